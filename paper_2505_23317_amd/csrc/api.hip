// C ABI of the library: context, validation, and the launch sequences of
// A1 (coarse encode), A2 (selection), A2+A3 (mixed-granularity varlen encode).
#include "../../include/cfdetr.h"

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "kernels.h"

using namespace cfdetr;

struct cfdetr_ctx {
  cfdetr_config cfg;
  cfdetr_weights w;
  Pyramid pyr;
  int device = 0;
  int n0 = 0;          // coarse cells per frame
  int nonfinest = 0;   // cells of all levels but the finest, per frame
  bool bf16 = true;
  size_t esz = 2;      // bytes per activation element

  // one device allocation, carved up
  void* arena = nullptr;
  uint64_t arena_bytes = 0;
  float* x = nullptr;      // residual stream [Tm, d] fp32
  void* a = nullptr;       // LayerNorm output [Tm, d]
  void* qkv = nullptr;     // [Tm, 3d]
  void* o = nullptr;       // attention output [Tm, d]
  void* h = nullptr;       // FFN hidden [Tm, F]
  void* vt = nullptr;      // bf16 mode: V feature-major [d, vt_ld], frames padded to 64
  int vt_ld = 0;
  int32_t* pcu = nullptr;  // padded sequence offsets into vt
  int32_t* cu_all = nullptr;  // sequence offsets of the encoder run in flight
  int32_t* m_all = nullptr;   // its token total
  uint64_t tok_cap = 0;       // rows of the activation buffers
  float* x0 = nullptr;     // coarse-token cache of cfdetr_multilevel_batch [Bmax*N0, d]
  float* pe_row[kMaxLevels] = {};
  float* pe_col[kMaxLevels] = {};
  int32_t* coarse_desc = nullptr;  // static token table of the coarse grid, Bmax frames
  int32_t* coarse_cu = nullptr;    // i * N0
  uint8_t* hit[2] = {};   // selection flags; the two arrays alternate between calls
  int hit_bytes = 0;
  int parity = 0;
  int32_t* items = nullptr;   // attention work items, 8 * cap8 entries of four words
  int cap8 = 0;               // entries per queue (one queue per XCD)
  int32_t* queue_heads = nullptr;   // 8 fetch counters per layer, set by the plan kernel
  int attn_grid = 0;                // workgroups of an attention launch
  int32_t* m_seen = nullptr;        // pinned host: row totals of earlier runs (merged, fine only), copied back without a wait
  int32_t* n_roi = nullptr;         // regions per frame (scratch of the region proposal)
  int32_t* tok_pad = nullptr;       // padded token table, offsets and true lengths of the
  int32_t* cu_pad = nullptr;        // padded form of the fine pass
  int32_t* kv_len = nullptr;
  int block_q = 0;
  int32_t* err_flag = nullptr;
  int32_t* vt_pos = nullptr;     // position of every row of the run in vt (first LayerNorm writes it)
  void* tail_packed = nullptr;   // w_o, w_ff1, w_ff2 of every layer in the fused kernel's order
  uint64_t tail_packed_layer = 0;   // bytes per layer; 0: the shape has no fused kernel
  void* head_packed = nullptr;      // w_qkv of the first layer in the same layout

  // decoder (cfdetr_decoder_attach): its own allocation
  bool has_dec = false;
  cfdetr_decoder_weights dw;
  void* dec_arena = nullptr;
  float* dx = nullptr;        // residual stream of the queries [Bmax*Q, d] fp32
  void* da = nullptr;         // LayerNorm output / head input [Bmax*Q, d] bf16
  void* dqkv = nullptr;       // [Bmax*Q, 3d] bf16 (self-attention), first third reused for
                              // the cross-attention queries
  void* d_o = nullptr;        // attention output [Bmax*Q, d]
  void* dh = nullptr;         // FFN hidden [Bmax*Q, F]; also the box head's hidden rows
  void* dvt = nullptr;        // V of the queries, feature-major
  int dvt_ld = 0;
  int32_t* dcu = nullptr;     // i * Q
  int32_t* dcu_all = nullptr; // plan outputs for the query sequences
  int32_t* dm_all = nullptr;
  int32_t* dpcu = nullptr;
  int32_t* ditems = nullptr;
  int dcap8 = 0;
  int dgrid = 0;
  void* dmid_packed = nullptr;   // per layer: first out-projection and cross-attention query projection, packed
  void* dk_all = nullptr;     // keys of the tokens for every decoder layer, [L][max_tokens_total, d]
  void* dvt_all = nullptr;    // their values, feature-major, [L][d, vt_ld]
  int32_t* dqueue = nullptr;  // 8 counters per attention launch (two per layer)
  void* dtail_packed = nullptr;   // per layer: w_o2, w_ff1, w_ff2, next w_qkv in the fused
  uint64_t dtail_packed_layer = 0;   // kernel's order (0: no fused kernel for this shape)
  void* dhead_packed = nullptr;   // w_qkv of the first layer
  float* dz = nullptr;            // final LayerNorm of the queries in fp32 (fused path)

  std::string err;

  bool prof = false;
  std::vector<hipEvent_t> ev;   // pairs
  std::vector<int> ev_kind;
  size_t ev_used = 0;
};

namespace {

// Error text of the last failed cfdetr_create of this thread (no context exists then).
thread_local std::string g_create_err;

// Scratch memory of cfdetr_select_fine_static, the entry point for callers that cannot
// allocate: the cell flags of one selection (B frames times the cells of all levels but the
// finest, one byte each).  Every GPU the library runs
// on holds its own copy until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress; kernels get the device address that call returns.
constexpr uint64_t kStaticFlagBytes = 1u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticFlagBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up once per device, with that
// device current); returns an error text, or null on success.
const char* static_scratch(unsigned char** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return "cannot identify the current device";
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p)
      return "hipGetSymbolAddress of the static scratch array failed";
    g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
  }
  *out = g_scratch_ptr[dev];
  return nullptr;
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* __restrict__ p, uint64_t n16,
                                                        int32_t* __restrict__ word) {
  const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) p[i] = make_uint4(0, 0, 0, 0);
  if (i == 0) *word = 0;
}

// Clears the first `bytes` bytes at p (rounded up to 16; p is 256-byte aligned and the
// array is longer than any count this is called with) and *word.
hipError_t launch_fill_zero(unsigned char* p, uint64_t bytes, int32_t* word, hipStream_t s) {
  const uint64_t n16 = (bytes + 15) / 16;
  const unsigned blocks = (unsigned)((n16 + 255) / 256);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks ? blocks : 1), dim3(256), 0, s,
                     reinterpret_cast<uint4*>(p), n16, word);
  return hipGetLastError();
}

cfdetr_status fail(cfdetr_ctx* c, cfdetr_status st, const std::string& msg) {
  if (c) c->err = msg;
  return st;
}

cfdetr_status fail_create(cfdetr_status st, const std::string& msg) {
  g_create_err = msg;
  return st;
}

cfdetr_status fail_hip(cfdetr_ctx* c, const char* what, hipError_t e) {
  return fail(c, CFDETR_EDEVICE, std::string(what) + ": " + hipGetErrorString(e));
}

bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

const char* check_config(const cfdetr_config& c) {
  if (c.n_levels < 1 || c.n_levels > kMaxLevels) return "n_levels must be 1..3";
  for (int l = 0; l < c.n_levels; ++l) {
    if (!is_pow2(c.patch[l]) || c.patch[l] < 8) return "patch sizes must be powers of two >= 8";
    if (l > 0 && c.patch[l] * 2 != c.patch[l - 1]) return "each patch size must halve the previous";
  }
  if (c.img_h <= 0 || c.img_w <= 0 || c.img_h % c.patch[0] || c.img_w % c.patch[0])
    return "frame sides must be positive multiples of patch[0]";
  if (c.img_h / c.patch[c.n_levels - 1] > 16384 || c.img_w / c.patch[c.n_levels - 1] > 16384)
    return "a grid has more than 16384 cells per side";
  if (c.d_model <= 0 || c.d_model % 64 || c.d_model > 1024) return "d_model must be a multiple of 64, at most 1024";
  if (c.n_heads <= 0 || c.d_model % c.n_heads) return "d_model must be a multiple of n_heads";
  if (c.d_model / c.n_heads != 32 && c.d_model / c.n_heads != 64) return "head width must be 32 or 64";
  if (c.n_heads > 32) return "at most 32 heads";
  if (c.d_ffn <= 0 || c.d_ffn % 64) return "d_ffn must be a multiple of 64";
  if (c.n_layers < 1) return "n_layers must be >= 1";
  if (c.max_batch < 1 || c.max_batch > kMaxBatch) return "max_batch must be 1..64";
  const long n0 = (long)(c.img_h / c.patch[0]) * (c.img_w / c.patch[0]);
  if ((long)c.max_tokens_total < (long)c.max_batch * n0)
    return "max_tokens_total must hold the coarse grids of max_batch frames";
  if ((long)c.max_tokens_total > (1L << 24) * 64) return "max_tokens_total too large";
  return nullptr;
}

struct Carver {
  uint64_t off = 0;
  uint64_t take(uint64_t bytes) {
    uint64_t at = off;
    off += (bytes + 255) & ~uint64_t(255);
    return at;
  }
};

// --- profiling ---------------------------------------------------------------
void prof_open(cfdetr_ctx* c, int kind, hipStream_t s) {
  if (!c->prof || c->ev_used + 2 > c->ev.size()) return;
  hipEventRecord(c->ev[c->ev_used], s);
  c->ev_kind[c->ev_used / 2] = kind;
}
void prof_close(cfdetr_ctx* c, hipStream_t s) {
  if (!c->prof || c->ev_used + 2 > c->ev.size()) return;
  hipEventRecord(c->ev[c->ev_used + 1], s);
  c->ev_used += 2;
}

#define CF_LAUNCH(kind, expr)                                       \
  do {                                                              \
    prof_open(ctx, (kind), s);                                      \
    hipError_t e__ = (expr);                                        \
    prof_close(ctx, s);                                             \
    if (e__ != hipSuccess) return fail_hip(ctx, #expr, e__);        \
  } while (0)

cfdetr_status check_call(cfdetr_ctx* ctx, int B) {
  if (!ctx) return CFDETR_EINVAL;
  if (B < 1) return fail(ctx, CFDETR_EINVAL, "B must be >= 1");
  if (B > ctx->cfg.max_batch) return fail(ctx, CFDETR_ECAPACITY, "B exceeds max_batch");
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(ctx, "hipGetDevice", e);
  if (dev != ctx->device) return fail(ctx, CFDETR_EINVAL, "context belongs to another device");
  return CFDETR_OK;
}

// Patch embedding of the tokens of one level into ctx->x (and optionally out2).
cfdetr_status embed_level(cfdetr_ctx* ctx, const void* images, int level,
                          const int32_t* tok_desc, const int32_t* cu, int B, float* out,
                          float* out2, const int32_t* m_ptr, int m_host, int m_cap,
                          hipStream_t s) {
  EmbedArgs a;
  a.images = images;
  a.image_is_bf16 = ctx->cfg.image_dtype == CFDETR_BF16;
  a.level = level;
  a.patch = ctx->cfg.patch[level];
  a.img_h = ctx->cfg.img_h;
  a.img_w = ctx->cfg.img_w;
  a.tok_desc = tok_desc;
  a.cu_seqlens = cu;
  a.B = B;
  a.pe_row = ctx->pe_row[level];
  a.pe_col = ctx->pe_col[level];
  a.out = out;
  a.out2 = out2;
  CF_LAUNCH(CFDETR_K_EMBED, launch_embed(a, ctx->w.w_embed[level], ctx->w.b_embed[level],
                                         ctx->cfg.d_model, ctx->bf16, m_ptr, m_host, m_cap, s));
  return CFDETR_OK;
}

// All layers + final LayerNorm over the tokens in ctx->x.  The sequences are
// n_prefix coarse grids (n0 tokens each) followed by the B sequences of cu; the
// plan kernel turns that into ctx->cu_all / ctx->m_all, which every kernel reads
// on the device.  Output rows below split_row go to y0, the others to y1.
// The plan of an encoder run over n_prefix coarse grids followed by the caller's sequences.
PlanArgs encoder_plan(const cfdetr_ctx* ctx, int n_prefix) {
  PlanArgs p{};
  p.n_prefix = n_prefix;
  p.prefix_len = ctx->n0;
  p.block_q = ctx->block_q;
  p.heads = ctx->cfg.n_heads;
  p.items = ctx->items;
  p.cap8 = ctx->cap8;
  p.cu_all = ctx->cu_all;
  p.m_all = ctx->m_all;
  p.pcu = ctx->pcu;
  p.queue_heads = ctx->queue_heads;
  p.n_heads_q = 8 * ctx->cfg.n_layers;
  p.queue_start = ctx->attn_grid / 8;
  return p;
}

cfdetr_status run_encoder(cfdetr_ctx* ctx, const int32_t* cu, int B, int n_prefix, int m_cap,
                          float* y0, int split_row, float* y1, hipStream_t s,
                          const int32_t* kv_len = nullptr, bool plan_done = false) {
  const cfdetr_config& c = ctx->cfg;
  const cfdetr_weights& w = ctx->w;
  const int d = c.d_model, F = c.d_ffn;
  const size_t es = ctx->esz;
  const float eps = c.ln_eps;
  const bool bf = ctx->bf16;
  const int nseq = n_prefix + B;
  const int32_t* cu_all = ctx->cu_all;
  const int32_t* m_ptr = ctx->m_all;
  // The contraction launchers choose their tiles by the rows they expect.  The count of this
  // run is on the device; the count of the previous run of the same kind (copied back
  // without waiting for it) is a good guess in a stream of frames.  A coarse-only run has
  // exactly its capacity.
  int m_hint = 0;
  int32_t* m_seen = nullptr;
  if (cu == ctx->coarse_cu && n_prefix == 0) {
    m_hint = m_cap;
  } else if (ctx->m_seen && bf && !(gemm_residual_ln_supported(d, bf) && ctx->tail_packed_layer != 0)) {
    m_seen = ctx->m_seen + (n_prefix > 0 ? 0 : kv_len ? 2 : 1);
    m_hint = *static_cast<volatile int32_t*>(m_seen);
  }
  if (!plan_done)   // (the selection kernel of a merged run has made the plan already)
    CF_LAUNCH(CFDETR_K_PLAN, launch_plan(cu, B, encoder_plan(ctx, n_prefix), s,
                                         m_cap - n_prefix * ctx->n0, 0, ctx->err_flag));
  if (m_seen) {
    hipError_t e = hipMemcpyAsync(m_seen, ctx->m_all, 4, hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return fail_hip(ctx, "copy of the row count", e);
  }
  // Where a workgroup can own whole rows, the residual contractions also apply the
  // LayerNorm that follows them, and only the very first one is a launch of its own.
  const bool fused_ln = gemm_residual_ln_supported(d, bf);
  const bool fused_tail = fused_ln && ctx->tail_packed_layer != 0;
  for (int l = 0; l < c.n_layers; ++l) {
    const char* wqkv = static_cast<const char*>(w.w_qkv) + (size_t)l * 3 * d * d * es;
    const char* wo = static_cast<const char*>(w.w_o) + (size_t)l * d * d * es;
    const char* w1 = static_cast<const char*>(w.w_ff1) + (size_t)l * F * d * es;
    const char* w2 = static_cast<const char*>(w.w_ff2) + (size_t)l * d * F * es;
    const bool last = l + 1 == c.n_layers;
    if (fused_tail && l == 0)
      // first LayerNorm and q/k/v projection in one kernel
      CF_LAUNCH(CFDETR_K_QKV,
                launch_layer_head(ctx->x, ctx->head_packed, w.ln1_g, w.ln1_b, eps, w.b_qkv,
                                  attention_q_scale(d / c.n_heads), ctx->qkv, ctx->vt, ctx->vt_ld,
                                  cu_all, ctx->pcu, nseq, d, m_ptr, 0, m_cap, s));
    else if (!fused_ln || l == 0) {
      // the first LayerNorm of a bf16 run also lists where every row goes in vt
      const RowPositions rp{ctx->vt_pos, cu_all, ctx->pcu, nseq};
      const bool list = bf && l == 0 && d % 4 == 0;
      CF_LAUNCH(CFDETR_K_LN,
                launch_layernorm(ctx->x, w.ln1_g + (size_t)l * d, w.ln1_b + (size_t)l * d, ctx->a,
                                 bf, d, eps, m_ptr, 0, m_cap, 0, nullptr, s, list ? &rp : nullptr));
    }
    if (fused_tail) {
      // q, k, v of this layer came out of the kernel before (the previous layer's last)
    } else if (bf)
      CF_LAUNCH(CFDETR_K_QKV,
                launch_gemm_qkv(ctx->a, wqkv, w.b_qkv + (size_t)l * 3 * d, d,
                                attention_q_scale(d / c.n_heads), ctx->qkv, ctx->vt,
                                ctx->vt_ld, cu_all, ctx->pcu, nseq, m_ptr, m_hint, m_cap, s,
                                d % 4 == 0 ? ctx->vt_pos : nullptr));
    else
      CF_LAUNCH(CFDETR_K_QKV, launch_gemm(ctx->a, wqkv, w.b_qkv + (size_t)l * 3 * d, 3 * d, d,
                                          Epilogue::kBias, ctx->qkv, nullptr, bf, m_ptr, m_hint, m_cap,
                                          s));
    CF_LAUNCH(CFDETR_K_ATTN,
              launch_attention(ctx->qkv, ctx->vt, ctx->vt_ld, ctx->o, d, c.n_heads, ctx->items, ctx->cap8, ctx->queue_heads + 8 * l,
                               ctx->attn_grid, ctx->block_q, bf, kv_len, s));
    if (fused_tail) {
      // out-projection, LayerNorm, feed-forward block and the LayerNorm after it (the next
      // layer's first one, or the final one) in one kernel
      LayerTailArgs ta{};
      ta.O = ctx->o;
      ta.packed = static_cast<const char*>(ctx->tail_packed) + (size_t)l * ctx->tail_packed_layer;
      ta.b_o = w.b_o + (size_t)l * d;
      ta.ln2_g = w.ln2_g + (size_t)l * d;
      ta.ln2_b = w.ln2_b + (size_t)l * d;
      ta.b_ff1 = w.b_ff1 + (size_t)l * F;
      ta.b_ff2 = w.b_ff2 + (size_t)l * d;
      ta.resid = ctx->x;
      ta.ln_g = last ? w.lnf_g : w.ln1_g + (size_t)(l + 1) * d;
      ta.ln_b = last ? w.lnf_b : w.ln1_b + (size_t)(l + 1) * d;
      ta.eps = eps;
      ta.last = last;
      ta.out = y0;
      ta.split_row = split_row;
      ta.out2 = y1;
      ta.b_qkv = last ? nullptr : w.b_qkv + (size_t)(l + 1) * 3 * d;
      ta.q_scale = attention_q_scale(d / c.n_heads);
      ta.qk = ctx->qkv;
      ta.vt = ctx->vt;
      ta.vt_ld = ctx->vt_ld;
      ta.cu = cu_all;
      ta.pcu = ctx->pcu;
      ta.B = nseq;
      CF_LAUNCH(CFDETR_K_FF2, launch_layer_tail(ta, d, F, m_ptr, 0, m_cap, s));
      continue;
    }
    if (fused_ln) {
      CF_LAUNCH(CFDETR_K_OUT,
                launch_gemm_residual_ln(ctx->o, wo, w.b_o + (size_t)l * d, d, d, ctx->x,
                                        w.ln2_g + (size_t)l * d, w.ln2_b + (size_t)l * d, eps,
                                        ctx->a, true, 0, nullptr, m_ptr, 0, m_cap, s));
    } else {
      CF_LAUNCH(CFDETR_K_OUT, launch_gemm(ctx->o, wo, w.b_o + (size_t)l * d, d, d,
                                          Epilogue::kBiasResidual, nullptr, ctx->x, bf, m_ptr, m_hint,
                                          m_cap, s));
      CF_LAUNCH(CFDETR_K_LN,
                launch_layernorm(ctx->x, w.ln2_g + (size_t)l * d, w.ln2_b + (size_t)l * d, ctx->a,
                                 bf, d, eps, m_ptr, 0, m_cap, 0, nullptr, s));
    }
    CF_LAUNCH(CFDETR_K_FF1, launch_gemm(ctx->a, w1, w.b_ff1 + (size_t)l * F, F, d,
                                        Epilogue::kBiasGelu, ctx->h, nullptr, bf, m_ptr, m_hint, m_cap,
                                        s));
    if (fused_ln && !last)
      CF_LAUNCH(CFDETR_K_FF2,
                launch_gemm_residual_ln(ctx->h, w2, w.b_ff2 + (size_t)l * d, d, F, ctx->x,
                                        w.ln1_g + (size_t)(l + 1) * d,
                                        w.ln1_b + (size_t)(l + 1) * d, eps, ctx->a, true, 0,
                                        nullptr, m_ptr, 0, m_cap, s));
    else if (fused_ln)
      CF_LAUNCH(CFDETR_K_FF2,
                launch_gemm_residual_ln(ctx->h, w2, w.b_ff2 + (size_t)l * d, d, F, ctx->x, w.lnf_g,
                                        w.lnf_b, eps, y0, false, split_row, y1, m_ptr, 0, m_cap,
                                        s));
    else
      CF_LAUNCH(CFDETR_K_FF2, launch_gemm(ctx->h, w2, w.b_ff2 + (size_t)l * d, d, F,
                                          Epilogue::kBiasResidual, nullptr, ctx->x, bf, m_ptr, m_hint,
                                          m_cap, s));
  }
  if (!fused_ln)
    CF_LAUNCH(CFDETR_K_LN, launch_layernorm(ctx->x, w.lnf_g, w.lnf_b, y0, false, d, eps, m_ptr, 0,
                                            m_cap, split_row, y1, s));
  return CFDETR_OK;
}

cfdetr_status coarse_impl(cfdetr_ctx* ctx, const void* images, int B, float* x0_out,
                          float* y_coarse, hipStream_t s) {
  const int M = B * ctx->n0;
  cfdetr_status st = embed_level(ctx, images, 0, ctx->coarse_desc, ctx->coarse_cu, B, ctx->x,
                                 x0_out, nullptr, M, M, s);
  if (st != CFDETR_OK) return st;
  return run_encoder(ctx, ctx->coarse_cu, B, 0, M, y_coarse, 0, nullptr, s);
}

cfdetr_status select_impl(cfdetr_ctx* ctx, const int32_t* boxes, const uint8_t* tier,
                          const int32_t* box_offsets, int B, int32_t* tok_desc,
                          int32_t* cu_seqlens, int32_t* level_counts, hipStream_t s,
                          const PlanArgs* plan = nullptr, const int32_t* hard = nullptr) {
  uint8_t* cur = ctx->hit[ctx->parity];
  uint8_t* next = ctx->hit[ctx->parity ^ 1];
  ctx->parity ^= 1;
  CF_LAUNCH(CFDETR_K_SELECT,
            launch_select(ctx->pyr, boxes, tier, box_offsets, B, ctx->nonfinest, cur, next,
                          ctx->hit_bytes, ctx->cfg.max_tokens_total, tok_desc, cu_seqlens, level_counts,
                          ctx->err_flag, s, plan, hard));
  return CFDETR_OK;
}

// Tokens of the mixed-granularity sets into rows [row0, row0 + cu[B]) of ctx->x.
cfdetr_status fine_embed(cfdetr_ctx* ctx, const void* images, int B, const int32_t* tok_desc,
                         const int32_t* cu, const float* x0_cache, int row0, hipStream_t s) {
  const int cap = ctx->cfg.max_tokens_total;
  const int32_t* m_ptr = cu + B;
  float* dst = ctx->x + (size_t)row0 * ctx->cfg.d_model;
  int first = 0;
  if (x0_cache) {
    CF_LAUNCH(CFDETR_K_GATHER,
              launch_gather_coarse(tok_desc, cu, B, x0_cache, ctx->n0, ctx->pyr.cols[0],
                                   ctx->cfg.d_model, dst, cap, s));
    first = 1;
  }
  for (int l = first; l < ctx->cfg.n_levels; ++l) {
    cfdetr_status st =
        embed_level(ctx, images, l, tok_desc, cu, B, dst, nullptr, m_ptr, 0, cap, s);
    if (st != CFDETR_OK) return st;
  }
  return CFDETR_OK;
}

cfdetr_status fine_impl(cfdetr_ctx* ctx, const void* images, int B, const int32_t* tok_desc,
                        const int32_t* cu, const float* x0_cache, float* y_mixed,
                        hipStream_t s) {
  // The offsets are the caller's: the plan checks them first (a bad length or a total beyond
  // the capacity empties the run and raises the error flag), and every kernel after it,
  // the embedding included, reads the checked copy.
  const int cap = ctx->cfg.max_tokens_total;
  CF_LAUNCH(CFDETR_K_PLAN, launch_plan(cu, B, encoder_plan(ctx, 0), s, cap, 0, ctx->err_flag));
  cfdetr_status st = fine_embed(ctx, images, B, tok_desc, ctx->cu_all, x0_cache, 0, s);
  if (st != CFDETR_OK) return st;
  return run_encoder(ctx, ctx->cu_all, B, 0, cap, y_mixed, 0, nullptr, s, nullptr, true);
}

// A3 as the paper states it: every frame's token set brought to t_pad tokens (repeats of
// its last token, which cost what any padding token costs), all B*t_pad rows through every
// kernel, padded keys masked in the attention.  Row f*t_pad + j of y is token j of frame f.
cfdetr_status padded_impl(cfdetr_ctx* ctx, const void* images, int B, const int32_t* tok_desc,
                          const int32_t* cu, const float* x0_cache, int t_pad, float* y_padded,
                          hipStream_t s) {
  // the caller's offsets are checked first (as in fine_impl); the padding reads the checked copy
  CF_LAUNCH(CFDETR_K_PLAN, launch_plan(cu, B, encoder_plan(ctx, 0), s, ctx->cfg.max_tokens_total, 0,
                                       ctx->err_flag));
  CF_LAUNCH(CFDETR_K_SELECT, launch_pad_tokens(tok_desc, ctx->cu_all, B, t_pad, ctx->tok_pad,
                                               ctx->cu_pad, ctx->kv_len, ctx->err_flag, s));
  cfdetr_status st = fine_embed(ctx, images, B, ctx->tok_pad, ctx->cu_pad, x0_cache, 0, s);
  if (st != CFDETR_OK) return st;
  return run_encoder(ctx, ctx->cu_pad, B, 0, B * t_pad, y_padded, 0, nullptr, s, ctx->kv_len);
}

// Decoder over the encoded tokens `memory` of B frames (Sec. II-A).  The token side (bf16
// copy of the tokens, their keys and feature-major values) lives in the encoder's work
// space, which is idle here; the query side has the decoder's own buffers.
cfdetr_status decode_impl(cfdetr_ctx* ctx, const float* memory, const int32_t* cu, int B,
                          float* queries, hipStream_t s) {
  const cfdetr_config& c = ctx->cfg;
  const cfdetr_decoder_weights& w = ctx->dw;
  const int d = c.d_model, F = c.d_ffn, Q = w.n_queries, L = w.n_layers;
  const int Mq = B * Q, cap_m = c.max_tokens_total;
  const float eps = c.ln_eps;
  const float qs = attention_q_scale(d / c.n_heads);
  // token sequences: offsets, total and padded offsets (the work list is not used).  The
  // offsets are the caller's: the plan checks them, and after an error the second plan
  // hands the attention kernels no work.
  {
    PlanArgs p = encoder_plan(ctx, 0);
    p.n_heads_q = 8;
    CF_LAUNCH(CFDETR_K_PLAN, launch_plan(cu, B, p, s, cap_m, 1, ctx->err_flag, nullptr));
  }
  CF_LAUNCH(CFDETR_K_DEC, launch_cast_bf16(memory, ctx->a, d, ctx->m_all, cap_m, s));
  // query sequences: B times Q rows, work list for both attentions of every layer
  {
    PlanArgs p{};
    p.block_q = ctx->block_q;
    p.heads = c.n_heads;
    p.items = ctx->ditems;
    p.cap8 = ctx->dcap8;
    p.cu_all = ctx->dcu_all;
    p.m_all = ctx->dm_all;
    p.pcu = ctx->dpcu;
    p.queue_heads = ctx->dqueue;
    p.n_heads_q = 16 * L;
    p.queue_start = ctx->dgrid / 8;
    CF_LAUNCH(CFDETR_K_PLAN, launch_plan(ctx->dcu, B, p, s, 0, 0, nullptr, ctx->err_flag));
  }
  CF_LAUNCH(CFDETR_K_DEC, launch_broadcast_rows(w.query_embed, ctx->dx, Q, d, B, s));
  // The tokens' keys and values for the cross-attention of every layer depend on the tokens
  // and the weights only: one contraction for all layers, ahead of the loop.
  const size_t k_stride = (size_t)cap_m * d, v_stride = (size_t)d * ctx->vt_ld;
  CF_LAUNCH(CFDETR_K_DEC,
            launch_gemm_kv_layers(ctx->a, w.w_kv, w.b_kv, d, L, ctx->dk_all, k_stride, ctx->dvt_all,
                                  v_stride, ctx->vt_ld, ctx->cu_all, ctx->pcu, B, ctx->m_all, 0,
                                  cap_m, s));
  const char* wqkv = static_cast<const char*>(w.w_qkv);
  const char* wo = static_cast<const char*>(w.w_o);
  const char* wq = static_cast<const char*>(w.w_q);
  const char* wo2 = static_cast<const char*>(w.w_o2);
  const char* w1 = static_cast<const char*>(w.w_ff1);
  const char* w2 = static_cast<const char*>(w.w_ff2);
  // With the fused layer kernels (width 256) a layer is four launches: self-attention, one
  // kernel for its out-projection, the LayerNorm behind it and the query projection,
  // cross-attention, and one kernel for the second out-projection, the feed-forward block,
  // the LayerNorm after it and the next layer's q/k/v projection.
  const bool fused = ctx->dtail_packed_layer != 0;
  for (int l = 0; l < L; ++l) {
    const bool last = l + 1 == L;
    // self-attention among the queries of a frame
    if (fused && l == 0) {
      CF_LAUNCH(CFDETR_K_QKV,
                launch_layer_head(ctx->dx, ctx->dhead_packed, w.ln1_g, w.ln1_b, eps, w.b_qkv, qs,
                                  ctx->dqkv, ctx->dvt, ctx->dvt_ld, ctx->dcu_all, ctx->dpcu, B, d,
                                  nullptr, Mq, Mq, s));
    } else if (!fused) {
      CF_LAUNCH(CFDETR_K_LN, launch_layernorm(ctx->dx, w.ln1_g + (size_t)l * d, w.ln1_b + (size_t)l * d,
                                              ctx->da, true, d, eps, nullptr, Mq, Mq, 0, nullptr, s));
      CF_LAUNCH(CFDETR_K_QKV,
                launch_gemm_qkv(ctx->da, wqkv + (size_t)l * 3 * d * d * 2, w.b_qkv + (size_t)l * 3 * d,
                                d, qs, ctx->dqkv, ctx->dvt, ctx->dvt_ld, ctx->dcu_all, ctx->dpcu, B,
                                nullptr, Mq, Mq, s));
    }
    CF_LAUNCH(CFDETR_K_ATTN,
              launch_attention(ctx->dqkv, ctx->dvt, ctx->dvt_ld, ctx->d_o, d, c.n_heads, ctx->ditems, ctx->dcap8, ctx->dqueue + 16 * l,
                               ctx->dgrid, ctx->block_q, true, nullptr, s));
    // cross-attention: the queries read the tokens of their frame
    if (fused) {
      // first out-projection, LayerNorm and the query projection in one kernel
      CF_LAUNCH(CFDETR_K_OUT,
                launch_layer_mid(ctx->d_o, static_cast<const char*>(ctx->dmid_packed) + (size_t)l * 2 * d * d * 2,
                                 w.b_o + (size_t)l * d, w.ln2_g + (size_t)l * d, w.ln2_b + (size_t)l * d,
                                 eps, ctx->dx, w.b_q + (size_t)l * d, qs, ctx->dh, d, nullptr, Mq, Mq, s));
    } else {
      CF_LAUNCH(CFDETR_K_OUT, launch_gemm(ctx->d_o, wo + (size_t)l * d * d * 2, w.b_o + (size_t)l * d,
                                          d, d, Epilogue::kBiasResidual, nullptr, ctx->dx, true,
                                          nullptr, Mq, Mq, s));
      CF_LAUNCH(CFDETR_K_LN, launch_layernorm(ctx->dx, w.ln2_g + (size_t)l * d, w.ln2_b + (size_t)l * d,
                                              ctx->da, true, d, eps, nullptr, Mq, Mq, 0, nullptr, s));
    }
    if (!fused)
      CF_LAUNCH(CFDETR_K_QKV, launch_gemm(ctx->da, wq + (size_t)l * d * d * 2, w.b_q + (size_t)l * d, d,
                                          d, Epilogue::kBias, ctx->dh, nullptr, true, nullptr, Mq,
                                          Mq, s, qs));
    CF_LAUNCH(CFDETR_K_ATTN,
              launch_cross_attention(ctx->dh, static_cast<const bf16_t*>(ctx->dk_all) + l * k_stride,
                                     static_cast<const bf16_t*>(ctx->dvt_all) + l * v_stride,
                                     ctx->vt_ld, ctx->d_o,
                                     ctx->cu_all, ctx->pcu, d, c.n_heads, ctx->ditems,
                                     ctx->dcap8, ctx->dqueue + 16 * l + 8, ctx->dgrid, s));
    if (fused) {
      LayerTailArgs ta{};
      ta.O = ctx->d_o;
      ta.packed = static_cast<const char*>(ctx->dtail_packed) + (size_t)l * ctx->dtail_packed_layer;
      ta.b_o = w.b_o2 + (size_t)l * d;
      ta.ln2_g = w.ln3_g + (size_t)l * d;
      ta.ln2_b = w.ln3_b + (size_t)l * d;
      ta.b_ff1 = w.b_ff1 + (size_t)l * F;
      ta.b_ff2 = w.b_ff2 + (size_t)l * d;
      ta.resid = ctx->dx;
      ta.ln_g = last ? w.lnf_g : w.ln1_g + (size_t)(l + 1) * d;
      ta.ln_b = last ? w.lnf_b : w.ln1_b + (size_t)(l + 1) * d;
      ta.eps = eps;
      ta.last = last;
      ta.out = ctx->dz;
      ta.split_row = 0;
      ta.out2 = nullptr;
      ta.b_qkv = last ? nullptr : w.b_qkv + (size_t)(l + 1) * 3 * d;
      ta.q_scale = qs;
      ta.qk = ctx->dqkv;
      ta.vt = ctx->dvt;
      ta.vt_ld = ctx->dvt_ld;
      ta.cu = ctx->dcu_all;
      ta.pcu = ctx->dpcu;
      ta.B = B;
      CF_LAUNCH(CFDETR_K_FF2, launch_layer_tail(ta, d, F, nullptr, Mq, Mq, s));
      continue;
    }
    CF_LAUNCH(CFDETR_K_OUT, launch_gemm(ctx->d_o, wo2 + (size_t)l * d * d * 2, w.b_o2 + (size_t)l * d,
                                        d, d, Epilogue::kBiasResidual, nullptr, ctx->dx, true,
                                        nullptr, Mq, Mq, s));
    // feed-forward
    CF_LAUNCH(CFDETR_K_LN, launch_layernorm(ctx->dx, w.ln3_g + (size_t)l * d, w.ln3_b + (size_t)l * d,
                                            ctx->da, true, d, eps, nullptr, Mq, Mq, 0, nullptr, s));
    CF_LAUNCH(CFDETR_K_FF1, launch_gemm(ctx->da, w1 + (size_t)l * F * d * 2, w.b_ff1 + (size_t)l * F,
                                        F, d, Epilogue::kBiasGelu, ctx->dh, nullptr, true, nullptr,
                                        Mq, Mq, s));
    CF_LAUNCH(CFDETR_K_FF2, launch_gemm(ctx->dh, w2 + (size_t)l * d * F * 2, w.b_ff2 + (size_t)l * d,
                                        d, F, Epilogue::kBiasResidual, nullptr, ctx->dx, true,
                                        nullptr, Mq, Mq, s));
  }
  // heads: z = final LayerNorm (bf16); box perceptron hidden rows in dqkv / d_o
  if (fused)
    CF_LAUNCH(CFDETR_K_DEC, launch_cast_bf16(ctx->dz, ctx->da, d, ctx->dm_all, Mq, s));
  else
    CF_LAUNCH(CFDETR_K_LN, launch_layernorm(ctx->dx, w.lnf_g, w.lnf_b, ctx->da, true, d, eps, nullptr,
                                            Mq, Mq, 0, nullptr, s));
  CF_LAUNCH(CFDETR_K_DEC, launch_gemm(ctx->da, w.w_box1, w.b_box1, d, d, Epilogue::kBiasRelu,
                                      ctx->dqkv, nullptr, true, nullptr, Mq, Mq, s));
  CF_LAUNCH(CFDETR_K_DEC, launch_gemm(ctx->dqkv, w.w_box2, w.b_box2, d, d, Epilogue::kBiasRelu,
                                      ctx->d_o, nullptr, true, nullptr, Mq, Mq, s));
  CF_LAUNCH(CFDETR_K_DEC, launch_decoder_heads(ctx->da, ctx->d_o, w.w_cls, w.b_cls, w.w_box3,
                                               w.b_box3, d, Mq, queries, s));
  return CFDETR_OK;
}

// A1 -> A2 -> A3 with ONE encoder run: the B coarse grids and the B mixed token sets
// are 2B independent sequences of the same variable-length batch (same weights), so
// every layer kernel is launched once for both.  Only the coarse embedding has to
// come first (the mixed sets reuse its tokens); the selection needs the boxes only.
cfdetr_status merged_impl(cfdetr_ctx* ctx, const void* images, int B, const int32_t* boxes,
                          const uint8_t* tier, const int32_t* box_offsets, float* y_coarse,
                          float* y_mixed, int32_t* tok_desc, int32_t* cu_seqlens,
                          int32_t* level_counts, hipStream_t s) {
  const int Mc = B * ctx->n0;
  cfdetr_status st = embed_level(ctx, images, 0, ctx->coarse_desc, ctx->coarse_cu, B, ctx->x,
                                 ctx->x0, nullptr, Mc, Mc, s);
  if (st != CFDETR_OK) return st;
  // the selection also plans the run over the B coarse grids and the B mixed sets
  const PlanArgs plan = encoder_plan(ctx, B);
  st = select_impl(ctx, boxes, tier, box_offsets, B, tok_desc, cu_seqlens, level_counts, s, &plan);
  if (st != CFDETR_OK) return st;
  st = fine_embed(ctx, images, B, tok_desc, cu_seqlens, ctx->x0, Mc, s);
  if (st != CFDETR_OK) return st;
  return run_encoder(ctx, cu_seqlens, B, B, Mc + ctx->cfg.max_tokens_total, y_coarse, Mc,
                     y_mixed, s, nullptr, true);
}

}  // namespace

extern "C" {

CFDETR_API cfdetr_status cfdetr_create(const cfdetr_config* cfg, const cfdetr_weights* w, cfdetr_ctx** out) {
  if (out) *out = nullptr;
  if (!cfg || !w || !out) return fail_create(CFDETR_EINVAL, "null argument");
  if (const char* why = check_config(*cfg)) return fail_create(CFDETR_ESHAPE, why);
  if ((cfg->image_dtype != CFDETR_BF16 && cfg->image_dtype != CFDETR_FP32) ||
      (cfg->act_dtype != CFDETR_BF16 && cfg->act_dtype != CFDETR_FP32) || !(cfg->ln_eps > 0.f))
    return fail_create(CFDETR_EINVAL, "bad dtype or ln_eps");
  for (int l = 0; l < cfg->n_levels; ++l)
    if (!w->w_embed[l] || !w->b_embed[l] || !aligned16(w->w_embed[l]))
      return fail_create(CFDETR_EINVAL, "null or misaligned embedding weight");
  const void* ptrs[] = {w->ln1_g, w->ln1_b, w->w_qkv, w->b_qkv, w->w_o,   w->b_o,   w->ln2_g,
                        w->ln2_b, w->w_ff1, w->b_ff1, w->w_ff2, w->b_ff2, w->lnf_g, w->lnf_b};
  for (const void* p : ptrs)
    if (!p || !aligned16(p)) return fail_create(CFDETR_EINVAL, "null or misaligned weight");

  cfdetr_ctx* c = new (std::nothrow) cfdetr_ctx();
  if (!c) return fail_create(CFDETR_ENOMEM, "host allocation failed");
  c->cfg = *cfg;
  c->w = *w;
  c->bf16 = cfg->act_dtype == CFDETR_BF16;
  c->esz = c->bf16 ? 2 : 4;
  hipError_t e = hipGetDevice(&c->device);
  if (e != hipSuccess) {
    delete c;
    return fail_create(CFDETR_EDEVICE, std::string("hipGetDevice: ") + hipGetErrorString(e));
  }
  Pyramid& p = c->pyr;
  p.n_levels = cfg->n_levels;
  p.img_h = cfg->img_h;
  p.img_w = cfg->img_w;
  for (int l = 0; l < kMaxLevels; ++l) {
    p.patch[l] = l < cfg->n_levels ? cfg->patch[l] : 1;
    p.rows[l] = l < cfg->n_levels ? cfg->img_h / cfg->patch[l] : 0;
    p.cols[l] = l < cfg->n_levels ? cfg->img_w / cfg->patch[l] : 0;
  }
  c->n0 = p.rows[0] * p.cols[0];
  c->nonfinest = 0;
  for (int l = 0; l + 1 < cfg->n_levels; ++l) c->nonfinest += p.rows[l] * p.cols[l];
  c->block_q = attention_block_q();
  // Activation buffers hold one merged run: max_batch coarse grids + the mixed sets.
  c->tok_cap = (uint64_t)cfg->max_tokens_total + (uint64_t)cfg->max_batch * c->n0;
  {
    // Query tiles of a whole run, and of its longest possible sequence; an XCD never
    // gets more than (all items)/8 + (tiles of the longest sequence) work items.
    const int tiles_all = (int)((c->tok_cap + c->block_q - 1) / c->block_q) + 2 * cfg->max_batch;
    const int longest = std::max(cfg->max_tokens_total, c->n0);
    c->cap8 = (tiles_all * cfg->n_heads + 7) / 8 + (longest + c->block_q - 1) / c->block_q;
  }
  c->attn_grid = attention_grid(cfg->d_model / cfg->n_heads, c->bf16, c->cap8);
  if (c->attn_grid < 8) {
    delete c;
    return fail_create(CFDETR_EDEVICE, "cannot size the attention grid for this device");
  }

  const uint64_t Tm = c->tok_cap, d = cfg->d_model, F = cfg->d_ffn;
  const uint64_t Bm = cfg->max_batch, D = d / 2;
  Carver cv;
  const uint64_t o_x = cv.take(Tm * d * 4), o_a = cv.take(Tm * d * c->esz);
  const uint64_t o_qkv = cv.take(Tm * 3 * d * c->esz), o_o = cv.take(Tm * d * c->esz);
  const uint64_t o_h = cv.take(Tm * F * c->esz), o_x0 = cv.take(Bm * c->n0 * d * 4);
  c->vt_ld = (int)((Tm + 64 * 2 * Bm + 63) & ~uint64_t(63));
  const uint64_t vt_bytes = c->bf16 ? d * (uint64_t)c->vt_ld * 2 : 256;
  const uint64_t o_vt = cv.take(vt_bytes), o_pcu = cv.take((2 * Bm + 1) * 4);
  const uint64_t o_cua = cv.take((2 * Bm + 1) * 4), o_mall = cv.take(4);
  uint64_t o_per[kMaxLevels], o_pec[kMaxLevels];
  for (int l = 0; l < cfg->n_levels; ++l) {
    o_per[l] = cv.take((uint64_t)p.rows[l] * D * 4);
    o_pec[l] = cv.take((uint64_t)p.cols[l] * D * 4);
  }
  const uint64_t o_cd = cv.take(Bm * c->n0 * 4), o_cc = cv.take((Bm + 1) * 4);
  const uint64_t hit_bytes = Bm * (uint64_t)(c->nonfinest > 0 ? c->nonfinest : 1);
  const uint64_t o_hit0 = cv.take(hit_bytes), o_hit1 = cv.take(hit_bytes);
  c->hit_bytes = (int)hit_bytes;
  const uint64_t o_items = cv.take((uint64_t)c->cap8 * 8 * 16), o_err = cv.take(4);
  const uint64_t o_vtpos = cv.take(Tm * 4);
  const uint64_t o_qh = cv.take((uint64_t)cfg->n_layers * 8 * 4);
  const uint64_t o_nroi = cv.take((uint64_t)kMaxBatch * 4);
  const uint64_t o_tpad = cv.take((uint64_t)cfg->max_tokens_total * 4);
  const uint64_t o_cupad = cv.take((uint64_t)(kMaxBatch + 1) * 4), o_kvlen = cv.take((uint64_t)kMaxBatch * 4);
  if (layer_tail_supported((int)d, (int)F, c->bf16))
    c->tail_packed_layer = layer_tail_packed_bytes((int)d, (int)F);
  const uint64_t o_pack = cv.take(c->tail_packed_layer * cfg->n_layers);
  const uint64_t o_hpack = cv.take(c->tail_packed_layer ? 3 * d * d * 2 : 0);
  c->arena_bytes = cv.off;
  e = hipMalloc(&c->arena, c->arena_bytes);
  if (e != hipSuccess) {
    delete c;
    return fail_create(CFDETR_ENOMEM, std::string("hipMalloc of the work space: ") +
                                          hipGetErrorString(e));
  }
  // three pinned words for row counts that come back from the device without a wait; the
  // library works without them (tiles are then chosen for the capacity)
  if (hipHostMalloc(reinterpret_cast<void**>(&c->m_seen), 3 * sizeof(int32_t), hipHostMallocDefault) == hipSuccess)
    c->m_seen[0] = c->m_seen[1] = c->m_seen[2] = 0;
  else
    c->m_seen = nullptr;
  char* base = static_cast<char*>(c->arena);
  c->x = reinterpret_cast<float*>(base + o_x);
  c->a = base + o_a;
  c->qkv = base + o_qkv;
  c->o = base + o_o;
  c->h = base + o_h;
  c->x0 = reinterpret_cast<float*>(base + o_x0);
  c->vt = base + o_vt;
  c->pcu = reinterpret_cast<int32_t*>(base + o_pcu);
  c->cu_all = reinterpret_cast<int32_t*>(base + o_cua);
  c->m_all = reinterpret_cast<int32_t*>(base + o_mall);
  for (int l = 0; l < cfg->n_levels; ++l) {
    c->pe_row[l] = reinterpret_cast<float*>(base + o_per[l]);
    c->pe_col[l] = reinterpret_cast<float*>(base + o_pec[l]);
  }
  c->coarse_desc = reinterpret_cast<int32_t*>(base + o_cd);
  c->coarse_cu = reinterpret_cast<int32_t*>(base + o_cc);
  c->hit[0] = reinterpret_cast<uint8_t*>(base + o_hit0);
  c->hit[1] = reinterpret_cast<uint8_t*>(base + o_hit1);
  c->items = reinterpret_cast<int32_t*>(base + o_items);
  c->err_flag = reinterpret_cast<int32_t*>(base + o_err);
  c->vt_pos = reinterpret_cast<int32_t*>(base + o_vtpos);
  c->queue_heads = reinterpret_cast<int32_t*>(base + o_qh);
  c->n_roi = reinterpret_cast<int32_t*>(base + o_nroi);
  c->tok_pad = reinterpret_cast<int32_t*>(base + o_tpad);
  c->cu_pad = reinterpret_cast<int32_t*>(base + o_cupad);
  c->kv_len = reinterpret_cast<int32_t*>(base + o_kvlen);
  c->tail_packed = base + o_pack;
  c->head_packed = base + o_hpack;

  // static tables: coarse grid descriptors, zeroed counters, position tables
  std::vector<int32_t> desc(Bm * c->n0), cu(Bm + 1);
  for (uint64_t b = 0; b < Bm; ++b)
    for (int r = 0; r < p.rows[0]; ++r)
      for (int q = 0; q < p.cols[0]; ++q) desc[b * c->n0 + r * p.cols[0] + q] = (r << 14) | q;
  for (uint64_t b = 0; b <= Bm; ++b) cu[b] = (int32_t)(b * c->n0);
  e = hipMemcpy(c->coarse_desc, desc.data(), desc.size() * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(c->coarse_cu, cu.data(), cu.size() * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemset(c->hit[0], 0, hit_bytes);
  if (e == hipSuccess) e = hipMemset(c->hit[1], 0, hit_bytes);
  // Padding positions of vt are read (with probability 0) by the attention kernel:
  // they must hold finite numbers.  Everything ever written there is finite, so
  // zeroing once is enough.
  if (e == hipSuccess) e = hipMemset(c->vt, 0, vt_bytes);
  if (e == hipSuccess) e = hipMemset(c->err_flag, 0, 4);
  for (int l = 0; l < cfg->n_levels && e == hipSuccess; ++l)
    e = launch_pe_tables(p.patch[l], p.rows[l], p.cols[l], p.img_h, p.img_w, (int)d, c->pe_row[l],
                         c->pe_col[l], nullptr);
  // the weights after attention in the order the fused kernel streams them
  for (int l = 0; l < cfg->n_layers && e == hipSuccess && c->tail_packed_layer; ++l)
    e = launch_layer_tail_pack(
        static_cast<const char*>(w->w_o) + (size_t)l * d * d * 2,
        static_cast<const char*>(w->w_ff1) + (size_t)l * F * d * 2,
        static_cast<const char*>(w->w_ff2) + (size_t)l * d * F * 2,
        l + 1 < cfg->n_layers ? static_cast<const char*>(w->w_qkv) + (size_t)(l + 1) * 3 * d * d * 2
                              : nullptr,
        (int)d, (int)F, static_cast<char*>(c->tail_packed) + (size_t)l * c->tail_packed_layer,
        nullptr);
  if (e == hipSuccess && c->tail_packed_layer)
    e = launch_layer_head_pack(w->w_qkv, (int)d, c->head_packed, nullptr);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    if (c->m_seen) hipHostFree(c->m_seen);
    hipFree(c->arena);
    delete c;
    return fail_create(CFDETR_EDEVICE, std::string("context set-up: ") + hipGetErrorString(e));
  }
  *out = c;
  return CFDETR_OK;
}

CFDETR_API void cfdetr_destroy(cfdetr_ctx* ctx) {
  if (!ctx) return;
  hipDeviceSynchronize();
  for (hipEvent_t ev : ctx->ev) hipEventDestroy(ev);
  if (ctx->m_seen) hipHostFree(ctx->m_seen);
  if (ctx->arena) hipFree(ctx->arena);
  if (ctx->dec_arena) hipFree(ctx->dec_arena);
  delete ctx;
}

CFDETR_API const char* cfdetr_last_error(const cfdetr_ctx* ctx) {
  return ctx ? ctx->err.c_str() : g_create_err.c_str();
}

CFDETR_API uint64_t cfdetr_workspace_bytes(const cfdetr_ctx* ctx) { return ctx ? ctx->arena_bytes : 0; }

CFDETR_API cfdetr_status cfdetr_sync_status(cfdetr_ctx* ctx, void* hip_stream) {
  if (!ctx) return CFDETR_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail_hip(ctx, "hipStreamSynchronize", e);
  int32_t flag = 0;
  e = hipMemcpy(&flag, ctx->err_flag, 4, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail_hip(ctx, "hipMemcpy", e);
  if (flag) {
    e = hipMemset(ctx->err_flag, 0, 4);
    if (e != hipSuccess) return fail_hip(ctx, "hipMemset", e);
    return fail(ctx, CFDETR_ECAPACITY, "a device-side check failed: more tokens or regions than the context holds, or bad sequence offsets");
  }
  return CFDETR_OK;
}

CFDETR_API cfdetr_status cfdetr_coarse_encode(cfdetr_ctx* ctx, const void* images, int32_t B,
                                   float* x0_cache, float* y_coarse, void* hip_stream) {
  cfdetr_status st = check_call(ctx, B);
  if (st != CFDETR_OK) return st;
  if (!images || !y_coarse) return fail(ctx, CFDETR_EINVAL, "null pointer");
  if (!aligned16(images) || !aligned16(y_coarse) || !aligned16(x0_cache))
    return fail(ctx, CFDETR_EINVAL, "pointers must be 16-byte aligned");
  return coarse_impl(ctx, images, B, x0_cache, y_coarse, static_cast<hipStream_t>(hip_stream));
}

CFDETR_API cfdetr_status cfdetr_propose_rois(cfdetr_ctx* ctx, const float* queries, int32_t B,
                                  int32_t Q, const cfdetr_roi_params* params,
                                  int32_t max_boxes, int32_t* boxes, uint8_t* tier,
                                  int32_t* box_offsets, int32_t* hard, float* mean_conf,
                                  void* hip_stream) {
  cfdetr_status st = check_call(ctx, B);
  if (st != CFDETR_OK) return st;
  if (!queries || !params || !boxes || !tier || !box_offsets || !hard || !mean_conf)
    return fail(ctx, CFDETR_EINVAL, "null pointer");
  if (!aligned16(queries) || !aligned16(boxes))
    return fail(ctx, CFDETR_EINVAL, "queries and boxes must be 16-byte aligned");
  if (Q < 1 || Q > 65536 || max_boxes < 0) return fail(ctx, CFDETR_EINVAL, "bad query or box count");
  if (!(params->tau_lo <= params->tau_hi) || !(params->scale >= 0.f) ||
      !(params->min_side >= 0.f) || params->tier < 0 || params->tier >= ctx->cfg.n_levels)
    return fail(ctx, CFDETR_EINVAL, "bad region parameters");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  CF_LAUNCH(CFDETR_K_ROI,
            launch_propose_rois(queries, B, Q, ctx->cfg.img_h, ctx->cfg.img_w, params->tau_hi,
                                params->tau_lo, params->scale, params->min_side, params->tier,
                                ctx->n_roi, max_boxes, boxes, tier, box_offsets, hard, mean_conf,
                                ctx->err_flag, s));
  return CFDETR_OK;
}

CFDETR_API cfdetr_status cfdetr_merge_detections(cfdetr_ctx* ctx, const float* coarse,
                                     const float* fine, const int32_t* hard, int32_t B,
                                     int32_t Q, float tau_hi, float tau_fine, float* det,
                                     uint8_t* src, int32_t* count, void* hip_stream) {
  cfdetr_status st = check_call(ctx, B);
  if (st != CFDETR_OK) return st;
  if (!coarse || !fine || !hard || !det || !src || !count)
    return fail(ctx, CFDETR_EINVAL, "null pointer");
  if (Q < 1 || Q > 65536) return fail(ctx, CFDETR_EINVAL, "bad query count");
  if (tau_hi != tau_hi || tau_fine != tau_fine) return fail(ctx, CFDETR_EINVAL, "threshold is not a number");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  CF_LAUNCH(CFDETR_K_ROI, launch_merge_detections(coarse, fine, hard, B, Q, tau_hi, tau_fine, det,
                                                  src, count, s));
  return CFDETR_OK;
}

CFDETR_API cfdetr_status cfdetr_select_fine(cfdetr_ctx* ctx, const int32_t* boxes, const uint8_t* tier,
                                 const int32_t* box_offsets, int32_t B, int32_t* tok_desc,
                                 int32_t* cu_seqlens, int32_t* level_counts, void* hip_stream) {
  cfdetr_status st = check_call(ctx, B);
  if (st != CFDETR_OK) return st;
  if (!boxes || !tier || !box_offsets || !tok_desc || !cu_seqlens)
    return fail(ctx, CFDETR_EINVAL, "null pointer");
  if (!aligned16(boxes)) return fail(ctx, CFDETR_EINVAL, "boxes must be 16-byte aligned");
  return select_impl(ctx, boxes, tier, box_offsets, B, tok_desc, cu_seqlens, level_counts,
                     static_cast<hipStream_t>(hip_stream));
}

CFDETR_API cfdetr_status cfdetr_select_fine_hard(cfdetr_ctx* ctx, const int32_t* boxes,
                                      const uint8_t* tier, const int32_t* box_offsets,
                                      const int32_t* hard, int32_t B, int32_t* tok_desc,
                                      int32_t* cu_seqlens, int32_t* level_counts,
                                      void* hip_stream) {
  cfdetr_status st = check_call(ctx, B);
  if (st != CFDETR_OK) return st;
  if (!boxes || !tier || !box_offsets || !hard || !tok_desc || !cu_seqlens)
    return fail(ctx, CFDETR_EINVAL, "null pointer");
  if (!aligned16(boxes)) return fail(ctx, CFDETR_EINVAL, "boxes must be 16-byte aligned");
  return select_impl(ctx, boxes, tier, box_offsets, B, tok_desc, cu_seqlens, level_counts,
                     static_cast<hipStream_t>(hip_stream), nullptr, hard);
}

CFDETR_API cfdetr_status cfdetr_select_fine_static(const cfdetr_config* cfg, const int32_t* boxes,
                                        const uint8_t* tier, const int32_t* box_offsets,
                                        int32_t B, int32_t* tok_desc, int32_t* cu_seqlens,
                                        int32_t* level_counts, int32_t* overflow,
                                        void* hip_stream) {
  if (!cfg || !boxes || !tier || !box_offsets || !tok_desc || !cu_seqlens || !overflow)
    return fail_create(CFDETR_EINVAL, "null pointer");
  if (const char* why = check_config(*cfg)) return fail_create(CFDETR_ESHAPE, why);
  if (B < 1) return fail_create(CFDETR_EINVAL, "B must be >= 1");
  if (B > cfg->max_batch) return fail_create(CFDETR_ECAPACITY, "B exceeds max_batch");
  if (!aligned16(boxes)) return fail_create(CFDETR_EINVAL, "boxes must be 16-byte aligned");
  Pyramid p;
  p.n_levels = cfg->n_levels;
  p.img_h = cfg->img_h;
  p.img_w = cfg->img_w;
  int nonfinest = 0;
  for (int l = 0; l < kMaxLevels; ++l) {
    p.patch[l] = l < cfg->n_levels ? cfg->patch[l] : 1;
    p.rows[l] = l < cfg->n_levels ? cfg->img_h / cfg->patch[l] : 0;
    p.cols[l] = l < cfg->n_levels ? cfg->img_w / cfg->patch[l] : 0;
    if (l + 1 < cfg->n_levels) nonfinest += p.rows[l] * p.cols[l];
  }
  const uint64_t flag_bytes = (uint64_t)B * (uint64_t)nonfinest;
  if (flag_bytes > kStaticFlagBytes)
    return fail_create(CFDETR_ECAPACITY,
                       "B times the cells of the non-finest levels exceeds the 1 MiB of static scratch");
  unsigned char* scratch_dev = nullptr;
  if (const char* why = static_scratch(&scratch_dev)) return fail_create(CFDETR_EDEVICE, why);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  uint8_t* flags = scratch_dev;
  // The array keeps what the last call left: the flags of this call's cells, and the
  // caller's overflow word, start from zero (a fill kernel, so that the call can be
  // captured into a graph).
  hipError_t e = launch_fill_zero(flags, flag_bytes, overflow, s);
  if (e == hipSuccess)
    e = launch_select(p, boxes, tier, box_offsets, B, nonfinest, flags, nullptr, 0,
                      cfg->max_tokens_total, tok_desc, cu_seqlens, level_counts, overflow, s);
  if (e != hipSuccess)
    return fail_create(CFDETR_EDEVICE, std::string("selection launch: ") + hipGetErrorString(e));
  return CFDETR_OK;
}

CFDETR_API cfdetr_status cfdetr_fine_encode(cfdetr_ctx* ctx, const void* images, int32_t B,
                                 const int32_t* tok_desc, const int32_t* cu_seqlens,
                                 const float* x0_cache, float* y_mixed, void* hip_stream) {
  cfdetr_status st = check_call(ctx, B);
  if (st != CFDETR_OK) return st;
  if (!images || !tok_desc || !cu_seqlens || !y_mixed) return fail(ctx, CFDETR_EINVAL, "null pointer");
  if (!aligned16(images) || !aligned16(y_mixed) || !aligned16(x0_cache))
    return fail(ctx, CFDETR_EINVAL, "pointers must be 16-byte aligned");
  return fine_impl(ctx, images, B, tok_desc, cu_seqlens, x0_cache, y_mixed,
                   static_cast<hipStream_t>(hip_stream));
}

CFDETR_API cfdetr_status cfdetr_fine_encode_padded(cfdetr_ctx* ctx, const void* images, int32_t B,
                                        const int32_t* tok_desc, const int32_t* cu_seqlens,
                                        const float* x0_cache, int32_t t_pad, float* y_padded,
                                        void* hip_stream) {
  cfdetr_status st = check_call(ctx, B);
  if (st != CFDETR_OK) return st;
  if (!images || !tok_desc || !cu_seqlens || !y_padded) return fail(ctx, CFDETR_EINVAL, "null pointer");
  if (!aligned16(images) || !aligned16(y_padded) || !aligned16(x0_cache))
    return fail(ctx, CFDETR_EINVAL, "pointers must be 16-byte aligned");
  if (t_pad < ctx->n0) return fail(ctx, CFDETR_EINVAL, "t_pad below the coarse grid size");
  if ((int64_t)B * t_pad > ctx->cfg.max_tokens_total)
    return fail(ctx, CFDETR_ECAPACITY, "B * t_pad exceeds max_tokens_total");
  return padded_impl(ctx, images, B, tok_desc, cu_seqlens, x0_cache, t_pad, y_padded,
                     static_cast<hipStream_t>(hip_stream));
}

CFDETR_API cfdetr_status cfdetr_multilevel_batch(cfdetr_ctx* ctx, const void* images, int32_t B,
                                      const int32_t* boxes, const uint8_t* tier,
                                      const int32_t* box_offsets, float* y_coarse, float* y_mixed,
                                      int32_t* tok_desc, int32_t* cu_seqlens,
                                      int32_t* level_counts, void* hip_stream) {
  cfdetr_status st = check_call(ctx, B);
  if (st != CFDETR_OK) return st;
  if (!images || !boxes || !tier || !box_offsets || !y_coarse || !y_mixed || !tok_desc ||
      !cu_seqlens)
    return fail(ctx, CFDETR_EINVAL, "null pointer");
  if (!aligned16(images) || !aligned16(y_coarse) || !aligned16(y_mixed) || !aligned16(boxes))
    return fail(ctx, CFDETR_EINVAL, "pointers must be 16-byte aligned");
  return merged_impl(ctx, images, B, boxes, tier, box_offsets, y_coarse, y_mixed, tok_desc,
                     cu_seqlens, level_counts, static_cast<hipStream_t>(hip_stream));
}

CFDETR_API cfdetr_status cfdetr_decoder_attach(cfdetr_ctx* ctx, const cfdetr_decoder_weights* w) {
  if (!ctx) return CFDETR_EINVAL;
  if (!w) return fail(ctx, CFDETR_EINVAL, "null argument");
  if (ctx->has_dec) return fail(ctx, CFDETR_EINVAL, "the context already has a decoder");
  if (!ctx->bf16) return fail(ctx, CFDETR_ESHAPE, "the decoder needs act_dtype bf16");
  if (w->n_queries < 1 || w->n_queries > 1024 || w->n_layers < 1)
    return fail(ctx, CFDETR_ESHAPE, "n_queries must be 1..1024 and n_layers >= 1");
  const void* ptrs[] = {w->query_embed, w->ln1_g, w->ln1_b, w->w_qkv, w->b_qkv, w->w_o,   w->b_o,
                        w->ln2_g,       w->ln2_b, w->w_q,  w->b_q,   w->w_kv,  w->b_kv, w->w_o2,
                        w->b_o2,        w->ln3_g, w->ln3_b, w->w_ff1, w->b_ff1, w->w_ff2, w->b_ff2,
                        w->lnf_g,       w->lnf_b, w->w_cls, w->b_cls, w->w_box1, w->b_box1,
                        w->w_box2,      w->b_box2, w->w_box3, w->b_box3};
  for (const void* p : ptrs)
    if (!p) return fail(ctx, CFDETR_EINVAL, "null decoder weight");
  const void* al[] = {w->query_embed, w->ln1_g, w->ln1_b, w->w_qkv, w->b_qkv, w->w_o, w->b_o,
                      w->ln2_g, w->ln2_b, w->w_q, w->b_q, w->w_kv, w->b_kv, w->w_o2, w->b_o2,
                      w->ln3_g, w->ln3_b, w->w_ff1, w->b_ff1, w->w_ff2, w->b_ff2, w->lnf_g,
                      w->lnf_b, w->w_box1, w->b_box1, w->w_box2, w->b_box2};
  for (const void* p : al)
    if (!aligned16(p)) return fail(ctx, CFDETR_EINVAL, "misaligned decoder weight");
  const cfdetr_config& c = ctx->cfg;
  const uint64_t Bm = c.max_batch, Q = w->n_queries, d = c.d_model, F = c.d_ffn;
  const uint64_t Mq = Bm * Q;
  // query tiles of a whole run; per queue at most all/8 + those of one sequence
  const int tiles_seq = (int)((Q + ctx->block_q - 1) / ctx->block_q);
  ctx->dcap8 = (int)((Bm * tiles_seq * c.n_heads + 7) / 8) + tiles_seq;
  ctx->dgrid = attention_grid(c.d_model / c.n_heads, true, ctx->dcap8);
  if (ctx->dgrid < 8) return fail(ctx, CFDETR_EDEVICE, "cannot size the attention grid");
  ctx->dvt_ld = (int)(Bm * ((Q + 63) & ~uint64_t(63)) + 64);
  Carver cv;
  const uint64_t o_x = cv.take(Mq * d * 4), o_a = cv.take(Mq * d * 2), o_qkv = cv.take(Mq * 3 * d * 2);
  const uint64_t o_o = cv.take(Mq * d * 2), o_h = cv.take(Mq * std::max(F, d) * 2);
  const uint64_t o_vt = cv.take(d * (uint64_t)ctx->dvt_ld * 2);
  const uint64_t o_cu = cv.take((Bm + 1) * 4), o_cua = cv.take((Bm + 1) * 4), o_m = cv.take(4);
  const uint64_t o_pcu = cv.take((Bm + 1) * 4), o_items = cv.take((uint64_t)ctx->dcap8 * 8 * 16);
  const uint64_t o_q = cv.take((uint64_t)w->n_layers * 16 * 4);
  const bool fused = layer_tail_supported((int)d, (int)F, true) && gemm_residual_ln_supported((int)d, true);
  const uint64_t tail_bytes = fused ? layer_tail_packed_bytes((int)d, (int)F) : 0;
  const uint64_t o_tail = cv.take(tail_bytes * w->n_layers);
  const uint64_t o_head = cv.take(fused ? 3 * d * d * 2 : 0), o_z = cv.take(fused ? Mq * d * 4 : 0);
  const uint64_t o_mid = cv.take(fused ? 2 * d * d * 2 * w->n_layers : 0);
  const uint64_t k_bytes = (uint64_t)c.max_tokens_total * d * 2, v_bytes = d * (uint64_t)ctx->vt_ld * 2;
  const uint64_t o_kall = cv.take(k_bytes * w->n_layers), o_vall = cv.take(v_bytes * w->n_layers);
  hipError_t e = hipMalloc(&ctx->dec_arena, cv.off);
  if (e != hipSuccess) return fail(ctx, CFDETR_ENOMEM, "hipMalloc of the decoder work space");
  char* base = static_cast<char*>(ctx->dec_arena);
  ctx->dx = reinterpret_cast<float*>(base + o_x);
  ctx->da = base + o_a;
  ctx->dqkv = base + o_qkv;
  ctx->d_o = base + o_o;
  ctx->dh = base + o_h;
  ctx->dvt = base + o_vt;
  ctx->dcu = reinterpret_cast<int32_t*>(base + o_cu);
  ctx->dcu_all = reinterpret_cast<int32_t*>(base + o_cua);
  ctx->dm_all = reinterpret_cast<int32_t*>(base + o_m);
  ctx->dpcu = reinterpret_cast<int32_t*>(base + o_pcu);
  ctx->ditems = reinterpret_cast<int32_t*>(base + o_items);
  ctx->dqueue = reinterpret_cast<int32_t*>(base + o_q);
  ctx->dtail_packed = base + o_tail;
  ctx->dhead_packed = base + o_head;
  ctx->dz = reinterpret_cast<float*>(base + o_z);
  ctx->dmid_packed = base + o_mid;
  ctx->dk_all = base + o_kall;
  ctx->dvt_all = base + o_vall;
  std::vector<int32_t> cu(Bm + 1);
  for (uint64_t b = 0; b <= Bm; ++b) cu[b] = (int32_t)(b * Q);
  e = hipMemcpy(ctx->dcu, cu.data(), cu.size() * 4, hipMemcpyHostToDevice);
  // padding positions of the feature-major V are read (with probability 0): keep them finite
  if (e == hipSuccess) e = hipMemset(ctx->dvt, 0, d * (uint64_t)ctx->dvt_ld * 2);
  if (e == hipSuccess) e = hipMemset(ctx->dvt_all, 0, v_bytes * w->n_layers);
  // the weights the fused layer kernels stream, in their order
  for (int l = 0; l < w->n_layers && e == hipSuccess && fused; ++l)
    e = launch_layer_tail_pack(
        static_cast<const char*>(w->w_o2) + (size_t)l * d * d * 2,
        static_cast<const char*>(w->w_ff1) + (size_t)l * F * d * 2,
        static_cast<const char*>(w->w_ff2) + (size_t)l * d * F * 2,
        l + 1 < w->n_layers ? static_cast<const char*>(w->w_qkv) + (size_t)(l + 1) * 3 * d * d * 2
                            : nullptr,
        (int)d, (int)F, static_cast<char*>(ctx->dtail_packed) + (size_t)l * tail_bytes, nullptr);
  if (e == hipSuccess && fused) e = launch_layer_head_pack(w->w_qkv, (int)d, ctx->dhead_packed, nullptr);
  for (int l = 0; l < w->n_layers && e == hipSuccess && fused; ++l)
    e = launch_layer_mid_pack(static_cast<const char*>(w->w_o) + (size_t)l * d * d * 2,
                              static_cast<const char*>(w->w_q) + (size_t)l * d * d * 2, (int)d,
                              static_cast<char*>(ctx->dmid_packed) + (size_t)l * 2 * d * d * 2, nullptr);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    hipFree(ctx->dec_arena);
    ctx->dec_arena = nullptr;
    return fail_hip(ctx, "decoder work space set-up", e);
  }
  ctx->dw = *w;
  ctx->dtail_packed_layer = tail_bytes;
  ctx->has_dec = true;
  return CFDETR_OK;
}

CFDETR_API cfdetr_status cfdetr_decode(cfdetr_ctx* ctx, const float* memory,
                            const int32_t* cu_seqlens, int32_t B, float* queries,
                            void* hip_stream) {
  cfdetr_status st = check_call(ctx, B);
  if (st != CFDETR_OK) return st;
  if (!ctx->has_dec) return fail(ctx, CFDETR_EINVAL, "no decoder attached");
  if (!memory || !cu_seqlens || !queries) return fail(ctx, CFDETR_EINVAL, "null pointer");
  if (!aligned16(memory)) return fail(ctx, CFDETR_EINVAL, "memory must be 16-byte aligned");
  return decode_impl(ctx, memory, cu_seqlens, B, queries, static_cast<hipStream_t>(hip_stream));
}

CFDETR_API cfdetr_status cfdetr_profile_begin(cfdetr_ctx* ctx) {
  if (!ctx) return CFDETR_EINVAL;
  if (ctx->ev.empty()) {
    const size_t want = 2 * 8192;
    ctx->ev.reserve(want);
    for (size_t i = 0; i < want; ++i) {
      hipEvent_t ev;
      hipError_t e = hipEventCreate(&ev);
      if (e != hipSuccess) return fail_hip(ctx, "hipEventCreate", e);
      ctx->ev.push_back(ev);
    }
    ctx->ev_kind.assign(want / 2, 0);
  }
  ctx->ev_used = 0;
  ctx->prof = true;
  return CFDETR_OK;
}

CFDETR_API cfdetr_status cfdetr_profile_end(cfdetr_ctx* ctx, float* total_ms, int32_t* launches) {
  if (!ctx || !total_ms || !launches) return CFDETR_EINVAL;
  ctx->prof = false;
  for (int k = 0; k < CFDETR_K_COUNT; ++k) {
    total_ms[k] = 0.f;
    launches[k] = 0;
  }
  if (ctx->ev_used == 0) return CFDETR_OK;
  hipError_t e = hipEventSynchronize(ctx->ev[ctx->ev_used - 1]);
  if (e != hipSuccess) return fail_hip(ctx, "hipEventSynchronize", e);
  for (size_t i = 0; i < ctx->ev_used; i += 2) {
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, ctx->ev[i], ctx->ev[i + 1]);
    if (e != hipSuccess) return fail_hip(ctx, "hipEventElapsedTime", e);
    int k = ctx->ev_kind[i / 2];
    total_ms[k] += ms;
    launches[k] += 1;
  }
  ctx->ev_used = 0;
  return CFDETR_OK;
}

}  // extern "C"
