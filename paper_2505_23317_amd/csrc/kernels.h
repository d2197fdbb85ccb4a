// Host-side launchers of the cfdetr kernels.  Every launcher enqueues on the
// given stream and returns the hipGetLastError() of its launches; none of them
// synchronises or allocates.
#pragma once
#include "common.h"

namespace cfdetr {

// What launch_plan writes and how (see there); also accepted by launch_select, whose last
// workgroup then makes the plan for the run that follows (the n_prefix prefix sequences plus
// the B token sets it has just counted).
struct PlanArgs {
  int n_prefix, prefix_len, block_q, heads;
  int32_t* items;
  int cap8;
  int32_t* cu_all;
  int32_t* m_all;
  int32_t* pcu;
  int32_t* queue_heads;
  int n_heads_q, queue_start;
};

// ---- A2 selection (select.hip) -------------------------------------------
// hard       (may be null) [B]: a frame with hard[f] == 0 skips the fine stage and gets no
//            token at all (length 0, counts 0).
// hit        [B, nonfinest] bytes, all zero on entry: flag of every cell of the levels
//            below the finest (level-major) that a box asking for a finer level
//            overlaps; hit_next (hit_bytes long) is the array of the following call
//            and is cleared.
hipError_t launch_select(const Pyramid& pyr, const int32_t* boxes, const uint8_t* tier,
                         const int32_t* box_offsets, int B, int nonfinest, uint8_t* hit,
                         uint8_t* hit_next, int hit_bytes, int max_tokens, int32_t* tok_desc,
                         int32_t* cu_seqlens, int32_t* level_counts, int32_t* err_flag,
                         hipStream_t s, const PlanArgs* plan = nullptr,
                         const int32_t* hard = nullptr);

// ---- A1 difficulty test + A2 region proposal (roi.hip) ----------------------
// queries [B, Q, 5] = (cx, cy, w, h, c), centre and size as fractions of the frame.
// Frame f is hard unless the average of its confidences not above tau_hi is below
// tau_lo; a hard frame proposes, in query order, the box of every query with
// tau_lo < c <= tau_hi, scaled by `scale` about its centre, at least min_side pixels
// wide and high, rounded outward to pixels and clipped, with refinement level
// tier_value.  Writes hard[B], mean_conf[B], n_roi[B] (scratch), boxes/tier (at most
// max_boxes; a larger total proposes nothing and raises *err_flag) and box_offsets[B+1].
hipError_t launch_propose_rois(const float* queries, int B, int Q, int H, int W, float tau_hi,
                               float tau_lo, float scale, float min_side, int tier_value,
                               int32_t* n_roi, int max_boxes, int32_t* boxes, uint8_t* tier,
                               int32_t* box_offsets, int32_t* hard, float* mean_conf,
                               int32_t* err_flag, hipStream_t s);

// Final detections per frame: coarse queries with c > tau_hi, then (hard frames) fine-stage
// queries with c > tau_fine, both in query order, into det [B, 2Q, 5] / src [B, 2Q] (0
// coarse, 1 fine); rows past count[f] are cleared (0 / 255).
hipError_t launch_merge_detections(const float* coarse, const float* fine, const int32_t* hard,
                                   int B, int Q, float tau_hi, float tau_fine, float* det,
                                   uint8_t* src, int32_t* count, hipStream_t s);

// Padded copy of a token table (the paper's own form of A3: every frame's token set is
// brought to one length).  Frame f gets rows f*t_pad .. (f+1)*t_pad of tok_pad: its own
// tokens, then repeats of its last one.  cu_pad[f] = f*t_pad, kv_len[f] = its true
// length (t_pad and *err_flag = 1 if that exceeds t_pad).
hipError_t launch_pad_tokens(const int32_t* tok_desc, const int32_t* cu_seqlens, int B, int t_pad,
                             int32_t* tok_pad, int32_t* cu_pad, int32_t* kv_len,
                             int32_t* err_flag, hipStream_t s);

// Sequence list and attention work list of one encoder run.  The sequences are
// n_prefix sequences of prefix_len tokens (coarse grids of a merged run; may be 0)
// followed by the B sequences delimited by cu_seqlens.  Writes cu_all[0..nseq] and
// m_all (offsets and total), pcu[0..nseq] (offsets with every sequence padded to a
// multiple of 64: the layout of the feature-major copy of V), and items[0..8*cap8)
// entries of four words (so items holds 32*cap8 words): the attention work item of
// workgroup w (sequence<<24 | head<<19 | query tile, or -1) followed by the offset,
// length and padded offset of its sequence, arranged so that all tiles of one
// (sequence, head) run on the same XCD.
// Also sets queue_heads[0..n_heads_q), the fetch counters of the attention launches
// that follow (eight per launch), to queue_start = (attention grid) / 8: the entries
// before that are handed out by workgroup index; or to -1 for a queue with no entries
// beyond those.
// max_total > 0 checks offsets that a caller wrote: a length below min_len, or a total above
// max_total, gives every one of the B sequences length 0 (the run then computes and writes
// nothing for them) and sets *err_flag.  gate (may be null): if
// *gate is not 0 the work list comes out empty, so that the attention launches that
// follow do nothing after an earlier kernel has raised the error flag.
hipError_t launch_plan(const int32_t* cu_seqlens, int B, const PlanArgs& plan, hipStream_t s,
                       int max_total = 0, int min_len = 0, int32_t* err_flag = nullptr,
                       const int32_t* gate = nullptr);

// ---- row-wise kernels (rowwise.hip) ----------------------------------------
// Position tables of one level: pe_row [rows, d/2], pe_col [cols, d/2] (fp32).
hipError_t launch_pe_tables(int patch, int rows, int cols, int img_h, int img_w, int d,
                            float* pe_row, float* pe_col, hipStream_t s);
// Where the rows of a run sit in the feature-major copy of V: out[m] = pcu[f] + (m - cu[f])
// for row m of sequence f (cu, pcu: nseq + 1 offsets from launch_plan).
struct RowPositions {
  int32_t* out;
  const int32_t* cu;
  const int32_t* pcu;
  int nseq;
};
// out = LayerNorm(x) * g + b for rows < M, M = *m_ptr if m_ptr else m_host.
// out_is_bf16 selects bf16 bit patterns or fp32 for `out`.  Rows >= split_row go to
// out2 (row - split_row) instead, when out2 is given.  With `positions` (widths that are
// multiples of 4 only) the kernel also fills that table for its rows: every row's frame is
// found once per run instead of once per projection.
hipError_t launch_layernorm(const float* x, const float* g, const float* b, void* out,
                            bool out_is_bf16, int d, float eps, const int32_t* m_ptr,
                            int m_host, int m_capacity, int split_row, void* out2,
                            hipStream_t s, const RowPositions* positions = nullptr);
// out (bf16 bit patterns) = in (fp32) for the first M * d elements, M = *m_ptr.
hipError_t launch_cast_bf16(const float* in, void* out, int d, const int32_t* m_ptr,
                            int m_capacity, hipStream_t s);
// dst[f*rows .. (f+1)*rows) = src[0 .. rows) for f < copies (rows of d floats).
hipError_t launch_broadcast_rows(const float* src, float* dst, int rows, int d, int copies,
                                 hipStream_t s);
// Heads of the decoder: out[m] = (sigmoid(hb[m] . w_box[0..3] + b_box), sigmoid(z[m] . w_cls
// + b_cls)) for m < M; z and hb [M, d] and the weight rows in bf16, out [M, 5] fp32.
hipError_t launch_decoder_heads(const void* z, const void* hb, const void* w_cls,
                                const float* b_cls, const void* w_box, const float* b_box, int d,
                                int M, float* out, hipStream_t s);
// x[t] = x0[frame(t)*n0 + row*cols0 + col] for every level-0 token t < cu[B].
hipError_t launch_gather_coarse(const int32_t* tok_desc, const int32_t* cu_seqlens, int B,
                                const float* x0, int n0, int cols0, int d, float* x,
                                int m_capacity, hipStream_t s);

// ---- contractions (gemm.hip) -----------------------------------------------
struct EmbedArgs {
  const void* images;     // [B,3,H,W]
  bool image_is_bf16;
  int level;              // tokens of this level only; other rows are left untouched
  int patch;              // pixels per side at this level
  int img_h, img_w;
  const int32_t* tok_desc;
  const int32_t* cu_seqlens;
  int B;
  const float* pe_row;    // [rows, d/2]
  const float* pe_col;    // [cols, d/2]
  float* out;             // [M, d] fp32
  float* out2;            // optional second copy (may be nullptr)
};
// Patch gather + projection + bias + position for the tokens of one level.
// w [d, 3*patch^2] in bf16 (use_bf16) or fp32.
hipError_t launch_embed(const EmbedArgs& a, const void* w, const float* bias, int d,
                        bool use_bf16, const int32_t* m_ptr, int m_host, int m_capacity,
                        hipStream_t s);

enum class Epilogue { kBias, kBiasGelu, kBiasRelu, kBiasResidual };
// C = (A[M,K] . W[N,K]^T + bias) * scale (scale: bf16 path only), then per `epi`:
//   kBias         -> out_act (activation dtype)
//   kBiasGelu     -> GELU, out_act
//   kBiasRelu     -> max(., 0), out_act (bf16 path only)
//   kBiasResidual -> resid[M,N] (fp32) += result, in place (no scale)
hipError_t launch_gemm(const void* A, const void* W, const float* bias, int N, int K,
                       Epilogue epi, void* out_act, float* resid, bool use_bf16,
                       const int32_t* m_ptr, int m_host, int m_capacity, hipStream_t s,
                       float scale = 1.0f);

// bf16 key/value projections of the decoder's cross-attention for `layers` layers at once
// (the tokens are the same for all of them): W [layers * 2d, d] and bias [layers * 2d] stack
// the layers' key and value rows; layer l's keys go token-major to k + l * k_stride
// (elements, [M, d] each), its values feature-major to vt + l * vt_stride like
// launch_gemm_qkv.  d must be a multiple of 64.
hipError_t launch_gemm_kv_layers(const void* A, const void* W, const float* bias, int d, int layers,
                                 void* k, size_t k_stride, void* vt, size_t vt_stride, int vt_ld,
                                 const int32_t* cu_seqlens, const int32_t* pcu, int B,
                                 const int32_t* m_ptr, int m_host, int m_capacity, hipStream_t s);

// Residual contraction followed by LayerNorm of the updated rows, in one kernel (bf16
// operands): resid[M,d] += A[M,K] . W[d,K]^T + bias, then
// out = LayerNorm(resid) * ln_g + ln_b in bf16 (out_is_bf16) or fp32; rows >= split_row
// go to out2 (row - split_row) when out2 is given.  Only for the widths
// gemm_residual_ln_supported names.
bool gemm_residual_ln_supported(int d, bool use_bf16);
hipError_t launch_gemm_residual_ln(const void* A, const void* W, const float* bias, int d, int K,
                                   float* resid, const float* ln_g, const float* ln_b, float eps,
                                   void* out, bool out_is_bf16, int split_row, void* out2,
                                   const int32_t* m_ptr, int m_host, int m_capacity,
                                   hipStream_t s);

// Everything of a layer after attention, with the LayerNorm that follows it, in one
// kernel:  resid[M,d] += O[M,d] . Wo[d,d]^T + b_o;  a = LayerNorm(resid) * ln2_g + ln2_b;
// resid += GELU(a . W1[F,d]^T + b_ff1) . W2[d,F]^T + b_ff2;  n = LayerNorm(resid) * ln_g + ln_b.
// last: n goes to out in fp32 (rows >= split_row to out2 at row - split_row when out2 is
// given).  Otherwise the kernel goes on with the next layer's query/key/value projection
// of n (bias b_qkv [3d]) and writes q, k, v exactly as launch_gemm_qkv does; n itself is
// not written.  The matrices are read from a packed copy (layer_tail_packed_bytes) that
// launch_layer_tail_pack writes once (Wqkv_next null for the last layer).  Only for the
// shapes layer_tail_supported names.
struct LayerTailArgs {
  const void* O;
  const void* packed;
  const float *b_o, *ln2_g, *ln2_b, *b_ff1, *b_ff2;
  float* resid;
  const float *ln_g, *ln_b;
  float eps;
  bool last;
  float* out;      // last only
  int split_row;
  float* out2;
  const float* b_qkv;   // the rest: not last only
  float q_scale;
  void* qk;
  void* vt;
  int vt_ld;
  const int32_t* cu;
  const int32_t* pcu;
  int B;
};
bool layer_tail_supported(int d, int F, bool use_bf16);
uint64_t layer_tail_packed_bytes(int d, int F);
hipError_t launch_layer_tail_pack(const void* Wo, const void* W1, const void* W2,
                                  const void* Wqkv_next, int d, int F, void* packed,
                                  hipStream_t s);
hipError_t launch_layer_tail(const LayerTailArgs& a, int d, int F, const int32_t* m_ptr,
                             int m_host, int m_capacity, hipStream_t s);

// The first layer's LayerNorm and query/key/value projection in the same style (width
// 256, bf16): q, k, v of LayerNorm(x) * ln_g + ln_b, written as launch_gemm_qkv writes
// them.  The matrix is read from a packed copy (3 d d elements) that
// launch_layer_head_pack writes once.
hipError_t launch_layer_head_pack(const void* Wqkv, int d, void* packed, hipStream_t s);
hipError_t launch_layer_head(const float* x, const void* packed, const float* ln_g,
                             const float* ln_b, float eps, const float* b_qkv, float q_scale,
                             void* qk, void* vt, int vt_ld, const int32_t* cu, const int32_t* pcu,
                             int B, int d, const int32_t* m_ptr, int m_host, int m_capacity,
                             hipStream_t s);

// Between the decoder's two attentions, in the same style (width 256, bf16): the output
// projection of the first with its residual, the LayerNorm behind it and the query
// projection of the second:  resid[M,d] += O . Wo^T + b_o;  q_out[M,d] (bf16) =
// ((LayerNorm(resid) * ln_g + ln_b) . Wq^T + b_q) * q_scale.  Both matrices are read from a
// packed copy (2 d d elements) that launch_layer_mid_pack writes once.
hipError_t launch_layer_mid_pack(const void* Wo, const void* Wq, int d, void* packed, hipStream_t s);
hipError_t launch_layer_mid(const void* O, const void* packed, const float* b_o, const float* ln_g,
                            const float* ln_b, float eps, float* resid, const float* b_q,
                            float q_scale, void* q_out, int d, const int32_t* m_ptr, int m_host,
                            int m_capacity, hipStream_t s);

// bf16 query/key/value projection: q and k go to qk [M, 3d] (columns 0..2d, bias added,
// q multiplied by q_scale = attention_q_scale(d_head) so that the attention kernel gets
// base-2 logits straight from its first MFMA); v goes feature-major to vt [d, vt_ld] at
// position pcu[frame] + (token - cu[frame]); vt_pos (may be null) holds those positions
// for all rows already (launch_layernorm with `positions`).
hipError_t launch_gemm_qkv(const void* A, const void* W, const float* bias, int d,
                           float q_scale, void* qk, void* vt, int vt_ld,
                           const int32_t* cu_seqlens, const int32_t* pcu, int B,
                           const int32_t* m_ptr, int m_host, int m_capacity, hipStream_t s,
                           const int32_t* vt_pos = nullptr);
// log2(e) / sqrt(d_head): the factor the bf16 attention kernel expects folded into q.
float attention_q_scale(int d_head);

// ---- attention (attention.hip) -----------------------------------------------
// qkv [M, 3d] (q | k | v, head h at columns h*dh), out [M, d], both in the activation
// dtype.  The bf16 kernel takes v from vt (see launch_gemm_qkv) instead of the last
// third of qkv and expects q pre-multiplied by attention_q_scale; its grid_size
// (= attention_grid) workgroups serve eight queues (items[x + 8j], j = 0, 1, ... for
// queue x): workgroup w takes entry w/8 of queue w%8 and then fetches through the
// counter queue_heads[w%8], which must be grid_size/8 at launch and is used up by it
// (-1: the queue has no further entries and is not asked).
// The fp32 kernel maps workgroup w to entry w (grid_size = 8*cap8).
// Softmax over the keys of the same frame only; with kv_len (may be null) only over the
// first kv_len[i] keys of sequence i, the rest being padding.
// The sequences' offsets come with the work items (launch_plan).
hipError_t launch_attention(const void* qkv, const void* vt, int vt_ld, void* out, int d, int heads,
                            const int32_t* items, int cap8, int32_t* queue_heads, int grid_size,
                            int block_q, bool use_bf16, const int32_t* kv_len, hipStream_t s);
// bf16 attention of query rows over the keys and values of another set of rows (the
// decoder's cross-attention): q [Mq, d] and k [Mk, d] (head h at columns h*dh, q
// pre-multiplied by attention_q_scale), v feature-major in vt at the padded offsets pcu_k
// of the key sequences; query sequence i attends to sequence i of cu_k.  Work items and
// counters as for launch_attention, planned over the query sequences.
hipError_t launch_cross_attention(const void* q, const void* k, const void* vt, int vt_ld,
                                  void* out, const int32_t* cu_k,
                                  const int32_t* pcu_k, int d, int heads, const int32_t* items,
                                  int cap8, int32_t* queue_heads, int grid_size, hipStream_t s);
// Grid of launch_attention on the current device: a multiple of 8, at most 8*cap8;
// 0 if the device cannot be queried.
int attention_grid(int d_head, bool use_bf16, int cap8);
// Queries per work item of both attention kernels.
int attention_block_q();

}  // namespace cfdetr
