// Contractions of the encoder: C[M,N] = A[M,K] . W[N,K]^T with fused epilogues.
//
// Both operands have K innermost, which is what the 32x32x16 bf16 MFMA wants: a
// lane supplies 8 consecutive k of one row.  The product is computed TRANSPOSED
// (MFMA A-operand = rows of W, B-operand = rows of the activations), so that in
// the result layout a lane owns one output ROW (token) and its registers hold runs
// of four consecutive output columns: the epilogue then works on 8- or 16-byte
// pieces (bias as float4, residual read-modify-write as float4, bf16 output as
// 4 packed values) and row validity is a per-lane question.
//
// Two bf16 kernels share that orientation:
//  * gemm_bf16_direct_kernel: activations x weights, and the patch embedding of bf16
//    frames (the A rows are then patch pixels: an implicit im2col).  K-slabs of 64 go
//    from global memory straight into LDS (global_load_lds, 16 bytes per lane, no VGPR
//    round trip) through a ring of two or four buffers, one barrier per slab.  LDS rows
//    are 128 bytes, unpadded; the 16-byte chunks of row r are stored at position
//    chunk ^ ((r/2) & 7), which keeps the operand reads of 16 consecutive rows (what
//    one LDS cycle serves) on disjoint banks.  The swizzle costs nothing: the lane that
//    fills LDS position p of row r simply fetches logical chunk p ^ ((r/2) & 7) from
//    global memory.
//  * gemm_bf16_gather_kernel: the patch embedding of fp32 frames.  The A rows are
//    pixels gathered patch by patch, converted and staged through registers into
//    padded LDS rows.
// A workgroup -> tile mapping that gives each XCD (own L2) a contiguous run of tiles,
// M read from device memory (grids are sized for the capacity; surplus workgroups
// leave at once), and an all-fp32 kernel for the check mode complete the file.
#include "kernels.h"

namespace cfdetr {

namespace {

constexpr int BK = 64;
constexpr int LDS_LD = BK + 8;  // padded row (elements) of the register-staged kernel

// ---------------------------------------------------------------------------
// Epilogues work on four consecutive columns n..n+3 of row m.  Loads and stores are
// separate calls:
//   row_info(m)                    per-row datum (position of the token, descriptor);
//   bias4(n)                       per-column addend, the same for every row;
//   extra4(m, n, info)             per-element addend (residual, position) or zero;
//   store4(m, n, v, b, x, info)    combines and stores, and loads nothing.
// Loads and stores share one in-order counter on this hardware: a load issued after a
// store cannot be waited for without waiting for the store as well, so alternating them
// costs a memory round trip per piece.  The kernels therefore fetch row_info and bias4
// before their main loop and extra4 in one batch per 32-row tile, ahead of its stores.
// ---------------------------------------------------------------------------
constexpr bool kNoExtra = false, kHasExtra = true;
__device__ __forceinline__ float gelu_erf(float x) {
  return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f));
}

// x * Phi(x) for the bf16 path, with Phi(x) ~ 1 / (1 + exp(-x (a + b x^2 + c x^4))),
// coefficients fitted to the erf form (maximum absolute error of the product 2.6e-5 over
// all x, two orders below the bf16 resolution of the values that matter); x is clamped
// to [-8, 8] inside the exponent, where the quartic is still positive.  The epilogue of
// the first FFN contraction evaluates this once per output element, and with K = d the
// main loop is short: seven plain operations and two transcendental ones per element
// keep it well below the cost of the MFMA loop.
__device__ __forceinline__ float gelu_fast(float x) {
  const float xc = __builtin_amdgcn_fmed3f(x, -8.0f, 8.0f);
  const float x2 = xc * xc;
  // -log2(e) * (a, b, c)
  const float t = fmaf(fmaf(1.0142780e-03f, x2, -1.0677580e-01f), x2, -2.3011212e+00f) * xc;
  return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t));
}

constexpr int kActNone = 0, kActGelu = 1, kActRelu = 2;

template <typename TAct, int kAct>
struct EpiAct;

// out = act((v + bias) * scale) in bf16
template <int kAct>
struct EpiAct<bf16_t, kAct> {
  const float* bias;
  bf16_t* out;
  int ldc;
  float scale;
  __device__ __forceinline__ float act(float r) const {
    r *= scale;
    if (kAct == kActGelu) return gelu_fast(r);
    if (kAct == kActRelu) return fmaxf(r, 0.f);
    return r;
  }
  static constexpr bool kExtra = kNoExtra;
  __device__ __forceinline__ int32_t row_info(int) const { return 0; }
  __device__ __forceinline__ bool row_ok(int32_t) const { return true; }
  __device__ __forceinline__ float4 bias4(int n) const {
    return *reinterpret_cast<const float4*>(bias + n);
  }
  __device__ __forceinline__ float4 extra4(int, int, int32_t) const {
    return make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __device__ __forceinline__ void store4(int m, int n, const float* v, const float4& b,
                                         const float4&, int32_t) const {
    const float r0 = act(v[0] + b.x), r1 = act(v[1] + b.y), r2 = act(v[2] + b.z),
                r3 = act(v[3] + b.w);
    uint2 w = make_uint2(pack_bf16x2(r0, r1), pack_bf16x2(r2, r3));
    *reinterpret_cast<uint2*>(out + (size_t)m * ldc + n) = w;
  }
  // staged form: the finished bf16 values go to LDS, rows leave it 16 bytes per lane
  static constexpr int kStageElem = 2;
  __device__ __forceinline__ bool staged(int) const { return true; }
  __device__ __forceinline__ void stage4(unsigned char* p, int, const float* v,
                                         const float4& b) const {
    const float r0 = act(v[0] + b.x), r1 = act(v[1] + b.y), r2 = act(v[2] + b.z),
                r3 = act(v[3] + b.w);
    *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(r0, r1), pack_bf16x2(r2, r3));
  }
  __device__ __forceinline__ void copy16(int m, int n, const uint4& d, const float4&) const {
    *reinterpret_cast<uint4*>(out + (size_t)m * ldc + n) = d;
  }
};

template <int kAct>
struct EpiAct<float, kAct> {
  const float* bias;
  float* out;
  int ldc;
  static constexpr bool kExtra = kNoExtra;
  __device__ __forceinline__ float4 bias4(int n) const {
    return *reinterpret_cast<const float4*>(bias + n);
  }
  __device__ __forceinline__ float4 extra4(int, int, int32_t) const {
    return make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __device__ __forceinline__ void store4(int m, int n, const float* v, const float4& b,
                                         const float4&, int32_t) const {
    float4 r = make_float4(v[0] + b.x, v[1] + b.y, v[2] + b.z, v[3] + b.w);
    if (kAct == kActGelu) r = make_float4(gelu_erf(r.x), gelu_erf(r.y), gelu_erf(r.z), gelu_erf(r.w));
    *reinterpret_cast<float4*>(out + (size_t)m * ldc + n) = r;
  }
};

struct EpiResidual {
  const float* bias;
  float* resid;
  int ldc;
  static constexpr bool kExtra = kHasExtra;
  __device__ __forceinline__ int32_t row_info(int) const { return 0; }
  __device__ __forceinline__ bool row_ok(int32_t) const { return true; }
  __device__ __forceinline__ float4 bias4(int n) const {
    return *reinterpret_cast<const float4*>(bias + n);
  }
  __device__ __forceinline__ float4 extra4(int m, int n, int32_t) const {
    return *reinterpret_cast<const float4*>(resid + (size_t)m * ldc + n);
  }
  __device__ __forceinline__ void store4(int m, int n, const float* v, const float4& b,
                                         const float4& xin, int32_t) const {
    float4 x = xin;
    x.x += v[0] + b.x;
    x.y += v[1] + b.y;
    x.z += v[2] + b.z;
    x.w += v[3] + b.w;
    *reinterpret_cast<float4*>(resid + (size_t)m * ldc + n) = x;
  }
  // staged form: v + bias goes to LDS in fp32; the residual rows are then read, updated
  // and written 16 bytes per lane (extra4 fetches the old values, same arithmetic)
  static constexpr int kStageElem = 4;
  __device__ __forceinline__ bool staged(int) const { return true; }
  __device__ __forceinline__ void stage4(unsigned char* p, int, const float* v,
                                         const float4& b) const {
    *reinterpret_cast<float4*>(p) = make_float4(v[0] + b.x, v[1] + b.y, v[2] + b.z, v[3] + b.w);
  }
  __device__ __forceinline__ void copy16(int m, int n, const uint4& d, const float4& xin) const {
    float4 x = xin;
    x.x += __uint_as_float(d.x);
    x.y += __uint_as_float(d.y);
    x.z += __uint_as_float(d.z);
    x.w += __uint_as_float(d.w);
    *reinterpret_cast<float4*>(resid + (size_t)m * ldc + n) = x;
  }
};

// Query/key/value projection: q and k columns (n < 2d) go token-major to qk [M, 3d];
// v columns go feature-major to vt [d, vt_ld], token m of frame f at position
// pcu[f] + (m - cu[f]).  row_info(m) is that position.
struct EpiQkv {
  const float* bias;
  bf16_t* qk;
  int ldc;    // 3d
  int d2;     // first v column (2d for q|k|v, d for k|v)
  int q_cols; // columns below this are queries (d, or 0 when there are none)
  float q_scale;   // queries leave multiplied by this
  bf16_t* vt;
  int vt_ld;
  const int32_t* cu;
  const int32_t* pcu;
  int B;
  const int32_t* vt_pos;   // the positions of all rows, if a kernel before has listed them
  __device__ __forceinline__ int32_t row_info(int m) const {
    if (vt_pos != nullptr) return vt_pos[m];
    const int f = frame_of_token(cu, B, m);
    return pcu[f] + (m - cu[f]);
  }
  __device__ __forceinline__ bool row_ok(int32_t) const { return true; }
  static constexpr bool kExtra = kNoExtra;
  __device__ __forceinline__ float4 bias4(int n) const {
    return *reinterpret_cast<const float4*>(bias + n);
  }
  __device__ __forceinline__ float4 extra4(int, int, int32_t) const {
    return make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __device__ __forceinline__ void store4(int m, int n, const float* v, const float4& b,
                                         const float4&, int32_t pos) const {
    float r0 = v[0] + b.x, r1 = v[1] + b.y, r2 = v[2] + b.z, r3 = v[3] + b.w;
    if (n < d2) {
      if (n < q_cols) {
        r0 *= q_scale;
        r1 *= q_scale;
        r2 *= q_scale;
        r3 *= q_scale;
      }
      *reinterpret_cast<uint2*>(qk + (size_t)m * ldc + n) =
          make_uint2(pack_bf16x2(r0, r1), pack_bf16x2(r2, r3));
    } else {
      bf16_t* p = vt + (size_t)(n - d2) * vt_ld + pos;
      p[0] = f32_to_bf16(r0);
      p[(size_t)vt_ld] = f32_to_bf16(r1);
      p[(size_t)2 * vt_ld] = f32_to_bf16(r2);
      p[(size_t)3 * vt_ld] = f32_to_bf16(r3);
    }
  }
  // staged form for the q and k columns (a wavefront's columns are all on one side of
  // 2d); the v columns keep store4: with a token per lane their feature-major stores are
  // already runs of 32 consecutive positions
  static constexpr int kStageElem = 2;
  __device__ __forceinline__ bool staged(int n_first) const { return n_first < d2; }
  __device__ __forceinline__ void stage4(unsigned char* p, int n, const float* v,
                                         const float4& b) const {
    float r0 = v[0] + b.x, r1 = v[1] + b.y, r2 = v[2] + b.z, r3 = v[3] + b.w;
    if (n < q_cols) {
      r0 *= q_scale;
      r1 *= q_scale;
      r2 *= q_scale;
      r3 *= q_scale;
    }
    *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(r0, r1), pack_bf16x2(r2, r3));
  }
  __device__ __forceinline__ void copy16(int m, int n, const uint4& d, const float4&) const {
    *reinterpret_cast<uint4*>(qk + (size_t)m * ldc + n) = d;
  }
};

// Key and value projections of several layers in one contraction (the decoder's cross-
// attention: the tokens are the same for every layer).  Column n belongs to layer
// n / (2d); inside a layer the first d columns are keys (token-major, k + layer *
// k_stride), the others values (feature-major, vt + layer * vt_stride, like EpiQkv).
struct EpiKvLayers {
  const float* bias;
  bf16_t* k;
  size_t k_stride;
  int d;
  bf16_t* vt;
  size_t vt_stride;
  int vt_ld;
  const int32_t* cu;
  const int32_t* pcu;
  int B;
  __device__ __forceinline__ int32_t row_info(int m) const {
    const int f = frame_of_token(cu, B, m);
    return pcu[f] + (m - cu[f]);
  }
  __device__ __forceinline__ bool row_ok(int32_t) const { return true; }
  static constexpr bool kExtra = kNoExtra;
  __device__ __forceinline__ float4 bias4(int n) const {
    return *reinterpret_cast<const float4*>(bias + n);
  }
  __device__ __forceinline__ float4 extra4(int, int, int32_t) const {
    return make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __device__ __forceinline__ void store4(int m, int n, const float* v, const float4& b,
                                         const float4&, int32_t pos) const {
    const float r0 = v[0] + b.x, r1 = v[1] + b.y, r2 = v[2] + b.z, r3 = v[3] + b.w;
    const int layer = n / (2 * d), nn = n - layer * 2 * d;
    if (nn < d) {
      *reinterpret_cast<uint2*>(k + layer * k_stride + (size_t)m * d + nn) =
          make_uint2(pack_bf16x2(r0, r1), pack_bf16x2(r2, r3));
    } else {
      bf16_t* p = vt + layer * vt_stride + (size_t)(nn - d) * vt_ld + pos;
      p[0] = f32_to_bf16(r0);
      p[(size_t)vt_ld] = f32_to_bf16(r1);
      p[(size_t)2 * vt_ld] = f32_to_bf16(r2);
      p[(size_t)3 * vt_ld] = f32_to_bf16(r3);
    }
  }
  // staged form for the key columns (a wavefront's columns are all keys or all values of
  // one layer: d is a multiple of its 64 columns)
  static constexpr int kStageElem = 2;
  __device__ __forceinline__ bool staged(int n_first) const { return n_first % (2 * d) < d; }
  __device__ __forceinline__ void stage4(unsigned char* p, int, const float* v,
                                         const float4& b) const {
    *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(v[0] + b.x, v[1] + b.y),
                                              pack_bf16x2(v[2] + b.z, v[3] + b.w));
  }
  __device__ __forceinline__ void copy16(int m, int n, const uint4& data, const float4&) const {
    const int layer = n / (2 * d), nn = n - layer * 2 * d;
    *reinterpret_cast<uint4*>(k + layer * k_stride + (size_t)m * d + nn) = data;
  }
};

struct EpiEmbed {
  const float* bias;
  const float* pe_row;
  const float* pe_col;
  float* out;
  float* out2;
  int d;
  const int32_t* tok_desc;   // for row_info (direct-load kernel); the other kernels pass
  int level;                 // the descriptor themselves
  static constexpr bool kExtra = kHasExtra;
  static constexpr int kStageElem = 0;   // rows of other levels lie in between: stores stay per row
  // descriptor of token m if it is a token of `level`, else -1 (row not to be written)
  __device__ __forceinline__ int32_t row_info(int m) const {
    const int32_t desc = tok_desc[m];
    return tok_level(desc) == level ? desc : -1;
  }
  __device__ __forceinline__ bool row_ok(int32_t info) const { return info >= 0; }
  __device__ __forceinline__ float4 bias4(int n) const {
    return *reinterpret_cast<const float4*>(bias + n);
  }
  __device__ __forceinline__ float4 extra4(int, int n, int32_t desc) const {
    const int D = d >> 1;  // a multiple of 32: a run of four never straddles the halves
    const float* pe = (n < D) ? pe_row + tok_row(desc) * D + n : pe_col + tok_col(desc) * D + (n - D);
    return *reinterpret_cast<const float4*>(pe);
  }
  __device__ __forceinline__ void store4(int m, int n, const float* v, const float4& b,
                                         const float4& e, int32_t) const {
    const float4 r = make_float4(v[0] + b.x + e.x, v[1] + b.y + e.y, v[2] + b.z + e.z,
                                 v[3] + b.w + e.w);
    *reinterpret_cast<float4*>(out + (size_t)m * d + n) = r;
    if (out2) *reinterpret_cast<float4*>(out2 + (size_t)m * d + n) = r;
  }
};

// The patch embedding contracts K in two halves and adds them (first + second) whenever K
// is a multiple of 128, in every form of the kernel: small problems give the halves to two
// groups of wavefronts, and a token must come out the same, bit for bit, whichever form
// embedded it (the coarse-stage result is reused for the coarse tokens of the mixed batch).
template <typename EP>
struct SumHalves { static constexpr bool value = false; };
template <>
struct SumHalves<EpiEmbed> { static constexpr bool value = true; };

// Maps a workgroup id to a tile id such that each of the 8 XCDs (workgroups are dealt
// to them round-robin) works on a contiguous run of tiles and its L2 sees the same
// activation rows again and again.
__device__ __forceinline__ int xcd_tile_order(int pid, int total) {
  const int per = total >> 3;
  return (pid < (per << 3)) ? (pid & 7) * per + (pid >> 3) : pid;
}

// ---------------------------------------------------------------------------
// Activations x weights, direct global -> LDS.
// ---------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

// 16 bytes per lane from global memory straight into LDS at lds_base + 16*lane
// (lds_base wave-uniform), issued in a form the compiler does not track: it then adds
// no wait of its own before LDS reads, and the caller orders fills and reads with
// explicit vmcnt waits and barriers.
__device__ __forceinline__ void dma16_untracked(const void* gptr, const unsigned char* lds_base) {
  // the low half of a flat pointer into LDS is the LDS address
  const uint32_t m0v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds_base);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(m0v), "v"(gptr)
               : "memory");   // M0 is reserved: the compiler keeps nothing in it
}

// The same with the address split into a wave-uniform base (kept in scalar registers,
// so that advancing it costs no vector instruction) and a 32-bit per-lane byte offset;
// lds_addr is the wave-uniform LDS byte address.
__device__ __forceinline__ void dma16_untracked_s(const void* sbase, uint32_t voff,
                                                  uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(sbase)
               : "memory");
}

// Where the rows of the A operand come from, as the three parts of a byte address that a
// load of 8 consecutive elements needs: base() + slab_off(k0) is the same for a whole
// wavefront (k0: first element of a K-slab of 64) and stays in scalar registers;
// row_off(r, M, ok) + lane_off(a) is the lane's own 32-bit part (row r; a: first of the
// lane's 8 elements inside the slab, a multiple of 8).  Rows that are not to be computed
// get ok = false and the offset of some valid row.  The callers see to it that the
// matrix (the batch of frames) is smaller than 4 GB.
struct DenseRows {   // an activation matrix [M, K], K innermost
  const bf16_t* A;
  int K;
  static constexpr bool kSparse = false;
  __device__ __forceinline__ const unsigned char* base() const {
    return reinterpret_cast<const unsigned char*>(A);
  }
  __device__ __forceinline__ uint32_t row_off(int r, int M, bool& ok) const {
    ok = r < M;
    return (uint32_t)min(r, M - 1) * (uint32_t)K * 2u;
  }
  __device__ __forceinline__ size_t slab_off(int k0) const { return (size_t)k0 * 2; }
  __device__ __forceinline__ uint32_t lane_off(int a) const { return (uint32_t)a * 2u; }
};

// Patch pixels of bf16 frames as rows (implicit im2col): row m is the patch of token m
// flattened (channel, row, column), for the tokens of one level only.  8 consecutive
// elements are 8 consecutive pixels of one patch row (patches are at least 8 wide).  A
// slab of 64 elements starts at a multiple of 64 and the patch side P is a power of two,
// so a slab lies in one channel and covers whole patch rows (P < 64) or a piece of one:
// element k0 + a is (a / P) image rows and a % P pixels behind element k0.
struct PatchPixelRows {
  const bf16_t* images;
  const int32_t* tok_desc;
  const int32_t* cu;
  int B, level, log2p, img_h, img_w;
  static constexpr bool kSparse = true;
  __device__ __forceinline__ const unsigned char* base() const {
    return reinterpret_cast<const unsigned char*>(images);
  }
  __device__ __forceinline__ uint32_t row_off(int r, int M, bool& ok) const {
    uint32_t off = 0;   // not ok: frame 0's first patch, in bounds, result discarded
    ok = r < M;
    if (ok) {
      const int32_t desc = tok_desc[r];
      ok = tok_level(desc) == level;
      if (ok) {
        const int frame = frame_of_token(cu, B, r);
        off = ((uint32_t)(frame * 3 * img_h + (tok_row(desc) << log2p)) * (uint32_t)img_w +
               (uint32_t)(tok_col(desc) << log2p)) * 2u;
      }
    }
    return off;
  }
  __device__ __forceinline__ size_t slab_off(int k0) const {
    const int c = k0 >> (2 * log2p);
    const int r = (k0 >> log2p) & ((1 << log2p) - 1);
    const int x = k0 & ((1 << log2p) - 1);
    return (((size_t)c * img_h + r) * img_w + x) * 2;
  }
  __device__ __forceinline__ uint32_t lane_off(int a) const {
    return ((uint32_t)(a >> log2p) * (uint32_t)img_w + (uint32_t)(a & ((1 << log2p) - 1))) * 2u;
  }
};

// Swizzle key of LDS row r for rows of ROWB bytes: the 16-byte chunks of a row are
// stored at position chunk ^ key, which keeps the operand reads of 16 consecutive rows
// (what one LDS cycle serves) on disjoint banks.
template <int ROWB>
__device__ __forceinline__ int lds_row_key(int r) {
  return ROWB == 128 ? ((r >> 1) & 7) : ((r >> 2) & 3);
}

template <int BM, int BN, int NWM, int NWN, int kStages, int BKT, typename AROWS, typename EP, int KS = 1, int WPE = 1>
__global__ __launch_bounds__(64 * NWM * NWN * KS, WPE) void gemm_bf16_direct_kernel(
    AROWS arows, const bf16_t* __restrict__ W, int N, int K, EP ep,
    const int32_t* __restrict__ m_ptr, int m_host) {
  constexpr int NW = NWM * NWN;
  constexpr int WTM = BM / NWM, WTN = BN / NWN;      // wavefront tile
  constexpr int MT = WTM / 32, NT = WTN / 32;        // 32x32 MFMA tiles, each way
  constexpr int ROWB = BKT * 2;                      // bytes of an LDS row (one K-slab of a row)
  constexpr int CPR = ROWB / 16;                     // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;                      // rows one wave instruction fills (1 KB)
  constexpr int A_INST = BM / (RPI * NW), B_INST = BN / (RPI * NW);
  constexpr int LPW = A_INST + B_INST;               // loads a wavefront issues per slab
  constexpr int STAGE = (BM + BN) * ROWB;            // bytes of one ring buffer (A rows, then W rows)
  static_assert(BKT == 32 || BKT == 64, "slab width");
  static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "tile / wavefront mismatch");
  static_assert(kStages >= 2 && kStages <= 4 && (kStages - 2) * LPW < 64, "ring depth");
  // KS = 2: a second group of wavefronts with a ring of its own contracts the second half
  // of K for the same tile, and the halves are added (first + second) at the end.  For
  // problems of fewer tiles than CUs, where a wavefront per SIMD leaves every unit idle
  // most of the time.  K must be a multiple of 2 BKT.
  static_assert(KS == 1 || (KS == 2 && MT * NT == 1 && kStages == 4 && BKT == 64 && EP::kStageElem == 0),
                "K split: single-tile wavefronts, direct epilogue");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_direct[];

  const int M = m_ptr ? *m_ptr : m_host;
  const int n_blocks = N / BN;
  const int total = ((M + BM - 1) / BM) * n_blocks;
  if ((int)blockIdx.x >= total) return;
  const int pid = xcd_tile_order(blockIdx.x, total);
  const int m0 = (pid / n_blocks) * BM;
  const int n0 = (pid % n_blocks) * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, and known to be
  const int grp = KS == 1 ? 0 : wave_all / NW;   // which part of K
  const int wave = KS == 1 ? wave_all : wave_all % NW;
  const int wm = wave / NWN, wn = wave % NWN;
  // Loader role: a wave instruction fills RPI consecutive LDS rows (1 KB).  Lane ->
  // (row lane/CPR of the group, LDS chunk position lane%CPR) and fetches the logical
  // chunk position ^ swizzle key of that row.  Of an address only the lane's 32-bit
  // offset lives in a vector register; what changes from slab to slab is wave-uniform
  // and is kept (and advanced) in scalar registers.
  const int lrow = lane / CPR, lpos = lane % CPR;
  uint32_t avo[A_INST], wvo[B_INST];
  bool any_row = false;
#pragma unroll
  for (int j = 0; j < A_INST; ++j) {
    const int rt = (wave * A_INST + j) * RPI + lrow;      // row inside the tile
    bool ok;
    avo[j] = arows.row_off(m0 + rt, M, ok) + arows.lane_off((lpos ^ lds_row_key<ROWB>(rt)) * 8);
    any_row |= ok;
  }
  if (AROWS::kSparse) {
    // a tile without a single row to compute (no token of the level) leaves at once
    if (!__syncthreads_or(any_row)) return;
  }
#pragma unroll
  for (int j = 0; j < B_INST; ++j) {
    const int rt = (wave * B_INST + j) * RPI + lrow;
    wvo[j] = ((uint32_t)(n0 + rt) * (uint32_t)K + (uint32_t)((lpos ^ lds_row_key<ROWB>(rt)) * 8)) * 2u;
  }
  // the low half of a flat pointer into LDS is the LDS address
  unsigned char* const ring = smem_direct + grp * (kStages * STAGE);
  const uint32_t lds0 = (uint32_t)(uintptr_t)ring;

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int l32 = lane & 31, g = lane >> 5;
  const int nk = K / (BKT * KS);
  const int kbase = grp * nk * BKT;   // first k of this group's part
  // one group and two halves: the sums so far are set aside in front of slab it_half
  constexpr bool kHalves = SumHalves<EP>::value && KS == 1;
  const int it_half = (kHalves && K % (2 * BKT) == 0) ? nk / 2 : -1;
  f32x16 lo[kHalves ? MT : 1][kHalves ? NT : 1];
#define CFDETR_SET_ASIDE(it_)                                                  \
  if (kHalves && (it_) == it_half) {                                           \
    _Pragma("unroll") for (int i = 0; i < MT; ++i)                             \
    _Pragma("unroll") for (int j = 0; j < NT; ++j)                             \
    _Pragma("unroll") for (int r = 0; r < 16; ++r) {                           \
      lo[kHalves ? i : 0][kHalves ? j : 0][r] = acc[i][j][r];                  \
      acc[i][j][r] = 0.f;                                                      \
    }                                                                          \
  }

  // What the epilogue needs per row and per column is requested now and arrives while
  // the main loop runs.  Result layout (transposed product): lane -> row l32 of each
  // 32-row tile, register r -> column 8*(r/4) + 4*g + (r%4) of each 32-column tile.
  int32_t info[MT];
  float4 bias_r[NT][4];
#pragma unroll
  for (int i = 0; i < MT; ++i) info[i] = ep.row_info(min(m0 + wm * WTM + i * 32 + l32, M - 1));
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int q = 0; q < 4; ++q) bias_r[j][q] = ep.bias4(n0 + wn * WTN + j * 32 + 8 * q + 4 * g);

  // K-slabs run through a ring of kStages buffers with kStages-1 slabs in flight: a slab
  // takes its transfer time plus the memory latency to arrive, which is more than one
  // slab of MFMA work, so a ring of two would wait on every slab.  The loads are issued
  // in a form the compiler does not track, so the only waits are the explicit ones: vmcnt
  // for the oldest slab, then a bare barrier that publishes it and retires every
  // wavefront's reads of the buffer the next issue overwrites.
#define CFDETR_ISSUE_SLAB(k0_, buf_)                                                          \
  do {                                                                                        \
    const unsigned char* ab_ = arows.base() + arows.slab_off(kbase + (k0_));                  \
    const unsigned char* wb_ =                                                                \
        reinterpret_cast<const unsigned char*>(W) + (size_t)(kbase + (k0_)) * 2;              \
    const uint32_t st_ = lds0 + (buf_) * STAGE;                                               \
    _Pragma("unroll") for (int j = 0; j < A_INST; ++j)                                        \
        dma16_untracked_s(ab_, avo[j], st_ + (wave * A_INST + j) * 1024);                     \
    _Pragma("unroll") for (int j = 0; j < B_INST; ++j)                                        \
        dma16_untracked_s(wb_, wvo[j], st_ + BM * ROWB + (wave * B_INST + j) * 1024);         \
  } while (0)

#pragma unroll
  for (int s = 0; s < kStages - 1; ++s)
    if (s < nk) CFDETR_ISSUE_SLAB(s * BKT, s);
  int buf = 0;   // ring position of slab `it`
  constexpr bool kChain = MT * NT == 1 && kStages == 4 && BKT == 64;
  if constexpr (kChain) {
    // A wavefront with a single 32x32 tile (small problems: a workgroup per CU, one
    // wavefront per SIMD) has four dependent MFMAs per slab and nothing to run beside
    // them, so the slab's operand reads, its MFMAs and the barrier would simply add up.
    // Here the operands of slab it + 1 are read while the MFMAs of slab it run (two sets
    // of operand registers, the loop unrolled twice so that they never move): slab it + 1
    // has landed and is published by the barrier of step it, slab it + 2 is in flight,
    // and the load issued in step it overwrites slab it - 1, which every wavefront has
    // consumed before it reaches that barrier.
    const int ra = wm * WTM + l32, rb = wn * WTN + l32;
    uint32_t oa[4], ob[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int c = 2 * ks + g;
      oa[ks] = ra * ROWB + ((c ^ lds_row_key<ROWB>(ra)) << 4);
      ob[ks] = BM * ROWB + rb * ROWB + ((c ^ lds_row_key<ROWB>(rb)) << 4);
    }
    bf16x8 fa0[4], fb0[4], fa1[4], fb1[4];
    auto read_slab = [&](int b, bf16x8(&fa)[4], bf16x8(&fb)[4]) {
      const unsigned char* p = ring + b * STAGE;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        fa[ks] = *reinterpret_cast<const bf16x8*>(p + oa[ks]);
        fb[ks] = *reinterpret_cast<const bf16x8*>(p + ob[ks]);
      }
    };
    auto step = [&](int it, bf16x8(&ca)[4], bf16x8(&cb)[4], bf16x8(&na)[4], bf16x8(&nb)[4]) {
      CFDETR_SET_ASIDE(it)
      if (it + 2 < nk)
        __builtin_amdgcn_s_waitcnt(0x0F70 | (LPW & 15) | ((LPW >> 4) << 14));
      else
        __builtin_amdgcn_s_waitcnt(0x0F70);
      __builtin_amdgcn_s_barrier();
      if (it + 3 < nk) CFDETR_ISSUE_SLAB((it + 3) * BKT, (it + 3) & 3);
      // each MFMA is followed by two of the next slab's reads: the reads are issued while
      // the MFMA before them runs, and the one wait for operands (ahead of the first MFMA)
      // finds only reads that are a whole step old
      // (behind the last slab they read a buffer that holds nothing new: never used)
      const unsigned char* p = ring + ((it + 1) & 3) * STAGE;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cb[ks], ca[ks], acc[0][0], 0, 0, 0);
        na[ks] = *reinterpret_cast<const bf16x8*>(p + oa[ks]);
        nb[ks] = *reinterpret_cast<const bf16x8*>(p + ob[ks]);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    };
    if (nk >= 3)
      __builtin_amdgcn_s_waitcnt(0x0F70 | ((2 * LPW) & 15) | (((2 * LPW) >> 4) << 14));
    else if (nk == 2)
      __builtin_amdgcn_s_waitcnt(0x0F70 | (LPW & 15) | ((LPW >> 4) << 14));
    else
      __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_s_barrier();
    read_slab(0, fa0, fb0);
    for (int it = 0; it < nk; it += 2) {
      step(it, fa0, fb0, fa1, fb1);
      if (it + 1 < nk) step(it + 1, fa1, fb1, fa0, fb0);
    }
  }
  if constexpr (KS == 2) {
    // the second group's sums cross through its ring (free now), register by register
    __syncthreads();
    float* const xs = reinterpret_cast<float*>(smem_direct + kStages * STAGE) + wave * (16 * 64) + lane;
    if (grp == 1) {
#pragma unroll
      for (int r = 0; r < 16; ++r) xs[r * 64] = acc[0][0][r];
    }
    __syncthreads();
    if (grp == 1) return;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][0][r] += xs[r * 64];
  }
  for (int it = 0; !kChain && it < nk; ++it) {
    CFDETR_SET_ASIDE(it)
    const int ahead = min(kStages - 2, nk - 1 - it);   // later slabs that may stay in flight
    if (kStages == 4 && ahead >= 2)
      __builtin_amdgcn_s_waitcnt(0x0F70 | ((2 * LPW) & 15) | (((2 * LPW) >> 4) << 14));
    else if (kStages >= 3 && ahead >= 1)
      __builtin_amdgcn_s_waitcnt(0x0F70 | (LPW & 15) | ((LPW >> 4) << 14));
    else
      __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_s_barrier();
    if (it + kStages - 1 < nk) {
      const int nb = buf == 0 ? kStages - 1 : buf - 1;   // (buf + kStages - 1) % kStages
      CFDETR_ISSUE_SLAB((it + kStages - 1) * BKT, nb);
    }
    const unsigned char* pa = smem_direct + buf * STAGE;
    const unsigned char* pb = pa + BM * ROWB;
    buf = buf + 1 == kStages ? 0 : buf + 1;
    // Operands of 16 k at a time, two sets of registers: the reads of the next 16 k are
    // issued between the MFMAs of the current ones, one read behind each MFMA, so that the
    // wavefront's MFMAs do not stop for the LDS latency inside a slab.
    bf16x8 fa[2][MT], fb[2][NT];
    auto read_ops = [&](int ks, bf16x8(&oa)[MT], bf16x8(&ob)[NT]) {
      const int c = 2 * ks + g;  // logical 16-byte chunk of this lane's 8 k
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int r = wm * WTM + i * 32 + l32;
        oa[i] = *reinterpret_cast<const bf16x8*>(pa + r * ROWB + ((c ^ lds_row_key<ROWB>(r)) << 4));
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int r = wn * WTN + j * 32 + l32;
        ob[j] = *reinterpret_cast<const bf16x8*>(pb + r * ROWB + ((c ^ lds_row_key<ROWB>(r)) << 4));
      }
    };
    read_ops(0, fa[0], fb[0]);
    __builtin_amdgcn_sched_group_barrier(0x100, MT + NT, 0);
#pragma unroll
    for (int ks = 0; ks < BKT / 16; ++ks) {
      if (ks + 1 < BKT / 16) read_ops(ks + 1, fa[(ks + 1) & 1], fb[(ks + 1) & 1]);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks & 1][j], fa[ks & 1][i], acc[i][j], 0, 0, 0);
      if (ks + 1 < BKT / 16) {
#pragma unroll
        for (int t = 0; t < MT + NT; ++t) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, MT * NT - (MT + NT), 0);
      } else {
        __builtin_amdgcn_sched_group_barrier(0x008, MT * NT, 0);
      }
    }
  }
#undef CFDETR_ISSUE_SLAB
#undef CFDETR_SET_ASIDE
  if (kHalves && it_half >= 0) {
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          acc[i][j][r] = lo[kHalves ? i : 0][kHalves ? j : 0][r] + acc[i][j][r];
  }

  // Epilogue, one 32-row tile of the wavefront at a time.  With a row per lane a store
  // instruction would touch 32 rows with 16 bytes each; instead the finished values
  // pass through a small LDS area of the wavefront's own (the ring is free now), from
  // which rows leave as runs of 128 bytes and more, 16 bytes per lane.  LDS serves a
  // wavefront's instructions in order, so its reads see its earlier writes.
  const int nw0 = n0 + wn * WTN;
  if constexpr (EP::kStageElem > 0) {
    constexpr int ES = EP::kStageElem;                    // bytes per staged element
    constexpr int ROWBYTES = WTN * ES;
    constexpr int STRIDE = ROWBYTES + 16;   // keeps the 16-byte reads aligned; the 8-byte bf16
                                            // writes of rows r and r+16 share banks (2-way)
    constexpr int LPR = ROWBYTES / 16;                    // lanes that copy one row
    constexpr int RPC = 64 / LPR;                         // rows per copy instruction
    constexpr int NCOPY = 32 / RPC;
    static_assert(NW * 32 * STRIDE <= kStages * STAGE, "staging area exceeds the ring");
    __builtin_amdgcn_s_barrier();   // every wavefront is done reading the ring
    if (ep.staged(nw0)) {
      unsigned char* stg = smem_direct + wave * (32 * STRIDE);
      const int crow = lane / LPR, cchunk = lane % LPR;
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int mb = m0 + wm * WTM + i * 32;
        if (mb >= M) break;
        float4 xin[NCOPY];
        if (EP::kExtra) {
#pragma unroll
          for (int t = 0; t < NCOPY; ++t)
            xin[t] = ep.extra4(min(mb + t * RPC + crow, M - 1), nw0 + cchunk * (16 / ES), info[i]);
        }
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int nl = j * 32 + 8 * q + 4 * g;
            const float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                                acc[i][j][4 * q + 3]};
            ep.stage4(stg + l32 * STRIDE + nl * ES, nw0 + nl, v, bias_r[j][q]);
          }
#pragma unroll
        for (int t = 0; t < NCOPY; ++t) {
          const int row = t * RPC + crow;
          const uint4 d = *reinterpret_cast<const uint4*>(stg + row * STRIDE + cchunk * 16);
          if (mb + row < M) ep.copy16(mb + row, nw0 + cchunk * (16 / ES), d, xin[t]);
        }
      }
      return;
    }
  }
  // direct form: the per-element addends of the tile in one batch, then its stores
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int m = m0 + wm * WTM + i * 32 + l32;
    if (m >= M || !ep.row_ok(info[i])) continue;
    float4 extra[NT][4];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        extra[j][q] = ep.extra4(m, n0 + wn * WTN + j * 32 + 8 * q + 4 * g, info[i]);
#pragma unroll
    for (int j = 0; j < NT; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn * WTN + j * 32 + 8 * q + 4 * g;
        const float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                            acc[i][j][4 * q + 3]};
        ep.store4(m, n, v, bias_r[j][q], extra[j][q], info[i]);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// The same contraction for the layer matrices at large row counts, as a kernel whose
// workgroups stay: the grid is what the chip holds at once and workgroup w walks over the
// tiles w, w + grid, w + 2 grid, ... of the XCD-grouped order.  What a tile costs besides
// its main loop is thereby paid once per workgroup (the row count from device memory) or
// hidden: together with a tile's last slab being worked on, the first slab of the next tile
// is requested into the free ring buffer; it is waited for before the epilogue's stores are
// issued (the wait counter is in order: behind them the wait would last until they are
// done), so the next tile starts computing at once and its second slab comes in behind the
// stores.  The epilogue's staging area is the other ring buffer.  A staging row is 128
// bytes (64 bf16 or 32 fp32 columns, the latter in two passes per 64 columns), so the area
// of all wavefronts fits one buffer.
// K is contracted in ascending slabs of BKT by every tile shape, so a result does not
// depend on the tile that produced it.
// ---------------------------------------------------------------------------
template <int BM, int BN, int NWM, int NWN, int BKT, typename EP, int WPE = 1>
__global__ __launch_bounds__(64 * NWM * NWN, WPE) void gemm_bf16_persist_kernel(
    DenseRows arows, const bf16_t* __restrict__ W, int N, int K, EP ep,
    const int32_t* __restrict__ m_ptr, int m_host) {
  constexpr int kStages = 2;
  constexpr int NW = NWM * NWN;
  constexpr int WTM = BM / NWM, WTN = BN / NWN;
  constexpr int MT = WTM / 32, NT = WTN / 32;
  constexpr int ROWB = BKT * 2;
  constexpr int CPR = ROWB / 16;
  constexpr int RPI = 64 / CPR;
  constexpr int A_INST = BM / (RPI * NW), B_INST = BN / (RPI * NW);
  constexpr int STAGE = (BM + BN) * ROWB;
  static_assert(BKT == 64, "slab width");
  static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "tile / wavefront mismatch");
  static_assert(EP::kStageElem == 2 || EP::kStageElem == 4, "staged epilogues only");
  static_assert(WTN == 64, "a wavefront's tile is 64 columns wide");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_persist[];

  const int M = m_ptr ? *m_ptr : m_host;
  const int n_blocks = N / BN;
  const int total = ((M + BM - 1) / BM) * n_blocks;
  int v = blockIdx.x;
  if (v >= total) return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / NWN, wn = wave % NWN;
  const int lrow = lane / CPR, lpos = lane % CPR;
  const int l32 = lane & 31, g = lane >> 5;
  const int nk = K / BKT;
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem_persist;

  uint32_t avo[A_INST], wvo[B_INST];
  // loader offsets of the tile with first row m0_ and first column n0_
#define CFDETR_SET_TILE(m0_, n0_)                                                              \
  do {                                                                                         \
    _Pragma("unroll") for (int j = 0; j < A_INST; ++j) {                                       \
      const int rt = (wave * A_INST + j) * RPI + lrow;                                         \
      bool ok;                                                                                 \
      avo[j] = arows.row_off((m0_) + rt, M, ok) +                                              \
               arows.lane_off((lpos ^ lds_row_key<ROWB>(rt)) * 8);                             \
    }                                                                                          \
    _Pragma("unroll") for (int j = 0; j < B_INST; ++j) {                                       \
      const int rt = (wave * B_INST + j) * RPI + lrow;                                         \
      wvo[j] = ((uint32_t)((n0_) + rt) * (uint32_t)K +                                         \
                (uint32_t)((lpos ^ lds_row_key<ROWB>(rt)) * 8)) * 2u;                          \
    }                                                                                          \
  } while (0)
#define CFDETR_ISSUE_SLAB(k0_, buf_)                                                          \
  do {                                                                                        \
    const unsigned char* ab_ = arows.base() + arows.slab_off(k0_);                            \
    const unsigned char* wb_ = reinterpret_cast<const unsigned char*>(W) + (size_t)(k0_) * 2; \
    const uint32_t st_ = lds0 + (buf_) * STAGE;                                               \
    _Pragma("unroll") for (int j = 0; j < A_INST; ++j)                                        \
        dma16_untracked_s(ab_, avo[j], st_ + (wave * A_INST + j) * 1024);                     \
    _Pragma("unroll") for (int j = 0; j < B_INST; ++j)                                        \
        dma16_untracked_s(wb_, wvo[j], st_ + BM * ROWB + (wave * B_INST + j) * 1024);         \
  } while (0)

  int pid = xcd_tile_order(v, total);
  int m0 = (pid / n_blocks) * BM, n0 = (pid % n_blocks) * BN;
  CFDETR_SET_TILE(m0, n0);
  CFDETR_ISSUE_SLAB(0, 0);
  int buf = 0;                // ring buffer of the slab that is computed next
  bool first_ready = false;   // that slab is the tile's first and is in LDS already (below)

  for (;;) {
    // what the epilogue needs per row and per column arrives while the main loop runs
    int32_t info[MT];
    float4 bias_r[NT][4];
#pragma unroll
    for (int i = 0; i < MT; ++i) info[i] = ep.row_info(min(m0 + wm * WTM + i * 32 + l32, M - 1));
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) bias_r[j][q] = ep.bias4(n0 + wn * WTN + j * 32 + 8 * q + 4 * g);

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // the tile after this one: its first slab is requested behind this tile's last one
    const int vn = v + (int)gridDim.x;
    const bool more = vn < total;
    const int m0_cur = m0, n0_cur = n0;
    for (int it = 0; it < nk; ++it) {
      // a tile's first slab that came in under the previous epilogue needs no wait; the
      // barrier then only retires that epilogue's reads of its staging rows
      if (!(it == 0 && first_ready)) __builtin_amdgcn_s_waitcnt(0x0F70);
      __builtin_amdgcn_s_barrier();
      if (it + 1 < nk) {
        CFDETR_ISSUE_SLAB((it + 1) * BKT, buf ^ 1);
      } else if (more) {
        pid = xcd_tile_order(vn, total);
        m0 = (pid / n_blocks) * BM;
        n0 = (pid % n_blocks) * BN;
        CFDETR_SET_TILE(m0, n0);
        CFDETR_ISSUE_SLAB(0, buf ^ 1);
      }
      const unsigned char* pa = smem_persist + buf * STAGE;
      const unsigned char* pb = pa + BM * ROWB;
      buf ^= 1;
      bf16x8 fa[2][MT], fb[2][NT];
      auto read_ops = [&](int ks, bf16x8(&oa)[MT], bf16x8(&ob)[NT]) {
        const int c = 2 * ks + g;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
          const int r = wm * WTM + i * 32 + l32;
          oa[i] = *reinterpret_cast<const bf16x8*>(pa + r * ROWB + ((c ^ lds_row_key<ROWB>(r)) << 4));
        }
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          const int r = wn * WTN + j * 32 + l32;
          ob[j] = *reinterpret_cast<const bf16x8*>(pb + r * ROWB + ((c ^ lds_row_key<ROWB>(r)) << 4));
        }
      };
      read_ops(0, fa[0], fb[0]);
      __builtin_amdgcn_sched_group_barrier(0x100, MT + NT, 0);
#pragma unroll
      for (int ks = 0; ks < BKT / 16; ++ks) {
        if (ks + 1 < BKT / 16) read_ops(ks + 1, fa[(ks + 1) & 1], fb[(ks + 1) & 1]);
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks & 1][j], fa[ks & 1][i], acc[i][j], 0, 0, 0);
        if (ks + 1 < BKT / 16) {
#pragma unroll
          for (int t = 0; t < MT + NT; ++t) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          }
          __builtin_amdgcn_sched_group_barrier(0x008, MT * NT - (MT + NT), 0);
        } else {
          __builtin_amdgcn_sched_group_barrier(0x008, MT * NT, 0);
        }
      }
    }
    // The next tile's first slab was requested one slab ago into the buffer `buf`; it has to
    // be in LDS before the epilogue's stores are issued: the wait counter is in order, and a
    // wait for it behind them would last until they are done.  The barrier also tells that
    // every wavefront is done reading the ring; the staging rows are in the other buffer.
    if (more) __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_s_barrier();
    const int stage_buf = buf ^ 1;

    // Epilogue of the finished tile, one 32-row block of the wavefront at a time; the
    // finished values pass through the wavefront's staging rows in buffer 1, from which
    // rows leave as 128-byte runs, 16 bytes per lane.
    {
      constexpr int ES = EP::kStageElem;
      constexpr int CPP = 128 / ES;          // columns per staging pass: 64 bf16 or 32 fp32
      constexpr int NPASS = WTN / CPP;
      constexpr int STRIDE = 128 + 16;
      constexpr int NCOPY = 4;               // 8 lanes copy a row, 8 rows per instruction
      static_assert(NW * 32 * STRIDE <= STAGE, "staging area exceeds a ring buffer");
      const int nw0 = n0_cur + wn * WTN;
      if (ep.staged(nw0)) {
        unsigned char* stg = smem_persist + stage_buf * STAGE + wave * (32 * STRIDE);
        const int crow = lane >> 3, cchunk = lane & 7;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
          const int mb = m0_cur + wm * WTM + i * 32;
          if (mb >= M) break;
#pragma unroll
          for (int ps = 0; ps < NPASS; ++ps) {
            const int nc0 = nw0 + ps * CPP;   // first column of this pass
            float4 xin[NCOPY];
            if (EP::kExtra) {
#pragma unroll
              for (int t = 0; t < NCOPY; ++t)
                xin[t] = ep.extra4(min(mb + t * 8 + crow, M - 1), nc0 + cchunk * (16 / ES), info[i]);
            }
#pragma unroll
            for (int jj = 0; jj < CPP / 32; ++jj) {
              const int j = ps * (CPP / 32) + jj;
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const int nl = jj * 32 + 8 * q + 4 * g;   // column inside the pass
                const float v4[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                                     acc[i][j][4 * q + 3]};
                ep.stage4(stg + l32 * STRIDE + nl * ES, nc0 + nl, v4, bias_r[j][q]);
              }
            }
#pragma unroll
            for (int t = 0; t < NCOPY; ++t) {
              const int row = t * 8 + crow;
              const uint4 dd = *reinterpret_cast<const uint4*>(stg + row * STRIDE + cchunk * 16);
              if (mb + row < M) ep.copy16(mb + row, nc0 + cchunk * (16 / ES), dd, xin[t]);
            }
          }
        }
      } else {
        // direct form (columns that do not leave as rows): per-element stores
#pragma unroll
        for (int i = 0; i < MT; ++i) {
          const int m = m0_cur + wm * WTM + i * 32 + l32;
          if (m >= M || !ep.row_ok(info[i])) continue;
#pragma unroll
          for (int j = 0; j < NT; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int n = nw0 + j * 32 + 8 * q + 4 * g;
              const float v4[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                                   acc[i][j][4 * q + 3]};
              ep.store4(m, n, v4, bias_r[j][q], ep.extra4(m, n, info[i]), info[i]);
            }
          }
        }
      }
    }
    if (!more) break;
    v = vn;
    first_ready = true;
  }
#undef CFDETR_SET_TILE
#undef CFDETR_ISSUE_SLAB
}

// Sum over each group of 16 consecutive lanes, delivered to all 16 (quad swaps, then the
// mirror of each half-row and of the row: a fixed order, no LDS).
__device__ __forceinline__ float row16_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true));
  return v;
}

// ---------------------------------------------------------------------------
// Residual contraction + LayerNorm of the new residual rows in one kernel.
// ---------------------------------------------------------------------------
// x[m, :] += A[m, :] . W^T + bias;  out[m, :] = LayerNorm(x[m, :]) * g + b.
// A workgroup owns BM complete rows (all D = N output columns), so the row statistics
// are at hand in the epilogue.  The accumulators (a row per lane) first pass through a
// per-wavefront LDS area and come back with 16 lanes per row and four consecutive
// columns per lane: in that form the old residual is read, the new one and the
// normalised row are written as runs of 128-256 bytes, a row's sum is a 16-lane
// reduction plus one pass through LDS across the four wavefronts (wavefront w owns
// columns [w*D/4, (w+1)*D/4)), and bias, gain and offset are one float4 each per lane.
// Mean first, then the variance of the centred values, like the stand-alone kernel.
//
// Few rows per workgroup means one workgroup per CU and one wavefront per SIMD, so
// latency is hidden by depth instead of occupancy: K-slabs of 64 run through a ring of
// kStages (3 or 4) LDS buffers (one static array each, which lets the compiler see that the
// slab being filled is not the slab being read), with kStages-1 slabs in flight, an
// explicit vmcnt wait for the oldest one and a bare barrier per slab.
template <int BM, int D, int kStages, bool kOutBf16>
__global__ __launch_bounds__(256) void gemm_bf16_rowln_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, int K,
    const float* __restrict__ bias, float* __restrict__ resid, const float* __restrict__ ln_g,
    const float* __restrict__ ln_b, float eps, void* __restrict__ out, int split_row,
    void* __restrict__ out2, const int32_t* __restrict__ m_ptr, int m_host) {
  constexpr int MT = BM / 32;                  // 32-row MFMA tiles per wavefront
  constexpr int WTN = D / 4, NT = WTN / 32;    // columns per wavefront, 32-column tiles
  constexpr int A_INST = BM / 32, B_INST = D / 32;   // 1 KB load instructions per wavefront
  constexpr int LPW = A_INST + B_INST;         // loads a wavefront issues per slab
  static_assert(BM % 32 == 0 && D % 128 == 0, "tile shape");   // 32 columns per MFMA tile, 4 wavefronts
  static_assert(kStages == 3 || kStages == 4, "ring of 3 or 4 buffers");
  static_assert((kStages - 2) * LPW < 64, "vmcnt is a 6-bit counter");
  __shared__ __attribute__((aligned(1024))) unsigned char sA0[BM * 128], sA1[BM * 128],
      sA2[BM * 128], sA3[BM * 128];
  __shared__ __attribute__((aligned(1024))) unsigned char sB0[D * 128], sB1[D * 128],
      sB2[D * 128], sB3[D * 128];
  __shared__ __attribute__((aligned(16))) float s_red[2][BM][4];   // [pass][row][wavefront]
#define CFDETR_RING(arr_, s_) ((s_) == 0 ? arr_##0 : (s_) == 1 ? arr_##1 : (s_) == 2 ? arr_##2 : arr_##3)

  const int M = m_ptr ? *m_ptr : m_host;
  const int total = (M + BM - 1) / BM;
  if ((int)blockIdx.x >= total) return;   // surplus workgroup: the grid covers the capacity
  // same workgroup -> XCD -> row range map as the contraction that produced A: its rows
  // are then still in this XCD's L2
  const int m0 = xcd_tile_order(blockIdx.x, total) * BM;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int lrow = lane >> 3, lpos = lane & 7;
  const bf16_t* ag[A_INST];
  const bf16_t* wg[B_INST];
#pragma unroll
  for (int j = 0; j < A_INST; ++j) {
    const int rt = (wave * A_INST + j) * 8 + lrow;
    const int r = min(m0 + rt, M - 1);   // rows past M: any valid row, never stored
    ag[j] = A + (size_t)r * K + (lpos ^ ((rt >> 1) & 7)) * 8;
  }
#pragma unroll
  for (int j = 0; j < B_INST; ++j) {
    const int rt = (wave * B_INST + j) * 8 + lrow;
    wg[j] = W + (size_t)rt * K + (lpos ^ ((rt >> 1) & 7)) * 8;
  }

#define CFDETR_ISSUE_RING(k0_, s_)                                                            \
  do {                                                                                        \
    _Pragma("unroll") for (int j = 0; j < A_INST; ++j)                                        \
        dma16_untracked(ag[j] + (k0_), CFDETR_RING(sA, s_) + (wave * A_INST + j) * 1024);     \
    _Pragma("unroll") for (int j = 0; j < B_INST; ++j)                                        \
        dma16_untracked(wg[j] + (k0_), CFDETR_RING(sB, s_) + (wave * B_INST + j) * 1024);     \
  } while (0)

  const int nk = K / BK;
#pragma unroll
  for (int s = 0; s < kStages - 1; ++s)
    if (s < nk) CFDETR_ISSUE_RING(s * BK, s);

  // Everything the epilogue reads is requested now and arrives during the main loop, in
  // the epilogue's own layout: lane -> row crow (+ RPC per step) of a 32-row tile and
  // columns cn .. cn+3 of the wavefront's WTN.
  constexpr int LPR = WTN / 4;          // lanes per row (4 columns each); 16 for D = 256
  constexpr int RPC = 64 / LPR;         // rows per step
  constexpr int NSTEP = 32 / RPC;
  static_assert(LPR == 16, "the row sums assume 16 lanes per row");
  const int crow = lane / LPR, cn = wave * WTN + (lane % LPR) * 4;
  const float4 bias4 = *reinterpret_cast<const float4*>(bias + cn);
  const float4 gain4 = *reinterpret_cast<const float4*>(ln_g + cn);
  const float4 offs4 = *reinterpret_cast<const float4*>(ln_b + cn);
  float4 xin[MT][NSTEP];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int t = 0; t < NSTEP; ++t)
      xin[i][t] = *reinterpret_cast<const float4*>(
          resid + (size_t)min(m0 + i * 32 + t * RPC + crow, M - 1) * D + cn);

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  for (int it0 = 0; it0 < nk; it0 += kStages) {
#pragma unroll
    for (int b = 0; b < kStages; ++b) {   // ring position: a constant after unrolling
      const int it = it0 + b;
      if (it >= nk) break;
      // Slabs issued after slab `it` and still allowed in flight: up to kStages-2.
      const int ahead = min(kStages - 2, nk - 1 - it);
      if (kStages == 4 && ahead >= 2)
        __builtin_amdgcn_s_waitcnt(0x0F70 | ((2 * LPW) & 15) | (((2 * LPW) >> 4) << 14));
      else if (ahead == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | (LPW & 15) | ((LPW >> 4) << 14));
      else __builtin_amdgcn_s_waitcnt(0x0F70);
      // Everybody's part of slab `it` is in LDS, and everybody is done reading the
      // buffer that the next issue overwrites (it was read in the previous step).
      __builtin_amdgcn_s_barrier();
      if (it + kStages - 1 < nk)
        CFDETR_ISSUE_RING((it + kStages - 1) * BK, (b + kStages - 1) % kStages);
      const unsigned char* pa = CFDETR_RING(sA, b);
      const unsigned char* pb = CFDETR_RING(sB, b);
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        const int c = 2 * ks + g;
        bf16x8 fa[MT], fb[NT];
#pragma unroll
        for (int i = 0; i < MT; ++i) {
          const int r = i * 32 + l32;
          fa[i] = *reinterpret_cast<const bf16x8*>(pa + r * 128 + ((c ^ ((r >> 1) & 7)) << 4));
        }
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          const int r = wave * WTN + j * 32 + l32;
          fb[j] = *reinterpret_cast<const bf16x8*>(pb + r * 128 + ((c ^ ((r >> 1) & 7)) << 4));
        }
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
      }
    }
  }
#undef CFDETR_ISSUE_RING
#undef CFDETR_RING
  // Epilogue.  Accumulators -> LDS (lane = row l32, register r of tile j = column
  // 32*j + 8*(r/4) + 4*g + r%4 of the wavefront's WTN) -> back with 16 lanes per row.
  // The area is the wavefront's own and LDS serves its instructions in order; the ring it
  // overlays is free once every wavefront has passed the barrier.
  constexpr int STRIDE = WTN * 4 + 16;   // bytes; rows 16 bytes apart in bank space
  static_assert(2 * 32 * STRIDE <= (int)sizeof(sB0), "staging area exceeds a ring buffer");
  __builtin_amdgcn_s_barrier();
  unsigned char* stg = (wave < 2 ? sB0 : sB1) + (wave & 1) * (32 * STRIDE);
  float4 v[MT][NSTEP];
#pragma unroll
  for (int i = 0; i < MT; ++i) {
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(stg + l32 * STRIDE + (j * 32 + 8 * q + 4 * g) * 4) =
            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                        acc[i][j][4 * q + 3]);
#pragma unroll
    for (int t = 0; t < NSTEP; ++t) {
      const int row = t * RPC + crow;
      const float4 a4 = *reinterpret_cast<const float4*>(stg + row * STRIDE + (lane % LPR) * 16);
      float4 r;
      r.x = a4.x + bias4.x + xin[i][t].x;
      r.y = a4.y + bias4.y + xin[i][t].y;
      r.z = a4.z + bias4.z + xin[i][t].z;
      r.w = a4.w + bias4.w + xin[i][t].w;
      v[i][t] = r;
      const int m = m0 + i * 32 + row;
      if (m < M) *reinterpret_cast<float4*>(resid + (size_t)m * D + cn) = r;
      const float part = row16_sum((r.x + r.y) + (r.z + r.w));
      if (lane % LPR == 0) s_red[0][i * 32 + row][wave] = part;
    }
  }
  __syncthreads();
  float mean[MT][NSTEP];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int t = 0; t < NSTEP; ++t) {
      const int row = i * 32 + t * RPC + crow;
      const float4 p = *reinterpret_cast<const float4*>(&s_red[0][row][0]);
      mean[i][t] = ((p.x + p.y) + (p.z + p.w)) * (1.0f / (float)D);
      const float cx = v[i][t].x - mean[i][t], cy = v[i][t].y - mean[i][t];
      const float cz = v[i][t].z - mean[i][t], cw = v[i][t].w - mean[i][t];
      const float part = row16_sum(fmaf(cx, cx, cy * cy) + fmaf(cz, cz, cw * cw));
      if (lane % LPR == 0) s_red[1][row][wave] = part;
    }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int t = 0; t < NSTEP; ++t) {
      const int row = i * 32 + t * RPC + crow;
      const int m = m0 + row;
      if (m >= M) continue;
      const float4 p = *reinterpret_cast<const float4*>(&s_red[1][row][0]);
      const float rstd = rsqrtf(((p.x + p.y) + (p.z + p.w)) * (1.0f / (float)D) + eps);
      const float r0 = (v[i][t].x - mean[i][t]) * rstd * gain4.x + offs4.x;
      const float r1 = (v[i][t].y - mean[i][t]) * rstd * gain4.y + offs4.y;
      const float r2 = (v[i][t].z - mean[i][t]) * rstd * gain4.z + offs4.z;
      const float r3 = (v[i][t].w - mean[i][t]) * rstd * gain4.w + offs4.w;
      const bool second = out2 != nullptr && m >= split_row;
      const size_t at = (size_t)(second ? m - split_row : m) * D + cn;
      void* obase = second ? out2 : out;
      if (kOutBf16)
        *reinterpret_cast<uint2*>(static_cast<bf16_t*>(obase) + at) =
            make_uint2(pack_bf16x2(r0, r1), pack_bf16x2(r2, r3));
      else
        *reinterpret_cast<float4*>(static_cast<float*>(obase) + at) = make_float4(r0, r1, r2, r3);
    }
}

// Phase time stamps of layer_tail_kernel for a development harness that defines these
// macros before including this file; compiled out otherwise.
#ifndef CFDETR_TL
#define CFDETR_TL(i)
#define CFDETR_TLX(i)
#endif

// The weights that layer_tail_kernel streams, in its order and layout: 1 KB blocks, each
// the 64 x 16 bytes that one 32x32x16 MFMA of one wavefront takes as its weight operand
// (lane (l32, g) holds 8 consecutive k of weight row l32), 16 blocks per wavefront and
// group, 8 wavefronts per group of 128 KB.  Block i of wavefront w in group c:
//   c = 0: the output projection: Wo[32 w + l32][16 i + 8 g ..];
//   c = 1 .. F/128: chunk c - 1 of 128 hidden units.  Wavefronts 0-3 produce the hidden
//     chunk: W1[128 (c-1) + 32 w + l32][16 i + 8 g ..].  Wavefronts 4-7 consume it, each
//     for 64 output columns as two tiles: W2[64 (w-4) + 32 (i % 2) + l32][128 (c-1) + 16 (i / 2) + 8 g ..];
//   c = F/128 + 1 .. + 3: the next layer's query/key/value projection, 48 blocks per
//     wavefront: block b = 16 (c - F/128 - 1) + i is k-step b / 3 of the wavefront's column
//     tile b % 3: Wqkv[96 w + 32 (b % 3) + l32][16 (b / 3) + 8 g ..]; skipped when Wqkv is
//     null.
// One thread per 16 bytes.
__global__ __launch_bounds__(256) void layer_tail_pack_kernel(const bf16_t* __restrict__ Wo,
                                                              const bf16_t* __restrict__ W1,
                                                              const bf16_t* __restrict__ W2,
                                                              const bf16_t* __restrict__ Wqkv,
                                                              int F, bf16_t* __restrict__ out) {
  constexpr int D = 256, FC = 128;
  const int u = blockIdx.x * blockDim.x + threadIdx.x;   // 16-byte unit of the output
  if (u >= (4 * D * D + F * D * 2) / 8) return;
  const int lane = u & 63, i = (u >> 6) & 15, w = (u >> 10) & 7, c = u >> 13;
  const int l32 = lane & 31, g = lane >> 5;
  const int nchunk = F / FC;
  const bf16_t* src;
  if (c == 0) {
    src = Wo + (size_t)(w * 32 + l32) * D + i * 16 + g * 8;
  } else if (c <= nchunk) {
    if (w < 4)
      src = W1 + (size_t)((c - 1) * FC + w * 32 + l32) * D + i * 16 + g * 8;
    else
      src = W2 + (size_t)((w - 4) * 64 + (i & 1) * 32 + l32) * F + (c - 1) * FC + (i >> 1) * 16 + g * 8;
  } else {
    if (Wqkv == nullptr) return;
    const int b = 16 * (c - nchunk - 1) + i;
    src = Wqkv + (size_t)(w * 96 + (b % 3) * 32 + l32) * D + (b / 3) * 16 + g * 8;
  }
  reinterpret_cast<uint4*>(out)[u] = *reinterpret_cast<const uint4*>(src);
}

// The first layer's q/k/v projection in the same layout (three groups of 128 KB), for
// layer_head_kernel.
__global__ __launch_bounds__(256) void layer_head_pack_kernel(const bf16_t* __restrict__ Wqkv,
                                                              bf16_t* __restrict__ out) {
  constexpr int D = 256;
  const int u = blockIdx.x * blockDim.x + threadIdx.x;   // 16-byte unit of the output
  if (u >= 3 * D * D / 8) return;
  const int lane = u & 63, i = (u >> 6) & 15, w = (u >> 10) & 7, b = (u >> 13) * 16 + i;
  reinterpret_cast<uint4*>(out)[u] = *reinterpret_cast<const uint4*>(
      Wqkv + (size_t)(w * 96 + (b % 3) * 32 + (lane & 31)) * D + (b / 3) * 16 + (lane >> 5) * 8);
}

// Two 256 x 256 matrices (an output projection and the projection behind the LayerNorm
// that follows it) in the layout of group 0 above, 128 KB each, for layer_mid_kernel.
__global__ __launch_bounds__(256) void layer_mid_pack_kernel(const bf16_t* __restrict__ Wo,
                                                             const bf16_t* __restrict__ Wq,
                                                             bf16_t* __restrict__ out) {
  constexpr int D = 256;
  const int u = blockIdx.x * blockDim.x + threadIdx.x;   // 16-byte unit of the output
  if (u >= 2 * D * D / 8) return;
  const int lane = u & 63, i = (u >> 6) & 15, w = (u >> 10) & 7, c = u >> 13;
  const bf16_t* src = c == 0 ? Wo : Wq;
  reinterpret_cast<uint4*>(out)[u] = *reinterpret_cast<const uint4*>(
      src + (size_t)(32 * w + (lane & 31)) * D + 16 * i + 8 * (lane >> 5));
}

// Sum over each group of 8 consecutive lanes, delivered to all 8.
__device__ __forceinline__ float row8_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));
  return v;
}

// Rows of layer_tail_kernel and layer_head_kernel live spread over 8 lanes, four
// consecutive columns per lane: a lane of wavefront w holds columns 32 w + 4 (lane % 8) ..
// of rows 8 t + lane / 8, t = 0..3.  A 32 x 32 accumulator tile (lane (l32, g), register
// r = row l32, column 8 (r / 4) + 4 g + r % 4) gets into that form through a 4.5 KB LDS
// area: tail_tile_put writes the tile, tail_rows_take reads it back as v = tile + bias + xin.
constexpr int kTailStride = 32 * 4 + 16;   // bytes of a staging row

__device__ __forceinline__ void tail_tile_put(const f32x16& acc, unsigned char* stg, int lane) {
  const int l32 = lane & 31, g = lane >> 5;
#pragma unroll
  for (int q = 0; q < 4; ++q)
    *reinterpret_cast<float4*>(stg + l32 * kTailStride + (8 * q + 4 * g) * 4) =
        make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
}

__device__ __forceinline__ void tail_rows_take(const unsigned char* stg, const float4& bias4,
                                               const float4 (&xin)[4], int lane, float4 (&v)[4]) {
  const int crow = lane >> 3, lp = lane & 7;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const float4 a4 = *reinterpret_cast<const float4*>(stg + (t * 8 + crow) * kTailStride + lp * 16);
    v[t].x = a4.x + bias4.x + xin[t].x;
    v[t].y = a4.y + bias4.y + xin[t].y;
    v[t].z = a4.z + bias4.z + xin[t].z;
    v[t].w = a4.w + bias4.w + xin[t].w;
  }
}

// tail_rows_stats: mean and 1/sigma of the complete 256-wide rows.  Every wavefront has
// 32 columns of a row (8 lanes x 4): it takes their sum and the sum of squares around
// their own mean (two 8-lane reductions), the eight pairs meet in LDS, and the row's mean
// and variance follow from them (the sum of squares around the common mean is the sum of
// the partial ones plus 32 (mean_w - mean)^2 for each part): as exact as centring on the
// row's mean first, with one barrier instead of two.  All 512 threads must call it.
__device__ __forceinline__ void tail_rows_stats(const float4 (&v)[4], float (*s_red)[32][8],
                                                int wave, int lane, float eps, float (&mean)[4],
                                                float (&rstd)[4]) {
  const int crow = lane >> 3, lp = lane & 7;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const float part = row8_sum((v[t].x + v[t].y) + (v[t].z + v[t].w));
    const float mw = part * (1.0f / 32.0f);
    const float cx = v[t].x - mw, cy = v[t].y - mw, cz = v[t].z - mw, cw = v[t].w - mw;
    const float sq = row8_sum(fmaf(cx, cx, cy * cy) + fmaf(cz, cz, cw * cw));
    if (lp == 0) {
      s_red[0][t * 8 + crow][wave] = part;
      s_red[1][t * 8 + crow][wave] = sq;
    }
  }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int row = t * 8 + crow;
    const float4 p0 = *reinterpret_cast<const float4*>(&s_red[0][row][0]);
    const float4 p1 = *reinterpret_cast<const float4*>(&s_red[0][row][4]);
    const float4 q0 = *reinterpret_cast<const float4*>(&s_red[1][row][0]);
    const float4 q1 = *reinterpret_cast<const float4*>(&s_red[1][row][4]);
    mean[t] = (((p0.x + p0.y) + (p0.z + p0.w)) + ((p1.x + p1.y) + (p1.z + p1.w))) * (1.0f / 256.0f);
    const float m32 = mean[t] * 32.0f;   // a part's sum if it had the row's mean
    const float d0 = p0.x - m32, d1 = p0.y - m32, d2 = p0.z - m32, d3 = p0.w - m32;
    const float d4 = p1.x - m32, d5 = p1.y - m32, d6 = p1.z - m32, d7 = p1.w - m32;
    const float within = ((q0.x + q0.y) + (q0.z + q0.w)) + ((q1.x + q1.y) + (q1.z + q1.w));
    const float between = (fmaf(d0, d0, d1 * d1) + fmaf(d2, d2, d3 * d3)) +
                          (fmaf(d4, d4, d5 * d5) + fmaf(d6, d6, d7 * d7));
    const float var = fmaf(between, 1.0f / 32.0f, within) * (1.0f / 256.0f);
    rstd[t] = rsqrtf(var + eps);
  }
}

// Normalised rows (v - mean) * rstd * gain + offs of this lane, as bf16 into the
// operand buffer sA: 512 bytes a row, 16-byte chunks swizzled with the row.
__device__ __forceinline__ void tail_rows_to_operand(const float4 (&v)[4], const float (&mean)[4],
                                                     const float (&rstd)[4], const float4& gain4,
                                                     const float4& offs4, unsigned char* sA,
                                                     int wave, int lane) {
  const int crow = lane >> 3, lp = lane & 7;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int row = t * 8 + crow;
    const float r0 = (v[t].x - mean[t]) * rstd[t] * gain4.x + offs4.x;
    const float r1 = (v[t].y - mean[t]) * rstd[t] * gain4.y + offs4.y;
    const float r2 = (v[t].z - mean[t]) * rstd[t] * gain4.z + offs4.z;
    const float r3 = (v[t].w - mean[t]) * rstd[t] * gain4.w + offs4.w;
    const int idx = wave * 4 + (lp >> 1);
    *reinterpret_cast<uint2*>(sA + row * 512 + (((idx & ~7) | ((idx ^ row) & 7)) << 4) + (lp & 1) * 8) =
        make_uint2(pack_bf16x2(r0, r1), pack_bf16x2(r2, r3));
  }
}

// The 32 rows in sA as operand of sixteen 32x32x16 MFMAs: lane (l32, g) gets elements
// 16 ks + 8 g .. of row l32.
__device__ __forceinline__ void tail_operand_load(const unsigned char* sA, int lane,
                                                  bf16x8 (&a)[16]) {
  const int l32 = lane & 31, g = lane >> 5;
#pragma unroll
  for (int ks = 0; ks < 16; ++ks) {
    const int idx = 2 * ks + g;
    a[ks] = *reinterpret_cast<const bf16x8*>(sA + l32 * 512 + (((idx & ~7) | ((idx ^ l32) & 7)) << 4));
  }
}

// Where the q/k/v projection of layer_tail_kernel and layer_head_kernel writes.
struct TailQkv {
  const float* bias;   // [768]
  float q_scale;
  bf16_t* qk;
  bf16_t* vt;
  int vt_ld;
  const int32_t* cu;
  const int32_t* pcu;
  int B;
};

// The q/k/v projection of the 32 rows in sA (bf16, as tail_rows_to_operand leaves them;
// the caller has passed a barrier since): q (multiplied by q_scale) and k go to
// qk [M, 768] in bf16, v feature-major to vt (position pcu[f] + m - cu[f] of its frame
// f), as the stand-alone projection writes them.  Wavefront w owns columns 96 w ..
// 96 w + 95 as three 32-column tiles.  Its 48 weight blocks of 1 KB (block b = k-step
// b / 3 of tile b % 3, see layer_tail_pack_kernel) lie at qsrc + (b / 16) * 128 KB +
// (b % 16) * 1 KB + voff; the first 16 are in wreg already, and each register takes
// block b + 16 as soon as block b has been used.
// Start values of the three accumulator tiles of tail_project_qkv: the bias of the columns
// a lane holds (register r of lane group g: column 8 (r / 4) + 4 g + r % 4 of the tile), and
// the position of the lane's row in the feature-major copy of v.  Both are loads from global
// memory: a caller asks for them well before the projection, so that they have arrived.
__device__ __forceinline__ void tail_qkv_prepare(const TailQkv& qkv, int m0, int M, int wave,
                                                 int lane, f32x16 (&pacc)[3], int& vpos) {
  const int l32 = lane & 31, g = lane >> 5;
#pragma unroll
  for (int j = 0; j < 3; ++j)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 b4 = *reinterpret_cast<const float4*>(qkv.bias + wave * 96 + j * 32 + 8 * q + 4 * g);
      pacc[j][4 * q] = b4.x;
      pacc[j][4 * q + 1] = b4.y;
      pacc[j][4 * q + 2] = b4.z;
      pacc[j][4 * q + 3] = b4.w;
    }
  const int mrow = m0 + l32;
  vpos = 0;
  if (mrow < M && wave * 96 + 95 >= 512) {   // only wavefronts with v columns need it
    const int f = frame_of_token(qkv.cu, qkv.B, mrow);
    vpos = qkv.pcu[f] + (mrow - qkv.cu[f]);
  }
}

__device__ __forceinline__ void tail_project_qkv(const unsigned char* sA, bf16x8 (&wreg)[16],
                                                 const unsigned char* qsrc, uint32_t voff,
                                                 const TailQkv& qkv, unsigned char* stg, int m0,
                                                 int M, int wave, int lane, f32x16 (&pacc)[3],
                                                 int vpos) {
  constexpr int D = 256;
  const int l32 = lane & 31, g = lane >> 5, crow = lane >> 3, lp = lane & 7;
  bf16x8 qreg[16];
  tail_operand_load(sA, lane, qreg);
#pragma unroll
  for (int b = 0; b < 48; ++b) {
    pacc[b % 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[b & 15], qreg[b / 3], pacc[b % 3], 0, 0, 0);
    if (b + 16 < 48)
      wreg[b & 15] = *reinterpret_cast<const bf16x8*>(qsrc + (size_t)((b + 16) >> 4) * 131072 +
                                                      (b & 15) * 1024 + voff);
  }
  const int mrow = m0 + l32;
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const int n0 = wave * 96 + j * 32;   // 32 columns, all q, all k or all v
    if (n0 < 2 * D) {
      // through the wavefront's staging area: 8 lanes per row, 4 columns per lane
      tail_tile_put(pacc[j], stg, lane);
      const float sc = n0 < D ? qkv.q_scale : 1.0f;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int row = t * 8 + crow;
        const float4 a4 = *reinterpret_cast<const float4*>(stg + row * kTailStride + lp * 16);
        if (m0 + row < M)
          *reinterpret_cast<uint2*>(qkv.qk + (size_t)(m0 + row) * (3 * D) + n0 + lp * 4) =
              make_uint2(pack_bf16x2(a4.x * sc, a4.y * sc), pack_bf16x2(a4.z * sc, a4.w * sc));
      }
    } else if (mrow < M) {
      // a token per lane: the feature-major stores are runs of 32 consecutive positions
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + 8 * q + 4 * g;
        bf16_t* p = qkv.vt + (size_t)(n - 2 * D) * qkv.vt_ld + vpos;
        p[0] = f32_to_bf16(pacc[j][4 * q]);
        p[(size_t)qkv.vt_ld] = f32_to_bf16(pacc[j][4 * q + 1]);
        p[(size_t)2 * qkv.vt_ld] = f32_to_bf16(pacc[j][4 * q + 2]);
        p[(size_t)3 * qkv.vt_ld] = f32_to_bf16(pacc[j][4 * q + 3]);
      }
    }
  }
}

// LayerNorm and q/k/v projection of the first layer (width 256): the same rows-per-
// workgroup scheme as layer_tail_kernel, of which this is the last stage on its own.
// Wp: the 48 weight blocks per wavefront in the packed layout (three groups of 128 KB).
__global__ __launch_bounds__(512) void layer_head_kernel(
    const float* __restrict__ x, const bf16_t* __restrict__ Wp, const float* __restrict__ ln_g,
    const float* __restrict__ ln_b, float eps, TailQkv qkv, const int32_t* __restrict__ m_ptr,
    int m_host) {
  constexpr int D = 256, BM = 32, NW = 8;
  __shared__ __attribute__((aligned(16))) unsigned char sA[BM * D * 2];
  __shared__ __attribute__((aligned(16))) unsigned char s_stage[NW * 32 * kTailStride];
  __shared__ __attribute__((aligned(16))) float s_red[2][BM][NW];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const unsigned char* const wsrc = reinterpret_cast<const unsigned char*>(Wp) + (size_t)wave * 16384;
  const uint32_t voff = lane * 16;
  bf16x8 wreg[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) wreg[i] = *reinterpret_cast<const bf16x8*>(wsrc + i * 1024 + voff);
  const int M = m_ptr ? *m_ptr : m_host;
  const int total = (M + BM - 1) / BM;
  if ((int)blockIdx.x >= total) return;   // surplus workgroup: the grid covers the capacity
  const int m0 = xcd_tile_order(blockIdx.x, total) * BM;
  const int crow = lane >> 3, lp = lane & 7, cn = wave * 32 + lp * 4;
  const float4 gain4 = *reinterpret_cast<const float4*>(ln_g + cn);
  const float4 offs4 = *reinterpret_cast<const float4*>(ln_b + cn);
  float4 v[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
    v[t] = *reinterpret_cast<const float4*>(x + (size_t)min(m0 + t * 8 + crow, M - 1) * D + cn);
  f32x16 pacc[3];
  int vpos;
  tail_qkv_prepare(qkv, m0, M, wave, lane, pacc, vpos);
  float mean[4], rstd[4];
  tail_rows_stats(v, s_red, wave, lane, eps, mean, rstd);
  tail_rows_to_operand(v, mean, rstd, gain4, offs4, sA, wave, lane);
  __syncthreads();
  tail_project_qkv(sA, wreg, wsrc, voff, qkv, s_stage + wave * (32 * kTailStride), m0, M, wave, lane,
                   pacc, vpos);
}

// Output projection of an attention block, the LayerNorm behind it and a projection of the
// normalised rows, in one kernel (width 256; the decoder between its two attentions):
//   x[m, :] += O[m, :] . Wo^T + bo;   q[m, :] = ((LayerNorm(x[m, :]) * g + b) . Wq^T + bq) * q_scale
// Same scheme as layer_tail_kernel: 32 rows per workgroup, wavefront w owns 32 output
// columns of either product, weights packed by layer_mid_pack_kernel.
__global__ __launch_bounds__(512) void layer_mid_kernel(
    const bf16_t* __restrict__ O, const bf16_t* __restrict__ Wp, const float* __restrict__ bo,
    const float* __restrict__ ln_g, const float* __restrict__ ln_b, float eps,
    float* __restrict__ resid, const float* __restrict__ bq, float q_scale,
    bf16_t* __restrict__ q_out, const int32_t* __restrict__ m_ptr, int m_host) {
  constexpr int D = 256, BM = 32, NW = 8;
  __shared__ __attribute__((aligned(16))) unsigned char sA[BM * D * 2];
  __shared__ __attribute__((aligned(16))) unsigned char s_stage[NW * 32 * kTailStride];
  __shared__ __attribute__((aligned(16))) float s_red[2][BM][NW];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g = lane >> 5;
  const unsigned char* const wsrc = reinterpret_cast<const unsigned char*>(Wp) + (size_t)wave * 16384;
  const uint32_t voff = lane * 16;
  bf16x8 wreg[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) wreg[i] = *reinterpret_cast<const bf16x8*>(wsrc + i * 1024 + voff);
  const int M = m_ptr ? *m_ptr : m_host;
  const int total = (M + BM - 1) / BM;
  if ((int)blockIdx.x >= total) return;   // surplus workgroup: the grid covers the capacity
  const int m0 = xcd_tile_order(blockIdx.x, total) * BM;
  const int crow = lane >> 3, lp = lane & 7, cn = wave * 32 + lp * 4;
  unsigned char* const stg = s_stage + wave * (32 * kTailStride);
  // the 32 rows of O once per workgroup, through the operand buffer (as in layer_tail_kernel)
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = wave * 4 + 2 * j + (lane >> 5), p = lane & 31;
    const int c = (p & ~7) | ((p ^ row) & 7);
    dma16_untracked(O + (size_t)min(m0 + row, M - 1) * D + c * 8, sA + (wave * 4 + 2 * j) * 512);
  }
  const float4 bo4 = *reinterpret_cast<const float4*>(bo + cn);
  const float4 gain4 = *reinterpret_cast<const float4*>(ln_g + cn);
  const float4 offs4 = *reinterpret_cast<const float4*>(ln_b + cn);
  const float4 bq4 = *reinterpret_cast<const float4*>(bq + cn);
  float4 xin[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
    xin[t] = *reinterpret_cast<const float4*>(resid + (size_t)min(m0 + t * 8 + crow, M - 1) * D + cn);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // this wavefront's rows of O are in LDS
  __syncthreads();
  bf16x8 oreg[16];
  tail_operand_load(sA, lane, oreg);
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
  for (int ks = 0; ks < 16; ++ks) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[ks], oreg[ks], acc, 0, 0, 0);
    wreg[ks] = *reinterpret_cast<const bf16x8*>(wsrc + 131072 + ks * 1024 + voff);   // Wq
  }
  float4 v[4];
  float mean[4], rstd[4];
  tail_tile_put(acc, stg, lane);
  tail_rows_take(stg, bo4, xin, lane, v);
#pragma unroll
  for (int t = 0; t < 4; ++t)
    if (m0 + t * 8 + crow < M)
      *reinterpret_cast<float4*>(resid + (size_t)(m0 + t * 8 + crow) * D + cn) = v[t];
  tail_rows_stats(v, s_red, wave, lane, eps, mean, rstd);
  tail_rows_to_operand(v, mean, rstd, gain4, offs4, sA, wave, lane);
  __syncthreads();
  bf16x8 areg[16];
  tail_operand_load(sA, lane, areg);
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
  for (int ks = 0; ks < 16; ++ks)
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[ks], areg[ks], acc, 0, 0, 0);
  // through the wavefront's staging area (its own reads of the first tile are done: LDS
  // serves a wavefront's instructions in order): 8 lanes per row, 4 columns per lane
  tail_tile_put(acc, stg, lane);
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int row = t * 8 + crow;
    const float4 a4 = *reinterpret_cast<const float4*>(stg + row * kTailStride + lp * 16);
    if (m0 + row < M)
      *reinterpret_cast<uint2*>(q_out + (size_t)(m0 + row) * D + cn) =
          make_uint2(pack_bf16x2((a4.x + bq4.x) * q_scale, (a4.y + bq4.y) * q_scale),
                     pack_bf16x2((a4.z + bq4.z) * q_scale, (a4.w + bq4.w) * q_scale));
  }
}

// ---------------------------------------------------------------------------
// Everything of a layer that follows attention, in one kernel (width 256).
// ---------------------------------------------------------------------------
//   x[m, :] += O[m, :] . Wo^T + bo;            a = LayerNorm(x) * g2 + b2
//   x[m, :] += GELU(a . W1^T + b1) . W2^T + bf;  n = LayerNorm(x[m, :]) * g + b
//   kLast: out = n (fp32; rows from split_row on to out2); otherwise q, k, v of the next
//   layer from n (tail_project_qkv), n itself is not written.
// All of it is local to a row, so a workgroup that owns 32 complete rows can do it
// without the residual stream, the normalised rows or the hidden activations leaving
// the CU in between.  Eight wavefronts; in the output projection and in q/k/v wavefront
// w owns a 32 (96) column slice of the output.
//
// The feed-forward block walks the hidden width in chunks of 128 with a split of
// roles: wavefronts 0-3 produce the hidden chunk (each 32 hidden columns: 16 MFMAs
// against the normalised rows it holds in registers, then bias, GELU, bf16, into LDS),
// wavefronts 4-7 consume it (each 64 output columns: 16 MFMAs with the chunk from LDS as
// operand).  Every SIMD holds one wavefront of each kind, and while the consumers work
// on chunk c the producers are already at chunk c + 1, so that one kind's MFMAs run
// under the other's GELU arithmetic instead of all eight wavefronts doing the same thing
// at the same time.  Two LDS buffers alternate between chunks and one barrier per chunk
// orders them: the producers pass barrier c after writing chunk c, the consumers before
// reading it; chunk c + 2 lands in the buffer of chunk c only after barrier c + 1, which
// a consumer reaches when it is done with chunk c.
//
// No wavefront shares a weight with another, so the weights do not pass through LDS at
// all: they are packed beforehand (layer_tail_pack_kernel) so that a plain 16-byte load
// per lane delivers an MFMA operand, 1 KB contiguous per instruction, and every operand
// register is reloaded for the next chunk right after the MFMA that used it: 16 KB of
// weights per wavefront are in flight at any time.  LDS carries only the normalised rows
// and the hidden chunk.
//
// The sums run over K in ascending order like the separate kernels', so a row's result
// does not depend on the batch it is in.
template <bool kLast>
__global__ __launch_bounds__(512) void layer_tail_kernel(
    const bf16_t* __restrict__ O, const bf16_t* __restrict__ Wp, const float* __restrict__ bo,
    const float* __restrict__ ln2_g, const float* __restrict__ ln2_b,
    const float* __restrict__ b1, const float* __restrict__ bf, int F,
    float* __restrict__ resid, const float* __restrict__ ln_g, const float* __restrict__ ln_b,
    float eps, float* __restrict__ out, int split_row, float* __restrict__ out2, TailQkv qkv,
    const int32_t* __restrict__ m_ptr, int m_host) {
  constexpr int D = 256, BM = 32, FC = 128, NW = 8, WTN = 32;
  constexpr int kMaxF = 2048;
  __shared__ __attribute__((aligned(16))) unsigned char sA[BM * D * 2];
  __shared__ __attribute__((aligned(16))) unsigned char sH0[BM * FC * 2], sH1[BM * FC * 2];
  __shared__ __attribute__((aligned(16))) unsigned char s_stage[NW * 32 * kTailStride];
  __shared__ __attribute__((aligned(16))) float s_b1[kMaxF];
  __shared__ __attribute__((aligned(16))) float s_red[2][BM][NW];   // [pass][row][wavefront]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, and known to be
  const int l32 = lane & 31, g = lane >> 5;     // MFMA operands: row, k half
  const int nchunk = F / FC;
  CFDETR_TLX(0);

  // weight operands: group c (0: output projection, 1..: hidden chunks, then q/k/v), 16
  // blocks of 1 KB per wavefront; a wave-uniform base and a 32-bit lane offset
  const unsigned char* const wsrc = reinterpret_cast<const unsigned char*>(Wp) + (size_t)wave * 16384;
  const uint32_t voff = lane * 16;
#define CFDETR_TAIL_W(c_, i_) \
  (*reinterpret_cast<const bf16x8*>(wsrc + (size_t)(c_) * 131072 + (i_) * 1024 + voff))
  bf16x8 wreg[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) wreg[i] = CFDETR_TAIL_W(0, i);

  const int M = m_ptr ? *m_ptr : m_host;
  const int total = (M + BM - 1) / BM;
  if ((int)blockIdx.x >= total) return;   // surplus workgroup: the grid covers the capacity
  const int m0 = xcd_tile_order(blockIdx.x, total) * BM;
  // rows and columns of this lane where rows are spread over 8 lanes (4 columns each)
  const int crow = lane >> 3, lp = lane & 7, cn = wave * WTN + lp * 4;
  float4 v[4];      // the residual rows in that form
  float mean[4], rstd[4];
  unsigned char* const stg = s_stage + wave * (32 * kTailStride);
  {
    // ---- attention output times Wo.  The 32 rows of O come in once per workgroup (four
    // rows per wavefront, straight into the operand buffer: lane -> LDS chunk position,
    // fetching the chunk that the row's swizzle puts there); every wavefront then takes
    // them as operands (lane (l32, g): elements 16 ks + 8 g .. of row l32) from LDS.
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int row = wave * 4 + 2 * j + (lane >> 5), p = lane & 31;
      const int c = (p & ~7) | ((p ^ row) & 7);
      dma16_untracked(O + (size_t)min(m0 + row, M - 1) * D + c * 8, sA + (wave * 4 + 2 * j) * 512);
    }
    const float4 bo4 = *reinterpret_cast<const float4*>(bo + cn);
    const float4 gain4 = *reinterpret_cast<const float4*>(ln2_g + cn);
    const float4 offs4 = *reinterpret_cast<const float4*>(ln2_b + cn);
    float4 xin[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
      xin[t] = *reinterpret_cast<const float4*>(resid + (size_t)min(m0 + t * 8 + crow, M - 1) * D + cn);
    for (int i = tid * 4; i < F; i += 2048)
      *reinterpret_cast<float4*>(s_b1 + i) = *reinterpret_cast<const float4*>(b1 + i);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // this wavefront's rows of O are in LDS
    __syncthreads();
    bf16x8 oreg[16];
    tail_operand_load(sA, lane, oreg);
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[ks], oreg[ks], acc, 0, 0, 0);
      wreg[ks] = CFDETR_TAIL_W(1, ks);
    }
    CFDETR_TLX(1);
    tail_tile_put(acc, stg, lane);
    tail_rows_take(stg, bo4, xin, lane, v);
    tail_rows_stats(v, s_red, wave, lane, eps, mean, rstd);
    tail_rows_to_operand(v, mean, rstd, gain4, offs4, sA, wave, lane);
    __syncthreads();
  }
  CFDETR_TLX(2);

  if (wave < 4) {
    // ---- producers: hidden columns 32 wave .. of every chunk.  The MFMAs of chunk c + 1
    // are issued between the GELU evaluations of chunk c (one MFMA, then one element's
    // arithmetic): a wavefront issues in order, and sixteen dependent MFMAs in a row would
    // hold back everything behind them for their whole run time.
    bf16x8 areg[16];
    tail_operand_load(sA, lane, areg);
    f32x16 hid;
#define CFDETR_TAIL_BIAS(c_)                                                                  \
  _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                             \
    const float4 b = *reinterpret_cast<const float4*>(s_b1 + (c_) * FC + wave * 32 + 8 * q + 4 * g); \
    hid[4 * q] = b.x;                                                                         \
    hid[4 * q + 1] = b.y;                                                                     \
    hid[4 * q + 2] = b.z;                                                                     \
    hid[4 * q + 3] = b.w;                                                                     \
  }
    CFDETR_TAIL_BIAS(0)
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
      hid = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[ks], areg[ks], hid, 0, 0, 0);
      wreg[ks] = CFDETR_TAIL_W(nchunk > 1 || !kLast ? 2 : 1, ks);
    }
    for (int c = 0; c < nchunk; ++c) {
      // the group whose weights are fetched while chunk c + 1 is computed: chunk c + 2,
      // behind the last chunk the projection (the last layer fetches a chunk once more:
      // in bounds, never used)
      const int cnext = (kLast ? min(c + 2, nchunk - 1) : min(c + 2, nchunk)) + 1;
      unsigned char* const sH = (c & 1) ? sH1 : sH0;
      CFDETR_TL(0);
      const f32x16 cur = hid;
      float gel[16];
      if (c + 1 < nchunk) {
        CFDETR_TAIL_BIAS(c + 1)
#pragma unroll
        for (int ks = 0; ks < 16; ++ks) {
          hid = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[ks], areg[ks], hid, 0, 0, 0);
          wreg[ks] = CFDETR_TAIL_W(cnext, ks);
          gel[ks] = gelu_fast(cur[ks]);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
          __builtin_amdgcn_sched_group_barrier(0x002, 9, 0);   // one element's arithmetic
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // the weight load
        }
      } else {
#pragma unroll
        for (int ks = 0; ks < 16; ++ks) gel[ks] = gelu_fast(cur[ks]);
      }
      CFDETR_TL(1);
      // bf16, into the chunk buffer: lane = row, 4 consecutive columns per store
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint2 pk = make_uint2(pack_bf16x2(gel[4 * q], gel[4 * q + 1]),
                                    pack_bf16x2(gel[4 * q + 2], gel[4 * q + 3]));
        *reinterpret_cast<uint2*>(sH + l32 * (FC * 2) + (((wave * 4 + q) ^ (l32 & 7)) << 4) + g * 8) = pk;
      }
      CFDETR_TL(2);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __builtin_amdgcn_s_barrier();
      CFDETR_TL(3);
    }
#undef CFDETR_TAIL_BIAS
  } else {
    // ---- consumers: output columns 64 (wave - 4) .. as two tiles
    f32x16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    for (int c = 0; c < nchunk; ++c) {
      const int cnext = (kLast ? min(c + 1, nchunk - 1) : c + 1) + 1;
      const unsigned char* const sH = (c & 1) ? sH1 : sH0;
      CFDETR_TL(0);
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      CFDETR_TL(1);
      // the whole chunk as operand first (eight reads in flight), then the MFMAs
      bf16x8 fa[8];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const int hc = 2 * ks + g;     // 16-byte chunk of the hidden row
        fa[ks] = *reinterpret_cast<const bf16x8*>(sH + l32 * (FC * 2) + ((hc ^ (l32 & 7)) << 4));
      }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[2 * ks + j], fa[ks], acc[j], 0, 0, 0);
          wreg[2 * ks + j] = CFDETR_TAIL_W(cnext, 2 * ks + j);
        }
      }
      CFDETR_TL(2);
    }
    // the two tiles go to the staging areas of the wavefronts that own their columns in
    // what follows (32 per wavefront)
    tail_tile_put(acc[0], s_stage + (2 * (wave - 4)) * (32 * kTailStride), lane);
    tail_tile_put(acc[1], s_stage + (2 * (wave - 4) + 1) * (32 * kTailStride), lane);
  }
  __syncthreads();
  CFDETR_TLX(3);
  // ---- x = x + FFN; the new residual rows go out, and their LayerNorm
  const float4 bf4 = *reinterpret_cast<const float4*>(bf + cn);
  const float4 gain4 = *reinterpret_cast<const float4*>(ln_g + cn);
  const float4 offs4 = *reinterpret_cast<const float4*>(ln_b + cn);
  float4 x2[4];
  tail_rows_take(stg, bf4, v, lane, x2);
  // asked for behind the loads the rows above wait for, used after the LayerNorm
  f32x16 pacc[3];
  int vpos = 0;
  if (!kLast) tail_qkv_prepare(qkv, m0, M, wave, lane, pacc, vpos);
#pragma unroll
  for (int t = 0; t < 4; ++t)
    if (m0 + t * 8 + crow < M)
      *reinterpret_cast<float4*>(resid + (size_t)(m0 + t * 8 + crow) * D + cn) = x2[t];
  tail_rows_stats(x2, s_red, wave, lane, eps, mean, rstd);
  if (kLast) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int m = m0 + t * 8 + crow;
      if (m >= M) continue;
      const float r0 = (x2[t].x - mean[t]) * rstd[t] * gain4.x + offs4.x;
      const float r1 = (x2[t].y - mean[t]) * rstd[t] * gain4.y + offs4.y;
      const float r2 = (x2[t].z - mean[t]) * rstd[t] * gain4.z + offs4.z;
      const float r3 = (x2[t].w - mean[t]) * rstd[t] * gain4.w + offs4.w;
      const bool second = out2 != nullptr && m >= split_row;
      float* obase = second ? out2 : out;
      *reinterpret_cast<float4*>(obase + (size_t)(second ? m - split_row : m) * D + cn) =
          make_float4(r0, r1, r2, r3);
    }
    CFDETR_TLX(4);
    return;
  }
  // ---- the next layer's q, k, v of these rows (sA is free: the producers have taken
  // their copy long ago)
  tail_rows_to_operand(x2, mean, rstd, gain4, offs4, sA, wave, lane);
  __syncthreads();
  tail_project_qkv(sA, wreg, wsrc + (size_t)(nchunk + 1) * 131072, voff, qkv, stg, m0, M, wave, lane,
                   pacc, vpos);
#undef CFDETR_TAIL_W
  CFDETR_TLX(4);
}

// ---------------------------------------------------------------------------
// Patch embedding: rows of A are gathered pixels.
// ---------------------------------------------------------------------------
// Pixels of one patch, flattened (channel, row, column).  P is a power of two.
template <typename TPix>
struct PatchRows {
  const TPix* images;
  const int32_t* tok_desc;
  const int32_t* cu;
  int B, level, log2p, img_h, img_w;
  // Pixel offset of the patch of token m, or 0 (frame 0's first patch: in bounds,
  // result discarded) with valid = false when m is not a token of this level.
  __device__ size_t prepare(int m, bool& valid) const {
    size_t off = 0;
    if (valid) {
      const int32_t desc = tok_desc[m];
      valid = tok_level(desc) == level;
      if (valid) {
        const int frame = frame_of_token(cu, B, m);
        off = ((size_t)frame * 3 * img_h + ((size_t)tok_row(desc) << log2p)) * img_w +
              ((size_t)tok_col(desc) << log2p);
      }
    }
    return off;
  }
  __device__ size_t pix_off(int k) const {
    const int c = k >> (2 * log2p);
    const int r = (k >> log2p) & ((1 << log2p) - 1);
    const int x = k & ((1 << log2p) - 1);
    return ((size_t)c * img_h + r) * img_w + x;
  }
  __device__ uint4 load8(size_t row_off, int k) const;
  __device__ float load1(size_t row_off, int k) const;
};
template <>
__device__ uint4 PatchRows<bf16_t>::load8(size_t row_off, int k) const {
  return *reinterpret_cast<const uint4*>(images + row_off + pix_off(k));
}
template <>
__device__ uint4 PatchRows<float>::load8(size_t row_off, int k) const {
  const float4* p = reinterpret_cast<const float4*>(images + row_off + pix_off(k));
  const float4 a = p[0], b = p[1];
  return make_uint4(pack_bf16x2(a.x, a.y), pack_bf16x2(a.z, a.w), pack_bf16x2(b.x, b.y),
                    pack_bf16x2(b.z, b.w));
}
template <>
__device__ float PatchRows<bf16_t>::load1(size_t row_off, int k) const {
  return bf16_to_f32(images[row_off + pix_off(k)]);
}
template <>
__device__ float PatchRows<float>::load1(size_t row_off, int k) const {
  return images[row_off + pix_off(k)];
}

template <int BM, int BN>
constexpr size_t gather_lds_bytes() {
  return (size_t)2 * (BM + BN) * LDS_LD * sizeof(bf16_t) + BM * sizeof(int32_t) + 16;
}

// Register-staged, double-buffered (global -> registers -> padded LDS rows, one
// barrier per slab).  The staging registers are plain unrolled arrays; closures over
// them would push them into scratch memory.
template <int BM, int BN, int NWM, int NWN, typename TPix>
__global__ __launch_bounds__(64 * NWM * NWN) void gemm_bf16_gather_kernel(
    PatchRows<TPix> al, const bf16_t* __restrict__ W, int N, int K, EpiEmbed ep,
    const int32_t* __restrict__ m_ptr, int m_host) {
  constexpr int THREADS = 64 * NWM * NWN;
  constexpr int WTM = BM / NWM, WTN = BN / NWN;
  constexpr int MT = WTM / 32, NT = WTN / 32;
  constexpr int PASS_ROWS = THREADS / 8;  // rows staged per pass (8 x 16 B per row)
  constexpr int A_LOADS = BM / PASS_ROWS, B_LOADS = BN / PASS_ROWS;
  static_assert(BM % PASS_ROWS == 0 && BN % PASS_ROWS == 0, "tile / thread mismatch");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_gather[];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_gather);                 // [2][BM * LDS_LD]
  bf16_t* sB = sA + 2 * BM * LDS_LD;                                   // [2][BN * LDS_LD]
  int32_t* s_desc = reinterpret_cast<int32_t*>(sB + 2 * BN * LDS_LD);  // [BM], -1 = not ours
  int32_t* s_any = s_desc + BM;

  const int M = m_ptr ? *m_ptr : m_host;
  const int n_blocks = N / BN;
  const int total = ((M + BM - 1) / BM) * n_blocks;
  if ((int)blockIdx.x >= total) return;
  const int pid = xcd_tile_order(blockIdx.x, total);
  const int m0 = (pid / n_blocks) * BM;
  const int n0 = (pid % n_blocks) * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / NWN, wn = wave % NWN;
  const int chunk = tid & 7, srow = tid >> 3;

  if (tid == 0) *s_any = 0;
  __syncthreads();
  size_t arow[A_LOADS];
  bool any_valid = false;
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int r = srow + PASS_ROWS * j;
    bool valid = (m0 + r) < M;
    arow[j] = al.prepare(m0 + r, valid);
    if (chunk == 0) s_desc[r] = valid ? al.tok_desc[m0 + r] : -1;
    any_valid |= valid;
  }
  if (any_valid) *s_any = 1;
  __syncthreads();
  if (!*s_any) return;  // no token of this level in the tile
  const bf16_t* wrow[B_LOADS];
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j)
    wrow[j] = W + (size_t)(n0 + srow + PASS_ROWS * j) * K + chunk * 8;

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int l32 = lane & 31, g = lane >> 5;
  const int a_off = (wm * WTM + l32) * LDS_LD + g * 8;
  const int b_off = (wn * WTN + l32) * LDS_LD + g * 8;
  const int st_off = srow * LDS_LD + chunk * 8;

  uint4 ra[A_LOADS], rb[B_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) ra[j] = al.load8(arow[j], chunk * 8);
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) rb[j] = *reinterpret_cast<const uint4*>(wrow[j]);
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j)
    *reinterpret_cast<uint4*>(sA + st_off + PASS_ROWS * j * LDS_LD) = ra[j];
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j)
    *reinterpret_cast<uint4*>(sB + st_off + PASS_ROWS * j * LDS_LD) = rb[j];
  __syncthreads();

  const int nk = K / BK;
  for (int it = 0; it < nk; ++it) {
    // The last pass fetches its own slab again (unused) so that the loop body is
    // free of conditionals around the register arrays.
    const int kn = min(it + 1, nk - 1) * BK;
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) ra[j] = al.load8(arow[j], kn + chunk * 8);
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) rb[j] = *reinterpret_cast<const uint4*>(wrow[j] + kn);
    const bf16_t* pa = sA + (it & 1) * BM * LDS_LD + a_off;
    const bf16_t* pb = sB + (it & 1) * BN * LDS_LD + b_off;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[MT], fb[NT];
#pragma unroll
      for (int i = 0; i < MT; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(pa + i * 32 * LDS_LD + ks * 16);
#pragma unroll
      for (int j = 0; j < NT; ++j)
        fb[j] = *reinterpret_cast<const bf16x8*>(pb + j * 32 * LDS_LD + ks * 16);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    bf16_t* qa = sA + ((it + 1) & 1) * BM * LDS_LD + st_off;
    bf16_t* qb = sB + ((it + 1) & 1) * BN * LDS_LD + st_off;
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j)
      *reinterpret_cast<uint4*>(qa + PASS_ROWS * j * LDS_LD) = ra[j];
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j)
      *reinterpret_cast<uint4*>(qb + PASS_ROWS * j * LDS_LD) = rb[j];
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int ml = wm * WTM + i * 32 + l32;
    const int32_t desc = s_desc[ml];
    if (desc < 0) continue;
    float4 bias_r[NT][4], extra[NT][4];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn * WTN + j * 32 + 8 * q + 4 * g;
        bias_r[j][q] = ep.bias4(n);
        extra[j][q] = ep.extra4(m0 + ml, n, desc);
      }
#pragma unroll
    for (int j = 0; j < NT; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn * WTN + j * 32 + 8 * q + 4 * g;
        const float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                            acc[i][j][4 * q + 3]};
        ep.store4(m0 + ml, n, v, bias_r[j][q], extra[j][q], desc);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// fp32 check-mode kernel: 64x64 tile, 256 threads, 4x4 outputs per thread.
// ---------------------------------------------------------------------------
struct PlainF32 {
  const float* A;
  int lda;
  __device__ size_t prepare(int m, bool&) const { return (size_t)m * lda; }
  __device__ float load1(size_t row_off, int k) const { return A[row_off + k]; }
};

template <typename AL>
struct IsPatch { static constexpr bool value = false; };
template <typename T>
struct IsPatch<PatchRows<T>> { static constexpr bool value = true; };

template <typename AL, typename EP>
__global__ __launch_bounds__(256) void gemm_f32_kernel(AL al, const float* __restrict__ W, int N,
                                                       int K, EP ep,
                                                       const int32_t* __restrict__ m_ptr,
                                                       int m_host, const int32_t* tok_desc) {
  constexpr int T = 64, KK = 16;
  __shared__ float sA[KK][T + 4];
  __shared__ float sB[KK][T + 4];
  __shared__ int32_t s_desc[T];
  __shared__ int s_any;
  const int M = m_ptr ? *m_ptr : m_host;
  const int n_blocks = N / T;
  const int m0 = (blockIdx.x / n_blocks) * T;
  const int n0 = (blockIdx.x % n_blocks) * T;
  if (m0 >= M) return;
  const int tid = threadIdx.x;
  const int lrow = tid >> 2;     // staged row 0..63
  const int lk = (tid & 3) * 4;  // 4 consecutive k of a 16-wide slab
  if (tid == 0) s_any = 0;
  __syncthreads();
  bool valid = (m0 + lrow) < M;
  const size_t arow = al.prepare(valid ? m0 + lrow : M - 1, valid);
  if ((tid & 3) == 0) {
    int32_t desc = -1;
    if (valid) desc = IsPatch<AL>::value ? tok_desc[m0 + lrow] : 0;
    s_desc[lrow] = desc;
  }
  if (valid) s_any = 1;
  __syncthreads();
  if (!s_any) return;
  const float* wrow = W + (size_t)(n0 + lrow) * K;
  const int ty = tid >> 4, tx = tid & 15;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += KK) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      sA[lk + q][lrow] = al.load1(arow, k0 + lk + q);
      sB[lk + q][lrow] = wrow[k0 + lk + q];
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        a[q] = sA[kk][ty * 4 + q];
        b[q] = sB[kk][tx * 4 + q];
      }
#pragma unroll
      for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[p][q] = fmaf(a[p], b[q], acc[p][q]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int ml = ty * 4 + p;
    const int32_t desc = s_desc[ml];
    if (desc < 0) continue;
    ep.store4(m0 + ml, n0 + tx * 4, acc[p], ep.bias4(n0 + tx * 4),
              ep.extra4(m0 + ml, n0 + tx * 4, desc), desc);
  }
}

int ilog2(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

template <typename Kern>
hipError_t allow_lds(Kern kern, size_t bytes, bool* configured) {
  if (*configured) return hipSuccess;   // the attribute is sticky
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) *configured = true;
  return e;
}

template <int BM, int BN, int NWM, int NWN, int S, int BKT, int KS = 1, int WPE = 1, typename AROWS, typename EP>
hipError_t launch_direct_tile(const AROWS& a, const bf16_t* w, int N, int K, const EP& ep,
                              const int32_t* m_ptr, int m_host, int m_capacity, hipStream_t s) {
  auto kern = gemm_bf16_direct_kernel<BM, BN, NWM, NWN, S, BKT, AROWS, EP, KS, WPE>;
  if (K % (BKT * KS) != 0) return hipErrorInvalidValue;
  // the kernel addresses the weights with 32-bit byte offsets (the rows: see the callers)
  if ((size_t)N * K * 2 >= ((size_t)1 << 32)) return hipErrorInvalidValue;
  constexpr size_t lds = (size_t)KS * S * (BM + BN) * BKT * 2;
  static_assert(lds <= 160 * 1024, "ring exceeds the LDS");
  static bool configured = false;
  hipError_t e = allow_lds(kern, lds, &configured);
  if (e != hipSuccess) return e;
  dim3 grid(((m_capacity + BM - 1) / BM) * (N / BN));
  hipLaunchKernelGGL(kern, grid, dim3(64 * NWM * NWN * KS), lds, s, a, w, N, K, ep, m_ptr, m_host);
  return hipSuccess;
}

int cu_count() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      cus = 256;
  }
  return cus;
}

// Launch of the staying-workgroup form: the grid is `per_cu` workgroups per CU (what the
// tile's LDS ring allows), a multiple of 8, and no more than the tiles the capacity yields.
template <int BM, int BN, int NWM, int NWN, int WPE = 1, typename EP>
hipError_t launch_persist_tile(const DenseRows& a, const bf16_t* w, int N, int K, const EP& ep,
                               const int32_t* m_ptr, int m_host, int m_capacity, int per_cu,
                               hipStream_t s) {
  auto kern = gemm_bf16_persist_kernel<BM, BN, NWM, NWN, 64, EP, WPE>;
  if (K % 64 != 0 || N % BN != 0) return hipErrorInvalidValue;
  if ((size_t)N * K * 2 >= ((size_t)1 << 32)) return hipErrorInvalidValue;
  constexpr size_t lds = (size_t)2 * (BM + BN) * 64 * 2;
  static_assert(lds <= 160 * 1024, "ring exceeds the LDS");
  static bool configured = false;
  hipError_t e = allow_lds(kern, lds, &configured);
  if (e != hipSuccess) return e;
  const long tiles = (long)((m_capacity + BM - 1) / BM) * (N / BN);
  long grid = ((long)cu_count() * per_cu) & ~7L;
  if (grid < 8) grid = 8;
  if (tiles < grid) grid = tiles;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * NWM * NWN), lds, s, a, w, N, K, ep, m_ptr,
                     m_host);
  return hipSuccess;
}

// Tile choice by problem size: 256x256 (8 wavefronts, 128x64 each) or 192x256 (96x64
// each) for wide outputs over many rows, 192x128 or 128x128 (4 wavefronts, 96x64 or 64x64
// each, two workgroups per CU) while that still yields a workgroup per CU, else 64x64
// (2 wavefronts, 32x64 each).  All are the staying-workgroup kernel.  The rows that count
// are the likely ones: with the row count on the device (m_ptr), m_host > 0 is the caller's
// estimate of it (the kernels do not read it) and the capacity stands in otherwise.  A CU
// holds one large tile or two of the four-wavefront tiles; against a pair of 128-tiles a
// 256-tile is twice the work per CU and takes about 1.8 times as long, a 192x256 tile or a
// pair of 192x128 tiles 1.5 times the work in about 1.45 to 1.5 times as long, so what
// decides at a few rounds is how full the last round is: the estimate is rounds x time per
// round.  (24 470 rows x 384 columns are 576 tiles of 128x128 for 512 places, two rounds
// of which the second is an eighth full, and 384 tiles of 192x128, one round.)
template <typename EP>
hipError_t launch_direct(const void* A, const void* W, int N, int K, const EP& ep,
                         const int32_t* m_ptr, int m_host, int m_capacity, hipStream_t s) {
  const DenseRows a{static_cast<const bf16_t*>(A), K};
  const bf16_t* w = static_cast<const bf16_t*>(W);
  if ((size_t)m_capacity * K * 2 >= ((size_t)1 << 32)) return hipErrorInvalidValue;
  const int m = m_ptr ? (m_host > 0 && m_host < m_capacity ? m_host : m_capacity) : m_host;
  const long cus = cu_count();
  const long tiles128 = (long)((m + 127) / 128) * (N / 128);
  const long tiles256 = (long)((m + 255) / 256) * (N / 256);
  const long tiles192 = (long)((m + 191) / 192) * (N / 256);
  const long tiles192n = (long)((m + 191) / 192) * (N / 128);
  const long rounds128 = (tiles128 + 2 * cus - 1) / (2 * cus), rounds256 = (tiles256 + cus - 1) / cus;
  const long rounds192 = (tiles192 + cus - 1) / cus, rounds192n = (tiles192n + 2 * cus - 1) / (2 * cus);
  const long t128 = 100 * rounds128, t192n = 150 * rounds192n;
  const bool narrow_ok = N % 128 == 0 && tiles128 >= cus;
  // A deeper ring (3 or 4 buffers, also with slabs of 32) measured no faster for these
  // tiles: their main loops are bound by LDS traffic, not by the latency of the loads.
  if (N % 256 == 0 && m >= 8192) {
    const long t256 = 180 * rounds256, t192 = 145 * rounds192;
    const long tn = t192n < t128 ? t192n : t128;
    if (t192 < t256 && t192 <= tn)
      return launch_persist_tile<192, 256, 2, 4>(a, w, N, K, ep, m_ptr, m_host, m_capacity, 1, s);
    if (t256 <= tn)
      return launch_persist_tile<256, 256, 2, 4>(a, w, N, K, ep, m_ptr, m_host, m_capacity, 1, s);
  }
  if (narrow_ok && m >= 8192 && t192n < t128)
    return launch_persist_tile<192, 128, 2, 2, 2>(a, w, N, K, ep, m_ptr, m_host, m_capacity, 2, s);
  if (narrow_ok)
    return launch_persist_tile<128, 128, 2, 2>(a, w, N, K, ep, m_ptr, m_host, m_capacity, 2, s);
  // small problems: 64 x 64 tiles of two wavefronts (32 x 64 each), several per CU
  return launch_persist_tile<64, 64, 2, 1>(a, w, N, K, ep, m_ptr, m_host, m_capacity, 4, s);
}

template <int BM, int BN, typename TPix>
hipError_t launch_gather_tile(const PatchRows<TPix>& al, const bf16_t* w, int N, int K,
                              const EpiEmbed& ep, const int32_t* m_ptr, int m_host,
                              int m_capacity, hipStream_t s) {
  auto kern = gemm_bf16_gather_kernel<BM, BN, 2, 2, TPix>;
  constexpr size_t lds = gather_lds_bytes<BM, BN>();
  static bool configured = false;
  hipError_t e = allow_lds(kern, lds, &configured);
  if (e != hipSuccess) return e;
  dim3 grid(((m_capacity + BM - 1) / BM) * (N / BN));
  hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, al, w, N, K, ep, m_ptr, m_host);
  return hipSuccess;
}

template <typename TPix>
hipError_t launch_gather(const PatchRows<TPix>& al, const void* W, int N, int K,
                         const EpiEmbed& ep, const int32_t* m_ptr, int m_host, int m_capacity,
                         hipStream_t s) {
  const bf16_t* w = static_cast<const bf16_t*>(W);
  const long tiles128 = (long)((m_capacity + 127) / 128) * (N / 128);
  if (N % 128 == 0 && tiles128 >= 256)
    return launch_gather_tile<128, 128>(al, w, N, K, ep, m_ptr, m_host, m_capacity, s);
  return launch_gather_tile<64, 64>(al, w, N, K, ep, m_ptr, m_host, m_capacity, s);
}

template <typename AL, typename EP>
hipError_t launch_f32(const AL& al, const void* W, int N, int K, const EP& ep,
                      const int32_t* m_ptr, int m_host, int m_capacity,
                      const int32_t* tok_desc, hipStream_t s) {
  dim3 grid(((m_capacity + 63) / 64) * (N / 64));
  hipLaunchKernelGGL((gemm_f32_kernel<AL, EP>), grid, dim3(256), 0, s, al,
                     static_cast<const float*>(W), N, K, ep, m_ptr, m_host, tok_desc);
  return hipSuccess;
}

}  // namespace

// Width 384 would fit too (three ring buffers), but a workgroup then streams 48 KB of
// weights per 32 rows and slab, and the pair of separate kernels is faster (measured).
bool gemm_residual_ln_supported(int d, bool use_bf16) { return use_bf16 && d == 256; }

namespace {

template <int D, int S>
hipError_t launch_rowln(const bf16_t* a, const bf16_t* w, const float* bias, int K, float* resid,
                        const float* ln_g, const float* ln_b, float eps, void* out,
                        bool out_is_bf16, int split_row, void* out2, const int32_t* m_ptr,
                        int m_host, int m_capacity, hipStream_t s) {
  constexpr int BM = 32;
  dim3 grid((m_capacity + BM - 1) / BM);
  if (out_is_bf16)
    hipLaunchKernelGGL((gemm_bf16_rowln_kernel<BM, D, S, true>), grid, dim3(256), 0, s, a, w, K,
                       bias, resid, ln_g, ln_b, eps, out, split_row, out2, m_ptr, m_host);
  else
    hipLaunchKernelGGL((gemm_bf16_rowln_kernel<BM, D, S, false>), grid, dim3(256), 0, s, a, w, K,
                       bias, resid, ln_g, ln_b, eps, out, split_row, out2, m_ptr, m_host);
  return hipGetLastError();
}

}  // namespace

// The ring takes as many buffers of (32 + d) rows x 128 bytes as the 160 KB of LDS hold.
hipError_t launch_gemm_residual_ln(const void* A, const void* W, const float* bias, int d, int K,
                                   float* resid, const float* ln_g, const float* ln_b, float eps,
                                   void* out, bool out_is_bf16, int split_row, void* out2,
                                   const int32_t* m_ptr, int m_host, int m_capacity,
                                   hipStream_t s) {
  if (K % BK != 0) return hipErrorInvalidValue;
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* w = static_cast<const bf16_t*>(W);
  if (d == 256)
    return launch_rowln<256, 4>(a, w, bias, K, resid, ln_g, ln_b, eps, out, out_is_bf16, split_row,
                                out2, m_ptr, m_host, m_capacity, s);
  return hipErrorInvalidValue;
}

bool layer_tail_supported(int d, int F, bool use_bf16) {
  return use_bf16 && d == 256 && F % 128 == 0 && F <= 2048;
}

uint64_t layer_tail_packed_bytes(int d, int F) {
  return (4 * (uint64_t)d * d + 2 * (uint64_t)F * d) * 2;
}

hipError_t launch_layer_tail_pack(const void* Wo, const void* W1, const void* W2,
                                  const void* Wqkv_next, int d, int F, void* packed,
                                  hipStream_t s) {
  if (!layer_tail_supported(d, F, true)) return hipErrorInvalidValue;
  const int units = (int)(layer_tail_packed_bytes(d, F) / 16);
  hipLaunchKernelGGL(layer_tail_pack_kernel, dim3((units + 255) / 256), dim3(256), 0, s,
                     static_cast<const bf16_t*>(Wo), static_cast<const bf16_t*>(W1),
                     static_cast<const bf16_t*>(W2), static_cast<const bf16_t*>(Wqkv_next), F,
                     static_cast<bf16_t*>(packed));
  return hipGetLastError();
}

hipError_t launch_layer_head_pack(const void* Wqkv, int d, void* packed, hipStream_t s) {
  if (d != 256) return hipErrorInvalidValue;
  hipLaunchKernelGGL(layer_head_pack_kernel, dim3(3 * 256 * 256 / 8 / 256), dim3(256), 0, s,
                     static_cast<const bf16_t*>(Wqkv), static_cast<bf16_t*>(packed));
  return hipGetLastError();
}

hipError_t launch_layer_head(const float* x, const void* packed, const float* ln_g,
                             const float* ln_b, float eps, const float* b_qkv, float q_scale,
                             void* qk, void* vt, int vt_ld, const int32_t* cu, const int32_t* pcu,
                             int B, int d, const int32_t* m_ptr, int m_host, int m_capacity,
                             hipStream_t s) {
  if (d != 256) return hipErrorInvalidValue;
  TailQkv q{b_qkv, q_scale, static_cast<bf16_t*>(qk), static_cast<bf16_t*>(vt), vt_ld, cu, pcu, B};
  hipLaunchKernelGGL(layer_head_kernel, dim3((m_capacity + 31) / 32), dim3(512), 0, s, x,
                     static_cast<const bf16_t*>(packed), ln_g, ln_b, eps, q, m_ptr, m_host);
  return hipGetLastError();
}

hipError_t launch_layer_mid_pack(const void* Wo, const void* Wq, int d, void* packed, hipStream_t s) {
  if (d != 256) return hipErrorInvalidValue;
  hipLaunchKernelGGL(layer_mid_pack_kernel, dim3(2 * 256 * 256 / 8 / 256), dim3(256), 0, s,
                     static_cast<const bf16_t*>(Wo), static_cast<const bf16_t*>(Wq),
                     static_cast<bf16_t*>(packed));
  return hipGetLastError();
}

hipError_t launch_layer_mid(const void* O, const void* packed, const float* b_o, const float* ln_g,
                            const float* ln_b, float eps, float* resid, const float* b_q,
                            float q_scale, void* q_out, int d, const int32_t* m_ptr, int m_host,
                            int m_capacity, hipStream_t s) {
  if (d != 256) return hipErrorInvalidValue;
  hipLaunchKernelGGL(layer_mid_kernel, dim3((m_capacity + 31) / 32), dim3(512), 0, s,
                     static_cast<const bf16_t*>(O), static_cast<const bf16_t*>(packed), b_o, ln_g,
                     ln_b, eps, resid, b_q, q_scale, static_cast<bf16_t*>(q_out), m_ptr, m_host);
  return hipGetLastError();
}

hipError_t launch_layer_tail(const LayerTailArgs& a, int d, int F, const int32_t* m_ptr,
                             int m_host, int m_capacity, hipStream_t s) {
  if (!layer_tail_supported(d, F, true)) return hipErrorInvalidValue;
  dim3 grid((m_capacity + 31) / 32);
  const bf16_t* o = static_cast<const bf16_t*>(a.O);
  const bf16_t* wp = static_cast<const bf16_t*>(a.packed);
  TailQkv q{a.b_qkv, a.q_scale, static_cast<bf16_t*>(a.qk), static_cast<bf16_t*>(a.vt), a.vt_ld,
            a.cu, a.pcu, a.B};
  if (a.last)
    hipLaunchKernelGGL((layer_tail_kernel<true>), grid, dim3(512), 0, s, o, wp, a.b_o, a.ln2_g,
                       a.ln2_b, a.b_ff1, a.b_ff2, F, a.resid, a.ln_g, a.ln_b, a.eps, a.out,
                       a.split_row, a.out2, q, m_ptr, m_host);
  else
    hipLaunchKernelGGL((layer_tail_kernel<false>), grid, dim3(512), 0, s, o, wp, a.b_o, a.ln2_g,
                       a.ln2_b, a.b_ff1, a.b_ff2, F, a.resid, a.ln_g, a.ln_b, a.eps, a.out,
                       a.split_row, a.out2, q, m_ptr, m_host);
  return hipGetLastError();
}

hipError_t launch_embed(const EmbedArgs& a, const void* w, const float* bias, int d,
                        bool use_bf16, const int32_t* m_ptr, int m_host, int m_capacity,
                        hipStream_t s) {
  const int K = 3 * a.patch * a.patch;
  EpiEmbed ep{bias, a.pe_row, a.pe_col, a.out, a.out2, d, a.tok_desc, a.level};
  hipError_t e = hipSuccess;
  // the direct kernel addresses pixels with 32-bit byte offsets from the first frame
  const bool frames_fit = (size_t)a.B * 3 * a.img_h * a.img_w * 2 < ((size_t)1 << 32);
  if (a.image_is_bf16 && use_bf16 && !frames_fit) {
    PatchRows<bf16_t> al{static_cast<const bf16_t*>(a.images), a.tok_desc, a.cu_seqlens, a.B,
                         a.level, ilog2(a.patch), a.img_h, a.img_w};
    e = launch_gather(al, w, d, K, ep, m_ptr, m_host, m_capacity, s);
  } else if (a.image_is_bf16 && use_bf16) {
    // bf16 pixels need no conversion: patch rows go straight from the frames into LDS,
    // through a deep ring when the problem is too small to hide latency by occupancy
    const PatchPixelRows rows{static_cast<const bf16_t*>(a.images), a.tok_desc, a.cu_seqlens, a.B,
                              a.level, ilog2(a.patch), a.img_h, a.img_w};
    const bf16_t* wb = static_cast<const bf16_t*>(w);
    // the coarse grid has a row count the host knows; the finer levels only a capacity
    const int m_likely = m_ptr ? m_capacity : m_host;
    const long tiles128 = (long)((m_likely + 127) / 128) * (d / 128);
    const long tiles64 = (long)((m_likely + 63) / 64) * (d / 64);
    if (d % 128 == 0 && tiles128 >= 256)
      e = launch_direct_tile<128, 128, 2, 2, 2, 64>(rows, wb, d, K, ep, m_ptr, m_host, m_capacity, s);
    else if ((tiles64 <= cu_count() || K >= 6144) && K % 128 == 0)
      // a workgroup per CU at most, or a very long contraction (patches of 64 x 64): two
      // groups of wavefronts share the contraction of a tile
      e = launch_direct_tile<64, 64, 2, 2, 4, 64, 2>(rows, wb, d, K, ep, m_ptr, m_host, m_capacity, s);
    else
      e = launch_direct_tile<64, 64, 2, 2, 4, 64>(rows, wb, d, K, ep, m_ptr, m_host, m_capacity, s);
  } else if (a.image_is_bf16) {
    PatchRows<bf16_t> al{static_cast<const bf16_t*>(a.images), a.tok_desc, a.cu_seqlens, a.B,
                         a.level, ilog2(a.patch), a.img_h, a.img_w};
    e = launch_f32(al, w, d, K, ep, m_ptr, m_host, m_capacity, a.tok_desc, s);
  } else {
    PatchRows<float> al{static_cast<const float*>(a.images), a.tok_desc, a.cu_seqlens, a.B,
                        a.level, ilog2(a.patch), a.img_h, a.img_w};
    if (use_bf16) e = launch_gather(al, w, d, K, ep, m_ptr, m_host, m_capacity, s);
    else e = launch_f32(al, w, d, K, ep, m_ptr, m_host, m_capacity, a.tok_desc, s);
  }
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

hipError_t launch_gemm_qkv(const void* A, const void* W, const float* bias, int d,
                           float q_scale, void* qk, void* vt, int vt_ld, const int32_t* cu_seqlens, const int32_t* pcu,
                           int B, const int32_t* m_ptr, int m_host, int m_capacity,
                           hipStream_t s, const int32_t* vt_pos) {
  EpiQkv ep{bias, static_cast<bf16_t*>(qk), 3 * d, 2 * d, d, q_scale, static_cast<bf16_t*>(vt),
            vt_ld, cu_seqlens, pcu, B, vt_pos};
  hipError_t e = launch_direct(A, W, 3 * d, d, ep, m_ptr, m_host, m_capacity, s);
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

hipError_t launch_gemm_kv_layers(const void* A, const void* W, const float* bias, int d, int layers,
                                 void* k, size_t k_stride, void* vt, size_t vt_stride, int vt_ld,
                                 const int32_t* cu_seqlens, const int32_t* pcu, int B,
                                 const int32_t* m_ptr, int m_host, int m_capacity, hipStream_t s) {
  if (d % 64 != 0) return hipErrorInvalidValue;   // a wavefront's columns must not straddle k | v
  EpiKvLayers ep{bias, static_cast<bf16_t*>(k), k_stride, d, static_cast<bf16_t*>(vt), vt_stride,
                 vt_ld, cu_seqlens, pcu, B};
  hipError_t e = launch_direct(A, W, layers * 2 * d, d, ep, m_ptr, m_host, m_capacity, s);
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

hipError_t launch_gemm(const void* A, const void* W, const float* bias, int N, int K,
                       Epilogue epi, void* out_act, float* resid, bool use_bf16,
                       const int32_t* m_ptr, int m_host, int m_capacity, hipStream_t s,
                       float scale) {
  hipError_t e = hipSuccess;
  if (use_bf16) {
    bf16_t* o = static_cast<bf16_t*>(out_act);
    switch (epi) {
      case Epilogue::kBias:
        e = launch_direct(A, W, N, K, EpiAct<bf16_t, kActNone>{bias, o, N, scale}, m_ptr, m_host,
                          m_capacity, s);
        break;
      case Epilogue::kBiasGelu:
        e = launch_direct(A, W, N, K, EpiAct<bf16_t, kActGelu>{bias, o, N, scale}, m_ptr, m_host,
                          m_capacity, s);
        break;
      case Epilogue::kBiasRelu:
        e = launch_direct(A, W, N, K, EpiAct<bf16_t, kActRelu>{bias, o, N, scale}, m_ptr, m_host,
                          m_capacity, s);
        break;
      case Epilogue::kBiasResidual:
        e = launch_direct(A, W, N, K, EpiResidual{bias, resid, N}, m_ptr, m_host, m_capacity, s);
        break;
    }
  } else {
    PlainF32 al{static_cast<const float*>(A), K};
    float* o = static_cast<float*>(out_act);
    switch (epi) {
      case Epilogue::kBias:
        e = launch_f32(al, W, N, K, EpiAct<float, kActNone>{bias, o, N}, m_ptr, m_host, m_capacity,
                       nullptr, s);
        break;
      case Epilogue::kBiasGelu:
        e = launch_f32(al, W, N, K, EpiAct<float, kActGelu>{bias, o, N}, m_ptr, m_host, m_capacity,
                       nullptr, s);
        break;
      case Epilogue::kBiasRelu:
        return hipErrorInvalidValue;   // only the bf16 path has it
      case Epilogue::kBiasResidual:
        e = launch_f32(al, W, N, K, EpiResidual{bias, resid, N}, m_ptr, m_host, m_capacity, nullptr,
                       s);
        break;
    }
  }
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

}  // namespace cfdetr
