// Contractions of the encoder: C[M,N] = A[M,K] . W[N,K]^T with fused epilogues.
//
// Both operands have K innermost, which is what the 32x32x16 bf16 MFMA wants: a
// lane supplies 8 consecutive k of one row.  A workgroup of four wavefronts
// (2 x 2) owns a BM x BN tile of C; K is walked in slabs of 64 that are staged
// through LDS (rows padded by 8 elements so that the 16-byte operand reads of
// eight consecutive rows fall into disjoint banks) while the next slab is
// already in flight from global memory into registers.
//
// The A operand comes from a loader: either a plain row-major activation matrix
// or the pixels of a frame gathered patch by patch (patch embedding as an
// implicit-im2col GEMM).  The epilogue is a functor as well: bias, bias+GELU,
// bias+residual, or bias+position for the embedding.
//
// M may live on the device (the token total after selection): the grid is sized
// for the capacity and workgroups beyond the real M leave at once.
//
// An all-fp32 variant of the same contractions (no matrix cores) serves the
// check mode.
#include "kernels.h"

namespace cfdetr {

namespace {

constexpr int BK = 64;
constexpr int LDS_LD = BK + 8;  // bf16 elements per staged row

// ---------------------------------------------------------------------------
// A loaders.  prepare(m, valid) is called once per staged row by the thread that
// stages it; load8(ctx, k) returns 8 consecutive k as bf16; load1 serves fp32 mode.
// ---------------------------------------------------------------------------
struct PlainBf16 {
  const bf16_t* A;
  int lda;
  struct Row { const bf16_t* p; };
  __device__ Row prepare(int m) const { return Row{A + (size_t)m * lda}; }
  __device__ uint4 load8(const Row& r, int k) const {
    return *reinterpret_cast<const uint4*>(r.p + k);
  }
};

struct PlainF32 {
  const float* A;
  int lda;
  struct Row { const float* p; };
  __device__ Row prepare(int m) const { return Row{A + (size_t)m * lda}; }
  __device__ float load1(const Row& r, int k) const { return r.p[k]; }
};

// Pixels of one patch, flattened (channel, row, column).  P is a power of two.
template <typename TPix>
struct PatchRows {
  const TPix* images;
  const int32_t* tok_desc;
  const int32_t* cu;
  int B, level, log2p, img_h, img_w;
  struct Row { const TPix* p; };
  // Rows that are not tokens of this level read frame 0's first patch (in bounds,
  // result discarded).
  __device__ Row prepare(int m, bool& valid) const {
    size_t off = 0;
    if (valid) {
      int32_t desc = tok_desc[m];
      valid = tok_level(desc) == level;
      if (valid) {
        int frame = frame_of_token(cu, B, m);
        off = ((size_t)frame * 3 * img_h + ((size_t)tok_row(desc) << log2p)) * img_w +
              ((size_t)tok_col(desc) << log2p);
      }
    }
    return Row{images + off};
  }
  __device__ size_t pix_off(int k) const {
    int c = k >> (2 * log2p);
    int r = (k >> log2p) & ((1 << log2p) - 1);
    int x = k & ((1 << log2p) - 1);
    return ((size_t)c * img_h + r) * img_w + x;
  }
  __device__ uint4 load8(const Row& row, int k) const;
  __device__ float load1(const Row& row, int k) const;
};
template <>
__device__ uint4 PatchRows<bf16_t>::load8(const Row& row, int k) const {
  return *reinterpret_cast<const uint4*>(row.p + pix_off(k));
}
template <>
__device__ uint4 PatchRows<float>::load8(const Row& row, int k) const {
  const float4* p = reinterpret_cast<const float4*>(row.p + pix_off(k));
  float4 a = p[0], b = p[1];
  return make_uint4(pack_bf16x2(a.x, a.y), pack_bf16x2(a.z, a.w), pack_bf16x2(b.x, b.y),
                    pack_bf16x2(b.z, b.w));
}
template <>
__device__ float PatchRows<bf16_t>::load1(const Row& row, int k) const {
  return bf16_to_f32(row.p[pix_off(k)]);
}
template <>
__device__ float PatchRows<float>::load1(const Row& row, int k) const {
  return row.p[pix_off(k)];
}

// ---------------------------------------------------------------------------
// Epilogues.  store(m, n, v, info) with info = the staged row's descriptor.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float gelu_exact(float x) {
  return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f));
}

template <typename TAct>
__device__ __forceinline__ void store_act(TAct* p, float v);
template <>
__device__ __forceinline__ void store_act<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_act<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

template <typename TAct, bool kGelu>
struct EpiAct {
  const float* bias;
  TAct* out;
  int ldc;
  __device__ void store(int m, int n, float v, int32_t) const {
    v += bias[n];
    if (kGelu) v = gelu_exact(v);
    store_act<TAct>(out + (size_t)m * ldc + n, v);
  }
};

struct EpiResidual {
  const float* bias;
  float* resid;
  int ldc;
  __device__ void store(int m, int n, float v, int32_t) const {
    float* p = resid + (size_t)m * ldc + n;
    *p = *p + (v + bias[n]);
  }
};

struct EpiEmbed {
  const float* bias;
  const float* pe_row;
  const float* pe_col;
  float* out;
  float* out2;
  int d;
  __device__ void store(int m, int n, float v, int32_t desc) const {
    const int D = d >> 1;
    float pe = (n < D) ? pe_row[tok_row(desc) * D + n] : pe_col[tok_col(desc) * D + (n - D)];
    v += bias[n] + pe;
    out[(size_t)m * d + n] = v;
    if (out2) out2[(size_t)m * d + n] = v;
  }
};

template <typename AL>
struct IsPatch { static constexpr bool value = false; };
template <typename T>
struct IsPatch<PatchRows<T>> { static constexpr bool value = true; };

template <typename AL>
__device__ __forceinline__ auto prepare_row(const AL& al, int m, bool& valid, int M) {
  if constexpr (IsPatch<AL>::value) {
    return al.prepare(m, valid);
  } else {
    return al.prepare(valid ? m : (M - 1));
  }
}

// ---------------------------------------------------------------------------
// bf16 MFMA kernel.  NWM x NWN wavefronts; each owns a (BM/NWM) x (BN/NWN) block
// of 32x32 MFMA tiles.  LDS holds two K-slabs of A and W (double buffer): while the
// MFMAs run on one, the next one travels global -> registers -> the other buffer,
// with a single barrier per slab.  All per-thread staging state lives in fully
// unrolled register arrays (no closures over them: those end up in scratch memory).
// ---------------------------------------------------------------------------
template <int BM, int BN>
constexpr size_t gemm_lds_bytes() {
  return (size_t)2 * (BM + BN) * LDS_LD * sizeof(bf16_t) + BM * sizeof(int32_t) + 16;
}

template <int BM, int BN, int NWM, int NWN, typename AL, typename EP>
__global__ __launch_bounds__(64 * NWM * NWN) void gemm_bf16_kernel(
    AL al, const bf16_t* __restrict__ W, int N, int K, EP ep, const int32_t* __restrict__ m_ptr,
    int m_host, const int32_t* tok_desc) {
  constexpr int THREADS = 64 * NWM * NWN;
  constexpr int WTM = BM / NWM, WTN = BN / NWN;   // wavefront tile
  constexpr int MT = WTM / 32, NT = WTN / 32;     // 32x32 tiles per wavefront, each way
  constexpr int PASS_ROWS = THREADS / 8;          // rows staged per pass (8 x 16 B per row)
  constexpr int A_LOADS = BM / PASS_ROWS, B_LOADS = BN / PASS_ROWS;
  static_assert(BM % PASS_ROWS == 0 && BN % PASS_ROWS == 0, "tile / thread mismatch");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_raw);          // [2][BM * LDS_LD]
  bf16_t* sB = sA + 2 * BM * LDS_LD;                         // [2][BN * LDS_LD]
  int32_t* s_desc = reinterpret_cast<int32_t*>(sB + 2 * BN * LDS_LD);   // [BM]
  int32_t* s_any = s_desc + BM;

  const int M = m_ptr ? *m_ptr : m_host;
  const int n_blocks = N / BN;
  const int total = ((M + BM - 1) / BM) * n_blocks;
  int pid = blockIdx.x;
  if (pid >= total) return;
  // Workgroups are dealt round-robin to the 8 XCDs.  Give each XCD a contiguous run
  // of tiles so that neighbours in tile order (same rows of A) share one L2.
  {
    const int per = total >> 3;
    if (pid < (per << 3)) pid = (pid & 7) * per + (pid >> 3);
  }
  const int m0 = (pid / n_blocks) * BM;
  const int n0 = (pid % n_blocks) * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / NWN, wn = wave % NWN;
  const int chunk = tid & 7;     // which 8-element piece of a 64-wide slab row
  const int srow = tid >> 3;     // staged row (plus PASS_ROWS * j)

  if (tid == 0) *s_any = 0;
  __syncthreads();
  typename AL::Row arow[A_LOADS];
  bool any_valid = false;
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int r = srow + PASS_ROWS * j;
    bool valid = (m0 + r) < M;
    arow[j] = prepare_row(al, m0 + r, valid, M);
    if (chunk == 0) {
      int32_t desc = -1;
      if (valid) desc = IsPatch<AL>::value ? tok_desc[m0 + r] : 0;
      s_desc[r] = desc;
    }
    any_valid |= valid;
  }
  if (IsPatch<AL>::value) {
    if (any_valid) *s_any = 1;
    __syncthreads();
    if (!*s_any) return;  // no token of this level in the tile
  }
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
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
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

  // C layout of the 32x32 MFMA: lane -> column l32, register r -> row 8*(r/4)+4*g+(r%4).
#pragma unroll
  for (int i = 0; i < MT; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int ml = wm * WTM + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
      const int32_t desc = s_desc[ml];
      if (desc < 0) continue;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int n = n0 + wn * WTN + j * 32 + l32;
        ep.store(m0 + ml, n, acc[i][j][r], desc);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// fp32 check-mode kernel: 64x64 tile, 256 threads, 4x4 outputs per thread.
// ---------------------------------------------------------------------------
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
  const int lrow = tid >> 2;        // staged row 0..63
  const int lk = (tid & 3) * 4;     // 4 consecutive k of a 16-wide slab
  if (tid == 0) s_any = 0;
  __syncthreads();
  bool valid = (m0 + lrow) < M;
  typename AL::Row arow = prepare_row(al, m0 + lrow, valid, M);
  if ((tid & 3) == 0) {
    int32_t desc = -1;
    if (valid) desc = IsPatch<AL>::value ? tok_desc[m0 + lrow] : 0;
    s_desc[lrow] = desc;
  }
  if (IsPatch<AL>::value) {
    if (valid) s_any = 1;
    __syncthreads();
    if (!s_any) return;
  }
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
#pragma unroll
    for (int q = 0; q < 4; ++q) ep.store(m0 + ml, n0 + tx * 4 + q, acc[p][q], desc);
  }
}

int ilog2(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

template <int BM, int BN, int NWM, int NWN, typename AL, typename EP>
hipError_t launch_bf16_tile(const AL& al, const bf16_t* w, int N, int K, const EP& ep,
                            const int32_t* m_ptr, int m_host, int m_capacity,
                            const int32_t* tok_desc, hipStream_t s) {
  auto kern = gemm_bf16_kernel<BM, BN, NWM, NWN, AL, EP>;
  constexpr size_t lds = gemm_lds_bytes<BM, BN>();
  static bool configured = false;   // per instantiation; the attribute is sticky
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  dim3 grid(((m_capacity + BM - 1) / BM) * (N / BN));
  hipLaunchKernelGGL(kern, grid, dim3(64 * NWM * NWN), lds, s, al, w, N, K, ep, m_ptr, m_host,
                     tok_desc);
  return hipSuccess;
}

template <typename AL, typename EP>
hipError_t launch_bf16(const AL& al, const void* W, int N, int K, const EP& ep,
                       const int32_t* m_ptr, int m_host, int m_capacity,
                       const int32_t* tok_desc, hipStream_t s) {
  const bf16_t* w = static_cast<const bf16_t*>(W);
  // Large tiles when they still give every CU work, small tiles otherwise.
  const long tiles128 = (long)((m_capacity + 127) / 128) * (N / 128);
  if (N % 128 == 0 && tiles128 >= 256)
    return launch_bf16_tile<128, 128, 2, 2>(al, w, N, K, ep, m_ptr, m_host, m_capacity, tok_desc, s);
  return launch_bf16_tile<64, 64, 2, 2>(al, w, N, K, ep, m_ptr, m_host, m_capacity, tok_desc, s);
}

template <typename AL, typename EP>
hipError_t launch_f32(const AL& al, const void* W, int N, int K, const EP& ep, const int32_t* m_ptr,
                int m_host, int m_capacity, const int32_t* tok_desc, hipStream_t s) {
  dim3 grid(((m_capacity + 63) / 64) * (N / 64));
  hipLaunchKernelGGL((gemm_f32_kernel<AL, EP>), grid, dim3(256), 0, s, al,
                     static_cast<const float*>(W), N, K, ep, m_ptr, m_host, tok_desc);
  return hipSuccess;
}

}  // namespace

hipError_t launch_embed(const EmbedArgs& a, const void* w, const float* bias, int d,
                        bool use_bf16, const int32_t* m_ptr, int m_host, int m_capacity,
                        hipStream_t s) {
  const int K = 3 * a.patch * a.patch;
  EpiEmbed ep{bias, a.pe_row, a.pe_col, a.out, a.out2, d};
  hipError_t e = hipSuccess;
  if (a.image_is_bf16) {
    PatchRows<bf16_t> al{static_cast<const bf16_t*>(a.images), a.tok_desc, a.cu_seqlens, a.B,
                         a.level, ilog2(a.patch), a.img_h, a.img_w};
    if (use_bf16) e = launch_bf16(al, w, d, K, ep, m_ptr, m_host, m_capacity, a.tok_desc, s);
    else e = launch_f32(al, w, d, K, ep, m_ptr, m_host, m_capacity, a.tok_desc, s);
  } else {
    PatchRows<float> al{static_cast<const float*>(a.images), a.tok_desc, a.cu_seqlens, a.B,
                        a.level, ilog2(a.patch), a.img_h, a.img_w};
    if (use_bf16) e = launch_bf16(al, w, d, K, ep, m_ptr, m_host, m_capacity, a.tok_desc, s);
    else e = launch_f32(al, w, d, K, ep, m_ptr, m_host, m_capacity, a.tok_desc, s);
  }
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

hipError_t launch_gemm(const void* A, const void* W, const float* bias, int N, int K,
                       Epilogue epi, void* out_act, float* resid, bool use_bf16,
                       const int32_t* m_ptr, int m_host, int m_capacity, hipStream_t s) {
  hipError_t e = hipSuccess;
  if (use_bf16) {
    PlainBf16 al{static_cast<const bf16_t*>(A), K};
    bf16_t* o = static_cast<bf16_t*>(out_act);
    switch (epi) {
      case Epilogue::kBias:
        e = launch_bf16(al, W, N, K, EpiAct<bf16_t, false>{bias, o, N}, m_ptr, m_host, m_capacity,
                    nullptr, s);
        break;
      case Epilogue::kBiasGelu:
        e = launch_bf16(al, W, N, K, EpiAct<bf16_t, true>{bias, o, N}, m_ptr, m_host, m_capacity,
                    nullptr, s);
        break;
      case Epilogue::kBiasResidual:
        e = launch_bf16(al, W, N, K, EpiResidual{bias, resid, N}, m_ptr, m_host, m_capacity, nullptr,
                    s);
        break;
    }
  } else {
    PlainF32 al{static_cast<const float*>(A), K};
    float* o = static_cast<float*>(out_act);
    switch (epi) {
      case Epilogue::kBias:
        e = launch_f32(al, W, N, K, EpiAct<float, false>{bias, o, N}, m_ptr, m_host, m_capacity,
                   nullptr, s);
        break;
      case Epilogue::kBiasGelu:
        e = launch_f32(al, W, N, K, EpiAct<float, true>{bias, o, N}, m_ptr, m_host, m_capacity,
                   nullptr, s);
        break;
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
