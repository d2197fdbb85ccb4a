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
// bf16 MFMA kernel.  256 threads = 4 wavefronts in a 2 x 2 arrangement.
// ---------------------------------------------------------------------------
template <int BM, int BN, typename AL, typename EP>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(AL al, const bf16_t* __restrict__ W,
                                                        int N, int K, EP ep,
                                                        const int32_t* __restrict__ m_ptr,
                                                        int m_host, const int32_t* tok_desc) {
  constexpr int MT = BM / 64, NT = BN / 64;       // 32x32 tiles per wavefront, each way
  constexpr int A_LOADS = BM / 32, B_LOADS = BN / 32;
  __shared__ __attribute__((aligned(16))) bf16_t sA[BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) bf16_t sB[BN * LDS_LD];
  __shared__ int32_t s_desc[BM];
  __shared__ int s_any;

  const int M = m_ptr ? *m_ptr : m_host;
  const int n_blocks = N / BN;
  const int m0 = (blockIdx.x / n_blocks) * BM;
  const int n0 = (blockIdx.x % n_blocks) * BN;
  if (m0 >= M) return;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int chunk = tid & 7;     // which 8-element piece of a 64-wide slab row
  const int srow = tid >> 3;     // staged row (plus 32*j)

  if (tid == 0) s_any = 0;
  __syncthreads();
  typename AL::Row arow[A_LOADS];
  bool any_valid = false;
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    int r = srow + 32 * j;
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
    if (any_valid) s_any = 1;
    __syncthreads();
    if (!s_any) return;  // no token of this level in the tile
  }
  const bf16_t* wrow[B_LOADS];
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) wrow[j] = W + (size_t)(n0 + srow + 32 * j) * K + chunk * 8;

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[A_LOADS], rb[B_LOADS];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) ra[j] = al.load8(arow[j], k0 + chunk * 8);
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) rb[j] = *reinterpret_cast<const uint4*>(wrow[j] + k0);
  };
  auto stage = [&]() {
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j)
      *reinterpret_cast<uint4*>(&sA[(srow + 32 * j) * LDS_LD + chunk * 8]) = ra[j];
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j)
      *reinterpret_cast<uint4*>(&sB[(srow + 32 * j) * LDS_LD + chunk * 8]) = rb[j];
  };

  const int l32 = lane & 31, g = lane >> 5;
  const bf16_t* pa = &sA[(wm * (BM / 2) + l32) * LDS_LD + g * 8];
  const bf16_t* pb = &sB[(wn * (BN / 2) + l32) * LDS_LD + g * 8];

  fetch(0);
  stage();
  __syncthreads();
  for (int k0 = 0; k0 < K; k0 += BK) {
    const bool more = (k0 + BK) < K;
    if (more) fetch(k0 + BK);
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
    __syncthreads();
    if (more) {
      stage();
      __syncthreads();
    }
  }

  // C layout of the 32x32 MFMA: lane -> column l32, register r -> row 8*(r/4)+4*g+(r%4).
#pragma unroll
  for (int i = 0; i < MT; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int ml = wm * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
      const int32_t desc = s_desc[ml];
      if (desc < 0) continue;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int n = n0 + wn * (BN / 2) + j * 32 + l32;
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

template <typename AL, typename EP>
void launch_bf16(const AL& al, const void* W, int N, int K, const EP& ep, const int32_t* m_ptr,
                 int m_host, int m_capacity, const int32_t* tok_desc, hipStream_t s) {
  const bf16_t* w = static_cast<const bf16_t*>(W);
  // Large tiles when they still give every CU work, small tiles otherwise.
  const long tiles128 = (long)((m_capacity + 127) / 128) * (N / 128);
  if (N % 128 == 0 && tiles128 >= 512) {
    dim3 grid(((m_capacity + 127) / 128) * (N / 128));
    hipLaunchKernelGGL((gemm_bf16_kernel<128, 128, AL, EP>), grid, dim3(256), 0, s, al, w, N, K,
                       ep, m_ptr, m_host, tok_desc);
  } else {
    dim3 grid(((m_capacity + 63) / 64) * (N / 64));
    hipLaunchKernelGGL((gemm_bf16_kernel<64, 64, AL, EP>), grid, dim3(256), 0, s, al, w, N, K, ep,
                       m_ptr, m_host, tok_desc);
  }
}

template <typename AL, typename EP>
void launch_f32(const AL& al, const void* W, int N, int K, const EP& ep, const int32_t* m_ptr,
                int m_host, int m_capacity, const int32_t* tok_desc, hipStream_t s) {
  dim3 grid(((m_capacity + 63) / 64) * (N / 64));
  hipLaunchKernelGGL((gemm_f32_kernel<AL, EP>), grid, dim3(256), 0, s, al,
                     static_cast<const float*>(W), N, K, ep, m_ptr, m_host, tok_desc);
}

}  // namespace

hipError_t launch_embed(const EmbedArgs& a, const void* w, const float* bias, int d,
                        bool use_bf16, const int32_t* m_ptr, int m_host, int m_capacity,
                        hipStream_t s) {
  const int K = 3 * a.patch * a.patch;
  EpiEmbed ep{bias, a.pe_row, a.pe_col, a.out, a.out2, d};
  if (a.image_is_bf16) {
    PatchRows<bf16_t> al{static_cast<const bf16_t*>(a.images), a.tok_desc, a.cu_seqlens, a.B,
                         a.level, ilog2(a.patch), a.img_h, a.img_w};
    if (use_bf16) launch_bf16(al, w, d, K, ep, m_ptr, m_host, m_capacity, a.tok_desc, s);
    else launch_f32(al, w, d, K, ep, m_ptr, m_host, m_capacity, a.tok_desc, s);
  } else {
    PatchRows<float> al{static_cast<const float*>(a.images), a.tok_desc, a.cu_seqlens, a.B,
                        a.level, ilog2(a.patch), a.img_h, a.img_w};
    if (use_bf16) launch_bf16(al, w, d, K, ep, m_ptr, m_host, m_capacity, a.tok_desc, s);
    else launch_f32(al, w, d, K, ep, m_ptr, m_host, m_capacity, a.tok_desc, s);
  }
  return hipGetLastError();
}

hipError_t launch_gemm(const void* A, const void* W, const float* bias, int N, int K,
                       Epilogue epi, void* out_act, float* resid, bool use_bf16,
                       const int32_t* m_ptr, int m_host, int m_capacity, hipStream_t s) {
  if (use_bf16) {
    PlainBf16 al{static_cast<const bf16_t*>(A), K};
    bf16_t* o = static_cast<bf16_t*>(out_act);
    switch (epi) {
      case Epilogue::kBias:
        launch_bf16(al, W, N, K, EpiAct<bf16_t, false>{bias, o, N}, m_ptr, m_host, m_capacity,
                    nullptr, s);
        break;
      case Epilogue::kBiasGelu:
        launch_bf16(al, W, N, K, EpiAct<bf16_t, true>{bias, o, N}, m_ptr, m_host, m_capacity,
                    nullptr, s);
        break;
      case Epilogue::kBiasResidual:
        launch_bf16(al, W, N, K, EpiResidual{bias, resid, N}, m_ptr, m_host, m_capacity, nullptr,
                    s);
        break;
    }
  } else {
    PlainF32 al{static_cast<const float*>(A), K};
    float* o = static_cast<float*>(out_act);
    switch (epi) {
      case Epilogue::kBias:
        launch_f32(al, W, N, K, EpiAct<float, false>{bias, o, N}, m_ptr, m_host, m_capacity,
                   nullptr, s);
        break;
      case Epilogue::kBiasGelu:
        launch_f32(al, W, N, K, EpiAct<float, true>{bias, o, N}, m_ptr, m_host, m_capacity,
                   nullptr, s);
        break;
      case Epilogue::kBiasResidual:
        launch_f32(al, W, N, K, EpiResidual{bias, resid, N}, m_ptr, m_host, m_capacity, nullptr,
                   s);
        break;
    }
  }
  return hipGetLastError();
}

}  // namespace cfdetr
