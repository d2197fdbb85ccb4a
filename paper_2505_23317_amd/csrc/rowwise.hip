// Row-wise kernels: position tables, LayerNorm, reuse of cached coarse tokens.
#include "kernels.h"

namespace cfdetr {

namespace {

// Centre-based 2-D sinusoidal position, separable: the first half of a token's
// vector depends on its row only, the second half on its column only.  With
// D = d/2 and pair index j = i/2 < D/2 the frequency is 10000^(-2j/D); even i
// holds sin, odd i holds cos of 2*pi*coord*frequency, coord = (index+0.5)*P/extent.
// Evaluated once, in double, at context creation.
__global__ void pe_table_kernel(int patch, int count, int extent, int D,
                                float* __restrict__ table) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= count * D) return;
  int cell = idx / D, i = idx - cell * D;
  double coord = (cell + 0.5) * (double)patch / (double)extent;
  double omega = pow(10000.0, -2.0 * (double)(i >> 1) / (double)D);
  double arg = 2.0 * 3.14159265358979323846 * coord * omega;
  table[idx] = (float)((i & 1) ? cos(arg) : sin(arg));
}

constexpr int kLnMaxPairs = 8;  // pairs of elements per lane: d <= 1024

__device__ __forceinline__ void store_pair(float* p, float a, float b) {
  *reinterpret_cast<float2*>(p) = make_float2(a, b);
}
__device__ __forceinline__ void store_pair(bf16_t* p, float a, float b) {
  *reinterpret_cast<uint32_t*>(p) = pack_bf16x2(a, b);
}

// One wavefront per row; the row lives in registers (two elements per lane and step)
// between the two passes: mean first, then the variance of the centred values.
template <typename TOut>
__global__ __launch_bounds__(256) void layernorm_kernel(
    const float* __restrict__ x, const float* __restrict__ g, const float* __restrict__ b,
    TOut* __restrict__ out, int d, float eps, const int32_t* __restrict__ m_ptr, int m_host,
    int split_row, TOut* __restrict__ out2) {
  const int M = m_ptr ? *m_ptr : m_host;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const int lane = threadIdx.x & 63;
  const int pairs = d >> 1;
  const float2* xr = reinterpret_cast<const float2*>(x + (size_t)row * d);
  float2 v[kLnMaxPairs];
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < kLnMaxPairs; ++j) {
    const int i = lane + 64 * j;
    v[j] = (i < pairs) ? xr[i] : make_float2(0.f, 0.f);
    sum += v[j].x + v[j].y;
  }
  const float mean = wave_sum(sum) / (float)d;
  float sq = 0.f;
#pragma unroll
  for (int j = 0; j < kLnMaxPairs; ++j) {
    if (lane + 64 * j < pairs) {
      const float cx = v[j].x - mean, cy = v[j].y - mean;
      sq += cx * cx + cy * cy;
    }
  }
  const float rstd = rsqrtf(wave_sum(sq) / (float)d + eps);
  TOut* orow = (out2 != nullptr && row >= split_row) ? out2 + (size_t)(row - split_row) * d
                                                     : out + (size_t)row * d;
  const float2* g2 = reinterpret_cast<const float2*>(g);
  const float2* b2 = reinterpret_cast<const float2*>(b);
#pragma unroll
  for (int j = 0; j < kLnMaxPairs; ++j) {
    const int i = lane + 64 * j;
    if (i < pairs) {
      const float2 gg = g2[i], bb = b2[i];
      store_pair(orow + 2 * i, (v[j].x - mean) * rstd * gg.x + bb.x,
                 (v[j].y - mean) * rstd * gg.y + bb.y);
    }
  }
}

// The same with four elements per lane and step (16-byte loads, 8- or 16-byte stores), for
// widths that are a multiple of four.  (Two rows per wavefront, both requested before either
// is reduced, measured no faster.)
constexpr int kLnMaxQuads = kLnMaxPairs / 2;

__device__ __forceinline__ void store_quad(float* p, float a, float b, float c, float d) {
  *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
}
__device__ __forceinline__ void store_quad(bf16_t* p, float a, float b, float c, float d) {
  *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(a, b), pack_bf16x2(c, d));
}

template <typename TOut>
__global__ __launch_bounds__(256) void layernorm4_kernel(
    const float* __restrict__ x, const float* __restrict__ g, const float* __restrict__ b,
    TOut* __restrict__ out, int d, float eps, const int32_t* __restrict__ m_ptr, int m_host,
    int split_row, TOut* __restrict__ out2, RowPositions rp) {
  const int M = m_ptr ? *m_ptr : m_host;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const int lane = threadIdx.x & 63;
  if (rp.out != nullptr && lane == 0) {
    // position of the row in the feature-major copy of V, for the projections that follow
    const int f = frame_of_token(rp.cu, rp.nseq, row);
    rp.out[row] = rp.pcu[f] + (row - rp.cu[f]);
  }
  const int quads = d >> 2;
  const float4* xr = reinterpret_cast<const float4*>(x + (size_t)row * d);
  float4 v[kLnMaxQuads];
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < kLnMaxQuads; ++j) {
    const int i = lane + 64 * j;
    v[j] = (i < quads) ? xr[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    sum += (v[j].x + v[j].y) + (v[j].z + v[j].w);
  }
  const float mean = wave_sum(sum) / (float)d;
  float sq = 0.f;
#pragma unroll
  for (int j = 0; j < kLnMaxQuads; ++j) {
    if (lane + 64 * j < quads) {
      const float cx = v[j].x - mean, cy = v[j].y - mean, cz = v[j].z - mean, cw = v[j].w - mean;
      sq += (cx * cx + cy * cy) + (cz * cz + cw * cw);
    }
  }
  const float rstd = rsqrtf(wave_sum(sq) / (float)d + eps);
  TOut* orow = (out2 != nullptr && row >= split_row) ? out2 + (size_t)(row - split_row) * d
                                                     : out + (size_t)row * d;
  const float4* g4 = reinterpret_cast<const float4*>(g);
  const float4* b4 = reinterpret_cast<const float4*>(b);
#pragma unroll
  for (int j = 0; j < kLnMaxQuads; ++j) {
    const int i = lane + 64 * j;
    if (i < quads) {
      const float4 gg = g4[i], bb = b4[i];
      store_quad(orow + 4 * i, (v[j].x - mean) * rstd * gg.x + bb.x,
                 (v[j].y - mean) * rstd * gg.y + bb.y, (v[j].z - mean) * rstd * gg.z + bb.z,
                 (v[j].w - mean) * rstd * gg.w + bb.w);
    }
  }
}

// One wavefront per token: level-0 tokens take their row of the coarse cache.
__global__ __launch_bounds__(256) void gather_coarse_kernel(
    const int32_t* __restrict__ tok_desc, const int32_t* __restrict__ cu, int B,
    const float* __restrict__ x0, int n0, int cols0, int d, float* __restrict__ x) {
  const int M = cu[B];
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= M) return;
  const int32_t desc = tok_desc[t];
  if (tok_level(desc) != 0) return;
  const int frame = frame_of_token(cu, B, t);
  const float* src = x0 + ((size_t)frame * n0 + tok_row(desc) * cols0 + tok_col(desc)) * d;
  float* dst = x + (size_t)t * d;
  for (int e = (threadIdx.x & 63) * 4; e < d; e += 256)
    *reinterpret_cast<float4*>(dst + e) = *reinterpret_cast<const float4*>(src + e);
}

__global__ __launch_bounds__(256) void cast_bf16_kernel(const float* __restrict__ in,
                                                        bf16_t* __restrict__ out, int d,
                                                        const int32_t* __restrict__ m_ptr) {
  const size_t n = (size_t)(*m_ptr) * d;
  const size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 8;
  if (i >= n) return;   // d is a multiple of 64, so n is a multiple of 8
  const float4 a = *reinterpret_cast<const float4*>(in + i);
  const float4 b = *reinterpret_cast<const float4*>(in + i + 4);
  *reinterpret_cast<uint4*>(out + i) = make_uint4(pack_bf16x2(a.x, a.y), pack_bf16x2(a.z, a.w),
                                                  pack_bf16x2(b.x, b.y), pack_bf16x2(b.z, b.w));
}

__global__ __launch_bounds__(256) void broadcast_rows_kernel(const float* __restrict__ src,
                                                             float* __restrict__ dst, int n4) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n4)
    reinterpret_cast<float4*>(dst)[(size_t)blockIdx.y * n4 + i] =
        reinterpret_cast<const float4*>(src)[i];
}

// One wavefront per query row: five dot products of length d, then the logistic function.
__global__ __launch_bounds__(256) void decoder_heads_kernel(
    const bf16_t* __restrict__ z, const bf16_t* __restrict__ hb, const bf16_t* __restrict__ w_cls,
    const float* __restrict__ b_cls, const bf16_t* __restrict__ w_box,
    const float* __restrict__ b_box, int d, int M, float* __restrict__ out) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const int lane = threadIdx.x & 63;
  float acc[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
  for (int e = lane; e < d; e += 64) {
    const float hv = bf16_to_f32(hb[(size_t)row * d + e]);
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = fmaf(hv, bf16_to_f32(w_box[(size_t)c * d + e]), acc[c]);
    acc[4] = fmaf(bf16_to_f32(z[(size_t)row * d + e]), bf16_to_f32(w_cls[e]), acc[4]);
  }
#pragma unroll
  for (int c = 0; c < 5; ++c) acc[c] = wave_sum(acc[c]);
  if (lane < 5) {
    const float u = acc[lane] + (lane < 4 ? b_box[lane] : b_cls[0]);
    out[(size_t)row * 5 + lane] = 1.0f / (1.0f + __expf(-u));
  }
}

}  // namespace

hipError_t launch_cast_bf16(const float* in, void* out, int d, const int32_t* m_ptr,
                            int m_capacity, hipStream_t s) {
  const size_t n8 = ((size_t)m_capacity * d + 7) / 8;
  hipLaunchKernelGGL(cast_bf16_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, s, in,
                     static_cast<bf16_t*>(out), d, m_ptr);
  return hipGetLastError();
}

hipError_t launch_broadcast_rows(const float* src, float* dst, int rows, int d, int copies,
                                 hipStream_t s) {
  const int n4 = rows * d / 4;
  hipLaunchKernelGGL(broadcast_rows_kernel, dim3((n4 + 255) / 256, copies), dim3(256), 0, s, src,
                     dst, n4);
  return hipGetLastError();
}

hipError_t launch_decoder_heads(const void* z, const void* hb, const void* w_cls,
                                const float* b_cls, const void* w_box, const float* b_box, int d,
                                int M, float* out, hipStream_t s) {
  hipLaunchKernelGGL(decoder_heads_kernel, dim3((M + 3) / 4), dim3(256), 0, s,
                     static_cast<const bf16_t*>(z), static_cast<const bf16_t*>(hb),
                     static_cast<const bf16_t*>(w_cls), b_cls, static_cast<const bf16_t*>(w_box),
                     b_box, d, M, out);
  return hipGetLastError();
}

hipError_t launch_pe_tables(int patch, int rows, int cols, int img_h, int img_w, int d,
                            float* pe_row, float* pe_col, hipStream_t s) {
  const int D = d / 2;
  hipLaunchKernelGGL(pe_table_kernel, dim3((rows * D + 255) / 256), dim3(256), 0, s, patch,
                     rows, img_h, D, pe_row);
  hipLaunchKernelGGL(pe_table_kernel, dim3((cols * D + 255) / 256), dim3(256), 0, s, patch,
                     cols, img_w, D, pe_col);
  return hipGetLastError();
}

hipError_t launch_layernorm(const float* x, const float* g, const float* b, void* out,
                            bool out_is_bf16, int d, float eps, const int32_t* m_ptr,
                            int m_host, int m_capacity, int split_row, void* out2,
                            hipStream_t s, const RowPositions* positions) {
  dim3 grid((m_capacity + 3) / 4);
  const RowPositions none{nullptr, nullptr, nullptr, 0};
  if (d % 4 == 0) {
    const RowPositions rp = positions ? *positions : none;
    if (out_is_bf16)
      hipLaunchKernelGGL(layernorm4_kernel<bf16_t>, grid, dim3(256), 0, s, x, g, b,
                         static_cast<bf16_t*>(out), d, eps, m_ptr, m_host, split_row,
                         static_cast<bf16_t*>(out2), rp);
    else
      hipLaunchKernelGGL(layernorm4_kernel<float>, grid, dim3(256), 0, s, x, g, b,
                         static_cast<float*>(out), d, eps, m_ptr, m_host, split_row,
                         static_cast<float*>(out2), rp);
    return hipGetLastError();
  }
  if (positions) return hipErrorInvalidValue;
  if (out_is_bf16)
    hipLaunchKernelGGL(layernorm_kernel<bf16_t>, grid, dim3(256), 0, s, x, g, b,
                       static_cast<bf16_t*>(out), d, eps, m_ptr, m_host, split_row,
                       static_cast<bf16_t*>(out2));
  else
    hipLaunchKernelGGL(layernorm_kernel<float>, grid, dim3(256), 0, s, x, g, b,
                       static_cast<float*>(out), d, eps, m_ptr, m_host, split_row,
                       static_cast<float*>(out2));
  return hipGetLastError();
}

hipError_t launch_gather_coarse(const int32_t* tok_desc, const int32_t* cu_seqlens, int B,
                                const float* x0, int n0, int cols0, int d, float* x,
                                int m_capacity, hipStream_t s) {
  hipLaunchKernelGGL(gather_coarse_kernel, dim3((m_capacity + 3) / 4), dim3(256), 0, s,
                     tok_desc, cu_seqlens, B, x0, n0, cols0, d, x);
  return hipGetLastError();
}

}  // namespace cfdetr
