// Variable-length multi-head self-attention (Sec. II-A: every token attends to
// every token of its own frame; A3, Sec. III-B: several frames in one batch).
// Frames are addressed by offsets, so no padding token is ever computed.
//
// bf16 kernel, flash style.  A workgroup owns kBlockQ queries of one (frame, head);
// each of its four wavefronts owns 32 of them.  Keys/values are walked in tiles of
// 64 staged in LDS.  Everything is computed transposed so that a query is a LANE:
//   S^T[key, q] = K . Q^T          (MFMA A = K rows from LDS, B = Q rows in registers)
//   O^T[dh, q] += V^T . P^T        (MFMA A = V^T rows from LDS, B = P from registers)
// In the MFMA result layout a lane then holds 16 keys of ONE query, so the running
// max, the running sum and the rescale factor are per-lane scalars, the only
// cross-lane step is one exchange between lane l and l^32, and the probabilities
// feed the second MFMA straight from registers.  For that to work the 8 keys a
// lane contributes to one k-step must sit in 8 consecutive result registers: rows
// of a 32-key sub-tile are therefore staged in LDS with bits 2 and 3 of the key
// index swapped (result register r of lane group g holds row 8*(r/4)+4*g+r%4, which
// then is key 16*(r/8)+8*g+r%8).  V is staged transposed ([dh][key]) so that its
// operand read is one 16-byte access too.
//
// The fp32 kernel (check mode) is the same online softmax with one query per thread.
#include "kernels.h"

namespace cfdetr {

namespace {

constexpr int kBlockQ = 128;
constexpr int kBlockKV = 64;

__device__ __forceinline__ int swap_bits_2_3(int i) {
  return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1);
}

template <int DH>
__global__ __launch_bounds__(256) void attention_bf16_kernel(
    const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out, const int32_t* __restrict__ cu,
    int d, const int32_t* __restrict__ tiles, const int32_t* __restrict__ n_tiles,
    float scale_log2e) {
  constexpr int LDK = DH + 8;         // sK row stride (elements)
  constexpr int LDV = kBlockKV + 8;   // sVt row stride
  constexpr int KS = DH / 16;         // k-steps of Q.K^T
  constexpr int MO = DH / 32;         // 32-row blocks of O^T
  __shared__ __attribute__((aligned(16))) bf16_t sK[2 * kBlockKV * LDK];   // double buffer
  __shared__ __attribute__((aligned(16))) bf16_t sVt[2 * DH * LDV];

  if ((int)blockIdx.x >= *n_tiles) return;
  const int32_t tile = tiles[blockIdx.x];
  const int frame = tile >> 24, qt = tile & 0xFFFFFF;
  const int head = blockIdx.y;
  const int seq0 = cu[frame], T = cu[frame + 1] - seq0;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int ld = 3 * d;
  const bf16_t* qbase = qkv + (size_t)seq0 * ld + head * DH;
  const bf16_t* kbase = qbase + d;
  const bf16_t* vbase = qbase + 2 * d;

  // Q operand: lane = query, 8 consecutive dh per k-step.
  const int q_local = qt * kBlockQ + wave * 32 + l32;
  const int q_load = min(q_local, T - 1);
  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qf[ks] = *reinterpret_cast<const bf16x8*>(qbase + (size_t)q_load * ld + ks * 16 + g * 8);

  // Staging roles.  K: one 16-byte piece of one key row per thread and pass.
  constexpr int K_PIECES = DH / 8;
  constexpr int K_PASSES = kBlockKV * K_PIECES / 256;   // 2 for DH=64, 1 for DH=32
  const int k_piece = tid % K_PIECES, k_row = tid / K_PIECES;
  constexpr int K_ROWS_PER_PASS = 256 / K_PIECES;
  // V: one unit = 2 consecutive keys x 8 consecutive dh; 32 key pairs x DH/8 pieces.
  constexpr int V_UNITS = 32 * (DH / 8);
  const bool v_active = tid < V_UNITS;
  const int v_pair = tid & 31, v_piece = tid >> 5;

  // Global -> register fetch of one K/V tile and its (permuted / transposed) store to
  // LDS, written out twice below without closures so the registers stay registers.
  uint4 rk[K_PASSES], rv0 = make_uint4(0, 0, 0, 0), rv1 = make_uint4(0, 0, 0, 0);
#define CFDETR_ATTN_FETCH(kv0_)                                                              \
  do {                                                                                       \
    _Pragma("unroll") for (int p = 0; p < K_PASSES; ++p) {                                   \
      int key = min((kv0_) + k_row + p * K_ROWS_PER_PASS, T - 1);                            \
      rk[p] = *reinterpret_cast<const uint4*>(kbase + (size_t)key * ld + k_piece * 8);       \
    }                                                                                        \
    if (v_active) {                                                                          \
      int key0 = min((kv0_) + 2 * v_pair, T - 1), key1 = min((kv0_) + 2 * v_pair + 1, T - 1); \
      rv0 = *reinterpret_cast<const uint4*>(vbase + (size_t)key0 * ld + v_piece * 8);        \
      rv1 = *reinterpret_cast<const uint4*>(vbase + (size_t)key1 * ld + v_piece * 8);        \
    }                                                                                        \
  } while (0)
#define CFDETR_ATTN_STAGE(sk_, sv_)                                                          \
  do {                                                                                       \
    _Pragma("unroll") for (int p = 0; p < K_PASSES; ++p) {                                   \
      int r = k_row + p * K_ROWS_PER_PASS;                                                   \
      int rr = (r & 32) | swap_bits_2_3(r & 31);                                             \
      *reinterpret_cast<uint4*>((sk_) + rr * LDK + k_piece * 8) = rk[p];                     \
    }                                                                                        \
    if (v_active) {                                                                          \
      const uint32_t a0 = rv0.x, a1 = rv0.y, a2 = rv0.z, a3 = rv0.w;                         \
      const uint32_t b0 = rv1.x, b1 = rv1.y, b2 = rv1.z, b3 = rv1.w;                         \
      bf16_t* vd = (sv_) + (v_piece * 8) * LDV + 2 * v_pair;                                 \
      /* dh 2e: (key0,key1) from the low halves; dh 2e+1 from the high halves */             \
      *reinterpret_cast<uint32_t*>(vd + 0 * LDV) = (a0 & 0xFFFFu) | (b0 << 16);              \
      *reinterpret_cast<uint32_t*>(vd + 1 * LDV) = (a0 >> 16) | (b0 & 0xFFFF0000u);          \
      *reinterpret_cast<uint32_t*>(vd + 2 * LDV) = (a1 & 0xFFFFu) | (b1 << 16);              \
      *reinterpret_cast<uint32_t*>(vd + 3 * LDV) = (a1 >> 16) | (b1 & 0xFFFF0000u);          \
      *reinterpret_cast<uint32_t*>(vd + 4 * LDV) = (a2 & 0xFFFFu) | (b2 << 16);              \
      *reinterpret_cast<uint32_t*>(vd + 5 * LDV) = (a2 >> 16) | (b2 & 0xFFFF0000u);          \
      *reinterpret_cast<uint32_t*>(vd + 6 * LDV) = (a3 & 0xFFFFu) | (b3 << 16);              \
      *reinterpret_cast<uint32_t*>(vd + 7 * LDV) = (a3 >> 16) | (b3 & 0xFFFF0000u);          \
    }                                                                                        \
  } while (0)

  f32x16 acc_o[MO];
#pragma unroll
  for (int i = 0; i < MO; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_o[i][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  CFDETR_ATTN_FETCH(0);
  CFDETR_ATTN_STAGE(sK, sVt);
  __syncthreads();
  const int n_kv = (T + kBlockKV - 1) / kBlockKV;
  for (int it = 0; it < n_kv; ++it) {
    const int kv0 = it * kBlockKV;
    // the last pass refetches its own tile (unused): no conditionals around the registers
    const int kv_next = min(it + 1, n_kv - 1) * kBlockKV;
    CFDETR_ATTN_FETCH(kv_next);
    const bf16_t* cK = sK + (it & 1) * (kBlockKV * LDK);
    const bf16_t* cV = sVt + (it & 1) * (DH * LDV);

    // S^T for the two 32-key sub-tiles
    f32x16 s[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[sub][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 kf = *reinterpret_cast<const bf16x8*>(cK + (sub * 32 + l32) * LDK + ks * 16 + g * 8);
        s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[sub], 0, 0, 0);
      }
    }
    // mask keys past the end of the frame (last tile only)
    if (kv0 + kBlockKV > T) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int key = kv0 + sub * 32 + 16 * (r >> 3) + 8 * g + (r & 7);
          if (key >= T) s[sub][r] = -INFINITY;
        }
    }
    float m_tile = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) m_tile = fmaxf(m_tile, s[sub][r]);
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, kWave));
    const float m_new = fmaxf(m_run, m_tile);
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2e);
    const float mc = m_new * scale_log2e;
    const bool grew = m_new > m_run;
    m_run = m_new;
    float psum = 0.f;
    bf16x8 pf[2][2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float p0 = __builtin_amdgcn_exp2f(fmaf(s[sub][8 * t + 2 * e], scale_log2e, -mc));
          float p1 = __builtin_amdgcn_exp2f(fmaf(s[sub][8 * t + 2 * e + 1], scale_log2e, -mc));
          psum += p0 + p1;
          w[e] = pack_bf16x2(p0, p1);
        }
        uint4 packed = make_uint4(w[0], w[1], w[2], w[3]);
        pf[sub][t] = *reinterpret_cast<bf16x8*>(&packed);
      }
    l_run = l_run * alpha + psum;
    // Rescale the accumulators only when some query of the wavefront saw a new
    // maximum (alpha is exactly 1 otherwise); after the first tiles that is rare.
    if (__any(grew)) {
#pragma unroll
      for (int i = 0; i < MO; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[i][r] *= alpha;
    }
    // O^T += V^T . P^T
#pragma unroll
    for (int i = 0; i < MO; ++i)
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          bf16x8 vf = *reinterpret_cast<const bf16x8*>(cV + (i * 32 + l32) * LDV + sub * 32 +
                                                       t * 16 + g * 8);
          acc_o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sub][t], acc_o[i], 0, 0, 0);
        }
    CFDETR_ATTN_STAGE(sK + ((it + 1) & 1) * (kBlockKV * LDK), sVt + ((it + 1) & 1) * (DH * LDV));
    __syncthreads();
  }
#undef CFDETR_ATTN_FETCH
#undef CFDETR_ATTN_STAGE

  const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
  const float inv = 1.0f / l_tot;
  if (q_local < T) {
    bf16_t* orow = out + (size_t)(seq0 + q_local) * d + head * DH;
#pragma unroll
    for (int i = 0; i < MO; ++i)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        // registers 4*rq..4*rq+3 of lane group g are dh = 32*i + 8*rq + 4*g + 0..3
        uint2 w;
        w.x = pack_bf16x2(acc_o[i][4 * rq] * inv, acc_o[i][4 * rq + 1] * inv);
        w.y = pack_bf16x2(acc_o[i][4 * rq + 2] * inv, acc_o[i][4 * rq + 3] * inv);
        *reinterpret_cast<uint2*>(orow + i * 32 + rq * 8 + g * 4) = w;
      }
  }
}

// fp32 check mode: one query per thread, keys in tiles of 32 through LDS.
template <int DH>
__global__ __launch_bounds__(128) void attention_f32_kernel(
    const float* __restrict__ qkv, float* __restrict__ out, const int32_t* __restrict__ cu, int d,
    const int32_t* __restrict__ tiles, const int32_t* __restrict__ n_tiles, float scale) {
  constexpr int TK = 32;
  __shared__ float sK[TK][DH];
  __shared__ float sV[TK][DH];
  if ((int)blockIdx.x >= *n_tiles) return;
  const int32_t tile = tiles[blockIdx.x];
  const int frame = tile >> 24, qt = tile & 0xFFFFFF;
  const int head = blockIdx.y;
  const int seq0 = cu[frame], T = cu[frame + 1] - seq0;
  const int ld = 3 * d;
  const float* qbase = qkv + (size_t)seq0 * ld + head * DH;
  const int q_local = qt * kBlockQ + threadIdx.x;
  const int q_load = min(q_local, T - 1);
  float q[DH], o[DH];
#pragma unroll
  for (int i = 0; i < DH; ++i) {
    q[i] = qbase[(size_t)q_load * ld + i] * scale;
    o[i] = 0.f;
  }
  float m_run = -INFINITY, l_run = 0.f;
  for (int kv0 = 0; kv0 < T; kv0 += TK) {
    __syncthreads();
    for (int e = threadIdx.x; e < TK * DH; e += 128) {
      int r = e / DH, c = e - r * DH;
      int key = min(kv0 + r, T - 1);
      sK[r][c] = qbase[(size_t)key * ld + d + c];
      sV[r][c] = qbase[(size_t)key * ld + 2 * d + c];
    }
    __syncthreads();
    float s[TK];
    float m_tile = -INFINITY;
#pragma unroll
    for (int r = 0; r < TK; ++r) {
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < DH; ++i) acc = fmaf(q[i], sK[r][i], acc);
      s[r] = (kv0 + r < T) ? acc : -INFINITY;
      m_tile = fmaxf(m_tile, s[r]);
    }
    const float m_new = fmaxf(m_run, m_tile);
    const float alpha = expf(m_run - m_new);
    m_run = m_new;
    l_run *= alpha;
#pragma unroll
    for (int i = 0; i < DH; ++i) o[i] *= alpha;
#pragma unroll
    for (int r = 0; r < TK; ++r) {
      float p = expf(s[r] - m_new);
      l_run += p;
#pragma unroll
      for (int i = 0; i < DH; ++i) o[i] = fmaf(p, sV[r][i], o[i]);
    }
  }
  if (q_local < T) {
    float* orow = out + (size_t)(seq0 + q_local) * d + head * DH;
    const float inv = 1.0f / l_run;
#pragma unroll
    for (int i = 0; i < DH; ++i) orow[i] = o[i] * inv;
  }
}

}  // namespace

int attention_block_q(int, bool) { return kBlockQ; }

hipError_t launch_attention(const void* qkv, void* out, const int32_t* cu_seqlens, int B, int d,
                            int heads, const int32_t* tiles, const int32_t* n_tiles,
                            int tile_capacity, int block_q, bool use_bf16, hipStream_t s) {
  (void)B;
  if (block_q != kBlockQ) return hipErrorInvalidValue;
  const int dh = d / heads;
  const float scale = 1.0f / sqrtf((float)dh);
  dim3 grid(tile_capacity, heads);
  if (use_bf16) {
    const float c = scale * 1.44269504088896340736f;
    const bf16_t* in = static_cast<const bf16_t*>(qkv);
    bf16_t* o = static_cast<bf16_t*>(out);
    if (dh == 64)
      hipLaunchKernelGGL(attention_bf16_kernel<64>, grid, dim3(256), 0, s, in, o, cu_seqlens, d,
                         tiles, n_tiles, c);
    else if (dh == 32)
      hipLaunchKernelGGL(attention_bf16_kernel<32>, grid, dim3(256), 0, s, in, o, cu_seqlens, d,
                         tiles, n_tiles, c);
    else
      return hipErrorInvalidValue;
  } else {
    const float* in = static_cast<const float*>(qkv);
    float* o = static_cast<float*>(out);
    if (dh == 64)
      hipLaunchKernelGGL(attention_f32_kernel<64>, grid, dim3(128), 0, s, in, o, cu_seqlens, d,
                         tiles, n_tiles, scale);
    else if (dh == 32)
      hipLaunchKernelGGL(attention_f32_kernel<32>, grid, dim3(128), 0, s, in, o, cu_seqlens, d,
                         tiles, n_tiles, scale);
    else
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace cfdetr
