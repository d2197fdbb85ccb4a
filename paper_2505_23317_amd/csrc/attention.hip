// Variable-length multi-head self-attention (Sec. II-A: every token attends to
// every token of its own frame; A3, Sec. III-B: several frames in one batch).
// Frames are addressed by offsets, so no padding token is ever computed.
//
// bf16 kernel, flash style.  A workgroup owns 128*QW queries of one (frame, head);
// each of its four wavefronts owns QW groups of 32 of them.  Keys/values are walked
// in tiles of 64 that go from global memory straight into LDS (global_load_lds,
// double-buffered, one barrier per tile).  Everything is computed transposed so that
// a query is a LANE:
//   S^T[key, q] = K . Q^T          (MFMA A = K rows from LDS, B = Q rows in registers)
//   O^T[dh, q] += V^T . P^T        (MFMA A = V^T rows from LDS, B = P from registers)
// In the MFMA result layout a lane then holds 16 keys of ONE query, so the running
// max, the running sum and the rescale factor are per-lane scalars, the only
// cross-lane step is one exchange between lane l and l^32, and the probabilities
// feed the second MFMA straight from registers.  For that to work the 8 keys a
// lane contributes to one k-step must sit in 8 consecutive result registers: LDS row
// rho of a 32-key sub-tile therefore holds the key whose index is rho with bits 2
// and 3 swapped (result register r of lane group g holds row 8*(r/4)+4*g+r%4, which
// then is key 16*(r/8)+8*g+r%8); with direct loads that permutation is free, the
// lane that fills row rho simply fetches that key.  V^T comes from a feature-major
// copy of V ([d][positions], each frame padded to a multiple of 64 positions) that
// the QKV projection writes, so its tiles are plain row copies too.  LDS rows are
// unpadded; 16-byte chunks are XOR-swizzled by row so that operand reads of 16
// consecutive rows hit disjoint banks.
//
// The fp32 kernel (check mode) is the same online softmax with one query per thread.
#include "kernels.h"

namespace cfdetr {

namespace {

constexpr int kBlockKV = 64;

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

__device__ __forceinline__ int swap_bits_2_3(int i) {
  return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1);
}

// Swizzle key of LDS row r: 128-byte rows have 8 chunks and two rows cover the 64
// banks, 64-byte rows have 4 chunks and four rows cover them.
template <int ROWB>
__device__ __forceinline__ int swz(int r) {
  return ROWB == 128 ? ((r >> 1) & 7) : ((r >> 2) & 3);
}

template <int DH, int QW>
__global__ __launch_bounds__(256) void attention_bf16_kernel(
    const bf16_t* __restrict__ qk, const bf16_t* __restrict__ vt, int vt_ld,
    bf16_t* __restrict__ out, const int32_t* __restrict__ cu, const int32_t* __restrict__ pcu,
    int d, const int32_t* __restrict__ items, float scale_log2e) {
  constexpr int BQ = 128 * QW;
  constexpr int KS = DH / 16;          // k-steps of Q.K^T
  constexpr int MO = DH / 32;          // 32-row blocks of O^T
  constexpr int KROWB = DH * 2;        // bytes per K row in LDS
  constexpr int KCPR = KROWB / 16;     // chunks per K row
  constexpr int KRPI = 1024 / KROWB;   // K rows per wave load instruction
  constexpr int KI = kBlockKV / KRPI / 4;   // K load instructions per wavefront
  constexpr int VI = DH / 8 / 4;            // V^T load instructions per wavefront (8 rows each)
  constexpr int KBYTES = kBlockKV * KROWB, VBYTES = DH * 128;
  __shared__ __attribute__((aligned(1024))) unsigned char sK[2 * KBYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char sV[2 * VBYTES];

  const int32_t item = items[blockIdx.x];
  if (item < 0) return;
  const int frame = item >> 24, head = (item >> 19) & 31, qt = item & 0x7FFFF;
  const int seq0 = cu[frame], T = cu[frame + 1] - seq0;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int ld = 3 * d;
  const bf16_t* qbase = qk + (size_t)seq0 * ld + head * DH;
  const bf16_t* kbase = qbase + d;

  // Q operands: lane = query, 8 consecutive dh per k-step.
  bf16x8 qf[QW][KS];
#pragma unroll
  for (int qs = 0; qs < QW; ++qs) {
    const int q_load = min(qt * BQ + (wave * QW + qs) * 32 + l32, T - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[qs][ks] = *reinterpret_cast<const bf16x8*>(qbase + (size_t)q_load * ld + ks * 16 + g * 8);
  }

  // Loader roles.  K: LDS row rho <- key (rho & 32) | swap23(rho & 31), chunk swizzled.
  int k_key[KI];
  int k_chunk[KI];
#pragma unroll
  for (int j = 0; j < KI; ++j) {
    const int rho = (wave * KI + j) * KRPI + lane / KCPR;
    k_key[j] = (rho & 32) | swap_bits_2_3(rho & 31);
    k_chunk[j] = (lane % KCPR) ^ swz<KROWB>(rho);
  }
  // V^T: LDS row rho = dh index; 64 keys = 8 chunks of 8.
  const bf16_t* v_src[VI];
#pragma unroll
  for (int j = 0; j < VI; ++j) {
    const int rho = (wave * VI + j) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ swz<128>(rho);
    v_src[j] = vt + (size_t)(head * DH + rho) * vt_ld + pcu[frame] + chunk * 8;
  }

#define CFDETR_ATTN_ISSUE(kv0_, buf_)                                                        \
  do {                                                                                       \
    _Pragma("unroll") for (int j = 0; j < KI; ++j) {                                         \
      const int key = min((kv0_) + k_key[j], T - 1);                                         \
      __builtin_amdgcn_global_load_lds(                                                      \
          (global_void_ptr)(kbase + (size_t)key * ld + k_chunk[j] * 8),                      \
          (lds_void_ptr)(sK + (buf_) * KBYTES + (wave * KI + j) * 1024), 16, 0, 0);          \
    }                                                                                        \
    _Pragma("unroll") for (int j = 0; j < VI; ++j) __builtin_amdgcn_global_load_lds(         \
        (global_void_ptr)(v_src[j] + (kv0_)),                                                \
        (lds_void_ptr)(sV + (buf_) * VBYTES + (wave * VI + j) * 1024), 16, 0, 0);            \
  } while (0)

  f32x16 acc_o[QW][MO];
  float m_run[QW], l_run[QW];
#pragma unroll
  for (int qs = 0; qs < QW; ++qs) {
    m_run[qs] = -INFINITY;
    l_run[qs] = 0.f;
#pragma unroll
    for (int i = 0; i < MO; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_o[qs][i][r] = 0.f;
  }

  const int n_kv = (T + kBlockKV - 1) / kBlockKV;
  CFDETR_ATTN_ISSUE(0, 0);
  for (int it = 0; it < n_kv; ++it) {
    const int kv0 = it * kBlockKV;
    // vmcnt(0): this wavefront's part of tile `it` is in LDS; the barrier publishes
    // every wavefront's part and retires all reads of the other buffer.
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (it + 1 < n_kv) CFDETR_ATTN_ISSUE(kv0 + kBlockKV, (it + 1) & 1);
    const unsigned char* cK = sK + (it & 1) * KBYTES;
    const unsigned char* cV = sV + (it & 1) * VBYTES;

    // S^T for the two 32-key sub-tiles
    f32x16 s[QW][2];
#pragma unroll
    for (int qs = 0; qs < QW; ++qs)
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[qs][sub][r] = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const int rho = sub * 32 + l32;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(
            cK + rho * KROWB + (((2 * ks + g) ^ swz<KROWB>(rho)) << 4));
#pragma unroll
        for (int qs = 0; qs < QW; ++qs)
          s[qs][sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qs][ks], s[qs][sub], 0, 0, 0);
      }
    }
    // mask keys past the end of the frame (last tile only)
    if (kv0 + kBlockKV > T) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + sub * 32 + 16 * (r >> 3) + 8 * g + (r & 7);
          if (key >= T) {
#pragma unroll
            for (int qs = 0; qs < QW; ++qs) s[qs][sub][r] = -INFINITY;
          }
        }
    }
    bf16x8 pf[QW][2][2];
#pragma unroll
    for (int qs = 0; qs < QW; ++qs) {
      float m_tile = -INFINITY;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) m_tile = fmaxf(m_tile, s[qs][sub][r]);
      m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, kWave));
      const float m_new = fmaxf(m_run[qs], m_tile);
      const float alpha = __builtin_amdgcn_exp2f((m_run[qs] - m_new) * scale_log2e);
      const float mc = m_new * scale_log2e;
      const bool grew = m_new > m_run[qs];
      m_run[qs] = m_new;
      float psum = 0.f;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          uint32_t w[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(s[qs][sub][8 * t + 2 * e], scale_log2e, -mc));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(s[qs][sub][8 * t + 2 * e + 1], scale_log2e, -mc));
            psum += p0 + p1;
            w[e] = pack_bf16x2(p0, p1);
          }
          uint4 packed = make_uint4(w[0], w[1], w[2], w[3]);
          pf[qs][sub][t] = *reinterpret_cast<bf16x8*>(&packed);
        }
      l_run[qs] = l_run[qs] * alpha + psum;
      // Rescale the accumulators only when some query of the wavefront saw a new
      // maximum (alpha is exactly 1 otherwise); after the first tiles that is rare.
      if (__any(grew)) {
#pragma unroll
        for (int i = 0; i < MO; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_o[qs][i][r] *= alpha;
      }
    }
    // O^T += V^T . P^T
#pragma unroll
    for (int i = 0; i < MO; ++i) {
      const int rho = i * 32 + l32;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const bf16x8 vf = *reinterpret_cast<const bf16x8*>(
              cV + rho * 128 + (((4 * sub + 2 * t + g) ^ swz<128>(rho)) << 4));
#pragma unroll
          for (int qs = 0; qs < QW; ++qs)
            acc_o[qs][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qs][sub][t], acc_o[qs][i], 0, 0, 0);
        }
    }
  }
#undef CFDETR_ATTN_ISSUE

#pragma unroll
  for (int qs = 0; qs < QW; ++qs) {
    const float l_tot = l_run[qs] + __shfl_xor(l_run[qs], 32, kWave);
    const float inv = 1.0f / l_tot;
    const int q_local = qt * BQ + (wave * QW + qs) * 32 + l32;
    if (q_local < T) {
      bf16_t* orow = out + (size_t)(seq0 + q_local) * d + head * DH;
#pragma unroll
      for (int i = 0; i < MO; ++i)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          // registers 4*rq..4*rq+3 of lane group g are dh = 32*i + 8*rq + 4*g + 0..3
          uint2 w;
          w.x = pack_bf16x2(acc_o[qs][i][4 * rq] * inv, acc_o[qs][i][4 * rq + 1] * inv);
          w.y = pack_bf16x2(acc_o[qs][i][4 * rq + 2] * inv, acc_o[qs][i][4 * rq + 3] * inv);
          *reinterpret_cast<uint2*>(orow + i * 32 + rq * 8 + g * 4) = w;
        }
    }
  }
}

// fp32 check mode: one query per thread, keys in tiles of 32 through LDS.
template <int DH>
__global__ __launch_bounds__(256) void attention_f32_kernel(
    const float* __restrict__ qkv, float* __restrict__ out, const int32_t* __restrict__ cu, int d,
    const int32_t* __restrict__ items, float scale) {
  constexpr int TK = 32;
  __shared__ float sK[TK][DH];
  __shared__ float sV[TK][DH];
  const int32_t item = items[blockIdx.x];
  if (item < 0) return;
  const int frame = item >> 24, head = (item >> 19) & 31, qt = item & 0x7FFFF;
  const int seq0 = cu[frame], T = cu[frame + 1] - seq0;
  const int ld = 3 * d;
  const float* qbase = qkv + (size_t)seq0 * ld + head * DH;
  const int q_local = qt * (int)blockDim.x + threadIdx.x;   // block size = queries per tile
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
    for (int e = threadIdx.x; e < TK * DH; e += blockDim.x) {
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

int attention_block_q(int d_head, bool use_bf16, int tokens_per_frame) {
  (void)d_head;
  (void)use_bf16;
  (void)tokens_per_frame;
  return 128;
}

hipError_t launch_attention(const void* qkv, const void* vt, int vt_ld, void* out,
                            const int32_t* cu_seqlens, const int32_t* pcu, int d, int heads,
                            const int32_t* items, int cap8, int block_q, bool use_bf16,
                            hipStream_t s) {
  if (block_q != 128 && block_q != 256) return hipErrorInvalidValue;
  const int dh = d / heads;
  const float scale = 1.0f / sqrtf((float)dh);
  dim3 grid(8 * cap8);
  if (use_bf16) {
    const float c = scale * 1.44269504088896340736f;
    const bf16_t* in = static_cast<const bf16_t*>(qkv);
    const bf16_t* v = static_cast<const bf16_t*>(vt);
    bf16_t* o = static_cast<bf16_t*>(out);
#define CFDETR_LAUNCH_ATTN(DH_, QW_)                                                          \
  hipLaunchKernelGGL((attention_bf16_kernel<DH_, QW_>), grid, dim3(256), 0, s, in, v, vt_ld, o, \
                     cu_seqlens, pcu, d, items, c)
    if (dh == 64 && block_q == 256) CFDETR_LAUNCH_ATTN(64, 2);
    else if (dh == 64) CFDETR_LAUNCH_ATTN(64, 1);
    else if (dh == 32 && block_q == 256) CFDETR_LAUNCH_ATTN(32, 2);
    else if (dh == 32) CFDETR_LAUNCH_ATTN(32, 1);
    else return hipErrorInvalidValue;
#undef CFDETR_LAUNCH_ATTN
  } else {
    const float* in = static_cast<const float*>(qkv);
    float* o = static_cast<float*>(out);
    if (dh == 64)
      hipLaunchKernelGGL(attention_f32_kernel<64>, grid, dim3(block_q), 0, s, in, o, cu_seqlens, d,
                         items, scale);
    else if (dh == 32)
      hipLaunchKernelGGL(attention_f32_kernel<32>, grid, dim3(block_q), 0, s, in, o, cu_seqlens, d,
                         items, scale);
    else
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace cfdetr
