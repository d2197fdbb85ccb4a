// Variable-length multi-head self-attention (Sec. II-A: every token attends to
// every token of its own frame; A3, Sec. III-B: several frames in one batch).
// Frames are addressed by offsets, so no padding token is ever computed.
//
// bf16 kernel, flash style.  A work item is 128 queries of one (frame, head); each of
// the four wavefronts of a workgroup owns 32 of them.  Keys/values are walked in tiles
// of 64 that go from global memory straight into LDS (global_load_lds,
// double-buffered, one barrier per tile).  Everything is computed transposed so that
// a query is a LANE:
//   S^T[key, q] = K . Q^T          (MFMA A = K rows from LDS, B = Q rows in registers)
//   O^T[dh, q] += V^T . P^T        (MFMA A = V^T rows from LDS, B = P from registers)
// In the MFMA result layout a lane then holds 16 keys of ONE query, so the sum of its
// probabilities is a per-lane scalar, the only cross-lane step is one exchange between
// lane l and l^32 at the end, and the probabilities feed the second MFMA straight from
// registers.  For that to work the 8 keys a
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
// Softmax arithmetic per element is one exp2, one add and half a convert: q arrives
// multiplied by log2(e)/sqrt(dh), so S is a base-2 logit, and the probabilities are taken as
// 2^S, relative to the reference 0 and not to a running maximum: O / l is the same quotient
// for any reference, floating point keeps the same relative precision at any magnitude, and
// no maximum has to be tracked, compared or applied.  What a fixed reference cannot do is
// stay inside the exponent range: when a query's sum of probabilities ends outside
// [2^-64, 2^100] (or is no number), some probability that matters may have been flushed to
// zero or have overflowed; the workgroup then walks the item's keys again, once for the
// largest logit of every query and once with the probabilities relative to it, which is
// exact for any logits.  Trained or randomly initialised weights do not get there (|S| of
// a few tens); the parity tests force it.
//
// Work distribution: sequences differ in length by 2-3x, so a fixed item -> workgroup
// map leaves CUs idle while the longest items finish.  The grid is sized to what the
// chip holds at once (a multiple of 8) and workgroup w serves queue w mod 8: it starts
// with entry w/8 and fetches further entries (longest first) through an atomic counter
// until the queue is empty.  Every queue has grid/8 workgroups whatever the hardware's
// placement; with the usual round-robin placement those all sit on one XCD and share
// its L2.
//
// The fp32 kernel (check mode) is an online softmax (running maximum) with one query per
// thread.
#include <type_traits>

#include "kernels.h"

namespace cfdetr {

namespace {

constexpr int kBlockKV = 64;
// sums of probabilities (relative to the reference 0) outside this range send an item
// through the exact walk: below, probabilities that matter may have been flushed to zero
// (normal numbers end at 2^-126; 2^24 flushed ones add up to less than 2^-100); above, one
// may have overflowed
constexpr float kSumLow = 0x1p-64f, kSumHigh = 0x1p+100f;
constexpr int kFast = 0, kScan = 1, kExact = 2;

__device__ __forceinline__ int swap_bits_2_3(int i) {
  return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1);
}

// Swizzle key of LDS row r: 128-byte rows have 8 chunks and two rows cover the 64
// banks, 64-byte rows have 4 chunks and four rows cover them.
template <int ROWB>
__device__ __forceinline__ int swz(int r) {
  return ROWB == 128 ? ((r >> 1) & 7) : ((r >> 2) & 3);
}

// p = 2^s for the 32 logits of a lane, packed to bf16 MFMA operands; returns their sum.
__device__ __forceinline__ float exp_tile(const f32x16 (&s)[2], bf16x8 (&pf)[2][2]) {
  float psum = 0.f;
#pragma unroll
  for (int sub = 0; sub < 2; ++sub)
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float p0 = __builtin_amdgcn_exp2f(s[sub][8 * t + 2 * e]);
        const float p1 = __builtin_amdgcn_exp2f(s[sub][8 * t + 2 * e + 1]);
        psum += p0 + p1;
        w[e] = pack_bf16x2(p0, p1);
      }
      uint4 packed = make_uint4(w[0], w[1], w[2], w[3]);
      pf[sub][t] = *reinterpret_cast<bf16x8*>(&packed);
    }
  return psum;
}

// One 16-byte piece per lane from global memory straight into LDS (1 KB per wavefront at
// lds_addr, lane order): the address is a base in scalar registers plus the lane's 32-bit
// byte offset, so a tile that lies inside its sequence costs no vector arithmetic.  The
// compiler does not count these loads; the tile loop waits with vmcnt(0) itself.
__device__ __forceinline__ void attn_dma16(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(sbase)
               : "memory");
}

// Clears, in a V^T tile in LDS (row = feature, 8 chunks of 8 keys), the keys from `nvalid`
// on.  Not inlined on purpose: it runs once per work item, and inlined into the tile loop it
// costs the kernel an occupancy step (the loop's register budget is what sets it).
template <int DH>
__device__ __attribute__((noinline)) void clear_v_padding(unsigned char* wV, int nvalid, int tid) {
  for (int u = tid; u < DH * 8; u += 256) {
    const int rho = u >> 3, c = u & 7;   // row (feature), logical chunk of 8 keys
    const int n = nvalid - 8 * c;        // keys of this chunk inside the sequence
    if (n < 8) {
      uint4* q = reinterpret_cast<uint4*>(wV + rho * 128 + ((c ^ swz<128>(rho)) << 4));
      uint4 w = *q;
      uint32_t* e = reinterpret_cast<uint32_t*>(&w);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        e[j] &= (2 * j < n ? 0x0000FFFFu : 0u) | (2 * j + 1 < n ? 0xFFFF0000u : 0u);
      *q = w;
    }
  }
}

template <int DH>
__global__ __launch_bounds__(256) void attention_bf16_kernel(
    const bf16_t* __restrict__ qbuf, int q_ld, const bf16_t* __restrict__ kbuf, int k_ld,
    const bf16_t* __restrict__ vt, int vt_ld, bf16_t* __restrict__ out,
    const int32_t* __restrict__ cu_k, const int32_t* __restrict__ pcu_k, int d,
    const int4* __restrict__ items, int cap8, int32_t* __restrict__ queue_heads,
    const int32_t* __restrict__ kv_len) {
  constexpr int BQ = 128;
  constexpr int KS = DH / 16;          // k-steps of Q.K^T
  constexpr int MO = DH / 32;          // 32-row blocks of O^T
  constexpr int KROWB = DH * 2;        // bytes per K row in LDS
  constexpr int KCPR = KROWB / 16;     // chunks per K row
  constexpr int KRPI = 1024 / KROWB;   // K rows per wave load instruction
  constexpr int KI = kBlockKV / KRPI / 4;   // K load instructions per wavefront
  constexpr int VI = DH / 8 / 4;            // V^T load instructions per wavefront (8 rows each)
  constexpr int KBYTES = kBlockKV * KROWB, VBYTES = DH * 128;
  // One array per buffer and operand: the compiler then knows that a tile being
  // filled is not the tile being read, and does not wait for the fill before the reads.
  __shared__ __attribute__((aligned(1024))) unsigned char sK0[KBYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char sK1[KBYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char sV0[VBYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char sV1[VBYTES];
  __shared__ int32_t s_item;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g = lane >> 5;
  const int home = blockIdx.x & 7;   // queue of this workgroup; w mod 8 is also its XCD
  // first item: entry blockIdx/8 of the home queue; later ones through the counter, which
  // starts behind the entries handed out this way
  int entry = blockIdx.x >> 3;
  // -1: the queue holds no more entries than were handed out by index (launch_plan)
  const bool drained = queue_heads[home] < 0;

  // Loader roles, as byte offsets of the lane's piece from the tile's first key (K) or
  // first position (V^T).  K: LDS row rho <- key (rho & 32) | swap23(rho & 31), chunk
  // swizzled.  V^T: LDS row rho = dh index; 64 keys = 8 chunks of 8.
  uint32_t k_off[KI], v_off[VI];
#pragma unroll
  for (int j = 0; j < KI; ++j) {
    const int rho = (wave * KI + j) * KRPI + lane / KCPR;
    const int key = (rho & 32) | swap_bits_2_3(rho & 31);
    k_off[j] = (uint32_t)key * (uint32_t)(k_ld * 2) + (uint32_t)(((lane % KCPR) ^ swz<KROWB>(rho)) * 16);
  }
#pragma unroll
  for (int j = 0; j < VI; ++j) {
    const int rho = (wave * VI + j) * 8 + (lane >> 3);
    v_off[j] = ((uint32_t)rho * (uint32_t)vt_ld + (uint32_t)(((lane & 7) ^ swz<128>(rho)) * 8)) * 2u;
  }
  const uint32_t lds_k0 = (uint32_t)(uintptr_t)sK0, lds_k1 = (uint32_t)(uintptr_t)sK1;
  const uint32_t lds_v0 = (uint32_t)(uintptr_t)sV0, lds_v1 = (uint32_t)(uintptr_t)sV1;

  for (;;) {
    // An entry is four words: the item, then offset, length and padded offset of its
    // sequence; the index is uniform, so this is one scalar load and a workgroup needs
    // nothing else before it can ask for its queries and first keys.
    if (entry >= cap8) break;
    const int4 rec = items[home + 8 * entry];
    const int32_t item = rec.x;
    if (item < 0) break;   // entries are in use from the front: the queue is empty

    const int frame = item >> 24, head = (item >> 19) & 31, qt = item & 0x7FFFF;
    const int seq0 = rec.y, T = rec.z;
    // the keys come from sequence `frame` of cu_k (cross-attention) or are the queries' own
    // sequence, all of them unless the caller padded it
    const int kseq0 = cu_k ? cu_k[frame] : seq0;
    const int TKall = cu_k ? cu_k[frame + 1] - kseq0 : T;
    const int kpad0 = cu_k ? pcu_k[frame] : rec.w;
    const int TK = kv_len ? min(kv_len[frame], TKall) : TKall;
    const bf16_t* qbase = qbuf + (size_t)seq0 * q_ld + head * DH;
    const bf16_t* kbase = kbuf + (size_t)kseq0 * k_ld + head * DH;

    // Q operands: lane = query, 8 consecutive dh per k-step.
    bf16x8 qf[KS];
    {
      const int q_load = min(qt * BQ + wave * 32 + l32, T - 1);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        qf[ks] = *reinterpret_cast<const bf16x8*>(qbase + (size_t)q_load * q_ld + ks * 16 + g * 8);
    }
    const bf16_t* vbase = vt + (size_t)(head * DH) * vt_ld + kpad0;

    // Fill of the tile that starts at key kv0_: inside the sequence the lane offsets are the
    // constants above; the last, ragged tile clamps its keys to the sequence (the lanes that
    // would read past it fetch the last key again; their logits are masked).
#define CFDETR_ATTN_ISSUE(kv0_, buf_)                                                        \
  do {                                                                                       \
    const bf16_t* kb_ = kbase + (size_t)(kv0_) * k_ld;                                       \
    const uint32_t lk_ = ((buf_) ? lds_k1 : lds_k0) + wave * (KI * 1024);                    \
    if ((kv0_) + kBlockKV <= TK) {                                                           \
      _Pragma("unroll") for (int j = 0; j < KI; ++j) attn_dma16(kb_, k_off[j], lk_ + j * 1024); \
    } else {                                                                                 \
      _Pragma("unroll") for (int j = 0; j < KI; ++j) {                                       \
        const int rho = (wave * KI + j) * KRPI + lane / KCPR;                                \
        const int key = min((rho & 32) | swap_bits_2_3(rho & 31), TK - 1 - (kv0_));          \
        attn_dma16(kb_, (uint32_t)key * (uint32_t)(k_ld * 2) +                               \
                            (uint32_t)(((lane % KCPR) ^ swz<KROWB>(rho)) * 16), lk_ + j * 1024); \
      }                                                                                      \
    }                                                                                        \
    const bf16_t* vb_ = vbase + (kv0_);                                                      \
    const uint32_t lv_ = ((buf_) ? lds_v1 : lds_v0) + wave * (VI * 1024);                    \
    _Pragma("unroll") for (int j = 0; j < VI; ++j) attn_dma16(vb_, v_off[j], lv_ + j * 1024); \
  } while (0)

    // One walk over the key tiles of the item.  kFast: probabilities relative to the
    // reference 0.  kScan: only the largest logit of every query.  kExact: probabilities
    // relative to m_ref (that largest logit).  All wavefronts of the workgroup take the same
    // walks (the tiles and the barriers are shared).
    f32x16 acc_o[MO];
    float l_run = 0.f;    // sum of the probabilities of this lane's keys
    float m_ref = 0.f;
    const int n_kv = (TK + kBlockKV - 1) / kBlockKV;
    auto walk = [&](auto mode_tag) {
      constexpr int kMode = decltype(mode_tag)::value;
      float smax = -INFINITY;
      if (kMode != kScan) {
        l_run = 0.f;
#pragma unroll
        for (int i = 0; i < MO; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_o[i][r] = 0.f;
      }
      CFDETR_ATTN_ISSUE(0, 0);
      for (int it0 = 0; it0 < n_kv; it0 += 2) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {   // buffer index: a constant after unrolling
          const int it = it0 + b;
          if (it >= n_kv) break;
          const int kv0 = it * kBlockKV;
          // vmcnt(0): this wavefront's part of tile `it` is in LDS; the barrier publishes
          // every wavefront's part and retires all reads of the other buffer.
          __builtin_amdgcn_s_waitcnt(0x0F70);
          __syncthreads();
          if (it + 1 < n_kv) CFDETR_ATTN_ISSUE(kv0 + kBlockKV, b ^ 1);
          const unsigned char* cK = b ? sK1 : sK0;
          const unsigned char* cV = b ? sV1 : sV0;
          if (kMode != kScan && kv0 + kBlockKV > TK) {
            // Last, ragged tile (no fill is in flight any more): the V^T positions past the
            // end of the sequence are padding that nothing in this run wrote.  They only
            // meet probabilities that are exactly 0, but 0 * NaN is NaN, so they are cleared
            // here: whatever an earlier run left there cannot reach a result.
            clear_v_padding<DH>(b ? sV1 : sV0, TK - kv0, tid);
            __syncthreads();
          }

          // S^T for the two 32-key sub-tiles; keys past the end of the frame (last tile
          // only) get -inf.
          f32x16 s[2];
#pragma unroll
          for (int sub = 0; sub < 2; ++sub) {
            const int rho = sub * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[sub][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
              const bf16x8 kf = *reinterpret_cast<const bf16x8*>(
                  cK + rho * KROWB + (((2 * ks + g) ^ swz<KROWB>(rho)) << 4));
              s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[sub], 0, 0, 0);
            }
          }
          if (kv0 + kBlockKV > TK) {
            asm volatile("" ::: "memory");   // keeps this a branch: one tile per item comes here
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int key = kv0 + sub * 32 + 16 * (r >> 3) + 8 * g + (r & 7);
                if (key >= TK) s[sub][r] = -INFINITY;
              }
          }
          if (kMode == kScan) {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
              for (int r = 0; r < 16; ++r) smax = fmaxf(smax, s[sub][r]);
            continue;
          }
          if (kMode == kExact) {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
              for (int r = 0; r < 16; ++r) s[sub][r] -= m_ref;
          }
          bf16x8 pf[2][2];
          l_run += exp_tile(s, pf);
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
                acc_o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sub][t], acc_o[i], 0, 0, 0);
              }
          }
        }
      }
      return smax;
    };

    walk(std::integral_constant<int, kFast>{});
    float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    // A sum that left the range in which every probability that matters is a normal number
    // (some logit beyond +-100 or so in base 2; also inf and NaN): find every query's
    // largest logit first and take the probabilities relative to it.
    if (__syncthreads_or(!(l_tot >= kSumLow && l_tot <= kSumHigh))) {
      const float smax = walk(std::integral_constant<int, kScan>{});
      m_ref = fmaxf(smax, __shfl_xor(smax, 32, kWave));
      __syncthreads();   // every wavefront is done with the last tile of the scan
      walk(std::integral_constant<int, kExact>{});
      l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    }
#undef CFDETR_ATTN_ISSUE

    const float inv = 1.0f / l_tot;
    const int q_local = qt * BQ + wave * 32 + l32;
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
    // the next entry; the barriers also keep the next item's first fill behind every
    // wavefront's last reads of this one's tiles
    if (drained) break;
    __syncthreads();
    if (tid == 0) s_item = atomicAdd(&queue_heads[home], 1);
    __syncthreads();
    entry = __builtin_amdgcn_readfirstlane(s_item);
  }
}

// fp32 check mode: one query per thread, keys in tiles of 32 through LDS.
template <int DH>
__global__ __launch_bounds__(256) void attention_f32_kernel(
    const float* __restrict__ qkv, float* __restrict__ out, int d,
    const int4* __restrict__ items, float scale, const int32_t* __restrict__ kv_len) {
  constexpr int TILE = 32;
  __shared__ float sK[TILE][DH];
  __shared__ float sV[TILE][DH];
  const int4 rec = items[blockIdx.x];
  const int32_t item = rec.x;
  if (item < 0) return;
  const int frame = item >> 24, head = (item >> 19) & 31, qt = item & 0x7FFFF;
  const int seq0 = rec.y, T = rec.z;
  const int TK = kv_len ? min(kv_len[frame], T) : T;
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
  for (int kv0 = 0; kv0 < TK; kv0 += TILE) {
    __syncthreads();
    for (int e = threadIdx.x; e < TILE * DH; e += blockDim.x) {
      int r = e / DH, c = e - r * DH;
      int key = min(kv0 + r, TK - 1);
      sK[r][c] = qbase[(size_t)key * ld + d + c];
      sV[r][c] = qbase[(size_t)key * ld + 2 * d + c];
    }
    __syncthreads();
    float s[TILE];
    float m_tile = -INFINITY;
#pragma unroll
    for (int r = 0; r < TILE; ++r) {
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < DH; ++i) acc = fmaf(q[i], sK[r][i], acc);
      s[r] = (kv0 + r < TK) ? acc : -INFINITY;
      m_tile = fmaxf(m_tile, s[r]);
    }
    const float m_new = fmaxf(m_run, m_tile);
    const float alpha = expf(m_run - m_new);
    m_run = m_new;
    l_run *= alpha;
#pragma unroll
    for (int i = 0; i < DH; ++i) o[i] *= alpha;
#pragma unroll
    for (int r = 0; r < TILE; ++r) {
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

int attention_block_q() { return 128; }

float attention_q_scale(int d_head) {
  return 1.44269504088896340736f / sqrtf((float)d_head);
}

namespace {

// Workgroups the chip holds at once for a kernel: the size of a fetch-from-queue grid.
template <typename K>
int resident_grid(K kern) {
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 256, 0) != hipSuccess) return 0;
  if (cus <= 0 || per_cu <= 0) return 0;
  return (cus * per_cu + 7) & ~7;
}

}  // namespace

int attention_grid(int d_head, bool use_bf16, int cap8) {
  const long all = 8L * cap8;
  if (!use_bf16) return (int)all;
  int resident = 0;
  if (d_head == 64) resident = resident_grid(attention_bf16_kernel<64>);
  else if (d_head == 32) resident = resident_grid(attention_bf16_kernel<32>);
  if (resident <= 0) return 0;
  return (int)(all < resident ? all : resident);
}

hipError_t launch_attention(const void* qkv, const void* vt, int vt_ld, void* out, int d, int heads,
                            const int32_t* items, int cap8, int32_t* queue_heads, int grid_size,
                            int block_q, bool use_bf16, const int32_t* kv_len, hipStream_t s) {
  if (block_q != 128 || grid_size < 8 || grid_size % 8 != 0 || grid_size > 8 * cap8)
    return hipErrorInvalidValue;
  const int dh = d / heads;
  const int4* recs = reinterpret_cast<const int4*>(items);
  if (use_bf16) {
    const bf16_t* in = static_cast<const bf16_t*>(qkv);
    const bf16_t* v = static_cast<const bf16_t*>(vt);
    bf16_t* o = static_cast<bf16_t*>(out);
    dim3 grid(grid_size);
    // self-attention: queries and keys are thirds of the same rows
    if (dh == 64)
      hipLaunchKernelGGL(attention_bf16_kernel<64>, grid, dim3(256), 0, s, in, 3 * d, in + d, 3 * d,
                         v, vt_ld, o, nullptr, nullptr, d, recs, cap8, queue_heads, kv_len);
    else if (dh == 32)
      hipLaunchKernelGGL(attention_bf16_kernel<32>, grid, dim3(256), 0, s, in, 3 * d, in + d, 3 * d,
                         v, vt_ld, o, nullptr, nullptr, d, recs, cap8, queue_heads, kv_len);
    else
      return hipErrorInvalidValue;
  } else {
    const float scale = 1.0f / sqrtf((float)dh);
    dim3 grid(8 * cap8);
    const float* in = static_cast<const float*>(qkv);
    float* o = static_cast<float*>(out);
    if (dh == 64)
      hipLaunchKernelGGL(attention_f32_kernel<64>, grid, dim3(block_q), 0, s, in, o, d, recs, scale,
                         kv_len);
    else if (dh == 32)
      hipLaunchKernelGGL(attention_f32_kernel<32>, grid, dim3(block_q), 0, s, in, o, d, recs, scale,
                         kv_len);
    else
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_cross_attention(const void* q, const void* k, const void* vt, int vt_ld,
                                  void* out, const int32_t* cu_k,
                                  const int32_t* pcu_k, int d, int heads, const int32_t* items,
                                  int cap8, int32_t* queue_heads, int grid_size, hipStream_t s) {
  if (grid_size < 8 || grid_size % 8 != 0 || grid_size > 8 * cap8) return hipErrorInvalidValue;
  const int dh = d / heads;
  const int4* recs = reinterpret_cast<const int4*>(items);
  const bf16_t* qb = static_cast<const bf16_t*>(q);
  const bf16_t* kb = static_cast<const bf16_t*>(k);
  const bf16_t* v = static_cast<const bf16_t*>(vt);
  bf16_t* o = static_cast<bf16_t*>(out);
  dim3 grid(grid_size);
  if (dh == 64)
    hipLaunchKernelGGL(attention_bf16_kernel<64>, grid, dim3(256), 0, s, qb, d, kb, d, v, vt_ld, o,
                       cu_k, pcu_k, d, recs, cap8, queue_heads, nullptr);
  else if (dh == 32)
    hipLaunchKernelGGL(attention_bf16_kernel<32>, grid, dim3(256), 0, s, qb, d, kb, d, v, vt_ld, o,
                       cu_k, pcu_k, d, recs, cap8, queue_heads, nullptr);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace cfdetr
