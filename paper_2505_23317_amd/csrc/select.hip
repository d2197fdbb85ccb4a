// A2 of CF-DETR (Sec. III-B): which cells are re-partitioned into finer patches,
// and the ordered token table that results.  Integer work only.
//
// Split rule: a cell of a non-finest level l is replaced by its four children iff
// a box of the same frame with tier > l overlaps it.  Such a box then also overlaps
// every ancestor of the cell with a tier above the ancestor's level, so a "hit"
// cell always has split ancestors.  Two consequences used here:
//   * a cell (l, r, c) is a token iff (l == 0 or its parent is hit) and
//     (l == finest or it is not hit itself): no recursion needed;
//   * the number of tokens of a frame at level l is 4*S(l-1) - S(l), with S(l)
//     the number of hit cells at level l, S(finest) = 0 and 4*S(-1) := N0.
// Kernel 1 tests every non-finest cell against the boxes of its frame and counts
// hits per (frame, level); kernel 2 turns the counts into frame offsets and
// compacts the tokens with wavefront ballots and popcount prefix sums.
#include "kernels.h"

namespace cfdetr {

namespace {

constexpr int kHitThreads = 256;
constexpr int kCompactThreads = 1024;

// One thread per non-finest cell.  The boxes of the frame are clipped once and staged
// through LDS in chunks (tier 0 marks an empty or non-critical box), so the inner loop
// reads them as LDS broadcasts.
__global__ __launch_bounds__(kHitThreads) void select_hit_kernel(
    Pyramid pyr, const int32_t* __restrict__ boxes, const uint8_t* __restrict__ tier,
    const int32_t* __restrict__ box_offsets, int nonfinest, uint8_t* __restrict__ hit,
    int32_t* __restrict__ split_count) {
  __shared__ int4 s_box[kHitThreads];
  __shared__ int s_tier[kHitThreads];
  const int frame = blockIdx.y;
  int id = blockIdx.x * kHitThreads + threadIdx.x;
  const bool valid = id < nonfinest;
  int level = 0;
  if (valid) {
    while (id >= pyr.rows[level] * pyr.cols[level]) {
      id -= pyr.rows[level] * pyr.cols[level];
      ++level;
    }
  } else {
    id = 0;
  }
  const int P = pyr.patch[level];
  const int row = id / pyr.cols[level], col = id % pyr.cols[level];
  const int cx0 = col * P, cx1 = cx0 + P, cy0 = row * P, cy1 = cy0 + P;
  const int lo = box_offsets[frame], hi = box_offsets[frame + 1];
  bool flag = false;
  for (int base = lo; base < hi; base += kHitThreads) {
    const int b = base + threadIdx.x;
    int4 bx = make_int4(0, 0, 0, 0);
    int t = 0;
    if (b < hi) {
      const int4 raw = *reinterpret_cast<const int4*>(boxes + 4 * (size_t)b);
      bx = make_int4(max(raw.x, 0), max(raw.y, 0), min(raw.z, pyr.img_w), min(raw.w, pyr.img_h));
      t = (bx.z > bx.x && bx.w > bx.y) ? (int)tier[b] : 0;
    }
    __syncthreads();   // previous chunk fully consumed
    s_box[threadIdx.x] = bx;
    s_tier[threadIdx.x] = t;
    __syncthreads();
    const int n = min(kHitThreads, hi - base);
    for (int k = 0; k < n; ++k) {
      const int4 q = s_box[k];
      flag |= (s_tier[k] > level) && (q.x < cx1) && (q.z > cx0) && (q.y < cy1) && (q.w > cy0);
    }
  }
  flag = flag && valid;
  if (valid) hit[(size_t)frame * nonfinest + blockIdx.x * kHitThreads + threadIdx.x] = flag;
  for (int l = 0; l + 1 < pyr.n_levels; ++l) {
    unsigned long long m = __ballot(flag && level == l);
    if ((threadIdx.x & (kWave - 1)) == 0 && m != 0)
      atomicAdd(&split_count[frame * kMaxLevels + l], __popcll(m));
  }
}

__global__ __launch_bounds__(kCompactThreads) void select_compact_kernel(
    Pyramid pyr, int B, int nonfinest, const uint8_t* __restrict__ hit,
    const int32_t* __restrict__ split_cur, int32_t* __restrict__ split_next, int max_tokens,
    int32_t* __restrict__ tok_desc, int32_t* __restrict__ cu_seqlens,
    int32_t* __restrict__ level_counts, int32_t* __restrict__ err_flag) {
  __shared__ int s_cnt[kMaxBatch][kMaxLevels];
  __shared__ int s_wave[kCompactThreads / kWave];
  const int frame = blockIdx.x;
  const int tid = threadIdx.x;
  const int n = pyr.n_levels;
  if (tid < B) {
    int prev4 = pyr.rows[0] * pyr.cols[0];  // 4 * S(-1) := N0
    for (int l = 0; l < n; ++l) {
      int s = (l + 1 < n) ? split_cur[tid * kMaxLevels + l] : 0;
      s_cnt[tid][l] = prev4 - s;
      prev4 = 4 * s;
    }
  }
  __syncthreads();
  long long total = 0;
  int base = 0;
  for (int j = 0; j < B; ++j) {
    int tj = 0;
    for (int l = 0; l < n; ++l) tj += s_cnt[j][l];
    if (j < frame) base += tj;
    total += tj;
  }
  // counters of the call after this one start from zero
  if (tid < kMaxLevels) split_next[frame * kMaxLevels + tid] = 0;
  const bool overflow = total > (long long)max_tokens;
  if (tid == 0) {
    cu_seqlens[frame] = overflow ? 0 : base;
    if (frame == B - 1) cu_seqlens[B] = overflow ? 0 : (int)total;
    if (overflow && frame == 0) *err_flag = 1;
  }
  if (level_counts != nullptr && tid < n)
    level_counts[frame * n + tid] = overflow ? 0 : s_cnt[frame][tid];
  if (overflow) return;

  const uint8_t* fhit = hit + (size_t)frame * nonfinest;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  int running = base;
  int off_prev = 0, off_cur = 0;  // start of level l-1 / level l inside the hit array
  for (int l = 0; l < n; ++l) {
    const int rows = pyr.rows[l], cols = pyr.cols[l], nl = rows * cols;
    const int pcols = (l > 0) ? pyr.cols[l - 1] : 0;
    for (int start = 0; start < nl; start += kCompactThreads) {
      const int id = start + tid;
      bool leaf = false;
      int row = 0, col = 0;
      if (id < nl) {
        row = id / cols;
        col = id - row * cols;
        bool parent_ok = (l == 0) || fhit[off_prev + (row >> 1) * pcols + (col >> 1)];
        bool self_split = (l + 1 < n) && fhit[off_cur + id];
        leaf = parent_ok && !self_split;
      }
      unsigned long long m = __ballot(leaf);
      int before = __popcll(m & ((1ull << lane) - 1ull));
      if (lane == 0) s_wave[wave] = __popcll(m);
      __syncthreads();
      int wave_off = 0, chunk = 0;
      for (int w = 0; w < kCompactThreads / kWave; ++w) {
        int c = s_wave[w];
        if (w < wave) wave_off += c;
        chunk += c;
      }
      if (leaf) tok_desc[running + wave_off + before] = (l << 28) | (row << 14) | col;
      running += chunk;
      __syncthreads();
    }
    off_prev = off_cur;
    off_cur += nl;
  }
}

// Sequence list of one encoder run, and the attention work list over it.
// The sequences are `n_prefix` sequences of `prefix_len` tokens each (the coarse grids
// of a merged coarse+mixed run; n_prefix may be 0) followed by the B sequences that
// cu[0..B] delimits.  Outputs:
//   cu_all[0..nseq]  offsets of all sequences, m_all = their total
//   pcu[0..nseq]     offsets when every sequence is padded to a multiple of 64
//   tiles[i] = sequence<<24 | query-tile index, longest sequence first; n_tiles
__global__ __launch_bounds__(256) void plan_kernel(const int32_t* __restrict__ cu, int B,
                                                   int n_prefix, int prefix_len, int block_q,
                                                   int32_t* __restrict__ tiles,
                                                   int32_t* __restrict__ n_tiles, int capacity,
                                                   int32_t* __restrict__ cu_all,
                                                   int32_t* __restrict__ m_all,
                                                   int32_t* __restrict__ pcu) {
  __shared__ int s_len[2 * kMaxBatch];
  __shared__ int s_order[2 * kMaxBatch];
  __shared__ int s_start[2 * kMaxBatch + 1];
  const int tid = threadIdx.x;
  const int nseq = n_prefix + B;
  if (tid < nseq) s_len[tid] = tid < n_prefix ? prefix_len : cu[tid - n_prefix + 1] - cu[tid - n_prefix];
  __syncthreads();
  if (tid < nseq) {
    const int len = s_len[tid];
    int rank = 0;
    for (int j = 0; j < nseq; ++j) {
      const int lj = s_len[j];
      rank += (lj > len) || (lj == len && j < tid);
    }
    s_order[rank] = tid;
  }
  __syncthreads();
  if (tid == 0) {
    int acc = 0;
    for (int k = 0; k < nseq; ++k) {
      s_start[k] = acc;
      acc += (s_len[s_order[k]] + block_q - 1) / block_q;
    }
    s_start[nseq] = acc;
    *n_tiles = min(acc, capacity);
    int pos = 0, ppos = 0;
    for (int i = 0; i < nseq; ++i) {
      cu_all[i] = pos;
      pcu[i] = ppos;
      pos += s_len[i];
      ppos += (s_len[i] + 63) & ~63;
    }
    cu_all[nseq] = pos;
    pcu[nseq] = ppos;
    *m_all = pos;
  }
  __syncthreads();
  for (int k = 0; k < nseq; ++k) {
    const int f = s_order[k];
    const int nt = s_start[k + 1] - s_start[k];
    for (int q = tid; q < nt; q += blockDim.x) {
      const int idx = s_start[k] + q;
      if (idx < capacity) tiles[idx] = (f << 24) | q;
    }
  }
}

}  // namespace

hipError_t launch_select(const Pyramid& pyr, const int32_t* boxes, const uint8_t* tier,
                         const int32_t* box_offsets, int B, int nonfinest, uint8_t* hit,
                         int32_t* split_cur, int32_t* split_next, int max_tokens,
                         int32_t* tok_desc, int32_t* cu_seqlens, int32_t* level_counts,
                         int32_t* err_flag, hipStream_t s) {
  if (nonfinest > 0) {
    dim3 grid((nonfinest + kHitThreads - 1) / kHitThreads, B);
    hipLaunchKernelGGL(select_hit_kernel, grid, dim3(kHitThreads), 0, s, pyr, boxes, tier,
                       box_offsets, nonfinest, hit, split_cur);
  }
  hipLaunchKernelGGL(select_compact_kernel, dim3(B), dim3(kCompactThreads), 0, s, pyr, B,
                     nonfinest, hit, split_cur, split_next, max_tokens, tok_desc, cu_seqlens,
                     level_counts, err_flag);
  return hipGetLastError();
}

hipError_t launch_plan(const int32_t* cu_seqlens, int B, int n_prefix, int prefix_len,
                       int block_q, int32_t* tiles, int32_t* n_tiles, int tile_capacity,
                       int32_t* cu_all, int32_t* m_all, int32_t* pcu, hipStream_t s) {
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(256), 0, s, cu_seqlens, B, n_prefix, prefix_len,
                     block_q, tiles, n_tiles, tile_capacity, cu_all, m_all, pcu);
  return hipGetLastError();
}

}  // namespace cfdetr
