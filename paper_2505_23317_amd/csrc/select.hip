// A2 of CF-DETR (Sec. III-B): which cells are re-partitioned into finer patches,
// and the ordered token table that results.  Integer work only.
//
// Split rule: a cell of a non-finest level l is replaced by its four children iff
// a box of the same frame with tier > l overlaps it.  Such a box then also overlaps
// every ancestor of the cell with a tier above the ancestor's level, so a "hit"
// cell always has split ancestors.  Two consequences used here:
//   * a cell (l, r, c) is a token iff (l == 0 or its parent is hit) and
//     (l == finest or it is not hit itself): no recursion needed;
//   * a frame has N0 + 3 * (number of hit cells) tokens, and 4*S(l-1) - S(l) of them
//     at level l, with S(l) the hit cells of level l, S(finest) = 0, 4*S(-1) := N0.
// Kernel 1 tests every non-finest cell against the boxes of its frame (kBoxLanes
// threads share a cell, each taking every kBoxLanes-th box) and raises the cell's
// flag; kernel 2 counts the flags of all frames (offsets), then compacts the tokens
// of its own frame with wavefront ballots and popcount prefix sums, and clears the
// flag array that the NEXT call will use (two arrays alternate), so no memset is
// ever needed.
#include "kernels.h"

namespace cfdetr {

namespace {

constexpr int kHitThreads = 256;
constexpr int kBoxLanes = 8;
constexpr int kCompactThreads = 1024;

__global__ __launch_bounds__(kHitThreads) void select_hit_kernel(
    Pyramid pyr, const int32_t* __restrict__ boxes, const uint8_t* __restrict__ tier,
    const int32_t* __restrict__ box_offsets, int nonfinest, uint8_t* __restrict__ hit) {
  const int frame = blockIdx.y;
  const int cell = blockIdx.x * (kHitThreads / kBoxLanes) + threadIdx.x / kBoxLanes;
  const int boxlane = threadIdx.x % kBoxLanes;
  if (cell >= nonfinest) return;
  int id = cell, level = 0;
  while (id >= pyr.rows[level] * pyr.cols[level]) {
    id -= pyr.rows[level] * pyr.cols[level];
    ++level;
  }
  const int P = pyr.patch[level];
  const int row = id / pyr.cols[level], col = id % pyr.cols[level];
  const int cx0 = col * P, cx1 = cx0 + P, cy0 = row * P, cy1 = cy0 + P;
  const int lo = box_offsets[frame], hi = box_offsets[frame + 1];
  bool flag = false;
  for (int b = lo + boxlane; b < hi; b += kBoxLanes) {
    const int4 raw = *reinterpret_cast<const int4*>(boxes + 4 * (size_t)b);
    const int x0 = max(raw.x, 0), y0 = max(raw.y, 0);
    const int x1 = min(raw.z, pyr.img_w), y1 = min(raw.w, pyr.img_h);
    const bool nonempty = (x1 > x0) && (y1 > y0);
    flag |= nonempty && ((int)tier[b] > level) && (x0 < cx1) && (x1 > cx0) && (y0 < cy1) &&
            (y1 > cy0);
  }
  if (flag) hit[(size_t)frame * nonfinest + cell] = 1;   // several lanes may write the same 1
}

// Sequence list of one encoder run, and the attention work list over it.
// The sequences are `n_prefix` sequences of `prefix_len` tokens each (the coarse grids
// of a merged coarse+mixed run; n_prefix may be 0) followed by the B sequences that
// cu[0..B] delimits.  Outputs:
//   cu_all[0..nseq]  offsets of all sequences, m_all = their total
//   pcu[0..nseq]     offsets when every sequence is padded to a multiple of 64
//   items[0..8*cap8) attention work items of four words: sequence<<24 | head<<19 | query
//                    tile (or -1: no item), then the sequence's offset, length and padded
//                    offset, so that a workgroup gets all it needs to start in one load.
// Workgroups are dealt to the 8 XCDs round-robin (workgroup w runs on XCD w % 8), and
// every XCD has its own L2.  All query tiles of one (sequence, head) read the same
// keys and values, so a whole group goes to one XCD: groups are ordered longest
// sequence first and dealt round-robin, group G to XCD G % 8, whose workgroups
// 8*j + G%8 take its tiles in order.  Costs fall with G, so the XCD loads differ by at
// most one group, and no XCD gets more than total/8 + (tiles of the longest sequence)
// items, which is what cap8 provides.
constexpr int kMaxHeads = 32;

// The plan proper: the lengths of the nseq sequences are in s_len (shared, published by a
// barrier); all threads of a workgroup of at least 2 * kMaxBatch threads call it.
__device__ __forceinline__ void plan_body(const PlanArgs& p, int nseq, const int* s_len, bool gated) {
  __shared__ int s_order[2 * kMaxBatch];
  __shared__ int s_gstart[2 * kMaxBatch * kMaxHeads];
  __shared__ int s_count[8];
  __shared__ int s_cu[2 * kMaxBatch], s_pcu[2 * kMaxBatch];
  const int tid = threadIdx.x;
  const int heads = p.heads, block_q = p.block_q, cap8 = p.cap8;
  int4* const items4 = reinterpret_cast<int4*>(p.items);
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
  const int ngroups = nseq * heads;
  if (tid < 8) {   // XCD tid: slots of its groups
    int pos = 0;
    for (int G = tid; G < ngroups; G += 8) {
      s_gstart[G] = pos;
      pos += (s_len[s_order[G / heads]] + block_q - 1) / block_q;
    }
    s_count[tid] = gated ? 0 : min(pos, cap8);
  }
  if (tid == 8) {
    int pos = 0, ppos = 0;
    for (int i = 0; i < nseq; ++i) {
      p.cu_all[i] = pos;
      p.pcu[i] = ppos;
      s_cu[i] = pos;
      s_pcu[i] = ppos;
      pos += s_len[i];
      ppos += (s_len[i] + 63) & ~63;
    }
    p.cu_all[nseq] = pos;
    p.pcu[nseq] = ppos;
    *p.m_all = pos;
  }
  __syncthreads();
  for (int G = tid; G < ngroups; G += blockDim.x) {   // one thread per group
    const int f = s_order[G / heads], h = G % heads, x = G & 7;
    const int nt = (s_len[f] + block_q - 1) / block_q;
    const int j0 = s_gstart[G];
    for (int q = 0; q < nt && j0 + q < cap8; ++q)
      items4[8 * (j0 + q) + x] = make_int4((f << 24) | (h << 19) | q, s_cu[f], s_len[f], s_pcu[f]);
  }
  for (int i = tid; i < 8 * cap8; i += blockDim.x)
    if ((i >> 3) >= s_count[i & 7]) items4[i] = make_int4(-1, 0, 0, 0);
  // fetch counters: behind the entries handed out by workgroup index, or -1 where those
  // are the whole queue (nothing to fetch: a workgroup need not ask)
  for (int i = tid; i < p.n_heads_q; i += blockDim.x)
    p.queue_heads[i] = s_count[i & 7] <= p.queue_start ? -1 : p.queue_start;
}

__global__ __launch_bounds__(256) void plan_kernel(const int32_t* __restrict__ cu, int B, PlanArgs p,
                                                   int max_total, int min_len,
                                                   int32_t* __restrict__ err_flag,
                                                   const int32_t* __restrict__ gate) {
  __shared__ int s_len[2 * kMaxBatch];
  const int tid = threadIdx.x;
  const int nseq = p.n_prefix + B;
  if (tid < nseq) s_len[tid] = tid < p.n_prefix ? p.prefix_len : cu[tid - p.n_prefix + 1] - cu[tid - p.n_prefix];
  __syncthreads();
  if (max_total > 0) {
    // offsets a caller wrote: every length must be at least min_len and the total must fit;
    // otherwise the caller's sequences all get length 0 (nothing of them is computed or
    // written) and the error flag is raised
    if (tid == 0) {
      long long pos = 0;
      bool bad = false;
      for (int i = p.n_prefix; i < nseq; ++i) {
        const int len = s_len[i];
        if (len < min_len) bad = true;
        pos += len > 0 ? len : 0;
      }
      if (pos > (long long)max_total) bad = true;
      if (bad) {
        for (int i = p.n_prefix; i < nseq; ++i) s_len[i] = 0;
        *err_flag = 1;
      }
    }
    __syncthreads();
  }
  const bool gated = gate != nullptr && *gate != 0;   // an earlier kernel found an error
  plan_body(p, nseq, s_len, gated);
}

__global__ __launch_bounds__(kCompactThreads) void select_compact_kernel(
    Pyramid pyr, int B, int nonfinest, const uint8_t* __restrict__ hit,
    uint8_t* __restrict__ hit_next, int hit_bytes, int max_tokens,
    int32_t* __restrict__ tok_desc,
    int32_t* __restrict__ cu_seqlens, int32_t* __restrict__ level_counts,
    int32_t* __restrict__ err_flag, const int32_t* __restrict__ hard, PlanArgs plan) {
  __shared__ int s_split[kMaxBatch][kMaxLevels];   // hit cells per (frame, level)
  __shared__ int s_wave[kCompactThreads / kWave];
  // Workgroup B, if there is one (plan.items set), compacts nothing: the lengths that every
  // workgroup works out for its offset are all the attention plan needs, so it makes that
  // plan while the others compact, and the encoder that follows has no launch for it.
  const int frame = blockIdx.x;
  const int tid = threadIdx.x;
  const int n = pyr.n_levels;
  const int lane = tid & (kWave - 1), wave = tid / kWave;

  // hit cells of every frame and level (each workgroup needs all of them for its offset)
  for (int i = tid; i < kMaxBatch * kMaxLevels; i += kCompactThreads) (&s_split[0][0])[i] = 0;
  __syncthreads();
  {
    int bound[kMaxLevels];   // end of level l inside one frame's flag array
    int acc = 0;
    for (int l = 0; l < kMaxLevels; ++l) {
      if (l + 1 < n) acc += pyr.rows[l] * pyr.cols[l];
      bound[l] = acc;
    }
    const int total = B * nonfinest;
    for (int start = 0; start < total; start += kCompactThreads) {
      const int i = start + tid;
      int f = 0, l = 0;
      bool h = false;
      if (i < total) {
        f = i / nonfinest;
        const int c = i - f * nonfinest;
        while (c >= bound[l]) ++l;
        h = hit[i] != 0;
      }
      // frames and levels change rarely inside a wavefront: vote per (frame, level) of lane 0
      // and let the few stragglers add on their own
      const int f0 = __shfl(f, 0, kWave), l0 = __shfl(l, 0, kWave);
      const bool same = (f == f0) && (l == l0);
      const unsigned long long m = __ballot(h && same);
      if (lane == 0 && m != 0) atomicAdd(&s_split[f0][l0], __popcll(m));
      if (h && !same) atomicAdd(&s_split[f][l], 1);
    }
  }
  __syncthreads();
  // A frame marked easy (hard given and 0 for it) has no fine stage: no token at all.
  long long total_tokens = 0;
  int base = 0;
  for (int j = 0; j < B; ++j) {
    int sj = 0;
    for (int l = 0; l + 1 < n; ++l) sj += s_split[j][l];
    const int tj = (hard != nullptr && hard[j] == 0) ? 0 : pyr.rows[0] * pyr.cols[0] + 3 * sj;
    if (j < frame) base += tj;
    total_tokens += tj;
  }
  if (frame >= B) {
    __shared__ int s_len[2 * kMaxBatch];
    const bool too_many = total_tokens > (long long)max_tokens;   // then every length is 0
    if (tid < plan.n_prefix + B) {
      int len = plan.prefix_len;
      if (tid >= plan.n_prefix) {
        int sj = 0;
        for (int l = 0; l + 1 < n; ++l) sj += s_split[tid - plan.n_prefix][l];
        len = too_many ? 0 : pyr.rows[0] * pyr.cols[0] + 3 * sj;
        if (hard != nullptr && hard[tid - plan.n_prefix] == 0) len = 0;
      }
      s_len[tid] = len;
    }
    __syncthreads();
    plan_body(plan, plan.n_prefix + B, s_len, false);
    return;
  }
  // The flag array of the call after this one starts from zero: all of it (that call
  // may have more frames than this one), shared out among the workgroups.
  {
    const int share = (hit_bytes + B - 1) / B;
    const int lo = frame * share, hi = min(lo + share, hit_bytes);
    for (int i = lo + tid; i < hi; i += kCompactThreads) hit_next[i] = 0;
  }
  const bool overflow = total_tokens > (long long)max_tokens;
  const bool skipped = hard != nullptr && hard[frame] == 0;
  if (tid == 0) {
    cu_seqlens[frame] = overflow ? 0 : base;
    if (frame == B - 1) cu_seqlens[B] = overflow ? 0 : (int)total_tokens;
    if (overflow && frame == 0) *err_flag = 1;
  }
  if (level_counts != nullptr && tid < n) {
    const int prev4 = tid == 0 ? pyr.rows[0] * pyr.cols[0] : 4 * s_split[frame][tid - 1];
    const int cur = (tid + 1 < n) ? s_split[frame][tid] : 0;
    level_counts[frame * n + tid] = (overflow || skipped) ? 0 : prev4 - cur;
  }
  if (overflow || skipped) return;

  const uint8_t* fhit = hit + (size_t)frame * nonfinest;
  int running = base;
  int off_prev = 0, off_cur = 0;  // start of level l-1 / level l inside the flag array
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

__global__ __launch_bounds__(256) void pad_tokens_kernel(const int32_t* __restrict__ tok_desc,
                                                         const int32_t* __restrict__ cu, int B,
                                                         int t_pad, int32_t* __restrict__ tok_pad,
                                                         int32_t* __restrict__ cu_pad,
                                                         int32_t* __restrict__ kv_len,
                                                         int32_t* __restrict__ err_flag) {
  const int f = blockIdx.y;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int t0 = cu[f], len = cu[f + 1] - t0;
  if (j == 0) {
    cu_pad[f] = f * t_pad;
    if (f == B - 1) cu_pad[B] = B * t_pad;
    // a frame without tokens cannot be padded (its keys would all be masked): it gets one
    // key, the rows hold the first coarse cell, and the error flag is raised
    kv_len[f] = max(min(len, t_pad), 1);
    if (len > t_pad || len < 1) *err_flag = 1;
  }
  if (j < t_pad) tok_pad[(size_t)f * t_pad + j] = len > 0 ? tok_desc[t0 + min(j, len - 1)] : 0;
}

}  // namespace

hipError_t launch_pad_tokens(const int32_t* tok_desc, const int32_t* cu_seqlens, int B, int t_pad,
                             int32_t* tok_pad, int32_t* cu_pad, int32_t* kv_len,
                             int32_t* err_flag, hipStream_t s) {
  hipLaunchKernelGGL(pad_tokens_kernel, dim3((t_pad + 255) / 256, B), dim3(256), 0, s, tok_desc,
                     cu_seqlens, B, t_pad, tok_pad, cu_pad, kv_len, err_flag);
  return hipGetLastError();
}

hipError_t launch_select(const Pyramid& pyr, const int32_t* boxes, const uint8_t* tier,
                         const int32_t* box_offsets, int B, int nonfinest, uint8_t* hit,
                         uint8_t* hit_next, int hit_bytes, int max_tokens, int32_t* tok_desc,
                         int32_t* cu_seqlens, int32_t* level_counts, int32_t* err_flag,
                         hipStream_t s, const PlanArgs* plan, const int32_t* hard) {
  if (nonfinest > 0) {
    const int cells_per_block = kHitThreads / kBoxLanes;
    dim3 grid((nonfinest + cells_per_block - 1) / cells_per_block, B);
    hipLaunchKernelGGL(select_hit_kernel, grid, dim3(kHitThreads), 0, s, pyr, boxes, tier,
                       box_offsets, nonfinest, hit);
  }
  PlanArgs none{};
  hipLaunchKernelGGL(select_compact_kernel, dim3(B + (plan ? 1 : 0)), dim3(kCompactThreads), 0, s,
                     pyr, B, nonfinest, hit, hit_next, hit_bytes, max_tokens, tok_desc, cu_seqlens,
                     level_counts, err_flag, hard, plan ? *plan : none);
  return hipGetLastError();
}

hipError_t launch_plan(const int32_t* cu_seqlens, int B, const PlanArgs& plan, hipStream_t s,
                       int max_total, int min_len, int32_t* err_flag, const int32_t* gate) {
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(256), 0, s, cu_seqlens, B, plan, max_total, min_len,
                     err_flag, gate);
  return hipGetLastError();
}

}  // namespace cfdetr
