// Difficulty of a frame and regions of interest from the coarse stage's object queries
// (Sec. III-B: A1, frames are easy or hard by the average confidence of the queries that
// are not already certain; A2, the boxes of the queries of intermediate confidence are
// the regions that get finer patches).  Integer outputs feed the selection kernel
// directly, so the boxes never visit the host.
//
// Decisions are taken in fp64 on the fp32 inputs: thresholds compare exactly as in fp32,
// the average is a fp64 sum (fixed reduction tree), and a region's edges are
// centre*extent -/+ half with half = max(0.5*scale*size*extent, 0.5*min_side), every
// product and difference rounded on its own (no fused multiply-add), then rounded
// outward and clipped.
#include "kernels.h"

namespace cfdetr {

namespace {

constexpr int kRoiThreads = 256;

// Frame f: average of the confidences not above tau_hi, hard or easy, and how many
// regions it will propose (none when easy).
__global__ __launch_bounds__(kRoiThreads) void roi_stats_kernel(
    const float* __restrict__ queries, int Q, float tau_hi, float tau_lo,
    int32_t* __restrict__ hard, float* __restrict__ mean_conf, int32_t* __restrict__ n_roi) {
  __shared__ double s_sum[kRoiThreads];
  __shared__ int s_rest[kRoiThreads];
  __shared__ int s_mid[kRoiThreads];
  const int f = blockIdx.x, tid = threadIdx.x;
  const float* q = queries + (size_t)f * Q * 5;
  double sum = 0.0;
  int rest = 0, mid = 0;
  for (int k = tid; k < Q; k += kRoiThreads) {
    const float c = q[5 * k + 4];
    if (!(c > tau_hi)) {
      sum += (double)c;
      ++rest;
      mid += c > tau_lo;
    }
  }
  s_sum[tid] = sum;
  s_rest[tid] = rest;
  s_mid[tid] = mid;
  __syncthreads();
  for (int step = kRoiThreads / 2; step > 0; step >>= 1) {
    if (tid < step) {
      s_sum[tid] += s_sum[tid + step];
      s_rest[tid] += s_rest[tid + step];
      s_mid[tid] += s_mid[tid + step];
    }
    __syncthreads();
  }
  if (tid == 0) {
    const double mean = s_rest[0] > 0 ? s_sum[0] / (double)s_rest[0] : 0.0;
    const bool is_hard = !(mean < (double)tau_lo);
    hard[f] = is_hard ? 1 : 0;
    mean_conf[f] = (float)mean;
    n_roi[f] = is_hard ? s_mid[0] : 0;
  }
}

#pragma clang fp contract(off)
__device__ __forceinline__ int4 region_of(float cxf, float cyf, float wf, float hf, int H, int W,
                                          float scale, float min_side) {
  const double cx = cxf, cy = cyf, w = wf, h = hf, s = scale;
  const double half_min = 0.5 * (double)min_side;
  double half_w = 0.5 * s * w * (double)W;
  double half_h = 0.5 * s * h * (double)H;
  half_w = half_w > half_min ? half_w : half_min;
  half_h = half_h > half_min ? half_h : half_min;
  const double px = cx * (double)W, py = cy * (double)H;
  // clamp before the conversion: anything beyond the frame clips to its edge anyway
  const double lim = 1.0e9;
  const double fx0 = fmin(fmax(floor(px - half_w), -lim), lim);
  const double fx1 = fmin(fmax(ceil(px + half_w), -lim), lim);
  const double fy0 = fmin(fmax(floor(py - half_h), -lim), lim);
  const double fy1 = fmin(fmax(ceil(py + half_h), -lim), lim);
  int4 r;
  r.x = min(max((int)fx0, 0), W);
  r.y = min(max((int)fy0, 0), H);
  r.z = min(max((int)fx1, 0), W);
  r.w = min(max((int)fy1, 0), H);
  return r;
}

// Frame f writes its regions, in query order, behind those of the frames before it.
__global__ __launch_bounds__(kRoiThreads) void roi_emit_kernel(
    const float* __restrict__ queries, int B, int Q, int H, int W, float tau_hi, float tau_lo,
    float scale, float min_side, int tier_value, const int32_t* __restrict__ n_roi, int max_boxes,
    int32_t* __restrict__ boxes, uint8_t* __restrict__ tier, int32_t* __restrict__ box_offsets,
    int32_t* __restrict__ err_flag) {
  __shared__ int s_wave[kRoiThreads / 64];
  const int f = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int before = 0, total = 0;
  for (int g = 0; g < B; ++g) {
    const int n = n_roi[g];
    before += g < f ? n : 0;
    total += n;
  }
  if (total > max_boxes) {   // never truncate: propose nothing and raise the flag
    if (tid == 0) {
      box_offsets[f] = 0;
      if (f == 0) {
        box_offsets[B] = 0;
        *err_flag = 1;
      }
    }
    return;
  }
  if (tid == 0) {
    box_offsets[f] = before;
    if (f == B - 1) box_offsets[B] = total;
  }
  if (n_roi[f] == 0) return;   // easy frame (or nothing of intermediate confidence)
  const float* q = queries + (size_t)f * Q * 5;
  int base = before;
  for (int k0 = 0; k0 < Q; k0 += kRoiThreads) {
    const int k = k0 + tid;
    float c = 0.f;
    if (k < Q) c = q[5 * k + 4];
    const bool take = k < Q && !(c > tau_hi) && c > tau_lo;
    const unsigned long long ballot = __ballot(take);
    if (lane == 0) s_wave[wave] = __popcll(ballot);
    __syncthreads();
    int pos = base + __popcll(ballot & ((1ull << lane) - 1ull));
    int chunk = 0;
    for (int w = 0; w < kRoiThreads / 64; ++w) {
      pos += w < wave ? s_wave[w] : 0;
      chunk += s_wave[w];
    }
    if (take) {
      const int4 r = region_of(q[5 * k], q[5 * k + 1], q[5 * k + 2], q[5 * k + 3], H, W, scale,
                               min_side);
      *reinterpret_cast<int4*>(boxes + 4 * (size_t)pos) = r;
      tier[pos] = (uint8_t)tier_value;
    }
    base += chunk;
    __syncthreads();
  }
}

// Final detections of frame f (end of A2): its coarse queries with c > tau_hi in query
// order, then, if the frame is hard, its fine-stage queries with c > tau_fine in query
// order.  Rows past the count are cleared (det 0, src 255).  Candidate j of 2Q is coarse
// query j or fine query j - Q; one ordered compaction over all of them.
__global__ __launch_bounds__(kRoiThreads) void merge_detections_kernel(
    const float* __restrict__ coarse, const float* __restrict__ fine,
    const int32_t* __restrict__ hard, int Q, float tau_hi, float tau_fine,
    float* __restrict__ det, uint8_t* __restrict__ src, int32_t* __restrict__ count) {
  __shared__ int s_wave[kRoiThreads / 64];
  const int f = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool is_hard = hard[f] != 0;
  const float* qc = coarse + (size_t)f * Q * 5;
  const float* qf = fine + (size_t)f * Q * 5;
  float* out = det + (size_t)f * 2 * Q * 5;
  uint8_t* osrc = src + (size_t)f * 2 * Q;
  int base = 0;
  for (int j0 = 0; j0 < 2 * Q; j0 += kRoiThreads) {
    const int j = j0 + tid;
    const bool from_fine = j >= Q;
    const float* row = from_fine ? qf + 5 * (size_t)(j - Q) : qc + 5 * (size_t)j;
    bool take = false;
    if (j < 2 * Q && (!from_fine || is_hard)) take = row[4] > (from_fine ? tau_fine : tau_hi);
    const unsigned long long ballot = __ballot(take);
    if (lane == 0) s_wave[wave] = __popcll(ballot);
    __syncthreads();
    int pos = base + __popcll(ballot & ((1ull << lane) - 1ull));
    int chunk = 0;
    for (int w = 0; w < kRoiThreads / 64; ++w) {
      pos += w < wave ? s_wave[w] : 0;
      chunk += s_wave[w];
    }
    if (take) {
#pragma unroll
      for (int e = 0; e < 5; ++e) out[5 * (size_t)pos + e] = row[e];
      osrc[pos] = from_fine ? 1 : 0;
    }
    base += chunk;
    __syncthreads();
  }
  if (tid == 0) count[f] = base;
  for (int j = base + tid; j < 2 * Q; j += kRoiThreads) {
#pragma unroll
    for (int e = 0; e < 5; ++e) out[5 * (size_t)j + e] = 0.f;
    osrc[j] = 255;
  }
}

}  // namespace

hipError_t launch_merge_detections(const float* coarse, const float* fine, const int32_t* hard,
                                   int B, int Q, float tau_hi, float tau_fine, float* det,
                                   uint8_t* src, int32_t* count, hipStream_t s) {
  hipLaunchKernelGGL(merge_detections_kernel, dim3(B), dim3(kRoiThreads), 0, s, coarse, fine, hard,
                     Q, tau_hi, tau_fine, det, src, count);
  return hipGetLastError();
}

hipError_t launch_propose_rois(const float* queries, int B, int Q, int H, int W, float tau_hi,
                               float tau_lo, float scale, float min_side, int tier_value,
                               int32_t* n_roi, int max_boxes, int32_t* boxes, uint8_t* tier,
                               int32_t* box_offsets, int32_t* hard, float* mean_conf,
                               int32_t* err_flag, hipStream_t s) {
  hipLaunchKernelGGL(roi_stats_kernel, dim3(B), dim3(kRoiThreads), 0, s, queries, Q, tau_hi,
                     tau_lo, hard, mean_conf, n_roi);
  hipLaunchKernelGGL(roi_emit_kernel, dim3(B), dim3(kRoiThreads), 0, s, queries, B, Q, H, W,
                     tau_hi, tau_lo, scale, min_side, tier_value, n_roi, max_boxes, boxes, tier,
                     box_offsets, err_flag);
  return hipGetLastError();
}

}  // namespace cfdetr
