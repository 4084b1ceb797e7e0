// Batch-level kernels around the per-string encoder: length binning (which kernel variant encodes which
// string, longest strings first), the scan of token counts into out_offsets, and the packing of the
// per-string id runs into the dense output (the paper only says that the result is an id tensor,
// section 2.2; the dense ids + offsets layout is this library's).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bpe {

constexpr int kMaxTiers = 4;
constexpr int kLenBuckets = 64;                      // length classes inside a tier, longest first
constexpr int kBinKeys = kMaxTiers * kLenBuckets;

struct TierPlan {
  int n_tiers;
  int cap[kMaxTiers];                                // tier t takes strings with cap[t-1] < len <= cap[t]
};

// Control block at the start of the workspace.
struct Control {
  uint32_t tier_base[kMaxTiers + 1];                 // start of each tier's slice of the list
  uint32_t queue_head[kMaxTiers];                    // work-queue heads of the encode kernels
};

__device__ inline int bin_key(int len, const TierPlan& plan) {
  int lo = 0;
  for (int t = 0; t < plan.n_tiers; ++t) {
    const int cap = plan.cap[t];
    if (len <= cap) {
      // bucket 0 holds the longest strings of the tier
      const int span = cap - lo;
      int b = span > 0 ? (int)(((uint32_t)(cap - len) * (uint32_t)kLenBuckets) / (uint32_t)span) : 0;
      if (b >= kLenBuckets) b = kLenBuckets - 1;
      return t * kLenBuckets + b;
    }
    lo = cap;
  }
  return -1;                                         // longer than any launched variant: skipped
}

// One workgroup bins the whole batch: histogram of (class, length bucket) keys in LDS, exclusive scan of the
// 256 keys, then the scatter of string indices into the work list (class-major, longest bucket first).
// Also resets the work-queue heads.  A second pass over the offsets is cheaper than a second launch.
__global__ __launch_bounds__(1024) void bin_kernel(const int64_t* offsets, int batch, TierPlan plan, Control* c,
                                                   int32_t* list, int32_t* counts) {
  __shared__ uint32_t hist[kBinKeys], scan[kBinKeys], cursor[kBinKeys];
  const int t = threadIdx.x;
  if (t < kBinKeys) { hist[t] = 0; cursor[t] = 0; }
  __syncthreads();
  for (int s = t; s < batch; s += 1024) {
    const int64_t len = offsets[s + 1] - offsets[s];
    const int key = (len < 0 || len > 0x7FFFFFFF) ? -1 : bin_key((int)len, plan);
    if (key >= 0) atomicAdd(&hist[key], 1u);
    else counts[s] = 0;                              // never encoded: contributes no tokens
  }
  __syncthreads();
  if (t < kBinKeys) scan[t] = hist[t];
  __syncthreads();
  for (int step = 1; step < kBinKeys; step <<= 1) {  // inclusive scan, all threads reach the barriers
    uint32_t v = 0;
    if (t < kBinKeys && t >= step) v = scan[t - step];
    __syncthreads();
    if (t < kBinKeys) scan[t] += v;
    __syncthreads();
  }
  if (t <= kMaxTiers) c->tier_base[t] = t == 0 ? 0 : scan[(t <= plan.n_tiers ? t : plan.n_tiers) * kLenBuckets - 1];
  if (t < kMaxTiers) c->queue_head[t] = 0;
  for (int s = t; s < batch; s += 1024) {
    const int64_t len = offsets[s + 1] - offsets[s];
    const int key = (len < 0 || len > 0x7FFFFFFF) ? -1 : bin_key((int)len, plan);
    if (key < 0) continue;
    const uint32_t pos = (scan[key] - hist[key]) + atomicAdd(&cursor[key], 1u);
    list[pos] = s;
  }
}

// out_offsets[i] = sum of counts[0..i), out_offsets[batch] = total.  One workgroup walks the batch.
__global__ __launch_bounds__(1024) void offsets_scan_kernel(const int32_t* counts, int batch,
                                                            int64_t* out_offsets) {
  __shared__ int64_t wave_sum[16];
  __shared__ int64_t carry_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) { carry_s = 0; out_offsets[0] = 0; }
  __syncthreads();
  for (int base = 0; base < batch; base += 1024) {
    const int i = base + tid;
    int64_t v = i < batch ? (int64_t)counts[i] : 0;
    for (int step = 1; step < 64; step <<= 1) {
      int64_t o = __shfl_up(v, step, 64);
      if (lane >= step) v += o;
    }
    if (lane == 63) wave_sum[wave] = v;
    __syncthreads();
    int64_t before = carry_s;
    for (int w = 0; w < wave; ++w) before += wave_sum[w];
    if (i < batch) out_offsets[i + 1] = before + v;
    __syncthreads();
    if (tid == 1023) carry_s = before + v;
    __syncthreads();
  }
}

// One workgroup per string: copy its ids from the per-string staging area to the dense output.
__global__ __launch_bounds__(256) void pack_kernel(const int32_t* tmp_ids, const int64_t* offsets,
                                                   const int64_t* out_offsets, int batch, int32_t* out_ids) {
  for (int s = blockIdx.x; s < batch; s += gridDim.x) {
    const int64_t src = offsets[s], dst = out_offsets[s];
    const int k = (int)(out_offsets[s + 1] - dst);
    for (int i = threadIdx.x; i < k; i += blockDim.x) out_ids[dst + i] = tmp_ids[src + i];
  }
}

}  // namespace bpe
