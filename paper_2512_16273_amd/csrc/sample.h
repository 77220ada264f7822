// tslt_sample: inverse-CDF draws from truncated distributions (the sample step of Algorithm 2,
// Algorithm 4 for several candidates), one wave per row, fp64 throughout.
#pragma once
#include "common.h"
#include "exp64.h"

namespace tslt {

constexpr int kSamplePer = 16;   // entries per lane: 64 * 16 = TSLT_MAX_K_CAP

struct SampleParams {
  const int32_t* idx;
  const float* logit;
  const int32_t* count;
  int64_t rows;
  int k_cap;
  const float* u;
  int n_samples;
  int without_replacement;
  int32_t* out_token;
  int32_t* out_slot;
};

__global__ __launch_bounds__(64) void sample_kernel(const SampleParams p) {
  const int64_t row = blockIdx.x;
  const int lane = threadIdx.x;
  int count = p.count[row];
  if (count > p.k_cap) count = p.k_cap;
  if (count < 0) count = 0;
  const float* lg = p.logit + size_t(row) * p.k_cap;
  const int32_t* ix = p.idx + size_t(row) * p.k_cap;
  const int per = (count + 63) / 64;               // entries per lane, contiguous
  double w[kSamplePer];
  const double s0 = count > 0 ? double(lg[0]) : 0.0;
#pragma unroll
  for (int r = 0; r < kSamplePer; ++r) {
    const int i = lane * per + r;
    w[r] = (r < per && i < count) ? exp64(double(lg[i]) - s0) : 0.0;
  }
  for (int c = 0; c < p.n_samples; ++c) {
    double local = 0.0;
#pragma unroll
    for (int r = 0; r < kSamplePer; ++r) local += w[r];
    // inclusive scan of the lane totals
    const double inc = wave_incl_scan_f64(local);
    const double total = last_lane_f64(inc);
    int slot = -1;
    if (total > 0.0) {
      const double target = double(p.u[size_t(row) * p.n_samples + c]) * total;
      double run = inc - local;
      int not_above = 0, last_pos = -1;
#pragma unroll
      for (int r = 0; r < kSamplePer; ++r) {
        const int i = lane * per + r;
        if (r < per && i < count) {
          run += w[r];
          not_above += run > target ? 0 : 1;
          if (w[r] > 0.0) last_pos = i;
        }
      }
      slot = wave_sum_i32(not_above);   // prefix sums are non-decreasing: first bucket above the target
      if (slot >= count) {              // only for u >= 1: the last bucket that has weight
        slot = wave_max_i32(last_pos);
      }
      if (p.without_replacement) {
#pragma unroll
        for (int r = 0; r < kSamplePer; ++r)
          if (lane * per + r == slot) w[r] = 0.0;
      }
    }
    if (lane == 0) {
      const size_t o = size_t(row) * p.n_samples + c;
      p.out_token[o] = slot >= 0 ? ix[slot] : -1;
      if (p.out_slot) p.out_slot[o] = slot;
    }
  }
}

}  // namespace tslt
