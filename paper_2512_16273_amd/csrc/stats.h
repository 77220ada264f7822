// tslt_truncation_stats: what truncation to the first K entries of a set does to the acceptance rate
// (Section 3.2: beta_hat = sum_x min(q_hat(x), p(x)) = 1 - TV(q_hat, p), Lemma 1; the quantity Theorem 1
// bounds).  A set is in canonical order, so its first K entries are the Top-K set of the same draft
// distribution: one pass over the target row serves every K of a list.
#pragma once
#include "rowops.h"

namespace tslt {

constexpr int kMaxStatK = 32;     // values of K per call

struct StatsParams {
  const void* target;
  int64_t rows, V, row_stride;
  float rT, k2;
  const int32_t* q_idx;
  const float* q_logit;
  const int32_t* q_count;
  int k_cap;
  int n_k;
  int k_list[kMaxStatK];
  float* out_keep;      // [rows, n_k]
  float* out_beta;      // [rows, n_k]
  int32_t* status;      // [rows] or null
};

// One workgroup per row: the pass of the acceptance kernel (normaliser of the target row, p and q_hat at
// the set's entries), then per K two block sums over the prefix.
template <typename T>
__global__ __launch_bounds__(kBlock, kAccWavesPerSimd) void truncation_stats_kernel(const StatsParams p) {
  __shared__ VerifyShared sh;
  const int tid = threadIdx.x;
  const int64_t r = blockIdx.x;
  const void* row = reinterpret_cast<const char*>(p.target) + size_t(r) * size_t(p.row_stride) * ElemTraits<T>::kBytes;
  const RowSplit rs = split_row<T>(row, p.V);
  int count = p.q_count[r];
  count = count < 0 ? 0 : (count > p.k_cap ? p.k_cap : count);
  double p_s[kSetPer], q_s[kSetPer], p_out;
  int yi[kSetPer], st;
  bool ok;
  eval_row_on_set<T>(row, rs, p.V, p.rT, p.k2, p.q_idx + size_t(r) * p.k_cap, p.q_logit + size_t(r) * p.k_cap, count, sh,
                     p_s, q_s, yi, p_out, ok, st);
  if (ok && count == 0) { ok = false; st |= 2; }
  for (int j = 0; j < p.n_k; ++j) {
    int k = p.k_list[j];
    k = k < 1 ? 1 : (k > count ? count : k);
    double c = 0.0;
#pragma unroll
    for (int s = 0; s < kSetPer; ++s)
      if (tid + s * kBlock < k) c += q_s[s];
    c = block_sum_f64<kWaves>(c, sh.red);
    double b = 0.0;
#pragma unroll
    for (int s = 0; s < kSetPer; ++s) {
      if (tid + s * kBlock < k && c > 0.0) {
        const double qk = q_s[s] / c;
        b += qk < p_s[s] ? qk : p_s[s];
      }
    }
    b = block_sum_f64<kWaves>(b, sh.red);
    if (tid == 0) {
      p.out_keep[r * p.n_k + j] = ok ? float(c) : NAN;
      p.out_beta[r * p.n_k + j] = ok ? float(b) : NAN;
    }
  }
  if (tid == 0 && p.status) p.status[r] = st;
}

// tslt_multicandidate_stats: Section 4.3's stage acceptance rates beta^(j) = sum_x min(q_hat(x), p^(j)(x)),
// j = 1..k, and the total rate theta = beta^(1) + sum_{i>=2} beta^(i) prod_{j<i} (1 - beta^(j)), for
// Algorithm 5 as printed (the same q_hat at every stage).  p^(j+1) = norm(max(0, p^(j) - q_hat)) does not
// depend on which candidates were drawn, so one pass over the target row serves all k stages: with a sparse
// q_hat the distribution p^(j) is a vector a on the set and a scalar multiple c of p off it (as in the tree
// kernel), q_hat is 0 off the set, so every beta^(j) is a sum over the set.
struct McStatsParams {
  const void* target;
  int64_t rows, V, row_stride;
  float rT, k2;
  const int32_t* q_idx;
  const float* q_logit;
  const int32_t* q_count;
  int k_cap;
  int k;                // stages
  float* out_beta;      // [rows, k]
  float* out_theta;     // [rows]
  int32_t* status;      // [rows] or null
};

template <typename T>
__global__ __launch_bounds__(kBlock, kAccWavesPerSimd) void multicandidate_stats_kernel(const McStatsParams p) {
  __shared__ VerifyShared sh;
  const int tid = threadIdx.x;
  const int64_t r = blockIdx.x;
  const void* row = reinterpret_cast<const char*>(p.target) + size_t(r) * size_t(p.row_stride) * ElemTraits<T>::kBytes;
  const RowSplit rs = split_row<T>(row, p.V);
  int count = p.q_count[r];
  count = count < 0 ? 0 : (count > p.k_cap ? p.k_cap : count);
  double a_s[kSetPer], q_s[kSetPer], p_out;
  int yi[kSetPer], st;
  bool ok;
  eval_row_on_set<T>(row, rs, p.V, p.rT, p.k2, p.q_idx + size_t(r) * p.k_cap, p.q_logit + size_t(r) * p.k_cap, count, sh,
                     a_s, q_s, yi, p_out, ok, st);
  if (ok && count == 0) { ok = false; st |= 2; }
  double c = 1.0, theta = 0.0, reach = 1.0;
  bool live = ok;                                   // false once a stage's residual is empty (block-uniform)
  for (int j = 0; j < p.k; ++j) {
    double shared = 0.0, part = 0.0;
#pragma unroll
    for (int q = 0; q < kSetPer; ++q) {
      shared += a_s[q] < q_s[q] ? a_s[q] : q_s[q];
      const double d = a_s[q] - q_s[q];
      a_s[q] = d > 0.0 ? d : 0.0;
      part += a_s[q];
    }
    const double beta = block_sum_f64<kWaves>(shared, sh.red);
    const double Z = block_sum_f64<kWaves>(part, sh.red) + c * p_out;
    if (tid == 0) p.out_beta[r * p.k + j] = live ? float(beta) : NAN;
    if (live) {
      theta += beta * reach;
      reach *= 1.0 - beta;
    }
    if (Z > 0.0) {
      const double inv_Z = 1.0 / Z;
#pragma unroll
      for (int q = 0; q < kSetPer; ++q) a_s[q] *= inv_Z;
      c *= inv_Z;
    } else {
      live = false;
    }
  }
  if (tid == 0) {
    p.out_theta[r] = ok ? float(theta) : NAN;
    if (p.status) p.status[r] = st;
  }
}

}  // namespace tslt
