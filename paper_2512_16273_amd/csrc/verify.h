// tslt_verify: token-sequence verification (Algorithm 3) against sparse draft distributions.
//
// Kernel A, one workgroup per (sequence, draft position): eval_row_on_set over the target row, then
// the ratio p(x)/q_hat(x) of the draft token, the acceptance decision u < min(1, ratio) and Lemma 1's
// sum min(p, q_hat).
// Kernel B1, a few workgroups per sequence: finds the first rejected position j (or the bonus row)
// from kernel A's decisions and sweeps that one target row in fp64, each workgroup a segment.
// Kernel B2, one workgroup per sequence: inverse CDF of norm(max(0, p - q_hat)) (or of p for the bonus
// row) from the sweep's sums, and the sequence's outputs.  (Two kernels rather than a "last workgroup
// finishes" scheme: a device-scope fence per workgroup writes back and invalidates the L2 of the XCD,
// which costs far more than a launch.)
#pragma once
#include "rowops.h"

namespace tslt {

struct VerifyParams {
  const void* target;
  int64_t B, V, row_stride;
  int gamma;
  float rT, k2;
  const int32_t* q_idx;
  const float* q_logit;
  const int32_t* q_count;
  int k_cap;
  const int32_t* draft_tokens;
  const float* u_accept;
  const float* u_resample;
  int32_t* out_accept_len;
  int32_t* out_tokens;
  float* out_ratio;
  float* out_beta;
  int32_t* status;
  // workspace
  int32_t* flags;        // [B, gamma] 1 accepted, 0 rejected, 2 row unusable
  int32_t* row_status;   // [B, gamma]
  SegResult* segs;       // [B, n_seg + 2]
  double* subs;          // [B, n_seg, kSubChunks] mass of every run of a segment, in the segment's units
  int n_seg;             // body segments per row (upper bound used for the layout)
  int n_seg_grid;        // segment groups of kernel B1 per sequence
  int use_table;         // kernel B1 sums bf16 rows through the exp table
};

inline size_t verify_workspace_bytes(int64_t B, int64_t gamma, int64_t V, int k_cap) {
  (void)k_cap;
  const size_t n_seg = size_t(row_segments(V));
  return align256(size_t(B) * gamma * 4) * 2 + align256(size_t(B) * (n_seg + 2) * sizeof(SegResult)) +
         align256(size_t(B) * n_seg * kSubChunks * sizeof(double));
}
inline void verify_carve_workspace(VerifyParams& p, void* ws) {
  char* w = reinterpret_cast<char*>(ws);
  p.n_seg = row_segments(p.V);
  p.flags = reinterpret_cast<int32_t*>(w); w += align256(size_t(p.B) * p.gamma * 4);
  p.row_status = reinterpret_cast<int32_t*>(w); w += align256(size_t(p.B) * p.gamma * 4);
  p.segs = reinterpret_cast<SegResult*>(w); w += align256(size_t(p.B) * (p.n_seg + 2) * sizeof(SegResult));
  p.subs = reinterpret_cast<double*>(w);
}

template <typename T> __device__ __forceinline__ const void* target_row(const VerifyParams& p, int64_t b, int j) {
  return reinterpret_cast<const char*>(p.target) +
         (size_t(b) * (p.gamma + 1) + j) * size_t(p.row_stride) * ElemTraits<T>::kBytes;
}

// ---------------------------------------------------------------------------------------------
// Kernel A
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kBlock) void verify_accept_kernel(const VerifyParams p) {
  __shared__ VerifyShared sh;
  const int tid = threadIdx.x;
  const int64_t r = blockIdx.x;            // row index in [0, B*gamma)
  const int64_t b = r / p.gamma;
  const int j = int(r - b * p.gamma);
  const void* row = target_row<T>(p, b, j);
  const RowSplit rs = split_row<T>(row, p.V);
  int count = p.q_count[r];
  count = count < 0 ? 0 : (count > p.k_cap ? p.k_cap : count);
  double p_s[kSetPer], q_s[kSetPer], p_out;
  int yi[kSetPer], st;
  bool ok;
  eval_row_on_set<T>(row, rs, p.V, p.rT, p.k2, p.q_idx + size_t(r) * p.k_cap, p.q_logit + size_t(r) * p.k_cap, count, sh,
                     p_s, q_s, yi, p_out, ok, st);
  const int x = p.draft_tokens[r];
  double beta = 0.0;
  if (tid == 0) { sh.bcast_d[0] = -1.0; sh.bcast_i[0] = 0; }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kSetPer; ++k) {
    if (tid + k * kBlock < count && ok) {
      beta += p_s[k] < q_s[k] ? p_s[k] : q_s[k];
      if (yi[k] == x && q_s[k] > 0.0) {
        // the first matching entry decides (sets have distinct indices)
        if (atomicCAS(&sh.bcast_i[0], 0, 1) == 0) sh.bcast_d[0] = p_s[k] / q_s[k];
      }
    }
  }
  beta = block_sum_f64<kWaves>(beta, sh.red);
  if (tid == 0) {
    const double ratio = sh.bcast_d[0];
    int flag;
    if (!ok) flag = 2;
    else {
      if (sh.bcast_i[0] == 0) { st |= 4; flag = 0; }
      else {
        const double bound = ratio < 1.0 ? ratio : 1.0;
        flag = double(p.u_accept[r]) < bound ? 1 : 0;
      }
    }
    p.flags[r] = flag;
    p.row_status[r] = st;
    if (p.out_ratio) p.out_ratio[r] = ok ? float(ratio) : NAN;
    if (p.out_beta) p.out_beta[r] = ok ? float(beta) : NAN;
  }
}

// ---------------------------------------------------------------------------------------------
// Kernels B1 and B2
// ---------------------------------------------------------------------------------------------
// First rejected position of sequence b, or gamma when every draft token was accepted (block-wide).
__device__ __forceinline__ int first_rejection(const VerifyParams& p, int64_t b, VerifyShared& sh) {
  const int tid = threadIdx.x;
  int jstar = p.gamma;
  for (int j = tid; j < p.gamma; j += kBlock)
    if (p.flags[b * p.gamma + j] != 1) { jstar = j; break; }
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) { const int o = __shfl_xor(jstar, s, 64); jstar = o < jstar ? o : jstar; }
  __syncthreads();
  if (lane_id() == 0) sh.red.i[wave_id()] = jstar;
  __syncthreads();
  jstar = sh.red.i[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) jstar = sh.red.i[w] < jstar ? sh.red.i[w] : jstar;
  __syncthreads();
  return jstar;
}

// Workgroups are persistent: each builds the exp table once (bf16 rows) and then takes the
// (sequence, segment group) items blockIdx.x, blockIdx.x + gridDim.x, ...
template <typename T>
__global__ __launch_bounds__(kBlock) void verify_sweep_kernel(const VerifyParams p) {
  __shared__ VerifyShared sh;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  double* table = nullptr;
  if (std::is_same<T, Bf16>::value && p.use_table) {
    table = reinterpret_cast<double*>(dyn_lds);
    build_exp_table(table, p.rT);
  }
  const int n_seg_grid = p.n_seg_grid;      // segment groups per sequence (layout bound; rows may need fewer)
  const int64_t n_items = p.B * n_seg_grid;
  for (int64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int64_t b = item / n_seg_grid;
    const int seg = int(item - b * n_seg_grid);
    const int jstar = first_rejection(p, b, sh);
    if (jstar < p.gamma && p.flags[b * p.gamma + jstar] == 2) continue;   // unusable row: nothing to sample
    const void* row = target_row<T>(p, b, jstar);
    const RowSplit rs = split_row<T>(row, p.V);
    // a row that kernel A has accepted or rejected has been validated there; the bonus row is checked here
    sweep_group<T>(row, rs, seg, jstar == p.gamma, p.rT, table, p.segs + size_t(b) * (p.n_seg + 2),
                     p.subs + size_t(b) * p.n_seg * kSubChunks, sh);
    __syncthreads();
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void verify_finish_kernel(const VerifyParams p) {
  __shared__ VerifyShared sh;
  const int tid = threadIdx.x;
  const int64_t b = blockIdx.x;
  const int jstar = first_rejection(p, b, sh);
  int st = 0;
  for (int j = tid; j <= jstar && j < p.gamma; j += kBlock) st |= p.row_status[b * p.gamma + j];
  st = block_or_i32<kWaves>(st, sh.red);

  FinishArgs a;
  a.row = target_row<T>(p, b, jstar);
  a.rs = split_row<T>(a.row, p.V);
  a.n_seg_row = int((a.rs.nvec + kSegVecsTotal - 1) / kSegVecsTotal);
  a.V = p.V;
  a.rT = p.rT;
  a.segs = p.segs + size_t(b) * (p.n_seg + 2);
  a.subs = p.subs + size_t(b) * p.n_seg * kSubChunks;
  const bool residual = jstar < p.gamma;
  const int64_t r = b * p.gamma + (residual ? jstar : 0);
  int count = residual ? p.q_count[r] : 0;
  a.count = count < 0 ? 0 : (count > p.k_cap ? p.k_cap : count);
  a.qi = p.q_idx + size_t(r) * p.k_cap;
  a.ql = p.q_logit + size_t(r) * p.k_cap;
  a.stages = residual ? 1 : 0;
  a.u = p.u_resample[b * (p.gamma + 1) + jstar];
  a.unusable = residual && p.flags[b * p.gamma + jstar] == 2;
  const int token = finish_core<T>(a, sh, st);

  int32_t* ot = p.out_tokens + size_t(b) * (p.gamma + 1);
  for (int j = tid; j <= p.gamma; j += kBlock) {
    int v = -1;
    if (j < jstar) v = p.draft_tokens[b * p.gamma + j];
    else if (j == jstar) v = token;
    ot[j] = v;
  }
  if (tid == 0) {
    p.out_accept_len[b] = jstar;
    if (p.status) p.status[b] = st;
  }
}

// phases: bit 0 = kernel A (acceptance decisions), bit 1 = kernels B1 and B2 (resampling and outputs)
template <typename T> hipError_t launch_verify(VerifyParams p, hipStream_t s, int phases) {
  hipError_t e = hipSuccess;
  if (phases & 1) {
    hipLaunchKernelGGL(verify_accept_kernel<T>, dim3(unsigned(p.B * p.gamma)), dim3(kBlock), 0, s, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (phases & 2) {
    const int E = ElemTraits<T>::kPerVec;
    int n_seg = int((p.V / E + 1 + kSegVecsTotal - 1) / kSegVecsTotal);
    if (n_seg > p.n_seg) n_seg = p.n_seg;
    p.n_seg_grid = (n_seg + kGroupSegs - 1) / kGroupSegs;
    p.use_table = std::is_same<T, Bf16>::value && exp_table_usable(p.rT) ? 1 : 0;
    const int64_t grid = std::min<int64_t>(p.B * p.n_seg_grid, sweep_grid_limit());
    hipLaunchKernelGGL(verify_sweep_kernel<T>, dim3(unsigned(grid)), dim3(kBlock), p.use_table ? kTabBytes : 0, s, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(verify_finish_kernel<T>, dim3(unsigned(p.B)), dim3(kBlock), 0, s, p);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace tslt
