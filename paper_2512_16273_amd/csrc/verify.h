// tslt_verify: token-sequence verification (Algorithm 3) against sparse draft distributions.
//
// Kernel A, one workgroup per (sequence, draft position): one streaming pass over the target row
// for the softmax normaliser (fp32 partial sums of exp2(t*k2 - c), c referenced to the largest
// target logit found at the draft set's indices), then, in fp64 over the <= k_cap received entries,
// p at those indices, q_hat = softmax of the received values, the ratio p(x)/q_hat(x) of the draft
// token, the acceptance decision u < min(1, ratio) and Lemma 1's sum min(p, q_hat).
//
// Kernel B1, a few workgroups per sequence: finds the first rejected position j (or the bonus row)
// from kernel A's decisions and sweeps that one target row in fp64, each workgroup a segment.
// Kernel B2, one workgroup per sequence: combines the segment sums, applies the sparse corrections
// max(0, p - q_hat) - p at the draft set's indices, locates the segment, the 64-element chunk and
// finally the element at which the cumulative residual mass passes u * total, and writes the
// sequence's outputs.  (Two kernels rather than a "last workgroup finishes" scheme: a device-scope
// fence per workgroup writes back and invalidates the L2 of the XCD, which costs far more than a
// launch.)  fp64 is needed here: at V >= 128k the buckets of the inverse CDF are far
// narrower than fp32 prefix sums can resolve.
#pragma once
#include "common.h"
#include "exp64.h"

namespace tslt {

constexpr int kSegVecs = 4;                         // 16-byte vectors per thread in a kernel-B segment
constexpr int kSegVecsTotal = kSegVecs * kBlock;    // vectors per segment

constexpr int kSubChunks = kSegVecs * kWaves;       // runs of 64 consecutive vectors per segment

struct SegResult {       // one segment (or edge piece) of the resampled row
  double sum;            // sum of exp(s - smax) over the piece
  float smax;            // largest scaled logit of the piece (-inf if empty)
  int bad;               // NaN or +inf seen
};

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
  SegResult* segs;       // [B, n_pieces]
  double* subs;          // [B, n_seg, kSubChunks] sums of exp(s - smax of the segment) per run of 64 vectors
  int n_seg;             // body segments per row (upper bound used for the layout)
  int n_seg_grid;        // workgroups of kernel B1 per sequence
};

inline int verify_segments(int64_t V) {
  // body vectors are at most V / 4 (fp32); one more segment covers a ragged end
  const int64_t nvec_max = V / 4 + 1;
  return int((nvec_max + kSegVecsTotal - 1) / kSegVecsTotal);
}
inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }
inline size_t verify_workspace_bytes(int64_t B, int64_t gamma, int64_t V, int k_cap) {
  (void)k_cap;
  const size_t n_pieces = size_t(verify_segments(V)) + 2;
  return align256(size_t(B) * gamma * 4) * 2 + align256(size_t(B) * n_pieces * sizeof(SegResult)) +
         align256(size_t(B) * verify_segments(V) * kSubChunks * sizeof(double));
}
inline void verify_carve_workspace(VerifyParams& p, void* ws) {
  char* w = reinterpret_cast<char*>(ws);
  p.flags = reinterpret_cast<int32_t*>(w); w += align256(size_t(p.B) * p.gamma * 4);
  p.row_status = reinterpret_cast<int32_t*>(w); w += align256(size_t(p.B) * p.gamma * 4);
  p.n_seg = verify_segments(p.V);
  p.segs = reinterpret_cast<SegResult*>(w); w += align256(size_t(p.B) * (p.n_seg + 2) * sizeof(SegResult));
  p.subs = reinterpret_cast<double*>(w);
}

struct VerifyShared {
  BlockScratch red;
  double bcast_d[4];
  int bcast_i[4];
  double piece_val[kBlock];        // level 1: mass of every piece (n_pieces <= kBlock)
  double sub_val[kSubChunks];      // level 2: mass of every run of 64 vectors of the chosen segment
  double elem_corr[64 * 8];        // level 3: sparse correction per element of the chosen run
};

template <typename T> __device__ __forceinline__ const void* target_row(const VerifyParams& p, int64_t b, int j) {
  return reinterpret_cast<const char*>(p.target) +
         (size_t(b) * (p.gamma + 1) + j) * size_t(p.row_stride) * ElemTraits<T>::kBytes;
}

// ---------------------------------------------------------------------------------------------
// Kernel A
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kBlock) void verify_accept_kernel(const VerifyParams p) {
  constexpr int E = ElemTraits<T>::kPerVec;
  constexpr int kMaxPer = TSLT_MAX_K_CAP / kBlock;
  __shared__ VerifyShared sh;
  const int tid = threadIdx.x;
  const int64_t r = blockIdx.x;            // row index in [0, B*gamma)
  const int64_t b = r / p.gamma;
  const int j = int(r - b * p.gamma);
  const void* row = target_row<T>(p, b, j);
  const RowSplit rs = split_row<T>(row, p.V);
  const int n_edge = rs.head + rs.tail;
  const int64_t n_tiles = (rs.nvec + kBlock - 1) / kBlock;

  // ---- the received sparse set: gather the target logits at its indices -----------------------
  int count = p.q_count[r];
  count = count < 0 ? 0 : (count > p.k_cap ? p.k_cap : count);
  const int32_t* qi = p.q_idx + size_t(r) * p.k_cap;
  const float* ql = p.q_logit + size_t(r) * p.k_cap;
  float tv[kMaxPer];       // raw target logit at entry
  int yi[kMaxPer];
  float gmax = -INFINITY;
#pragma unroll
  for (int k = 0; k < kMaxPer; ++k) {
    const int i = tid + k * kBlock;
    tv[k] = -INFINITY; yi[k] = -1;
    if (i < count) {
      const int y = qi[i];
      if (y >= 0 && y < p.V) { yi[k] = y; tv[k] = load_elem<T>(row, y); }
      gmax = fmaxf(gmax, tv[k]);
    }
  }
  float vref = block_max_f32<kWaves>(gmax, sh.red);
  if (!(vref > -INFINITY && vref < INFINITY)) {
    // no usable reference in the set: take the start of the row
    float m0 = -INFINITY;
    for (int64_t i = tid; i < p.V && i < 4096; i += kBlock) m0 = fmaxf(m0, load_elem<T>(row, i));
    vref = block_max_f32<kWaves>(m0, sh.red);
  }
  int st = 0;
  double z_c = 0.0;
  float c_ref = __fmul_rn(vref, p.k2);
  bool ok = vref > -INFINITY && vref < INFINITY;
  if (ok) {
    const float k2 = p.k2, neg_c = -c_ref;
    float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
    constexpr int U = 4;
    for (int64_t t0 = 0; t0 < n_tiles; t0 += U) {
      uint4 d[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t vi = (t0 + u) * kBlock + tid;
        d[u] = neg_inf_vec<T>();
        if (vi < rs.nvec) d[u] = load_vec_stream(&rs.body[vi]);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float v[E];
        unpack<T>(d[u], v);
#pragma unroll
        for (int e = 0; e < E; e += 4) {
          acc0 += fast_exp2(__builtin_fmaf(v[e + 0], k2, neg_c));
          acc1 += fast_exp2(__builtin_fmaf(v[e + 1], k2, neg_c));
          acc2 += fast_exp2(__builtin_fmaf(v[e + 2], k2, neg_c));
          acc3 += fast_exp2(__builtin_fmaf(v[e + 3], k2, neg_c));
        }
      }
    }
    if (tid < n_edge) acc0 += fast_exp2(__builtin_fmaf(load_elem<T>(row, edge_index<T>(rs, tid)), k2, neg_c));
    z_c = block_sum_f64<kWaves>(double(acc0) + double(acc1) + double(acc2) + double(acc3), sh.red);
    ok = z_c > 0.0 && z_c < INFINITY;
  }
  if (!ok) {
    // exact redo: validity and true maximum first, then the sum referenced to it
    int bad = 0, fin = 0;
    float vmax = -INFINITY;
    for (int64_t i = tid; i < p.V; i += kBlock) {
      float v = load_elem<T>(row, i);
      if (v != v || v == INFINITY) bad = 1;
      else if (v > -INFINITY) { fin = 1; vmax = fmaxf(vmax, v); }
    }
    bad = block_sum_i32<kWaves>(bad, sh.red);
    fin = block_sum_i32<kWaves>(fin, sh.red);
    vmax = block_max_f32<kWaves>(vmax, sh.red);
    if (bad) st |= 1;
    else if (!fin) st |= 2;
    else {
      vref = vmax;
      c_ref = __fmul_rn(vref, p.k2);
      float acc = 0.f;
      for (int64_t i = tid; i < p.V; i += kBlock) acc += fast_exp2(__builtin_fmaf(load_elem<T>(row, i), p.k2, -c_ref));
      z_c = block_sum_f64<kWaves>(double(acc), sh.red);
      ok = true;
    }
  }

  // ---- fp64 over the set: p, q_hat, ratio, sum of min ------------------------------------------
  const float s_ref = __fmul_rn(vref, p.rT);
  const double ql0 = count > 0 ? double(ql[0]) : 0.0;
  double e64[kMaxPer], w64[kMaxPer];
  double sum_e = 0.0, sum_t32 = 0.0, sum_w = 0.0;
#pragma unroll
  for (int k = 0; k < kMaxPer; ++k) {
    const int i = tid + k * kBlock;
    e64[k] = 0.0; w64[k] = 0.0;
    if (i < count) {
      w64[k] = exp64(double(ql[i]) - ql0);
      sum_w += w64[k];
      if (yi[k] >= 0 && tv[k] > -INFINITY && ok) {
        e64[k] = exp64(double(__fmul_rn(tv[k], p.rT)) - double(s_ref));
        sum_e += e64[k];
        sum_t32 += double(fast_exp2(__builtin_fmaf(tv[k], p.k2, -c_ref)));
      }
    }
  }
  sum_e = block_sum_f64<kWaves>(sum_e, sh.red);
  sum_t32 = block_sum_f64<kWaves>(sum_t32, sh.red);
  sum_w = block_sum_f64<kWaves>(sum_w, sh.red);
  double tail = z_c - sum_t32;
  if (tail < 0.0) tail = 0.0;
  const double Z = tail * exp2(double(c_ref) - double(vref) * double(p.k2)) + sum_e;
  const int x = p.draft_tokens[r];
  double beta = 0.0;
  if (tid == 0) { sh.bcast_d[0] = -1.0; sh.bcast_i[0] = 0; }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kMaxPer; ++k) {
    const int i = tid + k * kBlock;
    if (i < count && ok) {
      const double pi = e64[k] / Z, qh = w64[k] / sum_w;
      beta += pi < qh ? pi : qh;
      if (yi[k] == x && qh > 0.0) {
        // the first matching entry decides (sets have distinct indices)
        if (atomicCAS(&sh.bcast_i[0], 0, 1) == 0) sh.bcast_d[0] = pi / qh;
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
// Kernel B
// ---------------------------------------------------------------------------------------------
// Piece index (0 head edge, 1..n body segments, n+1 tail edge) that holds element y of the row.
template <typename T> __device__ __forceinline__ int piece_of(const RowSplit& rs, int n_seg_row, int64_t y) {
  constexpr int E = ElemTraits<T>::kPerVec;
  if (y < rs.head) return 0;
  const int64_t v = (y - rs.head) / E;
  if (v >= rs.nvec) return n_seg_row + 1;
  return 1 + int(v / kSegVecsTotal);
}

template <typename T>
__device__ void resample_finish(const VerifyParams& p, VerifyShared& sh, int64_t b, int jstar, const void* row,
                                const RowSplit& rs, int n_seg_row, int broken_flag) {
  constexpr int E = ElemTraits<T>::kPerVec;
  constexpr int kMaxPer = TSLT_MAX_K_CAP / kBlock;
  constexpr int kRun = 64 * E;              // elements in a run of 64 vectors
  constexpr int kPerT = kRun / kBlock;      // elements per thread at level 3
  const int tid = threadIdx.x;
  const int n_pieces = n_seg_row + 2;
  const SegResult* segs = p.segs + size_t(b) * (p.n_seg + 2);
  int st = 0;
  for (int j = tid; j <= jstar && j < p.gamma; j += kBlock) st |= p.row_status[b * p.gamma + j];
  st = block_or_i32<kWaves>(st, sh.red);

  // maximum and validity of the row, from the pieces
  float smax = -INFINITY;
  int bad = 0;
  if (!broken_flag)
    for (int k = tid; k < n_pieces; k += kBlock) { smax = fmaxf(smax, segs[k].smax); bad |= segs[k].bad; }
  smax = block_max_f32<kWaves>(smax, sh.red);
  bad = __syncthreads_or(bad);
  int token = -1;
  const bool usable = !broken_flag && !bad && smax > -INFINITY;
  if (!broken_flag && bad) st |= 1;
  if (!broken_flag && !bad && !(smax > -INFINITY)) st |= 2;

  if (usable) {
    // unnormalised target mass of every piece, referenced to the row maximum, and their total z_p
    double zp = 0.0;
    for (int k = tid; k < n_pieces; k += kBlock) {
      const double t = segs[k].smax > -INFINITY ? segs[k].sum * exp64(double(segs[k].smax) - double(smax)) : 0.0;
      sh.piece_val[k] = t;
      zp += t;
    }
    zp = block_sum_f64<kWaves>(zp, sh.red);

    // sparse corrections at the draft set's indices (none for the bonus row):
    // residual(y) = max(0, e_y - z_p * q_hat(y)) replaces e_y
    const bool residual = jstar < p.gamma;
    const int64_t r = b * p.gamma + (residual ? jstar : 0);
    int count = residual ? p.q_count[r] : 0;
    count = count < 0 ? 0 : (count > p.k_cap ? p.k_cap : count);
    const int32_t* qi = p.q_idx + size_t(r) * p.k_cap;
    const float* ql = p.q_logit + size_t(r) * p.k_cap;
    const double ql0 = count > 0 ? double(ql[0]) : 0.0;
    double w64[kMaxPer], corr[kMaxPer];
    int yi[kMaxPer];
    double sum_w = 0.0;
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k) {
      const int i = tid + k * kBlock;
      w64[k] = 0.0; corr[k] = 0.0; yi[k] = -1;
      if (i < count) { w64[k] = exp64(double(ql[i]) - ql0); sum_w += w64[k]; }
    }
    sum_w = block_sum_f64<kWaves>(sum_w, sh.red);
    double sum_corr = 0.0;
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k) {
      const int i = tid + k * kBlock;
      if (i < count) {
        const int y = qi[i];
        if (y >= 0 && y < p.V) {
          yi[k] = y;
          const float t = load_elem<T>(row, y);
          const double e = t > -INFINITY ? exp64(double(__fmul_rn(t, p.rT)) - double(smax)) : 0.0;
          const double res = e - zp * (w64[k] / sum_w);
          corr[k] = (res > 0.0 ? res : 0.0) - e;
          sum_corr += corr[k];
        }
      }
    }
    sum_corr = block_sum_f64<kWaves>(sum_corr, sh.red);
    double total = zp + sum_corr;
    bool use_corr = true;
    if (!(total > 0.0)) {          // defensive: an all-zero residual falls back to p itself
#pragma unroll
      for (int k = 0; k < kMaxPer; ++k) corr[k] = 0.0;
      total = zp;
      use_corr = false;
    }
    const double target = double(p.u_resample[b * (p.gamma + 1) + jstar]) * total;

    // ---- level 1: which piece ---------------------------------------------------------------------
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k)
      if (yi[k] >= 0 && corr[k] != 0.0) atomicAdd(&sh.piece_val[piece_of<T>(rs, n_seg_row, yi[k])], corr[k]);
    __syncthreads();
    if (tid == 0) {
      double run = 0.0, before = 0.0, last_before = 0.0;
      int piece = -1, last_pos = -1;
      for (int k = 0; k < n_pieces; ++k) {
        const double t = sh.piece_val[k];
        if (t > 0.0) {
          last_pos = k; last_before = run;
          if (run + t > target) { piece = k; before = run; break; }
          run += t;
        }
      }
      if (piece < 0) { piece = last_pos; before = last_before; }
      sh.bcast_i[0] = piece;
      sh.bcast_d[0] = before;
    }
    __syncthreads();
    const int piece = sh.bcast_i[0];
    const double before_piece = sh.bcast_d[0];
    __syncthreads();

    if (piece == 0 || piece == n_pieces - 1) {
      // an edge piece: fewer than E elements, walked by one thread
      if (tid == 0) {
        const int e0 = piece == 0 ? 0 : rs.head, e1 = piece == 0 ? rs.head : rs.head + rs.tail;
        double run = before_piece;
        for (int e = e0; e < e1; ++e) {
          const int64_t y = edge_index<T>(rs, e);
          const float t = load_elem<T>(row, y);
          double v = t > -INFINITY ? exp64(double(__fmul_rn(t, p.rT)) - double(smax)) : 0.0;
          if (use_corr)
            for (int i = 0; i < count; ++i)
              if (qi[i] == y) {
                const double res = v - zp * (exp64(double(ql[i]) - ql0) / sum_w);
                v = res > 0.0 ? res : 0.0;
                break;
              }
          if (v > 0.0) {
            token = int(y);
            run += v;
            if (run > target) break;
          }
        }
        sh.bcast_i[3] = token;
      }
      __syncthreads();
      token = sh.bcast_i[3];
    } else if (piece > 0) {
      // ---- level 2: which run of 64 consecutive vectors of the body segment ------------------------
      const int seg = piece - 1;
      const int64_t seg_first_vec = int64_t(seg) * kSegVecsTotal;
      const int64_t seg_first_elem = rs.head + seg_first_vec * E;
      const double seg_scale = exp64(double(segs[piece].smax) - double(smax));
      const double* subs = p.subs + (size_t(b) * p.n_seg + seg) * kSubChunks;
      if (tid < kSubChunks) sh.sub_val[tid] = subs[tid] * seg_scale;
      __syncthreads();
#pragma unroll
      for (int k = 0; k < kMaxPer; ++k)
        if (yi[k] >= 0 && corr[k] != 0.0 && piece_of<T>(rs, n_seg_row, yi[k]) == piece)
          atomicAdd(&sh.sub_val[(yi[k] - seg_first_elem) / kRun], corr[k]);
      __syncthreads();
      if (tid == 0) {
        double run = before_piece, before = before_piece, last_before = before_piece;
        int sub = -1, last_pos = -1;
        for (int c = 0; c < kSubChunks; ++c) {
          const double t = sh.sub_val[c];
          if (t > 0.0) {
            last_pos = c; last_before = run;
            if (run + t > target) { sub = c; before = run; break; }
            run += t;
          }
        }
        if (sub < 0) { sub = last_pos; before = last_before; }
        sh.bcast_i[1] = sub;
        sh.bcast_d[1] = before;
      }
      for (int i = tid; i < kRun; i += kBlock) sh.elem_corr[i] = 0.0;
      __syncthreads();
      const int sub = sh.bcast_i[1];
      const double before_run = sh.bcast_d[1];
      if (sub >= 0) {
        // ---- level 3: which element of that run; thread t owns kPerT consecutive elements ------------
        const int64_t run_first = seg_first_elem + int64_t(sub) * kRun;
#pragma unroll
        for (int k = 0; k < kMaxPer; ++k)
          if (yi[k] >= run_first && yi[k] < run_first + kRun) sh.elem_corr[yi[k] - run_first] = corr[k];
        __syncthreads();
        double v[kPerT];
        double mine = 0.0;
#pragma unroll
        for (int q = 0; q < kPerT; ++q) {
          const int64_t y = run_first + tid * kPerT + q;
          v[q] = 0.0;
          if ((y - rs.head) / E < rs.nvec) {
            const float t = load_elem<T>(row, y);
            v[q] = exp64(double(__fmul_rn(t, p.rT)) - double(smax)) + sh.elem_corr[tid * kPerT + q];
            if (v[q] < 0.0) v[q] = 0.0;
          }
          mine += v[q];
        }
        double run_total;
        const double excl = block_excl_scan_f64<kWaves>(mine, sh.red, run_total);
        // element at which the cumulative mass passes the target, else the last one with mass
        int first_pass = 0x7FFFFFFF, last_mass = -1;
        double run = before_run + excl;
#pragma unroll
        for (int q = 0; q < kPerT; ++q) {
          if (v[q] > 0.0) {
            run += v[q];
            last_mass = tid * kPerT + q;
            if (run > target && first_pass == 0x7FFFFFFF) first_pass = tid * kPerT + q;
          }
        }
#pragma unroll
        for (int m = 32; m > 0; m >>= 1) {
          const int o = __shfl_xor(first_pass, m, 64); first_pass = o < first_pass ? o : first_pass;
          const int q = __shfl_xor(last_mass, m, 64); last_mass = q > last_mass ? q : last_mass;
        }
        __syncthreads();
        if (lane_id() == 0) { sh.red.i[wave_id()] = first_pass; sh.red.i[8 + wave_id()] = last_mass; }
        __syncthreads();
        first_pass = 0x7FFFFFFF; last_mass = -1;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          first_pass = sh.red.i[w] < first_pass ? sh.red.i[w] : first_pass;
          last_mass = sh.red.i[8 + w] > last_mass ? sh.red.i[8 + w] : last_mass;
        }
        const int pick = first_pass != 0x7FFFFFFF ? first_pass : last_mass;
        token = pick >= 0 ? int(run_first + pick) : -1;
      }
    }
  }

  // ---- outputs of the sequence --------------------------------------------------------------------
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

// Kernel B1: fp64 sweep of the row to resample, one segment per workgroup.
template <typename T>
__global__ __launch_bounds__(kBlock) void verify_sweep_kernel(const VerifyParams p) {
  constexpr int E = ElemTraits<T>::kPerVec;
  __shared__ VerifyShared sh;
  const int tid = threadIdx.x;
  const int n_seg_grid = p.n_seg_grid;      // workgroups per sequence (layout bound; rows may need fewer)
  const int64_t b = blockIdx.x / n_seg_grid;
  const int seg = int(blockIdx.x - b * n_seg_grid);
  const int jstar = first_rejection(p, b, sh);
  const int broken = jstar < p.gamma && p.flags[b * p.gamma + jstar] == 2;
  const void* row = target_row<T>(p, b, jstar);
  const RowSplit rs = split_row<T>(row, p.V);
  const int n_seg_row = int((rs.nvec + kSegVecsTotal - 1) / kSegVecsTotal);
  SegResult* segs = p.segs + size_t(b) * (p.n_seg + 2);

  if (!broken && seg < n_seg_row) {
    // ---- this workgroup's segment, held in registers: maximum first, then the fp64 sums
    uint4 d[kSegVecs];
    const int64_t vbase = int64_t(seg) * kSegVecsTotal;
#pragma unroll
    for (int i = 0; i < kSegVecs; ++i) {
      const int64_t vi = vbase + int64_t(i) * kBlock + tid;
      d[i] = neg_inf_vec<T>();
      if (vi < rs.nvec) d[i] = load_vec(&rs.body[vi]);
    }
    // this segment's own maximum is the reference of its sums; a row that kernel A has accepted or
    // rejected has been validated there, the bonus row is checked here
    float vmax = -INFINITY;
    int bad = 0;
    const bool check = jstar == p.gamma;
#pragma unroll
    for (int i = 0; i < kSegVecs; ++i) {
      float v[E];
      unpack<T>(d[i], v);
      if (check) {
#pragma unroll
        for (int e = 0; e < E; ++e) bad |= (v[e] != v[e] || v[e] == INFINITY) ? 1 : 0;
      }
#pragma unroll
      for (int e = 0; e < E; e += 2) vmax = max3f(vmax, v[e], v[e + 1]);
    }
    vmax = block_max_f32<kWaves>(vmax, sh.red);
    bad = __syncthreads_or(bad);
    const float smax = __fmul_rn(vmax, p.rT);      // scaling is monotone: the largest s is at the largest t
    double* subs = p.subs + (size_t(b) * p.n_seg + seg) * kSubChunks;
    double sum = 0.0;
    if (smax > -INFINITY && !bad) {
      const double m = double(smax);
#pragma unroll
      for (int i = 0; i < kSegVecs; ++i) {
        float v[E];
        unpack<T>(d[i], v);
        double s0 = 0.0, s1 = 0.0;
#pragma unroll
        for (int e = 0; e < E; e += 2) {            // -inf gives exactly 0
          s0 += exp64(double(__fmul_rn(v[e], p.rT)) - m);
          s1 += exp64(double(__fmul_rn(v[e + 1], p.rT)) - m);
        }
        const double run_sum = wave_sum_f64(s0 + s1);   // run (i, wave): 64 consecutive vectors
        if (lane_id() == 0) subs[i * kWaves + wave_id()] = run_sum;
        sum += run_sum;
      }
    } else if (tid < kSubChunks) {
      subs[tid] = 0.0;
    }
    // every lane of a wave holds its wave's total
    __syncthreads();
    if (lane_id() == 0) sh.red.d[wave_id()] = sum;
    __syncthreads();
    if (tid == 0) {
      double t = 0.0;
      for (int w = 0; w < kWaves; ++w) t += sh.red.d[w];
      segs[1 + seg].sum = t; segs[1 + seg].smax = smax; segs[1 + seg].bad = bad;
    }
  }
  if (!broken && seg == 0 && tid == 0) {
    // the two edge pieces (at most E-1 elements each)
    for (int piece = 0; piece < 2; ++piece) {
      const int e0 = piece == 0 ? 0 : rs.head, e1 = piece == 0 ? rs.head : rs.head + rs.tail;
      float smax = -INFINITY;
      int bad = 0;
      for (int e = e0; e < e1; ++e) {
        const float t = load_elem<T>(row, edge_index<T>(rs, e));
        if (t != t || t == INFINITY) bad = 1;
        smax = fmaxf(smax, __fmul_rn(t, p.rT));
      }
      double sum = 0.0;
      if (smax > -INFINITY && !bad)
        for (int e = e0; e < e1; ++e) {
          const float t = load_elem<T>(row, edge_index<T>(rs, e));
          if (t > -INFINITY) sum += exp64(double(__fmul_rn(t, p.rT)) - double(smax));
        }
      SegResult& o = segs[piece == 0 ? 0 : n_seg_row + 1];
      o.sum = sum; o.smax = smax; o.bad = bad;
    }
  }
}

// Kernel B2: one workgroup per sequence combines the segments and draws the token.
template <typename T>
__global__ __launch_bounds__(kBlock) void verify_finish_kernel(const VerifyParams p) {
  __shared__ VerifyShared sh;
  const int64_t b = blockIdx.x;
  const int jstar = first_rejection(p, b, sh);
  const int broken = jstar < p.gamma && p.flags[b * p.gamma + jstar] == 2;
  const void* row = target_row<T>(p, b, jstar);
  const RowSplit rs = split_row<T>(row, p.V);
  const int n_seg_row = int((rs.nvec + kSegVecsTotal - 1) / kSegVecsTotal);
  resample_finish<T>(p, sh, b, jstar, row, rs, n_seg_row, broken);
}

// phases: bit 0 = kernel A (acceptance decisions), bit 1 = kernel B (resampling and outputs)
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
    p.n_seg_grid = n_seg;
    hipLaunchKernelGGL(verify_sweep_kernel<T>, dim3(unsigned(p.B * n_seg)), dim3(kBlock), 0, s, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(verify_finish_kernel<T>, dim3(unsigned(p.B)), dim3(kBlock), 0, s, p);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace tslt
