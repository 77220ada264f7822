// tslt_verify: token-sequence verification (Algorithm 3) against sparse draft distributions.
//
// Kernel A, one workgroup per (sequence, draft position): eval_row_on_set over the target row, then
// the ratio p(x)/q_hat(x) of the draft token, the acceptance decision u < min(1, ratio) and Lemma 1's
// sum min(p, q_hat).
// Kernel B, one workgroup of 1024 threads per sequence: finds the first rejected position j (or the bonus
// row) from kernel A's decisions, sweeps that one target row in fp64 with all its waves, and then, on its
// first four waves, draws from norm(max(0, p - q_hat)) (or from p for the bonus row) by inverse CDF and
// writes the sequence's outputs.  One workgroup per row keeps the sweep's sums in LDS; splitting a row
// over workgroups would need a device-scope fence per workgroup, which writes back and invalidates the
// L2 of an XCD and costs far more than it saves.
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
  int32_t* flags;        // [B, gamma] 1 accepted, 0 rejected, 2 row unusable, 3 not examined (staged mode)
  int32_t* row_status;   // [B, gamma]
  int use_table;         // kernel B sums bf16 rows through the exp table
  int stage0;            // staged mode: positions in the first stage (0 = all positions in one launch)
  int j_begin, j_count;  // the positions one launch of kernel A covers
};
constexpr int kFlagSkipped = 3;

inline size_t verify_workspace_bytes(int64_t B, int64_t gamma, int64_t V, int k_cap) {
  (void)V; (void)k_cap;
  return align256(size_t(B) * gamma * 4) * 2;
}
inline void verify_carve_workspace(VerifyParams& p, void* ws) {
  char* w = reinterpret_cast<char*>(ws);
  p.flags = reinterpret_cast<int32_t*>(w); w += align256(size_t(p.B) * p.gamma * 4);
  p.row_status = reinterpret_cast<int32_t*>(w);
}

// row_status bit for kernel B only: a sample of the row lies largely outside the exp table's range
constexpr int kRowTablePoor = 1 << 20;

template <typename T> __device__ __forceinline__ const void* target_row(const VerifyParams& p, int64_t b, int j) {
  return reinterpret_cast<const char*>(p.target) +
         (size_t(b) * (p.gamma + 1) + j) * size_t(p.row_stride) * ElemTraits<T>::kBytes;
}

// ---------------------------------------------------------------------------------------------
// Kernel A
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kBlock, kAccWavesPerSimd) void verify_accept_kernel(const VerifyParams p) {
  __shared__ VerifyShared sh;
  const int tid = threadIdx.x;
  const int64_t b = blockIdx.x / p.j_count;
  const int j = p.j_begin + int(blockIdx.x - b * p.j_count);
  const int64_t r = b * p.gamma + j;       // row index in [0, B*gamma)
  if (p.j_begin > 0) {
    // a later stage: nothing to do for a sequence that an earlier stage has rejected
    int dead = 0;
    for (int i = tid; i < p.j_begin; i += kBlock) dead |= p.flags[b * p.gamma + i] != 1 ? 1 : 0;
    if (__syncthreads_or(dead)) {
      if (tid == 0) {
        p.flags[r] = kFlagSkipped;
        p.row_status[r] = 0;
        if (p.out_ratio) p.out_ratio[r] = NAN;
        if (p.out_beta) p.out_beta[r] = NAN;
      }
      return;
    }
  }
  const void* row = target_row<T>(p, b, j);
  const RowSplit rs = split_row<T>(row, p.V);
  int count = p.q_count[r];
  count = count < 0 ? 0 : (count > p.k_cap ? p.k_cap : count);
  double p_s[kSetPer], q_s[kSetPer], p_out;
  int yi[kSetPer], st;
  bool ok;
  // A format whose exp table covers a part of its range only: the first batch of the row (kAccVecs * kBlock
  // vectors) says whether kernel B should use the table on this row.  A wave pays for one value outside
  // the table as if its whole vector were outside, so the table loses to the direct path once about 1
  // value in 500 is outside.
  int miss = 0;
  eval_row_on_set<T>(row, rs, p.V, p.rT, p.k2, p.q_idx + size_t(r) * p.k_cap, p.q_logit + size_t(r) * p.k_cap, count, sh,
                     p_s, q_s, yi, p_out, ok, st, &miss);
  if constexpr (ExpTab<T>::kSampled) miss = wave_sum_i32(miss);
  const int x = p.draft_tokens[r];
  double beta = 0.0;
  if (tid == 0) { sh.bcast_d[0] = -1.0; sh.bcast_i[0] = 0; sh.bcast_i[1] = 0; }
  __syncthreads();
  if (ExpTab<T>::kSampled && miss && lane_id() == 0) atomicAdd(&sh.bcast_i[1], miss);
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
    if (ExpTab<T>::kSampled && sh.bcast_i[1] * 500 >= kAccVecs * 8 * kBlock) st |= kRowTablePoor;
    p.row_status[r] = st;
    if (p.out_ratio) p.out_ratio[r] = ok ? float(ratio) : NAN;
    if (p.out_beta) p.out_beta[r] = ok ? float(beta) : NAN;
  }
}

// ---------------------------------------------------------------------------------------------
// Kernel B: one workgroup of 1024 threads per sequence.  All 16 waves sweep the row to be sampled (wave
// w takes run w and then whichever run is next; the run sums stay in LDS), every thread takes one entry of
// the sequence's sparse set on the way, then waves 4..15 end and the first four do the inverse CDF
// (finish_core) and write the sequence's outputs.
// ---------------------------------------------------------------------------------------------
constexpr int kResThreads = 1024;
constexpr int kResWaves = kResThreads / 64;
constexpr int kMaxSegs = kBlock - 2;          // finish_core handles at most kBlock pieces (segments + 2 edges)

template <typename T>
__global__ __launch_bounds__(kResThreads) void verify_resample_kernel(const VerifyParams p) {
  constexpr int E = ElemTraits<T>::kPerVec;
  __shared__ VerifyShared sh;
  __shared__ double subs_l[kMaxSegs * kSubChunks];     // mass of every run, in its segment's units
  __shared__ SegResult segs_l[kMaxSegs + 2];
  __shared__ float run_max[kResWaves];
  __shared__ int flags_l, next_run;
  // the set's entries, one per thread of the workgroup (k_cap <= kResThreads), kept for the four waves that
  // finish; once those have taken their entries the space serves the finish as scratch
  __shared__ union SetSpace {
    struct { int yi[kResThreads]; float ql[kResThreads], tv[kResThreads]; };
    double item_val[kMaxItems];
  } set;
  static_assert(kResThreads >= kSetPer * kBlock, "one set entry per thread");
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int64_t b = blockIdx.x;

  // The decisions of the sequence's first 64 positions are requested first; a table that does not depend on
  // them is built while they travel.  Every wave then finds the first rejected position by itself (gamma
  // when every draft token was accepted): the words are few and nothing has to be handed round.
  const int32_t* fl_b = p.flags + b * p.gamma;
  int f0 = lane < p.gamma ? fl_b[lane] : 1;
  if (tid == 0) { flags_l = 0; next_run = kResWaves; }
  double* table = nullptr;
  if constexpr (ExpTab<T>::kHas && !ExpTab<T>::kSampled) {
    if (p.use_table) {
      table = reinterpret_cast<double*>(dyn_lds);
      build_exp_table<T>(table, p.rT, kResThreads, 0);      // the second half: behind the first requests of the sweep
    }
  }
  int j0 = f0 != 1 ? lane : p.gamma;
  if (p.gamma > 64 && ballot(f0 != 1) == 0) {
    for (int j = lane + 64; j < p.gamma; j += 64)
      if (fl_b[j] != 1) { j0 = j; break; }
  }
  const int jstar = -wave_max_i32(-j0);        // the smallest over the wave
  const bool residual = jstar < p.gamma;
  if constexpr (ExpTab<T>::kSampled) {
    // kernel A has looked at a sample of the row (the bonus row it has not seen: the table is tried)
    if (p.use_table && !(residual && (p.row_status[b * p.gamma + jstar] & kRowTablePoor))) {
      table = reinterpret_cast<double*>(dyn_lds);
      build_exp_table<T>(table, p.rT, kResThreads, 0);
    }
  }
  // the decision at that position, from the lane that holds it (a position beyond the first 64 is read again)
  const bool unusable = residual && (jstar < 64 ? __shfl(f0, jstar, 64) : fl_b[jstar]) == 2;
  const void* row = target_row<T>(p, b, jstar);
  const RowSplit rs = split_row<T>(row, p.V);
  const int n_seg_row = int((rs.nvec + kSegVecsTotal - 1) / kSegVecsTotal);
  const int n_runs = int((rs.nvec + kRunVecs - 1) / kRunVecs);
  const bool check = !residual;     // kernel A has validated the rows it decided on; the bonus row is new
  // What the finish needs is requested now and travels during the sweep: status words, the uniform, and the
  // set's entries, one per thread, each with the target logit at its index (a dependent request, issued
  // further down once the index is there).  Every request is unconditional (a slot beyond the set reads
  // the set's last slot, an index outside the vocabulary reads the row's first element).
  const int64_t r = b * p.gamma + (residual ? jstar : 0);
  const int st_first = p.row_status[b * p.gamma + (tid < p.gamma ? tid : p.gamma - 1)];   // positions beyond 1023: below
  const float u_res = p.u_resample[b * (p.gamma + 1) + jstar];
  int count = residual ? p.q_count[r] : 0;
  const int slot = tid < p.k_cap ? tid : p.k_cap - 1;
  const int my_y = p.q_idx[size_t(r) * p.k_cap + slot];
  const float my_ql = p.q_logit[size_t(r) * p.k_cap + slot];
  const float ql0 = p.q_logit[size_t(r) * p.k_cap];

  count = count < 0 ? 0 : (count > p.k_cap ? p.k_cap : count);
  const bool my_valid = tid < count && my_y >= 0 && my_y < p.V;
  float my_tv = -INFINITY;
  bool tv_requested = false;
  auto request_target_at_index = [&]() {
    my_tv = load_elem<T>(row, my_valid ? my_y : 0);
    tv_requested = true;
  };
  bool wrote_set = false;
  auto write_set = [&]() {          // this thread's set entry, for the waves that finish
    if (!tv_requested) request_target_at_index();
    set.yi[tid] = my_valid ? my_y : -1;
    set.ql[tid] = tid < count ? my_ql : 0.0f;
    set.tv[tid] = my_valid ? my_tv : -INFINITY;
    wrote_set = true;
  };
  bool direct = !unusable;          // the row is swept with fp64 exponentials (no table, or values beyond its domain)
  int tab_bad = 0;
  if constexpr (ExpTab<T>::kHas) {
    if (table != nullptr) {
      // ---- the sweep through the table.  A wave takes run `wave` first and then whichever run is next
      // (a counter in LDS), so that the waves end together.  Every request of the loop is unconditional (a
      // vector past the row's end is read from the row's last vector and its sum dropped; a run past the last
      // is the last one again, to no effect): with requests inside branches the number in flight is not
      // known where a wait is placed, and the wait for the current run would wait for the run requested
      // ahead as well.
      int flags = 0;
      if (!unusable && n_runs > 0) {
        const uint32_t last_vec = uint32_t(rs.nvec - 1), nvec = uint32_t(rs.nvec);
        auto request = [&](int run, uint4 (&q)[kSegVecs]) {
          const uint32_t vbase = uint32_t(run < n_runs ? run : n_runs - 1) * kRunVecs + lane;
#pragma unroll
          for (int i = 0; i < kSegVecs; ++i) {
            const uint32_t vi = vbase + i * 64;
            q[i] = load_vec(&rs.body[vi < last_vec ? vi : last_vec]);
          }
        };
        // the four vectors' lookups are independent: all are requested before any is added up, and one look
        // at the total says whether an element was outside the table
        auto consume = [&](int run, const uint4 (&q)[kSegVecs]) {
          const uint32_t vbase = uint32_t(run) * kRunVecs + lane;
          double sv[kSegVecs];
#pragma unroll
          for (int i = 0; i < kSegVecs; ++i) sv[i] = table_vec_sum_raw<T>(q[i], table);
#pragma unroll
          for (int i = 0; i < kSegVecs; ++i) sv[i] = vbase + i * 64 < nvec ? sv[i] : 0.0;
          double acc = (sv[0] + sv[1]) + (sv[2] + sv[3]);
          if (acc != acc) {
            acc = 0.0;
#pragma unroll
            for (int i = 0; i < kSegVecs; ++i)
              if (vbase + i * 64 < nvec) acc += sv[i] == sv[i] ? sv[i] : table_vec_redo<T>(q[i], p.rT, flags);
          }
          const double run_sum = wave_sum_f64(acc);
          if (lane == 0 && run < n_runs) subs_l[run] = run_sum;
        };
        auto next = [&]() {
          int nr = 0;
          if (lane == 0) nr = atomicAdd(&next_run, 1);
          return __builtin_amdgcn_readfirstlane(nr);
        };
        uint4 d[kSegVecs], dn[kSegVecs];
        int cur = wave;
        request(cur, d);
        build_exp_table<T>(table, p.rT, kResThreads, 1);    // the table's second half, while the requests travel
        __syncthreads();                    // the table is complete
        // the first run apart: behind it the set entry's target logit is requested, whose index has arrived
        // by then
        int nxt = next();
        request(nxt, dn);
        consume(cur, d);
        request_target_at_index();
#pragma unroll
        for (int i = 0; i < kSegVecs; ++i) d[i] = dn[i];
        cur = nxt;
        while (cur < n_runs) {
          nxt = next();
          request(nxt, dn);
          consume(cur, d);
#pragma unroll
          for (int i = 0; i < kSegVecs; ++i) d[i] = dn[i];
          cur = nxt;
        }
        flags = wave_or_i32(flags);
        if (lane == 0 && flags) atomicOr(&flags_l, flags);
      }
      write_set();
      __syncthreads();                      // run sums, flags and set entries are out
      const int fl = flags_l;
      direct = !unusable && (fl & 2) != 0;
      tab_bad = (fl & 1) && check ? 1 : 0;
    }
  }
  if (direct) {
    if (table == nullptr) __syncthreads();      // flags_l is set up (a table sweep has had its barriers)
    // a run's four vectors per lane; a vector past the row's end reads as -inf
    auto load_run = [&](int run, uint4 (&q)[kSegVecs]) {
      const int64_t vbase = int64_t(run) * kRunVecs + lane;
#pragma unroll
      for (int i = 0; i < kSegVecs; ++i) {
        q[i] = neg_inf_vec<T>();
        if (vbase + i * 64 < rs.nvec) q[i] = load_vec(&rs.body[vbase + i * 64]);
      }
    };
    // every term an fp64 exponential referenced to its segment's maximum; the four waves w, w+1, w+2,
    // w+3 (w a multiple of 4) hold the four runs of one segment
    for (int run0 = 0; run0 < n_seg_row * kSubChunks; run0 += kResWaves) {
      const int run = run0 + wave;
      const int seg = run / kSubChunks;
      uint4 d[kSegVecs];
      load_run(run, d);                       // vectors past the row's end read as -inf
      float vmax = -INFINITY;
      int bad = 0;
#pragma unroll
      for (int i = 0; i < kSegVecs; ++i) {
        float v[E];
        unpack<T>(d[i], v);
#pragma unroll
        for (int e = 0; e < E; ++e) {
          if (check) bad |= (v[e] != v[e] || v[e] == INFINITY) ? 1 : 0;
          vmax = fmaxf(vmax, v[e]);
        }
      }
      vmax = wave_max_f32(vmax);
      bad = wave_or_i32(bad);
      if (lane == 0) { run_max[wave] = vmax; if (bad) atomicOr(&flags_l, 4); }
      __syncthreads();
      const int w0 = wave & ~(kSubChunks - 1);
      float smax_v = run_max[w0];
#pragma unroll
      for (int k = 1; k < kSubChunks; ++k) smax_v = fmaxf(smax_v, run_max[w0 + k]);
      const float smax = __fmul_rn(smax_v, p.rT);      // scaling is monotone
      double acc = 0.0;
      if (smax > -INFINITY && smax < INFINITY) {
        const double m = double(smax);
#pragma unroll
        for (int i = 0; i < kSegVecs; ++i) {
          float v[E];
          unpack<T>(d[i], v);
#pragma unroll
          for (int e = 0; e < E; ++e) acc += exp64(double(__fmul_rn(v[e], p.rT)) - m);    // -inf gives exactly 0
        }
      }
      const double run_sum = wave_sum_f64(acc);
      if (lane == 0 && seg < n_seg_row) {
        subs_l[run] = run_sum;
        if ((wave & (kSubChunks - 1)) == 0) segs_l[1 + seg].smax = smax;
      }
      __syncthreads();                          // run_max is reused by the next round
    }
  }
  if (!wrote_set) {
    write_set();
    __syncthreads();
  } else if (direct) {
    __syncthreads();
  }
  if (__builtin_amdgcn_readfirstlane(wave) >= kWaves) return;     // whole waves end here

  // ---- the first four waves: the pieces' masses, inverse CDF and outputs --------------------------
  if (!unusable) {
    if (tid < n_seg_row) {
      SegResult& o = segs_l[1 + tid];
      double t = 0.0;
      if (direct) {
        const int bad_row = (flags_l & 4) ? 1 : 0;
        for (int r = tid * kSubChunks; r < (tid + 1) * kSubChunks; ++r) t += subs_l[r];
        o.sum = bad_row ? 0.0 : t;
        o.bad = bad_row;
      } else {
        // through the table the terms are referenced to 0: a segment reports that, or that it has no mass
        for (int r = tid * kSubChunks; r < (tid + 1) * kSubChunks && r < n_runs; ++r) t += subs_l[r];
        for (int r = n_runs; r < (tid + 1) * kSubChunks; ++r) if (r >= tid * kSubChunks) subs_l[r] = 0.0;
        o.sum = tab_bad ? 0.0 : t;
        o.smax = (t > 0.0 && !tab_bad) ? 0.0f : -INFINITY;
        o.bad = tab_bad;
      }
    }
    if (tid == 0) {
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
        SegResult& o = segs_l[piece == 0 ? 0 : n_seg_row + 1];
        o.sum = sum; o.smax = smax; o.bad = bad;
      }
    }
  }
  // status bits of the positions up to the one that decided; this thread holds those of positions tid + 256 k
  int st = 0;
  for (int j = tid; j <= jstar && j < p.gamma; j += kBlock)
    st |= (j == tid ? st_first : p.row_status[b * p.gamma + j]) & ~kRowTablePoor;
  SetEntries se;
  se.ql0 = count > 0 ? ql0 : 0.0f;
#pragma unroll
  for (int k = 0; k < kSetPer; ++k) {
    se.yi[k] = set.yi[tid + k * kBlock]; se.ql[k] = set.ql[tid + k * kBlock]; se.tv[k] = set.tv[tid + k * kBlock];
  }
  st = block_or_i32<kWaves>(st, sh.red);        // its barriers also end the reading of the entries
  FinishArgs a;
  a.item_val = set.item_val;
  a.row = row;
  a.rs = rs;
  a.n_seg_row = n_seg_row;
  a.V = p.V;
  a.rT = p.rT;
  a.segs = segs_l;
  a.subs = subs_l;
  a.count = count;
  a.qi = p.q_idx + size_t(r) * p.k_cap;
  a.ql = p.q_logit + size_t(r) * p.k_cap;
  a.stages = residual ? 1 : 0;
  a.cands = nullptr;
  a.n_cands = 0;
  a.u = u_res;
  a.unusable = unusable;
  a.table = direct ? nullptr : table;
  const int token = finish_core<T>(a, sh, st, &se);

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
    // stages of stage0, stage0, 2 * stage0, 4 * stage0, ... positions; one stage if stage0 is 0
    int len = p.stage0 > 0 ? p.stage0 : p.gamma;
    for (int j0 = 0, k = 0; j0 < p.gamma; ++k) {
      p.j_begin = j0;
      p.j_count = p.gamma - j0 < len ? p.gamma - j0 : len;
      hipLaunchKernelGGL(verify_accept_kernel<T>, dim3(unsigned(p.B * p.j_count)), dim3(kBlock), 0, s, p);
      if ((e = hipGetLastError()) != hipSuccess) return e;
      j0 += p.j_count;
      if (k > 0) len *= 2;
    }
  }
  if (phases & 2) {
    p.use_table = exp_table_usable<T>(p.rT) ? 1 : 0;
    const size_t lds = p.use_table ? ExpTab<T>::kBytes : 0;
    if (lds > 48 * 1024 && (e = allow_dynamic_lds<&verify_resample_kernel<T>>(int(lds))) != hipSuccess) return e;
    hipLaunchKernelGGL(verify_resample_kernel<T>, dim3(unsigned(p.B)), dim3(kResThreads), lds, s, p);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace tslt
