// Row-level building blocks shared by chain and tree verification (Algorithms 3, 5 and 8):
//   eval_row_on_set  one streaming pass over a target row for its softmax normaliser, then p and
//                    q_hat at the indices of a received sparse set, in fp64;
//   sweep_segment    fp64 sums of exp(s - s_max) over one segment of a row that has to be sampled;
//   finish_core      combines a row's segment sums, applies the sparse corrections of the residual
//                    distribution and finds, by inverse CDF, the token at which the cumulative mass
//                    passes u * total.
// fp64 is needed for the sampling: at V >= 128k the buckets of the inverse CDF are far narrower than
// fp32 prefix sums can resolve.
#pragma once
#include <algorithm>
#include <type_traits>
#include "common.h"
#include "exp64.h"

namespace tslt {

constexpr int kSegVecs = 4;                         // 16-byte vectors per thread in a sweep segment
constexpr int kSegVecsTotal = kSegVecs * kBlock;    // vectors per segment
constexpr int kRunVecs = kSegVecs * 64;             // a run: the consecutive vectors one wave holds
constexpr int kSubChunks = kWaves;                  // runs per segment
// eval_row_on_set keeps kAccDepth batches of kAccVecs 16-byte vectors in flight per thread.  Its kernels ask for
// eight waves per SIMD (64 registers): 2048 rows of the headline shape are then resident at once, eight
// workgroups per compute unit, instead of 1280 followed by a thinly occupied second round.
constexpr int kAccDepth = 4;
constexpr int kAccVecs = 2;
constexpr int kAccWavesPerSimd = 8;
constexpr int kSetPer = 1024 / kBlock;              // set entries per thread (TSLT_MAX_K_CAP / kBlock)

constexpr int kRowBadSet = 8;      // TSLT_ROW_BAD_SET

struct SegResult {       // one segment (or edge piece) of a row that is being sampled
  double sum;            // sum of exp(s - smax) over the piece (edge pieces; a segment's mass is in its runs' sums)
  float smax;            // largest scaled logit of the piece (-inf if empty)
  int bad;               // NaN or +inf seen
};

// Segments of a row of V elements, `per_vec` of them in a 16-byte vector (4 for fp32, the default, which
// bounds every type and sizes the workspaces; 8 for the 16-bit types).
inline int row_segments(int64_t V, int per_vec = 4) {
  // one more segment covers a ragged end
  const int64_t nvec_max = V / per_vec + 1;
  return int((nvec_max + kSegVecsTotal - 1) / kSegVecsTotal);
}
inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

struct VerifyShared {
  BlockScratch red;
  double bcast_d[4];
  int bcast_i[4];
};
constexpr int kMaxPieces = kBlock;                                 // segments of a row that is sampled, plus its two edges
constexpr int kMaxItems = (kMaxPieces - 2) * kSubChunks + 2;       // its runs, plus the two edges

// A table of exp(s), s = fl32(z / T), for every 16-bit logit z of a magnitude range that holds the bulk of
// a row: the fp64 sums over the row then cost one LDS read per element instead of an fp64 exponential.
//   bfloat16  2^-14 <= |z| < 2^7   5376 values, 42 KB  (logits centred on 0 have many small values)
//   binary16  2^-2 <= |z| < 2^5  14336 values, 112 KB
// With the 16 bits of an element rotated left by one (sign in bit 0), entry 1 + (rotated - 2*kLo) holds
// its value; entries 0 and kEntries + 1 hold NaN and stand for everything below and above the table's
// domain (tiny, huge, -inf, NaN), which is evaluated directly.  Terms are referenced to 0 rather than to
// the row maximum, which is safe while |s| <= kTabMaxS; a segment that holds a larger |s| is redone by
// the maximum-referenced path.
constexpr float kTabMaxS = 600.0f;
template <typename T> struct ExpTab {
  static constexpr bool kHas = false;
  static constexpr bool kSampled = false;
  static constexpr size_t kBytes = 0;
};
template <> struct ExpTab<Bf16> {
  static constexpr bool kHas = true;
  static constexpr int kLo = (127 - 14) << 7;      // bits of the smallest magnitude covered
  static constexpr int kSpan = 21 << 7;            // magnitudes covered
  static constexpr int kEntries = 2 * kSpan;
  static constexpr size_t kBytes = size_t(kEntries + 2) * sizeof(double);
  static constexpr float kMaxAbs = 128.0f;
  static constexpr uint32_t kInf = 0x7F80u;
  static constexpr bool kSampled = false;          // the range is wide enough for any plausible row
  static __device__ __forceinline__ float widen(uint32_t bits) { return __uint_as_float(bits << 16); }
};
template <> struct ExpTab<F16> {
  static constexpr bool kHas = true;
  static constexpr int kLo = (15 - 2) << 10;
  static constexpr int kSpan = 7 << 10;
  static constexpr int kEntries = 2 * kSpan;
  static constexpr size_t kBytes = size_t(kEntries + 2) * sizeof(double);
  static constexpr float kMaxAbs = 32.0f;
  static constexpr uint32_t kInf = 0x7C00u;
  static constexpr bool kSampled = true;           // a row whose bulk lies near 0 is mostly below the range
  static __device__ __forceinline__ float widen(uint32_t bits) { return f16_lo(bits); }
};
template <typename T> inline bool exp_table_usable(float rT) {
  if constexpr (ExpTab<T>::kHas) return ExpTab<T>::kMaxAbs * rT <= kTabMaxS;
  return false;
}

// Workgroups of a sweep launch: a few per compute unit, each looping over its share of the segments.
inline int64_t sweep_grid_limit() { return int64_t(compute_units()) * 4; }

template <typename T> __device__ __forceinline__ double exp_table_entry(int i, float rT) {
  using TB = ExpTab<T>;
  if (i < 1 || i > TB::kEntries) return __longlong_as_double(0x7FF8000000000000ll);
  const int j = i - 1;
  const uint32_t bits = (uint32_t(j & 1) << 15) | uint32_t(TB::kLo + (j >> 1));
  return exp64(double(__fmul_rn(TB::widen(bits), rT)));
}
// Fills the table with all `threads` threads of the workgroup; the caller synchronises.  `half` 0 / 1 fills the
// first / second half only (a kernel that has requests to make between the two does so: the entries are
// pure arithmetic, a good thing to have while data travels), -1 everything.
template <typename T> __device__ __forceinline__ void build_exp_table(double* table, float rT, int threads, int half = -1) {
  constexpr int n = ExpTab<T>::kEntries + 2;
  const int mid = ((n / 2 + threads - 1) / threads) * threads;
  const int lo = half == 1 ? mid : 0, hi = half == 0 ? mid : n;
  for (int i = lo + threadIdx.x; i < hi; i += threads) table[i] = exp_table_entry<T>(i, rT);
}

// Sum of exp(s) over the 8 elements of a 16-bit vector through the table.  The index arithmetic runs on
// both halves of a 32-bit word at once (16-bit lanes: rotate, saturating subtract, minimum).  An element
// outside the table's domain reads a NaN entry, which shows in the sum: table_vec_sum_raw returns that NaN
// (so that a caller can add several vectors up and look once), table_vec_redo evaluates a vector element by
// element.
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
template <typename T>
__device__ __forceinline__ double table_vec_sum_raw(const uint4& d, const double* table) {
  using TB = ExpTab<T>;
  const uint32_t w[4] = {d.x, d.y, d.z, d.w};
  const ushort2_t base = {uint16_t(2 * TB::kLo - 1), uint16_t(2 * TB::kLo - 1)};
  const ushort2_t top = {uint16_t(TB::kEntries + 1), uint16_t(TB::kEntries + 1)};
  const ushort2_t one = {1, 1}, fifteen = {15, 15};
  double s0 = 0.0, s1 = 0.0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const ushort2_t x = __builtin_bit_cast(ushort2_t, w[k]);
    const ushort2_t rot = (x << one) | (x >> fifteen);            // sign into bit 0 of each half
    ushort2_t i2 = __builtin_elementwise_sub_sat(rot, base);
    i2 = __builtin_elementwise_min(i2, top);
    if constexpr (TB::kBytes <= 65536) {      // byte offsets fit the 16-bit lanes
      const ushort2_t three = {3, 3};
      const uint32_t off = __builtin_bit_cast(uint32_t, i2 << three);
      const char* tb = reinterpret_cast<const char*>(table);
      const double t0 = *reinterpret_cast<const double*>(tb + (off & 0xFFFFu));
      const double t1 = *reinterpret_cast<const double*>(tb + (off >> 16));
      s0 = k == 0 ? t0 : s0 + t0;
      s1 = k == 0 ? t1 : s1 + t1;
    } else {
      const uint32_t ix = __builtin_bit_cast(uint32_t, i2);
      const double t0 = table[ix & 0xFFFFu], t1 = table[ix >> 16];
      s0 = k == 0 ? t0 : s0 + t0;
      s1 = k == 0 ? t1 : s1 + t1;
    }
  }
  return s0 + s1;
}
// Every element of a vector directly; branch-free, so that a wave in which some lane comes here for every
// vector (a row with many values outside the table) runs at the pace of the direct path and not at that of
// a divergent loop.  flags: 1 = NaN or +inf, 2 = |s| beyond kTabMaxS
template <typename T>
__device__ __forceinline__ double table_vec_redo(const uint4& d, float rT, int& flags) {
  using TB = ExpTab<T>;
  const uint32_t w[4] = {d.x, d.y, d.z, d.w};
  double s = 0.0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t b = (w[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
    const float sv = __fmul_rn(TB::widen(b), rT);
    const bool neg_inf = b == (0x8000u | TB::kInf);
    flags |= ((b & 0x7FFFu) > TB::kInf || b == TB::kInf) ? 1 : 0;
    flags |= (!neg_inf && fabsf(sv) > kTabMaxS) ? 2 : 0;
    s += exp64(double(sv));                                       // -inf gives exactly 0
  }
  return s;
}
// Three sums over the workgroup with one pair of barriers.
template <int NW>
__device__ __forceinline__ void block_sum3_f64(double& a, double& b, double& c, BlockScratch& s) {
  static_assert(NW <= 4, "the partial sums are laid out for at most four waves");
  a = wave_sum_f64(a); b = wave_sum_f64(b); c = wave_sum_f64(c);
  __syncthreads();
  if (lane_id() == 0) { s.d[wave_id()] = a; s.d[4 + wave_id()] = b; s.d[8 + wave_id()] = c; }
  __syncthreads();
  a = 0.0; b = 0.0; c = 0.0;
#pragma unroll
  for (int w = 0; w < NW; ++w) { a += s.d[w]; b += s.d[4 + w]; c += s.d[8 + w]; }
}

// ---------------------------------------------------------------------------------------------
// One pass over a target row: partial sums of exp2(t*k2 - c), c referenced to the largest target
// logit found at the set's indices; then, in fp64 over the <= 1024 received entries, p at those
// indices (the set's fp32 terms are replaced by fp64 ones in the normaliser) and q_hat = softmax of
// the received values.  Entry i of the set is held by thread i % 256, slot i / 256.
//   p_s, q_s  target and draft probability of the entry (0 where the entry is unused)
//   yi        token index of the entry, -1 if unused or out of range
//   p_out     target mass outside the set
//   ok / st   false with TSLT_ROW_* bits when the row is unusable (NaN, +inf, nothing above -inf) or the set is
//             (a value that is not finite, an index outside the vocabulary)
// ---------------------------------------------------------------------------------------------
// log2 of a softmax term relative to the reference c: one fma with k2 = fl32(log2(e) / T).  (The
// definition rounds s = t / T to fp32 first; not doing so here moves a term by at most 2^-24 of its
// exponent, a few 1e-8 of the normaliser after the set's own terms have been replaced by fp64 ones.)
__device__ __forceinline__ float scaled_arg(float v, float k2, float neg_c) { return __builtin_fmaf(v, k2, neg_c); }

template <typename T>
__device__ __forceinline__ void eval_row_on_set(const void* row, const RowSplit& rs, int64_t V, float rT, float k2,
                                                const int32_t* qi, const float* ql, int count, VerifyShared& sh,
                                                double (&p_s)[kSetPer], double (&q_s)[kSetPer], int (&yi)[kSetPer],
                                                double& p_out, bool& ok, int& st, int* table_miss = nullptr) {
  constexpr int E = ElemTraits<T>::kPerVec;
  const int tid = threadIdx.x;
  const int n_edge = rs.head + rs.tail;
  const int64_t n_tiles = (rs.nvec + kBlock - 1) / kBlock;
  // The pass keeps kAccDepth batches of U vectors in flight per thread; the first ones are requested
  // before anything else, so that they travel while the reference is looked up.
  constexpr int U = kAccVecs;
  const uint32_t n_full = uint32_t(rs.nvec / (U * kBlock));      // batches of U complete tiles
  uint4 pipe[kAccDepth][U];
  // Every request of the pipeline is unconditional: one past the row's end comes back as zeros and is never
  // used.  With conditional requests the number of loads in flight is not known where a wait is placed, and
  // each wait for one batch waits for all of them.
  const __amdgpu_buffer_rsrc_t body = row_buffer(rs.body, uint32_t(rs.nvec));
  const uint32_t lane_bytes = uint32_t(tid) * 16u;
  auto issue = [&](uint32_t b, uint4 (&q)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) q[u] = buffer_load_vec_stream(body, lane_bytes, (b * U + u) * (kBlock * 16u));
  };
  if (n_full > 0) {
#pragma unroll
    for (int s = 0; s < kAccDepth; ++s) issue(uint32_t(s), pipe[s]);
  }

  float tv[kSetPer];       // raw target logit at entry
  float gmax = -INFINITY;
#pragma unroll
  for (int k = 0; k < kSetPer; ++k) {
    const int i = tid + k * kBlock;
    tv[k] = -INFINITY; yi[k] = -1;
    if (i < count) {
      const int y = qi[i];
      if (y >= 0 && y < V) { yi[k] = y; tv[k] = load_elem<T>(row, y); }
      gmax = fmaxf(gmax, tv[k]);
    }
  }
  float vref = block_max_f32<kWaves>(gmax, sh.red);
  if (!(vref > -INFINITY && vref < INFINITY)) {
    // no usable reference in the set: take the start of the row
    float m0 = -INFINITY;
    for (int64_t i = tid; i < V && i < 4096; i += kBlock) m0 = fmaxf(m0, load_elem<T>(row, i));
    vref = block_max_f32<kWaves>(m0, sh.red);
  }
  st = 0;
  double z_c = 0.0;
  float c_ref = __fmul_rn(vref, k2);
  ok = vref > -INFINITY && vref < INFINITY;
  if (ok) {
    const float neg_c = -c_ref;
    // fp32 sums only within a batch of U vectors: a long-lived fp32 accumulator that has met one large
    // term rounds away the many small ones that follow, always downwards
    double dacc = 0.0;
    auto consume = [&](const uint4 (&q)[U]) {
      float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float v[E];
        unpack<T>(q[u], v);
#pragma unroll
        for (int e = 0; e < E; e += 4) {
          acc0 += fast_exp2(scaled_arg(v[e + 0], k2, neg_c));
          acc1 += fast_exp2(scaled_arg(v[e + 1], k2, neg_c));
          acc2 += fast_exp2(scaled_arg(v[e + 2], k2, neg_c));
          acc3 += fast_exp2(scaled_arg(v[e + 3], k2, neg_c));
        }
      }
      dacc += double((acc0 + acc1) + (acc2 + acc3));
    };
    if constexpr (ExpTab<T>::kSampled) {
      // how many values of the first batch lie outside the exp table's range (a hint for the sweep that
      // may follow; this thread's share, the caller adds them up)
      if (table_miss != nullptr && n_full > 0) {
        int miss = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const uint32_t w[4] = {pipe[0][u].x, pipe[0][u].y, pipe[0][u].z, pipe[0][u].w};
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint32_t m = ((w[e >> 1] >> ((e & 1) * 16)) & 0x7FFFu) - uint32_t(ExpTab<T>::kLo);
            miss += m >= uint32_t(ExpTab<T>::kSpan) ? 1 : 0;
          }
        }
        *table_miss = miss;
      }
    }
    for (uint32_t b = 0; b < n_full; b += kAccDepth) {
#pragma unroll
      for (int s = 0; s < kAccDepth; ++s) {
        if (b + s < n_full) consume(pipe[s]);
        issue(b + s + kAccDepth, pipe[s]);
      }
    }
    for (int64_t t0 = int64_t(n_full) * U; t0 < n_tiles; t0 += U) {      // the ragged end
      uint4 d[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t vi = (t0 + u) * kBlock + tid;
        d[u] = neg_inf_vec<T>();
        if (vi < rs.nvec) d[u] = load_vec_stream(&rs.body[vi]);
      }
      consume(d);
    }
    if (tid < n_edge) dacc += double(fast_exp2(scaled_arg(load_elem<T>(row, edge_index<T>(rs, tid)), k2, neg_c)));
    z_c = block_sum_f64<kWaves>(dacc, sh.red);
    ok = z_c > 0.0 && z_c < INFINITY;
  }
  if (!ok) {
    // exact redo: validity and true maximum first, then the sum referenced to it
    int bad = 0, fin = 0;
    float vmax = -INFINITY;
    for (int64_t i = tid; i < V; i += kBlock) {
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
      c_ref = __fmul_rn(vref, k2);
      double acc = 0.0;
      for (int64_t i = tid; i < V; i += kBlock) acc += double(fast_exp2(scaled_arg(load_elem<T>(row, i), k2, -c_ref)));
      z_c = block_sum_f64<kWaves>(acc, sh.red);
      ok = true;
    }
  }

  // ---- fp64 over the set ----------------------------------------------------------------------
  const float s_ref = __fmul_rn(vref, rT);
  const double ql0 = count > 0 ? double(ql[0]) : 0.0;
  double sum_e = 0.0, sum_t32 = 0.0, sum_w = 0.0;
#pragma unroll
  for (int k = 0; k < kSetPer; ++k) {
    const int i = tid + k * kBlock;
    p_s[k] = 0.0; q_s[k] = 0.0;
    if (i < count) {
      // a received value that is not finite, or a token index outside the vocabulary, makes the set unusable:
      // its weight is NaN, which shows in the sum below
      const float qv = ql[i];
      q_s[k] = (fabsf(qv) < INFINITY && yi[k] >= 0) ? exp64(double(qv) - ql0) : __longlong_as_double(0x7FF8000000000000ll);
      sum_w += q_s[k];
      if (yi[k] >= 0 && tv[k] > -INFINITY && ok) {
        p_s[k] = exp64(double(__fmul_rn(tv[k], rT)) - double(s_ref));
        sum_e += p_s[k];
        sum_t32 += double(fast_exp2(scaled_arg(tv[k], k2, -c_ref)));
      }
    }
  }
  block_sum3_f64<kWaves>(sum_e, sum_t32, sum_w, sh.red);
  if (sum_w != sum_w) { st |= kRowBadSet; ok = false; }
  double tail = z_c - sum_t32;
  if (tail < 0.0) tail = 0.0;
  tail *= exp64((double(c_ref) - double(vref) * double(k2)) * 0.69314718055994530942);   // to the reference of the fp64 terms
  const double Z = tail + sum_e;
  // (one reciprocal each instead of a division per entry: an fp64 division is some thirty instructions)
  const double inv_Z = ok ? 1.0 / Z : 0.0, inv_w = sum_w > 0.0 ? 1.0 / sum_w : 0.0;
  p_out = tail * inv_Z;
#pragma unroll
  for (int k = 0; k < kSetPer; ++k) {
    p_s[k] = ok ? p_s[k] * inv_Z : 0.0;
    q_s[k] = sum_w > 0.0 ? q_s[k] * inv_w : 0.0;
  }
}

// ---------------------------------------------------------------------------------------------
// fp64 sweep of a row that has to be sampled, in segments of kSegVecsTotal vectors.  Wave w holds run w
// of a segment: kRunVecs consecutive vectors, vector i*64 + lane in slot i.  A piece (segment or edge)
// reports (sum, smax), meaning a mass of sum * exp(smax), and every run its mass in the same units.
// `check` asks for NaN / +inf detection (rows that no earlier kernel has validated).
// ---------------------------------------------------------------------------------------------
constexpr int kGroupSegs = 4;     // consecutive segments a workgroup takes at a time

// Segments seg0 .. seg0 + n_here - 1 of a row with every term an fp64 exponential referenced to its segment's
// own maximum.  One barrier per segment (the four waves exchange their runs' maxima through LDS, two buffers in
// turn), the next segment's vectors requested before the current one is worked on; every request is
// unconditional (a vector past the row's end is read from the row's last vector and counts as -inf).
template <typename T>
__device__ __forceinline__ void sweep_segments_direct(const RowSplit& rs, int seg0, int n_here, bool check, float rT,
                                                      SegResult* segs, double* subs, VerifyShared& sh) {
  constexpr int E = ElemTraits<T>::kPerVec;
  const int lane = lane_id(), wave = wave_id();
  const uint32_t nvec = uint32_t(rs.nvec), last_vec = nvec - 1;       // nvec > 0: the row has segments
  auto request = [&](int seg, uint4 (&q)[kSegVecs]) {
    const uint32_t vbase = uint32_t(seg) * kSegVecsTotal + wave * kRunVecs + lane;
#pragma unroll
    for (int i = 0; i < kSegVecs; ++i) {
      const uint32_t vi = vbase + i * 64;
      q[i] = load_vec(&rs.body[vi < last_vec ? vi : last_vec]);
    }
  };
  uint4 d[kSegVecs], dn[kSegVecs];
  request(seg0, d);
  for (int k = 0; k < n_here; ++k) {
    const int seg = seg0 + k;
    request(k + 1 < n_here ? seg + 1 : seg, dn);
    const uint32_t vbase = uint32_t(seg) * kSegVecsTotal + wave * kRunVecs + lane;
    float vmax = -INFINITY;
    int bad = 0;
#pragma unroll
    for (int i = 0; i < kSegVecs; ++i) {
      if (vbase + i * 64 >= nvec) d[i] = neg_inf_vec<T>();
      float v[E];
      unpack<T>(d[i], v);
      if (check) {
#pragma unroll
        for (int e = 0; e < E; ++e) bad |= (v[e] != v[e] || v[e] == INFINITY) ? 1 : 0;
      }
#pragma unroll
      for (int e = 0; e < E; e += 2) vmax = max3f(vmax, v[e], v[e + 1]);
    }
    vmax = wave_max_f32(vmax);
    bad = wave_or_i32(bad);
    const int buf = (k & 1) * 8;
    if (lane == 0) { sh.red.f[buf + wave] = vmax; sh.red.i[buf + wave] = bad; }
    __syncthreads();
    float seg_max = sh.red.f[buf];
    int seg_bad = sh.red.i[buf];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) { seg_max = fmaxf(seg_max, sh.red.f[buf + w]); seg_bad |= sh.red.i[buf + w]; }
    const float smax = __fmul_rn(seg_max, rT);      // scaling is monotone: the largest s is at the largest t
    double run = 0.0;
    if (smax > -INFINITY && !seg_bad) {
      const double m = double(smax);
#pragma unroll
      for (int i = 0; i < kSegVecs; ++i) {
        float v[E];
        unpack<T>(d[i], v);
        double s0 = 0.0, s1 = 0.0;
#pragma unroll
        for (int e = 0; e < E; e += 2) {            // -inf gives exactly 0
          s0 += exp64(double(__fmul_rn(v[e], rT)) - m);
          s1 += exp64(double(__fmul_rn(v[e + 1], rT)) - m);
        }
        run += s0 + s1;
      }
    }
    const double run_sum = wave_sum_f64(run);
    if (lane == 0) {
      subs[size_t(seg) * kSubChunks + wave] = run_sum;
      if (wave == 0) { segs[1 + seg].sum = 0.0; segs[1 + seg].smax = smax; segs[1 + seg].bad = seg_bad; }
    }
#pragma unroll
    for (int i = 0; i < kSegVecs; ++i) d[i] = dn[i];
  }
  __syncthreads();      // the exchange buffers are free again
}

// Segments group*kGroupSegs .. +kGroupSegs-1 of a row (all 256 threads of a workgroup); group 0 also does
// the two edge pieces.  `table` is the bf16 exp table in LDS or null.  Through the table the terms are
// referenced to 0: a segment then reports smax = 0 (-inf if it has no mass).
template <typename T>
__device__ __forceinline__ void sweep_group(const void* row, const RowSplit& rs, int group, bool check, float rT,
                                            const double* table, SegResult* segs, double* subs, VerifyShared& sh) {
  const int tid = threadIdx.x;
  const int n_seg_row = int((rs.nvec + kSegVecsTotal - 1) / kSegVecsTotal);
  const int seg0 = group * kGroupSegs;
  const int n_here = n_seg_row - seg0 < kGroupSegs ? n_seg_row - seg0 : kGroupSegs;   // may be <= 0
  bool direct = n_here > 0;
  if constexpr (ExpTab<T>::kHas) {
    if (table != nullptr && n_here > 0) {
      // (every request unconditional: a vector past the row's end is read from the row's last vector and its
      // sum dropped; the four vectors' look-ups of a lane go out together and one look at their total says
      // whether a value was outside the table)
      int flags = 0;
      const uint32_t nvec = uint32_t(rs.nvec), last_vec = nvec - 1;
      auto request = [&](int seg, uint4 (&q)[kSegVecs]) {
        const uint32_t vb = uint32_t(seg) * kSegVecsTotal + wave_id() * kRunVecs + lane_id();
#pragma unroll
        for (int i = 0; i < kSegVecs; ++i) {
          const uint32_t vi = vb + i * 64;
          q[i] = load_vec(&rs.body[vi < last_vec ? vi : last_vec]);
        }
      };
      uint4 d[kSegVecs], dn[kSegVecs];
      request(seg0, d);
#pragma unroll
      for (int k = 0; k < kGroupSegs; ++k) {
        if (k < n_here) {
          request(k + 1 < n_here ? seg0 + k + 1 : seg0 + k, dn);
          const uint32_t vbase = uint32_t(seg0 + k) * kSegVecsTotal + wave_id() * kRunVecs + lane_id();
          double sv[kSegVecs];
#pragma unroll
          for (int i = 0; i < kSegVecs; ++i) sv[i] = table_vec_sum_raw<T>(d[i], table);
#pragma unroll
          for (int i = 0; i < kSegVecs; ++i) sv[i] = vbase + i * 64 < nvec ? sv[i] : 0.0;
          double run = (sv[0] + sv[1]) + (sv[2] + sv[3]);
          if (run != run) {
            run = 0.0;
#pragma unroll
            for (int i = 0; i < kSegVecs; ++i)
              if (vbase + i * 64 < nvec) run += sv[i] == sv[i] ? sv[i] : table_vec_redo<T>(d[i], rT, flags);
          }
          const double run_sum = wave_sum_f64(run);
          if (lane_id() == 0) {
            subs[size_t(seg0 + k) * kSubChunks + wave_id()] = run_sum;
            sh.red.d[k * kWaves + wave_id()] = run_sum;
          }
#pragma unroll
          for (int i = 0; i < kSegVecs; ++i) d[i] = dn[i];
        }
      }
      flags = block_or_i32<kWaves>(flags, sh.red);      // its barriers also publish the run sums
      direct = (flags & 2) != 0;
      if (!direct && tid < n_here) {
        const int bad = (flags & 1) && check ? 1 : 0;
        double t = 0.0;
        for (int w = 0; w < kWaves; ++w) t += sh.red.d[tid * kWaves + w];
        SegResult& o = segs[1 + seg0 + tid];
        o.sum = bad ? 0.0 : t; o.smax = (t > 0.0 && !bad) ? 0.0f : -INFINITY; o.bad = bad;
      }
      __syncthreads();
    }
  }
  if (direct) sweep_segments_direct<T>(rs, seg0, n_here, check, rT, segs, subs, sh);
  if (group == 0 && tid == 0) {
    // the two edge pieces (at most E-1 elements each)
    for (int piece = 0; piece < 2; ++piece) {
      const int e0 = piece == 0 ? 0 : rs.head, e1 = piece == 0 ? rs.head : rs.head + rs.tail;
      float smax = -INFINITY;
      int bad = 0;
      for (int e = e0; e < e1; ++e) {
        const float t = load_elem<T>(row, edge_index<T>(rs, e));
        if (t != t || t == INFINITY) bad = 1;
        smax = fmaxf(smax, __fmul_rn(t, rT));
      }
      double sum = 0.0;
      if (smax > -INFINITY && !bad)
        for (int e = e0; e < e1; ++e) {
          const float t = load_elem<T>(row, edge_index<T>(rs, e));
          if (t > -INFINITY) sum += exp64(double(__fmul_rn(t, rT)) - double(smax));
        }
      SegResult& o = segs[piece == 0 ? 0 : n_seg_row + 1];
      o.sum = sum; o.smax = smax; o.bad = bad;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Inverse CDF of one row from its piece and run sums.
// ---------------------------------------------------------------------------------------------
struct FinishArgs {
  const void* row;
  RowSplit rs;
  int n_seg_row;
  int64_t V;
  float rT;
  const SegResult* segs;    // n_seg_row + 2 pieces of this row
  const double* subs;       // [segment][kSubChunks] run sums of this row
  const int32_t* qi;        // the sparse set whose residual is sampled (ignored when stages == 0)
  const float* ql;
  int count;
  int stages;               // residual updates p <- norm(max(0, p - q_hat)) to apply; 0 samples p itself
  const int32_t* cands;     // candidates drawn without replacement: the tokens that were tested, in order
  int n_cands;              //   (-1 = absent); after update i the i-th of them leaves q_hat, which is
                            //   renormalised.  Null: the same q_hat at every update
  float u;
  int unusable;             // the row is known to be unusable: no token
  double* item_val;         // LDS scratch of the caller, kMaxItems doubles
  const double* table;      // the exp table in LDS if the row's run sums were made through it (then every
                            // piece is referenced to 0), else null
};

// The set's entries as finish_core needs them, one slot per (thread, k): token index (-1 if unused or out
// of range), received scaled logit, raw target logit at that index.  A caller with other work to do first
// (a sweep) can load them early, so that the dependent loads travel meanwhile.
struct SetEntries {
  int yi[kSetPer];
  float ql[kSetPer];
  float tv[kSetPer];
  float ql0;
};
template <typename T>
__device__ __forceinline__ void load_set_entries(const void* row, int64_t V, const int32_t* qi, const float* ql,
                                                 int count, SetEntries& se) {
  const int tid = threadIdx.x;
  se.ql0 = count > 0 ? ql[0] : 0.0f;
#pragma unroll
  for (int k = 0; k < kSetPer; ++k) {
    const int i = tid + k * kBlock;
    se.yi[k] = -1; se.ql[k] = 0.0f; se.tv[k] = -INFINITY;
    if (i < count) {
      se.ql[k] = ql[i];
      const int y = qi[i];
      if (y >= 0 && y < V) { se.yi[k] = y; se.tv[k] = load_elem<T>(row, y); }
    }
  }
}

// Returns the token (-1 if none) and ORs TSLT_ROW_* bits into st.  After m updates with the same q_hat
// the distribution is c * p outside the set and a_i on it, where a and c follow the recursion
// a <- max(0, a - q_hat) / Z, c <- c / Z, Z = sum(max(0, a - q_hat)) + c * p_out; in units of the row's
// unnormalised terms e_y that is e_y outside the set and a_i * z_p / c on it.
//
// The search runs over "items" in row order: the head edge, every run of the body, the tail edge.  Every
// thread lays out its share of the item masses in LDS, the set's corrections are added to the items they
// fall into, and then every wave finds the item at which the cumulative mass passes the target by itself (a
// scan over the wave, the same in all of them), so that nothing has to be handed round; the element inside
// the chosen run is found from one vector per thread.  Called by all kBlock threads of a workgroup.
template <typename T>
__device__ int finish_core(const FinishArgs& a, VerifyShared& sh, int& st, const SetEntries* pre = nullptr) {
  constexpr int E = ElemTraits<T>::kPerVec;
  constexpr int kMaxPer = kSetPer;
  constexpr int kRun = kRunVecs * E;        // elements in a run
  constexpr int kPerT = kRun / kBlock;      // consecutive elements per thread in the chosen run (one vector)
  __shared__ double elem_corr[kRunVecs * 8];   // sparse correction per element of the chosen run
  double* item_val = a.item_val;               // mass of every item
  const int tid = threadIdx.x;
  const int lane = lane_id();
  const RowSplit& rs = a.rs;
  const void* row = a.row;
  const int n_seg_row = a.n_seg_row;
  const int n_pieces = n_seg_row + 2;
  const int n_runs = n_seg_row * kSubChunks;       // runs past the row's end hold no mass
  const int n_items = n_runs + 2;
  const SegResult* segs = a.segs;
  const int broken_flag = a.unusable;
  const float rT = a.rT;
  for (int i = tid; i < kRun; i += kBlock) elem_corr[i] = 0.0;      // published by the first barrier below
  // maximum and validity of the row, from the pieces; every wave looks at all of them
  float smax = -INFINITY;
  int bad = 0;
  if (!broken_flag)
    for (int k = lane; k < n_pieces; k += 64) { smax = fmaxf(smax, segs[k].smax); bad |= segs[k].bad; }
  smax = wave_max_f32(smax);
  bad = wave_or_i32(bad);
  int token = -1;
  const bool usable = !broken_flag && !bad && smax > -INFINITY;
  if (!broken_flag && bad) st |= 1;
  if (!broken_flag && !bad && !(smax > -INFINITY)) st |= 2;

  if (usable) {
    // unnormalised target mass of every item, referenced to the row maximum, and their total z_p
    double zp = 0.0;
    for (int it = tid; it < n_items; it += kBlock) {
      double t;
      if (it == 0 || it == n_items - 1) {
        const SegResult& e = segs[it == 0 ? 0 : n_pieces - 1];
        t = e.smax > -INFINITY ? e.sum * exp64(double(e.smax) - double(smax)) : 0.0;
      } else {
        const float m = segs[1 + (it - 1) / kSubChunks].smax;
        t = m > -INFINITY ? a.subs[it - 1] * exp64(double(m) - double(smax)) : 0.0;
      }
      item_val[it] = t;
      zp += t;
    }

    // the set: after `stages` residual updates the mass of entry i is a_i * z_p / c instead of e_i
    const int stages = a.stages;
    int count = stages > 0 ? a.count : 0;
    SetEntries se_local;
    if (pre == nullptr) load_set_entries<T>(row, a.V, a.qi, a.ql, count, se_local);
    const SetEntries& se = pre ? *pre : se_local;
    const double ql0 = double(se.ql0);
    double w64[kMaxPer], corr[kMaxPer], e_s[kMaxPer];
    int yi[kMaxPer];
    double sum_w = 0.0, sum_e = 0.0;
    const int n_slots = (count + kBlock - 1) / kBlock;      // slots of a thread that can hold an entry
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k) {
      const int i = tid + k * kBlock;
      w64[k] = 0.0; corr[k] = 0.0; e_s[k] = 0.0; yi[k] = -1;
      if (k < n_slots && i < count) {
        w64[k] = exp64(double(se.ql[k]) - ql0);
        sum_w += w64[k];
        if (se.yi[k] >= 0) {
          yi[k] = se.yi[k];
          const float t = se.tv[k];
          e_s[k] = t > -INFINITY ? exp64(double(__fmul_rn(t, rT)) - double(smax)) : 0.0;
          sum_e += e_s[k];
        }
      }
    }
    block_sum3_f64<kWaves>(zp, sum_w, sum_e, sh.red);
    double sum_corr = 0.0;
    if (count > 0) {
      double av[kMaxPer];
      const double inv_zp = 1.0 / zp, inv_w = 1.0 / sum_w;
#pragma unroll
      for (int k = 0; k < kMaxPer; ++k) {
        av[k] = 0.0;
        if (k < n_slots) { av[k] = e_s[k] * inv_zp; w64[k] = w64[k] * inv_w; }
      }
      const double p_out = 1.0 - sum_e * inv_zp;
      double c = 1.0;
      double sum_av = sum_e / zp;               // sum of av over the set, kept up to date through the updates
      const int32_t* cands = a.cands;
      int ci = 0;
      double qscale = 1.0, removed = 0.0;       // the update's proposal is w64 * qscale
      for (int sgi = 0; sgi < stages; ++sgi) {
        double part = 0.0;
#pragma unroll
        for (int k = 0; k < kMaxPer; ++k) {
          if (k < n_slots) {
            const double d = av[k] - w64[k] * qscale;
            av[k] = (yi[k] >= 0 && d > 0.0) ? d : 0.0;
            part += av[k];
          }
        }
        part = block_sum_f64<kWaves>(part, sh.red);
        const double Zs = part + c * (p_out > 0.0 ? p_out : 0.0);
        sum_av = part;
        if (Zs > 0.0) {
          const double inv_Zs = 1.0 / Zs;
#pragma unroll
          for (int k = 0; k < kMaxPer; ++k) av[k] *= inv_Zs;
          c *= inv_Zs;
          sum_av = part * inv_Zs;
        }
        if (cands != nullptr) {
          // the candidate that this update rejected leaves the urn
          int x = -1;
          while (ci < a.n_cands && (x = cands[ci]) < 0) ++ci;
          ++ci;
          if (tid == 0) sh.bcast_d[2] = 0.0;
          __syncthreads();
#pragma unroll
          for (int k = 0; k < kMaxPer; ++k)
            if (x >= 0 && yi[k] == x && w64[k] > 0.0) { sh.bcast_d[2] = w64[k]; w64[k] = 0.0; }
          __syncthreads();
          removed += sh.bcast_d[2];
          const double rest = 1.0 - removed;
          qscale = rest > 0.0 ? 1.0 / rest : 0.0;
        }
      }
      const double zp_over_c = zp / c;
#pragma unroll
      for (int k = 0; k < kMaxPer; ++k)
        if (yi[k] >= 0) corr[k] = av[k] * zp_over_c - e_s[k];
      sum_corr = sum_av * zp_over_c - sum_e;    // the sum of the corrections, without another pass over the workgroup
    }
    double total = zp + sum_corr;
    bool use_corr = true;
    if (!(total > 0.0)) {          // defensive: an all-zero residual falls back to p itself
#pragma unroll
      for (int k = 0; k < kMaxPer; ++k) corr[k] = 0.0;
      total = zp;
      use_corr = false;
    }
    const double target = double(a.u) * total;

    // ---- which item: corrections into the items they fall into, then a scan per wave ------------------------
    auto item_of = [&](int y) {
      if (y < rs.head) return 0;
      const int64_t v = (int64_t(y) - rs.head) / E;
      return v >= rs.nvec ? n_items - 1 : 1 + int(v / kRunVecs);
    };
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k)
      if (yi[k] >= 0 && corr[k] != 0.0) atomicAdd(&item_val[item_of(yi[k])], corr[k]);
    __syncthreads();
    const int per = (n_items + 63) / 64;          // consecutive items per lane
    double lsum = 0.0;
    for (int q = 0; q < per; ++q) {
      const int it = lane * per + q;
      const double t = it < n_items ? item_val[it] : 0.0;
      lsum += t > 0.0 ? t : 0.0;
    }
    double run = wave_incl_scan_f64(lsum) - lsum;
    int found = -1, last_pos = -1;
    double found_before = 0.0, last_before = 0.0;
    for (int q = 0; q < per; ++q) {
      const int it = lane * per + q;
      const double t = it < n_items ? item_val[it] : 0.0;
      if (t > 0.0) {
        last_pos = it; last_before = run;
        if (run + t > target && found < 0) { found = it; found_before = run; }
        run += t;
      }
    }
    // the first lane that saw the target passed, else the last one that holds an item with mass
    const uint64_t hit = ballot(found >= 0), any = ballot(last_pos >= 0);
    int item = -1;
    double before_item = 0.0;
    if (hit != 0) {
      const int src = __ffsll((long long)hit) - 1;
      item = __shfl(found, src, 64);
      before_item = shfl_f64(found_before, src);
    } else if (any != 0) {
      const int src = 63 - __clzll((long long)any);
      item = __shfl(last_pos, src, 64);
      before_item = shfl_f64(last_before, src);
    }

    if (item == 0 || item == n_items - 1) {
      // an edge piece: fewer than E elements, walked by one thread
      const int piece = item == 0 ? 0 : n_pieces - 1;
      const int e0 = piece == 0 ? 0 : rs.head;
#pragma unroll
      for (int k = 0; k < kMaxPer; ++k)
        if (yi[k] >= 0 && item_of(yi[k]) == item) {
          const int e = yi[k] < rs.head ? yi[k] : rs.head + int(yi[k] - (rs.head + rs.nvec * E));
          elem_corr[e - e0] = corr[k];
        }
      __syncthreads();
      if (tid == 0) {
        const int e1 = piece == 0 ? rs.head : rs.head + rs.tail;
        double run_e = before_item;
        for (int e = e0; e < e1; ++e) {
          const int64_t y = edge_index<T>(rs, e);
          const float t = load_elem<T>(row, y);
          double v = t > -INFINITY ? exp64(double(__fmul_rn(t, rT)) - double(smax)) : 0.0;
          if (use_corr) {
            v += elem_corr[e - e0];
            if (v < 0.0) v = 0.0;
          }
          if (v > 0.0) {
            token = int(y);
            run_e += v;
            if (run_e > target) break;
          }
        }
        sh.bcast_i[3] = token;
      }
      __syncthreads();
      token = sh.bcast_i[3];
    } else if (item > 0) {
      // ---- which element of that run; thread t owns kPerT consecutive elements: one vector, requested
      // before the corrections are laid out, so that it travels meanwhile ------------------------------------
      static_assert(kPerT == E, "a thread's share of a run is one vector");
      const int r = item - 1;
      const int64_t run_first = rs.head + int64_t(r) * kRun;
      const int64_t my_vec = int64_t(r) * kRunVecs + tid;
      uint4 dv = neg_inf_vec<T>();
      if (my_vec < rs.nvec) dv = load_vec(&rs.body[my_vec]);
#pragma unroll
      for (int k = 0; k < kMaxPer; ++k)
        if (yi[k] >= run_first && yi[k] < run_first + kRun) elem_corr[yi[k] - run_first] = corr[k];
      __syncthreads();
      float tv[E];
      unpack<T>(dv, tv);
      double v[kPerT];
      double mine = 0.0;
      // the terms as the sweep made them: through the table where it was used (then smax is 0 and an entry is
      // the term itself), else the exponential
      bool by_table = false;
      if constexpr (ExpTab<T>::kHas) by_table = a.table != nullptr && smax == 0.0f;
#pragma unroll
      for (int q = 0; q < kPerT; ++q) {
        v[q] = 0.0;
        if (my_vec < rs.nvec) {
          double term = __longlong_as_double(0x7FF8000000000000ll);
          if constexpr (ExpTab<T>::kHas) {
            if (by_table) {
              const uint32_t w4[4] = {dv.x, dv.y, dv.z, dv.w};
              const uint32_t bits = (w4[q >> 1] >> ((q & 1) * 16)) & 0xFFFFu;
              const int rot = int(((bits << 1) & 0xFFFEu) | (bits >> 15)) - (2 * ExpTab<T>::kLo - 1);
              term = a.table[rot < 0 ? 0 : (rot > ExpTab<T>::kEntries + 1 ? ExpTab<T>::kEntries + 1 : rot)];
            }
          }
          if (term != term) term = exp64(double(__fmul_rn(tv[q], rT)) - double(smax));
          v[q] = term + elem_corr[tid * kPerT + q];
          if (v[q] < 0.0) v[q] = 0.0;
        }
        mine += v[q];
      }
      double run_total;
      const double excl = block_excl_scan_f64<kWaves>(mine, sh.red, run_total);
      // element at which the cumulative mass passes the target, else the last one with mass
      int first_pass = 0x7FFFFFFF, last_mass = -1;
      double run_e = before_item + excl;
#pragma unroll
      for (int q = 0; q < kPerT; ++q) {
        if (v[q] > 0.0) {
          run_e += v[q];
          last_mass = tid * kPerT + q;
          if (run_e > target && first_pass == 0x7FFFFFFF) first_pass = tid * kPerT + q;
        }
      }
      first_pass = -wave_max_i32(-first_pass);      // the smallest over the wave (0x7FFFFFFF = none)
      last_mass = wave_max_i32(last_mass);
      __syncthreads();
      if (lane == 0) { sh.red.i[wave_id()] = first_pass; sh.red.i[8 + wave_id()] = last_mass; }
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
  return token;
}

}  // namespace tslt
