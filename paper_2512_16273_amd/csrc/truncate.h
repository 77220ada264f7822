// tslt_truncate: Top-K / Top-rho truncation of draft logits (Section 3.1) and compaction to the
// sparse (index, logit) payload of Solution 1 (Section 3.2), one workgroup per row.
//
// One pass over the row.  The row's tiles are visited in batches of kBatch tiles taken at equal
// distances (tile b of every "quarter"), so that the first batch is a strided sample of the row.  From
// that sample a threshold tau0 is chosen that a little more than K elements of the whole row are
// expected to exceed.  The pass then does two things per 16-byte vector: it adds exp2(z*k2 - c) to the
// row's fp32 partial sums (the softmax normaliser, k2 = log2(e)/T, c a reference taken from the
// sample maximum), and, if any element of the vector is above tau0, it parks the vector in a small
// per-wave LDS ring; rings are expanded into (value, index) candidate records when they fill up.  If
// at least K elements were above tau0 the top-K set is among the candidates and is found exactly by
// sorting them; otherwise (ties, masked rows, unlucky sample, overflow of a buffer) the row is redone
// by an exact radix selection that makes several passes.  Either way the kept entries are then
// evaluated in fp64, which is also where Top-rho and the renormalisation are decided.
#pragma once
#include "common.h"
#include "wire.h"
#include "exp64.h"

namespace tslt {

constexpr int kTruncThreads = 256;   // threads of a truncate workgroup (one row each)
constexpr int kBatch = 4;        // tiles of the threshold sample, taken at equal distances over the row
constexpr int kGroup = 2;        // tiles (one 16-byte vector per thread each) in a stage of the pass's pipeline
// The kernel comes in two shapes.  "Wide": two stages in flight per thread and eight waves per SIMD asked of the
// compiler (64 registers), so that eight workgroups share a compute unit; for launches whose LDS footprint
// allows that many (k_cap of a few hundred).  "Deep": four stages in flight and four waves per SIMD; for the
// launches whose candidate arrays leave room for fewer workgroups (k_cap 1024: three per compute unit), which
// then need more requests in flight each to keep the memory busy.
constexpr int kStagesWide = 2, kWavesWide = 8;
constexpr int kStagesDeep = 4, kWavesDeep = 4;
constexpr int kRing = 96;      // vectors a wave can park
constexpr int kRingExpand = 58; // expanded when it holds more than this: one pass of 64 lanes, nearly all busy

struct TruncateParams {
  const void* logits;
  int64_t rows, V, row_stride;
  float rT;          // fl32(1/T)
  float k2;          // fl32(rT * log2(e))
  float top_p;       // 0 = off
  int k_sel;         // min(top_k (if on), k_cap)
  int k_cap;
  int payload;       // 0: the scaled logits as computed; 1 / 2: rounded to bfloat16 / binary16 before q_hat and the draws
  int jprime;        // rank (1-based) among the 256 per-thread sample maxima that gives tau0; 0 = always exact path
  int tau_bits;      // number of leading key bits resolved by the threshold search
  int sort_cap;      // capacity of the candidate array
  int lds_recs;      // records that fit in the candidate region; those past sort_cap are sort scratch
  int ring_bytes;    // size of the ring space at the start of dynamic LDS (ring_bytes_for the workgroup's waves)
  int tmp_in_ring;   // the sort scratch is the ring space behind the tables
  int32_t* out_idx;
  float* out_logit;
  float* out_prob;
  int32_t* out_count;
  float* out_mass;
  int32_t* status;
  // optional draws from q_hat in the same launch (null u = none)
  int without_replacement;
  const float* u;    // [rows, n_samples]
  int n_samples;
  int32_t* out_token;
  int32_t* out_slot;
};

// Dynamic LDS: [ rings ] [ candidates, then sort scratch ].  The ring space is
// reused for the sort's three 256-entry tables and, before the pass, for the per-thread sample maxima.
constexpr int ring_bytes_for(int n_waves) { return n_waves * (kRing * 20); }      // per slot a vector and its index
static_assert(ring_bytes_for(2) >= 3 * 256 * 4, "ring space must hold the sort tables");
inline size_t truncate_lds_bytes(int ring_bytes, int lds_recs) { return size_t(ring_bytes) + size_t(8) * lds_recs; }
inline int truncate_sort_scratch(int k_sel) { return k_sel + k_sel / 2 + 64; }   // records the sort may need

struct TruncateShared {
  BlockScratch red;
  int cand_count;
  int overflow;
  int bcast_i[4];
  double bcast_d[2];
};

// ---------------------------------------------------------------------------------------------
// Exact multi-pass selection, the last resort: the k_eff largest elements of the row in the canonical order, found
// by a 4x8-bit radix search for the k-th largest key and an index-ordered collection of the ties.
// Also recomputes the fp32 sum with the true maximum as reference.  Returns the number of
// candidates written to cand[] (exactly k_eff), or 0 with `st` set.
// ---------------------------------------------------------------------------------------------
template <typename T, int NT>
__device__ int exact_select(const void* row, int64_t V, int k_sel, float k2, uint64_t* cand, uint32_t* hist,
                            TruncateShared& sh, float& c_ref, double& z_c, int& st) {
  constexpr int NW = NT / 64;
  const int tid = threadIdx.x;
  // pass 1: validity, number of selectable elements, maximum
  int fin = 0, bad = 0;
  float vmax = -INFINITY;
  for (int64_t i = tid; i < V; i += NT) {
    float v = load_elem<T>(row, i);
    if (v != v || v == INFINITY) bad = 1;
    else if (v > -INFINITY) { ++fin; vmax = fmaxf(vmax, v); }
  }
  bad = block_sum_i32<NW>(bad, sh.red);
  fin = block_sum_i32<NW>(fin, sh.red);
  vmax = block_max_f32<NW>(vmax, sh.red);
  if (bad) { st |= 1; return 0; }
  if (fin == 0) { st |= 2; return 0; }
  const int k_eff = k_sel < fin ? k_sel : fin;

  // radix search, most significant digit first, over keys of elements > -inf
  uint32_t prefix = 0;
  int need = k_eff;
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int b = tid; b < 256; b += NT) hist[b] = 0;
    __syncthreads();
    const uint32_t hi_mask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
    for (int64_t i = tid; i < V; i += NT) {
      float v = load_elem<T>(row, i);
      uint32_t key = mono_key(v + 0.0f);
      if (v > -INFINITY && (key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid == 0) {
      int cum = 0, d = 255;
      for (; d > 0; --d) {
        int h = int(hist[d]);
        if (cum + h >= need) break;
        cum += h;
      }
      sh.bcast_i[0] = d;
      sh.bcast_i[1] = need - cum;
    }
    __syncthreads();
    prefix |= uint32_t(sh.bcast_i[0]) << shift;
    need = sh.bcast_i[1];
    __syncthreads();
  }
  const uint32_t key_k = prefix;   // key of the k_eff-th largest element; `need` ties are to be taken

  // collection in index order: everything above key_k, and the `need` lowest-index ties
  if (tid == 0) sh.cand_count = 0;
  __syncthreads();
  int eq_base = 0;
  constexpr int kChunk = 8;
  for (int64_t base = 0; base < V; base += int64_t(NT) * kChunk) {
    uint32_t eq_mask = 0;
    const int64_t i0 = base + int64_t(tid) * kChunk;
#pragma unroll
    for (int e = 0; e < kChunk; ++e) {
      int64_t i = i0 + e;
      if (i < V) {
        float v = load_elem<T>(row, i);
        uint32_t key = mono_key(v + 0.0f);
        if (v > -INFINITY) {
          if (key > key_k) {
            int pos = atomicAdd(&sh.cand_count, 1);
            cand[pos] = make_cand(v, uint32_t(i));
          } else if (key == key_k) {
            eq_mask |= 1u << e;
          }
        }
      }
    }
    int total;
    int off = block_excl_scan_i32<NW>(__popc(eq_mask), sh.red, total);
    if (eq_base < need) {
      int ord = eq_base + off;
#pragma unroll
      for (int e = 0; e < kChunk; ++e) {
        if ((eq_mask >> e) & 1u) {
          if (ord < need) {
            int pos = atomicAdd(&sh.cand_count, 1);
            cand[pos] = make_cand(load_elem<T>(row, i0 + e), uint32_t(i0 + e));
          }
          ++ord;
        }
      }
    }
    eq_base += total;
  }
  // the normaliser's fp32 partial sums, referenced to the true maximum
  c_ref = __fmul_rn(vmax, k2);
  double acc = 0.0;
  for (int64_t i = tid; i < V; i += NT) acc += double(fast_exp2(__builtin_fmaf(load_elem<T>(row, i), k2, -c_ref)));
  z_c = block_sum_f64<NW>(acc, sh.red);
  __syncthreads();
  return k_eff;
}

// ---------------------------------------------------------------------------------------------
// ---------------------------------------------------------------------------------------------
// Two-pass selection, the first fallback.  Pass 1 takes the maximum of 1024 disjoint groups of the
// row (4 per thread); the k-th largest of those maxima is a threshold that at least k elements reach,
// so the top-k set is among the elements >= it, of which there are only a few more than k unless the
// row is full of ties.  Pass 2 collects them.  Returns the number of candidates, 0 with `st` set for
// an unusable row, or -1 when the candidates do not fit (then the radix selection is used).
// ---------------------------------------------------------------------------------------------
template <typename T, int NT>
__device__ int two_pass_select(const void* row, const RowSplit& rs, int k_sel, float k2, uint64_t* cand, int cap,
                               uint64_t* sort_tmp, int sort_tmp_cap, uint32_t* tables, TruncateShared& sh,
                               bool need_sum, float& c_ref, double& z_c, int& st) {
  constexpr int E = ElemTraits<T>::kPerVec;
  constexpr int NW = NT / 64;
  constexpr int GPT = 1024 / NT;       // groups per thread
  const int tid = threadIdx.x;
  const int n_edge = rs.head + rs.tail;
  const int64_t n_tiles = (rs.nvec + NT - 1) / NT;
  if (cap < GPT * NT + 2 * E) return -1;
  // pass 1
  float gmax[GPT];
#pragma unroll
  for (int u = 0; u < GPT; ++u) gmax[u] = -INFINITY;
  int fin = 0, bad = 0;
  for (int64_t t0 = 0; t0 < n_tiles; t0 += GPT) {
    uint4 d[GPT];
#pragma unroll
    for (int u = 0; u < GPT; ++u) {
      const int64_t vi = (t0 + u) * NT + tid;
      d[u] = neg_inf_vec<T>();
      if (vi < rs.nvec) d[u] = load_vec(&rs.body[vi]);
    }
#pragma unroll
    for (int u = 0; u < GPT; ++u) {
      float v[E];
      unpack<T>(d[u], v);
#pragma unroll
      for (int e = 0; e < E; ++e) {
        bad |= (v[e] != v[e] || v[e] == INFINITY) ? 1 : 0;
        fin += v[e] > -INFINITY ? 1 : 0;
        gmax[u] = fmaxf(gmax[u], v[e]);
      }
    }
  }
  float edge_v = -INFINITY;
  int64_t edge_i = 0;
  if (tid < n_edge) {
    edge_i = edge_index<T>(rs, tid);
    edge_v = load_elem<T>(row, edge_i);
    bad |= (edge_v != edge_v || edge_v == INFINITY) ? 1 : 0;
    fin += edge_v > -INFINITY ? 1 : 0;
  }
  bad = block_or_i32<NW>(bad, sh.red);
  fin = block_sum_i32<NW>(fin, sh.red);
  if (bad) { st |= 1; return 0; }
  if (fin == 0) { st |= 2; return 0; }
  const int k_eff = k_sel < fin ? k_sel : fin;
  float vmax = gmax[0];
#pragma unroll
  for (int u = 1; u < GPT; ++u) vmax = fmaxf(vmax, gmax[u]);
  vmax = block_max_f32<NW>(fmaxf(vmax, edge_v), sh.red);
  // the k_eff-th largest group maximum (edge elements are groups of their own; empty groups are left out)
  if (tid == 0) sh.cand_count = 0;
  __syncthreads();
#pragma unroll
  for (int u = 0; u < GPT; ++u)
    if (gmax[u] > -INFINITY) cand[atomicAdd(&sh.cand_count, 1)] = make_cand(gmax[u], uint32_t(tid * GPT + u));
  if (tid < n_edge && edge_v > -INFINITY) cand[atomicAdd(&sh.cand_count, 1)] = make_cand(edge_v, uint32_t(GPT * NT + tid));
  __syncthreads();
  const int n_groups = sh.cand_count;
  float tau = -INFINITY;                               // fewer than k_eff non-empty groups: take everything
  if (n_groups >= k_eff) {
    if (!bucket_sort_desc<NT>(cand, n_groups, sort_tmp, sort_tmp_cap, cand, k_eff, tables, tables + 256, tables + 512,
                          sh.red))
      return -1;
    tau = cand_value(cand[k_eff - 1]);
  }
  __syncthreads();
  // pass 2
  if (tid == 0) sh.cand_count = 0;
  __syncthreads();
  if (need_sum) c_ref = __fmul_rn(vmax, k2);
  double acc = 0.0;
  for (int64_t t0 = 0; t0 < n_tiles; t0 += 4) {
    uint4 d[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t vi = (t0 + u) * NT + tid;
      d[u] = neg_inf_vec<T>();
      if (vi < rs.nvec) d[u] = load_vec(&rs.body[vi]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float v[E];
      unpack<T>(d[u], v);
      const uint32_t base = uint32_t(rs.head) + uint32_t((t0 + u) * NT + tid) * E;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        if (need_sum) acc += double(fast_exp2(__builtin_fmaf(v[e], k2, -c_ref)));
        if (v[e] >= tau && v[e] > -INFINITY) {
          const int pos = atomicAdd(&sh.cand_count, 1);
          if (pos < cap) cand[pos] = make_cand(v[e], base + e);
        }
      }
    }
  }
  if (tid < n_edge) {
    if (need_sum) acc += double(fast_exp2(__builtin_fmaf(edge_v, k2, -c_ref)));
    if (edge_v >= tau && edge_v > -INFINITY) {
      const int pos = atomicAdd(&sh.cand_count, 1);
      if (pos < cap) cand[pos] = make_cand(edge_v, uint32_t(edge_i));
    }
  }
  if (need_sum) z_c = block_sum_f64<NW>(acc, sh.red);
  __syncthreads();
  const int n = sh.cand_count;
  __syncthreads();
  return n <= cap ? n : -1;
}

// A ring slot holds a 16-byte vector of which at least one element is above tau0, and its index (in
// vectors, within the row's aligned body).
//
// Expands the n vectors parked in a wave's ring into candidate records (elements above tau0).  Lane s
// takes slot s: it marks which of the vector's elements are above tau0, a wave scan of the counts gives
// every lane its place behind a single reservation in the shared candidate array.  Nearly every slot holds
// one such element, so they are then written one per round (as many rounds as the fullest slot needs),
// each read back from the slot by its position, instead of one branch per element position.
template <typename T> __device__ __forceinline__ float ring_element(const uint4* ring, int slot, int e);
template <> __device__ __forceinline__ float ring_element<float>(const uint4* ring, int slot, int e) {
  return reinterpret_cast<const float*>(ring)[slot * 4 + e];
}
template <> __device__ __forceinline__ float ring_element<Bf16>(const uint4* ring, int slot, int e) {
  return as_f32(uint32_t(reinterpret_cast<const uint16_t*>(ring)[slot * 8 + e]) << 16);
}
template <> __device__ __forceinline__ float ring_element<F16>(const uint4* ring, int slot, int e) {
  return f16_lo(reinterpret_cast<const uint16_t*>(ring)[slot * 8 + e]);
}

template <typename T>
__device__ __forceinline__ void expand_ring(const uint4* ring, const uint32_t* ring_vidx, int n, float tau0,
                                            uint32_t head, uint64_t* cand, int cap, TruncateShared& sh) {
  constexpr int E = ElemTraits<T>::kPerVec;
  const int lane = lane_id();
  for (int s0 = 0; s0 < n; s0 += 64) {
    const int s = s0 + lane;
    uint32_t mask = 0, vi = 0;          // bit e: element e of this lane's vector is above tau0
    if (s < n) {
      float v[E];
      unpack<T>(ring[s], v);
      vi = ring_vidx[s];
#pragma unroll
      for (int e = 0; e < E; ++e) mask |= v[e] > tau0 ? (1u << e) : 0u;
    }
    const int cnt = __popc(mask);
    const int incl = wave_incl_scan_i32(cnt);
    const int total = last_lane_i32(incl);
    if (total == 0) continue;
    int base = 0;
    if (lane == 0) base = atomicAdd(&sh.cand_count, total);
    base = __builtin_amdgcn_readfirstlane(base);
    int pos = base + incl - cnt;
    const uint32_t idx0 = head + vi * E;
    const int rounds = wave_max_i32(cnt);
    for (int r = 0; r < rounds; ++r) {
      if (mask != 0) {
        const int e = __builtin_ctz(mask);
        mask &= mask - 1;
        if (pos < cap) cand[pos] = make_cand(ring_element<T>(ring, s, e), idx0 + uint32_t(e));
        ++pos;
      }
    }
  }
  // more candidates than `cap` show in sh.cand_count, which the caller checks
}

template <typename T> __device__ __forceinline__ float vec_max(const float (&v)[ElemTraits<T>::kPerVec]);
template <> __device__ __forceinline__ float vec_max<float>(const float (&v)[4]) {
  return max3f(max3f(v[0], v[1], v[2]), v[3], v[3]);
}
__device__ __forceinline__ float vec_max8(const float (&v)[8]) {
  return max3f(max3f(max3f(v[0], v[1], v[2]), v[3], v[4]), max3f(v[5], v[6], v[7]), v[5]);
}
template <> __device__ __forceinline__ float vec_max<Bf16>(const float (&v)[8]) { return vec_max8(v); }
template <> __device__ __forceinline__ float vec_max<F16>(const float (&v)[8]) { return vec_max8(v); }

template <typename T, int NT, int kStages, int kWavesPerSimd>
__global__ __launch_bounds__(NT, kWavesPerSimd) void truncate_kernel(const TruncateParams p) {
  constexpr int E = ElemTraits<T>::kPerVec;
  constexpr int NW = NT / 64;
  static_assert(kBatch == 4, "the sample tiles are handled as two pairs");
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  __shared__ TruncateShared sh;
  uint4* ring_all = reinterpret_cast<uint4*>(dyn_lds);
  uint32_t* ring_vidx_all = reinterpret_cast<uint32_t*>(dyn_lds + NW * kRing * 16);
  uint32_t* tables = reinterpret_cast<uint32_t*>(dyn_lds);          // 3 x 256 entries, aliasing the rings
  uint64_t* cand = reinterpret_cast<uint64_t*>(dyn_lds + p.ring_bytes);
  // sort scratch: what is left of the ring space behind the tables, or (if that is too small for the
  // requested k) the records behind the candidate capacity
  uint64_t* sort_tmp = p.tmp_in_ring ? reinterpret_cast<uint64_t*>(dyn_lds + 3 * 256 * 4) : cand + p.sort_cap;
  const int sort_tmp_cap = p.tmp_in_ring ? (p.ring_bytes - 3 * 256 * 4) / 8 : p.lds_recs - p.sort_cap;

  const int tid = threadIdx.x;
  const int lane = lane_id();
  const int wave = wave_id();
  const int64_t row_i = blockIdx.x;
  // The sample: the first tile of kBatch batches at equal distances; a row with fewer than 4*kBatch
  // complete batches uses its first kBatch tiles.
  // (Every load of the pass below is unconditional: an address past the row's end is replaced by that of
  // the row's last vector and the value by -inf afterwards.  With conditional loads the number of loads in
  // flight is not known where a wait is placed, and a wait for one batch waits for all that were
  // requested after it as well.)
  auto load_sample = [&](const RowSplit& r, uint4 (&q)[kBatch]) {
    const uint32_t nv = uint32_t(r.nvec);            // > 0 here
    const uint32_t nf = nv / (kBatch * NT);
    const uint32_t stride = nf >= 4 ? (nf / 4) * kBatch : 1;
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const uint32_t vi = u * stride * NT + tid;
      q[u] = load_vec_stream(&r.body[vi < nv ? vi : nv - 1]);
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u)
      if (u * stride * NT + tid >= nv) q[u] = neg_inf_vec<T>();
  };
  const void* row = reinterpret_cast<const char*>(p.logits) + size_t(row_i) * size_t(p.row_stride) * ElemTraits<T>::kBytes;
  const RowSplit rs = split_row<T>(row, p.V);
  const int n_edge = rs.head + rs.tail;
  const uint32_t nvec = uint32_t(rs.nvec);
  const uint32_t n_tiles = (nvec + NT - 1) / NT;
  const uint32_t n_full = nvec / (kBatch * NT);        // batches of kBatch complete, consecutive tiles
  const bool long_row = n_full >= 4;
  const uint32_t s_stride = long_row ? (n_full / 4) * kBatch : 1;   // distance of the sample tiles, in tiles

  int st = 0;
  int n_cand = 0;
  float c_ref = 0.0f;
  double z_c = 0.0;
  bool fast_ok = p.jprime > 0 && n_tiles > 0;
  if (tid == 0) { sh.cand_count = 0; sh.overflow = 0; }

  if (fast_ok) {
    // ---- the sample: per-thread maxima ----------------------------------------------------------
    uint4 d[kBatch];
    load_sample(rs, d);
    // The pass keeps kStages stages of kGroup tiles in flight per thread; the first ones are requested now, so
    // that they travel while the threshold is being worked out.  A sample tile is the first tile of its stage
    // (the sample tiles lie a multiple of kBatch tiles apart) and is not read again.  A long row's ragged end
    // (the last tile possibly incomplete, the last stage possibly half empty) is the last stage.
    static_assert(kBatch % kGroup == 0 && kGroup == 2, "a stage is a pair of tiles; sample tiles start a stage");
    uint4 pipe[kStages][kGroup];
    const uint32_t n_stage = long_row ? (n_tiles + kGroup - 1) / kGroup : 0u;
    uint32_t skip_g = 0, skips_left = kBatch;
    const uint32_t stride_g = s_stride / kGroup;
    const uint32_t last_vec = nvec - 1;
    auto issue = [&](uint32_t g, uint4 (&q)[kGroup]) {
      const uint32_t v0 = g * (kGroup * NT) + tid;
      // the first tile of a sample stage is in registers already: its slot repeats the second tile's load
      const bool skip = skips_left > 0 && g == skip_g;
      if (skip) { skip_g += stride_g; --skips_left; }
      const uint32_t va = skip ? v0 + NT : v0, vb = v0 + NT;
      q[0] = load_vec_stream(&rs.body[va < last_vec ? va : last_vec]);
      q[1] = load_vec_stream(&rs.body[vb < last_vec ? vb : last_vec]);
    };
    if (n_stage > 0) {
#pragma unroll
      for (int s = 0; s < kStages; ++s) issue(uint32_t(s), pipe[s]);
    }
    float tmax = -INFINITY;
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      float v[E];
      unpack<T>(d[u], v);
      tmax = fmaxf(tmax, vec_max<T>(v));
    }
    // the sample is looked at again after the threshold is known; it is to wait in its packed form (the
    // compiler would otherwise keep the unpacked values, twice the registers, across the threshold search)
#pragma unroll
    for (int u = 0; u < kBatch; ++u) asm volatile("" : "+v"(d[u].x), "+v"(d[u].y), "+v"(d[u].z), "+v"(d[u].w));
    tables[tid] = mono_key(tmax);
    __syncthreads();
    // ---- tau0: the jprime-th largest of the 256 per-thread sample maxima (every wave redundantly)
    uint32_t kq[NW];
#pragma unroll
    for (int q = 0; q < NW; ++q) kq[q] = tables[lane + 64 * q];
    uint32_t tau_key = 0;
    for (int bit = 31; bit >= 32 - p.tau_bits; --bit) {
      const uint32_t trial = tau_key | (1u << bit);
      int cnt = 0;
#pragma unroll
      for (int q = 0; q < NW; ++q) cnt += __popcll(ballot(kq[q] >= trial));
      if (cnt >= p.jprime) tau_key = trial;
    }
    uint32_t top_key = kq[0];   // the sample maximum
#pragma unroll
    for (int q = 1; q < NW; ++q) top_key = kq[q] > top_key ? kq[q] : top_key;
    top_key = wave_max_u32(top_key);
    const float smax = key_to_f32(top_key);
    const float tau0 = tau_key <= kKeyNegInf ? -INFINITY : key_to_f32(tau_key);
    fast_ok = smax > -INFINITY && smax < INFINITY;   // false for NaN too
    c_ref = __fmul_rn(smax, p.k2);
    __syncthreads();                                  // the maxima are read; the space becomes the rings

    if (fast_ok) {
      // ---- the pass -------------------------------------------------------------------------
      const float neg_c = -c_ref;
      const float k2 = p.k2;
      // fp32 sums live for a few vectors only and are then added to an fp64 total: a long-lived fp32
      // accumulator that has met one large term rounds away the many small ones that follow
      double dacc = 0.0;
      int wave_cnt = 0;                                // pairs parked in this wave's ring
      bool lost = false;                               // wave-uniform: a ring overflowed
      uint4* ring = ring_all + wave * kRing;
      uint32_t* ring_vidx = ring_vidx_all + wave * kRing;
      const uint32_t head = uint32_t(rs.head);

      // Two vectors at a time: their exp2 terms go to the partial sums; a vector with an element above
      // tau0 is parked in the ring, which is expanded when it holds about a wave's worth of vectors.
      // (returns the sum of the pair's exp2 terms)
      auto process_pair = [&](const uint4& w0, const uint4& w1, uint32_t vidx0, uint32_t vidx1) -> float {
        float a[E], b[E];
        unpack<T>(w0, a);
        unpack<T>(w1, b);
        const bool hit_a = vec_max<T>(a) > tau0, hit_b = vec_max<T>(b) > tau0;
        float t[2 * E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
          t[e] = fast_exp2(__builtin_fmaf(a[e], k2, neg_c));
          t[E + e] = fast_exp2(__builtin_fmaf(b[e], k2, neg_c));
        }
#pragma unroll
        for (int w = E; w >= 1; w >>= 1)          // a tree: 2E - 1 additions, none of them with a zero
#pragma unroll
          for (int e = 0; e < w; ++e) t[e] += t[e + w];
        const float pair_sum = t[0];
        const uint64_t mask_a = ballot(hit_a), mask_b = ballot(hit_b);
        if ((mask_a | mask_b) != 0) {
          const int n_a = __popcll(mask_a);
          const int pos_a = wave_cnt + lanes_below(mask_a);
          const int pos_b = wave_cnt + n_a + lanes_below(mask_b);
          if (hit_a) {
            if (pos_a < kRing) { ring[pos_a] = w0; ring_vidx[pos_a] = vidx0; }
          }
          if (hit_b) {
            if (pos_b < kRing) { ring[pos_b] = w1; ring_vidx[pos_b] = vidx1; }
          }
          wave_cnt += n_a + __popcll(mask_b);
          lost |= wave_cnt > kRing;                    // some vector found no slot
          if (wave_cnt > kRingExpand) {                // wave-uniform
            expand_ring<T>(ring, ring_vidx, wave_cnt < kRing ? wave_cnt : kRing, tau0, head, cand, p.sort_cap, sh);
            wave_cnt = 0;
          }
        }
        return pair_sum;
      };

      // the sample tiles, already in registers
      {
        const uint32_t t1 = s_stride, t2 = 2 * s_stride, t3 = 3 * s_stride;
        const float s01 = process_pair(d[0], d[1], tid, t1 * NT + tid);
        const float s23 = process_pair(d[2], d[3], t2 * NT + tid, t3 * NT + tid);
        dacc += double(s01 + s23);
      }
      uint32_t first_generic_tile = kBatch;             // short rows: everything after the sample tiles
      if (long_row) {
        uint32_t seen_g = 0, seen_left = kBatch;
        const uint32_t ragged_g = n_full * (kBatch / kGroup);        // from here on a vector may lie past the row's end
        static_assert(kStages % 2 == 0, "the fp32 sums of two stages are added up before they go to the fp64 total");
        for (uint32_t g0 = 0; g0 < n_stage; g0 += kStages) {
          float two = 0.0f;
#pragma unroll
          for (int s = 0; s < kStages; ++s) {
            const uint32_t g = g0 + s;
            if (g < n_stage) {                                        // wave-uniform, no loads inside
              const uint32_t v0 = g * (kGroup * NT) + tid;
              if (seen_left > 0 && g == seen_g) {                     // a sample stage: its first tile is done
                seen_g += stride_g; --seen_left;
                pipe[s][0] = neg_inf_vec<T>();
              }
              if (g >= ragged_g) {                                    // the ragged end
                if (v0 >= nvec) pipe[s][0] = neg_inf_vec<T>();
                if (v0 + NT >= nvec) pipe[s][1] = neg_inf_vec<T>();
              }
              const float ps = process_pair(pipe[s][0], pipe[s][1], v0, v0 + NT);
              two = (s & 1) ? two + ps : ps;
            }
            if ((s & 1) && g0 + s - 1 < n_stage) dacc += double(two);   // (a lone last stage left its sum in `two`)
            issue(g + kStages, pipe[s]);
          }
        }
        first_generic_tile = n_tiles;
      }
      // short rows: the tiles after the sample, which may be incomplete
      for (uint32_t t = first_generic_tile; t < n_tiles; t += 2) {
        const uint32_t v0 = t * NT + tid, v1 = v0 + NT;
        d[0] = neg_inf_vec<T>();
        d[1] = neg_inf_vec<T>();
        if (v0 < nvec) d[0] = load_vec_stream(&rs.body[v0]);
        if (v1 < nvec) d[1] = load_vec_stream(&rs.body[v1]);
        dacc += double(process_pair(d[0], d[1], v0, v1));
      }
      expand_ring<T>(ring, ring_vidx, wave_cnt < kRing ? wave_cnt : kRing, tau0, head, cand, p.sort_cap, sh);
      if (lost && lane == 0) sh.overflow = 1;
      // edge elements (row not 16-byte aligned, or V not a whole number of vectors)
      if (tid < n_edge) {
        const int64_t edge_i = edge_index<T>(rs, tid);
        const float edge_v = load_elem<T>(row, edge_i);
        dacc += double(fast_exp2(__builtin_fmaf(edge_v, k2, neg_c)));
        if (edge_v > tau0) {
          const int pos = atomicAdd(&sh.cand_count, 1);
          if (pos < p.sort_cap) cand[pos] = make_cand(edge_v, uint32_t(edge_i));
        }
      }
      z_c = block_sum_f64<NW>(dacc, sh.red);
      __syncthreads();
      n_cand = sh.cand_count;
      fast_ok = !sh.overflow && n_cand <= p.sort_cap && n_cand >= p.k_sel && z_c > 0.0 && z_c < INFINITY;
      __syncthreads();
    }
  }

  if (!fast_ok) {
    st |= 256;
    const bool need_sum = !(z_c > 0.0 && z_c < INFINITY);
    n_cand = two_pass_select<T, NT>(row, rs, p.k_sel, p.k2, cand, p.sort_cap, sort_tmp, sort_tmp_cap, tables, sh, need_sum,
                                c_ref, z_c, st);
    if (n_cand < 0) n_cand = exact_select<T, NT>(row, p.V, p.k_sel, p.k2, cand, tables, sh, c_ref, z_c, st);
  }

  // ---- sort the candidates into canonical order ------------------------------------------------
  __syncthreads();
  if (!bucket_sort_desc<NT>(cand, n_cand, sort_tmp, sort_tmp_cap, cand, p.k_sel, tables, tables + 256, tables + 512,
                        sh.red)) {
    // the bin at the k-th place is too crowded for the scratch space (a row full of ties): radix selection
    // delivers exactly k candidates, which always fit
    st |= 256;
    n_cand = exact_select<T, NT>(row, p.V, p.k_sel, p.k2, cand, tables, sh, c_ref, z_c, st);
    bucket_sort_desc<NT>(cand, n_cand, sort_tmp, sort_tmp_cap, cand, p.k_sel, tables, tables + 256, tables + 512, sh.red);
  }
  const int k_eff = n_cand < p.k_sel ? n_cand : p.k_sel;

  // ---- fp64 evaluation of the kept head: Top-rho, renormalisation, outputs -----------------------
  // thread t owns entries [t*per, t*per + per) so that a block scan gives prefix masses in order
  const int per = (k_eff + NT - 1) / NT;       // 0..kMaxPer
  constexpr int kMaxPer = 1024 / NT;
  double e64[kMaxPer];
  float s32[kMaxPer];
  uint32_t idx[kMaxPer];
  double local = 0.0, head32 = 0.0;
  float v0 = 0.0f, m_s = 0.0f;
  if (k_eff > 0) {
    v0 = cand_value(cand[0]);
    m_s = __fmul_rn(v0, p.rT);
  }
#pragma unroll
  for (int r = 0; r < kMaxPer; ++r) {
    e64[r] = 0.0; s32[r] = 0.0f; idx[r] = 0;
    const int i = tid * per + r;
    if (r < per && i < k_eff) {
      const uint64_t c = cand[i];
      const float v = cand_value(c);
      idx[r] = cand_index(c);
      s32[r] = __fmul_rn(v, p.rT);
      e64[r] = exp64(double(s32[r]) - double(m_s));
      local += e64[r];
      head32 += double(fast_exp2(__builtin_fmaf(v, p.k2, -c_ref)));
    }
  }
  double head64;
  const double excl = block_excl_scan_f64<NW>(local, sh.red, head64);
  head32 = block_sum_f64<NW>(head32, sh.red);
  // normaliser relative to the row maximum: fp32 tail rescaled to that reference + fp64 head
  double tail = z_c - head32;
  if (tail < 0.0) tail = 0.0;
  const double Z = k_eff > 0 ? tail * exp64((double(c_ref) - double(v0) * double(p.k2)) * 0.69314718055994530942) + head64 : 0.0;

  int count = k_eff;
  if (p.top_p > 0.0f && k_eff > 0) {
    const double thr = double(p.top_p) * Z;
    int below = 0;
    double run = excl;
#pragma unroll
    for (int r = 0; r < kMaxPer; ++r) {
      const int i = tid * per + r;
      if (r < per && i < k_eff) {
        run += e64[r];
        below += run < thr ? 1 : 0;
      }
    }
    below = block_sum_i32<NW>(below, sh.red);
    count = below + 1 < k_eff ? below + 1 : k_eff;
  }
  // mass of the kept set: inclusive prefix at entry count-1
  {
    double run = excl;
#pragma unroll
    for (int r = 0; r < kMaxPer; ++r) {
      const int i = tid * per + r;
      if (r < per && i < k_eff) {
        run += e64[r];
        if (i == count - 1) sh.bcast_d[0] = run;
      }
    }
  }
  __syncthreads();
  const double c_sel = count > 0 ? sh.bcast_d[0] : 1.0;

  // what prob and the draws are made of: the kept entries' terms, or, with a 16-bit payload, the terms of
  // the rounded values (q_hat is the softmax of what the receiver gets)
  double pw[kMaxPer];
  double p_excl = excl, p_total = c_sel;
#pragma unroll
  for (int r = 0; r < kMaxPer; ++r) pw[r] = e64[r];
  if (p.payload != kPayloadF32) {
    const double m_r = double(round_payload(m_s, p.payload));
    double mine = 0.0;
#pragma unroll
    for (int r = 0; r < kMaxPer; ++r) {
      const int i = tid * per + r;
      pw[r] = 0.0;
      if (r < per && i < count) {
        s32[r] = round_payload(s32[r], p.payload);
        pw[r] = exp64(double(s32[r]) - m_r);
        mine += pw[r];
      }
    }
    p_excl = block_excl_scan_f64<NW>(mine, sh.red, p_total);
    if (!(p_total > 0.0)) p_total = 1.0;
  }

  const size_t out0 = size_t(row_i) * size_t(p.k_cap);
  const double inv_total = 1.0 / p_total;        // one reciprocal instead of a division per entry
#pragma unroll
  for (int r = 0; r < kMaxPer; ++r) {
    const int i = tid * per + r;
    if (r < per && i < k_eff && i < count) {
      p.out_idx[out0 + i] = int32_t(idx[r]);
      p.out_logit[out0 + i] = s32[r];
      if (p.out_prob) p.out_prob[out0 + i] = float(pw[r] * inv_total);
    }
  }
  for (int i = count + tid; i < p.k_cap; i += NT) {
    p.out_idx[out0 + i] = -1;
    p.out_logit[out0 + i] = -INFINITY;
    if (p.out_prob) p.out_prob[out0 + i] = 0.0f;
  }
  if (tid == 0) {
    p.out_count[row_i] = count;
    if (p.out_mass) p.out_mass[row_i] = count > 0 ? float(c_sel / Z) : 0.0f;
    if (p.status) p.status[row_i] = st;
  }
  // ---- draws from q_hat: the first entry whose inclusive prefix exceeds u * (mass of the kept set) ---
  // Without replacement a drawn entry's weight becomes 0 and the prefix masses are scanned again, so the
  // next draw is from the renormalised rest; when nothing is left the draw gives -1.
  if (p.u) {
    double w_total = count > 0 ? p_total : 0.0;
    for (int c = 0; c < p.n_samples; ++c) {
      const size_t o = size_t(row_i) * p.n_samples + c;
      const double target = double(p.u[o]) * w_total;
      int not_above = 0, last_pos = -1;
      double run = p_excl;
#pragma unroll
      for (int r = 0; r < kMaxPer; ++r) {
        const int i = tid * per + r;
        if (r < per && i < count) {
          run += pw[r];
          not_above += run > target ? 0 : 1;
          if (pw[r] > 0.0) last_pos = i;
        }
      }
      int slot = w_total > 0.0 ? block_sum_i32<NW>(not_above, sh.red) : -1;
      if (slot >= count) slot = block_max_i32<NW>(last_pos, sh.red);   // only for u >= 1 (uniform branch)
#pragma unroll
      for (int r = 0; r < kMaxPer; ++r)
        if (r < per && tid * per + r == slot) p.out_token[o] = int32_t(idx[r]);
      if (tid == 0) {
        if (slot < 0) p.out_token[o] = -1;
        if (p.out_slot) p.out_slot[o] = slot;
      }
      if (p.without_replacement && c + 1 < p.n_samples && slot >= 0) {       // uniform
        double rest = 0.0;
#pragma unroll
        for (int r = 0; r < kMaxPer; ++r) {
          const int i = tid * per + r;
          if (r < per && i == slot) pw[r] = 0.0;
          if (r < per && i < count) rest += pw[r];
        }
        p_excl = block_excl_scan_f64<NW>(rest, sh.red, w_total);
      }
    }
  }
}

}  // namespace tslt
