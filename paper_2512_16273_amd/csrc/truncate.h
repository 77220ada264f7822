// tslt_truncate: Top-K / Top-rho truncation of draft logits (Section 3.1) and compaction to the
// sparse (index, logit) payload of Solution 1 (Section 3.2), one workgroup per row.
//
// One pass over the row.  A strided sample of tiles, kept in registers, gives a threshold tau0 that
// a little more than K elements of the whole row are expected to exceed; the pass then does two
// things per 16-byte vector: it adds exp2(z*k2 - c) to the row's fp32 partial sums (the softmax
// normaliser, k2 = log2(e)/T, c a reference taken from the sample maximum), and it copies the
// vector into an LDS buffer if any of its elements is above tau0.  If at least K elements were
// above tau0 the top-K set is among them and is found exactly by sorting those candidates;
// otherwise (ties, masked rows, unlucky sample, overflow of a buffer) the row is redone by an exact
// radix selection that makes several passes.  Either way the kept entries are then evaluated in
// fp64, which is also where Top-rho and the renormalisation are decided.
#pragma once
#include "common.h"
#include "exp64.h"

namespace tslt {

constexpr int kSampleTiles = 8;   // tiles of the row that form the threshold sample

struct TruncateParams {
  const void* logits;
  int64_t rows, V, row_stride;
  float rT;          // fl32(1/T)
  float k2;          // fl32(rT * log2(e))
  float top_p;       // 0 = off
  int k_sel;         // min(top_k (if on), k_cap)
  int k_cap;
  int jprime;        // rank (1-based) among the 256 per-thread sample maxima that gives tau0; 0 = always exact path
  int tau_bits;      // number of leading key bits resolved by the threshold search
  int wave_cap;      // capacity, in vectors, of one wave's hit buffer
  int sort_cap;      // capacity of the candidate array
  int region_a_bytes;  // size of the first dynamic-LDS region (hit buffers / sort scratch), multiple of 16
  int32_t* out_idx;
  float* out_logit;
  float* out_prob;
  int32_t* out_count;
  float* out_mass;
  int32_t* status;
};

struct TruncateShared {
  BlockScratch red;
  uint32_t smax_key[kBlock];   // per-thread maxima of the sample, as keys
  uint32_t hist[256];
  uint32_t cursor[256];
  int wave_count[kWaves];
  int cand_count;
  int bcast_i[4];
  double bcast_d[2];
};

// ---------------------------------------------------------------------------------------------
// Exact multi-pass selection: the k_eff largest elements of the row in the canonical order, found
// by a 4x8-bit radix search for the k-th largest key and an index-ordered collection of the ties.
// Also recomputes the fp32 sum with the true maximum as reference.  Returns the number of
// candidates written to cand[] (exactly k_eff), or 0 with `st` set.
// ---------------------------------------------------------------------------------------------
template <typename T>
__device__ int exact_select(const void* row, int64_t V, int k_sel, float k2, uint64_t* cand,
                            TruncateShared& sh, float& c_ref, double& z_c, int& st) {
  const int tid = threadIdx.x;
  // pass 1: validity, number of selectable elements, maximum
  int fin = 0, bad = 0;
  float vmax = -INFINITY;
  for (int64_t i = tid; i < V; i += kBlock) {
    float v = load_elem<T>(row, i);
    if (v != v || v == INFINITY) bad = 1;
    else if (v > -INFINITY) { ++fin; vmax = fmaxf(vmax, v); }
  }
  bad = block_sum_i32<kWaves>(bad, sh.red);
  fin = block_sum_i32<kWaves>(fin, sh.red);
  vmax = block_max_f32<kWaves>(vmax, sh.red);
  if (bad) { st |= 1; return 0; }
  if (fin == 0) { st |= 2; return 0; }
  const int k_eff = k_sel < fin ? k_sel : fin;

  // radix search, most significant digit first, over keys of elements > -inf
  uint32_t prefix = 0;
  int need = k_eff;
  for (int shift = 24; shift >= 0; shift -= 8) {
    sh.hist[tid] = 0;
    __syncthreads();
    const uint32_t hi_mask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
    for (int64_t i = tid; i < V; i += kBlock) {
      float v = load_elem<T>(row, i);
      uint32_t key = mono_key(v + 0.0f);
      if (v > -INFINITY && (key & hi_mask) == prefix) atomicAdd(&sh.hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid == 0) {
      int cum = 0, d = 255;
      for (; d > 0; --d) {
        int h = int(sh.hist[d]);
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
  for (int64_t base = 0; base < V; base += int64_t(kBlock) * kChunk) {
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
    int off = block_excl_scan_i32<kWaves>(__popc(eq_mask), sh.red, total);
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
  float acc = 0.0f;
  for (int64_t i = tid; i < V; i += kBlock) acc += fast_exp2(__builtin_fmaf(load_elem<T>(row, i), k2, -c_ref));
  z_c = block_sum_f64<kWaves>(double(acc), sh.red);
  __syncthreads();
  return k_eff;
}

// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kBlock) void truncate_kernel(const TruncateParams p) {
  constexpr int E = ElemTraits<T>::kPerVec;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  __shared__ TruncateShared sh;
  // dynamic LDS: region A holds the hit vectors and their vector indices during the pass and is the
  // sort's scratch afterwards; region B is the candidate array
  uint4* grp_data = reinterpret_cast<uint4*>(dyn_lds);
  uint32_t* grp_vidx = reinterpret_cast<uint32_t*>(grp_data + kWaves * p.wave_cap);
  uint64_t* sort_tmp = reinterpret_cast<uint64_t*>(dyn_lds);
  uint64_t* cand = reinterpret_cast<uint64_t*>(dyn_lds + p.region_a_bytes);

  const int tid = threadIdx.x;
  const int lane = lane_id();
  const int wave = wave_id();
  const int64_t row_i = blockIdx.x;
  const void* row = reinterpret_cast<const char*>(p.logits) + size_t(row_i) * size_t(p.row_stride) * ElemTraits<T>::kBytes;
  const RowSplit rs = split_row<T>(row, p.V);
  const int n_edge = rs.head + rs.tail;
  const int64_t n_tiles = (rs.nvec + kBlock - 1) / kBlock;

  int st = 0;
  int n_cand = 0;
  float c_ref = 0.0f;
  double z_c = 0.0;
  bool fast_ok = p.jprime > 0 && n_tiles > 0;

  if (fast_ok) {
    // ---- sample tiles into registers ------------------------------------------------------
    const int ns = n_tiles < kSampleTiles ? int(n_tiles) : kSampleTiles;
    uint4 smp[kSampleTiles];
    float tmax = -INFINITY;
#pragma unroll
    for (int k = 0; k < kSampleTiles; ++k) {
      smp[k] = neg_inf_vec<T>();
      if (k < ns) {
        int64_t vi = ((int64_t(k) * n_tiles) / ns) * kBlock + tid;
        if (vi < rs.nvec) smp[k] = load_vec_stream(&rs.body[vi]);
      }
    }
#pragma unroll
    for (int k = 0; k < kSampleTiles; ++k) {
      float v[E];
      unpack<T>(smp[k], v);
#pragma unroll
      for (int e = 0; e < E; ++e) tmax = fmaxf(tmax, v[e]);
    }
    sh.smax_key[tid] = mono_key(tmax);
    __syncthreads();
    // ---- tau0: the jprime-th largest of the 256 per-thread sample maxima (every wave redundantly)
    uint32_t kq[kWaves];
#pragma unroll
    for (int q = 0; q < kWaves; ++q) kq[q] = sh.smax_key[lane + 64 * q];
    uint32_t tau_key = 0;
    for (int bit = 31; bit >= 32 - p.tau_bits; --bit) {
      uint32_t trial = tau_key | (1u << bit);
      int cnt = 0;
#pragma unroll
      for (int q = 0; q < kWaves; ++q) cnt += __popcll(ballot(kq[q] >= trial));
      if (cnt >= p.jprime) tau_key = trial;
    }
    uint32_t top_key = kq[0];   // the sample maximum
#pragma unroll
    for (int q = 1; q < kWaves; ++q) top_key = kq[q] > top_key ? kq[q] : top_key;
    top_key = wave_max_u32(top_key);
    const float smax = key_to_f32(top_key);
    const float tau0 = tau_key <= kKeyNegInf ? -INFINITY : key_to_f32(tau_key);
    fast_ok = smax > -INFINITY && smax < INFINITY;   // false for NaN too
    c_ref = __fmul_rn(smax, p.k2);
    const float neg_c = -c_ref;
    const float k2 = p.k2;

    // ---- the pass ---------------------------------------------------------------------------
    float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
    int wave_cnt = 0;
    uint4* my_data = grp_data + wave * p.wave_cap;
    uint32_t* my_vidx = grp_vidx + wave * p.wave_cap;
    const int wave_cap = p.wave_cap;

    auto process = [&](const uint4& w, uint32_t vidx) {
      float v[E];
      unpack<T>(w, v);
      float mx = v[0];
#pragma unroll
      for (int e = 1; e < E; ++e) mx = fmaxf(mx, v[e]);
#pragma unroll
      for (int e = 0; e < E; e += 4) {
        acc0 += fast_exp2(__builtin_fmaf(v[e + 0], k2, neg_c));
        acc1 += fast_exp2(__builtin_fmaf(v[e + 1], k2, neg_c));
        acc2 += fast_exp2(__builtin_fmaf(v[e + 2], k2, neg_c));
        acc3 += fast_exp2(__builtin_fmaf(v[e + 3], k2, neg_c));
      }
      const bool hit = mx > tau0;
      const uint64_t mask = ballot(hit);
      if (mask != 0) {
        const int pos = wave_cnt + lanes_below(mask);
        if (hit && pos < wave_cap) {
          my_data[pos] = w;
          my_vidx[pos] = vidx;
        }
        wave_cnt += __popcll(mask);
      }
    };

    if (fast_ok) {
#pragma unroll
      for (int k = 0; k < kSampleTiles; ++k) {
        if (k < ns) {
          int64_t vi = ((int64_t(k) * n_tiles) / ns) * kBlock + tid;
          process(smp[k], uint32_t(vi));
        }
      }
      constexpr int U = 4;
      int next_k = 0;
      int64_t next_sample = 0;   // tile index of sample tile next_k
      for (int64_t t0 = 0; t0 < n_tiles; t0 += U) {
        uint4 d[U];
        bool use[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int64_t t = t0 + u;
          bool is_sample = false;
          if (next_k < ns && t == next_sample) {
            is_sample = true;
            ++next_k;
            next_sample = next_k < ns ? (int64_t(next_k) * n_tiles) / ns : -1;
          }
          use[u] = t < n_tiles && !is_sample;
          d[u] = neg_inf_vec<T>();
          const int64_t vi = t * kBlock + tid;
          if (use[u] && vi < rs.nvec) d[u] = load_vec_stream(&rs.body[vi]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (use[u]) process(d[u], uint32_t((t0 + u) * kBlock + tid));
        }
      }
      // edge elements (row not 16-byte aligned, or V not a whole number of vectors)
      float edge_v = -INFINITY;
      int64_t edge_i = 0;
      if (tid < n_edge) {
        edge_i = edge_index<T>(rs, tid);
        edge_v = load_elem<T>(row, edge_i);
        acc0 += fast_exp2(__builtin_fmaf(edge_v, k2, neg_c));
      }
      z_c = block_sum_f64<kWaves>(double(acc0) + double(acc1) + double(acc2) + double(acc3), sh.red);
      if (lane == 0) sh.wave_count[wave] = wave_cnt;
      if (tid == 0) sh.cand_count = 0;
      __syncthreads();
      bool overflow = false;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) overflow = overflow || sh.wave_count[w] > wave_cap;
      // ---- expand the hit vectors into candidate records -----------------------------------
      if (!overflow) {
        for (int g = lane; g < wave_cnt; g += 64) {
          float v[E];
          unpack<T>(my_data[g], v);
          const uint32_t base = uint32_t(rs.head) + my_vidx[g] * E;
#pragma unroll
          for (int e = 0; e < E; ++e) {
            if (v[e] > tau0) {
              int pos = atomicAdd(&sh.cand_count, 1);
              if (pos < p.sort_cap) cand[pos] = make_cand(v[e], base + e);
            }
          }
        }
        if (tid < n_edge && edge_v > tau0) {
          int pos = atomicAdd(&sh.cand_count, 1);
          if (pos < p.sort_cap) cand[pos] = make_cand(edge_v, uint32_t(edge_i));
        }
      }
      __syncthreads();
      n_cand = sh.cand_count;
      fast_ok = !overflow && n_cand <= p.sort_cap && n_cand >= p.k_sel && z_c > 0.0 && z_c < INFINITY;
      __syncthreads();
    }
  }

  if (!fast_ok) {
    st |= 256;
    n_cand = exact_select<T>(row, p.V, p.k_sel, p.k2, cand, sh, c_ref, z_c, st);
  }

  // ---- sort the candidates into canonical order ------------------------------------------------
  __syncthreads();
  bucket_sort_desc(cand, n_cand, sort_tmp, cand, p.k_sel, sh.hist, sh.smax_key, sh.cursor, sh.red);
  const int k_eff = n_cand < p.k_sel ? n_cand : p.k_sel;

  // ---- fp64 evaluation of the kept head: Top-rho, renormalisation, outputs -----------------------
  // thread t owns entries [t*per, t*per + per) so that a block scan gives prefix masses in order
  const int per = (k_eff + kBlock - 1) / kBlock;       // 0..4
  constexpr int kMaxPer = 4;
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
  const double excl = block_excl_scan_f64<kWaves>(local, sh.red, head64);
  head32 = block_sum_f64<kWaves>(head32, sh.red);
  // normaliser relative to the row maximum: fp32 tail rescaled to that reference + fp64 head
  double tail = z_c - head32;
  if (tail < 0.0) tail = 0.0;
  const double Z = k_eff > 0 ? tail * exp2(double(c_ref) - double(v0) * double(p.k2)) + head64 : 0.0;

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
    below = block_sum_i32<kWaves>(below, sh.red);
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

  const size_t out0 = size_t(row_i) * size_t(p.k_cap);
#pragma unroll
  for (int r = 0; r < kMaxPer; ++r) {
    const int i = tid * per + r;
    if (r < per && i < k_eff && i < count) {
      p.out_idx[out0 + i] = int32_t(idx[r]);
      p.out_logit[out0 + i] = s32[r];
      if (p.out_prob) p.out_prob[out0 + i] = float(e64[r] / c_sel);
    }
  }
  for (int i = count + tid; i < p.k_cap; i += kBlock) {
    p.out_idx[out0 + i] = -1;
    p.out_logit[out0 + i] = -INFINITY;
    if (p.out_prob) p.out_prob[out0 + i] = 0.0f;
  }
  if (tid == 0) {
    p.out_count[row_i] = count;
    if (p.out_mass) p.out_mass[row_i] = count > 0 ? float(c_sel / Z) : 0.0f;
    if (p.status) p.status[row_i] = st;
  }
}

}  // namespace tslt
