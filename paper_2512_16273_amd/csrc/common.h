// Device-side helpers shared by the TSLT kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace tslt {

// ---- host side: what is looked up or set once per device, so that a call after the first on a device is
// nothing but argument checks and launches ----------------------------------------------------------------
constexpr int kMaxDevices = 64;
inline int current_device_slot() {
  int d = 0;
  if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= kMaxDevices) d = 0;
  return d;
}
// Lets `Kernel` be launched with up to `bytes` of dynamic LDS on the current device (needed above 48 KB).
template <auto Kernel> inline hipError_t allow_dynamic_lds(int bytes) {
  static std::atomic<int> granted[kMaxDevices];
  const int d = current_device_slot();
  if (granted[d].load(std::memory_order_relaxed) >= bytes) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) granted[d].store(bytes, std::memory_order_relaxed);
  return e;
}
// Compute units of the current device (256 if the query fails).
inline int compute_units() {
  static std::atomic<int> cus[kMaxDevices];
  const int d = current_device_slot();
  int n = cus[d].load(std::memory_order_relaxed);
  if (n > 0) return n;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
    n = 256;
  cus[d].store(n, std::memory_order_relaxed);
  return n;
}

constexpr int kBlock = 256;            // threads per workgroup of the streaming kernels
constexpr int kWaves = kBlock / 64;
constexpr uint32_t kNegInfBits = 0xFF800000u;

struct Bf16 { uint16_t bits; };        // storage tag for bf16 rows
struct F16 { uint16_t bits; };         // storage tag for binary16 rows

template <typename T> struct ElemTraits;
template <> struct ElemTraits<float> {
  static constexpr int kPerVec = 4;    // elements per 16-byte vector
  static constexpr int kBytes = 4;
};
template <> struct ElemTraits<Bf16> {
  static constexpr int kPerVec = 8;
  static constexpr int kBytes = 2;
};
template <> struct ElemTraits<F16> {
  static constexpr int kPerVec = 8;
  static constexpr int kBytes = 2;
};

__device__ __forceinline__ float as_f32(uint32_t b) { return __uint_as_float(b); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __float_as_uint(f); }

// A pointer into device memory, typed as such.  Where the compiler cannot prove that a pointer is global
// it emits flat loads; those also count against the LDS counter, so that every wait for an LDS access
// waits for them too and a kernel that prefetches rows while it works in LDS loses the overlap.
template <typename U> __device__ __forceinline__ const U __attribute__((address_space(1)))* as_global(const U* p) {
  return (const U __attribute__((address_space(1)))*)p;
}

// Element i of a 16-byte vector, widened exactly to fp32.
template <typename T> __device__ __forceinline__ void unpack(const uint4& w, float (&v)[ElemTraits<T>::kPerVec]);
template <> __device__ __forceinline__ void unpack<float>(const uint4& w, float (&v)[4]) {
  v[0] = as_f32(w.x); v[1] = as_f32(w.y); v[2] = as_f32(w.z); v[3] = as_f32(w.w);
}
template <> __device__ __forceinline__ void unpack<Bf16>(const uint4& w, float (&v)[8]) {
  v[0] = as_f32(w.x << 16); v[1] = as_f32(w.x & 0xFFFF0000u);
  v[2] = as_f32(w.y << 16); v[3] = as_f32(w.y & 0xFFFF0000u);
  v[4] = as_f32(w.z << 16); v[5] = as_f32(w.z & 0xFFFF0000u);
  v[6] = as_f32(w.w << 16); v[7] = as_f32(w.w & 0xFFFF0000u);
}

__device__ __forceinline__ float f16_lo(uint32_t w) { return float(__builtin_bit_cast(_Float16, uint16_t(w))); }
__device__ __forceinline__ float f16_hi(uint32_t w) { return float(__builtin_bit_cast(_Float16, uint16_t(w >> 16))); }
template <> __device__ __forceinline__ void unpack<F16>(const uint4& w, float (&v)[8]) {
  v[0] = f16_lo(w.x); v[1] = f16_hi(w.x);
  v[2] = f16_lo(w.y); v[3] = f16_hi(w.y);
  v[4] = f16_lo(w.z); v[5] = f16_hi(w.z);
  v[6] = f16_lo(w.w); v[7] = f16_hi(w.w);
}

template <typename T> __device__ __forceinline__ uint4 neg_inf_vec();
template <> __device__ __forceinline__ uint4 neg_inf_vec<float>() {
  return make_uint4(kNegInfBits, kNegInfBits, kNegInfBits, kNegInfBits);
}
template <> __device__ __forceinline__ uint4 neg_inf_vec<Bf16>() {
  return make_uint4(0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u);
}

template <> __device__ __forceinline__ uint4 neg_inf_vec<F16>() {
  return make_uint4(0xFC00FC00u, 0xFC00FC00u, 0xFC00FC00u, 0xFC00FC00u);
}

// Scalar load of element i of a row, any alignment of the element type.
template <typename T> __device__ __forceinline__ float load_elem(const void* row, int64_t i);
template <> __device__ __forceinline__ float load_elem<float>(const void* row, int64_t i) {
  return as_global(reinterpret_cast<const float*>(row))[i];
}
template <> __device__ __forceinline__ float load_elem<Bf16>(const void* row, int64_t i) {
  return as_f32(uint32_t(as_global(reinterpret_cast<const uint16_t*>(row))[i]) << 16);
}

template <> __device__ __forceinline__ float load_elem<F16>(const void* row, int64_t i) {
  return f16_lo(as_global(reinterpret_cast<const uint16_t*>(row))[i]);
}

// Order-preserving map fp32 -> uint32 (larger value, larger key).  -0.0 must be folded into +0.0 by
// the caller (add 0.0f) when the two have to compare equal.
__device__ __forceinline__ uint32_t mono_key(float v) {
  uint32_t b = as_u32(v);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_to_f32(uint32_t k) {
  return as_f32((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}
constexpr uint32_t kKeyNegInf = 0x007FFFFFu;   // mono_key(-inf)
constexpr uint32_t kKeyPosInf = 0xFF800000u;   // mono_key(+inf)

// Candidate record: value key in the high word, inverted index in the low word, so that a plain
// descending sort of the 64-bit word gives "value descending, index ascending".
__device__ __forceinline__ uint64_t make_cand(float v, uint32_t idx) {
  return (uint64_t(mono_key(v + 0.0f)) << 32) | uint64_t(0xFFFFFFFFu - idx);
}
__device__ __forceinline__ float cand_value(uint64_t c) { return key_to_f32(uint32_t(c >> 32)); }
__device__ __forceinline__ uint32_t cand_index(uint64_t c) { return 0xFFFFFFFFu - uint32_t(c); }

// 16-byte streaming load (read-once data: do not keep it in the caches longer than needed).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_vec_stream(const uint4* p) {
  u32x4_t r = __builtin_nontemporal_load(as_global(reinterpret_cast<const u32x4_t*>(p)));
  return make_uint4(r.x, r.y, r.z, r.w);
}
__device__ __forceinline__ uint4 load_vec(const uint4* p) {
  u32x4_t r = *as_global(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(r.x, r.y, r.z, r.w);
}

// A row's aligned body as a buffer: 16-byte loads through a resource descriptor take the row's base and size
// from scalar registers, a per-thread byte offset that never changes (lane * 16) from a vector register and
// the moving part of the address from a scalar one, so that a streaming loop spends no vector instruction on
// addresses; a load that reaches past the body's end returns zeros instead of faulting (the hardware checks
// the range), and the loops give such vectors the value they need afterwards.  The body must be below 4 GiB.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_buffer(const uint4* body, uint32_t nvec) {
  // (third dword: raw buffer of 32-bit data, the setting of the GFX9 family)
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4*>(body), 0, int(nvec * 16u), 0x00020000);
}
__device__ __forceinline__ uint4 buffer_load_vec_stream(__amdgpu_buffer_rsrc_t r, uint32_t lane_bytes, uint32_t wave_bytes) {
  u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, int(lane_bytes), int(wave_bytes), 2);      // 2: nontemporal
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 buffer_load_vec(__amdgpu_buffer_rsrc_t r, uint32_t lane_bytes, uint32_t wave_bytes) {
  u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, int(lane_bytes), int(wave_bytes), 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// max of three without the NaN-quieting moves the compiler adds around fmaxf (NaNs are found by other means)
__device__ __forceinline__ float max3f(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

__device__ __forceinline__ uint64_t ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }
__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi(uint32_t(mask >> 32), __builtin_amdgcn_mbcnt_lo(uint32_t(mask), 0));
}

__device__ __forceinline__ double shfl_f64(double v, int src) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl(lo, src, 64); hi = __shfl(hi, src, 64);
  return __hiloint2double(hi, lo);
}

// Cross-lane moves on the VALU's data-parallel-primitive path (no LDS round trip).  A lane whose source lies
// outside its row of 16, or that the row / bank mask leaves out, gets `old`.  Controls used here:
// row_shr:n = 0x110 + n (lane i reads lane i - n of its row), row_bcast:15 = 0x142 (lane 15 of every row to
// the whole next row), row_bcast:31 = 0x143 (lane 31 to rows 2 and 3).
template <int CTRL, int ROW_MASK = 0xF, int BANK_MASK = 0xF>
__device__ __forceinline__ int dpp_i32(int old, int v) {
  return __builtin_amdgcn_update_dpp(old, v, CTRL, ROW_MASK, BANK_MASK, false);
}
template <int CTRL, int ROW_MASK = 0xF, int BANK_MASK = 0xF>
__device__ __forceinline__ double dpp_f64(double old, double v) {
  const int lo = dpp_i32<CTRL, ROW_MASK, BANK_MASK>(__double2loint(old), __double2loint(v));
  const int hi = dpp_i32<CTRL, ROW_MASK, BANK_MASK>(__double2hiint(old), __double2hiint(v));
  return __hiloint2double(hi, lo);
}
// Inclusive scan over the 64 lanes of a wave with an associative operation `op` whose identity is `id`:
// four steps inside every row of 16, then the row totals are carried into the later rows.  Lane 63 ends up
// with the reduction over the wave.
template <typename Op> __device__ __forceinline__ int wave_scan_i32(int v, int id, Op op) {
  v = op(v, dpp_i32<0x111>(id, v));
  v = op(v, dpp_i32<0x112>(id, v));
  v = op(v, dpp_i32<0x114>(id, v));
  v = op(v, dpp_i32<0x118>(id, v));
  v = op(v, dpp_i32<0x142, 0xA>(id, v));
  v = op(v, dpp_i32<0x143, 0xC>(id, v));
  return v;
}
template <typename Op> __device__ __forceinline__ double wave_scan_f64(double v, double id, Op op) {
  v = op(v, dpp_f64<0x111>(id, v));
  v = op(v, dpp_f64<0x112>(id, v));
  v = op(v, dpp_f64<0x114>(id, v));
  v = op(v, dpp_f64<0x118>(id, v));
  v = op(v, dpp_f64<0x142, 0xA>(id, v));
  v = op(v, dpp_f64<0x143, 0xC>(id, v));
  return v;
}
__device__ __forceinline__ int last_lane_i32(int v) { return __builtin_amdgcn_readlane(v, 63); }
__device__ __forceinline__ double last_lane_f64(double v) {
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 63), __builtin_amdgcn_readlane(__double2loint(v), 63));
}

__device__ __forceinline__ int wave_incl_scan_i32(int v) { return wave_scan_i32(v, 0, [](int a, int b) { return a + b; }); }
__device__ __forceinline__ double wave_incl_scan_f64(double v) {
  return wave_scan_f64(v, 0.0, [](double a, double b) { return a + b; });
}
// Reductions over a wave; every lane gets the result.
__device__ __forceinline__ double wave_sum_f64(double v) { return last_lane_f64(wave_incl_scan_f64(v)); }
__device__ __forceinline__ int wave_sum_i32(int v) { return last_lane_i32(wave_incl_scan_i32(v)); }
__device__ __forceinline__ float wave_max_f32(float v) {
  // on the bit patterns: the maximum of NaN-free floats through fmaxf, carried as ints by the moves
  const int r = wave_scan_i32(__float_as_int(v), __float_as_int(-INFINITY),
                              [](int a, int b) { return __float_as_int(fmaxf(__int_as_float(a), __int_as_float(b))); });
  return __int_as_float(last_lane_i32(r));
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  return uint32_t(last_lane_i32(wave_scan_i32(int(v), 0, [](int a, int b) { return int(uint32_t(a) > uint32_t(b) ? uint32_t(a) : uint32_t(b)); })));
}
__device__ __forceinline__ int wave_max_i32(int v) {
  return last_lane_i32(wave_scan_i32(v, int(0x80000000), [](int a, int b) { return a > b ? a : b; }));
}
__device__ __forceinline__ int wave_or_i32(int v) { return last_lane_i32(wave_scan_i32(v, 0, [](int a, int b) { return a | b; })); }

// Small per-block scratch for reductions and scans; one instance lives in static LDS.
// `NW` is the number of waves of the workgroup that calls the helpers.
struct BlockScratch {
  double d[16];
  float f[16];
  int i[16];
};

// Block-wide reductions.  Every thread of the block must call; the result is returned to all.
template <int NW> __device__ __forceinline__ double block_sum_f64(double v, BlockScratch& s) {
  v = wave_sum_f64(v);
  __syncthreads();
  if (lane_id() == 0) s.d[wave_id()] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int w = 0; w < NW; ++w) t += s.d[w];
  return t;
}
template <int NW> __device__ __forceinline__ float block_max_f32(float v, BlockScratch& s) {
  v = wave_max_f32(v);
  __syncthreads();
  if (lane_id() == 0) s.f[wave_id()] = v;
  __syncthreads();
  float t = s.f[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) t = fmaxf(t, s.f[w]);
  return t;
}
template <int NW> __device__ __forceinline__ int block_sum_i32(int v, BlockScratch& s) {
  v = wave_sum_i32(v);
  __syncthreads();
  if (lane_id() == 0) s.i[wave_id()] = v;
  __syncthreads();
  int t = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) t += s.i[w];
  return t;
}

template <int NW> __device__ __forceinline__ int block_max_i32(int v, BlockScratch& s) {
  v = wave_max_i32(v);
  __syncthreads();
  if (lane_id() == 0) s.i[wave_id()] = v;
  __syncthreads();
  int t = s.i[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) t = s.i[w] > t ? s.i[w] : t;
  return t;
}

template <int NW> __device__ __forceinline__ int block_or_i32(int v, BlockScratch& s) {
  v = wave_or_i32(v);
  __syncthreads();
  if (lane_id() == 0) s.i[wave_id()] = v;
  __syncthreads();
  int t = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) t |= s.i[w];
  return t;
}

// Block-wide exclusive scans in thread order; `total` receives the sum over the block.
template <int NW> __device__ __forceinline__ double block_excl_scan_f64(double v, BlockScratch& s, double& total) {
  const double inc = wave_incl_scan_f64(v);
  __syncthreads();
  if (lane_id() == 63) s.d[wave_id()] = inc;
  __syncthreads();
  double base = 0.0, t = 0.0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    if (w < wave_id()) base += s.d[w];
    t += s.d[w];
  }
  total = t;
  return base + inc - v;
}
template <int NW> __device__ __forceinline__ int block_excl_scan_i32(int v, BlockScratch& s, int& total) {
  const int inc = wave_incl_scan_i32(v);
  __syncthreads();
  if (lane_id() == 63) s.i[wave_id()] = inc;
  __syncthreads();
  int base = 0, t = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    if (w < wave_id()) base += s.i[w];
    t += s.i[w];
  }
  total = t;
  return base + inc - v;
}

// Sort of n candidate records held in LDS, descending, by a 256-bin counting sort on the value
// (bins divide the interval [min, max] of the values present evenly; any monotone binning keeps the
// result exact) followed by an exact rank inside each bin.  The largest min(n, k_keep) records end up
// in out[0..) in order.  Only the bins that can reach the first k_keep places are moved: `tmp` needs
// room for k_keep records plus the population of the bin that straddles that boundary; the function
// returns false, leaving `in` intact, when tmp_cap is too small for that.  `in` and `out` may be the
// same array; `tmp` must be distinct from both.  hist, start and cursor are 256-entry LDS arrays.
// Work per thread is about n/256 + k_keep/256 * mean bin population; values crowded into one bin cost
// more, bounded by n^2/256 comparisons per thread.  NT = threads of the workgroup (64, 128 or 256).
__device__ __forceinline__ int value_bin(uint64_t c, float vmin, float scale) {
  // fp32 subtraction and multiplication are monotone, which is all the binning has to be
  const int b = int((cand_value(c) - vmin) * scale);
  return b > 255 ? 255 : (b < 0 ? 0 : b);
}
template <int NT>
__device__ __forceinline__ bool bucket_sort_desc(const uint64_t* in, int n, uint64_t* tmp, int tmp_cap, uint64_t* out,
                                                 int k_keep, uint32_t* hist, uint32_t* start, uint32_t* cursor,
                                                 BlockScratch& red) {
  constexpr int NW = NT / 64;
  constexpr int BPT = 256 / NT;      // bins per thread: thread t owns bins 255 - t*BPT - j, j < BPT
  if (n <= 0) return true;
  const int tid = threadIdx.x;
  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
  for (int i = tid; i < n; i += NT) {
    const uint32_t k = uint32_t(in[i] >> 32);
    kmin = k < kmin ? k : kmin;
    kmax = k > kmax ? k : kmax;
  }
  kmax = wave_max_u32(kmax);
  kmin = ~wave_max_u32(~kmin);
  for (int b = tid; b < 256; b += NT) hist[b] = 0;
  if (lane_id() == 0) { red.i[wave_id()] = int(kmin); red.i[8 + wave_id()] = int(kmax); }
  __syncthreads();
  kmin = uint32_t(red.i[0]); kmax = uint32_t(red.i[8]);
#pragma unroll
  for (int w = 1; w < NW; ++w) {
    kmin = uint32_t(red.i[w]) < kmin ? uint32_t(red.i[w]) : kmin;
    kmax = uint32_t(red.i[8 + w]) > kmax ? uint32_t(red.i[8 + w]) : kmax;
  }
  const float vmin = key_to_f32(kmin);
  const float span = key_to_f32(kmax) - vmin;            // may overflow to +inf: then one bin
  const float scale = (span > 0.0f && span < 3.0e38f) ? 255.0f / span : 0.0f;
  for (int i = tid; i < n; i += NT) atomicAdd(&hist[value_bin(in[i], vmin, scale)], 1u);
  __syncthreads();
  int total;
  int h[BPT], mine = 0;
#pragma unroll
  for (int j = 0; j < BPT; ++j) { h[j] = int(hist[255 - tid * BPT - j]); mine += h[j]; }
  const int excl = block_excl_scan_i32<NW>(mine, red, total);   // bins in descending order
  int run = excl, moved = 0;
#pragma unroll
  for (int j = 0; j < BPT; ++j) {
    start[255 - tid * BPT - j] = uint32_t(run);
    cursor[255 - tid * BPT - j] = uint32_t(run);
    if (run < k_keep) moved += h[j];      // records in the bins that start before place k_keep
    run += h[j];
  }
  const int n_moved = block_sum_i32<NW>(moved, red);
  if (n_moved > tmp_cap) return false;
  __syncthreads();
  for (int i = tid; i < n; i += NT) {
    const uint64_t c = in[i];
    const int b = value_bin(c, vmin, scale);
    if (int(start[b]) < k_keep) tmp[atomicAdd(&cursor[b], 1u)] = c;
  }
  __syncthreads();
  for (int i = tid; i < n_moved; i += NT) {
    const uint64_t c = tmp[i];
    const int b = value_bin(c, vmin, scale);
    const int s0 = int(start[b]);
    const int s1 = s0 + int(hist[b]);
    int r = 0;
    for (int j = s0; j < s1; ++j) r += tmp[j] > c ? 1 : 0;
    if (s0 + r < k_keep) out[s0 + r] = c;
  }
  __syncthreads();
  return true;
}

// How a row of V elements splits into a 16-byte aligned body of whole vectors plus at most
// 2*(kPerVec-1) edge elements in front of and behind it.
struct RowSplit {
  int head;        // elements before the aligned body
  int64_t nvec;    // whole 16-byte vectors in the body
  int tail;        // elements after the body
  const uint4* body;
};
template <typename T> __device__ __forceinline__ RowSplit split_row(const void* row, int64_t V) {
  constexpr int E = ElemTraits<T>::kPerVec;
  RowSplit r;
  uintptr_t a = reinterpret_cast<uintptr_t>(row);
  int mis = int((a & 15u) / ElemTraits<T>::kBytes);
  int head = mis ? (E - mis) : 0;
  if (head > V) head = int(V);
  r.head = head;
  r.nvec = (V - head) / E;
  r.tail = int(V - head - r.nvec * E);
  r.body = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(row) + size_t(head) * ElemTraits<T>::kBytes);
  return r;
}
// Index (within the row) and value of edge element e in 0 .. head+tail-1.
template <typename T> __device__ __forceinline__ int64_t edge_index(const RowSplit& r, int e) {
  return e < r.head ? int64_t(e) : int64_t(r.head) + r.nvec * ElemTraits<T>::kPerVec + (e - r.head);
}

}  // namespace tslt
