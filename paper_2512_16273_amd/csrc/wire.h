// tslt_pack / tslt_unpack: the wire format of a batch of truncated sets (Section 2.2 fixes its size, K pairs
// of a b_idx-bit token id and a b_prob-bit value per position; the layout is defined here).
//
// The stream of one row, least significant bit first: 16 bits count, then per kept entry, in canonical
// order, b_idx = ceil(log2 V) bits of token id followed by the 16 bits of the value (binary16 or bfloat16).
// Rows are padded with zero bits to whole 32-bit words and concatenated; row_offset[r] is the first word of
// row r, row_offset[rows] the total.  Bit p of a row's stream is bit p % 32 of its word p / 32.
#pragma once
#include <hip/hip_fp16.h>
#include "common.h"

namespace tslt {

constexpr int kPayloadF32 = 0, kPayloadBf16 = 1, kPayloadF16 = 2;    // numbered as tslt_dtype
constexpr int kWireMaxEntryBits = 31 + 16;
constexpr int kWireMaxRowWords = (16 + 1024 * kWireMaxEntryBits + 31) / 32;

// A scaled logit as it travels: rounded to nearest-even to the 16-bit format, clamped to its finite range,
// and returned as the fp32 value the receiver decodes.
__device__ __forceinline__ float round_payload(float x, int payload) {
  if (payload == kPayloadBf16) {
    const float big = 3.3895313892515355e38f;                 // largest finite bfloat16
    x = fminf(fmaxf(x, -big), big);
    uint32_t b = __float_as_uint(x);
    b = (b + 0x7FFFu + ((b >> 16) & 1u)) & 0xFFFF0000u;
    return __uint_as_float(b);
  }
  if (payload == kPayloadF16) {
    x = fminf(fmaxf(x, -65504.0f), 65504.0f);
    return __half2float(__float2half_rn(x));
  }
  return x;
}
__device__ __forceinline__ uint32_t payload_bits16(float x, int payload) {
  x = round_payload(x, payload);
  if (payload == kPayloadF16) return uint32_t(__half_as_ushort(__float2half_rn(x)));
  return __float_as_uint(x) >> 16;
}
__device__ __forceinline__ float payload_from_bits16(uint32_t b, int payload) {
  if (payload == kPayloadF16) return __half2float(__ushort_as_half(static_cast<unsigned short>(b)));
  return __uint_as_float(b << 16);
}

inline int wire_index_bits(int64_t V) {
  int b = 0;
  while ((int64_t(1) << b) < V) ++b;
  return b;
}
inline int64_t wire_row_words(int64_t count, int b_idx) { return (16 + count * (b_idx + 16) + 31) / 32; }

struct WireParams {
  const int32_t* idx;
  const float* logit;
  const int32_t* count;
  int64_t rows;
  int k_cap;
  int b_idx;
  int payload;
  uint32_t* words;
  int64_t* row_offset;
  // unpack
  const uint32_t* in_words;
  const int64_t* in_row_offset;
  int32_t* out_idx;
  float* out_logit;
  int32_t* out_count;
};

__device__ __forceinline__ int wire_clamped_count(int c, int k_cap) { return c < 0 ? 0 : (c > k_cap ? k_cap : c); }

// row_offset[r] = words of rows 0..r-1: one workgroup of 1024 threads scans the rows in chunks.
__global__ __launch_bounds__(1024) void wire_offsets_kernel(const WireParams p) {
  __shared__ long long wave_tot[16];
  __shared__ long long base_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) base_s = 0;
  __syncthreads();
  for (int64_t r0 = 0; r0 < p.rows; r0 += 1024) {
    const int64_t r = r0 + tid;
    long long mine = 0;
    if (r < p.rows) mine = (16 + (long long)wire_clamped_count(p.count[r], p.k_cap) * (p.b_idx + 16) + 31) / 32;
    long long inc = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const long long up = __shfl_up(inc, d, 64);
      if (lane >= d) inc += up;
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    long long before = base_s;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    if (r < p.rows) p.row_offset[r] = before + inc - mine;
    __syncthreads();
    if (tid == 1023) base_s = before + inc;
    __syncthreads();
  }
  if (tid == 0) p.row_offset[p.rows] = base_s;
}

// One wave per row: the row's stream is assembled in LDS (entries never share a bit, so OR-ing their pieces
// into the words is order-free) and copied out.
__global__ __launch_bounds__(64) void wire_pack_kernel(const WireParams p) {
  __shared__ uint32_t buf[kWireMaxRowWords];
  const int64_t r = blockIdx.x;
  const int lane = threadIdx.x;
  const int c = wire_clamped_count(p.count[r], p.k_cap);
  const int E = p.b_idx + 16;
  const int n_words = int((16 + (long long)c * E + 31) / 32);
  for (int w = lane; w < n_words; w += 64) buf[w] = 0;
  __syncthreads();
  if (lane == 0) buf[0] = uint32_t(c);
  __syncthreads();
  const int32_t* ix = p.idx + size_t(r) * p.k_cap;
  const float* lg = p.logit + size_t(r) * p.k_cap;
  for (int i = lane; i < c; i += 64) {
    const uint64_t entry = (uint64_t(uint32_t(ix[i])) & ((uint64_t(1) << p.b_idx) - 1)) |
                           (uint64_t(payload_bits16(lg[i], p.payload)) << p.b_idx);
    const long long bit = 16 + (long long)i * E;
    const int w = int(bit >> 5), sh = int(bit & 31);
    atomicOr(&buf[w], uint32_t(entry << sh));
    const uint64_t rest = sh ? (entry >> (32 - sh)) : (entry >> 16 >> 16);
    if (uint32_t(rest) != 0u) atomicOr(&buf[w + 1], uint32_t(rest));
    if ((rest >> 32) != 0u) atomicOr(&buf[w + 2], uint32_t(rest >> 32));
  }
  __syncthreads();
  uint32_t* out = p.words + p.row_offset[r];
  for (int w = lane; w < n_words; w += 64) out[w] = buf[w];
}

__global__ __launch_bounds__(64) void wire_unpack_kernel(const WireParams p) {
  const int64_t r = blockIdx.x;
  const int lane = threadIdx.x;
  const uint32_t* in = p.in_words + p.in_row_offset[r];
  const int64_t n_words = p.in_row_offset[r + 1] - p.in_row_offset[r];
  const int E = p.b_idx + 16;
  int c = n_words > 0 ? int(in[0] & 0xFFFFu) : 0;
  // a count that its row's words cannot hold is cut to what they do hold
  const long long fits = n_words > 0 ? (n_words * 32 - 16) / E : 0;
  if (c > fits) c = int(fits);
  c = wire_clamped_count(c, p.k_cap);
  int32_t* ix = p.out_idx + size_t(r) * p.k_cap;
  float* lg = p.out_logit + size_t(r) * p.k_cap;
  for (int i = lane; i < p.k_cap; i += 64) {
    int id = -1;
    float v = -INFINITY;
    if (i < c) {
      const long long bit = 16 + (long long)i * E;
      const int64_t w = bit >> 5;
      const int sh = int(bit & 31);
      uint64_t lo = uint64_t(in[w]) | (w + 1 < n_words ? uint64_t(in[w + 1]) << 32 : 0);
      uint64_t entry = lo >> sh;
      if (sh + E > 64 && w + 2 < n_words) entry |= uint64_t(in[w + 2]) << (64 - sh);
      entry &= (uint64_t(1) << E) - 1;
      id = int(entry & ((uint64_t(1) << p.b_idx) - 1));
      v = payload_from_bits16(uint32_t(entry >> p.b_idx) & 0xFFFFu, p.payload);
    }
    ix[i] = id;
    lg[i] = v;
  }
  if (lane == 0) p.out_count[r] = c;
}

}  // namespace tslt
