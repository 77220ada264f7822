// C ABI of the TSLT hot path (see include/tslt.h): argument checks, launch plans, kernel launches.
#include "tslt.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <string>

#include "common.h"
#include "sample.h"
#include "truncate.h"
#include "wire.h"
#include "tree.h"
#include "verify.h"
#include "stats.h"
#include "calib.h"

// Scratch memory of tslt_verify_static: the per-position decisions and status words that tslt_verify keeps in
// its caller's workspace.  Every GPU the library runs on holds its own copy until the process ends.  In host
// code the name is only a handle for hipGetSymbolAddress; kernels are given the address that call returns.
#define TSLT_STATIC_SCRATCH_BYTES (2 * 4 * TSLT_STATIC_MAX_POSITIONS)
static __device__ __align__(256) unsigned char scratch[TSLT_STATIC_SCRATCH_BYTES];

namespace {

thread_local std::string g_last_error;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return code;
}

int hip_fail(hipError_t e, const char* what) {
  return fail(TSLT_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool valid_dtype(tslt_dtype dt) { return dt == TSLT_F32 || dt == TSLT_BF16 || dt == TSLT_F16; }
int elem_bytes(tslt_dtype dt) { return dt == TSLT_F32 ? 4 : 2; }
// a row is addressed with 32-bit byte offsets from its start
bool row_too_long(int64_t V, tslt_dtype dt) { return V > 0x7FFFFFFF || V * elem_bytes(dt) >= (int64_t(1) << 32); }

// fl32(1/T), the one scaling constant every side derives the same way
float reciprocal_temperature(float T) { return float(1.0 / double(T)); }
float log2e_over_T(float rT) { return float(double(rT) * 1.4426950408889634074); }

constexpr size_t kMaxLds = 160 * 1024;   // LDS of one gfx950 compute unit

// Launch plan of the truncate kernel: which rank among the per-thread sample maxima gives the
// threshold, and how large the candidate array has to be.  Returns the bytes of dynamic LDS.
size_t plan_truncate(tslt_dtype dt, int64_t V, int nt, tslt::TruncateParams& p) {
  const int E = 16 / elem_bytes(dt);
  const double G = nt;                                 // per-thread sample maxima
  const int64_t tile = int64_t(nt) * E;
  const int64_t n_tiles = (V + tile - 1) / tile;
  const int64_t ns = n_tiles < tslt::kBatch ? n_tiles : tslt::kBatch;
  const double n_sample = double(ns * tile < V ? ns * tile : V);
  const double f = n_sample / double(V);               // fraction of the row in the sample
  const double kp = p.k_sel * f;                       // expected sample elements inside the top-k
  const double j = f >= 1.0 ? kp + 1.0 : kp + 4.0 * std::sqrt(kp) + 4.0;
  const double jc = G * (1.0 - std::exp(-j / G));      // distinct threads holding the top j
  const int jprime = int(std::ceil(jc + 2.0 * std::sqrt(j > jc ? j - jc : 0.0) + 1.0));
  // every bf16 value is told apart by the leading 16 bits of its fp32 key, every binary16 value (11
  // significant bits) by the leading 19
  p.tau_bits = dt == TSLT_BF16 ? 16 : (dt == TSLT_F16 ? 19 : 20);
  p.jprime = 0;
  // candidate capacity: always room for the fallback's 1024 group maxima and for 2 * k_sel records.
  // The sort needs about 1.5 * k_sel records of scratch: the ring space behind the sort's tables if
  // that is large enough, else extra records behind the candidates.
  const int min_cap = (1024 + 16 > 2 * p.k_sel) ? 1024 + 16 : 2 * p.k_sel;
  const int scratch = tslt::truncate_sort_scratch(p.k_sel);
  p.ring_bytes = tslt::ring_bytes_for(nt / 64);
  p.tmp_in_ring = (p.ring_bytes - 3 * 256 * 4) / 8 >= scratch ? 1 : 0;
  const int extra = p.tmp_in_ring ? 0 : scratch;
  p.sort_cap = min_cap;
  p.lds_recs = min_cap + extra;
  if (jprime <= int(0.8 * G)) {
    const double j_eff = -G * std::log(1.0 - double(jprime) / G);
    int sort_cap = int((j_eff + 5.0 * std::sqrt(j_eff) + 4.0) / f) + 16;   // mean + 5 sigma of the hits
    if (sort_cap < min_cap) sort_cap = min_cap;
    if (tslt::truncate_lds_bytes(p.ring_bytes, sort_cap + extra) + sizeof(tslt::TruncateShared) + 256 <= kMaxLds) {
      p.jprime = jprime;
      p.sort_cap = sort_cap;
      p.lds_recs = sort_cap + extra;
    }
  }
  return tslt::truncate_lds_bytes(p.ring_bytes, p.lds_recs);
}

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
hipError_t scratch_on_current_device(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (ptr == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

constexpr int kLargeLds = int(kMaxLds - 4096);

// The two shapes of the truncation kernel for one element type (see truncate.h).
template <typename T, int NT, bool kWide> struct TruncKernel {
  static constexpr auto fn = kWide ? &tslt::truncate_kernel<T, NT, tslt::kStagesWide, tslt::kWavesWide>
                                   : &tslt::truncate_kernel<T, NT, tslt::kStagesDeep, tslt::kWavesDeep>;
  hipError_t allow(int bytes) const { return tslt::allow_dynamic_lds<fn>(bytes); }
};

}  // namespace

extern "C" {

int tslt_version(void) { return 100; }

const char* tslt_last_error(void) { return g_last_error.c_str(); }

size_t tslt_workspace_bytes(int op, int64_t n_outer, int64_t n_inner, int64_t V, int32_t k_cap) {
  if (n_outer <= 0 || V <= 0) return 0;
  switch (op) {
    case TSLT_OP_VERIFY:
      return tslt::verify_workspace_bytes(n_outer, n_inner, V, k_cap);
    case TSLT_OP_VERIFY_TREE:
      return n_inner > 0 ? tslt::tree_workspace_bytes(n_outer, n_inner, V, true) : 0;
    case TSLT_OP_VERIFY_TREE_PATH:
      return n_inner > 0 ? tslt::tree_workspace_bytes(n_outer, n_inner, V, false) : 0;
    default:
      return 0;
  }
}

// tslt_truncate and tslt_truncate_sample: the second also draws from q_hat in the same launch.
static int truncate_impl(const void* logits, tslt_dtype dt, int64_t rows, int64_t V, int64_t row_stride,
                         float temperature, int32_t top_k, float top_p, int32_t k_cap, tslt_dtype payload, int32_t* out_idx,
                         float* out_logit, float* out_prob, int32_t* out_count, float* out_mass, int32_t* status,
                         const float* u, int32_t n_samples, int32_t without_replacement, int32_t* out_token, int32_t* out_slot,
                         void* ws, size_t ws_bytes, void* stream) {
  if (!valid_dtype(dt)) return fail(TSLT_ERR_INVALID_ARG, "tslt_truncate: unknown dtype %d", int(dt));
  if (rows < 0 || V <= 0 || row_stride < V) return fail(TSLT_ERR_INVALID_ARG, "tslt_truncate: bad shape rows=%lld V=%lld stride=%lld", (long long)rows, (long long)V, (long long)row_stride);
  if (row_too_long(V, dt) || rows > 0x7FFFFFFF) return fail(TSLT_ERR_UNSUPPORTED, "tslt_truncate: rows must fit 31 bits, a row 4 GiB");
  if (!(temperature > 0.0f) || !std::isfinite(temperature)) return fail(TSLT_ERR_INVALID_ARG, "tslt_truncate: temperature must be > 0");
  if (k_cap < 1 || k_cap > TSLT_MAX_K_CAP) return fail(TSLT_ERR_UNSUPPORTED, "tslt_truncate: k_cap must be in 1..%d", TSLT_MAX_K_CAP);
  if (top_k < 0 || !(top_p >= 0.0f)) return fail(TSLT_ERR_INVALID_ARG, "tslt_truncate: top_k and top_p must be >= 0");
  if (payload != TSLT_F32 && payload != TSLT_BF16 && payload != TSLT_F16) return fail(TSLT_ERR_INVALID_ARG, "tslt_truncate: unknown payload format %d", int(payload));
  if (rows == 0) return TSLT_OK;
  if (!logits || !out_idx || !out_logit || !out_count) return fail(TSLT_ERR_INVALID_ARG, "tslt_truncate: null pointer");
  if (reinterpret_cast<uintptr_t>(logits) % elem_bytes(dt)) return fail(TSLT_ERR_INVALID_ARG, "tslt_truncate: logits not aligned to their element type");

  tslt::TruncateParams p{};
  p.logits = logits; p.rows = rows; p.V = V; p.row_stride = row_stride;
  p.rT = reciprocal_temperature(temperature);
  p.k2 = log2e_over_T(p.rT);
  p.top_p = (top_p > 0.0f && top_p < 1.0f) ? top_p : 0.0f;
  p.k_cap = k_cap;
  p.payload = int(payload);
  p.k_sel = (top_k > 0 && top_k < k_cap) ? top_k : k_cap;
  p.out_idx = out_idx; p.out_logit = out_logit; p.out_prob = out_prob; p.out_count = out_count;
  p.out_mass = out_mass; p.status = status;
  p.u = u; p.n_samples = n_samples; p.without_replacement = without_replacement ? 1 : 0;
  p.out_token = out_token; p.out_slot = out_slot;
  constexpr int NT = tslt::kTruncThreads;
  const size_t lds = plan_truncate(dt, V, NT, p);

  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  hipError_t e;
  const bool big_lds = lds + sizeof(tslt::TruncateShared) > 48 * 1024;
  (void)ws; (void)ws_bytes;
  const dim3 grid{unsigned(rows)}, block{unsigned(NT)};
  // eight workgroups of this footprint on a compute unit: the wide shape; else the deep one
  const bool wide = 8 * (lds + sizeof(tslt::TruncateShared) + 256) <= kMaxLds;
  auto launch = [&](auto kernel_wide, auto kernel_deep) -> hipError_t {
    if (wide) {
      hipLaunchKernelGGL(kernel_wide.fn, grid, block, lds, s, p);
      return hipSuccess;
    }
    if (big_lds) {
      const hipError_t err = kernel_deep.allow(kLargeLds);
      if (err != hipSuccess) return err;
    }
    hipLaunchKernelGGL(kernel_deep.fn, grid, block, lds, s, p);
    return hipSuccess;
  };
  if (dt == TSLT_BF16) e = launch(TruncKernel<tslt::Bf16, NT, true>{}, TruncKernel<tslt::Bf16, NT, false>{});
  else if (dt == TSLT_F16) e = launch(TruncKernel<tslt::F16, NT, true>{}, TruncKernel<tslt::F16, NT, false>{});
  else e = launch(TruncKernel<float, NT, true>{}, TruncKernel<float, NT, false>{});
  if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute");
  if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "tslt_truncate launch");
  return TSLT_OK;
}

int tslt_truncate(const void* logits, tslt_dtype dt, int64_t rows, int64_t V, int64_t row_stride,
                  float temperature, int32_t top_k, float top_p, int32_t k_cap, tslt_dtype payload, int32_t* out_idx,
                  float* out_logit, float* out_prob, int32_t* out_count, float* out_mass, int32_t* status,
                  void* ws, size_t ws_bytes, void* stream) {
  return truncate_impl(logits, dt, rows, V, row_stride, temperature, top_k, top_p, k_cap, payload, out_idx, out_logit, out_prob,
                       out_count, out_mass, status, nullptr, 0, 0, nullptr, nullptr, ws, ws_bytes, stream);
}

int tslt_truncate_sample(const void* logits, tslt_dtype dt, int64_t rows, int64_t V, int64_t row_stride,
                         float temperature, int32_t top_k, float top_p, int32_t k_cap, tslt_dtype payload, int32_t* out_idx,
                         float* out_logit, float* out_prob, int32_t* out_count, float* out_mass, int32_t* status,
                         const float* u, int32_t n_samples, int32_t without_replacement, int32_t* out_token, int32_t* out_slot,
                         void* ws, size_t ws_bytes, void* stream) {
  if (n_samples < 1 || n_samples > TSLT_MAX_BRANCH)
    return fail(TSLT_ERR_INVALID_ARG, "tslt_truncate_sample: n_samples must be in 1..%d", TSLT_MAX_BRANCH);
  if (rows > 0 && (!u || !out_token)) return fail(TSLT_ERR_INVALID_ARG, "tslt_truncate_sample: null pointer");
  return truncate_impl(logits, dt, rows, V, row_stride, temperature, top_k, top_p, k_cap, payload, out_idx, out_logit, out_prob,
                       out_count, out_mass, status, u, n_samples, without_replacement, out_token, out_slot, ws, ws_bytes, stream);
}

int64_t tslt_pack_bound_words(int64_t rows, int32_t k_cap, int64_t V) {
  if (rows <= 0 || k_cap < 1 || k_cap > TSLT_MAX_K_CAP || V < 1 || V > 0x7FFFFFFF) return 0;
  return rows * tslt::wire_row_words(k_cap, tslt::wire_index_bits(V));
}

int tslt_pack(const int32_t* idx, const float* logit, const int32_t* count, int64_t rows, int32_t k_cap, int64_t V,
              tslt_dtype payload, uint32_t* out_words, int64_t out_capacity_words, int64_t* out_row_offset,
              void* stream) {
  if (rows < 0 || V < 1 || V > 0x7FFFFFFF) return fail(TSLT_ERR_INVALID_ARG, "tslt_pack: bad shape");
  if (k_cap < 1 || k_cap > TSLT_MAX_K_CAP) return fail(TSLT_ERR_UNSUPPORTED, "tslt_pack: k_cap must be in 1..%d", TSLT_MAX_K_CAP);
  if (payload != TSLT_BF16 && payload != TSLT_F16) return fail(TSLT_ERR_INVALID_ARG, "tslt_pack: the value format must be bfloat16 or binary16");
  if (!out_row_offset) return fail(TSLT_ERR_INVALID_ARG, "tslt_pack: null pointer");
  if (rows > 0 && (!idx || !logit || !count || !out_words)) return fail(TSLT_ERR_INVALID_ARG, "tslt_pack: null pointer");
  if (out_capacity_words < tslt_pack_bound_words(rows, k_cap, V))
    return fail(TSLT_ERR_WORKSPACE, "tslt_pack: room for %lld words, %lld may be needed", (long long)out_capacity_words,
                (long long)tslt_pack_bound_words(rows, k_cap, V));
  tslt::WireParams p{};
  p.idx = idx; p.logit = logit; p.count = count; p.rows = rows; p.k_cap = k_cap; p.b_idx = tslt::wire_index_bits(V);
  p.payload = int(payload); p.words = out_words; p.row_offset = out_row_offset;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  hipError_t e;
  hipLaunchKernelGGL(tslt::wire_offsets_kernel, dim3(1), dim3(1024), 0, s, p);
  if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "tslt_pack launch");
  if (rows > 0) {
    hipLaunchKernelGGL(tslt::wire_pack_kernel, dim3(unsigned(rows)), dim3(64), 0, s, p);
    if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "tslt_pack launch");
  }
  return TSLT_OK;
}

int tslt_unpack(const uint32_t* words, const int64_t* row_offset, int64_t rows, int32_t k_cap, int64_t V,
                tslt_dtype payload, int32_t* out_idx, float* out_logit, int32_t* out_count, void* stream) {
  if (rows < 0 || V < 1 || V > 0x7FFFFFFF) return fail(TSLT_ERR_INVALID_ARG, "tslt_unpack: bad shape");
  if (k_cap < 1 || k_cap > TSLT_MAX_K_CAP) return fail(TSLT_ERR_UNSUPPORTED, "tslt_unpack: k_cap must be in 1..%d", TSLT_MAX_K_CAP);
  if (payload != TSLT_BF16 && payload != TSLT_F16) return fail(TSLT_ERR_INVALID_ARG, "tslt_unpack: the value format must be bfloat16 or binary16");
  if (rows == 0) return TSLT_OK;
  if (!words || !row_offset || !out_idx || !out_logit || !out_count) return fail(TSLT_ERR_INVALID_ARG, "tslt_unpack: null pointer");
  tslt::WireParams p{};
  p.in_words = words; p.in_row_offset = row_offset; p.rows = rows; p.k_cap = k_cap; p.b_idx = tslt::wire_index_bits(V);
  p.payload = int(payload); p.out_idx = out_idx; p.out_logit = out_logit; p.out_count = out_count;
  hipLaunchKernelGGL(tslt::wire_unpack_kernel, dim3(unsigned(rows)), dim3(64), 0, reinterpret_cast<hipStream_t>(stream), p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, "tslt_unpack launch");
  return TSLT_OK;
}

int tslt_sample(const int32_t* idx, const float* logit, const int32_t* count, int64_t rows, int32_t k_cap,
                const float* u, int32_t n_samples, int32_t without_replacement, int32_t* out_token,
                int32_t* out_slot, void* stream) {
  if (rows < 0 || rows > 0x7FFFFFFF) return fail(TSLT_ERR_INVALID_ARG, "tslt_sample: bad row count");
  if (k_cap < 1 || k_cap > TSLT_MAX_K_CAP) return fail(TSLT_ERR_UNSUPPORTED, "tslt_sample: k_cap must be in 1..%d", TSLT_MAX_K_CAP);
  if (n_samples < 0) return fail(TSLT_ERR_INVALID_ARG, "tslt_sample: n_samples < 0");
  if (rows == 0 || n_samples == 0) return TSLT_OK;
  if (!idx || !logit || !count || !u || !out_token) return fail(TSLT_ERR_INVALID_ARG, "tslt_sample: null pointer");
  tslt::SampleParams p{idx, logit, count, rows, k_cap, u, n_samples, without_replacement ? 1 : 0, out_token, out_slot};
  hipLaunchKernelGGL(tslt::sample_kernel, dim3(unsigned(rows)), dim3(64), 0, reinterpret_cast<hipStream_t>(stream), p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, "tslt_sample launch");
  return TSLT_OK;
}

static int verify_impl(int phases, int stage0, const char* name, const void* target_logits, tslt_dtype dt, int64_t B,
                       int32_t gamma, int64_t V, int64_t row_stride, float target_temperature, const int32_t* q_idx,
                       const float* q_logit, const int32_t* q_count, int32_t k_cap, const int32_t* draft_tokens,
                       const float* u_accept, const float* u_resample, int32_t* out_accept_len, int32_t* out_tokens,
                       float* out_ratio, float* out_beta, int32_t* status, void* ws, size_t ws_bytes, void* stream) {
  if (!valid_dtype(dt)) return fail(TSLT_ERR_INVALID_ARG, "%s: unknown dtype %d", name, int(dt));
  if (B < 0 || gamma < 1 || V <= 0 || row_stride < V) return fail(TSLT_ERR_INVALID_ARG, "%s: bad shape", name);
  if (V > 0x7FFFFFFF || B * (int64_t(gamma) + 1) > 0x7FFFFFFF) return fail(TSLT_ERR_UNSUPPORTED, "%s: sizes must fit 31 bits", name);
  if (gamma > 4096) return fail(TSLT_ERR_UNSUPPORTED, "%s: gamma > 4096", name);
  if (stage0 < 0) return fail(TSLT_ERR_INVALID_ARG, "%s: first_stage must be >= 0", name);
  if (tslt::row_segments(V, 16 / elem_bytes(dt)) + 2 > tslt::kBlock)
    return fail(TSLT_ERR_UNSUPPORTED, "%s: V too large (at most %d elements of this type)", name, (tslt::kBlock - 2) * tslt::kSegVecsTotal * (16 / elem_bytes(dt)) - 16);
  if (B * int64_t(tslt::row_segments(V)) > 0x7FFFFFFF) return fail(TSLT_ERR_UNSUPPORTED, "%s: B too large", name);
  if (!(target_temperature > 0.0f) || !std::isfinite(target_temperature)) return fail(TSLT_ERR_INVALID_ARG, "%s: temperature must be > 0", name);
  if (k_cap < 1 || k_cap > TSLT_MAX_K_CAP) return fail(TSLT_ERR_UNSUPPORTED, "%s: k_cap must be in 1..%d", name, TSLT_MAX_K_CAP);
  if (B == 0) return TSLT_OK;
  if (!target_logits || !q_idx || !q_logit || !q_count || !draft_tokens || !u_accept || !u_resample ||
      !out_accept_len || !out_tokens)
    return fail(TSLT_ERR_INVALID_ARG, "%s: null pointer", name);
  if (reinterpret_cast<uintptr_t>(target_logits) % elem_bytes(dt)) return fail(TSLT_ERR_INVALID_ARG, "%s: logits not aligned to their element type", name);
  const size_t need = tslt::verify_workspace_bytes(B, gamma, V, k_cap);
  if (!ws || ws_bytes < need || reinterpret_cast<uintptr_t>(ws) % 256)
    return fail(TSLT_ERR_WORKSPACE, "%s: workspace of %zu bytes, 256-byte aligned, required", name, need);

  tslt::VerifyParams p{};
  p.target = target_logits; p.B = B; p.gamma = gamma; p.V = V; p.row_stride = row_stride;
  p.rT = reciprocal_temperature(target_temperature);
  p.k2 = log2e_over_T(p.rT);
  p.q_idx = q_idx; p.q_logit = q_logit; p.q_count = q_count; p.k_cap = k_cap;
  p.draft_tokens = draft_tokens; p.u_accept = u_accept; p.u_resample = u_resample;
  p.out_accept_len = out_accept_len; p.out_tokens = out_tokens; p.out_ratio = out_ratio; p.out_beta = out_beta;
  p.status = status;
  p.stage0 = stage0 >= gamma ? 0 : stage0;
  tslt::verify_carve_workspace(p, ws);
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  hipError_t e = dt == TSLT_BF16 ? tslt::launch_verify<tslt::Bf16>(p, s, phases)
                 : dt == TSLT_F16 ? tslt::launch_verify<tslt::F16>(p, s, phases) : tslt::launch_verify<float>(p, s, phases);
  if (e != hipSuccess) return hip_fail(e, name);
  return TSLT_OK;
}

#define TSLT_VERIFY_ARGS                                                                                          \
  const void *target_logits, tslt_dtype dt, int64_t B, int32_t gamma, int64_t V, int64_t row_stride,             \
      float target_temperature, const int32_t *q_idx, const float *q_logit, const int32_t *q_count, int32_t k_cap, \
      const int32_t *draft_tokens, const float *u_accept, const float *u_resample, int32_t *out_accept_len,       \
      int32_t *out_tokens, float *out_ratio, float *out_beta, int32_t *status, void *ws, size_t ws_bytes, void *stream
#define TSLT_VERIFY_PASS                                                                                           \
  target_logits, dt, B, gamma, V, row_stride, target_temperature, q_idx, q_logit, q_count, k_cap, draft_tokens,   \
      u_accept, u_resample, out_accept_len, out_tokens, out_ratio, out_beta, status, ws, ws_bytes, stream

int tslt_verify(TSLT_VERIFY_ARGS) { return verify_impl(3, 0, "tslt_verify", TSLT_VERIFY_PASS); }
int tslt_verify_accept(TSLT_VERIFY_ARGS) { return verify_impl(1, 0, "tslt_verify_accept", TSLT_VERIFY_PASS); }
int tslt_verify_resample(TSLT_VERIFY_ARGS) { return verify_impl(2, 0, "tslt_verify_resample", TSLT_VERIFY_PASS); }
int tslt_verify_staged(TSLT_VERIFY_ARGS, int32_t first_stage) {
  return verify_impl(3, first_stage, "tslt_verify_staged", TSLT_VERIFY_PASS);
}
int tslt_verify_accept_staged(TSLT_VERIFY_ARGS, int32_t first_stage) {
  return verify_impl(1, first_stage, "tslt_verify_accept_staged", TSLT_VERIFY_PASS);
}

int tslt_verify_static(const void* target_logits, tslt_dtype dt, int64_t B, int32_t gamma, int64_t V, int64_t row_stride,
                       float target_temperature, const int32_t* q_idx, const float* q_logit, const int32_t* q_count,
                       int32_t k_cap, const int32_t* draft_tokens, const float* u_accept, const float* u_resample,
                       int32_t* out_accept_len, int32_t* out_tokens, float* out_ratio, float* out_beta, int32_t* status,
                       void* stream) {
  const char* name = "tslt_verify_static";
  if (B < 0 || gamma < 1) return fail(TSLT_ERR_INVALID_ARG, "%s: bad shape", name);
  if (B > TSLT_STATIC_MAX_POSITIONS || B * int64_t(gamma) > TSLT_STATIC_MAX_POSITIONS)
    return fail(TSLT_ERR_UNSUPPORTED, "%s: B * gamma = %lld positions, the static scratch array holds %d; use tslt_verify "
                "with a workspace", name, (long long)(B * int64_t(gamma)), TSLT_STATIC_MAX_POSITIONS);
  if (tslt::verify_workspace_bytes(B, gamma, V, k_cap) > size_t(TSLT_STATIC_SCRATCH_BYTES))
    return fail(TSLT_ERR_UNSUPPORTED, "%s: the static scratch array is too small for this call", name);
  void* ptr = nullptr;
  const hipError_t e = scratch_on_current_device(&ptr);
  if (e != hipSuccess) return hip_fail(e, "tslt_verify_static: address of the scratch array");
  // every position's decision and status word is written by the acceptance kernel before the resampling
  // kernel reads it, so nothing in the array has to start at zero
  return verify_impl(3, 0, name, target_logits, dt, B, gamma, V, row_stride, target_temperature, q_idx, q_logit, q_count,
                     k_cap, draft_tokens, u_accept, u_resample, out_accept_len, out_tokens, out_ratio, out_beta, status, ptr,
                     size_t(TSLT_STATIC_SCRATCH_BYTES), stream);
}

int tslt_calibrate_read(const void* src, size_t bytes, int32_t n_blocks, uint32_t* sink, void* stream) {
  const char* name = "tslt_calibrate_read";
  if (!src || !sink) return fail(TSLT_ERR_INVALID_ARG, "%s: null pointer", name);
  if (reinterpret_cast<uintptr_t>(src) % 16) return fail(TSLT_ERR_INVALID_ARG, "%s: the buffer must be 16-byte aligned", name);
  if (n_blocks < 1) return fail(TSLT_ERR_INVALID_ARG, "%s: n_blocks must be >= 1", name);
  const size_t chunk = size_t(16) * tslt::kCalibUnroll * tslt::kBlock;       // bytes one workgroup reads per round
  if (bytes == 0 || bytes % (chunk * size_t(n_blocks)) != 0)
    return fail(TSLT_ERR_INVALID_ARG, "%s: bytes must be a positive multiple of n_blocks * %zu", name, chunk);
  const uint64_t vecs_per_block = bytes / 16 / size_t(n_blocks);
  hipLaunchKernelGGL(tslt::calibrate_read_kernel, dim3(unsigned(n_blocks)), dim3(tslt::kBlock), 0,
                     reinterpret_cast<hipStream_t>(stream), reinterpret_cast<const uint4*>(src), vecs_per_block, sink);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, name);
  return TSLT_OK;
}

int tslt_truncation_stats(const void* target_logits, tslt_dtype dt, int64_t rows, int64_t V, int64_t row_stride,
                          float target_temperature, const int32_t* q_idx, const float* q_logit, const int32_t* q_count,
                          int32_t k_cap, const int32_t* k_list, int32_t n_k, float* out_keep, float* out_beta,
                          int32_t* status, void* stream) {
  const char* name = "tslt_truncation_stats";
  if (!valid_dtype(dt)) return fail(TSLT_ERR_INVALID_ARG, "%s: unknown dtype %d", name, int(dt));
  if (rows < 0 || V <= 0 || row_stride < V) return fail(TSLT_ERR_INVALID_ARG, "%s: bad shape", name);
  if (row_too_long(V, dt) || rows > 0x7FFFFFFF) return fail(TSLT_ERR_UNSUPPORTED, "%s: rows must fit 31 bits, a row 4 GiB", name);
  if (!(target_temperature > 0.0f) || !std::isfinite(target_temperature)) return fail(TSLT_ERR_INVALID_ARG, "%s: temperature must be > 0", name);
  if (k_cap < 1 || k_cap > TSLT_MAX_K_CAP) return fail(TSLT_ERR_UNSUPPORTED, "%s: k_cap must be in 1..%d", name, TSLT_MAX_K_CAP);
  if (n_k < 1 || n_k > tslt::kMaxStatK) return fail(TSLT_ERR_UNSUPPORTED, "%s: between 1 and %d values of K", name, tslt::kMaxStatK);
  if (!k_list) return fail(TSLT_ERR_INVALID_ARG, "%s: null pointer", name);
  if (rows == 0) return TSLT_OK;
  if (!target_logits || !q_idx || !q_logit || !q_count || !out_keep || !out_beta) return fail(TSLT_ERR_INVALID_ARG, "%s: null pointer", name);
  if (reinterpret_cast<uintptr_t>(target_logits) % elem_bytes(dt)) return fail(TSLT_ERR_INVALID_ARG, "%s: logits not aligned to their element type", name);
  tslt::StatsParams p{};
  p.target = target_logits; p.rows = rows; p.V = V; p.row_stride = row_stride;
  p.rT = reciprocal_temperature(target_temperature);
  p.k2 = log2e_over_T(p.rT);
  p.q_idx = q_idx; p.q_logit = q_logit; p.q_count = q_count; p.k_cap = k_cap;
  p.n_k = n_k;
  for (int j = 0; j < n_k; ++j) p.k_list[j] = k_list[j];
  p.out_keep = out_keep; p.out_beta = out_beta; p.status = status;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const dim3 grid{unsigned(rows)}, block{unsigned(tslt::kBlock)};
  if (dt == TSLT_BF16) hipLaunchKernelGGL(tslt::truncation_stats_kernel<tslt::Bf16>, grid, block, 0, s, p);
  else if (dt == TSLT_F16) hipLaunchKernelGGL(tslt::truncation_stats_kernel<tslt::F16>, grid, block, 0, s, p);
  else hipLaunchKernelGGL(tslt::truncation_stats_kernel<float>, grid, block, 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, name);
  return TSLT_OK;
}

int tslt_multicandidate_stats(const void* target_logits, tslt_dtype dt, int64_t rows, int64_t V, int64_t row_stride,
                              float target_temperature, const int32_t* q_idx, const float* q_logit, const int32_t* q_count,
                              int32_t k_cap, int32_t k, float* out_beta, float* out_theta, int32_t* status, void* stream) {
  const char* name = "tslt_multicandidate_stats";
  if (!valid_dtype(dt)) return fail(TSLT_ERR_INVALID_ARG, "%s: unknown dtype %d", name, int(dt));
  if (rows < 0 || V <= 0 || row_stride < V) return fail(TSLT_ERR_INVALID_ARG, "%s: bad shape", name);
  if (row_too_long(V, dt) || rows > 0x7FFFFFFF) return fail(TSLT_ERR_UNSUPPORTED, "%s: rows must fit 31 bits, a row 4 GiB", name);
  if (!(target_temperature > 0.0f) || !std::isfinite(target_temperature)) return fail(TSLT_ERR_INVALID_ARG, "%s: temperature must be > 0", name);
  if (k_cap < 1 || k_cap > TSLT_MAX_K_CAP) return fail(TSLT_ERR_UNSUPPORTED, "%s: k_cap must be in 1..%d", name, TSLT_MAX_K_CAP);
  if (k < 1 || k > TSLT_MAX_BRANCH) return fail(TSLT_ERR_UNSUPPORTED, "%s: between 1 and %d candidates", name, TSLT_MAX_BRANCH);
  if (rows == 0) return TSLT_OK;
  if (!target_logits || !q_idx || !q_logit || !q_count || !out_beta || !out_theta) return fail(TSLT_ERR_INVALID_ARG, "%s: null pointer", name);
  if (reinterpret_cast<uintptr_t>(target_logits) % elem_bytes(dt)) return fail(TSLT_ERR_INVALID_ARG, "%s: logits not aligned to their element type", name);
  tslt::McStatsParams p{};
  p.target = target_logits; p.rows = rows; p.V = V; p.row_stride = row_stride;
  p.rT = reciprocal_temperature(target_temperature);
  p.k2 = log2e_over_T(p.rT);
  p.q_idx = q_idx; p.q_logit = q_logit; p.q_count = q_count; p.k_cap = k_cap; p.k = k;
  p.out_beta = out_beta; p.out_theta = out_theta; p.status = status;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const dim3 grid{unsigned(rows)}, block{unsigned(tslt::kBlock)};
  if (dt == TSLT_BF16) hipLaunchKernelGGL(tslt::multicandidate_stats_kernel<tslt::Bf16>, grid, block, 0, s, p);
  else if (dt == TSLT_F16) hipLaunchKernelGGL(tslt::multicandidate_stats_kernel<tslt::F16>, grid, block, 0, s, p);
  else hipLaunchKernelGGL(tslt::multicandidate_stats_kernel<float>, grid, block, 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, name);
  return TSLT_OK;
}

int tslt_verify_tree(const void* target_logits, tslt_dtype dt, int64_t B, int64_t V, int64_t row_stride,
                     float target_temperature, int32_t depth, const int32_t* expansion, const int32_t* q_idx,
                     const float* q_logit, const int32_t* q_count, int32_t k_cap, const int32_t* cand_tokens,
                     const float* u_accept, const float* u_resample, int32_t without_replacement,
                     int32_t* out_node_token, int32_t* out_node_slot, int32_t* out_seq, int32_t* out_len,
                     float* out_ratio, float* out_beta, int32_t* status, void* ws, size_t ws_bytes, void* stream) {
  const char* name = "tslt_verify_tree";
  if (!valid_dtype(dt)) return fail(TSLT_ERR_INVALID_ARG, "%s: unknown dtype %d", name, int(dt));
  if (B < 0 || V <= 0 || row_stride < V) return fail(TSLT_ERR_INVALID_ARG, "%s: bad shape", name);
  if (depth < 1 || !expansion) return fail(TSLT_ERR_INVALID_ARG, "%s: depth must be >= 1 and expansion given", name);
  if (depth > TSLT_MAX_TREE_DEPTH) return fail(TSLT_ERR_UNSUPPORTED, "%s: depth > %d", name, TSLT_MAX_TREE_DEPTH);
  if (!(target_temperature > 0.0f) || !std::isfinite(target_temperature)) return fail(TSLT_ERR_INVALID_ARG, "%s: temperature must be > 0", name);
  if (k_cap < 1 || k_cap > TSLT_MAX_K_CAP) return fail(TSLT_ERR_UNSUPPORTED, "%s: k_cap must be in 1..%d", name, TSLT_MAX_K_CAP);
  if (tslt::row_segments(V, 16 / elem_bytes(dt)) + 2 > tslt::kBlock || V > 0x7FFFFFFF) return fail(TSLT_ERR_UNSUPPORTED, "%s: V too large", name);
  tslt::TreeParams p{};
  int64_t width = 1, n_nodes = 1;
  p.offsets[0] = 0;
  for (int l = 0; l < depth; ++l) {
    if (expansion[l] < 1 || expansion[l] > TSLT_MAX_BRANCH)
      return fail(TSLT_ERR_UNSUPPORTED, "%s: expansion[%d] must be in 1..%d", name, l, TSLT_MAX_BRANCH);
    p.expansion[l] = expansion[l];
    p.offsets[l + 1] = int(n_nodes);
    width *= expansion[l];
    n_nodes += width;
    if (n_nodes > (1 << 24)) return fail(TSLT_ERR_UNSUPPORTED, "%s: tree too large", name);
  }
  p.offsets[depth + 1] = int(n_nodes);
  p.n_nodes = int(n_nodes);
  p.n_int = int(n_nodes - width);
  p.depth = depth;
  const bool all_nodes = out_node_token != nullptr || out_node_slot != nullptr;
  p.all_nodes = all_nodes ? 1 : 0;
  p.tasks = all_nodes ? p.n_nodes : 1;
  if (B * int64_t(p.tasks) * tslt::row_segments(V) > 0x7FFFFFFF || B * n_nodes > 0x7FFFFFFF)
    return fail(TSLT_ERR_UNSUPPORTED, "%s: B * nodes too large", name);
  if (B == 0) return TSLT_OK;
  if (!target_logits || !q_idx || !q_logit || !q_count || !cand_tokens || !u_accept || !u_resample || !out_seq || !out_len)
    return fail(TSLT_ERR_INVALID_ARG, "%s: null pointer", name);
  if (reinterpret_cast<uintptr_t>(target_logits) % elem_bytes(dt)) return fail(TSLT_ERR_INVALID_ARG, "%s: logits not aligned to their element type", name);
  const size_t need = tslt::tree_workspace_bytes(B, n_nodes, V, all_nodes);
  if (!ws || ws_bytes < need || reinterpret_cast<uintptr_t>(ws) % 256)
    return fail(TSLT_ERR_WORKSPACE, "%s: workspace of %zu bytes, 256-byte aligned, required", name, need);
  p.target = target_logits; p.B = B; p.V = V; p.row_stride = row_stride;
  p.rT = reciprocal_temperature(target_temperature);
  p.k2 = log2e_over_T(p.rT);
  p.q_idx = q_idx; p.q_logit = q_logit; p.q_count = q_count; p.k_cap = k_cap;
  p.cand_tokens = cand_tokens; p.u_accept = u_accept; p.u_resample = u_resample;
  p.wor = without_replacement ? 1 : 0;
  p.out_node_token = out_node_token; p.out_node_slot = out_node_slot; p.out_seq = out_seq; p.out_len = out_len;
  p.out_ratio = out_ratio; p.out_beta = out_beta; p.status = status;
  tslt::tree_carve_workspace(p, ws);
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  hipError_t e = dt == TSLT_BF16 ? tslt::launch_verify_tree<tslt::Bf16>(p, s)
                 : dt == TSLT_F16 ? tslt::launch_verify_tree<tslt::F16>(p, s) : tslt::launch_verify_tree<float>(p, s);
  if (e != hipSuccess) return hip_fail(e, name);
  return TSLT_OK;
}

}  // extern "C"
