// Error reporting and version of the C ABI.
#include <string.h>

#include <mutex>
#include <vector>

#include "photon_host.h"

namespace photon {

char* error_buffer() {
  static thread_local char buf[512] = {0};
  return buf;
}

void clear_error() { error_buffer()[0] = 0; }

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(error_buffer(), 512, fmt, ap);
  va_end(ap);
  return code;
}

// ---- per-kernel-class timing -------------------------------------------------------------------
bool g_profile_on = false;
namespace {
struct ProfRec { int cls; hipEvent_t start, stop; };
std::mutex g_prof_mu;
std::vector<ProfRec> g_prof;
const char* const kClassNames[KC_COUNT] = {
    "coarse_attn_kernel", "coarse_merge_kernel", "local_attn_kernel", "linear_bf16_kernels", "gemm_f32_kernel",
    "reduce_splits_kernel", "chunker_gemm_bf16_kernel", "norm_rows_kernel", "rope_append_kernel", "silu_mul_kernel",
    "choose_token_kernel", "misc", "persistent_module_kernel"};
}  // namespace

// At most this many launches are timed between two resets (each holds two events); further launches go untimed.
constexpr size_t PROFILE_MAX_RECORDS = 1 << 16;

bool profile_pair(int cls, hipEvent_t* start, hipEvent_t* stop) {
  {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (g_prof.size() >= PROFILE_MAX_RECORDS) return false;
  }
  ProfRec r{cls, nullptr, nullptr};
  if (hipEventCreate(&r.start) != hipSuccess) return false;
  if (hipEventCreate(&r.stop) != hipSuccess) { (void)hipEventDestroy(r.start); return false; }
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof.push_back(r);
  *start = r.start;
  *stop = r.stop;
  return true;
}

}  // namespace photon

// ---- trivial streaming read: the bandwidth ceiling the attention kernels are compared with --------
namespace photon {
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void hbm_read_probe_kernel(const u32x4* __restrict__ buf, int64_t n16, uint32_t* __restrict__ sink) {
  u32x4 acc = u32x4{0, 0, 0, 0};
  const int64_t stride = (int64_t)gridDim.x * 256 * 4;
  for (int64_t i = (int64_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n16; i += stride) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t j = i + u * 256;
      if (j < n16) acc ^= __builtin_nontemporal_load(buf + j);
    }
  }
  const uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (r == 0x9e3779b9u) sink[0] = r;          // practically never: keeps the loads alive
}
}  // namespace photon

extern "C" int32_t photon_hbm_read_probe(const void* buf, size_t bytes, void* sink, void* stream) {
  using namespace photon;
  clear_error();
  PHOTON_REQUIRE_PTR(buf);
  PHOTON_REQUIRE(sink != nullptr && bytes >= 16, PHOTON_ERR_INVALID_ARG, "%s: sink is null or buffer too small", __func__);
  hipLaunchKernelGGL(hbm_read_probe_kernel, dim3(256 * 8), dim3(256), 0, (hipStream_t)stream, (const u32x4*)buf,
                     (int64_t)(bytes / 16), (uint32_t*)sink);
  return check_launch("hbm_read_probe_kernel");
}

// ---- matrix-core loop without memory traffic: the ceiling the MFMA kernels are compared with -------
namespace photon {
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
// One wave per SIMD, 16 independent 32x32 accumulators, operands fixed in registers.  random_operands: values
// spread like N(0,1) data in every lane and element (what a contraction of real activations toggles in the
// multipliers) instead of small constants; the chip's clock under the two differs.
__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, int random_operands, float* __restrict__ sink) {
  probe_f32x16 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  probe_bf16x8 a, b;
  uint32_t h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    h = h * 1664525u + 1013904223u;
    a[e] = random_operands ? (__bf16)(((int)(h >> 16) - 32768) / 16384.0f) : (__bf16)(float)(threadIdx.x & 3);
    h = h * 1664525u + 1013904223u;
    b[e] = random_operands ? (__bf16)(((int)(h >> 16) - 32768) / 16384.0f) : (__bf16)1.0f;
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  if (s == 1.2345e-30f) sink[0] = s;           // practically never: keeps the accumulators alive
}
}  // namespace photon

extern "C" double photon_mfma_probe(int32_t iters, int32_t random_operands, void* sink, void* stream) {
  using namespace photon;
  clear_error();
  if (sink == nullptr || iters < 1 || iters > (1 << 24)) {
    fail(PHOTON_ERR_INVALID_ARG, "%s: sink is null or iters=%d outside [1, 2^24]", __func__, iters);
    return 0.0;
  }
  constexpr int WGS = 256;                     // one workgroup of 4 waves per compute unit
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(WGS), dim3(256), 0, (hipStream_t)stream, (int)iters, (int)random_operands, (float*)sink);
  if (check_launch("mfma_probe_kernel") != PHOTON_OK) return 0.0;
  return (double)WGS * 4 * iters * 16 * (2.0 * 32 * 32 * 16);
}

extern "C" int32_t photon_profile_enable(int32_t on) {
  photon::g_profile_on = (on != 0);
  return PHOTON_OK;
}

extern "C" int32_t photon_profile_reset(void) {
  std::lock_guard<std::mutex> lk(photon::g_prof_mu);
  for (auto& r : photon::g_prof) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
  photon::g_prof.clear();
  return PHOTON_OK;
}

extern "C" int32_t photon_profile_num_classes(void) { return photon::KC_COUNT; }

extern "C" const char* photon_profile_class_name(int32_t cls) {
  return (cls >= 0 && cls < photon::KC_COUNT) ? photon::kClassNames[cls] : "";
}

extern "C" int32_t photon_profile_get(int32_t cls, int64_t* launches, double* total_ms) {
  using namespace photon;
  clear_error();
  PHOTON_REQUIRE(cls >= 0 && cls < KC_COUNT && launches && total_ms, PHOTON_ERR_INVALID_ARG, "%s: bad class or null output", __func__);
  std::lock_guard<std::mutex> lk(g_prof_mu);
  int64_t n = 0;
  double ms = 0.0;
  for (auto& r : g_prof) {
    if (r.cls != cls) continue;
    if (hipEventSynchronize(r.stop) != hipSuccess) return fail(PHOTON_ERR_HIP, "%s: event synchronise failed", __func__);
    float t = 0.f;
    if (hipEventElapsedTime(&t, r.start, r.stop) != hipSuccess) return fail(PHOTON_ERR_HIP, "%s: elapsed time failed", __func__);
    ms += t;
    ++n;
  }
  *launches = n;
  *total_ms = ms;
  return PHOTON_OK;
}

extern "C" int32_t photon_version(void) { return 100; }

extern "C" const char* photon_last_error(void) { return photon::error_buffer(); }
