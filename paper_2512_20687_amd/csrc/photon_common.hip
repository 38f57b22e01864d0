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
    "choose_token_kernel", "misc"};
}  // namespace

bool profile_pair(int cls, hipEvent_t* start, hipEvent_t* stop) {
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
