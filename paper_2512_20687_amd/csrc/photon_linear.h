// Internal launch interface of the few-row linear maps.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace photon {

constexpr int LINEAR_MAX_KSPLIT = 16;
constexpr int LINEAR_TARGET_WORKGROUPS = 512;

// A product whose K-splits have not been added yet:
//   value[m][n] = sum_{s < ks} data[s*split_stride + m*ld + n]
struct Pending {
  const float* data = nullptr;
  int ks = 0;
  int64_t split_stride = 0;
  int64_t ld = 0;
};

// out[M,N] = x[M,K] * W[N,K]^T (+ bias[N]) (+ res[M,N]); out may alias res.
struct LinearArgs {
  const void* x = nullptr;     // fp32 (or bf16 when x_bf16) [M, K], row pitch ldx elements
  int64_t ldx = 0;
  bool x_bf16 = false;
  const void* W = nullptr;     // [N, K] row-major, bf16 when w_bf16 else fp32
  bool w_bf16 = false;
  const float* bias = nullptr;
  const float* res = nullptr;
  int64_t ldres = 0;
  float* out = nullptr;
  int64_t ldo = 0;
  int M = 0, N = 0, K = 0;
  void* workspace = nullptr;   // split-K scratch for the partial tiles (no initialisation needed)
  size_t workspace_bytes = 0;
};

size_t linear_workspace_bytes(int max_rows, int max_N);
int32_t launch_linear(const LinearArgs& a, Pending* pend, hipStream_t st);

}  // namespace photon
