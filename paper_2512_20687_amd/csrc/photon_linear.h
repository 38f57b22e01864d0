// Internal launch interface of the few-row linear maps.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace photon {

enum LinearEpilogue { EPI_PLAIN = 0, EPI_RESID = 1, EPI_SWIGLU = 2 };

// y = rmsnorm(x; gain, eps) * W^T (gain == nullptr: y = x * W^T), then
//   EPI_PLAIN : out = y + bias
//   EPI_RESID : out = res + y + bias            (out may alias res)
//   EPI_SWIGLU: out = silu(y[:, :N]) * y[:, N:] (W has 2N rows: gate rows, then up rows)
struct LinearArgs {
  const float* x = nullptr;    // fp32 [M, K], row pitch ldx elements (x_bf16: bf16 values behind the pointer)
  int64_t ldx = 0;
  bool x_bf16 = false;         // bf16 weights only, no norm, plain or residual epilogue: x is the MFMA operand as it stands
  const void* W = nullptr;     // [N, K] (2N for EPI_SWIGLU) row-major, bf16 when w_bf16 else fp32
  bool w_bf16 = false;
  const float* gain = nullptr; // [K] or nullptr
  float eps = 0.f;
  const float* bias = nullptr; // [N] or nullptr
  const float* res = nullptr;  // [M, N], row pitch ldres
  int64_t ldres = 0;
  float* out = nullptr;        // [M, N], row pitch ldo
  int64_t ldo = 0;
  bool out_bf16 = false;       // bf16 weights only: out holds bf16 values (rounded to nearest even), ldo in elements
  int M = 0, N = 0, K = 0;
  int epilogue = EPI_PLAIN;
};

int32_t launch_linear(const LinearArgs& a, hipStream_t st);

// bf16 weights, activations small enough to stay in LDS: issues the launch and returns true, else returns false
// (the caller then takes the streaming kernel).  Arguments must have passed launch_linear's checks.
bool launch_linear_resident(const LinearArgs& a, hipStream_t st);

// bf16 weights, fp32 activations of 17-32 rows, plain or SwiGLU epilogue, contraction length at most 2048: two row tiles of
// 16 per workgroup at the accuracy (and with the per-row arithmetic) of the 16-row kernel; the matrix is streamed once.
// Returns true when the launch was issued.
bool launch_linear_resident_x2(const LinearArgs& a, hipStream_t st);

// Many rows (dozens and up) with bf16 weights: row kernel (norm, rounding to bf16) + tiled MFMA
// contraction + (SwiGLU) row kernel.  `workspace` holds linear_many_workspace_bytes(rows, K_max, N2_max)
// bytes, K_max >= every K and N2_max >= every 2N of a SwiGLU call that will be issued with it.
size_t linear_many_workspace_bytes(int64_t rows, int K_max, int N2_max);
// The row kernel alone: xb[M, K] (dense bf16) = rmsnorm(x; gain, eps) (gain == nullptr: x), rounded to nearest even.
int32_t launch_norm_round_rows(const float* x, int64_t ldx, const float* gain, float eps, void* xb, int M, int K, hipStream_t st);
int32_t launch_linear_many(const LinearArgs& a, void* workspace, int K_max, hipStream_t st);

}  // namespace photon
