// Internal launch interface of the persistent module kernel: all blocks of a local decoder on a few rows in ONE
// launch (paper Section 2.3.3 step (i): a decode sub-step of G^(l), Eq. 6-7), the projections of a block meeting
// at grid barriers instead of kernel boundaries.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/photon.h"

namespace photon {

constexpr int PM_MAX_LAYERS = 16;          // blocks per module the kernel's argument block holds
constexpr int PM_MAX_ROWS = 16;            // rows of a pass (chunks in flight x rows per chunk)
constexpr int PM_MAX_WINDOW = 8;           // window positions the attention phase keeps in registers
constexpr int PM_BAR_WORDS = 9 * 64;       // one barrier slot: a global arrival counter and one per XCD, 256 bytes apart

struct PersistentModule {
  const photon_layer_weights* layers = nullptr;   // host array, bf16 matrices
  int n_layers = 0;
  const float* x_in = nullptr;     // rows entering the first block: row i at x_in + i * ld_in (D floats)
  int64_t ld_in = 0;
  float* h = nullptr;              // [M, D]   residual stream after each block; the result
  float* qkv = nullptr;            // [M, 3D]  q | k | v of a block; afterwards its first M*D floats hold the mid-block stream
  void* attn = nullptr;            // [M, D]   bf16 attention rows
  void* act = nullptr;             // [M, F]   bf16 hidden rows of the feed-forward
  float* lk = nullptr;             // local caches [n_layers][n_chunks][W][H][d_h] fp32
  float* lv = nullptr;
  size_t layer_cache = 0;          // elements per layer
  unsigned* bar = nullptr;         // PM_BAR_WORDS zeroed words no other launch in flight uses
  unsigned* err = nullptr;         // error word (non-zero: a barrier wait ran out; every workgroup then leaves)
  int M = 0, D = 0, F = 0, H = 0, d_h = 0;
  int64_t n_chunks = 0;
  int W = 0, q_len = 0, q_pos = 0;
  float eps = 0.f, scale = 0.f, theta = 0.f;
};

// True when a kernel instantiation exists for these sizes (bf16 matrices, d_ff > 0, at most 16 rows, head size 64 or
// 128, window of at most 8, a unit deal one of the compiled ones) and the device can hold its whole grid at once.
bool persistent_module_supported(const PersistentModule& a);

// Enqueues the launch.  PHOTON_ERR_UNSUPPORTED when persistent_module_supported() is false.
int32_t launch_persistent_module(const PersistentModule& a, hipStream_t st);

// Measurement aid: while `device_buffer` (room for 16 * PM_MAX_LAYERS clock values) is set, workgroup 0 of every
// launch notes the constant 100 MHz clock at the milestones of every phase (contraction done, stores and prefetch
// issued, barrier passed).  nullptr switches it off.
void persistent_module_set_stamps(unsigned long long* device_buffer);

// Bound of a barrier wait in ticks of the constant 100 MHz clock (default 10^9 = 10 s).
void persistent_module_set_spin_ticks(long long ticks);

}  // namespace photon
