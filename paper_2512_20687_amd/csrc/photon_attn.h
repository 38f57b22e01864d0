// Internal launch interface of the attention kernels (used by the C ABI
// entry points and by the decode-step composition).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace photon {

enum KvType { KV_F32 = 0, KV_BF16 = 1, KV_FP8 = 2 };   // KV_FP8: E4M3 bytes; q and out fp32

// Elements of one K/V cache row: the head size rounded up to 32, 64 or 128 (columns past d_h hold zeros); 0 = unsupported.
inline int kv_row_elems(int d_h) { return d_h < 1 ? 0 : d_h <= 32 ? 32 : d_h <= 64 ? 64 : d_h <= 128 ? 128 : 0; }

// q/out are fp32 when q_f32 (always the case for KV_F32), else bf16; rows of d_h elements.  Cache rows hold
// kv_row_elems(d_h) elements.
int32_t launch_coarse_attn(KvType kv, bool q_f32, int d_h, const void* q, const void* kc, const void* vc,
                           const int32_t* seq_len, void* out, int Bt, int H, int64_t S_max, float scale,
                           int n_splits, void* ws, hipStream_t st);
int32_t coarse_auto_splits(int Bt, int H, int64_t S_max);

int32_t launch_local_attn(bool f32, int d_h, const void* q, const void* k, const void* v, void* out,
                          int64_t n_chunks, int W, int q_len, int q_pos, int H, float scale, hipStream_t st);

// Fused decode sub-step of a local decoder: rotary + append to the local cache + causal attention for the
// q_len new rows of every chunk, read straight from the QKV projection output [rows, 3*H*d_h] (fp32).
int32_t launch_local_step_attn(int d_h, const float* qkv, float* lk, float* lv, float* out, int64_t n_chunks, int W, int q_len,
                               int q_pos, int H, float scale, float theta, bool out_bf16, hipStream_t st);

}  // namespace photon
