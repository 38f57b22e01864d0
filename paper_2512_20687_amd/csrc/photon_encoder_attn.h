// Internal launch interface of the encoders' whole-sequence causal attention.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/photon.h"

namespace photon {

// Scratch the bf16 path needs (rotated, split and re-laid-out operands); 0 for fp32.
size_t encoder_attn_workspace_bytes(int Bt, int64_t M, int H, int d_h, bool bf16);

// out[b*M + i, h*d_h ..] = causal attention of query i over keys 0..i of (sequence b, head h), q and k rotated
// at positions 0..M-1.  qkv fp32 [Bt*M, 3*H*d_h].  k_cache / v_cache (both or neither): [Bt][H][S_max][row elements]
// receive the rotated keys and the values of positions 0..M-1: fp32 (bf16 false), bf16, or E4M3 bytes (kv_fp8, with
// bf16 only).  out_bf16 (with bf16 only): `out` holds bf16 values, the result rounded to nearest even.
int32_t launch_encoder_attn(const float* qkv, float* out, int Bt, int64_t M, int H, int d_h, float theta, float scale, void* k_cache,
                            void* v_cache, int64_t S_max, void* workspace, bool bf16, bool kv_fp8, bool out_bf16, hipStream_t st);

}  // namespace photon
