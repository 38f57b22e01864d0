// Dense bf16 contractions on the matrix cores: out[M,N] = x[M,K] * W[N,K]^T (+ bias, + residual).
//   * the context-chunker projection (paper Eq. 4) at many-row shapes: bf16 in, bf16 out;
//   * the block projections of the prefill, and of a decode step once a level carries many rows (large
//     batches, deep hierarchies): a row kernel normalises the fp32 activations and rounds them to bf16, the
//     matrix cores' operand type (the few-row kernels keep a bf16 remainder as well; at many rows that second
//     pass over the matrix cores costs a fifth of the prefill and of a large-batch step, for accuracy far
//     beyond what bf16 matrices and a bf16 cache leave).
//
// One workgroup of 4 waves owns a (64 WT) x (64 WT) output tile, each wave a quadrant of WT x WT
// MFMA 32x32x16 tiles (WT = 4: 256x256 tile, 128x128 per wave, 256 fp32 accumulators per lane; WT = 2 and 1 for
// problems with too few big tiles to fill the chip).  K is walked in 64-wide slabs of x and W held in 2 LDS
// buffers (4 at the smaller tiles); the coming slabs are moved global -> LDS directly (no staging registers) while the current slab's MFMAs run, and operand fragments are
// double-buffered in registers.  LDS rows are 128 (64) bytes with the 16-byte column index XOR-ed with row bits,
// which keeps the 128-bit operand reads of 16 consecutive rows on distinct banks.  Workgroup ids are remapped so
// that the tiles resident on one XCD at a time share x row-blocks and W column-blocks in that XCD's L2.
// What bounds the kernel is the rate at which a compute unit takes its slabs in (about 40 bytes per ns), not the
// matrix cores: the tile is as large as the accumulator registers allow, and the gate/up projection forms SwiGLU
// in the accumulators instead of writing both halves.
#include <type_traits>

#include "photon_device.h"
#include "photon_host.h"
#include "photon_linear.h"

namespace photon {

typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int G_BK = 64;                                         // K must be a multiple of this
constexpr int G_THREADS = 256;

// Byte offset of (row, 16-byte column) in a staged slab whose rows hold BK bf16.  The column index is XOR-ed with row
// bits so that the 16 rows one quarter-wave reads together fall on distinct 16-byte slots of the 256-byte bank line
// (2 rows of 128 bytes, or 4 rows of 64 bytes, per line).
template <int BK> __device__ __forceinline__ int swz(int row, int col16) {
  if (BK == 64) return row * 128 + ((col16 ^ ((row >> 1) & 7)) << 4);
  return row * 64 + ((col16 ^ ((row >> 2) & 3)) << 4);
}

// 16 bytes per lane from global memory straight into LDS: lane l lands at lds_base + 16 l (lds_base: byte offset in
// LDS, wave-uniform).  Written as an instruction rather than through the compiler's builtin: the compiler treats
// the builtin as an access to both memories that may complete out of order, and while one is in flight it makes
// every wait for an LDS read a wait for ALL LDS reads, which serialises the operand prefetch below.  Completion is
// tracked by hand (s_waitcnt vmcnt) at the one place per slab where it matters.
// m0 (the LDS base of the load) is named as clobbered so that the compiler keeps no value of its own in it across the
// statement; it notes that m0 is a reserved register, which is the point here.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load16_to_lds(const void* gsrc, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gsrc), "s"(lds_base) : "memory", "m0");
}
#pragma clang diagnostic pop

// s_waitcnt immediate: at most `vm` vector-memory operations outstanding, all LDS reads done
constexpr int waitcnt_vm_lgkm0(int vm) { return (vm & 0xF) | ((vm >> 4) << 14) | (7 << 4); }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

enum GemmOut { GEMM_OUT_BF16 = 0, GEMM_OUT_F32 = 1, GEMM_OUT_SWIGLU = 2 };

// WT: MFMA tiles per wave and dimension (tile edge 64 WT).  OUT bf16: Cout bf16 [M, ldc] = acc + bias.  OUT fp32:
// Cout fp32 [M, ldc] = acc + bias + res.  OUT SwiGLU (WT even): B has 2N rows, gate rows then up rows; a tile covers
// 32 WT output columns and takes the gate rows of 32 columns into the even MFMA column tiles of a wave and the up
// rows of the same columns into the odd ones, so that silu(gate) * up is formed in registers:
// Cout bf16 [M, ldc] = silu(x Wg^T) * (x Wu^T).  BK: k per slab (64 or 32); NB: slab buffers in LDS (NB - 1 slabs are
// in flight while one is contracted).
template <int WT, int OUT, int BK, int NB>
__global__ __launch_bounds__(G_THREADS) void gemm_bf16_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, const float* __restrict__ bias,
    const float* __restrict__ res, int64_t ldres, void* __restrict__ Cout, int64_t ldc, int M, int N, int K, int tiles_m,
    int tiles_n) {
  constexpr int BM = 64 * WT;                                   // tile edge (rows and columns)
  constexpr int WE = 32 * WT;                                   // wave quadrant edge
  constexpr int TILE_BYTES = BM * BK * 2;                       // one operand slab
  constexpr int CPR = BK / 8;                                   // 16-byte columns per slab row
  constexpr int RPI = 64 / CPR;                                 // slab rows one load instruction covers
  constexpr int ROUNDS = BM / (4 * RPI);
  constexpr int OPS = 2;                                        // operand slabs per buffer: x, W
  constexpr int STAGE_BYTES = OPS * TILE_BYTES;
  constexpr int B_OFF = (OPS - 1) * TILE_BYTES;
  constexpr int LPS = OPS * ROUNDS;                             // load instructions per slab and wave
  extern __shared__ __align__(16) char lds[];                   // [NB buffers][A slab | B slab]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // scalar: the LDS targets of the direct loads are wave-uniform

  // XCD-aware raster: ids are dealt round-robin to 8 XCDs; give each XCD a contiguous run of tiles,
  // column tiles fastest, so concurrent workgroups of an XCD share x row-blocks.
  const int total = tiles_m * tiles_n;
  const int id = blockIdx.x;
  const int logical = (total % 8 == 0) ? (id & 7) * (total / 8) + (id >> 3) : id;   // ragged tile count: plain order
  const int tm = logical / tiles_n, tn = logical % tiles_n;
  constexpr bool GU = (OUT == GEMM_OUT_SWIGLU);
  static_assert(!GU || WT % 2 == 0, "the gate/up pairing needs an even number of column tiles per wave");
  const int m0 = tm * BM, n0 = tn * (GU ? BM / 2 : BM);

  // global -> LDS without passing through registers: one instruction moves 64 lanes x 16 B = RPI slab rows;
  // lane l lands at LDS row l/CPR, 16-byte column l%CPR, so it fetches the logical column that the XOR
  // swizzle maps there.  Round i of wave w covers slab rows (i*4 + w)*RPI .. +RPI.
  const int srow = lane / CPR, scol = lane % CPR;
  int64_t aoff[ROUNDS];
  const bf16_t* bptr[ROUNDS];
#pragma unroll
  for (int i = 0; i < ROUNDS; ++i) {
    const int r = (i * 4 + wave) * RPI + srow;
    const int c = (swz<BK>(r, scol) - r * (BK * 2)) >> 4;       // the swizzle is an involution on the column index
    int ra = m0 + r; ra = ra < M ? ra : M - 1;                   // clamped rows are never stored
    int rb = n0 + r;
    if (GU) {                                                   // tile row -> output column and gate / up
      const int rr = r % WE, jj = rr >> 5;
      rb = n0 + (r / WE) * (WE / 2) + (jj >> 1) * 32 + (rr & 31);
      rb = (rb < N ? rb : N - 1) + (jj & 1) * N;
    } else {
      rb = rb < N ? rb : N - 1;
    }
    aoff[i] = (int64_t)ra * K + c * 8;
    bptr[i] = B + (int64_t)rb * K + c * 8;
  }
  const int KT = K / BK;
  const int KT2 = KT;
  // Always issues its loads (past the end: the last slab again, into a buffer nobody reads any more), so that the
  // number of loads in flight at every wait is a compile-time constant.
  auto stage = [&](int kt, int buf) {
    kt = kt < KT2 ? kt : KT2 - 1;
    char* sa = lds + buf * STAGE_BYTES;
    const int64_t kk = (int64_t)kt * BK;
#pragma unroll
    for (int i = 0; i < ROUNDS; ++i) {
      const int off = (i * 4 + wave) * 1024;
      load16_to_lds(A + aoff[i] + kk, (uint32_t)(uintptr_t)(lptr_t)(sa + off));
      load16_to_lds(bptr[i] + kk, (uint32_t)(uintptr_t)(lptr_t)(sa + B_OFF + off));
    }
  };

  float16_t acc[WT][WT];
#pragma unroll
  for (int i = 0; i < WT; ++i)
#pragma unroll
    for (int j = 0; j < WT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int wm = (wave >> 1) * WE, wn = (wave & 1) * WE;         // wave quadrant inside the tile
  const int frow = lane & 31, fk = lane >> 5;                    // operand fragment: row, 8-wide k group

  // Pipeline over the K slabs with ONE barrier per slab, placed before the slab's last 16-wide step:
  //   MFMA(all steps but the last of slab kt)  [fragment reads of the next step issued ahead]
  //   wait for slab kt+1 (NB-2 younger slabs may still be in flight), barrier
  //     -> every wave has finished reading slab kt, so its buffer can take slab kt+NB right away
  //   issue slab kt+NB, read the first fragments of slab kt+1, MFMA(last step of slab kt)
  // so neither the load wait nor the first fragment reads of a slab leave the matrix cores idle.
  constexpr int KS = BK / 16;
  // The fragment reads of the next step are issued in two halves (x rows, then W rows) around the first row of
  // MFMAs: the counter of outstanding LDS operations holds 15 at most, and with the 2 WT reads of the next step
  // on top of the 2 WT of the current one the compiler could no longer wait for the older ones alone.
  bf16x8_t af[2][WT], bfr[2][WT];
  auto frags_a = [&](int buf, int ks, bf16x8_t (&a)[WT]) {
    const char* sa = lds + buf * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < WT; ++i)
      a[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4_t*>(sa + swz<BK>(wm + i * 32 + frow, ks * 2 + fk)));
  };
  auto frags_b = [&](int buf, int ks, bf16x8_t (&b)[WT]) {
    const char* sb = lds + buf * STAGE_BYTES + B_OFF;
#pragma unroll
    for (int i = 0; i < WT; ++i)
      b[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4_t*>(sb + swz<BK>(wn + i * 32 + frow, ks * 2 + fk)));
  };
  auto mfma_first = [&](const bf16x8_t (&a)[WT], const bf16x8_t (&b)[WT]) {
#pragma unroll
    for (int j = 0; j < WT; ++j) acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[j], acc[0][j], 0, 0, 0);
  };
  auto mfma_rest = [&](const bf16x8_t (&a)[WT], const bf16x8_t (&b)[WT]) {
#pragma unroll
    for (int i = 1; i < WT; ++i)
#pragma unroll
      for (int j = 0; j < WT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  };
  // one 16-wide step of register set `cur`: contract (x, W) while the fragments of the
  // following step (buffer nbuf, step nks) arrive in the other register set
  auto step = [&](int cur, int nbuf, int nks) {
    const int nx = cur ^ 1;
    frags_a(nbuf, nks, af[nx]);
    __builtin_amdgcn_sched_barrier(0);
    mfma_first(af[cur], bfr[cur]);
    __builtin_amdgcn_sched_barrier(0);
    frags_b(nbuf, nks, bfr[nx]);
    __builtin_amdgcn_sched_barrier(0);
    mfma_rest(af[cur], bfr[cur]);
    __builtin_amdgcn_sched_barrier(0);
  };

#pragma unroll
  for (int s = 0; s < NB; ++s) stage(s, s);
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NB - 1) * LPS)); // slab 0 has landed
  __syncthreads();
  frags_a(0, 0, af[0]);
  frags_b(0, 0, bfr[0]);
  int buf = 0;
  for (int kt = 0; kt < KT2; ++kt) {
    const int nxt = buf + 1 < NB ? buf + 1 : 0;
#pragma unroll
    for (int ks = 0; ks < KS - 1; ++ks) step(ks & 1, buf, ks + 1);
    // last step: slab kt is completely in registers / consumed from LDS
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NB - 2) * LPS)); // slab kt+1 landed, own LDS reads done
    __syncthreads();
    stage(kt + NB, buf);
    step((KS - 1) & 1, nxt, 0);                                  // after the last slab: a landed buffer, values unused
    buf = nxt;
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));               // the surplus loads of the tail land before the workgroup ends

  // acc[i][j][v] of lane l: row m = wm + i*32 + 8*(v/4) + 4*(l/32) + v%4, column n = wn + j*32 + l%32
  if constexpr (GU) {
#pragma unroll
    for (int j = 0; j < WT; j += 2) {
      const int n = n0 + (wn / WE) * (WE / 2) + (j >> 1) * 32 + (lane & 31);
      if (n >= N) continue;
#pragma unroll
      for (int i = 0; i < WT; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          if (m >= M) continue;
          reinterpret_cast<bf16_t*>(Cout)[(int64_t)m * ldc + n] = from_f32<bf16_t>(silu(acc[i][j][v]) * acc[i][j + 1][v]);
        }
      }
    }
    return;
  }
  // Row tiles that lie inside the matrix (all but a ragged last one) take the arm without per-row checks.
  auto epilogue = [&](auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
    for (int j = 0; j < WT; ++j) {
      const int n = n0 + wn + j * 32 + (lane & 31);
      if (n >= N) continue;
      const float bv = bias != nullptr ? bias[n] : 0.f;
#pragma unroll
      for (int i = 0; i < WT; ++i) {
        const int mb = m0 + wm + i * 32 + 4 * (lane >> 5);
        // Residual values are requested in groups, ahead of the group's stores: res and Cout never overlap (the
        // host checks), so nothing orders these loads behind the stores of the group before.
#pragma unroll
        for (int half = 0; half < 2; ++half) {                   // 8 at a time: the accumulators leave few registers
          float rv[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int v = half * 8 + u, m = mb + 8 * (v >> 2) + (v & 3);
            rv[u] = (OUT != GEMM_OUT_BF16 && res != nullptr && (FULL || m < M)) ? res[(int64_t)m * ldres + n] : 0.f;
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int v = half * 8 + u, m = mb + 8 * (v >> 2) + (v & 3);
            if (!FULL && m >= M) continue;
            const float y = acc[i][j][v] + bv + rv[u];
            if (OUT == GEMM_OUT_BF16) reinterpret_cast<bf16_t*>(Cout)[(int64_t)m * ldc + n] = from_f32<bf16_t>(y);
            else reinterpret_cast<float*>(Cout)[(int64_t)m * ldc + n] = y;
          }
        }
      }
    }
  };
  if (m0 + BM <= M) epilogue(std::true_type{}); else epilogue(std::false_type{});
}

// Row kernel in front of the contraction of fp32 activations: optional RMS norm with gain, then rounding to bf16
// (nearest even).  One workgroup per row.
__global__ __launch_bounds__(256) void norm_round_rows_kernel(const float* __restrict__ x, int64_t ldx, const float* __restrict__ gain,
                                                              float eps, bf16_t* __restrict__ xb, int K) {
  const int tid = threadIdx.x;
  const float* xr = x + (int64_t)blockIdx.x * ldx;
  float r = 1.f;
  if (gain != nullptr) {
    float ss = 0.f;
    for (int k = tid * 4; k < K; k += 1024) {
      const float4_t v = *reinterpret_cast<const float4_t*>(xr + k);
      ss = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, ss))));
    }
    ss = group_sum<32>(ss);
    ss += __shfl_xor(ss, 32);
    __shared__ float partsum[4];
    if ((tid & 63) == 0) partsum[tid >> 6] = ss;
    __syncthreads();
    r = 1.0f / sqrtf(((partsum[0] + partsum[1]) + (partsum[2] + partsum[3])) / (float)K + eps);
  }
  uint2* o = reinterpret_cast<uint2*>(xb + (int64_t)blockIdx.x * K);
  for (int k = tid * 4; k < K; k += 1024) {
    float4_t v = *reinterpret_cast<const float4_t*>(xr + k);    // second read of the row: it is in cache
    if (gain != nullptr) v = v * *reinterpret_cast<const float4_t*>(gain + k) * r;
    o[k >> 2] = uint2{pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w)};
  }
}

// out[m, n] = silu(gu[m, n]) * gu[m, N + n], gu fp32 [M, 2N], out bf16.
__global__ __launch_bounds__(256) void swiglu_rows_kernel(const float* __restrict__ gu, bf16_t* __restrict__ out, int64_t ldo, int N) {
  const float* g = gu + (int64_t)blockIdx.x * 2 * N;
  bf16_t* o = out + (int64_t)blockIdx.x * ldo;
  for (int n = threadIdx.x * 4; n < N; n += 1024) {
    const float4_t a = *reinterpret_cast<const float4_t*>(g + n);
    const float4_t u = *reinterpret_cast<const float4_t*>(g + N + n);
    float4_t y;
    y.x = silu(a.x) * u.x; y.y = silu(a.y) * u.y; y.z = silu(a.z) * u.z; y.w = silu(a.w) * u.w;
    *reinterpret_cast<uint2*>(o + n) = uint2{pack_bf16x2(y.x, y.y), pack_bf16x2(y.z, y.w)};
  }
}

__global__ __launch_bounds__(256) void copy_bytes16_kernel(const uint4_t* __restrict__ src, uint4_t* __restrict__ dst, int64_t n16) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx < n16) dst[idx] = src[idx];
}

template <int WT, int OUT, int BK, int NB>
static int32_t launch_gemm_v(int cls, const bf16_t* A, const bf16_t* B, const float* bias, const float* res,
                             int64_t ldres, void* out, int64_t ldc, int64_t M, int N, int K, hipStream_t st) {
  constexpr int BM = 64 * WT;
  constexpr int BN = (OUT == GEMM_OUT_SWIGLU) ? BM / 2 : BM;   // output columns of a tile
  const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (N + BN - 1) / BN;
  const int64_t grid = (int64_t)tiles_m * tiles_n;
  const size_t lds_bytes = (size_t)NB * 2 * BM * BK * 2;
  static bool attr_set = false;                                  // more than 64 KiB of dynamic LDS has to be allowed once
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_kernel<WT, OUT, BK, NB>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return fail(PHOTON_ERR_HIP, "gemm: cannot reserve %zu bytes of LDS: %s", lds_bytes, hipGetErrorString(e));
    attr_set = true;
  }
  PHOTON_LAUNCH(cls, st, (gemm_bf16_kernel<WT, OUT, BK, NB>), dim3((unsigned)grid), dim3(G_THREADS), lds_bytes, st, A, B, bias, res,
                ldres, out, ldc, (int)M, N, K, tiles_m, tiles_n);
  return check_launch("gemm_bf16_kernel");
}

// The 256-wide tile, measured: 64-wide slabs in two buffers.  32-wide slabs in three to five buffers (up to 128 KB in
// flight per compute unit instead of 64 KB) are no faster at the large shapes.
template <int WT, int OUT>
static int32_t launch_gemm_t(int cls, const bf16_t* A, const bf16_t* B, const float* bias, const float* res, int64_t ldres, void* out,
                             int64_t ldc, int64_t M, int N, int K, hipStream_t st) {
  // Small tiles come with few rows (a decode sub-step of a large batch): few slabs' worth of MFMA work per workgroup
  // and often fewer workgroups than compute units, so the wait for a slab is what a slab costs.  Four buffers
  // (three slabs in flight) instead of two: +11-12 % on whole decode steps with 128-256 sequences; six or eight
  // buffers at the 64-wide tile add nothing.
  // With more 128-wide tiles than compute units two buffers are kept: two workgroups then share a unit's LDS, which
  // hides the wait as well and fills the tail better.
  if constexpr (WT == 2) {
    constexpr int BN = (OUT == GEMM_OUT_SWIGLU) ? 64 : 128;
    if (((M + 127) / 128) * ((N + BN - 1) / BN) > 256) return launch_gemm_v<WT, OUT, 64, 2>(cls, A, B, bias, res, ldres, out, ldc, M, N, K, st);
  }
  if constexpr (WT <= 2) return launch_gemm_v<WT, OUT, 64, 4>(cls, A, B, bias, res, ldres, out, ldc, M, N, K, st);
  return launch_gemm_v<WT, OUT, 64, 2>(cls, A, B, bias, res, ldres, out, ldc, M, N, K, st);
}

// Largest tile that still gives the chip enough workgroups.
static int pick_tile(int64_t M, int N) {
  auto tiles = [&](int wt) { return ((M + 64 * wt - 1) / (64 * wt)) * ((N + 64 * wt - 1) / (64 * wt)); };
  if (tiles(4) >= 192) return 4;
  if (tiles(2) >= 128) return 2;
  return 1;
}

template <int OUT>
static int32_t launch_gemm(int cls, const bf16_t* A, const bf16_t* B, const float* bias, const float* res,
                           int64_t ldres, void* out, int64_t ldc, int64_t M, int N, int K, hipStream_t st) {
  switch (pick_tile(M, N)) {
    case 4: return launch_gemm_t<4, OUT>(cls, A, B, bias, res, ldres, out, ldc, M, N, K, st);
    case 2: return launch_gemm_t<2, OUT>(cls, A, B, bias, res, ldres, out, ldc, M, N, K, st);
    default: return launch_gemm_t<1, OUT>(cls, A, B, bias, res, ldres, out, ldc, M, N, K, st);
  }
}

// SwiGLU in the epilogue: N output columns from 2N rows of W.  Returns false when the problem is too small for a
// tile with paired column tiles (the caller then contracts into a [M, 2N] buffer and applies SwiGLU by rows).
static bool launch_gemm_swiglu(int cls, const bf16_t* A, const bf16_t* B, bf16_t* out, int64_t ldc, int64_t M, int N,
                               int K, hipStream_t st, int32_t* rc) {
  auto tiles = [&](int wt) { return ((M + 64 * wt - 1) / (64 * wt)) * ((N + 32 * wt - 1) / (32 * wt)); };
  if (tiles(4) >= 192) *rc = launch_gemm_t<4, GEMM_OUT_SWIGLU>(cls, A, B, nullptr, nullptr, 0, out, ldc, M, N, K, st);
  else if (tiles(2) >= 128) *rc = launch_gemm_t<2, GEMM_OUT_SWIGLU>(cls, A, B, nullptr, nullptr, 0, out, ldc, M, N, K, st);
  else return false;
  return true;
}

static int32_t launch_chunker_gemm(const void* x, const void* w, const float* bias, void* out, int64_t M, int N, int K, hipStream_t st) {
  return launch_gemm<GEMM_OUT_BF16>(KC_CHUNKER_GEMM, (const bf16_t*)x, (const bf16_t*)w, bias, nullptr, 0, out, N, M, N, K, st);
}

size_t linear_many_workspace_bytes(int64_t rows, int K_max, int N2_max) {
  // the activations as bf16, then the gate|up product rows (fp32) of the unfused SwiGLU
  return (size_t)rows * K_max * 2 + (size_t)rows * N2_max * sizeof(float);
}

int32_t launch_norm_round_rows(const float* x, int64_t ldx, const float* gain, float eps, void* xb, int M, int K, hipStream_t st) {
  if (K % 4 != 0 || ldx % 4 != 0) return fail(PHOTON_ERR_UNSUPPORTED, "row kernel: K=%d and the row pitch must be multiples of 4", K);
  PHOTON_LAUNCH(KC_NORM, st, norm_round_rows_kernel, dim3(M), dim3(256), 0, st, x, ldx, gain, eps, reinterpret_cast<bf16_t*>(xb), K);
  return check_launch("norm_round_rows_kernel");
}

int32_t launch_linear_many(const LinearArgs& a, void* workspace, int K_max, hipStream_t st) {
  if (!a.w_bf16 || a.K % G_BK != 0 || a.K > K_max || a.ldx % 4 != 0)
    return fail(PHOTON_ERR_UNSUPPORTED, "many-row linear: needs bf16 weights, K=%d a multiple of 64 and at most %d", a.K, K_max);
  if (a.epilogue == EPI_RESID) {
    const char *r0 = reinterpret_cast<const char*>(a.res), *o0 = reinterpret_cast<const char*>(a.out);
    const char *r1 = r0 + ((int64_t)(a.M - 1) * a.ldres + a.N) * 4, *o1 = o0 + ((int64_t)(a.M - 1) * a.ldo + a.N) * 4;
    if (r0 < o1 && o0 < r1) return fail(PHOTON_ERR_INVALID_ARG, "many-row linear: the residual rows must not overlap the output");
  }
  if (a.out_bf16 != (a.epilogue == EPI_SWIGLU))
    return fail(PHOTON_ERR_UNSUPPORTED, "many-row linear: the SwiGLU product, and only it, is written as bf16");
  if (a.x_bf16) {
    // bf16 rows are the operand as they stand: one pass of the plain contraction
    if (a.gain != nullptr || a.epilogue == EPI_SWIGLU || a.ldx != a.K)
      return fail(PHOTON_ERR_UNSUPPORTED, "many-row linear: bf16 activations come dense, without norm or SwiGLU");
    return launch_gemm<GEMM_OUT_F32>(KC_CHUNKER_GEMM, reinterpret_cast<const bf16_t*>(a.x), (const bf16_t*)a.W, a.bias,
                                     a.epilogue == EPI_RESID ? a.res : nullptr, a.ldres, a.out, a.ldo, a.M, a.N, a.K, st);
  }
  bf16_t* xb = reinterpret_cast<bf16_t*>(workspace);
  float* gu = reinterpret_cast<float*>(xb + (size_t)a.M * K_max);
  PHOTON_LAUNCH(KC_NORM, st, norm_round_rows_kernel, dim3(a.M), dim3(256), 0, st, a.x, a.ldx, a.gain, a.eps, xb, a.K);
  PHOTON_TRY(check_launch("norm_round_rows_kernel"));
  if (a.epilogue == EPI_SWIGLU) {
    if (a.N % 4 != 0) return fail(PHOTON_ERR_UNSUPPORTED, "many-row linear: SwiGLU width %d must be a multiple of 4", a.N);
    int32_t rc = PHOTON_OK;
    bf16_t* act = reinterpret_cast<bf16_t*>(a.out);
    if (launch_gemm_swiglu(KC_CHUNKER_GEMM, xb, (const bf16_t*)a.W, act, a.ldo, a.M, a.N, a.K, st, &rc)) return rc;
    PHOTON_TRY(launch_gemm<GEMM_OUT_F32>(KC_CHUNKER_GEMM, xb, (const bf16_t*)a.W, nullptr, nullptr, 0, gu, 2 * (int64_t)a.N, a.M, 2 * a.N,
                                         a.K, st));
    PHOTON_LAUNCH(KC_SILU_MUL, st, swiglu_rows_kernel, dim3(a.M), dim3(256), 0, st, gu, act, a.ldo, a.N);
    return check_launch("swiglu_rows_kernel");
  }
  return launch_gemm<GEMM_OUT_F32>(KC_CHUNKER_GEMM, xb, (const bf16_t*)a.W, a.bias, a.epilogue == EPI_RESID ? a.res : nullptr, a.ldres,
                                   a.out, a.ldo, a.M, a.N, a.K, st);
}

}  // namespace photon

using namespace photon;

extern "C" int32_t photon_chunker_project(const void* x, const void* w, const float* bias, void* out, int64_t rows,
                                          int32_t C, int32_t d_in, int32_t d_out, photon_dtype dt, void* stream) {
  clear_error();
  PHOTON_REQUIRE(valid_dtype(dt), PHOTON_ERR_UNSUPPORTED, "%s: unknown dtype %d", __func__, (int)dt);
  PHOTON_REQUIRE(rows >= 0 && C >= 1 && d_in >= 1 && d_out >= 1, PHOTON_ERR_INVALID_ARG,
                 "%s: rows=%lld C=%d d_in=%d d_out=%d invalid", __func__, (long long)rows, C, d_in, d_out);
  const int64_t K64 = (int64_t)C * d_in;
  PHOTON_REQUIRE(K64 <= (1 << 24) && rows <= (1LL << 24), PHOTON_ERR_UNSUPPORTED, "%s: problem too large for one launch", __func__);
  const int K = (int)K64;
  if (rows == 0) return PHOTON_OK;
  PHOTON_REQUIRE_PTR(x);
  PHOTON_REQUIRE_PTR(out);
  hipStream_t st = (hipStream_t)stream;
  if (w == nullptr) {
    PHOTON_REQUIRE(d_out == K, PHOTON_ERR_INVALID_ARG, "%s: concatenation without projection needs d_out == C*d_in (%d != %d)",
                   __func__, d_out, K);
    PHOTON_REQUIRE(bias == nullptr, PHOTON_ERR_INVALID_ARG, "%s: bias without a projection matrix", __func__);
    const int64_t bytes = rows * K * (int64_t)dtype_size(dt);
    PHOTON_REQUIRE(bytes % 16 == 0, PHOTON_ERR_UNSUPPORTED, "%s: rows*C*d_in*elem must be a multiple of 16 bytes", __func__);
    PHOTON_LAUNCH(KC_MISC, st, copy_bytes16_kernel, dim3((unsigned)((bytes / 16 + 255) / 256)), dim3(256), 0, st, (const uint4_t*)x,
                       (uint4_t*)out, bytes / 16);
    return check_launch("copy_bytes16_kernel");
  }
  PHOTON_REQUIRE_PTR(w);
  if (dt == PHOTON_F32) {
    PHOTON_REQUIRE(K % 4 == 0, PHOTON_ERR_UNSUPPORTED, "%s: fp32 path needs C*d_in (%d) to be a multiple of 4", __func__, K);
    LinearArgs a;
    a.x = (const float*)x; a.ldx = K; a.W = w; a.bias = bias; a.out = (float*)out; a.ldo = d_out; a.M = (int)rows; a.N = d_out; a.K = K;
    return launch_linear(a, st);
  }
  PHOTON_REQUIRE(K % 64 == 0 && d_out % 16 == 0, PHOTON_ERR_UNSUPPORTED,
                 "%s: bf16 path needs C*d_in (%d) to be a multiple of 64 and d_out (%d) of 16", __func__, K, d_out);
  return launch_chunker_gemm(x, w, bias, out, rows, d_out, K, st);
}
