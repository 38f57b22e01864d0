// Context-chunker projection (paper Eq. 4) at many-row shapes: a dense bf16
// contraction out[M,N] = x[M,K] * W[N,K]^T + bias on the matrix cores.
//
// One workgroup of 4 waves owns a 256x256 output tile; each wave owns a 128x128
// quadrant as 4x4 MFMA 32x32x16 tiles (256 fp32 accumulators per lane).  K is
// walked in 64-wide slabs, double-buffered in LDS (2 x 64 KB); the next slab is
// moved global -> LDS directly (no staging registers) while the current slab's
// MFMAs run, and operand fragments are double-buffered in registers.  LDS rows
// are 128 bytes with the 16-byte column index XOR-ed by (row>>1)&7, which keeps
// the 128-bit operand reads of 16 consecutive rows on distinct banks.  Workgroup ids are remapped so that the tiles resident on one
// XCD at a time share x row-blocks and W column-blocks in that XCD's L2.
#include "photon_device.h"
#include "photon_host.h"
#include "photon_linear.h"

namespace photon {

typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int G_BM = 256, G_BN = 256, G_BK = 64;
constexpr int G_THREADS = 256;
constexpr int G_TILE_BYTES = G_BM * G_BK * 2;          // 32 KB per operand slab

__device__ __forceinline__ int swz(int row, int col16) { return row * 128 + ((col16 ^ ((row >> 1) & 7)) << 4); }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

__global__ __launch_bounds__(G_THREADS) void chunker_gemm_bf16_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, const float* __restrict__ bias, bf16_t* __restrict__ Cout,
    int M, int N, int K, int tiles_m, int tiles_n) {
  extern __shared__ __align__(16) char lds[];                   // [2 buffers][A slab | B slab]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

  // XCD-aware raster: ids are dealt round-robin to 8 XCDs; give each XCD a contiguous run of tiles,
  // column tiles fastest, so concurrent workgroups of an XCD share x row-blocks.
  const int total = tiles_m * tiles_n;
  const int id = blockIdx.x;
  const int logical = (total % 8 == 0) ? (id & 7) * (total / 8) + (id >> 3) : id;   // ragged tile count: plain order
  const int tm = logical / tiles_n, tn = logical % tiles_n;
  const int m0 = tm * G_BM, n0 = tn * G_BN;

  // global -> LDS without passing through registers: one instruction moves 64 lanes x 16 B = 8 slab rows;
  // lane l lands at LDS row l/8, 16-byte column l%8, so it fetches the logical column that the XOR
  // swizzle maps there.  Round i of wave w covers slab rows i*32 + w*8 .. +8.
  const int srow = lane >> 3, scol = lane & 7;
  const bf16_t* aptr[8];
  const bf16_t* bptr[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = i * 32 + wave * 8 + srow;
    const int c = scol ^ ((r >> 1) & 7);
    int ra = m0 + r; ra = ra < M ? ra : M - 1;                   // clamped rows are never stored
    int rb = n0 + r; rb = rb < N ? rb : N - 1;
    aptr[i] = A + (int64_t)ra * K + c * 8;
    bptr[i] = B + (int64_t)rb * K + c * 8;
  }
  auto stage = [&](int kt, int buf) {
    char* sa = lds + buf * 2 * G_TILE_BYTES;
    char* sb = sa + G_TILE_BYTES;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int off = (i * 32 + wave * 8) * 128;
      __builtin_amdgcn_global_load_lds((gptr_t)(aptr[i] + (int64_t)kt * G_BK), (lptr_t)(sa + off), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((gptr_t)(bptr[i] + (int64_t)kt * G_BK), (lptr_t)(sb + off), 16, 0, 0);
    }
  };

  float16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;       // wave quadrant inside the tile
  const int frow = lane & 31, fk = lane >> 5;                    // operand fragment: row, 8-wide k group

  // Pipeline over 64-wide K slabs with ONE barrier per slab, placed before the slab's last quarter:
  //   MFMA(ks=0..2 of slab kt)  [reads of ks+1 issued ahead]
  //   wait for slab kt+1 (its global->LDS loads were issued a whole slab ago), barrier
  //     -> every wave has finished reading slab kt, so its buffer can take slab kt+2 right away
  //   issue slab kt+2, read the first fragments of slab kt+1, MFMA(ks=3 of slab kt)
  // so neither the load wait nor the first fragment reads of a slab leave the matrix cores idle.
  const int KT = K / G_BK;
  constexpr int KS = G_BK / 16;
  bf16x8_t af[2][4], bfr[2][4];
  auto frags = [&](int buf, int ks, bf16x8_t (&a)[4], bf16x8_t (&b)[4]) {
    const char* sa = lds + buf * 2 * G_TILE_BYTES;
    const char* sb = sa + G_TILE_BYTES;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4_t*>(sa + swz(wm + i * 32 + frow, ks * 2 + fk)));
      b[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4_t*>(sb + swz(wn + i * 32 + frow, ks * 2 + fk)));
    }
  };
  auto mfma16 = [&](const bf16x8_t (&a)[4], const bf16x8_t (&b)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  };

  stage(0, 0);
  if (KT > 1) stage(1, 1);
  __builtin_amdgcn_s_waitcnt(0);                                 // both slabs have landed (vmcnt(0))
  __syncthreads();
  frags(0, 0, af[0], bfr[0]);
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
#pragma unroll
    for (int ks = 0; ks < KS - 1; ++ks) {
      frags(buf, ks + 1, af[(ks + 1) & 1], bfr[(ks + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);
      mfma16(af[ks & 1], bfr[ks & 1]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // last quarter: slab kt is completely in registers / consumed from LDS
    __builtin_amdgcn_s_waitcnt(0);                               // slab kt+1 landed, own LDS reads done
    __syncthreads();
    if (kt + 2 < KT) stage(kt + 2, buf);
    if (kt + 1 < KT) frags(buf ^ 1, 0, af[KS & 1], bfr[KS & 1]);
    __builtin_amdgcn_sched_barrier(0);
    mfma16(af[(KS - 1) & 1], bfr[(KS - 1) & 1]);
    __builtin_amdgcn_sched_barrier(0);
  }

  // acc[i][j][v] of lane l: row m = wm + i*32 + 8*(v/4) + 4*(l/32) + v%4, column n = wn + j*32 + l%32
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int n = n0 + wn + j * 32 + (lane & 31);
    if (n >= N) continue;
    const float bv = bias != nullptr ? bias[n] : 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (m < M) Cout[(int64_t)m * N + n] = from_f32<bf16_t>(acc[i][j][v] + bv);
      }
    }
  }
}

__global__ __launch_bounds__(256) void copy_bytes16_kernel(const uint4_t* __restrict__ src, uint4_t* __restrict__ dst, int64_t n16) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx < n16) dst[idx] = src[idx];
}

static int32_t launch_chunker_gemm(const void* x, const void* w, const float* bias, void* out, int64_t M, int N, int K, hipStream_t st) {
  const int tiles_m = (int)((M + G_BM - 1) / G_BM), tiles_n = (N + G_BN - 1) / G_BN;
  const int64_t grid = (int64_t)tiles_m * tiles_n;
  static bool attr_set = false;
  const size_t lds_bytes = 4 * G_TILE_BYTES;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(chunker_gemm_bf16_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return fail(PHOTON_ERR_HIP, "chunker gemm: cannot reserve %zu bytes of LDS: %s", lds_bytes, hipGetErrorString(e));
    attr_set = true;
  }
  PHOTON_LAUNCH(KC_CHUNKER_GEMM, st, chunker_gemm_bf16_kernel, dim3((unsigned)grid), dim3(G_THREADS), lds_bytes, st, (const bf16_t*)x,
                     (const bf16_t*)w, bias, (bf16_t*)out, (int)M, N, K, tiles_m, tiles_n);
  return check_launch("chunker_gemm_bf16_kernel");
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
