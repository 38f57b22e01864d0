// Linear maps of the decode path, y[M,N] = x[M,K] * W[N,K]^T (+ bias) (+ residual),
// for few rows M (decode sub-steps carry one row per chunk in flight).
//
// These are weight-streaming kernels: every weight byte is read once per call
// and the M activations ride along.  bf16 weights go through the matrix cores
// only because the per-byte arithmetic (M multiply-adds per weight) would
// otherwise occupy the vector ALUs; the kernel is HBM-bound by construction:
//   * each lane issues 2 x 128-bit loads per 64-wide k block so that every
//     weight row is fetched in whole 128-byte lines,
//   * the k order inside a block is permuted identically for both MFMA
//     operands (a contraction does not care), which is what makes those
//     contiguous loads line up with the 16x16x32 operand layout,
//   * fp32 activations are split into a bf16 head and a bf16 remainder and
//     both are multiplied (two MFMAs per weight fragment), so the result is as
//     accurate as an fp32-activation x bf16-weight product,
//   * K is split over workgroups to fill the chip; each split writes its partial
//     tile to a workspace and whichever kernel consumes the result (a norm, the
//     rotary/append kernel, the SwiGLU gate, or the plain reduce kernel below)
//     adds the splits in split order.  No atomics, no in-kernel fences: the
//     kernel boundary is the synchronisation, and the result is deterministic.
#include "photon_linear.h"

#include "photon_device.h"
#include "photon_host.h"

namespace photon {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int SK_THREADS = 256;
constexpr int SK_WAVES = 4;
constexpr int SK_KBLOCK = 64;                 // k elements per block: 128 bytes of a weight row
constexpr int SK_CHUNK_BLOCKS = 4;            // blocks staged in LDS at a time (256 k)
constexpr int SK_NB = 16 * SK_WAVES;          // output columns per workgroup

__device__ __forceinline__ bf16x8_t as_bf16x8(const uint4_t& v) { return __builtin_bit_cast(bf16x8_t, v); }

// Split 8 fp32 values into bf16 heads and bf16 remainders, packed for one MFMA operand each.
__device__ __forceinline__ void split_hi_lo(const float (&v)[8], uint4_t& hi, uint4_t& lo) {
  uint32_t h[8], l[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    h[i] = f32_to_bf16_bits(v[i]);
    const float rem = v[i] - __uint_as_float(h[i] << 16);
    l[i] = f32_to_bf16_bits(rem);
  }
  hi.x = h[0] | (h[1] << 16); hi.y = h[2] | (h[3] << 16); hi.z = h[4] | (h[5] << 16); hi.w = h[6] | (h[7] << 16);
  lo.x = l[0] | (l[1] << 16); lo.y = l[2] | (l[3] << 16); lo.z = l[4] | (l[5] << 16); lo.w = l[6] | (l[7] << 16);
}

template <typename TX> struct XLoad;
template <> struct XLoad<float> {
  static constexpr bool SPLIT = true;
  __device__ static __forceinline__ void load8(const float* p, float (&v)[8]) {
    const float4_t a = *reinterpret_cast<const float4_t*>(p);
    const float4_t b = *reinterpret_cast<const float4_t*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};
template <> struct XLoad<bf16_t> {
  static constexpr bool SPLIT = false;
  __device__ static __forceinline__ void load8(const bf16_t* p, float (&v)[8]) { unpack16<bf16_t>(load16(p), v); }
};

// MT = number of 16-row activation tiles (M <= 16*MT).
template <typename TX, int MT>
__global__ __launch_bounds__(SK_THREADS) void skinny_gemm_bf16_kernel(
    const TX* __restrict__ x, int64_t ldx, const bf16_t* __restrict__ W, const float* __restrict__ bias,
    const float* res, int64_t ldres, float* out, int64_t ldo,
    int M, int N, int K, int direct, int blocks_per_split, float* __restrict__ partial, int64_t split_stride) {
  constexpr bool SPLIT = XLoad<TX>::SPLIT;
  constexpr int CB = SK_CHUNK_BLOCKS;
  // operand fragments of the activations: [m-tile][block][half][lane] x 16 bytes
  __shared__ uint4_t xh[MT][CB][2][64];
  __shared__ uint4_t xl[SPLIT ? MT : 1][SPLIT ? CB : 1][SPLIT ? 2 : 1][SPLIT ? 64 : 1];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nblock = blockIdx.x, ks = blockIdx.y;
  const int n0 = nblock * SK_NB + wave * 16;
  const bool wave_live = n0 < N;                       // N is a multiple of 16
  const int lrow = lane & 15, lq = lane >> 4;

  const int total_blocks = K / SK_KBLOCK;
  const int blk_begin = ks * blocks_per_split;
  const int blk_end = min(blk_begin + blocks_per_split, total_blocks);

  float4_t acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = float4_t{0.f, 0.f, 0.f, 0.f};

  const bf16_t* wrow = W + (int64_t)(wave_live ? n0 + lrow : 0) * K + lq * 16;

  uint4_t wf[CB][2];
  auto load_w = [&](int blk0) {
#pragma unroll
    for (int b = 0; b < CB; ++b) {
      int blk = blk0 + b;
      blk = blk < blk_end ? blk : blk_end - 1;                 // clamped: stays in bounds, result unused
      const bf16_t* p = wrow + (int64_t)blk * SK_KBLOCK;
      wf[b][0] = load16_stream(p);
      wf[b][1] = load16_stream(p + 8);
    }
  };

  for (int blk0 = blk_begin; blk0 < blk_end; blk0 += CB) {
    if (wave_live) load_w(blk0);                               // weight loads fly while x is staged
    __syncthreads();                                           // previous chunk's fragments are consumed
    // stage activations: groups of 8 consecutive k of one row -> one operand fragment
    constexpr int GROUPS = MT * 16 * CB * 8;
    for (int idx = tid; idx < GROUPS; idx += SK_THREADS) {
      const int m = idx / (CB * 8), kg = idx % (CB * 8);
      const int b = kg >> 3, gi = kg & 7, q = gi >> 1, half = gi & 1;
      const int blk = blk0 + b;
      float v[8];
      if (m < M && blk < blk_end) {
        XLoad<TX>::load8(x + (int64_t)m * ldx + (int64_t)blk * SK_KBLOCK + gi * 8, v);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = 0.f;
      }
      const int slot = q * 16 + (m & 15);
      if (SPLIT) {
        uint4_t hi, lo;
        split_hi_lo(v, hi, lo);
        xh[m >> 4][b][half][slot] = hi;
        xl[m >> 4][b][half][slot] = lo;
      } else {
        uint4_t hi;
        hi.x = pack_bf16x2(v[0], v[1]); hi.y = pack_bf16x2(v[2], v[3]);
        hi.z = pack_bf16x2(v[4], v[5]); hi.w = pack_bf16x2(v[6], v[7]);
        xh[m >> 4][b][half][slot] = hi;
      }
    }
    __syncthreads();
    if (wave_live) {
#pragma unroll
      for (int b = 0; b < CB; ++b) {
        if (blk0 + b < blk_end) {
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const bf16x8_t a = as_bf16x8(wf[b][half]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
              acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, as_bf16x8(xh[mt][b][half][lane]), acc[mt], 0, 0, 0);
              if (SPLIT)
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, as_bf16x8(xl[mt][b][half][lane]), acc[mt], 0, 0, 0);
            }
          }
        }
      }
    }
  }

  // acc[mt] of lane l holds y[m = mt*16 + l%16][n = n0 + (l/16)*4 + 0..3]
  const int n_out = n0 + lq * 4;
  auto finish = [&](int m, float4_t v) {
    if (bias != nullptr) {
      const float4_t bv = *reinterpret_cast<const float4_t*>(bias + n_out);
      v += bv;
    }
    if (res != nullptr) {
      const float4_t rv = *reinterpret_cast<const float4_t*>(res + (int64_t)m * ldres + n_out);
      v += rv;
    }
    *reinterpret_cast<float4_t*>(out + (int64_t)m * ldo + n_out) = v;
  };

  if (direct) {
    if (wave_live) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + lrow;
        if (m < M) finish(m, acc[mt]);
      }
    }
    return;
  }

  // split-K: park the partial tile [ks][m][n]; the consumer adds the splits
  if (wave_live) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = mt * 16 + lrow;
      if (m < M) *reinterpret_cast<float4_t*>(partial + (int64_t)ks * split_stride + (int64_t)m * N + n_out) = acc[mt];
    }
  }
}

// out[m, n] = sum_s part[s][m][n] (+ bias[n]) (+ res[m, n])
__global__ __launch_bounds__(256) void reduce_splits_kernel(const float* __restrict__ part, int ks, int64_t split_stride,
                                                            const float* __restrict__ bias, const float* res, int64_t ldres,
                                                            float* out, int64_t ldo, int M, int N) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)M * N) return;
  const int n = (int)(idx % N);
  const int64_t m = idx / N;
  float v = 0.f;
  for (int s2 = 0; s2 < ks; ++s2) v += part[(int64_t)s2 * split_stride + m * N + n];
  if (bias != nullptr) v += bias[n];
  if (res != nullptr) v += res[m * ldres + n];
  out[m * ldo + n] = v;
}

// fp32 weights (the small all-fp32 configuration): one wave per output column,
// lanes stride over k with 128-bit loads, up to 16 rows accumulate per pass.
constexpr int F32_ROWS = 16;
template <int DUMMY>
__global__ __launch_bounds__(256) void gemm_f32_kernel(
    const float* __restrict__ x, int64_t ldx, const float* __restrict__ W, const float* __restrict__ bias,
    const float* res, int64_t ldres, float* out, int64_t ldo, int M, int N, int K) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int m0 = blockIdx.y * F32_ROWS;
  if (n >= N) return;
  float acc[F32_ROWS];
#pragma unroll
  for (int r = 0; r < F32_ROWS; ++r) acc[r] = 0.f;
  const float* wr = W + (int64_t)n * K;
  for (int k = lane * 4; k < K; k += 256) {
    const float4_t w4 = *reinterpret_cast<const float4_t*>(wr + k);
#pragma unroll
    for (int r = 0; r < F32_ROWS; ++r) {
      if (m0 + r < M) {
        const float4_t x4 = *reinterpret_cast<const float4_t*>(x + (int64_t)(m0 + r) * ldx + k);
        acc[r] = fmaf(w4.x, x4.x, acc[r]);
        acc[r] = fmaf(w4.y, x4.y, acc[r]);
        acc[r] = fmaf(w4.z, x4.z, acc[r]);
        acc[r] = fmaf(w4.w, x4.w, acc[r]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < F32_ROWS; ++r) {
    float v = group_sum<32>(acc[r]);
    v += __shfl_xor(v, 32);
    if (lane == 0 && m0 + r < M) {
      if (bias != nullptr) v += bias[n];
      if (res != nullptr) v += res[(int64_t)(m0 + r) * ldres + n];
      out[(int64_t)(m0 + r) * ldo + n] = v;
    }
  }
}

size_t linear_workspace_bytes(int max_rows, int max_N) {
  const size_t mpad = (size_t)(max_rows + 15) / 16 * 16;
  if (max_rows > 64) return mpad * (size_t)max_N * sizeof(float);            // many rows: K is not split
  return mpad * (size_t)(LINEAR_TARGET_WORKGROUPS * SK_NB + max_N + SK_NB) * sizeof(float);
}

static int choose_ksplit(int n_blocks, int total_kblocks) {
  int ks = (LINEAR_TARGET_WORKGROUPS + n_blocks - 1) / n_blocks;
  const int max_by_k = (total_kblocks + SK_CHUNK_BLOCKS - 1) / SK_CHUNK_BLOCKS;
  if (ks > max_by_k) ks = max_by_k;
  if (ks > LINEAR_MAX_KSPLIT) ks = LINEAR_MAX_KSPLIT;
  if (ks < 1) ks = 1;
  return ks;
}

template <typename TX>
static int32_t launch_skinny(const LinearArgs& a, int m0, int m_rows, int ks, int bps, bool direct, float* partial,
                             int64_t split_stride, hipStream_t st) {
  const int n_blocks = (a.N + SK_NB - 1) / SK_NB;
  const size_t xsz = sizeof(TX);
  const TX* x = reinterpret_cast<const TX*>(reinterpret_cast<const char*>(a.x) + (size_t)m0 * a.ldx * xsz);
  const float* res = (direct && a.res) ? a.res + (int64_t)m0 * a.ldres : nullptr;
  const float* bias = direct ? a.bias : nullptr;
  float* out = direct ? a.out + (int64_t)m0 * a.ldo : nullptr;
  float* part = direct ? nullptr : partial + (int64_t)m0 * a.N;
  dim3 grid(n_blocks, ks);
  const int mt = (m_rows + 15) / 16;
#define PHOTON_SK_LAUNCH(MTV)                                                                                    \
  PHOTON_LAUNCH(KC_SKINNY_GEMM, st, (skinny_gemm_bf16_kernel<TX, MTV>), grid, dim3(SK_THREADS), 0, st, x, a.ldx, (const bf16_t*)a.W, \
                     bias, res, a.ldres, out, a.ldo, m_rows, a.N, a.K, direct ? 1 : 0, bps, part, split_stride)
  switch (mt) {
    case 1: PHOTON_SK_LAUNCH(1); break;
    case 2: PHOTON_SK_LAUNCH(2); break;
    case 3: PHOTON_SK_LAUNCH(3); break;
    case 4: PHOTON_SK_LAUNCH(4); break;
    default: return fail(PHOTON_ERR_UNSUPPORTED, "linear: %d rows in one pass", m_rows);
  }
#undef PHOTON_SK_LAUNCH
  return check_launch("skinny_gemm_bf16_kernel");
}

// Enqueue the product.  With pend == nullptr the complete result (bias, residual) lands in a.out.
// With pend != nullptr the caller's next kernel consumes *pend: value = sum_s data[s*split_stride + m*ld + n],
// bias and residual are NOT applied and a.out is not written.
int32_t launch_linear(const LinearArgs& a, Pending* pend, hipStream_t st) {
  if (a.M <= 0) { if (pend) *pend = Pending{}; return PHOTON_OK; }
  if (a.w_bf16) {
    if (a.K % SK_KBLOCK != 0 || a.N % 16 != 0)
      return fail(PHOTON_ERR_UNSUPPORTED, "linear (bf16): K=%d must be a multiple of 64 and N=%d of 16", a.K, a.N);
    const int n_blocks = (a.N + SK_NB - 1) / SK_NB;
    const int total_kblocks = a.K / SK_KBLOCK;
    int ks = a.M > 64 ? 1 : choose_ksplit(n_blocks, total_kblocks);
    int bps = (total_kblocks + ks - 1) / ks;
    bps = (bps + SK_CHUNK_BLOCKS - 1) / SK_CHUNK_BLOCKS * SK_CHUNK_BLOCKS;
    ks = (total_kblocks + bps - 1) / bps;
    const int64_t mpad = (int64_t)(a.M + 15) / 16 * 16;
    const int64_t split_stride = mpad * a.N;
    const size_t need = (size_t)ks * split_stride * sizeof(float);
    const bool have_ws = a.workspace != nullptr && a.workspace_bytes >= need;
    if (!have_ws) {
      if (pend) return fail(PHOTON_ERR_WORKSPACE, "linear: %zu bytes of workspace needed (got %zu)", need, a.workspace_bytes);
      ks = 1; bps = total_kblocks;
    }
    const bool direct = (pend == nullptr) && ks == 1;
    float* partial = reinterpret_cast<float*>(a.workspace);
    for (int m0 = 0; m0 < a.M; m0 += 64) {
      const int rows = a.M - m0 < 64 ? a.M - m0 : 64;
      const int32_t rc = a.x_bf16 ? launch_skinny<bf16_t>(a, m0, rows, ks, bps, direct, partial, split_stride, st)
                                  : launch_skinny<float>(a, m0, rows, ks, bps, direct, partial, split_stride, st);
      if (rc != PHOTON_OK) return rc;
    }
    if (pend) { pend->data = partial; pend->ks = ks; pend->split_stride = split_stride; pend->ld = a.N; return PHOTON_OK; }
    if (direct) return PHOTON_OK;
    const int64_t total = (int64_t)a.M * a.N;
    PHOTON_LAUNCH(KC_REDUCE_SPLITS, st, reduce_splits_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, partial, ks, split_stride,
                       a.bias, a.res, a.ldres, a.out, a.ldo, a.M, a.N);
    return check_launch("reduce_splits_kernel");
  }
  if (a.x_bf16) return fail(PHOTON_ERR_UNSUPPORTED, "linear: bf16 activations need bf16 weights");
  if (a.K % 4 != 0) return fail(PHOTON_ERR_UNSUPPORTED, "linear (fp32): K=%d must be a multiple of 4", a.K);
  dim3 grid((a.N + 3) / 4, (a.M + F32_ROWS - 1) / F32_ROWS);
  if (pend) {
    const size_t need = (size_t)a.M * a.N * sizeof(float);
    if (a.workspace == nullptr || a.workspace_bytes < need)
      return fail(PHOTON_ERR_WORKSPACE, "linear: %zu bytes of workspace needed (got %zu)", need, a.workspace_bytes);
    float* partial = reinterpret_cast<float*>(a.workspace);
    PHOTON_LAUNCH(KC_GEMM_F32, st, (gemm_f32_kernel<0>), grid, dim3(256), 0, st, (const float*)a.x, a.ldx, (const float*)a.W,
                       (const float*)nullptr, (const float*)nullptr, (int64_t)0, partial, (int64_t)a.N, a.M, a.N, a.K);
    pend->data = partial; pend->ks = 1; pend->split_stride = (int64_t)a.M * a.N; pend->ld = a.N;
    return check_launch("gemm_f32_kernel");
  }
  PHOTON_LAUNCH(KC_GEMM_F32, st, (gemm_f32_kernel<0>), grid, dim3(256), 0, st, (const float*)a.x, a.ldx, (const float*)a.W, a.bias,
                     a.res, a.ldres, a.out, a.ldo, a.M, a.N, a.K);
  return check_launch("gemm_f32_kernel");
}

}  // namespace photon

using namespace photon;

extern "C" size_t photon_linear_workspace_bytes(int32_t M, int32_t N) {
  if (M <= 0 || N <= 0) return 0;
  return linear_workspace_bytes(M, N);
}

extern "C" int32_t photon_linear(const float* x, const void* w, const float* bias, const float* res, float* out, int32_t M,
                                 int32_t N, int32_t K, void* workspace, size_t workspace_bytes, photon_dtype dt, void* stream) {
  clear_error();
  PHOTON_REQUIRE(valid_dtype(dt), PHOTON_ERR_UNSUPPORTED, "%s: unknown dtype %d", __func__, (int)dt);
  PHOTON_REQUIRE(M >= 0 && N > 0 && K > 0, PHOTON_ERR_INVALID_ARG, "%s: M=%d N=%d K=%d invalid", __func__, M, N, K);
  if (M == 0) return PHOTON_OK;
  PHOTON_REQUIRE_PTR(x);
  PHOTON_REQUIRE_PTR(w);
  PHOTON_REQUIRE_PTR(out);
  PHOTON_REQUIRE(workspace == nullptr || aligned16(workspace), PHOTON_ERR_WORKSPACE, "%s: workspace is misaligned", __func__);
  LinearArgs a;
  a.x = x; a.ldx = K; a.W = w; a.w_bf16 = (dt == PHOTON_BF16); a.bias = bias; a.res = res; a.ldres = N; a.out = out; a.ldo = N;
  a.M = M; a.N = N; a.K = K; a.workspace = workspace; a.workspace_bytes = workspace_bytes;
  return launch_linear(a, nullptr, (hipStream_t)stream);
}
