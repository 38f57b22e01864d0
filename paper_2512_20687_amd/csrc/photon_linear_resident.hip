// Few-row linear maps, variant with the activations resident in LDS.
//
// What bounds a few-row linear map on this chip is not HBM alone but the bytes
// each compute unit has to take in: its share of the weights plus ALL of the
// activations it multiplies them with (every workgroup needs every k).  With
// one output tile per workgroup the fp32 activations (64 B per k at 16 rows)
// outweigh a tile's weights (32 B per k), and they are re-read, re-scaled and
// re-split for every tile.  This kernel therefore
//   * spreads the output columns evenly over (up to) one workgroup per compute
//     unit, in units of 8 weight rows, several units per workgroup.  A unit is
//     one MFMA tile: 8 output columns, or for SwiGLU the 4 gate rows and the 4
//     matching up rows of 4 output columns; the two halves of every 128-byte
//     line are folded into the tile's two row halves (one load instruction then fetches whole
//     lines and no lane carries a duplicate: a compute unit's load path is the
//     scarce resource, and a load that hits in cache costs it as much as one
//     that misses);
//   * reads, normalises and splits the activations ONCE per workgroup into
//     MFMA operand order (bf16 head + bf16 remainder) and keeps them in LDS,
//     each of the 8 waves holding the k chunks it contracts over;
//   * then only streams weights: per k chunk the operand fragments come out of
//     LDS once and meet every tile's weight fragments.
// It applies whenever the split activations fit in LDS; larger cases take the
// streaming kernel.  Summation order is fixed (waves in order), as there.
#include "photon_linear.h"

#include "photon_device.h"
#include "photon_host.h"

namespace photon {

namespace {

constexpr int RL_WAVES = 8;
constexpr int RL_THREADS = RL_WAVES * 64;
constexpr int RL_KBLOCK = 64;                  // k per block: 128 bytes of a weight row
constexpr int RL_CB = 2;                       // blocks per chunk
constexpr int RL_CHUNK_K = RL_CB * RL_KBLOCK;
constexpr int RL_LDS_LIMIT = 156 * 1024;

// bytes of one fragment group (one 8-k group of ROWS rows, 16 bytes each) incl. padding that spreads groups over banks
__host__ __device__ constexpr int rl_group_pitch(int rows) { return rows * 16 + 16; }
// one chunk of one wave: 16 groups of heads, then 16 groups of remainders
__host__ __device__ constexpr int rl_chunk_bytes(int rows) { return 2 * 16 * rl_group_pitch(rows); }

// EPI as in LinearEpilogue; XP: live slab pieces per lane (rows = 2*XP of the 16-row tile are live);
// NORM: RMS pre-norm with gain; TMAX: units per workgroup (register-resident accumulators).
// XB: the activations are bf16 already (the feed-forward's hidden rows): they ARE the operand, so each lane
// loads its fragments (8 consecutive k of its row, 16 bytes) straight from memory beside the weights of the
// same chunk; nothing is staged, normalised or split, LDS only carries the final reduction, and K is not
// limited by LDS.  Rows beyond M are not loaded (their accumulator columns are never stored).
//
// Columns are dealt in units of 8 (SwiGLU: 4): workgroup g owns units [u0, u0 + cnt).  A unit's 8 weight rows form one
// MFMA tile (SwiGLU: 4 gate rows, then the 4 up rows of the same columns): tile row r and r + 8 are weight row r;
// lanes of rows 0..7 load the first 64 bytes of a k block's 128-byte line, lanes of rows 8..15 the second 64,
// so one load per block fetches whole lines.  The first MFMA of a block uses the registers as loaded, the second
// after a rotation by 8 lanes inside each row of 16, which brings the second half under rows 0..7.  Accumulator
// rows 8..15 are meaningless; a unit's 8 weight rows sit in rows 0..7 (lanes 0..31).
// RT (bf16 activations only): row tiles of 16 per workgroup.  With 32-127 rows every weight fragment, once in registers,
// meets the fragments of RT row tiles, so the weights are streamed once per RT*16 rows instead of once per 16.
template <int EPI, int XP, bool NORM, int TMAX, bool XB, int RT = 1>
__global__ __launch_bounds__(RL_THREADS) void resident_linear_bf16_kernel(
    const float* __restrict__ x, int64_t ldx, const bf16_t* __restrict__ W, const float* __restrict__ gain, float eps,
    const float* __restrict__ bias, const float* res, int64_t ldres, float* out, int64_t ldo, int M, int N, int K,
    int unit_base, int unit_rem, int wave_bytes, int out_bf16) {
  static_assert(!XB || !NORM, "bf16 activations come without a pre-norm");
  static_assert(XB || RT == 1, "several row tiles per workgroup: bf16 activations only");
  constexpr int CB = RL_CB;
  constexpr int ROWS = 2 * XP;
  constexpr int GP = rl_group_pitch(ROWS);
  constexpr int CHUNK_BYTES = rl_chunk_bytes(ROWS);
  constexpr int TT = TMAX;                                         // MFMA tiles, one per unit
  constexpr int UC = (EPI == EPI_SWIGLU) ? 4 : 8;                  // output columns of a unit
  extern __shared__ __align__(16) char smem[];                     // [8 waves][wave_bytes], then row statistics [8][16]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lrow = lane & 15, lq = lane >> 4;
  const int m0 = blockIdx.y * (16 * RT);
  char* my_area = smem + wave * wave_bytes;
  float* ssum = reinterpret_cast<float*>(smem + RL_WAVES * wave_bytes);

  const int g = blockIdx.x;
  const int u_cnt = unit_base + (g < unit_rem ? 1 : 0);
  const int u0 = g * unit_base + (g < unit_rem ? g : unit_rem);
  const int tiles = u_cnt;                                         // 1 .. TMAX
  const int n0 = u0 * UC;

  // weight row of this lane in every tile, as a byte offset from W (host checks that all of W is below 4 GiB)
  uint32_t w_lane[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int uu = t < tiles ? t : tiles - 1;                      // surplus units repeat the last one (loaded, never stored)
    const int r = lrow & 7;
    // SwiGLU: tile rows 0..3 are gate rows, 4..7 the up rows of the same columns (stored after the N gate rows)
    const int n = (EPI == EPI_SWIGLU) ? (r < 4 ? 0 : N) + n0 + uu * 4 + (r & 3) : n0 + uu * 8 + r;
    w_lane[t] = ((uint32_t)n * (uint32_t)K + (uint32_t)(lq + 4 * (lrow >> 3)) * 8u) * 2u;
  }
  const char* w_base = reinterpret_cast<const char*>(W);

  const int total_blocks = K / RL_KBLOCK;
  const int chunks = (total_blocks + CB - 1) / CB;
  const int n_my = wave < chunks ? (chunks - wave + RL_WAVES - 1) / RL_WAVES : 0;   // this wave contracts chunks wave, wave+8, ..

  struct Operands {
    uint4_t w[TT][CB];                                             // weight fragments of one chunk
    uint4_t xf[RT][XB ? CB : 1][2];                                // XB: its activation fragments, per row tile
  };
  float4_t acc[RT][TT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int t = 0; t < TT; ++t) acc[rt][t] = float4_t{0.f, 0.f, 0.f, 0.f};
  float ss[XP];
#pragma unroll
  for (int i = 0; i < XP; ++i) ss[i] = 0.f;

  // ---- loads: unconditional, clamped into bounds, so that the load counter can be waited on exactly ----
  // bf16 activations: fragment (block b, half) of this lane = k b*64 + half*32 + lq*8 .. +8 of row m0 + lrow
  bool xf_live[RT];
  const char* xf_lane[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    xf_live[rt] = m0 + rt * 16 + lrow < M;
    xf_lane[rt] = reinterpret_cast<const char*>(x) + ((int64_t)(xf_live[rt] ? m0 + rt * 16 + lrow : 0) * ldx + lq * 8) * 2;
  }
  auto load_w = [&](int j, Operands& o) {
    const int chunk = wave + j * RL_WAVES;
    if (XB) {                                                      // the (cached) activations first, as below
#pragma unroll
      for (int b = 0; b < CB; ++b) {
        int blk = chunk * CB + b;
        blk = blk < total_blocks ? blk : total_blocks - 1;
#pragma unroll
        for (int half2 = 0; half2 < 2; ++half2)
#pragma unroll
          for (int rt = 0; rt < RT; ++rt) {
            o.xf[rt][b][half2] = uint4_t{0u, 0u, 0u, 0u};
            if (xf_live[rt]) o.xf[rt][b][half2] = load16(xf_lane[rt] + (int64_t)blk * (RL_KBLOCK * 2) + half2 * 64);
          }
      }
    }
#pragma unroll
    for (int b = 0; b < CB; ++b) {
      int blk = chunk * CB + b;
      blk = blk < total_blocks ? blk : total_blocks - 1;
      const char* wb = w_base + (int64_t)blk * (RL_KBLOCK * 2);
#pragma unroll
      for (int t = 0; t < TT; ++t) o.w[t][b] = load16_stream(wb + w_lane[t]);   // used once: keep it from displacing the activations
                                                                                // (ordinary loads: the whole decode step 4 % slower)
    }
  };
  // slab piece i of a lane: row i*2 + lane/32, k offset (lane%32)*4 inside the chunk
  const int c4 = lane & 31;
  uint32_t x_lane[XP];
#pragma unroll
  for (int i = 0; i < XP; ++i) {
    int m = m0 + i * 2 + (lane >> 5);
    m = m < M ? m : M - 1;
    x_lane[i] = (uint32_t)((int64_t)(m - m0) * ldx + (c4 & 15) * 4) * 4u;
  }
  const char* x_tile = reinterpret_cast<const char*>(x + (int64_t)m0 * ldx);
  auto load_x = [&](int j, float4_t (&xr)[XP + 1]) {
    if (XB) return;
    const int chunk = wave + j * RL_WAVES;
    int blk = chunk * CB + (c4 >> 4);
    blk = blk < total_blocks ? blk : total_blocks - 1;
    const uint32_t kb = (uint32_t)blk * (RL_KBLOCK * 4);
#pragma unroll
    for (int i = 0; i < XP; ++i) xr[i] = *reinterpret_cast<const float4_t*>(x_tile + (x_lane[i] + kb));
    if (NORM) xr[XP] = *reinterpret_cast<const float4_t*>(reinterpret_cast<const char*>(gain) + (kb + (c4 & 15) * 16));
  };
  // scale, split and store chunk j in operand order: group (block, half, q) holds k = b*64 + half*32 + q*8 .. +8 of every row
  auto stage = [&](int j, const float4_t (&xr)[XP + 1]) {
    if (XB) return;
    const int chunk = wave + j * RL_WAVES;
    char* hi = my_area + j * CHUNK_BYTES;
    char* lo = hi + 16 * GP;
    const bool k_live = chunk * RL_CHUNK_K + c4 * 4 < K;
    const int group = c4 >> 1;
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const int row = i * 2 + (lane >> 5);
      float4_t v = (k_live && m0 + row < M) ? xr[i] : float4_t{0.f, 0.f, 0.f, 0.f};
      ss[i] = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, ss[i]))));
      if (NORM) v *= xr[XP];
      uint32_t h01, l01, h23, l23;
      split_bf16x2(v.x, v.y, h01, l01);
      split_bf16x2(v.z, v.w, h23, l23);
      const int off = group * GP + row * 16 + (c4 & 1) * 8;
      *reinterpret_cast<uint2*>(hi + off) = uint2{h01, h23};
      *reinterpret_cast<uint2*>(lo + off) = uint2{l01, l23};
    }
  };
  const int frag_row = (lrow & (ROWS - 1)) * 16;                   // dead rows read a live row's fragment: never stored
  auto mma = [&](int j, const Operands& o) {
    const int chunk = wave + j * RL_WAVES;
    const char* hi = my_area + j * CHUNK_BYTES;
    const char* lo = hi + 16 * GP;
#pragma unroll
    for (int b = 0; b < CB; ++b) {
      if (chunk * CB + b < total_blocks) {
#pragma unroll
        for (int half2 = 0; half2 < 2; ++half2) {
          if constexpr (XB) {
#pragma unroll
            for (int t = 0; t < TT; ++t) {
              const bf16x8_t a = as_bf16x8(half2 ? rotate8(o.w[t][b]) : o.w[t][b]);
#pragma unroll
              for (int rt = 0; rt < RT; ++rt)
                acc[rt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, as_bf16x8(o.xf[rt][b][half2]), acc[rt][t], 0, 0, 0);
            }
          } else {
            const int off = ((b * 2 + half2) * 4 + lq) * GP + frag_row;
            const bf16x8_t bh = as_bf16x8(*reinterpret_cast<const uint4_t*>(hi + off));
            const bf16x8_t bl = as_bf16x8(*reinterpret_cast<const uint4_t*>(lo + off));
#pragma unroll
            for (int t = 0; t < TT; ++t) {
              const bf16x8_t a = as_bf16x8(half2 ? rotate8(o.w[t][b]) : o.w[t][b]);
              acc[0][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bh, acc[0][t], 0, 0, 0);
              acc[0][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bl, acc[0][t], 0, 0, 0);
            }
          }
        }
      }
    }
  };

  if constexpr (XB) {
    // Nothing is staged: a ring of NB chunks in flight per wave (measured at the 5120-long down projection: four
    // instead of two change nothing).
    constexpr int NB = 2;
    Operands ring[NB];
#pragma unroll
    for (int s = 0; s < NB; ++s)
      if (s < n_my) load_w(s, ring[s]);
    for (int j = 0; j < n_my; j += NB) {
#pragma unroll
      for (int s = 0; s < NB; ++s) {
        if (j + s < n_my) {
          mma(j + s, ring[s]);
          if (j + s + NB < n_my) load_w(j + s + NB, ring[s]);
        }
      }
    }
  }
  Operands wa, wb;
  float4_t xa[XP + 1], xb[XP + 1];
  if (!XB && n_my > 0) {
    // Activations are requested before the weights: loads return in order, and the (cached) activations must
    // not queue behind weight lines coming from HBM.  Both arms keep the number of loads in flight static.
    // The common depths (one or two chunks per wave) are written out straight.
    if (n_my == 1) {
      load_x(0, xa);
      load_w(0, wa);
      stage(0, xa);
      mma(0, wa);
    } else if (n_my == 2) {
      load_x(0, xa);
      load_x(1, xb);
      load_w(0, wa);
      stage(0, xa);
      stage(1, xb);
      load_w(1, wb);                                               // after staging: the slabs' registers are free again, and
                                                                   // the load path has been busy with the requests above anyway
      mma(0, wa);
      mma(1, wb);
    } else {
      load_x(0, xa);
      load_x(1, xb);
      load_w(0, wa);
      stage(0, xa);
      stage(1, xb);
      // further slabs: one in flight while the previous one is staged
      int j = 2;
      load_x(j, xa);
      while (true) {
        if (j + 1 < n_my) { load_x(j + 1, xb); stage(j, xa); } else { stage(j, xa); break; }
        if (j + 2 < n_my) { load_x(j + 2, xa); stage(j + 1, xb); } else { stage(j + 1, xb); break; }
        j += 2;
      }
      load_w(1, wb);
      // weights: wa holds chunk j, wb chunk j + 1; each arm issues a fixed number of loads between a request and its use
      j = 0;
      while (true) {
        mma(j, wa);
        if (j + 2 < n_my) {
          load_w(j + 2, wa);
          mma(j + 1, wb);
          if (j + 3 < n_my) { load_w(j + 3, wb); } else { mma(j + 2, wa); break; }
        } else {
          mma(j + 1, wb);
          break;
        }
        j += 2;
      }
    }
  }

  // row statistics: piece i of a lane belongs to row i*2 + lane/32; add the 32 lanes of each half-wave
#pragma unroll
  for (int i = 0; i < XP; ++i) {
    float v = group_sum<32>(ss[i]);
    if ((lane & 31) == 0) ssum[wave * 16 + i * 2 + (lane >> 5)] = v;
  }
  __syncthreads();                                                 // every wave is done with its operands: the area is reused
  float4_t* red = reinterpret_cast<float4_t*>(my_area);
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int t = 0; t < TT; ++t) red[(rt * TT + t) * 64 + lane] = acc[rt][t];
  __syncthreads();

  // wave t finishes tile t (of every row tile): partial tiles added in wave order, 1/rms, epilogue.
  // acc of lane l holds y[row m0 + l%16][tile row (l/16)*4 + 0..3] (tile row = weight row = output column)
  if (wave >= TMAX || wave >= tiles) return;
  const int t = wave;
  if (lq >= (EPI == EPI_SWIGLU ? 1 : 2)) return;                   // accumulator rows 8..15 are meaningless; SwiGLU: rows 4..7 are
                                                                   // the up values, read from the lanes that hold them below
  const int n_out = n0 + t * UC + lq * 4;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int m = m0 + rt * 16 + lrow;
    if (m >= M) continue;
    float4_t extra = float4_t{0.f, 0.f, 0.f, 0.f};                 // bias and residual, fetched while the partials are added
    if (bias != nullptr) extra = *reinterpret_cast<const float4_t*>(bias + n_out);
    if (EPI == EPI_RESID) extra += *reinterpret_cast<const float4_t*>(res + (int64_t)m * ldres + n_out);
    float4_t y = float4_t{0.f, 0.f, 0.f, 0.f}, yu = float4_t{0.f, 0.f, 0.f, 0.f};
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < RL_WAVES; ++w) {
      const float4_t* rw = reinterpret_cast<const float4_t*>(smem + w * wave_bytes);
      y += rw[(rt * TT + t) * 64 + lane];
      if (EPI == EPI_SWIGLU) yu += rw[(rt * TT + t) * 64 + lane + 16];
      tot += ssum[w * 16 + lrow];
    }
    if (NORM) {
      const float r = 1.0f / sqrtf(tot / (float)K + eps);
      y *= r;
      yu *= r;
    }
    if (EPI == EPI_SWIGLU) {
      y.x = silu(y.x) * yu.x; y.y = silu(y.y) * yu.y; y.z = silu(y.z) * yu.z; y.w = silu(y.w) * yu.w;
    }
    y += extra;
    if (out_bf16)
      *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(out) + (int64_t)m * ldo + n_out) = uint2{pack_bf16x2(y.x, y.y), pack_bf16x2(y.z, y.w)};
    else
      *reinterpret_cast<float4_t*>(out + (int64_t)m * ldo + n_out) = y;
  }
}

// Two row tiles of 16 with fp32 activations (17-32 rows): the weights, once in registers, meet both tiles, so the matrix
// is streamed once for up to 32 rows at the accuracy of the 16-row kernel (bf16 head + remainder of every activation;
// every row's arithmetic, chunk assignment and summation order are those of the kernel above, so a row's result does
// not depend on which of the two kernels computed it).  The contraction length is at most 2048 (two chunks per wave):
// chunk 0 of both tiles is staged, contracted, then chunk 1 is staged over it (LDS operations of a wave execute in
// order), so LDS holds one staging slot per tile and wave: 139 KB, as the 16-row kernel with its two chunks.
template <int EPI, bool NORM, int TMAX>
__global__ __launch_bounds__(RL_THREADS) void resident_linear_f32x2_kernel(
    const float* __restrict__ x, int64_t ldx, const bf16_t* __restrict__ W, const float* __restrict__ gain, float eps,
    const float* __restrict__ bias, float* out, int64_t ldo, int M, int N, int K, int unit_base, int unit_rem, int wave_bytes, int out_bf16) {
  constexpr int CB = RL_CB, XP = 8, ROWS = 16, RT = 2;
  constexpr int GP = rl_group_pitch(ROWS);
  constexpr int SLOT = rl_chunk_bytes(ROWS);
  constexpr int TT = TMAX;
  constexpr int UC = (EPI == EPI_SWIGLU) ? 4 : 8;
  extern __shared__ __align__(16) char smem[];                     // [8 waves][wave_bytes], then row statistics [2 tiles][8][16]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lrow = lane & 15, lq = lane >> 4;
  char* my_area = smem + wave * wave_bytes;
  float* ssum = reinterpret_cast<float*>(smem + RL_WAVES * wave_bytes);

  const int g = blockIdx.x;
  const int u_cnt = unit_base + (g < unit_rem ? 1 : 0);
  const int u0 = g * unit_base + (g < unit_rem ? g : unit_rem);
  const int tiles = u_cnt;
  const int n0 = u0 * UC;
  uint32_t w_lane[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int uu = t < tiles ? t : tiles - 1;
    const int r = lrow & 7;
    const int n = (EPI == EPI_SWIGLU) ? (r < 4 ? 0 : N) + n0 + uu * 4 + (r & 3) : n0 + uu * 8 + r;
    w_lane[t] = ((uint32_t)n * (uint32_t)K + (uint32_t)(lq + 4 * (lrow >> 3)) * 8u) * 2u;
  }
  const char* w_base = reinterpret_cast<const char*>(W);
  const int total_blocks = K / RL_KBLOCK;
  const int chunks = (total_blocks + CB - 1) / CB;
  const int n_my = wave < chunks ? (chunks - wave + RL_WAVES - 1) / RL_WAVES : 0;   // 0, 1 or 2 (host-checked)

  float4_t acc[RT][TT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int t = 0; t < TT; ++t) acc[rt][t] = float4_t{0.f, 0.f, 0.f, 0.f};
  float ss[RT][XP];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int i = 0; i < XP; ++i) ss[rt][i] = 0.f;

  auto load_w = [&](int j, auto& w) {
    const int chunk = wave + j * RL_WAVES;
#pragma unroll
    for (int b = 0; b < CB; ++b) {
      int blk = chunk * CB + b;
      blk = blk < total_blocks ? blk : total_blocks - 1;
      const char* wp = w_base + (int64_t)blk * (RL_KBLOCK * 2);
#pragma unroll
      for (int t = 0; t < TT; ++t) w[t][b] = load16_stream(wp + w_lane[t]);
    }
  };
  const int c4 = lane & 31;
  auto load_x = [&](int j, int rt, float4_t (&xr)[XP + 1]) {
    const int chunk = wave + j * RL_WAVES;
    int blk = chunk * CB + (c4 >> 4);
    blk = blk < total_blocks ? blk : total_blocks - 1;
    const uint32_t kb = (uint32_t)blk * (RL_KBLOCK * 4);
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      int m = rt * 16 + i * 2 + (lane >> 5);
      m = m < M ? m : M - 1;
      xr[i] = *reinterpret_cast<const float4_t*>(reinterpret_cast<const char*>(x) + ((int64_t)m * ldx + (c4 & 15) * 4) * 4 + kb);
    }
    if (NORM) xr[XP] = *reinterpret_cast<const float4_t*>(reinterpret_cast<const char*>(gain) + (kb + (c4 & 15) * 16));
  };
  auto stage = [&](int j, int rt, const float4_t (&xr)[XP + 1]) {
    const int chunk = wave + j * RL_WAVES;
    char* hi = my_area + rt * SLOT;
    char* lo = hi + 16 * GP;
    const bool k_live = chunk * RL_CHUNK_K + c4 * 4 < K;
    const int group = c4 >> 1;
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const int row = i * 2 + (lane >> 5);
      float4_t v = (k_live && rt * 16 + row < M) ? xr[i] : float4_t{0.f, 0.f, 0.f, 0.f};
      ss[rt][i] = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, ss[rt][i]))));
      if (NORM) v *= xr[XP];
      uint32_t h01, l01, h23, l23;
      split_bf16x2(v.x, v.y, h01, l01);
      split_bf16x2(v.z, v.w, h23, l23);
      const int off = group * GP + row * 16 + (c4 & 1) * 8;
      *reinterpret_cast<uint2*>(hi + off) = uint2{h01, h23};
      *reinterpret_cast<uint2*>(lo + off) = uint2{l01, l23};
    }
  };
  auto mma = [&](int j, const auto& w) {
    const int chunk = wave + j * RL_WAVES;
#pragma unroll
    for (int b = 0; b < CB; ++b) {
      if (chunk * CB + b < total_blocks) {
#pragma unroll
        for (int half2 = 0; half2 < 2; ++half2) {
          const int off = ((b * 2 + half2) * 4 + lq) * GP + lrow * 16;
          bf16x8_t bh[RT], bl[RT];
#pragma unroll
          for (int rt = 0; rt < RT; ++rt) {
            bh[rt] = as_bf16x8(*reinterpret_cast<const uint4_t*>(my_area + rt * SLOT + off));
            bl[rt] = as_bf16x8(*reinterpret_cast<const uint4_t*>(my_area + rt * SLOT + 16 * GP + off));
          }
#pragma unroll
          for (int t = 0; t < TT; ++t) {
            const bf16x8_t a = as_bf16x8(half2 ? rotate8(w[t][b]) : w[t][b]);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
              acc[rt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bh[rt], acc[rt][t], 0, 0, 0);
              acc[rt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bl[rt], acc[rt][t], 0, 0, 0);
            }
          }
        }
      }
    }
  };

  // With four or five tiles per workgroup the registers do not hold both chunks' weights beside the activations of
  // two row tiles: chunk 1's weights are then requested only once chunk 0's are in the matrix cores (into the same
  // registers); their latency is partly covered by chunk 0's MFMAs and the staging of chunk 1.
  constexpr bool LATE_W = TMAX >= 4;
  uint4_t wa[TT][CB], wb[LATE_W ? 1 : TT][CB];
  float4_t xa[XP + 1], xb[XP + 1];
  if (n_my > 0) {
    load_x(0, 0, xa);                                              // activations first: loads return in order
    load_x(0, 1, xb);
    load_w(0, wa);
    stage(0, 0, xa);
    stage(0, 1, xb);
    if (n_my > 1) {
      load_x(1, 0, xa);
      load_x(1, 1, xb);
      if constexpr (!LATE_W) load_w(1, wb);
    }
    mma(0, wa);
    if (n_my > 1) {
      if constexpr (LATE_W) load_w(1, wa);
      stage(1, 0, xa);                                             // over chunk 0's slots: its operand reads were issued before
      stage(1, 1, xb);
      if constexpr (LATE_W) mma(1, wa); else mma(1, wb);
    }
  }

#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const float v = group_sum<32>(ss[rt][i]);
      if ((lane & 31) == 0) ssum[(rt * RL_WAVES + wave) * 16 + i * 2 + (lane >> 5)] = v;
    }
  __syncthreads();
  float4_t* red = reinterpret_cast<float4_t*>(my_area);
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int t = 0; t < TT; ++t) red[(rt * TT + t) * 64 + lane] = acc[rt][t];
  __syncthreads();

  if (wave >= TMAX || wave >= tiles) return;
  const int t = wave;
  if (lq >= (EPI == EPI_SWIGLU ? 1 : 2)) return;
  const int n_out = n0 + t * UC + lq * 4;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int m = rt * 16 + lrow;
    if (m >= M) continue;
    float4_t extra = float4_t{0.f, 0.f, 0.f, 0.f};
    if (bias != nullptr) extra = *reinterpret_cast<const float4_t*>(bias + n_out);
    float4_t y = float4_t{0.f, 0.f, 0.f, 0.f}, yu = float4_t{0.f, 0.f, 0.f, 0.f};
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < RL_WAVES; ++w) {
      const float4_t* rw = reinterpret_cast<const float4_t*>(smem + w * wave_bytes);
      y += rw[(rt * TT + t) * 64 + lane];
      if (EPI == EPI_SWIGLU) yu += rw[(rt * TT + t) * 64 + lane + 16];
      tot += ssum[(rt * RL_WAVES + w) * 16 + lrow];
    }
    if (NORM) {
      const float r = 1.0f / sqrtf(tot / (float)K + eps);
      y *= r;
      yu *= r;
    }
    if (EPI == EPI_SWIGLU) {
      y.x = silu(y.x) * yu.x; y.y = silu(y.y) * yu.y; y.z = silu(y.z) * yu.z; y.w = silu(y.w) * yu.w;
    }
    y += extra;
    if (out_bf16)
      *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(out) + (int64_t)m * ldo + n_out) = uint2{pack_bf16x2(y.x, y.y), pack_bf16x2(y.z, y.w)};
    else
      *reinterpret_cast<float4_t*>(out + (int64_t)m * ldo + n_out) = y;
  }
}

template <int EPI, bool NORM, int TMAX>
bool launch_f32x2_t(const LinearArgs& a, hipStream_t st, int G, int ub, int ur, int wave_bytes, size_t lds) {
  auto kern = resident_linear_f32x2_kernel<EPI, NORM, TMAX>;
  static bool attr_done = false;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, RL_LDS_LIMIT) != hipSuccess) {
      (void)hipGetLastError();
      return false;
    }
    attr_done = true;
  }
  PHOTON_LAUNCH(KC_SKINNY_GEMM, st, kern, dim3(G), dim3(RL_THREADS), lds, st, a.x, a.ldx, (const bf16_t*)a.W, a.gain, a.eps, a.bias, a.out,
                a.ldo, a.M, a.N, a.K, ub, ur, wave_bytes, a.out_bf16 ? 1 : 0);
  return true;
}

template <int EPI, bool NORM>
bool launch_f32x2_e(const LinearArgs& a, hipStream_t st, int tmax, int G, int ub, int ur, int wave_bytes, size_t lds) {
  switch (tmax) {
    case 1: return launch_f32x2_t<EPI, NORM, 1>(a, st, G, ub, ur, wave_bytes, lds);
    case 2: return launch_f32x2_t<EPI, NORM, 2>(a, st, G, ub, ur, wave_bytes, lds);
    case 3: return launch_f32x2_t<EPI, NORM, 3>(a, st, G, ub, ur, wave_bytes, lds);
    case 4: return launch_f32x2_t<EPI, NORM, 4>(a, st, G, ub, ur, wave_bytes, lds);
    case 5: return launch_f32x2_t<EPI, NORM, 5>(a, st, G, ub, ur, wave_bytes, lds);
  }
  return false;
}

template <int EPI, int XP, bool NORM, int TMAX, bool XB = false, int RT = 1>
bool launch_resident_t(const LinearArgs& a, hipStream_t st, int G, int unit_base, int unit_rem, int wave_bytes, size_t lds) {
  auto kern = resident_linear_bf16_kernel<EPI, XP, NORM, TMAX, XB, RT>;
  static bool attr_done = false;                                   // more than 64 KiB of dynamic LDS has to be allowed once
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, RL_LDS_LIMIT) != hipSuccess) {
      (void)hipGetLastError();
      return false;
    }
    attr_done = true;
  }
  dim3 grid(G, (a.M + 16 * RT - 1) / (16 * RT));
  PHOTON_LAUNCH(KC_SKINNY_GEMM, st, kern, grid, dim3(RL_THREADS), lds, st, a.x, a.ldx, (const bf16_t*)a.W, a.gain, a.eps, a.bias,
                a.res, a.ldres, a.out, a.ldo, a.M, a.N, a.K, unit_base, unit_rem, wave_bytes, a.out_bf16 ? 1 : 0);
  return true;
}

template <int EPI, int XP, bool NORM>
bool launch_resident_x(const LinearArgs& a, hipStream_t st, int tmax, int G, int ub, int ur, int wave_bytes, size_t lds) {
  switch (tmax) {
    case 1: return launch_resident_t<EPI, XP, NORM, 1>(a, st, G, ub, ur, wave_bytes, lds);
    case 2: return launch_resident_t<EPI, XP, NORM, 2>(a, st, G, ub, ur, wave_bytes, lds);
    case 3: return launch_resident_t<EPI, XP, NORM, 3>(a, st, G, ub, ur, wave_bytes, lds);
    case 4: return launch_resident_t<EPI, XP, NORM, 4>(a, st, G, ub, ur, wave_bytes, lds);
    case 5: return launch_resident_t<EPI, XP, NORM, 5>(a, st, G, ub, ur, wave_bytes, lds);
    case 6: return launch_resident_t<EPI, XP, NORM, 6>(a, st, G, ub, ur, wave_bytes, lds);
    default: return launch_resident_t<EPI, XP, NORM, 8>(a, st, G, ub, ur, wave_bytes, lds);
  }
}

// bf16 activations: one instantiation per epilogue, unit count and row tiles per workgroup (live rows are a run-time
// mask).  Four row tiles are instantiated up to three units, two up to six: what the registers hold.
template <int EPI, int RT>
bool launch_resident_xb_rt(const LinearArgs& a, hipStream_t st, int tmax, int G, int ub, int ur, int wave_bytes, size_t lds) {
  switch (tmax) {
    case 1: return launch_resident_t<EPI, 8, false, 1, true, RT>(a, st, G, ub, ur, wave_bytes, lds);
    case 2: return launch_resident_t<EPI, 8, false, 2, true, RT>(a, st, G, ub, ur, wave_bytes, lds);
    case 3: return launch_resident_t<EPI, 8, false, 3, true, RT>(a, st, G, ub, ur, wave_bytes, lds);
  }
  if constexpr (RT <= 2) {
    switch (tmax) {
      case 4: return launch_resident_t<EPI, 8, false, 4, true, RT>(a, st, G, ub, ur, wave_bytes, lds);
      case 5: return launch_resident_t<EPI, 8, false, 5, true, RT>(a, st, G, ub, ur, wave_bytes, lds);
      default: return launch_resident_t<EPI, 8, false, 6, true, RT>(a, st, G, ub, ur, wave_bytes, lds);
    }
  }
  return false;
}

template <int EPI>
bool launch_resident_xb(const LinearArgs& a, hipStream_t st, int rt, int tmax, int G, int ub, int ur, int wave_bytes, size_t lds) {
  switch (rt) {
    case 4: return launch_resident_xb_rt<EPI, 4>(a, st, tmax, G, ub, ur, wave_bytes, lds);
    case 2: return launch_resident_xb_rt<EPI, 2>(a, st, tmax, G, ub, ur, wave_bytes, lds);
    default: return launch_resident_xb_rt<EPI, 1>(a, st, tmax, G, ub, ur, wave_bytes, lds);
  }
}

template <int EPI, bool NORM>
bool launch_resident_e(const LinearArgs& a, hipStream_t st, int xp, int tmax, int G, int ub, int ur, int wave_bytes, size_t lds) {
  switch (xp) {
    case 2: return launch_resident_x<EPI, 2, NORM>(a, st, tmax, G, ub, ur, wave_bytes, lds);
    case 4: return launch_resident_x<EPI, 4, NORM>(a, st, tmax, G, ub, ur, wave_bytes, lds);
    default: return launch_resident_x<EPI, 8, NORM>(a, st, tmax, G, ub, ur, wave_bytes, lds);
  }
}

}  // namespace

// Returns true when the launch was issued here; false leaves the case to the streaming kernel.
bool launch_linear_resident(const LinearArgs& a, hipStream_t st) {
  if (!a.w_bf16 || a.K % RL_KBLOCK != 0 || a.N % 8 != 0) return false;
  if (a.ldx % (a.x_bf16 ? 8 : 4) != 0 || a.ldo % 4 != 0 || (a.res && a.ldres % 4 != 0)) return false;
  const bool norm = a.gain != nullptr;
  if (a.x_bf16 && norm) return false;
  // instantiated combinations: the ones the decode path uses
  const bool combo = (a.epilogue == EPI_PLAIN) || (a.epilogue == EPI_RESID && !norm) || (a.epilogue == EPI_SWIGLU && (norm || a.x_bf16));
  if (!combo) return false;
  const int64_t w_rows = (a.epilogue == EPI_SWIGLU) ? 2 * (int64_t)a.N : a.N;
  if (w_rows * a.K * 2 >= ((int64_t)1 << 32)) return false;       // 32-bit weight offsets
  const int rows_live = a.M < 16 ? a.M : 16;
  const int xp = rows_live <= 4 ? 2 : rows_live <= 8 ? 4 : 8;
  // SwiGLU deals columns in units of 4 (a tile holds 4 gate rows and their 4 up rows): the same bytes per unit as
  // 8 plain columns, and a finer deal, which evens out what the workgroups stream
  const int units = a.N / ((a.epilogue == EPI_SWIGLU) ? 4 : 8);
  // one workgroup per compute unit when there are enough units; more rounds only when a workgroup would exceed the
  // 8 tiles its registers hold
  constexpr int CUS = 256;
  const int cap = a.x_bf16 ? 6 : 8;                               // bf16 activations: the fragments take registers too
  const int rounds = (units + CUS * cap - 1) / (CUS * cap);
  const int G = units < CUS * rounds ? units : CUS * rounds;
  const int ub = units / G, ur = units % G;
  int tmax = ub + (ur ? 1 : 0);
  if (tmax > 6) tmax = 8;                                          // instantiated: 1 .. 6 and 8 (surplus tiles repeat the last)
  const int chunks = (a.K / RL_KBLOCK + RL_CB - 1) / RL_CB;
  const int n_my_max = (chunks + RL_WAVES - 1) / RL_WAVES;
  // bf16 activations with more than 16 rows: several row tiles per workgroup, as many as the registers hold
  const int rt = !a.x_bf16 || a.M <= 16 ? 1 : (a.M > 32 && tmax <= 3) ? 4 : 2;
  int wave_bytes = a.x_bf16 ? 0 : n_my_max * rl_chunk_bytes(2 * xp);
  if (wave_bytes < rt * tmax * 1024) wave_bytes = rt * tmax * 1024;   // the partial tiles reuse the area
  const size_t lds = (size_t)RL_WAVES * wave_bytes + RL_WAVES * 16 * sizeof(float);
  if (lds > (size_t)RL_LDS_LIMIT) return false;
  if (a.x_bf16) {
    switch (a.epilogue) {
      case EPI_PLAIN: return launch_resident_xb<EPI_PLAIN>(a, st, rt, tmax, G, ub, ur, wave_bytes, lds);
      case EPI_RESID: return launch_resident_xb<EPI_RESID>(a, st, rt, tmax, G, ub, ur, wave_bytes, lds);
      default: return launch_resident_xb<EPI_SWIGLU>(a, st, rt, tmax, G, ub, ur, wave_bytes, lds);
    }
  }
  switch (a.epilogue) {
    case EPI_PLAIN:
      return norm ? launch_resident_e<EPI_PLAIN, true>(a, st, xp, tmax, G, ub, ur, wave_bytes, lds)
                  : launch_resident_e<EPI_PLAIN, false>(a, st, xp, tmax, G, ub, ur, wave_bytes, lds);
    case EPI_RESID: return launch_resident_e<EPI_RESID, false>(a, st, xp, tmax, G, ub, ur, wave_bytes, lds);
    default: return launch_resident_e<EPI_SWIGLU, true>(a, st, xp, tmax, G, ub, ur, wave_bytes, lds);
  }
}

// fp32 activations of 17-32 rows at the accuracy of the 16-row kernel (see resident_linear_f32x2_kernel): plain (with an
// optional pre-norm and bias) and SwiGLU epilogues, contraction length at most 2048, at most 5 tiles per workgroup.
// Returns true when the launch was issued here.
bool launch_linear_resident_x2(const LinearArgs& a, hipStream_t st) {
  if (!a.w_bf16 || a.x_bf16 || a.M <= 16 || a.M > 32 || a.K % RL_KBLOCK != 0 || a.N % 8 != 0) return false;
  if (a.K > RL_WAVES * 2 * RL_CHUNK_K) return false;                // two chunks per wave
  if (a.ldx % 4 != 0 || a.ldo % 4 != 0) return false;
  if (a.epilogue == EPI_RESID || (a.epilogue == EPI_SWIGLU && a.gain == nullptr)) return false;
  const bool norm = a.gain != nullptr;
  const int64_t w_rows = (a.epilogue == EPI_SWIGLU) ? 2 * (int64_t)a.N : a.N;
  if (w_rows * a.K * 2 >= ((int64_t)1 << 32)) return false;
  const int units = a.N / ((a.epilogue == EPI_SWIGLU) ? 4 : 8);
  constexpr int CUS = 256;
  if (units > CUS * 5) return false;
  const int G = units < CUS ? units : CUS;
  const int ub = units / G, ur = units % G;
  const int tmax = ub + (ur ? 1 : 0);
  int wave_bytes = 2 * rl_chunk_bytes(16);
  if (wave_bytes < 2 * tmax * 1024) wave_bytes = 2 * tmax * 1024;
  const size_t lds = (size_t)RL_WAVES * wave_bytes + 2 * RL_WAVES * 16 * sizeof(float);
  if (lds > (size_t)RL_LDS_LIMIT) return false;
  if (a.epilogue == EPI_SWIGLU) return launch_f32x2_e<EPI_SWIGLU, true>(a, st, tmax, G, ub, ur, wave_bytes, lds);
  return norm ? launch_f32x2_e<EPI_PLAIN, true>(a, st, tmax, G, ub, ur, wave_bytes, lds)
              : launch_f32x2_e<EPI_PLAIN, false>(a, st, tmax, G, ub, ur, wave_bytes, lds);
}

}  // namespace photon
