// Few-row linear maps of the decode path with fused pre-norm and epilogue:
//
//     y[m, :] = rmsnorm(x[m, :]; gain) * W^T                     (gain optional)
//     plain    : out = y + bias
//     residual : out = res + y (+ bias)
//     swiglu   : out = silu(y_gate) * y_up          (W = [gate rows; up rows])
//
// Decode sub-steps carry one row per chunk in flight, so these are
// weight-streaming kernels: every weight byte is read once and the (<= 16 per
// workgroup) activation rows ride along.  bf16 weights go through the matrix
// cores only because M multiply-adds per weight would otherwise occupy the
// vector ALUs.  This file holds the streaming kernel, which takes any shape;
// shapes whose split activations fit in LDS go to the resident-activation
// kernel (photon_linear_resident.hip) first.
//   * a workgroup owns a few 16-column output tiles and the whole contraction;
//     its 8 waves take interleaved k chunks and meet once, in LDS, at the end.
//     Nothing crosses workgroups, so the output is complete when the kernel
//     ends (bias, residual, SwiGLU gate applied in place) and the summation
//     order is fixed: results are run-to-run deterministic;
//   * each lane issues 2 x 128-bit loads per 64-wide k block so that every
//     weight row is fetched in whole 128-byte lines; the k order inside a block
//     is permuted identically for both MFMA operands (a contraction does not
//     care), which is what makes those loads line up with the 16x16x32 operand
//     layout;
//   * activations stay fp32 in memory; each wave loads its k slab coalesced,
//     scales by the norm gain, splits it into a bf16 head and a bf16 remainder
//     (two MFMAs per weight fragment, so the product is as accurate as
//     fp32-activation x bf16-weight) and reshapes it to the operand layout
//     through a wave-private LDS area; rows beyond M are neither loaded nor
//     staged (a compute unit's load path is the scarce resource here: a load
//     that hits in cache costs it as much as one that misses);
//   * every load of a chunk, the gain slice included, is issued before the
//     next chunk's prefetch, so each wait names an exact number of younger
//     loads and never drains the prefetch;
//   * the RMS statistic of each row is accumulated from the same loads (every
//     wave sees a disjoint k range), reduced with the tiles, and applied to the
//     finished dot products, so a pre-norm costs no extra pass or launch.
#include "photon_linear.h"

#include "photon_device.h"
#include "photon_host.h"

namespace photon {


constexpr int FL_WAVES = 8;
constexpr int FL_THREADS = FL_WAVES * 64;
constexpr int FL_KBLOCK = 64;                 // k elements per block: 128 bytes of a weight row

// NT output tiles (16 columns each) per workgroup; a chunk is CB = 2 k blocks (128 k).
// One workgroup row (blockIdx.y) = 16 activation rows.
//
// Activations of a chunk reach the MFMA operand layout through a wave-private LDS area: the wave
// loads its 16 x 128 fp32 slab with coalesced 128-bit loads (a lane-per-fragment gather straight from
// memory would touch 64 cache lines per load instruction), scales by the gain, splits into bf16
// head/remainder, and writes 8-byte pieces into fragment order; the fragments come back with one
// 128-bit LDS read each.  No workgroup barrier is involved: only the owning wave touches its area.
constexpr int FL_CB = 2;
constexpr int FL_FRAG_PITCH = 16 * 16 + 16;                 // bytes per (block, half, q) group of 16 fragments, padded
constexpr int FL_STAGE_BYTES = FL_CB * 2 * 4 * FL_FRAG_PITCH;   // one of hi / lo

// XP: slab pieces per lane that hold live rows (rows m0 .. m0 + 2*XP - 1); dead rows are neither loaded nor staged,
// their MFMA columns then carry whatever the staging area held and are never stored.
// FOLD (one tile, not SwiGLU): the workgroup owns 8 columns; tile row r and r + 8 are weight row r, lanes of rows 0..7
// load the first 64 bytes of a block's line and lanes of rows 8..15 the second 64, so one load per block fetches
// whole lines; the second MFMA of a block takes the registers rotated by 8 lanes.  Accumulator rows 8..15 are
// meaningless.  Used when 16-column tiles would leave compute units without a workgroup.
template <int NT, int EPI, bool FOLD, int XP, bool NORM>
__global__ __launch_bounds__(FL_THREADS, (NT == 1 && EPI != EPI_SWIGLU && XP == 2) ? 4 : 2) void fused_linear_bf16_kernel(
    const float* __restrict__ x, int64_t ldx, const bf16_t* __restrict__ W, const float* __restrict__ gain, float eps,
    const float* __restrict__ bias, const float* res, int64_t ldres, float* out, int64_t ldo, int M, int N, int K, int out_bf16) {
  constexpr int CB = FL_CB;
  constexpr bool XPF = true;
  constexpr int TL = (EPI == EPI_SWIGLU) ? 2 * NT : NT;            // MFMA tiles per wave
  constexpr int RED_BYTES = TL * 64 * 16;
  constexpr int AREA = (2 * FL_STAGE_BYTES > RED_BYTES) ? 2 * FL_STAGE_BYTES : RED_BYTES;
  __shared__ __align__(16) char area[FL_WAVES][AREA];              // per wave: staging (hi | lo), later its partial tiles
  __shared__ float ssum[FL_WAVES][16];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);       // wave-uniform: chunk arithmetic stays on the scalar unit
  const int lrow = lane & 15, lq = lane >> 4;
  const int m0 = blockIdx.y * 16;
  static_assert(!FOLD || (NT == 1 && EPI != EPI_SWIGLU), "folded tiles: one per workgroup, no gate/up pairing");
  constexpr int WL = FOLD ? 1 : 2;                                 // weight loads per k block and tile
  const int n_base = blockIdx.x * (FOLD ? 8 : NT * 16);
  char* stage_hi = area[wave];
  char* stage_lo = area[wave] + FL_STAGE_BYTES;

  // Addresses are a wave-uniform base plus a 32-bit lane offset that does not change over the loop.
  const char* wtile[TL];                                           // first weight row of each tile
  bool tile_live[TL];
#pragma unroll
  for (int t = 0; t < TL; ++t) {
    const int n_rel = n_base + (t % NT) * 16;
    tile_live[t] = n_rel < N;                                      // N is a multiple of 16
    const int n_w = (t < NT ? 0 : N) + n_rel;                      // swiglu: up rows follow the N gate rows
    wtile[t] = reinterpret_cast<const char*>(W + (int64_t)(tile_live[t] ? n_w : 0) * K);
  }
  // row lrow of the tile, 16-byte group lq of a block half (folded: row lrow % 8, group lq of the half lrow / 8)
  const uint32_t w_lane = FOLD ? (uint32_t)((lrow & 7) * K + (lq + 4 * (lrow >> 3)) * 8) * 2u : (uint32_t)(lrow * K + lq * 8) * 2u;

  const int total_blocks = K / FL_KBLOCK;
  const int chunks = (total_blocks + CB - 1) / CB;

  float4_t acc[TL];
#pragma unroll
  for (int t = 0; t < TL; ++t) acc[t] = float4_t{0.f, 0.f, 0.f, 0.f};
  float ss[XP];                                                    // this lane's slab pieces belong to rows i*2 + lane/32
#pragma unroll
  for (int i = 0; i < XP; ++i) ss[i] = 0.f;

  uint4_t wa[TL][CB][WL], wb[TL][CB][WL];
  float4_t xa[XP + 1], xb[XP + 1];                                 // last element: the chunk's slice of the norm gain
  auto load_w = [&](int chunk, uint4_t (&wf)[TL][CB][WL]) {
#pragma unroll
    for (int b = 0; b < CB; ++b) {
      int blk = chunk * CB + b;
      blk = blk < total_blocks ? blk : total_blocks - 1;           // clamped: in bounds, result unused
#pragma unroll
      for (int t = 0; t < TL; ++t) {
        const char* p = wtile[t] + (int64_t)blk * (FL_KBLOCK * 2) + w_lane;
        // bytes 0..63 of the row's 128-byte line; folded: all of it, and non-temporal (whole lines used once
        // stream past the caches; for half lines the cached path measured faster)
        wf[t][b][0] = FOLD ? load16_stream(p) : load16(p);
        if (!FOLD) wf[t][b][1] = load16(p + 64);                   // bytes 64..127
      }
    }
  };
  // slab piece i of this lane: row i*2 + lane/32, k offset (lane%32)*4 inside the chunk
  const int c4 = lane & 31;
  // Loads are unconditional (row and k clamped into bounds, dead pieces zeroed at use) so that the
  // hardware load counter can be waited on precisely while the next chunk is in flight.
  uint32_t x_lane[XP];
#pragma unroll
  for (int i = 0; i < XP; ++i) {
    int m = m0 + i * 2 + (lane >> 5);
    m = m < M ? m : M - 1;
    x_lane[i] = (uint32_t)((int64_t)(m - m0) * ldx + (c4 & 15) * 4) * 4u;
  }
  const char* x_tile = reinterpret_cast<const char*>(x + (int64_t)m0 * ldx);
  auto load_x = [&](int chunk, float4_t (&xr)[XP + 1]) {
    int blk = chunk * CB + (c4 >> 4);                              // the k block this lane's pieces fall in
    blk = blk < total_blocks ? blk : total_blocks - 1;
    const uint32_t kb = (uint32_t)blk * (FL_KBLOCK * 4);
#pragma unroll
    for (int i = 0; i < XP; ++i) xr[i] = *reinterpret_cast<const float4_t*>(x_tile + (x_lane[i] + kb));
    // fetched with the slab, not at its use: a load issued after the next chunk's prefetch could only be
    // waited for by draining that prefetch as well
    if (NORM) xr[XP] = *reinterpret_cast<const float4_t*>(reinterpret_cast<const char*>(gain) + (kb + (c4 & 15) * 16));
  };
  auto stage = [&](int chunk, const float4_t (&xr)[XP + 1]) {
    // fragment fragment (block b, half, q) slot `row` holds k = b*64 + half*32 + q*8 .. +8 of that row
    const int k_in = c4 * 4;
    const int b_ = k_in >> 6, half = (k_in >> 5) & 1, q = (k_in >> 3) & 3;
    const int group = (b_ * 2 + half) * 4 + q;
    const int kabs = chunk * (CB * FL_KBLOCK) + k_in;
    const bool k_live = kabs < K;
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const int row = i * 2 + (lane >> 5);
      float4_t v = (k_live && m0 + row < M) ? xr[i] : float4_t{0.f, 0.f, 0.f, 0.f};
      ss[i] = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, ss[i]))));
      if (NORM) v *= xr[XP];
      uint32_t h01, l01, h23, l23;
      split_bf16x2(v.x, v.y, h01, l01);
      split_bf16x2(v.z, v.w, h23, l23);
      const int off = group * FL_FRAG_PITCH + row * 16 + (c4 & 1) * 8;
      *reinterpret_cast<uint2*>(stage_hi + off) = uint2{h01, h23};
      *reinterpret_cast<uint2*>(stage_lo + off) = uint2{l01, l23};
    }
    __builtin_amdgcn_wave_barrier();
  };
  auto mma = [&](int chunk, const uint4_t (&wf)[TL][CB][WL]) {
#pragma unroll
    for (int b = 0; b < CB; ++b) {
      if (chunk * CB + b < total_blocks) {
#pragma unroll
        for (int half2 = 0; half2 < 2; ++half2) {
          const int off = ((b * 2 + half2) * 4 + lq) * FL_FRAG_PITCH + lrow * 16;
          const bf16x8_t bh = as_bf16x8(*reinterpret_cast<const uint4_t*>(stage_hi + off));
          const bf16x8_t bl = as_bf16x8(*reinterpret_cast<const uint4_t*>(stage_lo + off));
#pragma unroll
          for (int t = 0; t < TL; ++t) {
            const bf16x8_t a = as_bf16x8(FOLD ? (half2 ? rotate8(wf[t][b][0]) : wf[t][b][0]) : wf[t][b][WL - 1 < half2 ? WL - 1 : half2]);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bh, acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bl, acc[t], 0, 0, 0);
          }
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  };

  // waves take chunks round-robin; the next chunk's weights and activations are in flight while this one is multiplied
  int chunk = wave;
  if (chunk < chunks) {
    load_w(chunk, wa);
    load_x(chunk, xa);
    if (XPF) {
      while (true) {
        const int c1 = chunk + FL_WAVES;
        if (c1 < chunks) { load_w(c1, wb); load_x(c1, xb); stage(chunk, xa); mma(chunk, wa); } else { stage(chunk, xa); mma(chunk, wa); break; }
        const int c2 = c1 + FL_WAVES;
        if (c2 < chunks) { load_w(c2, wa); load_x(c2, xa); stage(c1, xb); mma(c1, wb); } else { stage(c1, xb); mma(c1, wb); break; }
        chunk = c2;
      }
    } else {
      // one activation buffer: the next slab is requested as soon as this one sits in the staging area
      while (true) {
        const int c1 = chunk + FL_WAVES;
        if (c1 < chunks) { load_w(c1, wb); stage(chunk, xa); load_x(c1, xa); mma(chunk, wa); } else { stage(chunk, xa); mma(chunk, wa); break; }
        const int c2 = c1 + FL_WAVES;
        if (c2 < chunks) { load_w(c2, wa); stage(c1, xa); load_x(c2, xa); mma(c1, wb); } else { stage(c1, xa); mma(c1, wb); break; }
        chunk = c2;
      }
    }
  }

  // row statistics: piece i of a lane belongs to row i*2 + lane/32; add the 32 lanes of each half-wave
#pragma unroll
  for (int i = 0; i < XP; ++i) {
    float v = group_sum<32>(ss[i]);
    if ((lane & 31) == 0) ssum[wave][i * 2 + (lane >> 5)] = v;
  }
  float4_t* red = reinterpret_cast<float4_t*>(area[wave]);         // the staging area is free now
#pragma unroll
  for (int t = 0; t < TL; ++t) red[t * 64 + lane] = acc[t];
  __syncthreads();

  // wave t finishes output tile t: add the 8 partial tiles in wave order, scale by the row's 1/rms, epilogue.
  // acc of lane l holds y[row m0 + l%16][columns n0 + (l/16)*4 + 0..3]
  if (wave >= NT) return;
  const int t = wave;
  const int m = m0 + lrow;
  if (!tile_live[t] || m >= M) return;
  if (FOLD && lq >= 2) return;                                     // folded tile: accumulator rows 8..15 are meaningless
  const int n_out = n_base + t * 16 + lq * 4;
  float4_t extra = float4_t{0.f, 0.f, 0.f, 0.f};                   // bias and residual, fetched while the partials are added
  if (bias != nullptr) extra = *reinterpret_cast<const float4_t*>(bias + n_out);
  if (EPI == EPI_RESID) extra += *reinterpret_cast<const float4_t*>(res + (int64_t)m * ldres + n_out);
  float4_t y = float4_t{0.f, 0.f, 0.f, 0.f}, yu = float4_t{0.f, 0.f, 0.f, 0.f};
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < FL_WAVES; ++w) {
    const float4_t* rw = reinterpret_cast<const float4_t*>(area[w]);
    y += rw[t * 64 + lane];
    if (EPI == EPI_SWIGLU) yu += rw[(NT + t) * 64 + lane];
    tot += ssum[w][lrow];
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

// fp32 weights (the small all-fp32 configuration): one wave per output column, lanes stride over k
// with 128-bit loads, up to 16 rows per pass; same fused pre-norm and epilogues.
constexpr int F32_ROWS = 16;
template <int EPI>
__global__ __launch_bounds__(256) void fused_linear_f32_kernel(
    const float* __restrict__ x, int64_t ldx, const float* __restrict__ W, const float* __restrict__ gain, float eps,
    const float* __restrict__ bias, const float* res, int64_t ldres, float* out, int64_t ldo, int M, int N, int K) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int m0 = blockIdx.y * F32_ROWS;
  if (n >= N) return;
  float acc[F32_ROWS], accu[F32_ROWS], ss[F32_ROWS];
#pragma unroll
  for (int r = 0; r < F32_ROWS; ++r) acc[r] = accu[r] = ss[r] = 0.f;
  const float* wr = W + (int64_t)n * K;
  const float* wu = W + (int64_t)(N + n) * K;
  for (int k = lane * 4; k < K; k += 256) {
    float4_t w4 = *reinterpret_cast<const float4_t*>(wr + k);
    float4_t u4 = float4_t{0.f, 0.f, 0.f, 0.f};
    if (EPI == EPI_SWIGLU) u4 = *reinterpret_cast<const float4_t*>(wu + k);
    if (gain != nullptr) {
      const float4_t g4 = *reinterpret_cast<const float4_t*>(gain + k);
      w4 *= g4;
      u4 *= g4;
    }
#pragma unroll
    for (int r = 0; r < F32_ROWS; ++r) {
      if (m0 + r < M) {
        const float4_t x4 = *reinterpret_cast<const float4_t*>(x + (int64_t)(m0 + r) * ldx + k);
        acc[r] = fmaf(w4.x, x4.x, fmaf(w4.y, x4.y, fmaf(w4.z, x4.z, fmaf(w4.w, x4.w, acc[r]))));
        if (EPI == EPI_SWIGLU) accu[r] = fmaf(u4.x, x4.x, fmaf(u4.y, x4.y, fmaf(u4.z, x4.z, fmaf(u4.w, x4.w, accu[r]))));
        ss[r] = fmaf(x4.x, x4.x, fmaf(x4.y, x4.y, fmaf(x4.z, x4.z, fmaf(x4.w, x4.w, ss[r]))));
      }
    }
  }
#pragma unroll
  for (int r = 0; r < F32_ROWS; ++r) {
    float v = group_sum<32>(acc[r]);
    v += __shfl_xor(v, 32);
    float u = 0.f;
    if (EPI == EPI_SWIGLU) { u = group_sum<32>(accu[r]); u += __shfl_xor(u, 32); }
    float s = group_sum<32>(ss[r]);
    s += __shfl_xor(s, 32);
    if (lane == 0 && m0 + r < M) {
      if (gain != nullptr) {
        const float rs = 1.0f / sqrtf(s / (float)K + eps);
        v *= rs;
        u *= rs;
      }
      if (EPI == EPI_SWIGLU) v = silu(v) * u;
      if (bias != nullptr) v += bias[n];
      if (EPI == EPI_RESID) v += res[(int64_t)(m0 + r) * ldres + n];
      out[(int64_t)(m0 + r) * ldo + n] = v;
    }
  }
}

template <int NT, int EPI, bool FOLD, int XP>
static void launch_bf16_v(const LinearArgs& a, hipStream_t st) {
  constexpr int COLS = FOLD ? 8 : NT * 16;
  dim3 grid((a.N + COLS - 1) / COLS, (a.M + 15) / 16);
  if (a.gain != nullptr)
    PHOTON_LAUNCH(KC_SKINNY_GEMM, st, (fused_linear_bf16_kernel<NT, EPI, FOLD, XP, true>), grid, dim3(FL_THREADS), 0, st, a.x,
                  a.ldx, (const bf16_t*)a.W, a.gain, a.eps, a.bias, a.res, a.ldres, a.out, a.ldo, a.M, a.N, a.K, a.out_bf16 ? 1 : 0);
  else
    PHOTON_LAUNCH(KC_SKINNY_GEMM, st, (fused_linear_bf16_kernel<NT, EPI, FOLD, XP, false>), grid, dim3(FL_THREADS), 0, st, a.x,
                  a.ldx, (const bf16_t*)a.W, a.gain, a.eps, a.bias, a.res, a.ldres, a.out, a.ldo, a.M, a.N, a.K, a.out_bf16 ? 1 : 0);
}

template <int EPI, int XP>
static void launch_bf16_x(const LinearArgs& a, hipStream_t st) {
  if constexpr (EPI != EPI_SWIGLU) {                          // SwiGLU already carries two tiles (gate, up) per workgroup
    // more columns per workgroup (fewer re-reads of the activations) once there are enough workgroups to fill the chip
    if (a.N >= 6144) return launch_bf16_v<2, EPI, false, XP>(a, st);
    // too few 16-column tiles for the compute units: 8-column folded tiles
    if (a.N < 256 * 16) return launch_bf16_v<1, EPI, true, XP>(a, st);
  }
  return launch_bf16_v<1, EPI, false, XP>(a, st);
}

template <int EPI>
static void launch_bf16_e(const LinearArgs& a, hipStream_t st) {
  // few live rows (decode steps of the upper levels): the dead rows' loads are skipped
  if (a.M <= 4) return launch_bf16_x<EPI, 2>(a, st);
  if (a.M <= 8) return launch_bf16_x<EPI, 4>(a, st);
  return launch_bf16_x<EPI, 8>(a, st);
}

int32_t launch_linear(const LinearArgs& a, hipStream_t st) {
  if (a.M <= 0) return PHOTON_OK;
  if (a.epilogue < EPI_PLAIN || a.epilogue > EPI_SWIGLU) return fail(PHOTON_ERR_INVALID_ARG, "linear: unknown epilogue %d", a.epilogue);
  if (a.epilogue == EPI_RESID && a.res == nullptr) return fail(PHOTON_ERR_INVALID_ARG, "linear: residual epilogue without res");
  if (a.w_bf16) {
    if (a.K % FL_KBLOCK != 0 || a.N % 16 != 0 || a.ldx % 4 != 0 || a.ldo % 4 != 0 || (a.res && a.ldres % 4 != 0))
      return fail(PHOTON_ERR_UNSUPPORTED, "linear (bf16): K=%d must be a multiple of 64, N=%d of 16, row pitches of 4", a.K, a.N);
    if (launch_linear_resident_x2(a, st)) return check_launch("resident_linear_f32x2_kernel");   // 17-32 fp32 rows: one weight pass
    if (launch_linear_resident(a, st)) return check_launch("resident_linear_bf16_kernel");
    if (a.x_bf16) return fail(PHOTON_ERR_UNSUPPORTED, "linear: bf16 activations need a plain or residual epilogue without norm, N=%d a multiple of 8", a.N);
    switch (a.epilogue) {
      case EPI_PLAIN: launch_bf16_e<EPI_PLAIN>(a, st); break;
      case EPI_RESID: launch_bf16_e<EPI_RESID>(a, st); break;
      default: launch_bf16_e<EPI_SWIGLU>(a, st); break;
    }
    return check_launch("fused_linear_bf16_kernel");
  }
  if (a.x_bf16 || a.out_bf16) return fail(PHOTON_ERR_UNSUPPORTED, "linear (fp32): activations are fp32");
  if (a.K % 4 != 0 || a.ldx % 4 != 0) return fail(PHOTON_ERR_UNSUPPORTED, "linear (fp32): K=%d and the row pitch must be multiples of 4", a.K);
  dim3 grid((a.N + 3) / 4, (a.M + F32_ROWS - 1) / F32_ROWS);
#define PHOTON_F32_LAUNCH(E)                                                                                              \
  PHOTON_LAUNCH(KC_GEMM_F32, st, (fused_linear_f32_kernel<E>), grid, dim3(256), 0, st, a.x, a.ldx, (const float*)a.W, a.gain, \
                a.eps, a.bias, a.res, a.ldres, a.out, a.ldo, a.M, a.N, a.K)
  switch (a.epilogue) {
    case EPI_PLAIN: PHOTON_F32_LAUNCH(EPI_PLAIN); break;
    case EPI_RESID: PHOTON_F32_LAUNCH(EPI_RESID); break;
    default: PHOTON_F32_LAUNCH(EPI_SWIGLU); break;
  }
#undef PHOTON_F32_LAUNCH
  return check_launch("fused_linear_f32_kernel");
}

}  // namespace photon

using namespace photon;

extern "C" int32_t photon_linear(const void* x, const void* w, const float* gain, float rms_eps, const float* bias,
                                 const float* res, void* out, int32_t M, int32_t N, int32_t K, int32_t epilogue,
                                 photon_dtype dt, void* stream) {
  clear_error();
  const bool x_bf16 = (epilogue & PHOTON_LINEAR_X_BF16) != 0, out_bf16 = (epilogue & PHOTON_LINEAR_OUT_BF16) != 0;
  epilogue &= ~(PHOTON_LINEAR_X_BF16 | PHOTON_LINEAR_OUT_BF16);
  PHOTON_REQUIRE(!(x_bf16 || out_bf16) || dt == PHOTON_BF16, PHOTON_ERR_UNSUPPORTED, "%s: bf16 rows need dt = bf16", __func__);
  PHOTON_REQUIRE(valid_dtype(dt), PHOTON_ERR_UNSUPPORTED, "%s: unknown dtype %d", __func__, (int)dt);
  PHOTON_REQUIRE(M >= 0 && N > 0 && K > 0, PHOTON_ERR_INVALID_ARG, "%s: M=%d N=%d K=%d invalid", __func__, M, N, K);
  if (M == 0) return PHOTON_OK;
  PHOTON_REQUIRE_PTR(x);
  PHOTON_REQUIRE_PTR(w);
  PHOTON_REQUIRE_PTR(out);
  PHOTON_REQUIRE(gain == nullptr || aligned16(gain), PHOTON_ERR_INVALID_ARG, "%s: gain is misaligned", __func__);
  PHOTON_REQUIRE(bias == nullptr || aligned16(bias), PHOTON_ERR_INVALID_ARG, "%s: bias is misaligned", __func__);
  PHOTON_REQUIRE(res == nullptr || aligned16(res), PHOTON_ERR_INVALID_ARG, "%s: res is misaligned", __func__);
  LinearArgs a;
  a.x = reinterpret_cast<const float*>(x); a.x_bf16 = x_bf16; a.out_bf16 = out_bf16;
  a.ldx = K; a.W = w; a.w_bf16 = (dt == PHOTON_BF16); a.gain = gain; a.eps = rms_eps; a.bias = bias; a.res = res;
  a.ldres = N; a.out = reinterpret_cast<float*>(out); a.ldo = N; a.M = M; a.N = N; a.K = K; a.epilogue = epilogue;
  return launch_linear(a, (hipStream_t)stream);
}
