// Causal self-attention of a context encoder over whole sequences (the prefill
// form of paper Eq. 3; Section 2.3.1 prices it at O(M_l^2) per level).
//
// Input is the fused projection output qkv fp32 [Bt*M, 3*H*d_h] (row = b*M +
// position).  A row kernel applies the rotary encoding (module-local positions
// 0..M-1) and lays the operands out per (sequence, head); the attention kernel
// is a streaming-softmax tile kernel that never forms the M x M score matrix.
//
// bf16 configurations, d_h <= 64: matrix cores.
//   * S^T = K Q^T is computed (keys as MFMA rows, queries as columns) so that a
//     lane owns ONE query and 16 of a tile's 32 keys: the row maximum and sum
//     of the softmax are lane-local plus one exchange with lane^32.
//   * q, k and v enter as fp16 (one rounding of the fp32 projections each, 11
//     significant bits), the probabilities are rounded to fp16 as well, all
//     accumulation is fp32: two MFMAs per key tile and query tile.  Measured
//     against the float64 definition: normalised output error 4e-4 for
//     unit-variance q, k (score deviation 1), 1.5e-3 at deviation 4, 6e-3 at 16.
//     The alternative that was built first, bf16 head + remainder operands for
//     the scores (three MFMAs) with bf16 probabilities and values, costs 1.4x
//     the time and sits at 2-3e-3 whatever the scores' size: better only for
//     scores far larger than attention produces.  q is pre-scaled by
//     scale*log2(e) and exp2 is used.
//   * O^T = V^T P^T with P rounded straight from the score registers.
//     The key rows enter the score MFMA permuted (MFMA row 8i + 4g + r holds
//     key 16g + 4i + r of the tile) so that a lane ends up with 16 CONSECUTIVE
//     keys of the tile; V is stored transposed ([d_h][key]), so the matching
//     operand of the second MFMA is one 16-byte LDS read.  No data moves
//     between lanes and no register is repacked.
//   * the score accumulators start from minus the running maximum (kept as a
//     register vector that changes only when the maximum does), so the common
//     path per score is exp2, one add into the row sum and the fp16 pack.
//   * a workgroup = 12 waves = 384 queries of one (sequence, head) share every
//     key block of 64 (K, V^T: 16 KB = one 16-byte piece of each array per
//     thread of the first 8 waves; three waves per SIMD is what the kernel's
//     registers allow, and the phases of a wave - score MFMAs, softmax on the
//     vector ALUs, value MFMAs - are serial, so every further wave fills gaps:
//     measured +15 % at 32768 positions and +48 % at 8192 against 8 waves;
//     16 waves fit only with 128 registers per lane, which the compiler reaches
//     - queries kept in LDS, one register stage - at the price of a slower
//     schedule: 15 % behind 12 waves): what bounds the kernel is the K/V traffic into
//     the compute unit, so the query block is as large as the wave count
//     allows.  Blocks are requested two ahead into registers and written to a
//     double-buffered, XOR-swizzled LDS image one ahead (memory latency spans
//     more than one block's arithmetic); tiles entirely above the diagonal are
//     skipped per wave; the heavy (late) query blocks are scheduled first.
// fp32 configuration: a plain fp32 tile kernel on the vector ALUs (small sizes).
#include "photon_encoder_attn.h"

#include "photon_attn.h"
#include "photon_device.h"
#include "photon_host.h"

namespace photon {

namespace {

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

constexpr int EA_DH = 64;          // head size of the MFMA path
constexpr int EA_WAVES = 12;        // 3 per SIMD: what the kernel's registers allow
constexpr int EA_MOVERS = 8;        // waves that move the key blocks: 512 threads = one 16-byte piece of each array
constexpr int EA_BQ = EA_WAVES * 32; // queries per workgroup (32 per wave)
constexpr int EA_BK = 64;          // keys per block
constexpr int EA_THREADS = EA_WAVES * 64;
constexpr int EA_ARRAY = EA_BK * 128;                 // one staged array: 64 rows of 128 bytes
constexpr int EA_STAGE = 2 * EA_ARRAY;                // K | V^T

__host__ __device__ inline int64_t round_up64(int64_t m) { return (m + 63) / 64 * 64; }

// LDS layout of the staged arrays: 128-byte rows, the 16-byte column index XOR-ed with row bits.  A 128-bit LDS read
// is conflict-free when (measured with a read-only probe: 256 bytes per clock and compute unit, against 154 otherwise)
//   * the 16 lanes of a quarter-wave fall on distinct 16-byte slots of the 256-byte bank line, and
//   * lanes j and j + 16 of a half-wave agree in address bits 6 and 7 (the same quarter of the bank line).
// V^T is read by consecutive rows (lane j: row j of 32): XOR with row bits 1..3; rows r and r + 16 share the slot.
// K is read by permuted rows (quarter-wave 0: rows {0..7, 16..23}, quarter-wave 1: the same + 8): XOR with row bits
// 1..2 and, into bit 2, row bit 4; rows r and r + 8 share the slot.
__device__ __forceinline__ int swz_v(int row, int col16) { return row * 128 + ((col16 ^ ((row >> 1) & 7)) << 4); }
__device__ __forceinline__ int swz_k(int row, int col16) { return row * 128 + ((col16 ^ ((row >> 1) & 3) ^ ((row >> 2) & 4)) << 4); }

// ---- row kernel: rotary + operand layout ----------------------------------------------------------
// One workgroup = 64 positions of one (sequence, head).  Thread t: position t/4, quarter t%4 of the pairs
// (pairs i = quarter*8 .. +8).
// Outputs (fp16, saturated): qh, kh [Bt*H][Mp][64] (Mp = M rounded up to 64; rows >= M are zero), vt [Bt*H][64][Mp];
// q is multiplied by qscale (= softmax scale * log2 e) before the rounding.  kc / vc (optional): the layer's
// coarse cache [Bt][H][S_max][pitch] in bf16, positions 0..M-1, K rotated.
// PAD: head size d_h < 64 (a multiple of 4).  The operand rows stay 64 wide: of rotary pair i (i < d_h/2) the
// first member sits in column i and the second in column 32 + i, for q and k alike (a score does not depend on
// the order of the contraction index); V keeps its own column order, so the output columns are the head's; all
// other columns are zero.
// TC: storage type of the cache (bf16_t or fp8_t).
template <bool PAD, typename TC>
__global__ __launch_bounds__(256) void encoder_rope_split_kernel(const float* __restrict__ qkv, uint16_t* __restrict__ qh,
                                                                 uint16_t* __restrict__ kh, uint16_t* __restrict__ vt,
                                                                 TC* __restrict__ kc, TC* __restrict__ vc, int64_t M, int H,
                                                                 int d_h_rt, int pitch, int64_t S_max, float theta, float qscale) {
  __shared__ uint16_t vtile[64][64 + 2];                // [d][position], padded
  const int tid = threadIdx.x;
  const int bh = blockIdx.y, b = bh / H, h = bh % H;
  const int64_t Mp = round_up64(M);
  const int64_t p0 = (int64_t)blockIdx.x * 64;
  const int pl = tid >> 2, quarter = tid & 3;
  const int64_t pos = p0 + pl;
  const int d_h = PAD ? d_h_rt : EA_DH;
  const int hr = d_h / 2;                             // distance between the members of a rotary pair
  const int D = H * d_h;
  const bool live = pos < M;
  // q, k: [j] first and [8 + j] second member of pair quarter*8 + j; v: columns quarter*8 + j and 32 + quarter*8 + j
  float q[16], k[16], v[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) q[e] = k[e] = v[e] = 0.f;
  if (live) {
    const float* head = qkv + ((int64_t)b * M + pos) * 3 * D + h * d_h;
    const float* src = head + quarter * 8;
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int e = half * 8 + c * 4;
        if (!PAD) {
          const float4_t a = *reinterpret_cast<const float4_t*>(src + half * 32 + c * 4);
          const float4_t kk = *reinterpret_cast<const float4_t*>(src + D + half * 32 + c * 4);
          q[e] = a.x; q[e + 1] = a.y; q[e + 2] = a.z; q[e + 3] = a.w;
          k[e] = kk.x; k[e + 1] = kk.y; k[e + 2] = kk.z; k[e + 3] = kk.w;
        }
        if (!PAD || half * 32 + quarter * 8 + c * 4 < d_h) {
          const float4_t vv = *reinterpret_cast<const float4_t*>(src + 2 * D + half * 32 + c * 4);
          v[e] = vv.x; v[e + 1] = vv.y; v[e + 2] = vv.z; v[e + 3] = vv.w;
        }
      }
    if (PAD) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int i = quarter * 8 + j;
        if (i < hr) { q[j] = head[i]; q[8 + j] = head[i + hr]; k[j] = head[D + i]; k[8 + j] = head[D + i + hr]; }
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float c, s;
      rope_angle((int)pos, quarter * 8 + j, d_h, theta, c, s);
      const float qa = q[j], qb = q[8 + j], ka = k[j], kb = k[8 + j];
      q[j] = (qa * c - qb * s) * qscale; q[8 + j] = (qb * c + qa * s) * qscale;
      k[j] = ka * c - kb * s; k[8 + j] = kb * c + ka * s;
    }
  }
  const int64_t row = ((int64_t)bh * Mp + pos) * EA_DH;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int off = half * 32 + quarter * 8;
    const float* qs = q + half * 8;
    const float* ks = k + half * 8;
    uint4_t h4, kh4;
    h4.x = pack_f16x2(qs[0], qs[1]); h4.y = pack_f16x2(qs[2], qs[3]); h4.z = pack_f16x2(qs[4], qs[5]); h4.w = pack_f16x2(qs[6], qs[7]);
    kh4.x = pack_f16x2(ks[0], ks[1]); kh4.y = pack_f16x2(ks[2], ks[3]); kh4.z = pack_f16x2(ks[4], ks[5]); kh4.w = pack_f16x2(ks[6], ks[7]);
    *reinterpret_cast<uint4_t*>(qh + row + off) = h4;
    *reinterpret_cast<uint4_t*>(kh + row + off) = kh4;
    if (!PAD && kc != nullptr && live && pos < S_max) { // the cache holds its own rounding of the fp32 values
      const float* vs = v + half * 8;
      const int64_t slot = (((int64_t)b * H + h) * S_max + pos) * EA_DH + off;
      if (sizeof(TC) == 2) {
        uint4_t vv, kk;
        vv.x = pack_bf16x2(vs[0], vs[1]); vv.y = pack_bf16x2(vs[2], vs[3]); vv.z = pack_bf16x2(vs[4], vs[5]); vv.w = pack_bf16x2(vs[6], vs[7]);
        kk.x = pack_bf16x2(ks[0], ks[1]); kk.y = pack_bf16x2(ks[2], ks[3]); kk.z = pack_bf16x2(ks[4], ks[5]); kk.w = pack_bf16x2(ks[6], ks[7]);
        *reinterpret_cast<uint4_t*>(kc + slot) = kk;
        *reinterpret_cast<uint4_t*>(vc + slot) = vv;
      } else {
        uint2 vv, kk;
        vv.x = pack_fp8x2(vs[0], vs[1]) | (pack_fp8x2(vs[2], vs[3]) << 16); vv.y = pack_fp8x2(vs[4], vs[5]) | (pack_fp8x2(vs[6], vs[7]) << 16);
        kk.x = pack_fp8x2(ks[0], ks[1]) | (pack_fp8x2(ks[2], ks[3]) << 16); kk.y = pack_fp8x2(ks[4], ks[5]) | (pack_fp8x2(ks[6], ks[7]) << 16);
        *reinterpret_cast<uint2*>(kc + slot) = kk;
        *reinterpret_cast<uint2*>(vc + slot) = vv;
      }
    }
    if (PAD && kc != nullptr && live && pos < S_max) {  // cache rows in the head's own column order, zeros past d_h
      const int64_t slot = (((int64_t)b * H + h) * S_max + pos) * pitch;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int i = quarter * 8 + j;
        if (i < hr) kc[slot + half * hr + i] = from_f32<TC>(k[half * 8 + j]);
        const int col = half * 32 + i;
        if (col < pitch) vc[slot + col] = from_f32<TC>(v[half * 8 + j]);
        if (col >= d_h && col < pitch) kc[slot + col] = TC{};
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      vtile[half * 32 + quarter * 8 + j][pl] = (uint16_t)(pack_f16x2(v[half * 8 + j], 0.f) & 0xffffu);
  }
  __syncthreads();
  // transposed tile out: 64 rows (d) of 64 positions = 128 bytes each; thread t writes two 16-byte pieces
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int piece = tid + r * 256;
    const int d = piece >> 3, c8 = (piece & 7) * 8;
    uint4_t o;
    o.x = (uint32_t)vtile[d][c8 + 0] | ((uint32_t)vtile[d][c8 + 1] << 16); o.y = (uint32_t)vtile[d][c8 + 2] | ((uint32_t)vtile[d][c8 + 3] << 16);
    o.z = (uint32_t)vtile[d][c8 + 4] | ((uint32_t)vtile[d][c8 + 5] << 16); o.w = (uint32_t)vtile[d][c8 + 6] | ((uint32_t)vtile[d][c8 + 7] << 16);
    *reinterpret_cast<uint4_t*>(vt + ((int64_t)bh * EA_DH + d) * Mp + p0 + c8) = o;
  }
}

// ---- attention kernel (matrix cores) -----------------------------------------------------------------
// Operands are fp16: q (pre-scaled), k and V^T as the row kernel wrote them, probabilities rounded to fp16 from the
// score registers; accumulation in fp32.
__device__ __forceinline__ float16_t ea_mfma(const uint4_t& a, const uint4_t& b, const float16_t& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

__global__ __launch_bounds__(EA_THREADS) void encoder_attn_mfma_kernel(const uint16_t* __restrict__ qh, const uint16_t* __restrict__ kh,
                                                                       const uint16_t* __restrict__ vt, float* __restrict__ out, int64_t M,
                                                                       int H, int d_h, int n_qblocks, int out_bf16) {
  constexpr int STAGE = EA_STAGE;
  constexpr int V_OFF = EA_ARRAY;
  extern __shared__ __align__(16) char lds[];         // [4 buffers][K | V^T]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qb = n_qblocks - 1 - blockIdx.x;          // late query blocks carry the most keys: schedule them first
  const int bh = blockIdx.y, b = bh / H, h = bh % H;
  const int64_t Mp = round_up64(M);
  const int64_t q0 = (int64_t)qb * EA_BQ + wave * 32; // this wave's first query
  const int qcol = lane & 31, kg = lane >> 5;
  const int64_t qpos = q0 + qcol;                     // this lane's query (may be >= M in the last block: computed, not stored)

  // operand bases of this (sequence, head)
  const uint16_t* khb = kh + (int64_t)bh * Mp * EA_DH;
  const uint16_t* vtb = vt + (int64_t)bh * EA_DH * Mp;

  // this lane's query as MFMA B operand: Q[q][16 s + 8 kg .. +8] for the four k-steps s
  uint4_t qfh[4];
  {
    const int64_t qrow = qpos < Mp ? qpos : Mp - 1;   // rows up to Mp exist (zero padded)
    const uint16_t* qp = qh + ((int64_t)bh * Mp + qrow) * EA_DH + kg * 8;
#pragma unroll
    for (int s = 0; s < 4; ++s) qfh[s] = load16(qp + s * 16);
  }

  // A key block is 2 arrays of 64 rows x 128 bytes = 512 pieces of 16 bytes each: thread t moves piece (row t/8,
  // column t%8) of both arrays, global -> registers -> LDS (swizzled).
  const int prow = (tid >> 3) & 63, pcol = tid & 7;
  const int poff_k = swz_k(prow, pcol), poff_v = swz_v(prow, pcol);
  struct Pieces { uint4_t kh, vt; };
  auto fetch = [&](int kb, int n_kb_, Pieces& r) __attribute__((always_inline)) {
    if (wave >= EA_MOVERS) return;
    const int64_t k0 = (int64_t)(kb < n_kb_ ? kb : n_kb_ - 1) * EA_BK;      // past the end: the last block again (in bounds, unused)
    r.kh = load16(khb + (k0 + prow) * EA_DH + pcol * 8);
    r.vt = load16(vtb + (int64_t)prow * Mp + k0 + pcol * 8);
  };
  auto put = [&](const Pieces& r, int buf) __attribute__((always_inline)) {
    if (wave >= EA_MOVERS) return;
    char* base = lds + buf * STAGE;
    *reinterpret_cast<uint4_t*>(base + poff_k) = r.kh;
    *reinterpret_cast<uint4_t*>(base + V_OFF + poff_v) = r.vt;
  };

  float16_t o[2];                                     // O^T tiles: d = dt*32 + 8*(v/4) + 4*kg + v%4, query = lane%32
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
  // key blocks 0 .. last block that holds a key <= the workgroup's last query
  const int64_t wg_last_q = (int64_t)qb * EA_BQ + EA_BQ - 1;
  const int64_t last_key = wg_last_q < M - 1 ? wg_last_q : M - 1;
  const int n_kb = (int)(last_key / EA_BK) + 1;
  const int64_t wave_last_q = q0 + 31;

  // MFMA row m = 8i + 4g + r of a score tile holds key 16g + 4i + r, so lane half kg owns keys 16 kg + v, v = 0..15
  const int krow = 16 * ((qcol >> 2) & 1) + 4 * (qcol >> 3) + (qcol & 3);
  float16_t negm;                                     // -m_run in every element: the score accumulators start from it
#pragma unroll
  for (int e = 0; e < 16; ++e) negm[e] = 0.f;
  float m_run = 0.f, l_run = 0.f;                     // reference maximum (shared by both lane halves; set by block 0) and this half's partial sum

  auto compute = [&](int kb, int buf) __attribute__((always_inline)) {
    const int64_t k0 = (int64_t)kb * EA_BK;
    if (k0 > wave_last_q) return;                     // block entirely above this wave's diagonal (uniform per wave)
    const char* sk = lds + buf * STAGE;
    const char* sv = sk + V_OFF;
    const bool two = k0 + 32 <= wave_last_q;          // second key tile not entirely above this wave's diagonal

    // st[kt][v] = S^T[key k0 + kt*32 + 16 kg + v][query] - m_run; the two tiles' MFMA chains are interleaved
    float16_t st[2];
    if (two) {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const int o0 = swz_k(krow, s * 2 + kg), o1 = swz_k(32 + krow, s * 2 + kg);
        const uint4_t ah0 = *reinterpret_cast<const uint4_t*>(sk + o0);
        const uint4_t ah1 = *reinterpret_cast<const uint4_t*>(sk + o1);
        st[0] = ea_mfma(ah0, qfh[s], s == 0 ? negm : st[0]);
        st[1] = ea_mfma(ah1, qfh[s], s == 0 ? negm : st[1]);
      }
    } else {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const int o0 = swz_k(krow, s * 2 + kg);
        const uint4_t ah0 = *reinterpret_cast<const uint4_t*>(sk + o0);
        st[0] = ea_mfma(ah0, qfh[s], s == 0 ? negm : st[0]);
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) st[1][e] = NEG_BIG;     // contributes exp2(-huge) = 0
    }
    // causal mask: only in blocks that reach this wave's diagonal (a real branch, uniform per wave)
    if (k0 + EA_BK - 1 > q0) {
      const int rel = (int)(qpos - k0) - 16 * kg;     // v + 32 kt must not exceed rel
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (kt * 32 + v > rel) st[kt][v] = NEG_BIG;
    }
    // scores are relative to the running maximum: a positive one raises it (rare after the first blocks)
    float mx = st[0][0];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, st[kt][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const bool first = (kb == 0);                     // block 0 is every wave's first block: it sets the reference maximum
    if (first || __builtin_amdgcn_ballot_w64(mx > 0.f) != 0) {
      const float up = first ? mx : fmaxf(mx, 0.f);   // this lane's reference maximum moves by `up`
      m_run += up;
#pragma unroll
      for (int e = 0; e < 16; ++e) negm[e] = -m_run;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int v = 0; v < 16; ++v) st[kt][v] -= up;
      if (!first) {                                   // (the state is still zero in block 0)
        const float alpha = fast_exp2(-up);
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[dt][e] *= alpha;
      }
    }
    float psum = 0.f;
    uint4_t pf[2][2];                                 // P^T operands: [key tile][k-step]: keys 16 kg + 8 s + 0..7 of the tile
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        uint4_t pk;
        float p[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          // a masked score is about -1e30: exp2 gives exactly 0 (the query sees at least key k0 of every block it processes)
          p[j] = fast_exp2(st[kt][8 * s + j]);
          psum += p[j];
        }
        pk.x = pack_f16x2_unit(p[0], p[1]); pk.y = pack_f16x2_unit(p[2], p[3]); pk.z = pack_f16x2_unit(p[4], p[5]);
        pk.w = pack_f16x2_unit(p[6], p[7]);
        pf[kt][s] = pk;
      }
    l_run += psum;
    // O^T += V^T P^T: k-slot (kg, j) of step s stands for key kt*32 + 16 kg + 8 s + j: 16 consecutive bytes of a V^T row
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      if (kt == 1 && !two) continue;
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
          const uint4_t a = *reinterpret_cast<const uint4_t*>(sv + swz_v(dt * 32 + qcol, kt * 4 + 2 * kg + s));
          o[dt] = ea_mfma(a, pf[kt][s], o[dt]);
        }
    }
  };

  // Four buffers, one barrier per TWO key blocks: a round contracts the pair of buffers that the round before filled
  // and fills the other pair (last read before the barrier that ended that round) with the two blocks after.
  Pieces ra, rb;
  fetch(0, n_kb, ra);
  fetch(1, n_kb, rb);
  put(ra, 0);
  put(rb, 1);
  fetch(2, n_kb, ra);
  fetch(3, n_kb, rb);
  __syncthreads();
  for (int kb = 0; kb < n_kb; kb += 2) {
    const int cur = (kb >> 1) & 1;                    // buffers 2 cur, 2 cur + 1 hold blocks kb, kb + 1
    put(ra, 2 * (cur ^ 1));                           // blocks kb + 2, kb + 3
    put(rb, 2 * (cur ^ 1) + 1);
    fetch(kb + 4, n_kb, ra);
    fetch(kb + 5, n_kb, rb);
    compute(kb, 2 * cur);
    if (kb + 1 < n_kb) compute(kb + 1, 2 * cur + 1);
    __syncthreads();
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (qpos >= M) return;
  const float inv = 1.0f / l_tot;
  const int64_t dst_off = ((int64_t)b * M + qpos) * (H * d_h) + h * d_h;   // d_h <= 64: the columns past it are padding
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      float4_t y;
      y.x = o[dt][g4 * 4 + 0] * inv; y.y = o[dt][g4 * 4 + 1] * inv; y.z = o[dt][g4 * 4 + 2] * inv; y.w = o[dt][g4 * 4 + 3] * inv;
      const int col = dt * 32 + 8 * g4 + 4 * kg;
      if (col >= d_h) continue;
      if (out_bf16) *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(out) + dst_off + col) = uint2{pack_bf16x2(y.x, y.y), pack_bf16x2(y.z, y.w)};
      else *reinterpret_cast<float4_t*>(out + dst_off + col) = y;
    }
}

// ---- fp32 configuration: plain tile kernel -----------------------------------------------------------
// One workgroup = 64 queries of one (sequence, head); thread t owns query t and streams the keys 0..q
// through LDS tiles of 32 keys (rotated as they are staged).
template <int DH>
__global__ __launch_bounds__(64) void encoder_attn_f32_kernel(const float* __restrict__ qkv, float* __restrict__ out, float* __restrict__ kc,
                                                              float* __restrict__ vc, int64_t M, int H, int pitch, int64_t S_max,
                                                              float theta, float scale) {
  __shared__ float ks[32][DH + 1], vs[32][DH + 1];
  const int t = threadIdx.x;
  const int bh = blockIdx.y, b = bh / H, h = bh % H;
  const int D = H * DH, half = DH / 2;
  const int64_t q0 = (int64_t)blockIdx.x * 64;
  const int64_t qpos = q0 + t;
  const bool live = qpos < M;
  float q[DH], acc[DH];
#pragma unroll
  for (int d = 0; d < DH; ++d) { q[d] = 0.f; acc[d] = 0.f; }
  if (live) {
    const float* src = qkv + ((int64_t)b * M + qpos) * 3 * D + h * DH;
#pragma unroll
    for (int i = 0; i < half; ++i) {
      float c, s;
      rope_angle((int)qpos, i, DH, theta, c, s);
      const float a = src[i], bb = src[i + half];
      q[i] = (a * c - bb * s) * scale * LOG2E;
      q[i + half] = (bb * c + a * s) * scale * LOG2E;
    }
  }
  float m_run = NEG_BIG, l_run = 0.f;
  const int64_t last = (q0 + 63 < M - 1) ? q0 + 63 : M - 1;
  for (int64_t k0 = 0; k0 <= last; k0 += 32) {
    __syncthreads();
    // 64 threads load 32 keys: thread t -> key t/2, half (t%2) of the pairs
    {
      const int kr = t >> 1, part = t & 1;
      const int64_t kpos = k0 + kr;
      if (kpos < M) {
        const float* src = qkv + ((int64_t)b * M + kpos) * 3 * D + h * DH;
        for (int i = part * (half / 2); i < (part + 1) * (half / 2); ++i) {
          float c, s;
          rope_angle((int)kpos, i, DH, theta, c, s);
          const float a = src[D + i], bb = src[D + i + half];
          const float ka = a * c - bb * s, kb = bb * c + a * s;
          const float va = src[2 * D + i], vb = src[2 * D + i + half];
          ks[kr][i] = ka; ks[kr][i + half] = kb;
          vs[kr][i] = va; vs[kr][i + half] = vb;
        }
      } else {
        for (int i = part * (half / 2); i < (part + 1) * (half / 2); ++i) { ks[kr][i] = ks[kr][i + half] = 0.f; vs[kr][i] = vs[kr][i + half] = 0.f; }
      }
    }
    __syncthreads();
    if (!live) continue;
    for (int j = 0; j < 32; ++j) {
      const int64_t kpos = k0 + j;
      if (kpos > qpos) break;
      float s = 0.f;
#pragma unroll
      for (int d = 0; d < DH; ++d) s = fmaf(q[d], ks[j][d], s);
      const float m_new = fmaxf(m_run, s);
      const float alpha = fast_exp2(m_run - m_new), p = fast_exp2(s - m_new);
      m_run = m_new;
      l_run = l_run * alpha + p;
#pragma unroll
      for (int d = 0; d < DH; ++d) acc[d] = fmaf(acc[d], alpha, p * vs[j][d]);
    }
  }
  if (!live) return;
  const float inv = 1.0f / l_run;
  float* dst = out + ((int64_t)b * M + qpos) * D + h * DH;
#pragma unroll
  for (int d = 0; d < DH; ++d) dst[d] = acc[d] * inv;
  if (kc != nullptr && qpos < S_max) {                // this thread's own position: rotated key and value into the cache
    const float* src = qkv + ((int64_t)b * M + qpos) * 3 * D + h * DH;
    float* kd = kc + (((int64_t)b * H + h) * S_max + qpos) * pitch;   // cache rows hold pitch >= DH elements, zeros past DH
    float* vd = vc + (((int64_t)b * H + h) * S_max + qpos) * pitch;
    for (int p = DH; p < pitch; ++p) { kd[p] = 0.f; vd[p] = 0.f; }
#pragma unroll
    for (int i = 0; i < half; ++i) {
      float c, s;
      rope_angle((int)qpos, i, DH, theta, c, s);
      const float a = src[D + i], bb = src[D + i + half];
      kd[i] = a * c - bb * s; kd[i + half] = bb * c + a * s;
      vd[i] = src[2 * D + i]; vd[i + half] = src[2 * D + i + half];
    }
  }
}

}  // namespace

size_t encoder_attn_workspace_bytes(int Bt, int64_t M, int H, int d_h, bool bf16) {
  if (!bf16) return 0;
  (void)d_h;                                                           // the operand rows are 64 wide for every head size
  return (size_t)3 * Bt * H * round_up64(M) * EA_DH * sizeof(uint16_t);   // q, k, V^T
}

int32_t launch_encoder_attn(const float* qkv, float* out, int Bt, int64_t M, int H, int d_h, float theta, float scale, void* k_cache,
                            void* v_cache, int64_t S_max, void* workspace, bool bf16, bool kv_fp8, bool out_bf16, hipStream_t st) {
  if (Bt <= 0 || M <= 0) return PHOTON_OK;
  if (out_bf16 && !bf16) return fail(PHOTON_ERR_UNSUPPORTED, "encoder attention: bf16 output rows come with the bf16 path only");
  if ((int64_t)Bt * H > 65535) return fail(PHOTON_ERR_UNSUPPORTED, "encoder attention: Bt*H=%lld exceeds 65535", (long long)Bt * H);
  const int pitch = kv_row_elems(d_h);
  if (!bf16) {
    dim3 grid((unsigned)((M + 63) / 64), Bt * H);
#define PHOTON_EA_F32(DH)                                                                                                          \
    PHOTON_LAUNCH(KC_LOCAL_ATTN, st, encoder_attn_f32_kernel<DH>, grid, dim3(64), 0, st, qkv, out, (float*)k_cache, (float*)v_cache, M, H, \
                  pitch, S_max, theta, scale)
    switch (d_h) {
      case 16: PHOTON_EA_F32(16); break;
      case 20: PHOTON_EA_F32(20); break;
      case 24: PHOTON_EA_F32(24); break;
      case 28: PHOTON_EA_F32(28); break;
      case 32: PHOTON_EA_F32(32); break;
      case 36: PHOTON_EA_F32(36); break;
      case 40: PHOTON_EA_F32(40); break;
      case 44: PHOTON_EA_F32(44); break;
      case 48: PHOTON_EA_F32(48); break;
      case 52: PHOTON_EA_F32(52); break;
      case 56: PHOTON_EA_F32(56); break;
      case 60: PHOTON_EA_F32(60); break;
      case 64: PHOTON_EA_F32(64); break;
      default: return fail(PHOTON_ERR_UNSUPPORTED, "encoder attention (fp32): head size %d is not a multiple of 4 in [16, 64]", d_h);
    }
#undef PHOTON_EA_F32
    return check_launch("encoder_attn_f32_kernel");
  }
  if (d_h < 4 || d_h > EA_DH || d_h % 4 != 0)
    return fail(PHOTON_ERR_UNSUPPORTED, "encoder attention (bf16): head size %d is not a multiple of 4 in [4, 64]", d_h);
  const int64_t Mp = round_up64(M);
  const size_t arr = (size_t)Bt * H * Mp * EA_DH;
  uint16_t* qh = reinterpret_cast<uint16_t*>(workspace);
  uint16_t *kh = qh + arr, *vt = kh + arr;
#define PHOTON_EA_ROPE(PAD, TC)                                                                                                        \
  PHOTON_LAUNCH(KC_ROPE_APPEND, st, (encoder_rope_split_kernel<PAD, TC>), dim3((unsigned)(Mp / 64), Bt * H), dim3(256), 0, st, qkv, qh, \
                kh, vt, (TC*)k_cache, (TC*)v_cache, M, H, d_h, pitch, S_max, theta, scale * LOG2E)
  if (d_h == EA_DH) { if (kv_fp8) PHOTON_EA_ROPE(false, fp8_t); else PHOTON_EA_ROPE(false, bf16_t); }
  else { if (kv_fp8) PHOTON_EA_ROPE(true, fp8_t); else PHOTON_EA_ROPE(true, bf16_t); }
#undef PHOTON_EA_ROPE
  PHOTON_TRY(check_launch("encoder_rope_split_kernel"));
  const int n_qblocks = (int)((M + EA_BQ - 1) / EA_BQ);
  PHOTON_LAUNCH(KC_LOCAL_ATTN, st, encoder_attn_mfma_kernel, dim3(n_qblocks, Bt * H), dim3(EA_THREADS), 4 * EA_STAGE, st, qh, kh, vt, out, M,
                H, d_h, n_qblocks, out_bf16 ? 1 : 0);
  return check_launch("encoder_attn_mfma_kernel");
}

}  // namespace photon

using namespace photon;

extern "C" size_t photon_encoder_attn_workspace_bytes(int32_t Bt, int64_t M, int32_t H, int32_t d_h, photon_dtype dt) {
  if (Bt <= 0 || M <= 0 || H <= 0 || d_h <= 0) return 0;
  return encoder_attn_workspace_bytes(Bt, M, H, d_h, dt == PHOTON_BF16);
}

extern "C" int32_t photon_encoder_attn(const float* qkv, float* out, int32_t Bt, int64_t M, int32_t H, int32_t d_h, float rope_theta,
                                       float scale, void* k_cache, void* v_cache, int64_t S_max, void* workspace, size_t workspace_bytes,
                                       photon_dtype dt, void* stream) {
  clear_error();
  PHOTON_REQUIRE(valid_dtype(dt), PHOTON_ERR_UNSUPPORTED, "%s: unknown dtype %d", __func__, (int)dt);
  PHOTON_REQUIRE(Bt >= 0 && M >= 0 && H >= 1 && d_h >= 1, PHOTON_ERR_INVALID_ARG, "%s: Bt=%d M=%lld H=%d d_h=%d invalid", __func__, Bt,
                 (long long)M, H, d_h);
  PHOTON_REQUIRE(M <= (1 << 24), PHOTON_ERR_UNSUPPORTED, "%s: M=%lld exceeds 2^24 positions", __func__, (long long)M);
  if (Bt == 0 || M == 0) return PHOTON_OK;
  PHOTON_REQUIRE_PTR(qkv);
  PHOTON_REQUIRE_PTR(out);
  PHOTON_REQUIRE((k_cache == nullptr) == (v_cache == nullptr), PHOTON_ERR_INVALID_ARG, "%s: give both caches or neither", __func__);
  if (k_cache != nullptr) {
    PHOTON_REQUIRE(aligned16(k_cache) && aligned16(v_cache), PHOTON_ERR_INVALID_ARG, "%s: cache is misaligned", __func__);
    PHOTON_REQUIRE(S_max >= M, PHOTON_ERR_INVALID_ARG, "%s: cache pitch S_max=%lld is shorter than M=%lld", __func__, (long long)S_max,
                   (long long)M);
  }
  const size_t need = encoder_attn_workspace_bytes(Bt, M, H, d_h, dt == PHOTON_BF16);
  PHOTON_REQUIRE(workspace_bytes >= need, PHOTON_ERR_INVALID_ARG, "%s: workspace holds %zu bytes, %zu needed", __func__, workspace_bytes, need);
  if (need > 0) PHOTON_REQUIRE_PTR(workspace);
  return launch_encoder_attn(qkv, out, Bt, M, H, d_h, rope_theta, scale, k_cache, v_cache, S_max, workspace, dt == PHOTON_BF16, false, false,
                             (hipStream_t)stream);
}
