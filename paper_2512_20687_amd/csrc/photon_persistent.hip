// Persistent module kernel: every block of a local decoder G^(l) on the few rows of one decode sub-step (paper
// Section 2.3.3 step (i), Eq. 6-7) in ONE launch.
//
// A decode sub-step at small batch multiplies 4-16 rows with every matrix of a module: five dependent maps per
// block (QKV, attention, O, gate/up, down).  As separate launches each of them pays a kernel boundary (launch,
// first-byte latency, tail: about 4.5 us on this chip) and the memory system idles meanwhile.  Here one
// workgroup per compute unit stays resident for the whole module:
//   * the phases of a block are separated by a grid barrier: relaxed agent-scope counters, one per XCD plus a
//     global one, thread 0 of each workgroup arriving and spinning with a bound (a wait that runs out sets an
//     error word and every workgroup leaves: no wave ever waits forever);
//   * what one phase hands the next (a few rows: q|k|v, attention rows, the residual stream, hidden rows) is
//     written with agent-scope write-through stores, waited for before the arrival, and read with agent-scope
//     loads: the eight XCDs' L2 caches are not coherent with each other, these accesses are served beyond them;
//   * the weights of a phase do not depend on what the barrier protects, so a workgroup requests its share of a
//     matrix one to three phases ahead, in groups placed right behind the activation loads of those earlier phases
//     (vector-memory operations of a wave complete in order: a request placed anywhere else would hold back
//     either that phase's stores, and with them the barrier, or the next phase's activations); a wave's whole
//     share of a matrix sits in registers when its phase begins, and HBM streams while the phases before compute;
//   * a linear phase is the few-row resident-activation map (one MFMA tile per 8 output columns, 128-byte weight
//     lines folded into the tile's row halves, fp32 activations split into bf16 head + remainder in LDS, bf16
//     activations taken as fragments straight from memory); both k chunks of a wave are staged before its first
//     MFMA, so that the activations' landing registers are free while the accumulators are live (registers, not
//     LDS, are what this kernel runs out of: a spilled value comes back through the same in-order queue as the
//     weight prefetch and stalls its phase); the waves of a workgroup take their k chunks in an order rotated per
//     workgroup so that the workgroups of an XCD do not all ask for the same activation lines at once; partial
//     tiles are still summed in chunk order, so the arithmetic equals that of the separate launches.
#include "photon_persistent.h"

#include <mutex>

#include "photon_device.h"
#include "photon_host.h"
#include "photon_linear.h"

namespace photon {

namespace {

constexpr int PM_WAVES = 8;
constexpr int PM_THREADS = PM_WAVES * 64;
constexpr int PM_KBLOCK = 64;                  // k per block: 128 bytes of a weight row
constexpr int PM_CB = 2;                       // blocks per chunk
constexpr int PM_RING = 2;                     // chunks per wave of a contraction over the model width (at most 2048)
constexpr int PM_RING_D = 5;                   // chunks per wave of the down projection (d_ff at most 5120)
constexpr int PM_AGENT = 16;                   // cache policy of a buffer access at agent scope (sc1)
constexpr int PM_RSRC_WORD3 = 0x00020000;      // buffer descriptor: raw 32-bit data
constexpr int PM_LDS_LIMIT = 156 * 1024;
constexpr int PM_MAX_NEW_ROWS = 2;             // rows per chunk of a pass (a converter prefix of at most 2 vectors)

__host__ __device__ constexpr int pm_group_pitch(int rows) { return rows * 16 + 16; }
__host__ __device__ constexpr int pm_chunk_bytes(int rows) { return 2 * 16 * pm_group_pitch(rows); }

typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, PM_RSRC_WORD3);
}
// Agent-scope accesses: offsets beyond the descriptor's size read zeros and store nothing.
__device__ __forceinline__ uint4_t ld16_agent(rsrc_t r, uint32_t off) { return __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, PM_AGENT); }
__device__ __forceinline__ void st16_agent(rsrc_t r, uint32_t off, uint4_t v) { __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)off, 0, PM_AGENT); }
__device__ __forceinline__ void st8_agent(rsrc_t r, uint32_t off, uint2_t v) { __builtin_amdgcn_raw_buffer_store_b64(v, r, (int)off, 0, PM_AGENT); }
__device__ __forceinline__ float4_t as_f4(uint4_t v) { return __builtin_bit_cast(float4_t, v); }
__device__ __forceinline__ uint4_t as_u4(float4_t v) { return __builtin_bit_cast(uint4_t, v); }

struct PmLayer {
  const float* g1; const bf16_t* wqkv; const bf16_t* wo; const float* g2; const bf16_t* wgu; const bf16_t* wd;
};
struct PmDeal { int G, ub, ur; };              // workgroups of a phase; units per workgroup: ub, the first ur one more
struct PmArgs {
  PmLayer layer[PM_MAX_LAYERS];
  const float* x_in; int64_t ld_in;
  float* h; float* qkv; bf16_t* attn; bf16_t* act;
  float* lk; float* lv; int64_t layer_cache;
  unsigned* bar; unsigned* err;
  int M, D, F, H, n_layers, n_units, W, q_len, q_pos;
  int wave_bytes;
  float eps, scale_log2e;
  PmDeal dq, dout, dg, dd;
  // cosine and sine of the rotary angles of the (at most PM_MAX_NEW_ROWS) new window positions q_pos + r: entry i is
  // the pair (i, i + d_h/2), angle (q_pos + r) * theta^(-2i/d_h), formed in double on the host (identity for theta = 0)
  float rope_cos[PM_MAX_NEW_ROWS][64], rope_sin[PM_MAX_NEW_ROWS][64];
  long long spin_ticks;                        // bound of a barrier wait in ticks of the constant 100 MHz clock
  unsigned long long* stamps;                  // measurement aid, normally null: workgroup 0 notes the clock at every phase milestone
};

// ---- grid barrier ----------------------------------------------------------------------------------------------
// Workgroup g of G arrives for the round-th time.  bar[0]: arrivals of whole XCD groups; bar[64 * (1 + x)]:
// arrivals of the workgroups with g % 8 == x (the last of them reports the group).  Counters only grow within a
// launch.  Returns false when the wait ran out or another workgroup reported that: the caller leaves the kernel.
// YOUNGER: vector-memory loads this wave has issued, on every path, after its last store of the phase (the weight
// prefetch of later phases).  Vector-memory operations complete in order, so "at most YOUNGER outstanding" means the
// stores have completed while such a prefetch stays in flight across the barrier.  (The schedule in the kernel
// now places every prefetch group ahead of the stores of its phase, where it lands under the phase's arithmetic:
// YOUNGER is 0 at every barrier.)
constexpr int pm_wait_vm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }
template <int YOUNGER>
__device__ __forceinline__ bool grid_sync(unsigned* bar, unsigned* err, int* flag, int g, int G, unsigned round, long long spin_ticks) {
  static_assert(YOUNGER >= 0 && YOUNGER < 64, "the counter has six bits");
  asm volatile("" ::: "memory");               // no memory access moves across this point
  __builtin_amdgcn_s_waitcnt(pm_wait_vm(YOUNGER));   // this lane's write-through stores have completed
  asm volatile("" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    const int x = g & 7, per = (G + 7 - x) / 8;
    const unsigned old = __hip_atomic_fetch_add(bar + 64 * (1 + x), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1 == round * (unsigned)per) __hip_atomic_fetch_add(bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned want = round * (unsigned)(G < 8 ? G : 8);
    const long long t0 = wall_clock64();
    int ok = 1, spins = 0;
    while (__hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < want) {
      if ((spins++ & 63) == 0) {                                   // on the first unsuccessful poll, then every 64th
        if (__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) { ok = 0; break; }
        if (wall_clock64() - t0 > spin_ticks) {
          __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ok = 0;
          break;
        }
      }
      __builtin_amdgcn_s_sleep(1);
    }
    *flag = ok;
  }
  __syncthreads();
  return *flag != 0;
}

// ---- a linear phase --------------------------------------------------------------------------------------------
// What a workgroup and lane need to know about one linear phase; lives from the weight prefetch to the epilogue.
template <int TT> struct LinCtx {
  uint32_t w_lane[TT];                         // byte offset of this lane's weight row in every tile
  int tiles, n0, n_my, total_blocks;
  bool active;
};
template <int TT, int NCH = PM_RING> struct Ring { uint4_t w[NCH][TT][PM_CB]; };

struct LaneId { int g, wave, lane, lrow, lq, cw, rot; };

template <int EPI, int TT>
__device__ __forceinline__ void lin_begin(LinCtx<TT>& c, const PmDeal& d, const LaneId& id, int N, int K) {
  constexpr int UC = (EPI == EPI_SWIGLU) ? 4 : 8;
  c.active = id.g < d.G;
  const int gg = c.active ? id.g : 0;
  c.tiles = d.ub + (gg < d.ur ? 1 : 0);
  c.n0 = (gg * d.ub + (gg < d.ur ? gg : d.ur)) * UC;
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int uu = t < c.tiles ? t : c.tiles - 1;                  // surplus tiles repeat the last one (loaded, never stored)
    const int r = id.lrow & 7;
    const int n = (EPI == EPI_SWIGLU) ? (r < 4 ? 0 : N) + c.n0 + uu * 4 + (r & 3) : c.n0 + uu * 8 + r;
    c.w_lane[t] = ((uint32_t)n * (uint32_t)K + (uint32_t)(id.lq + 4 * (id.lrow >> 3)) * 8u) * 2u;
  }
  c.total_blocks = K / PM_KBLOCK;
  const int chunks = (c.total_blocks + PM_CB - 1) / PM_CB;
  c.n_my = (c.active && id.cw < chunks) ? (chunks - id.cw + PM_WAVES - 1) / PM_WAVES : 0;   // chunks cw, cw + 8, ..
}

// real == false below (a wave without such a chunk, a workgroup without work in the phase, no next block): every lane
// reads the matrix's first 16 bytes instead, so that the ring's registers are defined on every path (a conditionally
// written ring would stay live around the whole layer loop) at no cost.
// One group of a phase's first weight chunks: block b of chunk slot s, TT loads on every path.  The groups of a matrix
// are requested over the phases before its own, a few at a time (see the kernel), so that HBM streams through the
// barriers without any wave's queue holding back its stores or its activation loads for long.
template <int TT, int NCH>
__device__ __forceinline__ void pf_group(const LinCtx<TT>& c, const bf16_t* W, const LaneId& id, Ring<TT, NCH>& ring, int s, int b, bool real = true) {
  real = real && s < c.n_my;
  const int chunk = id.cw + s * PM_WAVES;
  int blk = chunk * PM_CB + b;
  blk = blk < c.total_blocks ? blk : c.total_blocks - 1;
  const char* wb = reinterpret_cast<const char*>(W) + (real ? (int64_t)blk * (PM_KBLOCK * 2) : 0);
#pragma unroll
  for (int t = 0; t < TT; ++t) ring.w[s][t][b] = load16_stream(wb + (real ? c.w_lane[t] : 0u));
}
template <int TT, int NCH>
__device__ __forceinline__ void lin_prefetch(const LinCtx<TT>& c, const bf16_t* W, const LaneId& id, Ring<TT, NCH>& ring, bool real = true) {
#pragma unroll
  for (int s = 0; s < NCH; ++s)
#pragma unroll
    for (int b = 0; b < PM_CB; ++b) pf_group(c, W, id, ring, s, b, real);
}

// Contraction with fp32 activations x[M, K] (row pitch ldx, read at agent scope): each wave loads its chunk of all
// rows, applies the norm gain, splits into bf16 head + remainder in its LDS slot, and meets the weights there.
// early(): called once the first activation loads are on their way (weight prefetch of later phases goes here: behind
// the activations in the wave's queue, ahead of everything else).
// staged(): called when the activations are staged and their landing registers are free (the last group of this
// phase's own weights may be requested there when registers are too scarce to hold it through the staging).
template <int XP, bool NORM, int TT, typename Early, typename Staged>
__device__ __forceinline__ void lin_contract_f32(const LinCtx<TT>& c, const bf16_t* W, const LaneId& id, Ring<TT>& ring, rsrc_t x_r,
                                                 int64_t ldx, const float* gain, int M, int K, char* my_area,
                                                 float4_t (&acc)[TT], float (&ss)[XP], Early&& early, Staged&& staged) {
  constexpr int ROWS = 2 * XP;
  constexpr int GP = pm_group_pitch(ROWS);
#pragma unroll
  for (int i = 0; i < XP; ++i) ss[i] = 0.f;
  const int lane = id.lane;
  const int c4 = lane & 31;
  const uint32_t row_pitch = (uint32_t)ldx * 4u;                   // bytes; a lane's pieces are rows (lane >> 5) + 2 i
  const uint32_t x_lane0 = (uint32_t)(lane >> 5) * row_pitch + (uint32_t)(c4 & 15) * 16u;
  auto load_x = [&](int j, float4_t (&xr)[XP + 1]) {
    const int chunk = id.cw + j * PM_WAVES;
    int blk = chunk * PM_CB + (c4 >> 4);
    blk = blk < c.total_blocks ? blk : c.total_blocks - 1;
    const uint32_t kb = (uint32_t)blk * (PM_KBLOCK * 4);
#pragma unroll
    for (int i = 0; i < XP; ++i)                                    // rows beyond M lie beyond the descriptor and read as zeros
      xr[i] = as_f4(ld16_agent(x_r, x_lane0 + (uint32_t)(2 * i) * row_pitch + kb));
    if (NORM) xr[XP] = *reinterpret_cast<const float4_t*>(reinterpret_cast<const char*>(gain) + (kb + (c4 & 15) * 16));
  };
  constexpr int SLOT = pm_chunk_bytes(ROWS);                       // two staging slots per wave: both chunks of a pair are staged
                                                                   // before the first MFMA, so the landing registers of the
                                                                   // activations are free while the accumulators are live
  auto stage = [&](int j, const float4_t (&xr)[XP + 1]) {
    char* hi = my_area + (j & 1) * SLOT;
    char* lo = hi + 16 * GP;
    const int chunk = id.cw + j * PM_WAVES;
    const bool k_live = chunk * (PM_CB * PM_KBLOCK) + c4 * 4 < K;
    const int group = c4 >> 1;
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const int row = i * 2 + (lane >> 5);
      float4_t v = (k_live && row < M) ? xr[i] : float4_t{0.f, 0.f, 0.f, 0.f};
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
  const int frag_row = (id.lrow & (ROWS - 1)) * 16;                // dead rows read a live row's fragment: never stored
  auto mma = [&](int j, const uint4_t (&w)[TT][PM_CB]) {
    const char* hi = my_area + (j & 1) * SLOT;
    const char* lo = hi + 16 * GP;
    const int chunk = id.cw + j * PM_WAVES;
#pragma unroll
    for (int b = 0; b < PM_CB; ++b) {
      if (chunk * PM_CB + b < c.total_blocks) {
#pragma unroll
        for (int half2 = 0; half2 < 2; ++half2) {
          const int off = ((b * 2 + half2) * 4 + id.lq) * GP + frag_row;
          const bf16x8_t bh = as_bf16x8(*reinterpret_cast<const uint4_t*>(hi + off));
          const bf16x8_t bl = as_bf16x8(*reinterpret_cast<const uint4_t*>(lo + off));
#pragma unroll
          for (int t = 0; t < TT; ++t) {
            const bf16x8_t aw = as_bf16x8(half2 ? rotate8(w[t][b]) : w[t][b]);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aw, bh, acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aw, bl, acc[t], 0, 0, 0);
          }
        }
      }
    }
  };
  // The contraction length here is the model width, at most 2048 (host-checked): a wave has at most two chunks.  Both
  // are requested at once, both are staged before the first MFMA (their landing registers are free again while the
  // accumulators are live), and no ring slot is refilled.
  const int n_my = c.n_my;
  float4_t xa[XP + 1], xb[XP + 1];
  if (n_my > 0) load_x(0, xa);
  if (n_my > 1) load_x(1, xb);
  asm volatile("" ::: "memory");
  early();
  asm volatile("" ::: "memory");
  if (n_my > 0) stage(0, xa);
  if (n_my > 1) stage(1, xb);
  asm volatile("" ::: "memory");
  staged();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int t = 0; t < TT; ++t) acc[t] = float4_t{0.f, 0.f, 0.f, 0.f};
  if (n_my > 0) mma(0, ring.w[0]);
  if (n_my > 1) mma(1, ring.w[1]);
}

// Contraction with bf16 activations x[M, K] (row pitch ldx elements, read at agent scope): they are the MFMA
// operand as they stand, each lane loads its fragments (8 consecutive k of its row) itself.  A wave's whole share of
// chunks (at most NCH, host-checked) is in flight at once: weights in the ring, fragments requested here in one go.
template <int TT, int NCH, typename Early>
__device__ __forceinline__ void lin_contract_bf16(const LinCtx<TT>& c, const LaneId& id, Ring<TT, NCH>& ring, rsrc_t x_r,
                                                  int64_t ldx, int M, float4_t (&acc)[TT], Early&& early) {
  const bool live = id.lrow < M;
  const uint32_t xf_lane = (uint32_t)((int64_t)(live ? id.lrow : 0) * ldx + id.lq * 8) * 2u;
  uint4_t xf[NCH][PM_CB][2];
#pragma unroll
  for (int s = 0; s < NCH; ++s) {
    const int chunk = id.cw + s * PM_WAVES;
#pragma unroll
    for (int b = 0; b < PM_CB; ++b) {
      int blk = chunk * PM_CB + b;
      blk = blk < c.total_blocks ? blk : c.total_blocks - 1;
#pragma unroll
      for (int half2 = 0; half2 < 2; ++half2) {
        xf[s][b][half2] = uint4_t{0u, 0u, 0u, 0u};
        if (live && s < c.n_my) xf[s][b][half2] = ld16_agent(x_r, xf_lane + (uint32_t)blk * (PM_KBLOCK * 2) + half2 * 64);
      }
    }
  }
  asm volatile("" ::: "memory");
  early();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int t = 0; t < TT; ++t) acc[t] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < NCH; ++s) {
    if (s < c.n_my) {
      const int chunk = id.cw + s * PM_WAVES;
#pragma unroll
      for (int b = 0; b < PM_CB; ++b) {
        if (chunk * PM_CB + b < c.total_blocks) {
#pragma unroll
          for (int half2 = 0; half2 < 2; ++half2) {
#pragma unroll
            for (int t = 0; t < TT; ++t) {
              const bf16x8_t aw = as_bf16x8(half2 ? rotate8(ring.w[s][t][b]) : ring.w[s][t][b]);
              acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aw, as_bf16x8(xf[s][b][half2]), acc[t], 0, 0, 0);
            }
          }
        }
      }
    }
  }
}

// End of a linear phase: the waves' partial tiles meet in LDS and are added in chunk order; 1/rms, residual or
// SiLU * up; the finished columns go out with agent-scope stores (fp32, or bf16 for the hidden rows).
template <int EPI, int XP, bool NORM, bool OUT_BF16, int TT>
__device__ __forceinline__ void lin_finish(const LinCtx<TT>& c, const LaneId& id, const float4_t (&acc)[TT], const float (&ss)[XP],
                                           char* smem, int wave_bytes, rsrc_t res_r, int64_t ldres, rsrc_t out_r, int64_t ldo,
                                           int M, int K, float eps) {
  constexpr int UC = (EPI == EPI_SWIGLU) ? 4 : 8;
  float* ssum = reinterpret_cast<float*>(smem + PM_WAVES * wave_bytes);
  const int lane = id.lane;
  if (NORM) {
#pragma unroll
    for (int i = 0; i < XP; ++i) {
      const float v = group_sum<32>(ss[i]);
      if ((lane & 31) == 0) ssum[id.cw * 16 + i * 2 + (lane >> 5)] = v;     // filed under the chunk lane, not the wave
    }
  }
  __syncthreads();                                                 // every wave is done with its staging slot: it is reused
  float4_t* red = reinterpret_cast<float4_t*>(smem + id.cw * wave_bytes);
#pragma unroll
  for (int t = 0; t < TT; ++t) red[t * 64 + lane] = acc[t];
  __syncthreads();
  // wave t finishes tile t.  acc of lane l holds y[row l % 16][tile row (l / 16) * 4 + 0..3] (tile row = output column)
  const int t = id.wave;
  if (c.active && t < TT && t < c.tiles && id.lq < (EPI == EPI_SWIGLU ? 1 : 2) && id.lrow < M) {
    const int m = id.lrow;
    const int n_out = c.n0 + t * UC + id.lq * 4;
    float4_t extra = float4_t{0.f, 0.f, 0.f, 0.f};
    if (EPI == EPI_RESID) extra = as_f4(ld16_agent(res_r, (uint32_t)((int64_t)m * ldres + n_out) * 4u));
    float4_t y = float4_t{0.f, 0.f, 0.f, 0.f}, yu = float4_t{0.f, 0.f, 0.f, 0.f};
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < PM_WAVES; ++w) {                           // chunk lanes in order: the order of the separate launches
      const float4_t* rw = reinterpret_cast<const float4_t*>(smem + w * wave_bytes);
      y += rw[t * 64 + lane];
      if (EPI == EPI_SWIGLU) yu += rw[t * 64 + lane + 16];
      if (NORM) tot += ssum[w * 16 + id.lrow];
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
    if (OUT_BF16)
      st8_agent(out_r, (uint32_t)((int64_t)m * ldo + n_out) * 2u, uint2_t{pack_bf16x2(y.x, y.y), pack_bf16x2(y.z, y.w)});
    else
      st16_agent(out_r, (uint32_t)((int64_t)m * ldo + n_out) * 4u, as_u4(y));
  }
}

// ---- the attention phase ---------------------------------------------------------------------------------------
// Rotary encoding of the q_len new rows of every chunk at their window positions, append of k and v to the chunk's
// local cache, causal attention over the window so far (Eq. 6-7).  One lane group per (chunk, head); the window
// (at most PM_MAX_WINDOW rows) lives in registers.  q|k|v come from the QKV phase (agent scope), the bf16
// attention rows go to the O phase (agent scope); the cache rows of earlier sub-steps were written by earlier
// launches and the new ones are read back by later launches only.
// The window rows of earlier sub-steps do not depend on this block's q | k | v: they are requested a phase ahead.
template <int NK> struct Window { float4_t k[NK], v[NK]; };
template <int DH, int NK>
__device__ __forceinline__ Window<NK> attn_window_load(const PmArgs& a, const LaneId& id, int G, const float* lk, const float* lv) {
  Window<NK> w;
  constexpr int VEC = 4, LPR = DH / 4, UPW = 64 / LPR;
  const int D = a.H * DH;
  const int col = (id.lane % LPR) * VEC;
  const int n_items = (a.n_units + UPW - 1) / UPW;
  const int item = id.wave * G + id.g;
  const bool has = item < n_items;
  int unit = item * UPW + id.lane / LPR;
  unit = unit < a.n_units ? unit : a.n_units - 1;
  const int chunk = unit / a.H, h = unit % a.H;
  const float* kcache = lk + ((int64_t)chunk * a.W * a.H + h) * DH + col;
  const float* vcache = lv + ((int64_t)chunk * a.W * a.H + h) * DH + col;
#pragma unroll
  for (int j = 0; j < NK; ++j) {
    const bool on = has && j < a.q_pos;                            // other rows: the first row again (in bounds), never used
    w.k[j] = *reinterpret_cast<const float4_t*>(kcache + (on ? (int64_t)j * D : 0));
    w.v[j] = *reinterpret_cast<const float4_t*>(vcache + (on ? (int64_t)j * D : 0));
  }
  return w;
}

template <int DH, int NK, typename Early>
__device__ __forceinline__ void attn_phase(const PmArgs& a, const LaneId& id, int G, rsrc_t qkv_r, rsrc_t attn_r, float* lk, float* lv,
                                           const Window<NK>& win, Early&& early) {
  constexpr int VEC = 4, LPR = DH / 4, UPW = 64 / LPR;
  float4_t kr[NK], vr[NK];
#pragma unroll
  for (int j = 0; j < NK; ++j) { kr[j] = win.k[j]; vr[j] = win.v[j]; }
  const int lane = id.lane;
  const int D = a.H * DH, half = DH / 2;
  const int col = (lane % LPR) * VEC;
  const bool upper = col >= half;                                  // this lane holds the i + d_h/2 members of the rotary pairs
  // one item (UPW units) per wave at most (host-checked: the grid's waves cover all units), spread over workgroups first
  const int n_items = (a.n_units + UPW - 1) / UPW;
  const int item = id.wave * G + id.g;
  const bool has = item < n_items;
  int unit = item * UPW + lane / LPR;
  const bool live = has && unit < a.n_units;
  unit = unit < a.n_units ? unit : a.n_units - 1;
  const int chunk = unit / a.H, h = unit % a.H;
  float* kcache = lk + ((int64_t)chunk * a.W * a.H + h) * DH + col;
  float* vcache = lv + ((int64_t)chunk * a.W * a.H + h) * DH + col;
  // q | k | v of every new row of the chunk, requested before anything else
  float4_t q4[PM_MAX_NEW_ROWS], k4[PM_MAX_NEW_ROWS], v4[PM_MAX_NEW_ROWS];
#pragma unroll
  for (int r = 0; r < PM_MAX_NEW_ROWS; ++r) {
    q4[r] = k4[r] = v4[r] = float4_t{0.f, 0.f, 0.f, 0.f};
    if (has && r < a.q_len) {
      const uint32_t off = (uint32_t)((int64_t)(chunk * a.q_len + r) * 3 * D + h * DH + col) * 4u;
      q4[r] = as_f4(ld16_agent(qkv_r, off));
      k4[r] = as_f4(ld16_agent(qkv_r, off + (uint32_t)D * 4u));
      v4[r] = as_f4(ld16_agent(qkv_r, off + (uint32_t)D * 8u));
    }
  }
  asm volatile("" ::: "memory");
  early();                                                         // weight prefetch of later phases: behind this phase's own loads
  asm volatile("" ::: "memory");
  if (!has) return;
#pragma unroll
  for (int r = 0; r < PM_MAX_NEW_ROWS; ++r) {
    if (r < a.q_len) {
      const int pos = a.q_pos + r;
      const int row = chunk * a.q_len + r;
      float qa[VEC] = {q4[r].x, q4[r].y, q4[r].z, q4[r].w}, ka[VEC] = {k4[r].x, k4[r].y, k4[r].z, k4[r].w};
      const float4_t cs4 = *reinterpret_cast<const float4_t*>(&a.rope_cos[r][col % half]);
      const float4_t sn4 = *reinterpret_cast<const float4_t*>(&a.rope_sin[r][col % half]);
      const float csv[VEC] = {cs4.x, cs4.y, cs4.z, cs4.w}, snv[VEC] = {sn4.x, sn4.y, sn4.z, sn4.w};
#pragma unroll
      for (int t = 0; t < VEC; ++t) {
        const float qb = __shfl_xor(qa[t], LPR / 2), kb = __shfl_xor(ka[t], LPR / 2);   // the partner sits LPR/2 lanes away
        const float sn = upper ? snv[t] : -snv[t];
        qa[t] = qa[t] * csv[t] + qb * sn;
        ka[t] = ka[t] * csv[t] + kb * sn;
      }
      const float4_t k_new = float4_t{ka[0], ka[1], ka[2], ka[3]};
      if (live) {
        *reinterpret_cast<float4_t*>(kcache + (int64_t)pos * D) = k_new;
        *reinterpret_cast<float4_t*>(vcache + (int64_t)pos * D) = v4[r];
      }
#pragma unroll
      for (int j = 0; j < NK; ++j)
        if (j == pos) { kr[j] = k_new; vr[j] = v4[r]; }
      float s[NK], mx = NEG_BIG;
#pragma unroll
      for (int j = 0; j < NK; ++j) {
        s[j] = NEG_BIG;
        if (j <= pos) {
          float acc = qa[0] * kr[j].x;
          acc = fmaf(qa[1], kr[j].y, acc);
          acc = fmaf(qa[2], kr[j].z, acc);
          acc = fmaf(qa[3], kr[j].w, acc);
          s[j] = group_sum<LPR>(acc) * a.scale_log2e;
          mx = fmaxf(mx, s[j]);
        }
      }
      float l = 0.f;
      float4_t o = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < NK; ++j) {
        if (j <= pos) {
          const float pw = fast_exp2(s[j] - mx);
          l += pw;
          o += pw * vr[j];
        }
      }
      o *= (1.f / l);
      if (live) st8_agent(attn_r, (uint32_t)((int64_t)row * D + h * DH + col) * 2u, uint2_t{pack_bf16x2(o.x, o.y), pack_bf16x2(o.z, o.w)});
    }
  }
}

// ---- the kernel ------------------------------------------------------------------------------------------------
// XP: live row pairs (rows <= 2 * XP); TQ / TO / TG / TD: MFMA tiles per workgroup of the QKV, O, gate/up and down
// phases; DH: head size; NK: window positions held in registers (4 or 8).
template <int XP, int TQ, int TO, int TG, int TD, int DH, int NK>
__global__ __launch_bounds__(PM_THREADS) void persistent_module_kernel(const PmArgs a) {
  extern __shared__ __align__(16) char smem[];                     // [8 waves][wave_bytes] | row statistics [8][16] | flag
  LaneId id;
  id.g = blockIdx.x;
  id.lane = threadIdx.x & 63;
  id.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  id.lrow = id.lane & 15;
  id.lq = id.lane >> 4;
  id.rot = (id.g >> 3) & 7;
  id.cw = (id.wave + id.rot) & 7;
  const int G = gridDim.x;
  int* flag = reinterpret_cast<int*>(smem + PM_WAVES * a.wave_bytes + PM_WAVES * 16 * sizeof(float));
  char* my_area = smem + id.cw * a.wave_bytes;
  const int M = a.M, D = a.D, F = a.F;

  const rsrc_t h_r = make_rsrc(a.h, (uint32_t)M * D * 4u);
  const rsrc_t qkv_r = make_rsrc(a.qkv, (uint32_t)M * 3u * D * 4u);
  const rsrc_t mid_r = make_rsrc(a.qkv, (uint32_t)M * D * 4u);     // the mid-block stream reuses the q|k|v buffer
  const rsrc_t attn_r = make_rsrc(a.attn, (uint32_t)M * D * 2u);
  const rsrc_t act_r = make_rsrc(a.act, (uint32_t)M * F * 2u);
  const rsrc_t in_r = make_rsrc(a.x_in, (uint32_t)(((int64_t)(M - 1) * a.ld_in + D) * 4));

  Ring<TQ> rq;                                                     // carried from one block to the next
  {
    LinCtx<TQ> cq0;
    lin_begin<EPI_PLAIN, TQ>(cq0, a.dq, id, 3 * D, D);
    lin_prefetch(cq0, a.layer[0].wqkv, id, rq);
  }

  // Weight prefetch schedule.  Vector-memory operations of a wave complete in order: whatever is requested before a
  // phase's stores holds their completion (and so the arrival at the barrier) back until it has landed, and whatever
  // is outstanding at a barrier holds back the next phase's activation loads.  So a matrix is requested in groups
  // (chunk slot, block) of about 2-10 MB over the chip, each right BEHIND the activation loads of an earlier phase,
  // where it has that phase's arithmetic and epilogue (about 3 us) to land: roughly a fifth of a block's bytes per phase.
  //   QKV phase    O (all groups), gate/up (0,0)
  //   attention    gate/up (0,1), (1,0)
  //   O phase      gate/up (1,1) [up to 8 rows], down chunks 0-1
  //   gate/up      once its activations are staged (registers are scarcest before): gate/up (1,1) [9-16 rows],
  //                down chunks 2-4, next QKV (0,0)
  //   down phase   next QKV (0,1), (1,0), (1,1)
  int n_stamp = 0;
  auto stamp = [&]() {
    if (a.stamps != nullptr && id.g == 0 && threadIdx.x == 0) a.stamps[n_stamp++] = wall_clock64();
  };
  unsigned round = 0;
  for (int i = 0; i < a.n_layers; ++i) {
    // Everything derived from the lane number is formed afresh in every block (the empty statement below hides the
    // lane number from the optimiser): hoisted out of the loop, these values would occupy registers, or be spilled,
    // around all phases, and a reload from scratch queues behind the weight prefetch like any other load.
    {
      int lane_v = threadIdx.x & 63;
      asm volatile("" : "+v"(lane_v));
      id.lane = lane_v;
      id.lrow = lane_v & 15;
      id.lq = lane_v >> 4;
    }
    LinCtx<TQ> cq; LinCtx<TO> co; LinCtx<TG> cg; LinCtx<TD> cd;
    lin_begin<EPI_PLAIN, TQ>(cq, a.dq, id, 3 * D, D);
    lin_begin<EPI_RESID, TO>(co, a.dout, id, D, D);
    lin_begin<EPI_SWIGLU, TG>(cg, a.dg, id, F, D);
    lin_begin<EPI_RESID, TD>(cd, a.dd, id, D, F);
    const PmLayer& L = a.layer[i];
    const bool more = i + 1 < a.n_layers;
    const bf16_t* wq_next = a.layer[more ? i + 1 : i].wqkv;
    const rsrc_t x_r = i == 0 ? in_r : h_r;                        // the block's input rows: the residual stream so far
    const int64_t ldx = i == 0 ? a.ld_in : D;
    float ss[XP];
    Ring<TO> ro; Ring<TG> rg; Ring<TD, PM_RING_D> rd;
    Window<NK> win;                                                // the attention's window rows of earlier sub-steps
    float* lk_i = a.lk + (int64_t)i * a.layer_cache;
    float* lv_i = a.lv + (int64_t)i * a.layer_cache;
    {                                                              // q | k | v = rmsnorm(x; g1) Wqkv^T
      float4_t acc[TQ];
      lin_contract_f32<XP, true, TQ>(cq, L.wqkv, id, rq, x_r, ldx, L.g1, M, D, my_area, acc, ss, [&]() {
        win = attn_window_load<DH, NK>(a, id, G, lk_i, lv_i);
        lin_prefetch(co, L.wo, id, ro);
        pf_group(cg, L.wgu, id, rg, 0, 0);
      }, []() {});
      stamp();
      lin_finish<EPI_PLAIN, XP, true, false, TQ>(cq, id, acc, ss, smem, a.wave_bytes, qkv_r, 0, qkv_r, 3 * D, M, D, a.eps);
      stamp();
    }
    if (!grid_sync<0>(a.bar, a.err, flag, id.g, G, ++round, a.spin_ticks)) return;
    stamp();
    attn_phase<DH, NK>(a, id, G, qkv_r, attn_r, lk_i, lv_i, win, [&]() { pf_group(cg, L.wgu, id, rg, 0, 1); pf_group(cg, L.wgu, id, rg, 1, 0); });
    stamp();
    if (!grid_sync<0>(a.bar, a.err, flag, id.g, G, ++round, a.spin_ticks)) return;
    stamp();
    {                                                              // mid = x + attn Wo^T
      float4_t acc[TO];
      lin_contract_bf16<TO, PM_RING>(co, id, ro, attn_r, D, M, acc, [&]() {
        if (XP < 8) pf_group(cg, L.wgu, id, rg, 1, 1);
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) { pf_group(cd, L.wd, id, rd, sl, 0); pf_group(cd, L.wd, id, rd, sl, 1); }
      });
      stamp();
      lin_finish<EPI_RESID, XP, false, false, TO>(co, id, acc, ss, smem, a.wave_bytes, x_r, ldx, mid_r, D, M, D, a.eps);
      stamp();
    }
    if (!grid_sync<0>(a.bar, a.err, flag, id.g, G, ++round, a.spin_ticks)) return;
    stamp();
    {                                                              // act = silu(n Wg^T) * (n Wu^T), n = rmsnorm(mid; g2)
      float4_t acc[TG];
      lin_contract_f32<XP, true, TG>(cg, L.wgu, id, rg, mid_r, D, L.g2, M, D, my_area, acc, ss, []() {}, [&]() {
        if (XP == 8) pf_group(cg, L.wgu, id, rg, 1, 1);
#pragma unroll
        for (int sl = 2; sl < PM_RING_D; ++sl) { pf_group(cd, L.wd, id, rd, sl, 0); pf_group(cd, L.wd, id, rd, sl, 1); }
        pf_group(cq, wq_next, id, rq, 0, 0, more);
      });
      stamp();
      lin_finish<EPI_SWIGLU, XP, true, true, TG>(cg, id, acc, ss, smem, a.wave_bytes, act_r, 0, act_r, F, M, D, a.eps);
      stamp();
    }
    if (!grid_sync<0>(a.bar, a.err, flag, id.g, G, ++round, a.spin_ticks)) return;
    stamp();
    {                                                              // h = mid + act Wd^T
      float4_t acc[TD];
      lin_contract_bf16<TD, PM_RING_D>(cd, id, rd, act_r, F, M, acc, [&]() {
        pf_group(cq, wq_next, id, rq, 0, 1, more);
        pf_group(cq, wq_next, id, rq, 1, 0, more);
        pf_group(cq, wq_next, id, rq, 1, 1, more);
      });
      stamp();
      lin_finish<EPI_RESID, XP, false, false, TD>(cd, id, acc, ss, smem, a.wave_bytes, mid_r, D, h_r, D, M, F, a.eps);
      stamp();
    }
    if (more && !grid_sync<0>(a.bar, a.err, flag, id.g, G, ++round, a.spin_ticks)) return;
    stamp();
  }
}

// ---- host side -------------------------------------------------------------------------------------------------
struct Deal { int units, G, ub, ur, tmax; };

// The unit deal of the few-row resident map: units of 8 output columns (SwiGLU: 4) over at most 256 workgroups.
Deal deal_units(int N, bool swiglu, bool x_bf16) {
  Deal d;
  d.units = N / (swiglu ? 4 : 8);
  constexpr int CUS = 256;
  const int cap = x_bf16 ? 6 : 8;
  const int rounds = (d.units + CUS * cap - 1) / (CUS * cap);
  d.G = d.units < CUS * rounds ? d.units : CUS * rounds;
  d.ub = d.units / d.G;
  d.ur = d.units % d.G;
  d.tmax = d.ub + (d.ur ? 1 : 0);
  return d;
}

struct Shape { int xp, tq, to, tg, td, dh, nk; Deal dq, dout, dg, dd; int grid, wave_bytes; size_t lds; };

bool plan_shape(const PersistentModule& a, Shape& s) {
  if (a.M < 1 || a.M > PM_MAX_ROWS || a.n_layers < 1 || a.n_layers > PM_MAX_LAYERS || a.F <= 0) return false;
  if (a.d_h != 64 && a.d_h != 128) return false;
  if (a.H * a.d_h != a.D || a.D % PM_KBLOCK != 0 || a.F % PM_KBLOCK != 0) return false;
  if (a.D > PM_WAVES * PM_RING * PM_CB * PM_KBLOCK) return false;  // a wave holds its whole share of chunks: two over the model width,
  if (a.F > PM_WAVES * PM_RING_D * PM_CB * PM_KBLOCK) return false;  // five over d_ff
  if (a.q_pos + a.q_len > PM_MAX_WINDOW || a.W > PM_MAX_WINDOW || a.q_len < 1 || a.q_len > PM_MAX_NEW_ROWS) return false;
  if (a.n_chunks * a.q_len != a.M) return false;
  if ((int64_t)a.M * a.ld_in * 4 >= ((int64_t)1 << 31) || a.ld_in % 4 != 0) return false;
  if ((int64_t)3 * a.D * a.D * 2 >= ((int64_t)1 << 32) || (int64_t)2 * a.F * a.D * 2 >= ((int64_t)1 << 32)) return false;   // 32-bit weight offsets
  s.xp = a.M <= 4 ? 2 : a.M <= 8 ? 4 : 8;
  s.dh = a.d_h;
  s.nk = a.W <= 4 ? 4 : 8;
  s.dq = deal_units(3 * a.D, false, false);
  s.dout = deal_units(a.D, false, true);
  s.dg = deal_units(a.F, true, false);
  s.dd = deal_units(a.D, false, true);
  if (s.dq.G > 256 || s.dout.G > 256 || s.dg.G > 256 || s.dd.G > 256) return false;
  s.tq = s.dq.tmax; s.to = s.dout.tmax; s.tg = s.dg.tmax; s.td = s.dd.tmax;
  s.grid = s.dq.G;
  if (s.dout.G > s.grid) s.grid = s.dout.G;
  if (s.dg.G > s.grid) s.grid = s.dg.G;
  if (s.dd.G > s.grid) s.grid = s.dd.G;
  {                                                                // attention: at most one item (64 lanes of units) per wave
    const int upw = 64 / (a.d_h / 4);
    const int64_t items = (a.n_chunks * a.H + upw - 1) / upw;
    if (items > (int64_t)s.grid * PM_WAVES) return false;
  }
  int tmax = s.tq > s.tg ? s.tq : s.tg;
  if (s.to > tmax) tmax = s.to;
  if (s.td > tmax) tmax = s.td;
  s.wave_bytes = 2 * pm_chunk_bytes(2 * s.xp);                     // two staging slots per wave
  if (s.wave_bytes < tmax * 1024) s.wave_bytes = tmax * 1024;      // the partial tiles reuse the staging slot
  s.lds = (size_t)PM_WAVES * s.wave_bytes + PM_WAVES * 16 * sizeof(float) + 16;
  return s.lds <= (size_t)PM_LDS_LIMIT;
}

typedef void (*PmKernel)(const PmArgs);

template <int XP, int TQ, int TO, int TG, int TD>
PmKernel kernel_for_dh(int dh, int nk) {
  // 9-16 rows with a window of 5-8 positions at the widest deals does not fit the register file without spilling, and
  // a reload from scratch would queue behind the weight prefetch: those passes keep the separate launches
  if constexpr (XP == 8 && TQ >= 3) {
    if (nk != 4) return nullptr;
    return dh == 64 ? persistent_module_kernel<XP, TQ, TO, TG, TD, 64, 4> : persistent_module_kernel<XP, TQ, TO, TG, TD, 128, 4>;
  }
  if (nk == 4) return dh == 64 ? persistent_module_kernel<XP, TQ, TO, TG, TD, 64, 4> : persistent_module_kernel<XP, TQ, TO, TG, TD, 128, 4>;
  return dh == 64 ? persistent_module_kernel<XP, TQ, TO, TG, TD, 64, 8> : persistent_module_kernel<XP, TQ, TO, TG, TD, 128, 8>;
}

template <int TQ, int TO, int TG, int TD>
PmKernel kernel_for_xp(int xp, int dh, int nk) {
  switch (xp) {
    case 2: return kernel_for_dh<2, TQ, TO, TG, TD>(dh, nk);
    case 4: return kernel_for_dh<4, TQ, TO, TG, TD>(dh, nk);
    default: return kernel_for_dh<8, TQ, TO, TG, TD>(dh, nk);
  }
}

// The compiled unit deals (tiles per workgroup of the QKV, O, gate/up, down phases).
PmKernel kernel_for(const Shape& s) {
  const int key = s.tq * 1000 + s.to * 100 + s.tg * 10 + s.td;
  switch (key) {
    case 1111: return kernel_for_xp<1, 1, 1, 1>(s.xp, s.dh, s.nk);       // widths up to 680
    case 1121: return kernel_for_xp<1, 1, 2, 1>(s.xp, s.dh, s.nk);       // D = 512, d_ff = 1280
    case 2131: return kernel_for_xp<2, 1, 3, 1>(s.xp, s.dh, s.nk);       // D = 1024, d_ff = 2560
    case 3141: return kernel_for_xp<3, 1, 4, 1>(s.xp, s.dh, s.nk);       // D = 1664, d_ff = 4096
    case 3151: return kernel_for_xp<3, 1, 5, 1>(s.xp, s.dh, s.nk);       // D = 1792 .. 2048, d_ff = 4608 .. 5120
  }
  return nullptr;
}

unsigned long long* g_pm_stamps = nullptr;                         // see persistent_module_set_stamps
long long g_pm_spin_ticks = 1000000000LL;                          // bound of a barrier wait: 10 s of the 100 MHz clock
struct KernelState { bool checked = false, ok = false; };
std::mutex g_pm_mu;
constexpr int PM_MAX_DEVICES = 64;
KernelState g_pm_state[PM_MAX_DEVICES][5][3][2][2];              // per device: attributes and occupancy are the device's

// One-time set-up of an instantiation: allow its dynamic LDS, and make sure the device holds the whole grid at once.
bool kernel_ready(PmKernel k, const Shape& s) {
  const int key = s.tq * 1000 + s.to * 100 + s.tg * 10 + s.td;
  const int ki = key == 1111 ? 0 : key == 1121 ? 1 : key == 2131 ? 2 : key == 3141 ? 3 : 4;
  const int xi = s.xp == 2 ? 0 : s.xp == 4 ? 1 : 2;
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= PM_MAX_DEVICES) {
    (void)hipGetLastError();
    return false;
  }
  std::lock_guard<std::mutex> lk(g_pm_mu);
  KernelState& st = g_pm_state[dev][ki][xi][s.dh == 64 ? 0 : 1][s.nk == 4 ? 0 : 1];
  if (st.checked) return st.ok;
  st.checked = true;
  st.ok = false;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, PM_LDS_LIMIT) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(k), PM_THREADS, PM_LDS_LIMIT) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  st.ok = per_cu >= 1 && (int64_t)per_cu * cus >= 256;               // every workgroup of the largest grid is resident at once
  return st.ok;
}

}  // namespace

void persistent_module_set_stamps(unsigned long long* device_buffer) { g_pm_stamps = device_buffer; }
void persistent_module_set_spin_ticks(long long ticks) { g_pm_spin_ticks = ticks > 0 ? ticks : 1; }

bool persistent_module_supported(const PersistentModule& a) {
  Shape s;
  if (!plan_shape(a, s)) return false;
  PmKernel k = kernel_for(s);
  return k != nullptr && kernel_ready(k, s);
}

int32_t launch_persistent_module(const PersistentModule& a, hipStream_t st) {
  Shape s;
  if (!plan_shape(a, s)) return fail(PHOTON_ERR_UNSUPPORTED, "persistent module: no kernel for these sizes");
  PmKernel k = kernel_for(s);
  if (k == nullptr || !kernel_ready(k, s)) return fail(PHOTON_ERR_UNSUPPORTED, "persistent module: no kernel for this unit deal, or the grid is not co-resident");
  PmArgs p;
  for (int i = 0; i < a.n_layers; ++i) {
    const photon_layer_weights& lw = a.layers[i];
    p.layer[i] = PmLayer{lw.g1, (const bf16_t*)lw.wqkv, (const bf16_t*)lw.wo, lw.g2, (const bf16_t*)lw.wgu, (const bf16_t*)lw.wd};
  }
  for (int i = a.n_layers; i < PM_MAX_LAYERS; ++i) p.layer[i] = p.layer[0];
  p.x_in = a.x_in; p.ld_in = a.ld_in;
  p.h = a.h; p.qkv = a.qkv; p.attn = (bf16_t*)a.attn; p.act = (bf16_t*)a.act;
  p.lk = a.lk; p.lv = a.lv; p.layer_cache = (int64_t)a.layer_cache;
  p.bar = a.bar; p.err = a.err;
  p.M = a.M; p.D = a.D; p.F = a.F; p.H = a.H; p.n_layers = a.n_layers; p.n_units = (int)(a.n_chunks * a.H);
  p.W = a.W; p.q_len = a.q_len; p.q_pos = a.q_pos;
  p.wave_bytes = s.wave_bytes;
  p.eps = a.eps; p.scale_log2e = a.scale * LOG2E;
  for (int r = 0; r < PM_MAX_NEW_ROWS; ++r)
    for (int i = 0; i < 64; ++i) {
      const double ang = (a.theta == 0.f || i >= a.d_h / 2) ? 0.0 : (double)(a.q_pos + r) * pow((double)a.theta, -2.0 * i / (double)a.d_h);
      p.rope_cos[r][i] = (float)cos(ang);
      p.rope_sin[r][i] = (float)sin(ang);
    }
  p.dq = PmDeal{s.dq.G, s.dq.ub, s.dq.ur};
  p.dout = PmDeal{s.dout.G, s.dout.ub, s.dout.ur};
  p.dg = PmDeal{s.dg.G, s.dg.ub, s.dg.ur};
  p.dd = PmDeal{s.dd.G, s.dd.ub, s.dd.ur};
  p.spin_ticks = g_pm_spin_ticks;
  p.stamps = g_pm_stamps;
  PHOTON_LAUNCH(KC_PERSISTENT, st, k, dim3(s.grid), dim3(PM_THREADS), s.lds, st, p);
  return check_launch("persistent_module_kernel");
}

}  // namespace photon
