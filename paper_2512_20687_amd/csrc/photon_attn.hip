// Attention kernels of the PHOTON decode path for gfx950.
//
//  * coarse_attn_kernel: single-query attention over the coarsest stream's KV
//    cache (STEP operator, paper Eq. 12-13).  HBM-bound streaming: every K/V
//    byte is used once, so the S axis is split over workgroups, each lane
//    issues 128-bit loads that together cover whole 128-byte+ rows, scores are
//    reduced inside lane groups with DPP moves, the online-softmax states of
//    the lane groups and waves are merged through shuffles and LDS, and the
//    splits through a small fp32 workspace in a fixed order.
//  * local_attn_kernel: chunk-local causal attention of the local decoders
//    (paper Eq. 6-7).  A window has at most 16 positions, so one lane group
//    keeps a whole (chunk, head) K/V tile in registers; nothing is re-read.
#include "photon_attn.h"

#include <mutex>

#include "photon_device.h"
#include "photon_host.h"

namespace photon {

// ------------------------------------------------------------------ coarse stream

constexpr int COARSE_WAVES_PER_WG = 8;   // measured: 8 waves x 4 loads in flight per buffer streams best
constexpr int COARSE_UNROLL = 4;

template <typename TKV, int DH> struct RowMap {
  static constexpr int VEC = 16 / sizeof(TKV);      // elements per 16-byte lane chunk
  static constexpr int LPR = DH / VEC;              // lanes that cover one row
  static constexpr int RPW = 64 / LPR;              // rows one wave covers per load
  static_assert(LPR >= 1 && LPR <= 32 && (LPR & (LPR - 1)) == 0, "row must map to 1..32 lanes");
};

// Online-softmax state of one lane group: running max m (log2 domain), sum l, weighted values o.
template <int VEC> struct SoftState {
  float m, l, o[VEC];
  __device__ __forceinline__ void init() {
    m = NEG_BIG; l = 0.f;
#pragma unroll
    for (int i = 0; i < VEC; ++i) o[i] = 0.f;
  }
};

// COARSE_WAVES waves per workgroup; U 16-byte K loads (and as many V loads) in flight per lane and register buffer.
// DH: elements of a cache row (32, 64 or 128); d_h <= DH: head size, the row length of q and out.  Cache columns
// d_h .. DH-1 hold zeros and meet zero query elements.
template <typename TKV, typename TQ, int DH, int COARSE_WAVES, int U>
__global__ __launch_bounds__(COARSE_WAVES * 64) void coarse_attn_kernel(
    const TQ* __restrict__ q, const TKV* __restrict__ kc, const TKV* __restrict__ vc,
    const int32_t* __restrict__ seq_len, TQ* __restrict__ out, float* __restrict__ ws,
    int H, int d_h, int64_t S_max, float scale_log2e, int n_splits) {
  using M = RowMap<TKV, DH>;
  constexpr int VEC = M::VEC, LPR = M::LPR, RPW = M::RPW;
  constexpr int TILE = RPW * U;                       // keys one wave consumes per buffer

  const int split = blockIdx.x;
  const int bh = blockIdx.y;
  const int b = bh / H;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int g = lane / LPR, c = lane % LPR;

  int64_t n = seq_len[b];
  n = n < 0 ? 0 : (n > S_max ? S_max : n);
  int64_t per = (n + n_splits - 1) / n_splits;
  per = (per + TILE - 1) / TILE * TILE;
  const int64_t begin = (int64_t)split * per;
  const int64_t end = begin + per < n ? begin + per : n;

  // the query is fetched first but only converted after the first K/V slab is in flight
  TQ qraw[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) qraw[i] = c * VEC + i < d_h ? q[(int64_t)bh * d_h + c * VEC + i] : TQ{};
  float qf[VEC];

  const TKV* kb = kc + (int64_t)bh * S_max * DH + c * VEC;
  const TKV* vb = vc + (int64_t)bh * S_max * DH + c * VEC;

  SoftState<VEC> st;
  st.init();

  // Loads use a clamped key index (always in bounds); keys past `end` get weight 0.
  auto load = [&](int64_t t0, uint4_t (&kr)[U], uint4_t (&vr)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int64_t key = t0 + u * RPW + g;
      key = key < end ? key : end - 1;
      kr[u] = load16_stream(kb + key * DH);
      vr[u] = load16_stream(vb + key * DH);
    }
  };
  auto consume = [&](int64_t t0, const uint4_t (&kr)[U], const uint4_t (&vr)[U]) {
    float s[U];
    float mx = st.m;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[VEC];
      unpack16<TKV>(kr[u], kf);
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc = fmaf(qf[i], kf[i], acc);
      s[u] = group_sum<LPR>(acc);
      const bool ok = t0 + u * RPW + g < end;
      s[u] = ok ? s[u] : NEG_BIG;
      mx = fmaxf(mx, s[u]);
    }
    const float alpha = fast_exp2(st.m - mx);
    st.m = mx;
    st.l *= alpha;
#pragma unroll
    for (int i = 0; i < VEC; ++i) st.o[i] *= alpha;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool ok = t0 + u * RPW + g < end;
      const float p = ok ? fast_exp2(s[u] - mx) : 0.f;
      st.l += p;
      float vf[VEC];
      unpack16<TKV>(vr[u], vf);
#pragma unroll
      for (int i = 0; i < VEC; ++i) st.o[i] = fmaf(p, vf[i], st.o[i]);
    }
  };

  // Waves take TILE-key slabs round-robin; two register buffers keep the next slab in flight.
  const int64_t stride = (int64_t)COARSE_WAVES * TILE;
  int64_t t0 = begin + (int64_t)wave * TILE;
  if (t0 < end) {
    uint4_t ka[U], va[U], kb2[U], vb2[U];
    load(t0, ka, va);
#pragma unroll
    for (int i = 0; i < VEC; ++i) qf[i] = to_f32<TQ>(qraw[i]) * scale_log2e;
    while (true) {
      const int64_t t1 = t0 + stride;
      const bool more1 = t1 < end;
      if (more1) load(t1, kb2, vb2);
      consume(t0, ka, va);
      if (!more1) break;
      const int64_t t2 = t1 + stride;
      const bool more2 = t2 < end;
      if (more2) load(t2, ka, va);
      consume(t1, kb2, vb2);
      if (!more2) break;
      t0 = t2;
    }
  }

  // Merge the RPW lane groups of the wave (lanes with equal c).
#pragma unroll
  for (int mask = LPR; mask < 64; mask <<= 1) {
    const float m2 = __shfl_xor(st.m, mask);
    const float mm = fmaxf(st.m, m2);
    const float a1 = fast_exp2(st.m - mm), a2 = fast_exp2(m2 - mm);
    st.l = st.l * a1 + __shfl_xor(st.l, mask) * a2;
#pragma unroll
    for (int i = 0; i < VEC; ++i) st.o[i] = st.o[i] * a1 + __shfl_xor(st.o[i], mask) * a2;
    st.m = mm;
  }

  // Merge the waves through LDS.
  __shared__ float sm[COARSE_WAVES], sl[COARSE_WAVES], so[COARSE_WAVES][DH];
  if (g == 0) {
#pragma unroll
    for (int i = 0; i < VEC; ++i) so[wave][c * VEC + i] = st.o[i];
    if (c == 0) { sm[wave] = st.m; sl[wave] = st.l; }
  }
  __syncthreads();
  if (tid < DH) {
    float mm = sm[0];
#pragma unroll
    for (int w = 1; w < COARSE_WAVES; ++w) mm = fmaxf(mm, sm[w]);
    float l = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < COARSE_WAVES; ++w) {
      const float a = fast_exp2(sm[w] - mm);
      l = fmaf(sl[w], a, l);
      o = fmaf(so[w][tid], a, o);
    }
    if (n_splits == 1) {
      if (tid < d_h) out[(int64_t)bh * d_h + tid] = from_f32<TQ>(l > 0.f ? o / l : 0.f);
    } else {
      float* p = ws + ((int64_t)bh * n_splits + split) * (DH + 2);
      if (tid == 0) { p[0] = mm; p[1] = l; }
      p[2 + tid] = o;
    }
  }
}

// Merge the split partials of one (b, h) stream in split order.
template <typename TQ, int DH>
__global__ __launch_bounds__(DH) void coarse_merge_kernel(const float* __restrict__ ws, TQ* __restrict__ out, int n_splits, int d_h) {
  const int bh = blockIdx.x, d = threadIdx.x;
  const float* p = ws + (int64_t)bh * n_splits * (DH + 2);
  float mm = NEG_BIG;
  for (int s = 0; s < n_splits; ++s) mm = fmaxf(mm, p[s * (DH + 2)]);
  float l = 0.f, o = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float a = fast_exp2(p[s * (DH + 2)] - mm);
    l = fmaf(p[s * (DH + 2) + 1], a, l);
    o = fmaf(p[s * (DH + 2) + 2 + d], a, o);
  }
  if (d < d_h) out[(int64_t)bh * d_h + d] = from_f32<TQ>(l > 0.f ? o / l : 0.f);
}

template <typename TKV, typename TQ, int DH, int WAVES, int U>
static int32_t launch_coarse_v(const void* q, const void* kc, const void* vc, const int32_t* seq_len, void* out,
                               int Bt, int H, int d_h, int64_t S_max, float scale, int n_splits, void* ws, hipStream_t st) {
  dim3 grid(n_splits, Bt * H);
  PHOTON_LAUNCH(KC_COARSE_ATTN, st, (coarse_attn_kernel<TKV, TQ, DH, WAVES, U>), grid, dim3(WAVES * 64), 0, st,
                     (const TQ*)q, (const TKV*)kc, (const TKV*)vc, seq_len, (TQ*)out, (float*)ws, H, d_h, S_max,
                     scale * LOG2E, n_splits);
  int32_t rc = check_launch("coarse_attn_kernel");
  if (rc != PHOTON_OK || n_splits == 1) return rc;
  PHOTON_LAUNCH(KC_COARSE_MERGE, st, (coarse_merge_kernel<TQ, DH>), dim3(Bt * H), dim3(DH), 0, st, (const float*)ws, (TQ*)out, n_splits, d_h);
  return check_launch("coarse_merge_kernel");
}

template <typename TKV, typename TQ, int DH>
static int32_t launch_coarse_t(const void* q, const void* kc, const void* vc, const int32_t* seq_len, void* out,
                               int Bt, int H, int d_h, int64_t S_max, float scale, int n_splits, void* ws, hipStream_t st) {
  return launch_coarse_v<TKV, TQ, DH, COARSE_WAVES_PER_WG, COARSE_UNROLL>(q, kc, vc, seq_len, out, Bt, H, d_h, S_max, scale,
                                                                          n_splits, ws, st);
}

template <typename TKV, typename TQ>
static int32_t launch_coarse_dh(int d_h, const void* q, const void* kc, const void* vc, const int32_t* seq_len, void* out,
                                int Bt, int H, int64_t S_max, float scale, int n_splits, void* ws, hipStream_t st) {
  switch (kv_row_elems(d_h)) {
    case 32: return launch_coarse_t<TKV, TQ, 32>(q, kc, vc, seq_len, out, Bt, H, d_h, S_max, scale, n_splits, ws, st);
    case 64: return launch_coarse_t<TKV, TQ, 64>(q, kc, vc, seq_len, out, Bt, H, d_h, S_max, scale, n_splits, ws, st);
    case 128: return launch_coarse_t<TKV, TQ, 128>(q, kc, vc, seq_len, out, Bt, H, d_h, S_max, scale, n_splits, ws, st);
  }
  return fail(PHOTON_ERR_UNSUPPORTED, "coarse attention: d_h=%d not in [1, 128]", d_h);
}

int32_t launch_coarse_attn(KvType kv, bool q_f32, int d_h, const void* q, const void* kc, const void* vc,
                           const int32_t* seq_len, void* out, int Bt, int H, int64_t S_max, float scale,
                           int n_splits, void* ws, hipStream_t st) {
  if (kv == KV_F32) return launch_coarse_dh<float, float>(d_h, q, kc, vc, seq_len, out, Bt, H, S_max, scale, n_splits, ws, st);
  if (kv == KV_FP8) return launch_coarse_dh<fp8_t, float>(d_h, q, kc, vc, seq_len, out, Bt, H, S_max, scale, n_splits, ws, st);
  if (q_f32) return launch_coarse_dh<bf16_t, float>(d_h, q, kc, vc, seq_len, out, Bt, H, S_max, scale, n_splits, ws, st);
  return launch_coarse_dh<bf16_t, bf16_t>(d_h, q, kc, vc, seq_len, out, Bt, H, S_max, scale, n_splits, ws, st);
}

int32_t coarse_auto_splits(int Bt, int H, int64_t S_max) {
  // Short streams (the benchmark shape: 128 streams x 8200 keys): about 768 workgroups (3 per CU), measured 80 %
  // of the HBM peak for any cache pitch (one workgroup per CU is as fast only when the pitch S_max*d_h is a
  // multiple of 16 KB: otherwise the streams start on skewed memory channels and few large splits collide; more
  // splits lengthen the merge).  Long streams (4096 keys or more per split): about 1024 workgroups (4 per CU, all
  // resident at once), measured 87 % against 81 % at 128 streams x 131072 keys.  Every split streams at least 512 keys.
  const int64_t streams = (int64_t)Bt * H;
  int64_t want = (1024 + streams - 1) / streams;
  if (S_max / want < 4096) want = (768 + streams - 1) / streams;
  int64_t cap = S_max / 512;
  if (cap < 1) cap = 1;
  if (want > cap) want = cap;
  if (want > 64) want = 64;
  if (want < 1) want = 1;
  return (int32_t)want;
}

// ------------------------------------------------------------------ chunk-local

constexpr int LOCAL_THREADS = 256;

// One lane group owns one (chunk, head) unit: it holds the unit's NK key and
// value rows in registers and walks over the query rows.  TILE: q_len == NK and
// q_pos == 0, fully unrolled.  DH: lanes * elements per lane of a group (32, 64, 128); d_h <= DH: head size (a
// multiple of the 16-byte lane chunk); lanes past d_h carry zero queries and store nothing.
template <typename T, int DH, int NK, bool TILE>
__global__ __launch_bounds__(LOCAL_THREADS) void local_attn_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, T* __restrict__ out,
    int64_t n_units, int H, int d_h, int W, int q_len_rt, int q_pos_rt, float scale_log2e) {
  using M = RowMap<T, DH>;
  constexpr int VEC = M::VEC, LPR = M::LPR, UPW = M::RPW;
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * (LOCAL_THREADS / 64) + (threadIdx.x >> 6);
  int64_t unit = wave * UPW + lane / LPR;
  const bool live = unit < n_units;
  unit = live ? unit : n_units - 1;
  const int64_t chunk = unit / H;
  const int h = (int)(unit % H);
  const bool col_live = (lane % LPR) * VEC < d_h;
  const int col = col_live ? (lane % LPR) * VEC : 0;               // surplus lanes repeat column 0 (in bounds)
  const int q_len = TILE ? NK : q_len_rt;
  const int q_pos = TILE ? 0 : q_pos_rt;
  const int64_t row = (int64_t)H * d_h;

  const T* kp = k + (chunk * W * H + h) * d_h + col;
  const T* vp = v + (chunk * W * H + h) * d_h + col;
  uint4_t kr[NK], vr[NK];
#pragma unroll
  for (int j = 0; j < NK; ++j) { kr[j] = load16_stream(kp + j * row); vr[j] = load16_stream(vp + j * row); }

  const T* qp = q + (chunk * q_len * H + h) * d_h + col;
  T* op = out + (chunk * q_len * H + h) * d_h + col;
  const float q_mul = col_live ? scale_log2e : 0.f;

  auto one_query = [&](int i, int nvis) {
    float qf[VEC];
    unpack16<T>(load16_stream(qp + i * row), qf);
#pragma unroll
    for (int t = 0; t < VEC; ++t) qf[t] *= q_mul;
    float s[NK];
    float mx = NEG_BIG;
#pragma unroll
    for (int j = 0; j < NK; ++j) {
      if (j < nvis) {
        float kf[VEC];
        unpack16<T>(kr[j], kf);
        float acc = 0.f;
#pragma unroll
        for (int t = 0; t < VEC; ++t) acc = fmaf(qf[t], kf[t], acc);
        s[j] = group_sum<LPR>(acc);
        mx = fmaxf(mx, s[j]);
      }
    }
    float l = 0.f, o[VEC];
#pragma unroll
    for (int t = 0; t < VEC; ++t) o[t] = 0.f;
#pragma unroll
    for (int j = 0; j < NK; ++j) {
      if (j < nvis) {
        const float p = fast_exp2(s[j] - mx);
        l += p;
        float vf[VEC];
        unpack16<T>(vr[j], vf);
#pragma unroll
        for (int t = 0; t < VEC; ++t) o[t] = fmaf(p, vf[t], o[t]);
      }
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int t = 0; t < VEC; ++t) o[t] *= inv;
    if (live && col_live) Vec16<T>::store(op + i * row, o);
  };

  if (TILE) {
#pragma unroll
    for (int i = 0; i < NK; ++i) one_query(i, i + 1);
  } else {
    for (int i = 0; i < q_len; ++i) one_query(i, q_pos + i + 1);
  }
}

// Decode sub-step of a local decoder, fused: for the q_len new rows of every chunk (window positions
// q_pos .. q_pos+q_len-1) take q, k, v from the QKV projection output, apply the rotary encoding at
// the window position, append k and v to the chunk's local cache, and attend causally over the window
// so far.  One lane group per (chunk, head); the window (<= 16 rows) lives in registers.  fp32.
// DH: 4 * lanes of a group.  PAD: the head size d_h is smaller than DH (a multiple of 4): surplus lanes carry
// zeros, and the rotary partner of an element (d_h/2 away, in general not a whole number of lanes) is read from
// memory instead of from a neighbour lane.
template <int DH, int NK, bool PAD>
__global__ __launch_bounds__(LOCAL_THREADS) void local_step_attn_kernel(
    const float* __restrict__ qkv, float* __restrict__ lk, float* __restrict__ lv, float* __restrict__ out,
    int64_t n_units, int H, int d_h_rt, int W, int q_len, int q_pos, float scale_log2e, double freq_ratio, int out_bf16) {
  constexpr int VEC = 4, LPR = DH / 4, UPW = 64 / LPR;
  const int d_h = PAD ? d_h_rt : DH;
  const int half = d_h / 2;
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * (LOCAL_THREADS / 64) + (threadIdx.x >> 6);
  int64_t unit = wave * UPW + lane / LPR;
  const bool unit_live = unit < n_units;
  unit = unit_live ? unit : n_units - 1;
  const int64_t chunk = unit / H;
  const int h = (int)(unit % H);
  const bool col_live = (lane % LPR) * VEC < d_h;
  const int col = col_live ? (lane % LPR) * VEC : 0;         // surplus lanes repeat column 0 (in bounds, never stored)
  const bool live = unit_live && col_live;
  const int D = H * d_h;

  float inv_freq[VEC];
  bool upper[VEC];                                           // this element is the i + d_h/2 member of its rotary pair
  int partner[VEC];
#pragma unroll
  for (int t = 0; t < VEC; ++t) {
    upper[t] = col + t >= half;
    partner[t] = upper[t] ? col + t - half : col + t + half;
    // rotary frequency theta^(-2i/d_h) = freq_ratio^i (freq_ratio = theta^(-2/d_h) from the host, 0 for no rotation):
    // i < 64, six squarings in double instead of a double-precision logarithm and power per element
    double base = freq_ratio, f = freq_ratio == 0.0 ? 0.0 : 1.0;
    int e = (col + t) % half;
#pragma unroll
    for (int b = 0; b < 6; ++b) {
      if (e & 1) f *= base;
      base *= base;
      e >>= 1;
    }
    inv_freq[t] = (float)f;
  }

  float4_t kr[NK], vr[NK];
  float* kcache = lk + (chunk * W * H + h) * d_h + col;
  float* vcache = lv + (chunk * W * H + h) * d_h + col;
#pragma unroll
  for (int j = 0; j < NK; ++j) {
    if (j < q_pos) {
      kr[j] = *reinterpret_cast<const float4_t*>(kcache + (int64_t)j * D);
      vr[j] = *reinterpret_cast<const float4_t*>(vcache + (int64_t)j * D);
    }
  }
  // The new rows' q, k, v (and, for padded heads, the rotary partners) are requested one row ahead: the first one
  // here, before the sine and cosine are formed, so that the arithmetic runs under the loads.
  float4_t q4, k4, v4;
  float qp[VEC], kp[VEC];
  auto fetch_row = [&](int64_t r) {
    const float* head = qkv + (chunk * q_len + r) * 3 * D + h * d_h;
    q4 = *reinterpret_cast<const float4_t*>(head + col);
    k4 = *reinterpret_cast<const float4_t*>(head + col + D);
    v4 = *reinterpret_cast<const float4_t*>(head + col + 2 * D);
    if (PAD) {
#pragma unroll
      for (int t = 0; t < VEC; ++t) { qp[t] = head[partner[t]]; kp[t] = head[D + partner[t]]; }
    }
  };
  fetch_row(0);
  // cosine and sine of the first new row's angle (window positions are small, j < 16: single precision is exact
  // enough); further new rows (a first sub-step with several converter rows) follow by the angle-addition formulas,
  // which keeps the unrolled row loop below free of the library routine.
  float rc[VEC], rs[VEC], dc[VEC], ds[VEC];
#pragma unroll
  for (int t = 0; t < VEC; ++t) {
    sincosf((float)q_pos * inv_freq[t], &rs[t], &rc[t]);
    dc[t] = 1.f; ds[t] = 0.f;
    if (q_len > 1) sincosf(inv_freq[t], &ds[t], &dc[t]);
  }
#pragma unroll
  for (int j = 0; j < NK; ++j) {
    if (j >= q_pos) {
      const int64_t row = chunk * q_len + (j - q_pos);
      // rotary: out[i] = x[i] c - x[i+h] s ; out[i+h] = x[i+h] c + x[i] s
      float qa[VEC] = {q4.x, q4.y, q4.z, q4.w}, ka[VEC] = {k4.x, k4.y, k4.z, k4.w};
      const float4_t v_row = v4;
      float qpr[VEC], kpr[VEC];
#pragma unroll
      for (int t = 0; t < VEC; ++t) { qpr[t] = PAD ? qp[t] : 0.f; kpr[t] = PAD ? kp[t] : 0.f; }
      if (j + 1 < NK) fetch_row(j + 1 - q_pos);              // the row after this one (exists: NK = q_pos + q_len)
#pragma unroll
      for (int t = 0; t < VEC; ++t) {
        float qb, kb;
        if (PAD) {
          qb = qpr[t];
          kb = kpr[t];
        } else {                                             // the partner sits LPR/2 lanes away
          qb = __shfl_xor(qa[t], LPR / 2);
          kb = __shfl_xor(ka[t], LPR / 2);
        }
        const float c = rc[t], sn = upper[t] ? rs[t] : -rs[t];
        qa[t] = col_live ? qa[t] * c + qb * sn : 0.f;
        ka[t] = ka[t] * c + kb * sn;
        const float c1 = rc[t] * dc[t] - rs[t] * ds[t];        // the next row's angle
        rs[t] = rs[t] * dc[t] + rc[t] * ds[t];
        rc[t] = c1;
      }
      kr[j] = float4_t{ka[0], ka[1], ka[2], ka[3]};
      vr[j] = v_row;
      if (live) {
        *reinterpret_cast<float4_t*>(kcache + (int64_t)j * D) = kr[j];
        *reinterpret_cast<float4_t*>(vcache + (int64_t)j * D) = v_row;
      }
      // attention of this row over window rows 0..j
      float s[NK], mx = NEG_BIG;
#pragma unroll
      for (int jj = 0; jj <= j; ++jj) {
        float acc = qa[0] * kr[jj].x;
        acc = fmaf(qa[1], kr[jj].y, acc);
        acc = fmaf(qa[2], kr[jj].z, acc);
        acc = fmaf(qa[3], kr[jj].w, acc);
        s[jj] = group_sum<LPR>(acc) * scale_log2e;
        mx = fmaxf(mx, s[jj]);
      }
      float l = 0.f;
      float4_t o = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int jj = 0; jj <= j; ++jj) {
        const float pw = fast_exp2(s[jj] - mx);
        l += pw;
        o += pw * vr[jj];
      }
      o *= (1.f / l);
      if (live) {
        if (out_bf16) *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(out) + row * D + h * d_h + col) = uint2{pack_bf16x2(o.x, o.y), pack_bf16x2(o.z, o.w)};
        else *reinterpret_cast<float4_t*>(out + row * D + h * d_h + col) = o;
      }
    }
  }
}

template <int DH, bool PAD>
static int32_t launch_local_step_dh(const float* qkv, float* lk, float* lv, float* out, int64_t n_chunks, int W, int q_len,
                                    int q_pos, int H, int d_h, float scale, float theta, bool out_bf16, hipStream_t st) {
  const double freq_ratio = theta == 0.f ? 0.0 : pow((double)theta, -2.0 / (double)d_h);
  const int64_t n_units = n_chunks * H;
  const int64_t units_per_block = (int64_t)(64 / (DH / 4)) * (LOCAL_THREADS / 64);
  const int64_t blocks = (n_units + units_per_block - 1) / units_per_block;
  if (blocks > 0x7fffffffLL) return fail(PHOTON_ERR_UNSUPPORTED, "chunk-local attention: too many chunks for one launch");
#define PHOTON_LS_CASE(N)                                                                                                   \
  case N:                                                                                                                   \
    PHOTON_LAUNCH(KC_LOCAL_ATTN, st, (local_step_attn_kernel<DH, N, PAD>), dim3((unsigned)blocks), dim3(LOCAL_THREADS), 0, st, qkv, \
                  lk, lv, out, n_units, H, d_h, W, q_len, q_pos, scale * LOG2E, freq_ratio, out_bf16 ? 1 : 0);                                    \
    break;
  switch (q_pos + q_len) {
    PHOTON_LS_CASE(1) PHOTON_LS_CASE(2) PHOTON_LS_CASE(3) PHOTON_LS_CASE(4)
    PHOTON_LS_CASE(5) PHOTON_LS_CASE(6) PHOTON_LS_CASE(7) PHOTON_LS_CASE(8)
    PHOTON_LS_CASE(9) PHOTON_LS_CASE(10) PHOTON_LS_CASE(11) PHOTON_LS_CASE(12)
    PHOTON_LS_CASE(13) PHOTON_LS_CASE(14) PHOTON_LS_CASE(15) PHOTON_LS_CASE(16)
    default: return fail(PHOTON_ERR_UNSUPPORTED, "chunk-local attention: window position %d out of range", q_pos + q_len);
  }
#undef PHOTON_LS_CASE
  return check_launch("local_step_attn_kernel");
}

int32_t launch_local_step_attn(int d_h, const float* qkv, float* lk, float* lv, float* out, int64_t n_chunks, int W, int q_len,
                               int q_pos, int H, float scale, float theta, bool out_bf16, hipStream_t st) {
  if (d_h % 4 != 0) return fail(PHOTON_ERR_UNSUPPORTED, "chunk-local attention: d_h=%d is not a multiple of 4", d_h);
  switch (d_h) {
    case 32: return launch_local_step_dh<32, false>(qkv, lk, lv, out, n_chunks, W, q_len, q_pos, H, d_h, scale, theta, out_bf16, st);
    case 64: return launch_local_step_dh<64, false>(qkv, lk, lv, out, n_chunks, W, q_len, q_pos, H, d_h, scale, theta, out_bf16, st);
    case 128: return launch_local_step_dh<128, false>(qkv, lk, lv, out, n_chunks, W, q_len, q_pos, H, d_h, scale, theta, out_bf16, st);
  }
  switch (kv_row_elems(d_h)) {
    case 32: return launch_local_step_dh<32, true>(qkv, lk, lv, out, n_chunks, W, q_len, q_pos, H, d_h, scale, theta, out_bf16, st);
    case 64: return launch_local_step_dh<64, true>(qkv, lk, lv, out, n_chunks, W, q_len, q_pos, H, d_h, scale, theta, out_bf16, st);
    case 128: return launch_local_step_dh<128, true>(qkv, lk, lv, out, n_chunks, W, q_len, q_pos, H, d_h, scale, theta, out_bf16, st);
  }
  return fail(PHOTON_ERR_UNSUPPORTED, "chunk-local attention: d_h=%d not in [4, 128]", d_h);
}

template <typename T, int DH, int NK>
static int32_t launch_local_nk(bool tile, const void* q, const void* k, const void* v, void* out, int64_t n_chunks,
                               int W, int q_len, int q_pos, int H, int d_h, float scale, hipStream_t st) {
  using M = RowMap<T, DH>;
  const int64_t n_units = n_chunks * H;
  const int64_t units_per_block = (int64_t)M::RPW * (LOCAL_THREADS / 64);
  const int64_t blocks = (n_units + units_per_block - 1) / units_per_block;
  if (blocks > 0x7fffffffLL) return fail(PHOTON_ERR_UNSUPPORTED, "chunk-local attention: too many chunks for one launch");
  if (tile)
    PHOTON_LAUNCH(KC_LOCAL_ATTN, st, (local_attn_kernel<T, DH, NK, true>), dim3((unsigned)blocks), dim3(LOCAL_THREADS), 0, st,
                       (const T*)q, (const T*)k, (const T*)v, (T*)out, n_units, H, d_h, W, q_len, q_pos, scale * LOG2E);
  else
    PHOTON_LAUNCH(KC_LOCAL_ATTN, st, (local_attn_kernel<T, DH, NK, false>), dim3((unsigned)blocks), dim3(LOCAL_THREADS), 0, st,
                       (const T*)q, (const T*)k, (const T*)v, (T*)out, n_units, H, d_h, W, q_len, q_pos, scale * LOG2E);
  return check_launch("local_attn_kernel");
}

template <typename T, int DH>
static int32_t launch_local_dh(const void* q, const void* k, const void* v, void* out, int64_t n_chunks,
                               int W, int q_len, int q_pos, int H, int d_h, float scale, hipStream_t st) {
  const int nk = q_pos + q_len;
  const bool tile = (q_pos == 0);
#define PHOTON_NK_CASE(N) \
  case N: return launch_local_nk<T, DH, N>(tile, q, k, v, out, n_chunks, W, q_len, q_pos, H, d_h, scale, st);
  switch (nk) {
    PHOTON_NK_CASE(1) PHOTON_NK_CASE(2) PHOTON_NK_CASE(3) PHOTON_NK_CASE(4)
    PHOTON_NK_CASE(5) PHOTON_NK_CASE(6) PHOTON_NK_CASE(7) PHOTON_NK_CASE(8)
    PHOTON_NK_CASE(9) PHOTON_NK_CASE(10) PHOTON_NK_CASE(11) PHOTON_NK_CASE(12)
    PHOTON_NK_CASE(13) PHOTON_NK_CASE(14) PHOTON_NK_CASE(15) PHOTON_NK_CASE(16)
  }
#undef PHOTON_NK_CASE
  return fail(PHOTON_ERR_UNSUPPORTED, "chunk-local attention: window position %d out of range", nk);
}

int32_t launch_local_attn(bool f32, int d_h, const void* q, const void* k, const void* v, void* out,
                          int64_t n_chunks, int W, int q_len, int q_pos, int H, float scale, hipStream_t st) {
  const int vec = f32 ? 4 : 8;                                // elements of a lane's 16-byte chunk
  if (d_h < vec || d_h > 128 || d_h % vec != 0)
    return fail(PHOTON_ERR_UNSUPPORTED, "chunk-local attention: d_h=%d must be a multiple of %d in [%d, 128]", d_h, vec, vec);
  const int lanes = kv_row_elems(d_h);
  if (f32) {
    switch (lanes) {
      case 32: return launch_local_dh<float, 32>(q, k, v, out, n_chunks, W, q_len, q_pos, H, d_h, scale, st);
      case 64: return launch_local_dh<float, 64>(q, k, v, out, n_chunks, W, q_len, q_pos, H, d_h, scale, st);
      default: return launch_local_dh<float, 128>(q, k, v, out, n_chunks, W, q_len, q_pos, H, d_h, scale, st);
    }
  }
  switch (lanes) {
    case 32: return launch_local_dh<bf16_t, 32>(q, k, v, out, n_chunks, W, q_len, q_pos, H, d_h, scale, st);
    case 64: return launch_local_dh<bf16_t, 64>(q, k, v, out, n_chunks, W, q_len, q_pos, H, d_h, scale, st);
    default: return launch_local_dh<bf16_t, 128>(q, k, v, out, n_chunks, W, q_len, q_pos, H, d_h, scale, st);
  }
}

}  // namespace photon

// ------------------------------------------------------------------ C ABI

using namespace photon;

extern "C" int32_t photon_kv_row_elems(int32_t d_h) { return kv_row_elems(d_h); }

extern "C" size_t photon_coarse_decode_attn_workspace_bytes(int32_t Bt, int32_t H, int32_t d_h, int32_t n_splits) {
  if (Bt <= 0 || H <= 0 || d_h <= 0 || d_h > 128 || n_splits <= 1) return 0;
  return (size_t)Bt * H * n_splits * (kv_row_elems(d_h) + 2) * sizeof(float);
}

extern "C" int32_t photon_coarse_decode_attn_auto_splits(int32_t Bt, int32_t H, int64_t S_max) {
  if (Bt <= 0 || H <= 0 || S_max <= 0) return 1;
  return coarse_auto_splits(Bt, H, S_max);
}

extern "C" int32_t photon_coarse_decode_attn(const void* q, const void* k_cache, const void* v_cache,
                                             const int32_t* seq_len, void* out, int32_t Bt, int32_t H, int32_t d_h,
                                             int64_t S_max, float scale, int32_t n_splits, void* workspace,
                                             size_t workspace_bytes, photon_dtype dt, void* stream) {
  clear_error();
  PHOTON_REQUIRE(valid_dtype(dt) || dt == PHOTON_FP8_E4M3, PHOTON_ERR_UNSUPPORTED, "%s: unknown dtype %d", __func__, (int)dt);
  PHOTON_REQUIRE(Bt > 0 && H > 0 && S_max > 0, PHOTON_ERR_INVALID_ARG, "%s: Bt=%d H=%d S_max=%lld must be positive",
                 __func__, Bt, H, (long long)S_max);
  PHOTON_REQUIRE((int64_t)Bt * H <= 65535, PHOTON_ERR_UNSUPPORTED, "%s: Bt*H=%lld exceeds 65535 streams per launch",
                 __func__, (long long)Bt * H);
  PHOTON_REQUIRE(d_h >= 1 && d_h <= 128, PHOTON_ERR_UNSUPPORTED, "%s: d_h=%d not in [1, 128]", __func__, d_h);
  PHOTON_REQUIRE(n_splits >= 0 && n_splits <= 1024, PHOTON_ERR_INVALID_ARG, "%s: n_splits=%d out of [0, 1024]", __func__, n_splits);
  PHOTON_REQUIRE_PTR(q);
  PHOTON_REQUIRE_PTR(k_cache);
  PHOTON_REQUIRE_PTR(v_cache);
  PHOTON_REQUIRE_PTR(out);
  PHOTON_REQUIRE(seq_len != nullptr, PHOTON_ERR_INVALID_ARG, "%s: seq_len is null", __func__);
  if (n_splits == 0) n_splits = coarse_auto_splits(Bt, H, S_max);
  if (n_splits > 1) {
    const size_t need = photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, n_splits);
    PHOTON_REQUIRE(workspace != nullptr && aligned16(workspace) && workspace_bytes >= need, PHOTON_ERR_WORKSPACE,
                   "%s: n_splits=%d needs a 16-byte aligned workspace of %zu bytes (got %zu)", __func__, n_splits, need,
                   workspace_bytes);
  }
  return launch_coarse_attn(dt == PHOTON_F32 ? KV_F32 : dt == PHOTON_BF16 ? KV_BF16 : KV_FP8, dt != PHOTON_BF16, d_h, q, k_cache, v_cache, seq_len, out,
                            Bt, H, S_max, scale, n_splits, workspace, (hipStream_t)stream);
}

// ------------------------------------------------------------------ entry point that allocates nothing
// The split partials of the coarse attention live in a file-scope device array instead of a caller workspace.
// Every GPU holds its own copy of the array at its own address: the address is looked up once per device, with
// that device current, and only that pointer (never the array's name, which on the host is a stand-in and no
// device address) goes to kernels.
namespace photon {
constexpr size_t COARSE_STATIC_BYTES = (size_t)4 << 20;
constexpr int COARSE_STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[COARSE_STATIC_BYTES];
static void* g_scratch_ptr[COARSE_STATIC_MAX_DEVICES] = {nullptr};
static std::mutex g_scratch_mu;

// Device address of this GPU's copy of `scratch` (nullptr + error text on failure).
static void* static_scratch_for_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= COARSE_STATIC_MAX_DEVICES) {
    (void)hipGetLastError();
    fail(PHOTON_ERR_HIP, "static scratch: cannot identify the current device (%d)", dev);
    return nullptr;
  }
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      fail(PHOTON_ERR_HIP, "static scratch: hipGetSymbolAddress failed on device %d: %s", dev, hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}
}  // namespace photon

extern "C" size_t photon_coarse_decode_attn_static_capacity(void) { return photon::COARSE_STATIC_BYTES; }

extern "C" int32_t photon_coarse_decode_attn_static(const void* q, const void* k_cache, const void* v_cache,
                                                    const int32_t* seq_len, void* out, int32_t Bt, int32_t H, int32_t d_h,
                                                    int64_t S_max, float scale, int32_t n_splits, photon_dtype dt, void* stream) {
  clear_error();
  PHOTON_REQUIRE(Bt > 0 && H > 0 && S_max > 0, PHOTON_ERR_INVALID_ARG, "%s: Bt=%d H=%d S_max=%lld must be positive", __func__, Bt, H,
                 (long long)S_max);
  PHOTON_REQUIRE(d_h >= 1 && d_h <= 128, PHOTON_ERR_UNSUPPORTED, "%s: d_h=%d not in [1, 128]", __func__, d_h);
  PHOTON_REQUIRE(n_splits >= 0 && n_splits <= 1024, PHOTON_ERR_INVALID_ARG, "%s: n_splits=%d out of [0, 1024]", __func__, n_splits);
  if (n_splits == 0) n_splits = coarse_auto_splits(Bt, H, S_max);
  const size_t need = photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, n_splits);
  PHOTON_REQUIRE(need <= COARSE_STATIC_BYTES, PHOTON_ERR_WORKSPACE,
                 "%s: Bt=%d H=%d d_h=%d n_splits=%d needs %zu bytes of split partials, the built-in scratch holds %zu; "
                 "use photon_coarse_decode_attn with a workspace", __func__, Bt, H, d_h, n_splits, need, COARSE_STATIC_BYTES);
  void* ws = nullptr;
  if (n_splits > 1) {
    ws = static_scratch_for_current_device();
    if (ws == nullptr) return PHOTON_ERR_HIP;
  }
  // every partial the merge reads is written by this call's attention kernel first: nothing has to start at zero
  return photon_coarse_decode_attn(q, k_cache, v_cache, seq_len, out, Bt, H, d_h, S_max, scale, n_splits, ws, need, dt, stream);
}

extern "C" int32_t photon_chunk_local_attn(const void* q, const void* k, const void* v, void* out, int64_t n_chunks,
                                           int32_t W, int32_t q_len, int32_t q_pos, int32_t H, int32_t d_h, float scale,
                                           photon_dtype dt, void* stream) {
  clear_error();
  PHOTON_REQUIRE(valid_dtype(dt), PHOTON_ERR_UNSUPPORTED, "%s: unknown dtype %d", __func__, (int)dt);
  PHOTON_REQUIRE(n_chunks >= 0 && H > 0, PHOTON_ERR_INVALID_ARG, "%s: n_chunks=%lld H=%d invalid", __func__,
                 (long long)n_chunks, H);
  PHOTON_REQUIRE(W >= 1 && W <= PHOTON_MAX_WINDOW, PHOTON_ERR_UNSUPPORTED, "%s: W=%d not in [1, %d]", __func__, W,
                 (int)PHOTON_MAX_WINDOW);
  PHOTON_REQUIRE(q_len >= 1 && q_pos >= 0 && q_pos + q_len <= W, PHOTON_ERR_INVALID_ARG,
                 "%s: queries [%d, %d) do not fit the window W=%d", __func__, q_pos, q_pos + q_len, W);
  {
    const int vec = dt == PHOTON_F32 ? 4 : 8;
    PHOTON_REQUIRE(d_h >= vec && d_h <= 128 && d_h % vec == 0, PHOTON_ERR_UNSUPPORTED,
                   "%s: d_h=%d must be a multiple of %d in [%d, 128]", __func__, d_h, vec, vec);
  }
  if (n_chunks == 0) return PHOTON_OK;
  PHOTON_REQUIRE_PTR(q);
  PHOTON_REQUIRE_PTR(k);
  PHOTON_REQUIRE_PTR(v);
  PHOTON_REQUIRE_PTR(out);
  return launch_local_attn(dt == PHOTON_F32, d_h, q, k, v, out, n_chunks, W, q_len, q_pos, H, scale, (hipStream_t)stream);
}
