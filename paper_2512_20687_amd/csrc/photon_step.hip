// photon_decode_step: one recursive-generation step (paper Section 2.3.3,
// Appendix A Definition 2) composed from the attention and linear kernels plus
// the small element-wise kernels below.  Everything is enqueued on one stream;
// sequence lengths and tokens stay in device memory, so the enqueue pattern does
// not depend on data and the whole step can be captured in a HIP graph.
#include "photon_attn.h"
#include "photon_encoder_attn.h"
#include "photon_device.h"
#include "photon_host.h"
#include "photon_linear.h"
#include "photon_persistent.h"

namespace photon {

// ------------------------------------------------------------------ small kernels

// out[i*out_mul + out_off] = rmsnorm(in[i*in_mul + in_off]) * g ; rows of D floats, D a multiple of 4.
__global__ __launch_bounds__(256) void norm_rows_kernel(const float* __restrict__ in, int in_mul, int in_off,
                                                        const float* __restrict__ g, float eps, float* __restrict__ out,
                                                        int out_mul, int out_off, int D) {
  extern __shared__ float4_t xrow[];
  const int i = blockIdx.x, tid = threadIdx.x;
  const float* x = in + ((int64_t)i * in_mul + in_off) * D;
  float ss = 0.f;
  for (int d = tid * 4; d < D; d += 1024) {
    const float4_t v = *reinterpret_cast<const float4_t*>(x + d);
    xrow[d >> 2] = v;
    ss = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, ss))));
  }
  ss = group_sum<32>(ss);
  ss += __shfl_xor(ss, 32);
  __shared__ float partsum[4];
  if ((tid & 63) == 0) partsum[tid >> 6] = ss;
  __syncthreads();
  const float tot = (partsum[0] + partsum[1]) + (partsum[2] + partsum[3]);
  const float r = 1.0f / sqrtf(tot / (float)D + eps);
  float* o = out + ((int64_t)i * out_mul + out_off) * D;
  for (int d = tid * 4; d < D; d += 1024) {
    const float4_t gv = *reinterpret_cast<const float4_t*>(g + d);
    *reinterpret_cast<float4_t*>(o + d) = xrow[d >> 2] * r * gv;
  }
}

// rows[i, :] = table[tokens[i], :] as fp32 (encoder-side embedding of the prompt).
template <typename TE>
__global__ __launch_bounds__(256) void embed_rows_kernel(const int32_t* __restrict__ tokens, const TE* __restrict__ table,
                                                         float* __restrict__ rows, int64_t n, int D, int vocab) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;       // one thread per 4 elements
  const int per_row = D / 4;
  if (idx >= n * per_row) return;
  const int64_t i = idx / per_row;
  const int d = (int)(idx % per_row) * 4;
  int t = tokens[i];
  t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);                      // out-of-range ids are clamped, never read out of bounds
  const TE* src = table + (int64_t)t * D + d;
  float4_t v;
  v.x = to_f32<TE>(src[0]); v.y = to_f32<TE>(src[1]); v.z = to_f32<TE>(src[2]); v.w = to_f32<TE>(src[3]);
  *reinterpret_cast<float4_t*>(rows + i * D + d) = v;
}

__global__ __launch_bounds__(256) void copy_f32x4_kernel(const float4_t* __restrict__ src, float4_t* __restrict__ dst, int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n4) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void fill_i32_kernel(int32_t* __restrict__ dst, int32_t value, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = value;
}

__global__ __launch_bounds__(256) void broadcast_rows_kernel(const float* __restrict__ src, float* __restrict__ dst, int rows, int D) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx < (int64_t)rows * D) dst[idx] = src[idx % D];
}

// Top-level STEP: position of sequence b is seq_len[b]-1 (the count already includes the new entry);
// k, v go to cache[b, h, pos, :] of this layer, whose rows hold `pitch` >= d_h elements (the surplus is zeroed).
template <typename TKV>
__global__ __launch_bounds__(256) void rope_append_coarse_kernel(const float* __restrict__ qkv, float* __restrict__ qrot,
                                                                 TKV* __restrict__ kc, TKV* __restrict__ vc,
                                                                 const int32_t* __restrict__ seq_len, int Bt, int H,
                                                                 int d_h, int pitch, int64_t S_max, float theta) {
  const int half = d_h >> 1, D = H * d_h;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)Bt * H * half) return;
  const int i = (int)(idx % half);
  const int h = (int)((idx / half) % H);
  const int b = (int)(idx / ((int64_t)half * H));
  const int pos = seq_len[b] - 1;
  float c, s;
  rope_angle(pos, i, d_h, theta, c, s);
  const float* src = qkv + (int64_t)b * 3 * D + h * d_h;
  const float qa = src[i], qb = src[i + half];
  const float ka = src[D + i], kb = src[D + i + half];
  float* qd = qrot + (int64_t)b * D + h * d_h;
  qd[i] = qa * c - qb * s;
  qd[i + half] = qb * c + qa * s;
  if (pos < 0 || pos >= S_max) return;                        // full cache: nothing is written out of bounds
  const int64_t slot = (((int64_t)b * H + h) * S_max + pos) * pitch;
  kc[slot + i] = from_f32<TKV>(ka * c - kb * s);
  kc[slot + i + half] = from_f32<TKV>(kb * c + ka * s);
  vc[slot + i] = from_f32<TKV>(src[2 * D + i]);
  vc[slot + i + half] = from_f32<TKV>(src[2 * D + i + half]);
  for (int p = d_h + i; p < pitch; p += half) { kc[slot + p] = TKV{}; vc[slot + p] = TKV{}; }
}

// Token choice for one row of logits (greedy, lowest index on ties, or the forced token), then the
// decoder-side embedding of that token as the next input row.
constexpr int CHOOSE_THREADS = 1024;
template <typename TE>
__global__ __launch_bounds__(CHOOSE_THREADS) void choose_token_kernel(const float* __restrict__ logits, int64_t ld_logits, int vocab,
                                                           const int32_t* __restrict__ forced, int32_t* __restrict__ tokens,
                                                           int tok_mul, int tok_off, const TE* __restrict__ E,
                                                           float* __restrict__ x_next, int D) {
  const int row = blockIdx.x, tid = threadIdx.x;
  const float* lg = logits + (int64_t)row * ld_logits;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int t0 = tid; t0 < vocab; t0 += 4 * CHOOSE_THREADS) {       // indices visited in increasing order: first maximum wins
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int t = t0 + u * CHOOSE_THREADS;
      v[u] = t < vocab ? lg[t] : -INFINITY;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (v[u] > best || (bi == 0x7fffffff && t0 + u * CHOOSE_THREADS < vocab)) { best = v[u]; bi = t0 + u * CHOOSE_THREADS; }
  }
#pragma unroll
  for (int mask = 1; mask < 64; mask <<= 1) {
    const float ov = __shfl_xor(best, mask);
    const int oi = __shfl_xor(bi, mask);
    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
  }
  __shared__ float sv[CHOOSE_THREADS / 64];
  __shared__ int si[CHOOSE_THREADS / 64];
  __shared__ int chosen;
  if ((tid & 63) == 0) { sv[tid >> 6] = best; si[tid >> 6] = bi; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < CHOOSE_THREADS / 64; ++w)
      if (sv[w] > best || (sv[w] == best && si[w] < bi)) { best = sv[w]; bi = si[w]; }
    const int64_t flat = (int64_t)row * tok_mul + tok_off;
    if (forced != nullptr) bi = forced[flat];
    bi = bi < 0 ? 0 : (bi >= vocab ? vocab - 1 : bi);
    tokens[flat] = bi;
    chosen = bi;
  }
  __syncthreads();
  if (x_next != nullptr) {
    const TE* e = E + (int64_t)chosen * D;
    for (int d = tid; d < D; d += CHOOSE_THREADS) x_next[(int64_t)row * D + d] = to_f32<TE>(e[d]);
  }
}

// Conditioning of the next lower level: sequence b's chunks hang off [carry[b], new[b,0], ..., new[b,n-2]];
// new[b,n-1] becomes the carry.  One launch: a thread reads the carry element it is about to replace.
__global__ __launch_bounds__(256) void shift_condition_kernel(const float* __restrict__ fresh, float* __restrict__ carry,
                                                              float* __restrict__ cond, int Bt, int n, int D) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)Bt * n * D) return;
  const int d = (int)(idx % D);
  const int i = (int)((idx / D) % n);
  const int b = (int)(idx / ((int64_t)D * n));
  if (i == 0) {                                           // the only reader and the only writer of carry[b, d]
    cond[idx] = carry[(int64_t)b * D + d];
    carry[(int64_t)b * D + d] = fresh[((int64_t)b * n + n - 1) * D + d];
  } else {
    cond[idx] = fresh[((int64_t)b * n + i - 1) * D + d];
  }
}

// Start of a step: count the entry this step will append to every sequence's coarse cache, and clear the barrier
// counters (and the error word behind them) of the step's persistent launches.
// A sequence whose cache is full (seq_len == S_cap on entry) keeps its count: its new entry then overwrites the last
// one, in bounds, and the caller's status word gets bit 0 (its results of this step are not valid).
__global__ __launch_bounds__(256) void step_begin_kernel(int32_t* __restrict__ seq_len, int Bt, int64_t S_cap, int32_t* __restrict__ status,
                                                         unsigned* __restrict__ bar, int bar_words) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (seq_len != nullptr && idx < Bt) {
    const int32_t n = seq_len[idx];
    if (n < S_cap) seq_len[idx] = n + 1;
    else if (status != nullptr) atomicOr(status, PHOTON_STATUS_CACHE_FULL);
  }
  for (int i = idx; i < bar_words; i += gridDim.x * 256) bar[i] = 0u;
}

// End of a step: a barrier wait of a persistent launch that ran out is reported in the caller's status word.
__global__ void step_end_kernel(const unsigned* __restrict__ err, int32_t* __restrict__ status) {
  if (threadIdx.x == 0 && blockIdx.x == 0 && err[0] != 0u) atomicOr(status, PHOTON_STATUS_BARRIER_TIMEOUT);
}

// Test and measurement switch: run every module pass as separate launches (photon_set_option).
bool g_no_persistent = false;

static inline unsigned blocks_for(int64_t n) { return (unsigned)((n + 255) / 256); }

// ------------------------------------------------------------------ workspace plan

// From this many rows on a linear map goes to the tiled MFMA contraction instead of the few-row kernels
// (which would re-read the weights once per 16 rows).
constexpr int LINEAR_MANY_ROWS = 128;
// Between the two, from this many rows on (more than one row tile of 16), the rows are normalised and rounded to
// bf16 by the row kernel and the few-row kernel takes several row tiles per workgroup: the weights are then streamed
// once per 32 or 64 rows instead of once per 16 (measured at 24 rows: QKV 17.2 -> 4.5 + 9.4 us, gate/up 23.7 -> 4.5 + 13.1).
constexpr int LINEAR_MID_ROWS = 17;

struct Plan {
  int L = 0;
  int64_t chunks[PHOTON_MAX_LEVELS + 1] = {0};   // chunks[l], l = 1..L: chunks decoded per step at level l
  int64_t rows_max = 0;
  int n_splits = 1;
  size_t coarse_ws = 0, coarse_ws_bytes = 0;
  size_t h = 0, attn = 0, qkv = 0, qrot = 0, act = 0, cond = 0, logits = 0, a_hat = 0;
  size_t h2 = 0, attn2 = 0, qkv2 = 0, qrot2 = 0, act2 = 0;   // second set for the main line of a hierarchy (top-level decoder, then STEP)
  int64_t rows2 = 0;                             // its rows: Bt chunks x R_L converter rows
  size_t cond_top = 0;                           // conditioning latents of the level-(L-1) chunks (written on the main line)
  size_t many = 0, many2 = 0;                    // scratch of the many-row linear path (0 rows: absent), main and STEP branch
  size_t hx[PHOTON_MAX_LEVELS] = {0}, hA = 0;    // hierarchical generation: encoder-side new units of level l, chunker outputs
  int many_K = 0;                                // widest contraction it is sized for
  size_t bar = 0;                                // barrier slots of the persistent launches of one step, then the error word
  int bar_slots = 0;
  size_t fresh[PHOTON_MAX_LEVELS] = {0};         // fresh[l]: new level-l units, l = 0..L-1
  size_t lk[PHOTON_MAX_LEVELS] = {0}, lv[PHOTON_MAX_LEVELS] = {0};   // local caches of level l (index l-1), all layers
  size_t total = 0;
};

static size_t bump(size_t& cur, size_t bytes) {
  const size_t at = cur;
  cur += (bytes + 255) / 256 * 256;
  return at;
}

static Plan make_plan(const photon_config& c, int Bt, int64_t S_max) {
  Plan p;
  p.L = c.L;
  p.chunks[c.L] = Bt;
  for (int l = c.L - 1; l >= 1; --l) p.chunks[l] = p.chunks[l + 1] * c.C[l];
  for (int l = 1; l <= c.L; ++l) {
    const int64_t r = p.chunks[l] * c.R[l - 1];
    if (r > p.rows_max) p.rows_max = r;
  }
  const int64_t D = c.D, F = c.d_ff;
  p.n_splits = coarse_auto_splits(Bt, c.H, S_max);
  size_t cur = 0;
  p.coarse_ws_bytes = photon_coarse_decode_attn_workspace_bytes(Bt, c.H, c.d_h, p.n_splits);
  p.coarse_ws = bump(cur, p.coarse_ws_bytes);
  const size_t f = sizeof(float);
  p.h = bump(cur, p.rows_max * D * f);
  p.attn = bump(cur, p.rows_max * D * f);
  p.qkv = bump(cur, p.rows_max * 3 * D * f);
  p.qrot = bump(cur, p.rows_max * D * f);
  p.act = bump(cur, p.rows_max * F * f);
  p.cond = bump(cur, p.rows_max * D * f);
  p.logits = bump(cur, (size_t)p.chunks[1] * c.vocab * f);
  p.a_hat = bump(cur, (size_t)Bt * D * f);
  p.hA = bump(cur, (size_t)p.chunks[1] * D * f);
  p.rows2 = (int64_t)Bt * c.R[c.L - 1];
  p.h2 = bump(cur, (size_t)p.rows2 * D * f);
  p.attn2 = bump(cur, (size_t)p.rows2 * D * f);
  p.qkv2 = bump(cur, (size_t)p.rows2 * 3 * D * f);
  p.qrot2 = bump(cur, (size_t)p.rows2 * D * f);
  p.act2 = bump(cur, (size_t)p.rows2 * F * f);
  p.cond_top = bump(cur, (size_t)(c.L >= 2 ? p.chunks[c.L - 1] : 1) * D * f);
  if (c.dt == PHOTON_BF16) {
    p.many_K = (int)(D > F ? D : F);
    if ((int64_t)c.C[c.L - 1] * D > p.many_K) p.many_K = (int)(c.C[c.L - 1] * D);   // the top chunker contracts over C_L * D
    if (p.rows_max >= LINEAR_MID_ROWS) p.many = bump(cur, linear_many_workspace_bytes(p.rows_max, p.many_K, (int)(2 * F)));
    if (p.rows2 >= LINEAR_MID_ROWS) p.many2 = bump(cur, linear_many_workspace_bytes(p.rows2, p.many_K, (int)(2 * F)));
  }
  for (int l = 1; l <= c.L; ++l) {
    p.fresh[l - 1] = bump(cur, (size_t)p.chunks[l] * c.C[l - 1] * D * f);
    p.hx[l - 1] = bump(cur, (size_t)p.chunks[l] * c.C[l - 1] * D * f);
    const int W = c.R[l - 1] + c.C[l - 1] - 1;
    const size_t cache = (size_t)c.n_layers * p.chunks[l] * W * D * f;
    p.lk[l - 1] = bump(cur, cache);
    p.lv[l - 1] = bump(cur, cache);
  }
  for (int l = 1; l <= c.L; ++l) p.bar_slots += c.C[l - 1];       // one launch per decode sub-step
  p.bar = bump(cur, ((size_t)p.bar_slots * PM_BAR_WORDS + 64) * sizeof(unsigned));
  p.total = cur;
  return p;
}

static int32_t validate_config(const photon_config* c, int Bt, int64_t S_max) {
  PHOTON_REQUIRE(c != nullptr, PHOTON_ERR_INVALID_ARG, "config is null");
  PHOTON_REQUIRE(valid_dtype(c->dt), PHOTON_ERR_UNSUPPORTED, "unknown dtype %d", (int)c->dt);
  PHOTON_REQUIRE(c->kv_dt == c->dt || (c->dt == PHOTON_BF16 && c->kv_dt == PHOTON_FP8_E4M3), PHOTON_ERR_UNSUPPORTED,
                 "kv_dt=%d must equal dt=%d, or be 8-bit with bf16 matrices", (int)c->kv_dt, (int)c->dt);
  PHOTON_REQUIRE(c->L >= 1 && c->L <= PHOTON_MAX_LEVELS, PHOTON_ERR_INVALID_ARG, "L=%d not in [1, %d]", c->L, (int)PHOTON_MAX_LEVELS);
  PHOTON_REQUIRE(Bt > 0 && S_max > 0, PHOTON_ERR_INVALID_ARG, "Bt=%d and S_max=%lld must be positive", Bt, (long long)S_max);
  PHOTON_REQUIRE(c->D > 0 && c->H > 0 && c->d_h > 0 && c->H * c->d_h == c->D, PHOTON_ERR_INVALID_ARG,
                 "D=%d must equal H*d_h=%d*%d", c->D, c->H, c->d_h);
  PHOTON_REQUIRE(c->d_h % 4 == 0 && c->d_h >= 4 && c->d_h <= 128, PHOTON_ERR_UNSUPPORTED, "d_h=%d must be a multiple of 4 in [4, 128]",
                 c->d_h);
  PHOTON_REQUIRE(c->n_layers >= 1 && c->vocab >= 1 && c->d_ff >= 0, PHOTON_ERR_INVALID_ARG, "n_layers=%d vocab=%d d_ff=%d invalid",
                 c->n_layers, c->vocab, c->d_ff);
  int64_t chunks = Bt;
  for (int l = c->L; l >= 1; --l) {
    const int C = c->C[l - 1], R = c->R[l - 1];
    PHOTON_REQUIRE(C >= 1 && R >= 1 && R + C - 1 <= PHOTON_MAX_WINDOW, PHOTON_ERR_UNSUPPORTED,
                   "level %d: C=%d R=%d need C, R >= 1 and R+C-1 <= %d", l, C, R, (int)PHOTON_MAX_WINDOW);
    chunks *= C;
    PHOTON_REQUIRE(chunks * R <= (1 << 20), PHOTON_ERR_UNSUPPORTED, "level %d: %lld rows per sub-step is too many", l, (long long)chunks * R);
  }
  if (c->dt == PHOTON_BF16) {
    PHOTON_REQUIRE(c->D % 64 == 0 && c->d_ff % 64 == 0 && c->vocab % 16 == 0, PHOTON_ERR_UNSUPPORTED,
                   "bf16 path needs D (%d) and d_ff (%d) multiples of 64 and vocab (%d) a multiple of 16", c->D, c->d_ff, c->vocab);
  } else {
    PHOTON_REQUIRE(c->D % 4 == 0 && c->d_ff % 4 == 0, PHOTON_ERR_UNSUPPORTED, "fp32 path needs D and d_ff multiples of 4");
  }
  PHOTON_REQUIRE((int64_t)Bt * c->H <= 65535, PHOTON_ERR_UNSUPPORTED, "Bt*H=%lld exceeds 65535", (long long)Bt * c->H);
  return PHOTON_OK;
}

// ------------------------------------------------------------------ composition

struct Ctx {
  const photon_config* c;
  const photon_weights* w;
  const photon_state* s;
  int Bt;
  hipStream_t st;
  Plan p;
  char* base;
  bool bf16;
  size_t o_h, o_attn, o_qkv, o_qrot, o_act;   // activation buffers of the branch this context drives
  size_t o_many;                              // its many-row linear scratch
  bool overlap;                               // run the top-level update beside the lower levels
  const photon_encoder_weights* ew = nullptr; // encoder-side weights (prefill, hierarchical generation)
  const photon_hier_state* hs = nullptr;      // lower-level encoder streams (hierarchical generation only)
  int* bar_next = nullptr;                    // next unused barrier slot (cleared slots: see step_begin_kernel); nullptr: none
  unsigned* bar_words() const { return reinterpret_cast<unsigned*>(base + p.bar); }
  int bar_word_count() const { return p.bar_slots * PM_BAR_WORDS + 64; }
  float* f(size_t off) const { return reinterpret_cast<float*>(base + off); }
};


// Rows entering a module pass: row i of the pass lives at in[i * ld] (D floats).
struct RowsIn {
  const float* ptr = nullptr;
  int64_t ld = 0;
};

static int32_t linear(const Ctx& x, const float* in, int64_t ldx, const void* W, const float* gain, const float* bias,
                      const float* res, int64_t ldres, float* out, int64_t ldo, int M, int N, int K, int epilogue,
                      bool in_bf16 = false, bool out_bf16 = false) {
  LinearArgs a;
  a.x_bf16 = in_bf16; a.out_bf16 = out_bf16;
  a.x = in; a.ldx = ldx; a.W = W; a.w_bf16 = x.bf16; a.gain = gain; a.eps = x.c->rms_eps; a.bias = bias; a.res = res;
  a.ldres = ldres; a.out = out; a.ldo = ldo; a.M = M; a.N = N; a.K = K; a.epilogue = epilogue;
  if (x.bf16 && M >= LINEAR_MANY_ROWS && K <= x.p.many_K && (epilogue != EPI_SWIGLU || 2 * N <= 2 * x.c->d_ff))
    return launch_linear_many(a, x.base + x.o_many, x.p.many_K, x.st);
  const int64_t w_bytes = (int64_t)(epilogue == EPI_SWIGLU ? 2 : 1) * N * K * 2;
  if (x.bf16 && M >= LINEAR_MID_ROWS && K <= x.p.many_K && w_bytes < ((int64_t)1 << 32)) {
    if (!in_bf16) {                                          // norm and rounding once, in front of the bf16-row kernel
      void* rows_bf16 = x.base + x.o_many;
      PHOTON_TRY(launch_norm_round_rows(in, ldx, gain, x.c->rms_eps, rows_bf16, M, K, x.st));
      a.x = reinterpret_cast<const float*>(rows_bf16); a.ldx = K; a.x_bf16 = true; a.gain = nullptr;
    }
    return launch_linear(a, x.st);
  }
  return launch_linear(a, x.st);
}

static int32_t norm(const Ctx& x, const float* in, int in_mul, int in_off, const float* g, float* out, int out_mul, int out_off,
                    int rows) {
  PHOTON_LAUNCH(KC_NORM, x.st, norm_rows_kernel, dim3(rows), dim3(256), x.c->D * sizeof(float), x.st, in, in_mul, in_off, g,
                x.c->rms_eps, out, out_mul, out_off, x.c->D);
  return check_launch("norm_rows_kernel");
}

// Tail of a block once the attention output sits in p.attn: O projection + residual, then the SwiGLU sub-layer,
// leaving the residual stream in p.h.  `in` is the block's input (the residual stream before the block: p.h from
// the second block on).  The stream between the two sub-layers lives in the q/k/v buffer, which the attention
// has finished with: no projection then adds a residual in place, which the many-row contraction does not allow
// (it requests residual values ahead of the stores of the tile before).
static int32_t block_tail(const Ctx& x, const photon_layer_weights& lw, RowsIn in, int rows, bool attn_bf16) {
  const photon_config& c = *x.c;
  float *h = x.f(x.o_h), *attn = x.f(x.o_attn), *act = x.f(x.o_act), *mid = x.f(x.o_qkv);
  PHOTON_TRY(linear(x, attn, c.D, lw.wo, nullptr, nullptr, in.ptr, in.ld, mid, c.D, rows, c.D, c.D, EPI_RESID, attn_bf16, false));
  if (c.d_ff == 0) {
    PHOTON_LAUNCH(KC_MISC, x.st, copy_f32x4_kernel, dim3((unsigned)(((int64_t)rows * c.D / 4 + 255) / 256)), dim3(256), 0, x.st,
                  reinterpret_cast<const float4_t*>(mid), reinterpret_cast<float4_t*>(h), (int64_t)rows * c.D / 4);
    return check_launch("copy_f32x4_kernel");
  }
  // with bf16 matrices the hidden rows are kept as bf16: they are the down projection's MFMA operand as they stand
  PHOTON_TRY(linear(x, mid, c.D, lw.wgu, lw.g2, nullptr, nullptr, 0, act, c.d_ff, rows, c.d_ff, c.D, EPI_SWIGLU, false, x.bf16));
  return linear(x, act, c.d_ff, lw.wd, nullptr, nullptr, mid, c.D, h, c.D, rows, c.D, c.d_ff, EPI_RESID, x.bf16, false);
}

// All blocks of the level-`level` local decoder on n_chunks * q_len rows (window positions
// q_pos .. q_pos+q_len-1 of every chunk).  Leaves the residual stream in p.h.
// alone: nothing else runs beside this pass (no STEP branch on the side stream).  The persistent kernel holds every
// compute unit's registers and most of its LDS, so kernels of another stream cannot run beside it: where the
// top-level update overlaps the lower levels, those levels keep the separate launches.
static int32_t local_module_pass(const Ctx& x, int level, int64_t n_chunks, int q_len, int q_pos, RowsIn in, bool alone = true) {
  const photon_config& c = *x.c;
  const photon_module_weights& mod = x.w->dec[level - 1];
  const int W = c.R[level - 1] + c.C[level - 1] - 1;
  const int rows = (int)(n_chunks * q_len);
  float *h = x.f(x.o_h), *qkv = x.f(x.o_qkv), *attn = x.f(x.o_attn);
  const size_t layer_cache = (size_t)n_chunks * W * c.D;
  const float scale = 1.0f / sqrtf((float)c.d_h);
  if (alone && x.bf16 && c.d_ff > 0 && rows <= PM_MAX_ROWS && x.bar_next != nullptr && *x.bar_next < x.p.bar_slots && !g_no_persistent) {
    // all blocks in one launch, the projections meeting at grid barriers instead of kernel boundaries
    PersistentModule pm;
    pm.layers = mod.layers; pm.n_layers = c.n_layers;
    pm.x_in = in.ptr; pm.ld_in = in.ld;
    pm.h = h; pm.qkv = qkv; pm.attn = attn; pm.act = x.f(x.o_act);
    pm.lk = x.f(x.p.lk[level - 1]); pm.lv = x.f(x.p.lv[level - 1]); pm.layer_cache = layer_cache;
    pm.bar = x.bar_words() + (size_t)(*x.bar_next) * PM_BAR_WORDS;
    pm.err = x.bar_words() + (size_t)x.p.bar_slots * PM_BAR_WORDS;
    pm.M = rows; pm.D = c.D; pm.F = c.d_ff; pm.H = c.H; pm.d_h = c.d_h;
    pm.n_chunks = n_chunks; pm.W = W; pm.q_len = q_len; pm.q_pos = q_pos;
    pm.eps = c.rms_eps; pm.scale = scale; pm.theta = c.rope_theta;
    if (persistent_module_supported(pm)) {
      ++*x.bar_next;
      return launch_persistent_module(pm, x.st);
    }
  }
  for (int i = 0; i < c.n_layers; ++i) {
    const photon_layer_weights& lw = mod.layers[i];
    float* lk = x.f(x.p.lk[level - 1]) + (size_t)i * layer_cache;
    float* lv = x.f(x.p.lv[level - 1]) + (size_t)i * layer_cache;
    PHOTON_TRY(linear(x, in.ptr, in.ld, lw.wqkv, lw.g1, nullptr, nullptr, 0, qkv, 3 * c.D, rows, 3 * c.D, c.D, EPI_PLAIN));
    // with bf16 matrices the attention rows are written as bf16: the O projection's MFMA operand as they stand
    PHOTON_TRY(launch_local_step_attn(c.d_h, qkv, lk, lv, attn, n_chunks, W, q_len, q_pos, c.H, scale, c.rope_theta, x.bf16, x.st));
    PHOTON_TRY(block_tail(x, lw, in, rows, x.bf16));
    in.ptr = h; in.ld = c.D;
  }
  return PHOTON_OK;
}

// STEP (Eq. 12-13) of one encoder stream on the Bt rows `in` (one new unit per sequence): appends K/V to the
// stream's cache at position seq_len - 1 (the count already includes the new unit) and writes the new state
// of sequence b to out[(b * out_mul + out_off) * D].
static int32_t stream_step(const Ctx& x, const photon_module_weights& mod, void* k_cache, void* v_cache, const int32_t* seq_len,
                           int64_t S_cap, RowsIn in, float* out, int out_mul, int out_off) {
  const photon_config& c = *x.c;
  const int rows = x.Bt;
  float *h = x.f(x.o_h), *qkv = x.f(x.o_qkv), *qrot = x.f(x.o_qrot), *attn = x.f(x.o_attn);
  const size_t esz = dtype_size(c.kv_dt);
  const int pitch = kv_row_elems(c.d_h);
  const size_t layer_cache = (size_t)x.Bt * c.H * S_cap * pitch * esz;
  const float scale = 1.0f / sqrtf((float)c.d_h);
  for (int i = 0; i < c.n_layers; ++i) {
    const photon_layer_weights& lw = mod.layers[i];
    char* kc = reinterpret_cast<char*>(k_cache) + (size_t)i * layer_cache;
    char* vc = reinterpret_cast<char*>(v_cache) + (size_t)i * layer_cache;
    PHOTON_TRY(linear(x, in.ptr, in.ld, lw.wqkv, lw.g1, nullptr, nullptr, 0, qkv, 3 * c.D, rows, 3 * c.D, c.D, EPI_PLAIN));
    const int64_t n_el = (int64_t)rows * c.H * (c.d_h / 2);
    if (c.kv_dt == PHOTON_FP8_E4M3)
      PHOTON_LAUNCH(KC_ROPE_APPEND, x.st, rope_append_coarse_kernel<fp8_t>, dim3(blocks_for(n_el)), dim3(256), 0, x.st, qkv, qrot,
                    (fp8_t*)kc, (fp8_t*)vc, seq_len, x.Bt, c.H, c.d_h, pitch, S_cap, c.rope_theta);
    else if (x.bf16)
      PHOTON_LAUNCH(KC_ROPE_APPEND, x.st, rope_append_coarse_kernel<bf16_t>, dim3(blocks_for(n_el)), dim3(256), 0, x.st, qkv, qrot,
                    (bf16_t*)kc, (bf16_t*)vc, seq_len, x.Bt, c.H, c.d_h, pitch, S_cap, c.rope_theta);
    else
      PHOTON_LAUNCH(KC_ROPE_APPEND, x.st, rope_append_coarse_kernel<float>, dim3(blocks_for(n_el)), dim3(256), 0, x.st, qkv, qrot,
                    (float*)kc, (float*)vc, seq_len, x.Bt, c.H, c.d_h, pitch, S_cap, c.rope_theta);
    PHOTON_TRY(check_launch("rope_append_coarse_kernel"));
    PHOTON_TRY(launch_coarse_attn(c.kv_dt == PHOTON_FP8_E4M3 ? KV_FP8 : x.bf16 ? KV_BF16 : KV_F32, true, c.d_h, qrot, kc, vc, seq_len, attn, x.Bt, c.H, S_cap, scale,
                                  x.p.n_splits, x.base + x.p.coarse_ws, x.st));
    PHOTON_TRY(block_tail(x, lw, in, rows, false));      // the coarse attention writes fp32 rows
    in.ptr = h; in.ld = c.D;
  }
  return norm(x, h, 1, 0, mod.g_final, out, out_mul, out_off, rows);
}

// STEP of the top-level encoder; leaves X^(L)_{g+1} in state.x_top.
static int32_t top_step(const Ctx& x, RowsIn in) {
  return stream_step(x, x.w->top, x.s->k_cache, x.s->v_cache, x.s->seq_len, x.s->S_max, in, x.s->x_top, 1, 0);
}

// Step 2 of hierarchical generation (Appendix A, Definition 1): re-encode the step's tokens bottom-up.  Every
// level l < L advances its stream by its new units, one STEP per unit (they are causally ordered).  Returns the
// encoder-side level-(L-1) block [Bt, C_L, D] (rows of sequence b contiguous).
static int32_t embed_rows(hipStream_t st, bool bf16, const int32_t* tokens, const void* table, float* rows, int64_t n, int width, int vocab) {
  if (bf16)
    PHOTON_LAUNCH(KC_MISC, st, embed_rows_kernel<bf16_t>, dim3(blocks_for(n * (width / 4))), dim3(256), 0, st, tokens, (const bf16_t*)table,
                  rows, n, width, vocab);
  else
    PHOTON_LAUNCH(KC_MISC, st, embed_rows_kernel<float>, dim3(blocks_for(n * (width / 4))), dim3(256), 0, st, tokens, (const float*)table,
                  rows, n, width, vocab);
  return check_launch("embed_rows_kernel");
}

static int32_t hier_reencode(const Ctx& x, const int32_t* tokens, const float** bottleneck) {
  const photon_config& c = *x.c;
  const int D = c.D, L = c.L, Bt = x.Bt;
  int64_t per_seq = 1;
  for (int l = 0; l < L; ++l) per_seq *= c.C[l];
  float* A = x.f(x.p.hA);
  // parameter-free level-1 chunker: the embeddings are D / C_1 wide and C_1 of them side by side ARE the unit
  const bool concat1 = L >= 2 && x.ew->chunker_w[0] == nullptr;
  float* X = concat1 ? A : x.f(x.p.hx[0]);                 // encoder-side level-0 states of the new tokens
  const int64_t n_tok = (int64_t)Bt * per_seq;
  PHOTON_TRY(embed_rows(x.st, x.bf16, tokens, x.ew->E_enc, X, n_tok, concat1 ? D / c.C[0] : D, c.vocab));
  for (int l = 1; l < L; ++l) {
    const int C = c.C[l - 1];
    per_seq /= C;                                          // new level-l units per sequence
    const int rows = (int)(Bt * per_seq);
    if (!(l == 1 && concat1))
      PHOTON_TRY(linear(x, X, (int64_t)C * D, x.ew->chunker_w[l - 1], nullptr, x.ew->chunker_b[l - 1], nullptr, 0, A, D, rows, D, C * D,
                        EPI_PLAIN));
    float* Xl = x.f(x.p.hx[l]);
    for (int j = 0; j < (int)per_seq; ++j) {
      PHOTON_LAUNCH(KC_MISC, x.st, step_begin_kernel, dim3(blocks_for(Bt)), dim3(256), 0, x.st, x.hs->seq_len[l - 1], Bt, x.hs->S_cap[l - 1],
                    x.s->status, (unsigned*)nullptr, 0);
      PHOTON_TRY(check_launch("step_begin_kernel"));
      RowsIn in;
      in.ptr = A + (int64_t)j * D; in.ld = per_seq * (int64_t)D;
      PHOTON_TRY(stream_step(x, x.ew->enc[l - 1], x.hs->k_cache[l - 1], x.hs->v_cache[l - 1], x.hs->seq_len[l - 1], x.hs->S_cap[l - 1], in,
                             Xl, (int)per_seq, j));
    }
    X = Xl;
  }
  *bottleneck = X;
  return PHOTON_OK;
}

// (ii) top chunker (Eq. 4) on the C_L new level-(L-1) units of every sequence, (iii) STEP (Eq. 13).
static int32_t chunk_and_step(const Ctx& x, const float* bottleneck, const photon_trace* tr) {
  const photon_config& c = *x.c;
  const int D = c.D, CL = c.C[c.L - 1];
  float* a_hat = (tr && tr->a_hat) ? tr->a_hat : x.f(x.p.a_hat);
  PHOTON_TRY(linear(x, bottleneck, (int64_t)CL * D, x.w->chunker_w, nullptr, x.w->chunker_b, nullptr, 0, a_hat, D, x.Bt, D, CL * D,
                    EPI_PLAIN));
  RowsIn top_in;
  top_in.ptr = a_hat; top_in.ld = D;
  return top_step(x, top_in);
}

// The top-level update depends only on the level-L decoder's output, not on the lower levels that turn it into
// tokens, so for L >= 2 it can run on a second stream beside them (fork after level L, join at the end of the
// step).  That stream and the two events belong to the caller (photon_state): the library creates nothing.
// All sub-steps of the level-l local decoder on this context's stream and buffers: n chunks, each conditioned on a row
// of cond_in; the new level-(l-1) units go to `units` ([n * C_l, D], item j of chunk ch at row ch * C_l + j); at level 1
// the logits, the token choice and the decoder-side embedding fed back.  after_converter: recorded on the stream once
// the converter, the only reader of cond_in, is enqueued (nullptr: nothing to record).
static int32_t decode_level(const Ctx& x, int l, const float* cond_in, float* units, const int32_t* forced, int32_t* out_tokens,
                            const photon_trace* tr, bool alone, hipEvent_t after_converter) {
  const photon_config& c = *x.c;
  const int D = c.D, L = c.L;
  const int C = c.C[l - 1], R = c.R[l - 1];
  const int64_t n = x.p.chunks[l];
  const photon_module_weights& mod = x.w->dec[l - 1];
  float* h = x.f(x.o_h);
  // sub-step 0: the converter's R vectors at window positions 0..R-1 (row ch*R + r of a flat [n*R, D] view of h)
  PHOTON_TRY(linear(x, cond_in, D, x.w->conv_w[l - 1], nullptr, x.w->conv_b[l - 1], nullptr, 0, h, (int64_t)R * D, (int)n, R * D, D,
                    EPI_PLAIN));
  if (after_converter != nullptr && hipEventRecord(after_converter, x.st) != hipSuccess)
    return fail(PHOTON_ERR_HIP, "decode step: cannot record the event that frees the conditioning buffer");
  RowsIn in;
  in.ptr = h; in.ld = D;
  for (int j = 0; j < C; ++j) {
    const int q_len = (j == 0) ? R : 1;
    const int q_pos = (j == 0) ? 0 : R + j - 1;
    PHOTON_TRY(local_module_pass(x, l, n, q_len, q_pos, in, alone));
    // item j = final norm of the last row of each chunk.  At the token level of a hierarchy the item only feeds the
    // vocabulary projection, which then applies the norm itself (one launch less per sub-step) unless the caller
    // asked to see the items.
    const bool norm_in_head = (l == 1 && L >= 2 && !(tr && tr->new_units[0]));
    if (!norm_in_head) PHOTON_TRY(norm(x, h, q_len, q_len - 1, mod.g_final, units, C, j, (int)n));
    if (l >= 2) {                                          // Eq. 6: the module's own output is the next input
      in.ptr = units + (int64_t)j * D; in.ld = (int64_t)C * D;
    } else {
      float* lg = (tr && tr->logits) ? tr->logits + (int64_t)j * c.vocab : x.f(x.p.logits);
      const int64_t ld = (tr && tr->logits) ? (int64_t)C * c.vocab : c.vocab;
      // logits of item j of every chunk: rows of `units` with pitch C*D
      if (norm_in_head)
        PHOTON_TRY(linear(x, h + (int64_t)(q_len - 1) * D, (int64_t)q_len * D, x.w->W_lm, mod.g_final, nullptr, nullptr, 0, lg, ld, (int)n,
                          c.vocab, D, EPI_PLAIN));
      else
        PHOTON_TRY(linear(x, units + (int64_t)j * D, (int64_t)C * D, x.w->W_lm, nullptr, nullptr, nullptr, 0, lg, ld, (int)n, c.vocab, D,
                          EPI_PLAIN));
      float* x_next = (j + 1 < C) ? h : nullptr;           // decoder-side embedding of the chosen token
      if (x.bf16)
        PHOTON_LAUNCH(KC_CHOOSE_TOKEN, x.st, choose_token_kernel<bf16_t>, dim3((unsigned)n), dim3(CHOOSE_THREADS), 0, x.st, lg, ld, c.vocab,
                      forced, out_tokens, C, j, (const bf16_t*)x.w->E_dec, x_next, D);
      else
        PHOTON_LAUNCH(KC_CHOOSE_TOKEN, x.st, choose_token_kernel<float>, dim3((unsigned)n), dim3(CHOOSE_THREADS), 0, x.st, lg, ld, c.vocab,
                      forced, out_tokens, C, j, (const float*)x.w->E_dec, x_next, D);
      PHOTON_TRY(check_launch("choose_token_kernel"));
      in.ptr = h; in.ld = D;
    }
  }
  return PHOTON_OK;
}

// Conditioning of the level-(l-1) chunks from the new level-(l-1) units of this step and the carry, which is updated.
static int32_t condition_lower(const Ctx& x, int l, const float* units, float* cond) {
  const photon_config& c = *x.c;
  const int64_t n = x.p.chunks[l];
  const int C = c.C[l - 1], D = c.D, Bt = x.Bt;
  const int64_t per_seq = n * C / Bt;
  float* carry = x.s->carry + (int64_t)(l - 2) * Bt * D;
  PHOTON_LAUNCH(KC_MISC, x.st, shift_condition_kernel, dim3(blocks_for(n * C * D)), dim3(256), 0, x.st, units, carry, cond, Bt, (int)per_seq, D);
  return check_launch("shift_condition_kernel");
}

// The levels below the top, in order, on this context's stream: level L-1 hangs off cond_top, every further level off
// the units of the level above it.
static int32_t decode_lower_levels(const Ctx& x, const float* cond_top, float* const* fresh, const int32_t* forced, int32_t* out_tokens,
                                   const photon_trace* tr, bool alone, hipEvent_t after_first_converter) {
  const float* cond_in = cond_top;
  for (int l = x.c->L - 1; l >= 1; --l) {
    PHOTON_TRY(decode_level(x, l, cond_in, fresh[l - 1], forced, out_tokens, tr, alone, l == x.c->L - 1 ? after_first_converter : nullptr));
    if (l >= 2) {
      PHOTON_TRY(condition_lower(x, l, fresh[l - 1], x.f(x.p.cond)));
      cond_in = x.f(x.p.cond);
    }
  }
  return PHOTON_OK;
}

// One step.  The recurrence of recursive generation runs through the top level only: X^(L)_g -> top-level decoder ->
// chunker -> STEP -> X^(L)_{g+1} (Section 2.3.3 (i)-(iii)); the lower levels, which turn the top-level decoder's
// output into tokens, hang off it as a leaf (the next step reads only the carries, which the main line itself
// updates).  With a side stream lent by the caller the lower levels run there, beside the chunker and STEP; in
// pipelined mode they are not joined at the end of the call, so that they also run beside the next step's top level.
static int32_t decode_step_impl(const Ctx& x, photon_state* st, const int32_t* forced, int32_t* out_tokens, const photon_trace* tr) {
  const photon_config& c = *x.c;
  const int L = c.L, Bt = x.Bt;

  PHOTON_LAUNCH(KC_MISC, x.st, step_begin_kernel, dim3(blocks_for(Bt)), dim3(256), 0, x.st, x.s->seq_len, Bt, x.s->S_max, x.s->status,
                x.bar_words(), x.bar_word_count());
  PHOTON_TRY(check_launch("step_begin_kernel"));

  float* fresh[PHOTON_MAX_LEVELS];
  for (int l = 0; l < L; ++l) fresh[l] = (tr && tr->new_units[l]) ? tr->new_units[l] : x.f(x.p.fresh[l]);

  const bool pipelined = x.overlap && st->pipeline != 0;
  // the main line of a hierarchy has its own activation buffers: the lower levels of this (or, pipelined, of the
  // previous) step work on the first set meanwhile
  Ctx top = x;
  if (L >= 2) {
    top.o_h = x.p.h2; top.o_attn = x.p.attn2; top.o_qkv = x.p.qkv2; top.o_qrot = x.p.qrot2; top.o_act = x.p.act2; top.o_many = x.p.many2;
  }
  // level L: one chunk per sequence, conditioned on X^(L)_g.  Persistent launches only when nothing runs beside them
  // (a pipelined state keeps the separate launches also while a profiler holds the step on one stream, so that what
  // is profiled is what is timed).
  PHOTON_TRY(decode_level(top, L, x.s->x_top, fresh[L - 1], forced, out_tokens, tr, st->pipeline == 0, nullptr));

  if (L >= 2) {
    float* cond_top = x.f(x.p.cond_top);
    hipStream_t side_st = (hipStream_t)st->side_stream;
    if (pipelined && st->lower_levels_pending != 0 &&
        hipStreamWaitEvent(x.st, (hipEvent_t)st->free_event, 0) != hipSuccess)      // the previous step's lower levels have read cond_top
      return fail(PHOTON_ERR_HIP, "decode step: cannot wait for the conditioning buffer");
    PHOTON_TRY(condition_lower(top, L, fresh[L - 1], cond_top));
    if (x.overlap && x.hs == nullptr) {
      if (hipEventRecord((hipEvent_t)st->fork_event, x.st) != hipSuccess || hipStreamWaitEvent(side_st, (hipEvent_t)st->fork_event, 0) != hipSuccess)
        return fail(PHOTON_ERR_HIP, "decode step: cannot fork the lower levels");
      Ctx side = x;
      side.st = side_st;
      side.bar_next = nullptr;
      PHOTON_TRY(decode_lower_levels(side, cond_top, fresh, forced, out_tokens, tr, false, pipelined ? (hipEvent_t)st->free_event : nullptr));
      PHOTON_TRY(chunk_and_step(top, fresh[L - 1], tr));
      if (pipelined) {
        st->lower_levels_pending = 1;
      } else if (hipEventRecord((hipEvent_t)st->join_event, side_st) != hipSuccess || hipStreamWaitEvent(x.st, (hipEvent_t)st->join_event, 0) != hipSuccess) {
        return fail(PHOTON_ERR_HIP, "decode step: cannot join the lower levels");
      }
    } else {
      // one stream: persistent launches where eligible, unless the state has a side stream and is merely held on one
      // stream by the profiler (what is profiled is then what is timed)
      const bool side_lent = st->side_stream != nullptr && st->fork_event != nullptr && st->join_event != nullptr;
      PHOTON_TRY(decode_lower_levels(x, cond_top, fresh, forced, out_tokens, tr, !side_lent || x.hs != nullptr, nullptr));
      if (x.hs != nullptr) {
        const float* bott = nullptr;
        PHOTON_TRY(hier_reencode(x, out_tokens, &bott));
        PHOTON_TRY(chunk_and_step(top, bott, tr));
      } else {
        PHOTON_TRY(chunk_and_step(top, fresh[L - 1], tr));
      }
    }
  } else if (x.hs != nullptr) {
    const float* bott = nullptr;
    PHOTON_TRY(hier_reencode(x, out_tokens, &bott));
    PHOTON_TRY(chunk_and_step(x, bott, tr));
  } else {
    PHOTON_TRY(chunk_and_step(x, fresh[L - 1], tr));
  }
  if (x.s->status != nullptr && x.bar_next != nullptr && *x.bar_next > 0) {
    PHOTON_LAUNCH(KC_MISC, x.st, step_end_kernel, dim3(1), dim3(64), 0, x.st,
                  (const unsigned*)(x.bar_words() + (size_t)x.p.bar_slots * PM_BAR_WORDS), x.s->status);
    PHOTON_TRY(check_launch("step_end_kernel"));
  }
  return PHOTON_OK;
}

}  // namespace photon

using namespace photon;

// ------------------------------------------------------------------ prefill

struct PrefillPlan {
  int64_t M[PHOTON_MAX_LEVELS + 1] = {0};        // M[l]: level-l units per sequence, M[0] = T
  size_t X[PHOTON_MAX_LEVELS + 1] = {0};         // X[l]: level-l encoder states [Bt*M[l], D]; X[0] = embeddings; X[L] unused
  size_t A = 0, h = 0, attn = 0, qkv = 0, act = 0, many = 0, ea = 0, pair = 0;
  int many_K = 0;
  size_t total = 0;
};

static PrefillPlan make_prefill_plan(const photon_config& c, int Bt, int64_t T) {
  PrefillPlan p;
  const int64_t D = c.D, F = c.d_ff;
  const size_t f = sizeof(float);
  p.M[0] = T;
  for (int l = 1; l <= c.L; ++l) p.M[l] = p.M[l - 1] / c.C[l - 1];
  size_t cur = 0;
  for (int l = 0; l < c.L; ++l) p.X[l] = bump(cur, (size_t)Bt * p.M[l] * D * f);
  const int64_t rows = (int64_t)Bt * p.M[1];     // the widest level
  p.A = bump(cur, rows * D * f);
  p.h = bump(cur, rows * D * f);
  p.attn = bump(cur, rows * D * f);
  p.qkv = bump(cur, rows * 3 * D * f);
  p.act = bump(cur, rows * F * f);
  p.pair = bump(cur, (size_t)2 * Bt * D * f);    // conditioning latent of the carry decode, and a spare
  if (c.dt == PHOTON_BF16) {
    p.many_K = (int)(D > F ? D : F);
    for (int l = 1; l <= c.L; ++l)
      if ((int64_t)c.C[l - 1] * D > p.many_K) p.many_K = (int)(c.C[l - 1] * D);
    if (rows >= LINEAR_MID_ROWS) p.many = bump(cur, linear_many_workspace_bytes(rows, p.many_K, (int)(2 * F)));
  }
  p.ea = bump(cur, encoder_attn_workspace_bytes(Bt, p.M[1], c.H, c.d_h, c.dt == PHOTON_BF16));
  p.total = cur;
  return p;
}

// Bottom-up encoder pass over the prompt, then the carries.  `x` is a decode-step context on the state's own
// workspace (the carry decode is a teacher-forced run of the decode sub-steps); `e` drives the big buffers.
static int32_t prefill_impl(const Ctx& x, Ctx e, const PrefillPlan& pp, const photon_encoder_weights& ew, const int32_t* tokens) {
  const photon_config& c = *x.c;
  const int D = c.D, L = c.L, Bt = x.Bt;
  const float scale = 1.0f / sqrtf((float)c.d_h);
  const size_t esz = dtype_size(c.kv_dt);

  float *A = e.f(pp.A), *h = e.f(pp.h), *qkv = e.f(pp.qkv), *attn = e.f(pp.attn);
  float* pair = e.f(pp.pair);
  // X^(0): encoder-side embeddings.  Parameter-free level-1 chunker: they are D / C_1 wide, and C_1 of them side
  // by side are A^(1) itself.
  const bool concat1 = L >= 2 && ew.chunker_w[0] == nullptr;
  const int64_t n_tok = (int64_t)Bt * pp.M[0];
  PHOTON_TRY(embed_rows(x.st, x.bf16, tokens, ew.E_enc, concat1 ? A : e.f(pp.X[0]), n_tok, concat1 ? D / c.C[0] : D, c.vocab));

  for (int l = 1; l <= L; ++l) {
    const int C = c.C[l - 1];
    const int64_t M = pp.M[l];
    const int rows = (int)(Bt * M);
    const photon_module_weights& mod = ew.enc[l - 1];
    // Eq. 4: C consecutive level-(l-1) states are one row of C*D inputs (the states are contiguous per sequence)
    if (!(l == 1 && concat1))
      PHOTON_TRY(linear(e, e.f(pp.X[l - 1]), (int64_t)C * D, ew.chunker_w[l - 1], nullptr, ew.chunker_b[l - 1], nullptr, 0, A, D, rows, D,
                        C * D, EPI_PLAIN));
    RowsIn in;
    in.ptr = A; in.ld = D;
    const size_t layer_cache = (size_t)Bt * c.H * x.s->S_max * kv_row_elems(c.d_h) * esz;
    for (int i = 0; i < c.n_layers; ++i) {
      const photon_layer_weights& lw = mod.layers[i];
      PHOTON_TRY(linear(e, in.ptr, in.ld, lw.wqkv, lw.g1, nullptr, nullptr, 0, qkv, 3 * D, rows, 3 * D, D, EPI_PLAIN));
      char *kc = nullptr, *vc = nullptr;
      int64_t cap = x.s->S_max;
      if (l == L) {
        kc = reinterpret_cast<char*>(x.s->k_cache) + (size_t)i * layer_cache;
        vc = reinterpret_cast<char*>(x.s->v_cache) + (size_t)i * layer_cache;
      } else if (x.hs != nullptr) {                        // hierarchical generation keeps every level's stream
        cap = x.hs->S_cap[l - 1];
        const size_t lc = (size_t)Bt * c.H * cap * kv_row_elems(c.d_h) * esz;
        kc = reinterpret_cast<char*>(x.hs->k_cache[l - 1]) + (size_t)i * lc;
        vc = reinterpret_cast<char*>(x.hs->v_cache[l - 1]) + (size_t)i * lc;
      }
      PHOTON_TRY(launch_encoder_attn(qkv, attn, Bt, M, c.H, c.d_h, c.rope_theta, scale, kc, vc, cap, e.base + pp.ea, x.bf16, c.kv_dt == PHOTON_FP8_E4M3, x.bf16, x.st));
      PHOTON_TRY(block_tail(e, lw, in, rows, x.bf16));
      in.ptr = h; in.ld = D;
    }
    if (l < L) {
      PHOTON_TRY(norm(e, in.ptr, 1, 0, mod.g_final, e.f(pp.X[l]), 1, 0, rows));
      if (x.hs != nullptr) {
        PHOTON_LAUNCH(KC_MISC, x.st, fill_i32_kernel, dim3(blocks_for(Bt)), dim3(256), 0, x.st, x.hs->seq_len[l - 1], (int32_t)M, Bt);
        PHOTON_TRY(check_launch("fill_i32_kernel"));
      }
    } else {
      // only two rows of X^(L) are ever used: the last one (the top state) and the one before it (conditions the carry decode)
      PHOTON_TRY(norm(e, in.ptr, (int)M, (int)M - 1, mod.g_final, x.s->x_top, 1, 0, Bt));
      if (L >= 2) {
        if (M >= 2) {
          PHOTON_TRY(norm(e, in.ptr, (int)M, (int)M - 2, mod.g_final, pair, 1, 0, Bt));
        } else {
          PHOTON_LAUNCH(KC_MISC, x.st, broadcast_rows_kernel, dim3(blocks_for((int64_t)Bt * D)), dim3(256), 0, x.st, ew.x0[L - 1], pair, Bt, D);
          PHOTON_TRY(check_launch("broadcast_rows_kernel"));
        }
      }
    }
  }
  PHOTON_LAUNCH(KC_MISC, x.st, fill_i32_kernel, dim3(blocks_for(Bt)), dim3(256), 0, x.st, x.s->seq_len, (int32_t)pp.M[L], Bt);
  PHOTON_TRY(check_launch("fill_i32_kernel"));

  // Carries: teacher-forced decode of the last chunk of every level l >= 2 (one chunk per sequence), on the
  // decode step's own buffers.  Inputs of sub-step j >= 1 are the encoder-side states of the chunk (reading G7).
  if (L >= 2) {
    PHOTON_LAUNCH(KC_MISC, x.st, step_begin_kernel, dim3(1), dim3(256), 0, x.st, (int32_t*)nullptr, 0, (int64_t)0, (int32_t*)nullptr,
                  x.bar_words(), x.bar_word_count());
    PHOTON_TRY(check_launch("step_begin_kernel"));
  }
  const float* cond = pair;                                // level-l latent before the last one, one row per sequence
  int64_t cond_ld = D;
  float* dh = x.f(x.o_h);
  float* units = x.f(x.p.fresh[0]);                        // [Bt * C, D] scratch: the items of the chunk
  for (int l = L; l >= 2; --l) {
    const int C = c.C[l - 1], R = c.R[l - 1];
    const photon_module_weights& mod = x.w->dec[l - 1];
    PHOTON_TRY(linear(x, cond, cond_ld, x.w->conv_w[l - 1], nullptr, x.w->conv_b[l - 1], nullptr, 0, dh, (int64_t)R * D, Bt, R * D, D,
                      EPI_PLAIN));
    RowsIn in;
    in.ptr = dh; in.ld = D;
    const float* teacher = e.f(pp.X[l - 1]) + (pp.M[l - 1] - C) * (int64_t)D;   // sequence b: + b * M[l-1] * D
    for (int j = 0; j < C; ++j) {
      const int q_len = (j == 0) ? R : 1;
      const int q_pos = (j == 0) ? 0 : R + j - 1;
      PHOTON_TRY(local_module_pass(x, l, Bt, q_len, q_pos, in));
      PHOTON_TRY(norm(x, dh, q_len, q_len - 1, mod.g_final, units, C, j, Bt));
      in.ptr = teacher + (int64_t)j * D; in.ld = pp.M[l - 1] * (int64_t)D;
    }
    // carry^(l-1) = the chunk's last item (C >= 2: the last sub-step had one row per sequence);
    // the item before it conditions the last chunk of the level below
    PHOTON_TRY(norm(x, dh, 1, 0, mod.g_final, x.s->carry + (size_t)(l - 2) * Bt * D, 1, 0, Bt));
    cond = units + (int64_t)(C - 2) * D;
    cond_ld = (int64_t)C * D;
  }
  return PHOTON_OK;
}

extern "C" size_t photon_decode_step_workspace_bytes(const photon_config* cfg, int32_t Bt, int64_t S_max) {
  clear_error();
  if (validate_config(cfg, Bt, S_max) != PHOTON_OK) return 0;
  return make_plan(*cfg, Bt, S_max).total;
}

static int32_t require_module(const photon_config& c, const photon_module_weights& mod, const char* what, int level) {
  PHOTON_REQUIRE(mod.layers && mod.g_final, PHOTON_ERR_INVALID_ARG, "%s module of level %d missing", what, level);
  for (int i = 0; i < c.n_layers; ++i) {
    const photon_layer_weights& lw = mod.layers[i];
    const bool ok = lw.g1 && lw.wqkv && aligned16(lw.wqkv) && lw.wo && aligned16(lw.wo) &&
                    (c.d_ff == 0 || (lw.g2 && lw.wgu && aligned16(lw.wgu) && lw.wd && aligned16(lw.wd)));
    PHOTON_REQUIRE(ok, PHOTON_ERR_INVALID_ARG, "%s module of level %d, layer %d has a null or misaligned weight", what, level, i);
  }
  return PHOTON_OK;
}

static int32_t validate_prefill(const photon_config& c, int Bt, int64_t T, int64_t S_max) {
  int64_t meta = 1;
  for (int l = 0; l < c.L; ++l) meta *= c.C[l];
  PHOTON_REQUIRE(T >= meta && T % meta == 0, PHOTON_ERR_INVALID_ARG, "prefill: T=%lld must be a positive multiple of prod(C)=%lld",
                 (long long)T, (long long)meta);
  PHOTON_REQUIRE(T / meta <= S_max, PHOTON_ERR_INVALID_ARG, "prefill: %lld top-level units do not fit S_max=%lld", (long long)(T / meta),
                 (long long)S_max);
  PHOTON_REQUIRE((int64_t)Bt * (T / c.C[0]) <= (1 << 24), PHOTON_ERR_UNSUPPORTED, "prefill: %lld level-1 rows exceed 2^24",
                 (long long)Bt * (T / c.C[0]));
  for (int l = 2; l <= c.L; ++l)
    PHOTON_REQUIRE(c.C[l - 1] >= 2, PHOTON_ERR_UNSUPPORTED, "prefill: level %d has C=%d; the carry decode needs C >= 2 above level 1", l,
                   c.C[l - 1]);
  return PHOTON_OK;
}

extern "C" size_t photon_prefill_workspace_bytes(const photon_config* cfg, int32_t Bt, int64_t T) {
  clear_error();
  if (cfg == nullptr || validate_config(cfg, Bt, 1) != PHOTON_OK) return 0;
  if (validate_prefill(*cfg, Bt, T, (int64_t)1 << 40) != PHOTON_OK) return 0;
  return make_prefill_plan(*cfg, Bt, T).total;
}

static int32_t require_hier_state(const photon_config& c, const photon_hier_state* hst) {
  for (int l = 1; l < c.L; ++l) {
    PHOTON_REQUIRE(hst->k_cache[l - 1] && aligned16(hst->k_cache[l - 1]) && hst->v_cache[l - 1] && aligned16(hst->v_cache[l - 1]) &&
                       hst->seq_len[l - 1] && hst->S_cap[l - 1] > 0,
                   PHOTON_ERR_INVALID_ARG, "stream of level %d: cache, seq_len or capacity missing or misaligned", l);
  }
  return PHOTON_OK;
}

static int32_t require_encoders(const photon_config& c, const photon_encoder_weights* ew) {
  PHOTON_REQUIRE_PTR(ew->E_enc);
  for (int l = 1; l <= c.L; ++l) {
    if (l == 1 && c.L >= 2 && ew->chunker_w[0] == nullptr) {   // parameter-free concatenation of D / C_1 wide embeddings
      PHOTON_REQUIRE(c.D % (4 * c.C[0]) == 0 && ew->chunker_b[0] == nullptr, PHOTON_ERR_INVALID_ARG,
                     "level-1 chunker without a matrix: D=%d must be a multiple of 4*C_1=%d, and there is no bias", c.D, 4 * c.C[0]);
      PHOTON_TRY(require_module(c, ew->enc[0], "encoder", 1));
      continue;
    }
    PHOTON_REQUIRE(ew->chunker_w[l - 1] && aligned16(ew->chunker_w[l - 1]), PHOTON_ERR_INVALID_ARG,
                   "chunker of level %d missing or misaligned", l);
    PHOTON_TRY(require_module(c, ew->enc[l - 1], "encoder", l));
  }
  return PHOTON_OK;
}

extern "C" int32_t photon_prefill(const photon_config* cfg, const photon_weights* w, const photon_encoder_weights* ew,
                                  const photon_state* st, const photon_hier_state* hst, int32_t Bt, const int32_t* tokens, int64_t T,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  PHOTON_REQUIRE(cfg && w && ew && st, PHOTON_ERR_INVALID_ARG, "%s: cfg, w, ew and st must not be null", __func__);
  PHOTON_TRY(validate_config(cfg, Bt, st->S_max));
  const photon_config& c = *cfg;
  PHOTON_TRY(validate_prefill(c, Bt, T, st->S_max));
  PHOTON_REQUIRE(tokens != nullptr, PHOTON_ERR_INVALID_ARG, "%s: tokens is null", __func__);
  PHOTON_REQUIRE(st->lower_levels_pending == 0, PHOTON_ERR_INVALID_ARG,
                 "%s: the lower levels of a pipelined step are still outstanding on this state: call photon_decode_join first", __func__);
  PHOTON_REQUIRE_PTR(st->k_cache);
  PHOTON_REQUIRE_PTR(st->v_cache);
  PHOTON_REQUIRE_PTR(st->x_top);
  PHOTON_REQUIRE(st->seq_len != nullptr, PHOTON_ERR_INVALID_ARG, "%s: state.seq_len is null", __func__);
  PHOTON_REQUIRE(c.L == 1 || (st->carry != nullptr && aligned16(st->carry)), PHOTON_ERR_INVALID_ARG,
                 "%s: state.carry must be a 16-byte aligned device pointer when L > 1", __func__);
  PHOTON_TRY(require_encoders(c, ew));
  for (int l = 2; l <= c.L; ++l) {
    PHOTON_REQUIRE(ew->x0[l - 1] != nullptr, PHOTON_ERR_INVALID_ARG, "%s: start latent of level %d missing", __func__, l);
    PHOTON_REQUIRE(w->conv_w[l - 1] && aligned16(w->conv_w[l - 1]) && w->conv_b[l - 1], PHOTON_ERR_INVALID_ARG,
                   "%s: converter of level %d missing or misaligned", __func__, l);
    PHOTON_TRY(require_module(c, w->dec[l - 1], "decoder", l));
  }
  if (hst != nullptr) {
    PHOTON_TRY(require_hier_state(c, hst));
    int64_t M = T;
    for (int l = 1; l < c.L; ++l) {
      M /= c.C[l - 1];
      PHOTON_REQUIRE(M <= hst->S_cap[l - 1], PHOTON_ERR_INVALID_ARG, "%s: %lld level-%d units do not fit its capacity %lld", __func__,
                     (long long)M, l, (long long)hst->S_cap[l - 1]);
    }
  }
  Ctx x;
  x.c = cfg; x.w = w; x.s = st; x.Bt = Bt; x.st = (hipStream_t)stream;
  x.p = make_plan(c, Bt, st->S_max);
  x.bf16 = (c.dt == PHOTON_BF16);
  x.overlap = false;
  x.ew = ew; x.hs = hst;
  x.o_h = x.p.h; x.o_attn = x.p.attn; x.o_qkv = x.p.qkv; x.o_qrot = x.p.qrot; x.o_act = x.p.act; x.o_many = x.p.many;
  PHOTON_REQUIRE(st->workspace != nullptr && aligned16(st->workspace) && st->workspace_bytes >= x.p.total, PHOTON_ERR_WORKSPACE,
                 "%s: state workspace of %zu bytes needed (got %zu)", __func__, x.p.total, st->workspace_bytes);
  x.base = reinterpret_cast<char*>(st->workspace);
  const PrefillPlan pp = make_prefill_plan(c, Bt, T);
  PHOTON_REQUIRE(workspace != nullptr && aligned16(workspace) && workspace_bytes >= pp.total, PHOTON_ERR_WORKSPACE,
                 "%s: workspace of %zu bytes needed (got %zu)", __func__, pp.total, workspace_bytes);
  int bar_next = 0;
  x.bar_next = &bar_next;
  Ctx e = x;                                               // same configuration and stream, the big buffers
  e.bar_next = nullptr;
  e.base = reinterpret_cast<char*>(workspace);
  e.o_h = pp.h; e.o_attn = pp.attn; e.o_qkv = pp.qkv; e.o_qrot = 0; e.o_act = pp.act; e.o_many = pp.many;
  e.p.many_K = pp.many_K;
  return prefill_impl(x, e, pp, *ew, tokens);
}

static int32_t decode_entry(const char* fn, const photon_config* cfg, const photon_weights* w, const photon_encoder_weights* ew,
                            photon_state* st, const photon_hier_state* hst, int32_t Bt, const int32_t* forced_tokens,
                            int32_t* out_tokens, const photon_trace* trace, void* stream) {
  PHOTON_REQUIRE(cfg && w && st, PHOTON_ERR_INVALID_ARG, "%s: cfg, w and st must not be null", fn);
  PHOTON_TRY(validate_config(cfg, Bt, st->S_max));
  const photon_config& c = *cfg;
  PHOTON_REQUIRE(out_tokens != nullptr, PHOTON_ERR_INVALID_ARG, "%s: out_tokens is null", fn);
  PHOTON_REQUIRE_PTR(st->k_cache);
  PHOTON_REQUIRE_PTR(st->v_cache);
  PHOTON_REQUIRE_PTR(st->x_top);
  PHOTON_REQUIRE(st->seq_len != nullptr, PHOTON_ERR_INVALID_ARG, "%s: state.seq_len is null", fn);
  PHOTON_REQUIRE(c.L == 1 || (st->carry != nullptr && aligned16(st->carry)), PHOTON_ERR_INVALID_ARG,
                 "%s: state.carry must be a 16-byte aligned device pointer when L > 1", fn);
  PHOTON_REQUIRE_PTR(w->E_dec);
  PHOTON_REQUIRE_PTR(w->W_lm);
  PHOTON_REQUIRE_PTR(w->chunker_w);
  PHOTON_TRY(require_module(c, w->top, "top", c.L));
  for (int l = 0; l < c.L; ++l) {
    PHOTON_REQUIRE(w->conv_w[l] && aligned16(w->conv_w[l]) && w->conv_b[l], PHOTON_ERR_INVALID_ARG,
                   "%s: converter of level %d missing or misaligned", fn, l + 1);
    PHOTON_TRY(require_module(c, w->dec[l], "decoder", l + 1));
  }
  if (hst != nullptr) {
    PHOTON_REQUIRE(ew != nullptr, PHOTON_ERR_INVALID_ARG, "%s: encoder-side weights are null", fn);
    PHOTON_TRY(require_encoders(c, ew));
    PHOTON_TRY(require_hier_state(c, hst));
  }
  Ctx x;
  x.c = cfg; x.w = w; x.s = st; x.Bt = Bt; x.st = (hipStream_t)stream;
  x.p = make_plan(c, Bt, st->S_max);
  x.bf16 = (c.dt == PHOTON_BF16);
  // the top-level update runs beside the lower levels when the caller lent a second stream and two events
  // (per-kernel timing wants one stream: concurrency would inflate the bracketed times)
  x.overlap = !g_profile_on && st->side_stream != nullptr && st->fork_event != nullptr && st->join_event != nullptr;
  PHOTON_REQUIRE(st->side_stream == nullptr || st->side_stream != stream, PHOTON_ERR_INVALID_ARG,
                 "%s: state.side_stream must differ from the stream of the call", fn);
  PHOTON_REQUIRE(st->pipeline == 0 || (hst == nullptr && st->side_stream != nullptr && st->fork_event != nullptr && st->join_event != nullptr &&
                                       st->free_event != nullptr),
                 PHOTON_ERR_INVALID_ARG, "%s: pipelined steps need side_stream, fork_event, join_event and free_event (recursive generation only)", fn);
  PHOTON_REQUIRE(st->pipeline != 0 || st->lower_levels_pending == 0, PHOTON_ERR_INVALID_ARG,
                 "%s: the lower levels of a pipelined step are still outstanding: call photon_decode_join first", fn);
  x.ew = ew; x.hs = hst;
  x.o_h = x.p.h; x.o_attn = x.p.attn; x.o_qkv = x.p.qkv; x.o_qrot = x.p.qrot; x.o_act = x.p.act; x.o_many = x.p.many;
  PHOTON_REQUIRE(st->workspace != nullptr && aligned16(st->workspace) && st->workspace_bytes >= x.p.total, PHOTON_ERR_WORKSPACE,
                 "%s: workspace of %zu bytes needed (got %zu)", fn, x.p.total, st->workspace_bytes);
  x.base = reinterpret_cast<char*>(st->workspace);
  int bar_next = 0;
  x.bar_next = &bar_next;
  return decode_step_impl(x, st, forced_tokens, out_tokens, trace);
}

extern "C" int32_t photon_set_persistent(int32_t on) {
  g_no_persistent = (on == 0);
  return PHOTON_OK;
}

extern "C" int32_t photon_persistent_trace(uint64_t* stamps) {
  persistent_module_set_stamps(reinterpret_cast<unsigned long long*>(stamps));
  return PHOTON_OK;
}

extern "C" int32_t photon_set_barrier_wait_limit(int64_t ticks) {
  clear_error();
  PHOTON_REQUIRE(ticks > 0, PHOTON_ERR_INVALID_ARG, "%s: ticks=%lld must be positive", __func__, (long long)ticks);
  persistent_module_set_spin_ticks(ticks);
  return PHOTON_OK;
}

extern "C" int32_t photon_decode_join(photon_state* st, void* stream) {
  clear_error();
  PHOTON_REQUIRE(st != nullptr, PHOTON_ERR_INVALID_ARG, "%s: st is null", __func__);
  if (st->lower_levels_pending == 0) return PHOTON_OK;
  PHOTON_REQUIRE(st->side_stream != nullptr && st->join_event != nullptr, PHOTON_ERR_INVALID_ARG, "%s: the state has no side stream", __func__);
  if (hipEventRecord((hipEvent_t)st->join_event, (hipStream_t)st->side_stream) != hipSuccess ||
      hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)st->join_event, 0) != hipSuccess)
    return fail(PHOTON_ERR_HIP, "%s: cannot join the lower levels", __func__);
  st->lower_levels_pending = 0;
  return PHOTON_OK;
}

extern "C" int32_t photon_decode_step(const photon_config* cfg, const photon_weights* w, photon_state* st, int32_t Bt,
                                      const int32_t* forced_tokens, int32_t* out_tokens, const photon_trace* trace,
                                      void* stream) {
  clear_error();
  return decode_entry(__func__, cfg, w, nullptr, st, nullptr, Bt, forced_tokens, out_tokens, trace, stream);
}

extern "C" int32_t photon_hiergen_step(const photon_config* cfg, const photon_weights* w, const photon_encoder_weights* ew,
                                       photon_state* st, const photon_hier_state* hst, int32_t Bt,
                                       const int32_t* forced_tokens, int32_t* out_tokens, const photon_trace* trace,
                                       void* stream) {
  clear_error();
  PHOTON_REQUIRE(hst != nullptr, PHOTON_ERR_INVALID_ARG, "%s: the lower-level streams are null", __func__);
  return decode_entry(__func__, cfg, w, ew, st, hst, Bt, forced_tokens, out_tokens, trace, stream);
}
