/*
 * photon.h -- C ABI of the MI355X (gfx950) implementation of the PHOTON
 * hierarchical decode hot path (arXiv 2512.20687).
 *
 * Notation follows the paper (Section 2.1, "Notation"): an L-level hierarchy,
 * level l groups C_l level-(l-1) units into one level-l unit; the converter of
 * level l expands one level-l vector into R_l conditioning vectors; the local
 * decoder of level l works on a window of W_l = R_l + C_l - 1 positions; all
 * levels share one width D = H * d_h.
 *
 * General rules for every entry point
 *  - Every pointer is a DEVICE pointer unless its comment says "host".
 *    Device pointers must be 16-byte aligned (the kernels use 128-bit accesses).
 *  - The library never allocates, frees or synchronises.  A call validates its
 *    arguments on the host, then only enqueues kernels on `stream` (a
 *    hipStream_t passed as void*; NULL is the default stream) and returns.
 *    Buffers must stay alive until the stream has run the work.
 *  - Return value: PHOTON_OK or a negative photon_status.  On error nothing has
 *    been enqueued (PHOTON_ERR_HIP excepted: a launch failed part-way) and
 *    photon_last_error() describes the problem (thread-local, host string).
 *  - dtype: PHOTON_F32 stores every tensor as IEEE fp32; PHOTON_BF16 stores
 *    matrices, embedding tables and K/V caches as bfloat16 (round to nearest
 *    even on store).  All arithmetic accumulates in fp32.
 *  - Linear maps are stored W[out, in] row-major (y = W x): the contraction
 *    index is contiguous.
 */
#ifndef PHOTON_H_
#define PHOTON_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define PHOTON_API __attribute__((visibility("default")))
#else
#define PHOTON_API
#endif

/* PHOTON_FP8_E4M3: 8-bit floating point (OCP E4M3: bias 7, no infinities, largest finite value 448), accepted only
 * as the storage type of a coarse K/V cache (photon_config.kv_dt, photon_coarse_decode_attn). */
typedef enum { PHOTON_F32 = 0, PHOTON_BF16 = 1, PHOTON_FP8_E4M3 = 2 } photon_dtype;

typedef enum {
  PHOTON_OK = 0,
  PHOTON_ERR_INVALID_ARG = -1, /* null/misaligned pointer, non-positive size, sizes that do not divide */
  PHOTON_ERR_UNSUPPORTED = -2, /* a size or dtype no kernel was compiled for */
  PHOTON_ERR_WORKSPACE = -3,   /* workspace missing or too small */
  PHOTON_ERR_HIP = -4          /* the HIP runtime refused a launch */
} photon_status;

enum { PHOTON_MAX_LEVELS = 4, PHOTON_MAX_WINDOW = 16 };

/* Library version: major*10000 + minor*100 + patch. */
PHOTON_API int32_t photon_version(void);

/* Host string describing the last error on the calling thread ("" if none). */
PHOTON_API const char* photon_last_error(void);

/* --------------------------------------------------------------------------
 * Context chunker (paper Eq. 4): fold C consecutive finer states into one
 * coarser state,
 *     out[r, :] = W_c * concat(x[r*C + 0, :], ..., x[r*C + C-1, :]) + bias .
 *   x     [rows*C, d_in]   dt   (read as [rows, C*d_in]: the concatenation is free)
 *   w     [d_out, C*d_in]  dt   or NULL: parameter-free concatenation (then
 *                               d_out must equal C*d_in; out is a copy of x)
 *   bias  [d_out]          fp32 or NULL
 *   out   [rows, d_out]    dt
 * bf16: fp32 accumulation on the matrix cores, one rounding on store.
 * bf16 requires C*d_in to be a multiple of 64 and d_out a multiple of 16;
 * fp32 requires C*d_in to be a multiple of 4.
 * rows == 0 is a no-op.
 * -------------------------------------------------------------------------- */
PHOTON_API int32_t photon_chunker_project(const void* x, const void* w, const float* bias, void* out,
                               int64_t rows, int32_t C, int32_t d_in, int32_t d_out,
                               photon_dtype dt, void* stream);

/* --------------------------------------------------------------------------
 * Coarsest-stream decode attention: the attention inside the STEP operator of
 * the top-level context encoder (paper Eq. 12-13, Appendix A.1).  One query
 * per (sequence, head) attends to the first seq_len[b] entries of that
 * stream's K/V cache (the entry appended by this step included):
 *     out[b,h,:] = softmax(scale * q[b,h,:] . K[b,h,0:seq_len[b],:]) V[b,h,0:seq_len[b],:]
 *   q        [Bt, H, d_h]          dt
 *   k_cache  [Bt, H, S_max, d_p]   dt   (each (b,h) stream contiguous)
 *   v_cache  [Bt, H, S_max, d_p]   dt
 *   seq_len  [Bt]                  int32, device; values in [0, S_max]; 0 gives zeros
 *   out      [Bt, H, d_h]          dt
 * d_h in [1, 128].  A cache row holds d_p = photon_kv_row_elems(d_h) elements:
 * d_h rounded up to 32, 64 or 128, so that rows are whole 64/128/256-byte
 * lines for the head sizes 52, 56 and 60 of the paper's models (Appendix,
 * tables "PHOTON (600M)" .. "(1.2B)") as well; columns d_h .. d_p-1 of every
 * row in use must hold zeros (the library's own cache writers do that).
 * The S axis is split over n_splits workgroups per
 * stream (0 = choose from Bt*H and S_max); partial softmax states are merged
 * in a fixed order, so the result is run-to-run deterministic for a given
 * n_splits.  dt PHOTON_FP8_E4M3: the caches hold E4M3 bytes (1 byte per element, same row length d_p), q and
 * out are fp32.  n_splits > 1 needs a workspace of
 * photon_coarse_decode_attn_workspace_bytes() bytes (contents need no
 * initialisation; calls that share a workspace must be stream-ordered).
 * -------------------------------------------------------------------------- */
PHOTON_API int32_t photon_kv_row_elems(int32_t d_h);   /* 0 when d_h is outside [1, 128] */
PHOTON_API size_t photon_coarse_decode_attn_workspace_bytes(int32_t Bt, int32_t H, int32_t d_h, int32_t n_splits);
PHOTON_API int32_t photon_coarse_decode_attn_auto_splits(int32_t Bt, int32_t H, int64_t S_max);
PHOTON_API int32_t photon_coarse_decode_attn(const void* q, const void* k_cache, const void* v_cache,
                                  const int32_t* seq_len, void* out,
                                  int32_t Bt, int32_t H, int32_t d_h, int64_t S_max, float scale,
                                  int32_t n_splits, void* workspace, size_t workspace_bytes,
                                  photon_dtype dt, void* stream);

/* --------------------------------------------------------------------------
 * photon_coarse_decode_attn for callers that cannot allocate device memory and
 * have no workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * photon_coarse_decode_attn, but the split partials go to a scratch array built
 * into the library (photon_coarse_decode_attn_static_capacity() bytes = 4 MiB,
 * held by every GPU the library runs on until the process ends) instead of a
 * caller workspace.  Nothing is allocated or freed, here or in the runtime.
 * A shape whose partials (photon_coarse_decode_attn_workspace_bytes()) exceed
 * the capacity is rejected with PHOTON_ERR_WORKSPACE.  All calls on one GPU
 * share that GPU's array: calls must be stream-ordered; calls that overlap on
 * one GPU (two streams, two host threads) race on the partials.
 * -------------------------------------------------------------------------- */
PHOTON_API size_t photon_coarse_decode_attn_static_capacity(void);
PHOTON_API int32_t photon_coarse_decode_attn_static(const void* q, const void* k_cache, const void* v_cache,
                                         const int32_t* seq_len, void* out,
                                         int32_t Bt, int32_t H, int32_t d_h, int64_t S_max, float scale,
                                         int32_t n_splits, photon_dtype dt, void* stream);

/* --------------------------------------------------------------------------
 * Chunk-local causal attention of the local decoders (paper Eq. 6-7): every
 * chunk is an independent window of W positions; query i (0 <= i < q_len) sits
 * at window position q_pos + i and attends to keys 0 .. q_pos + i of its own
 * chunk only.
 *   q    [n_chunks, q_len, H, d_h]   dt   (token-major, as a QKV projection writes it)
 *   k,v  [n_chunks, W,     H, d_h]   dt   (the chunk's local cache / K,V tile)
 *   out  [n_chunks, q_len, H, d_h]   dt
 * q_len == W, q_pos == 0: the whole W x W causal tile (teacher-forced / prefill).
 * q_len == 1: one decode sub-step at window position q_pos.
 * Requires q_pos + q_len <= W <= PHOTON_MAX_WINDOW; d_h <= 128 and a multiple
 * of 4 (fp32) or 8 (bf16): a head row is read in 16-byte pieces.
 * n_chunks == 0 is a no-op.
 * -------------------------------------------------------------------------- */
PHOTON_API int32_t photon_chunk_local_attn(const void* q, const void* k, const void* v, void* out,
                                int64_t n_chunks, int32_t W, int32_t q_len, int32_t q_pos,
                                int32_t H, int32_t d_h, float scale, photon_dtype dt, void* stream);

/* --------------------------------------------------------------------------
 * Causal self-attention of a context encoder over whole sequences: the
 * prefill form of the encoder (paper Eq. 3; cost O(M_l^2) per level, Section
 * 2.3.1).  Query i of sequence b attends to keys 0 .. i of the same sequence
 * and head; q and k receive the rotary encoding at positions 0 .. M-1.
 *   qkv  [Bt*M, 3*H*d_h]  fp32, device: rows b*M + i, columns [q | k | v],
 *                         head h at columns h*d_h .. of each third
 *   out  [Bt*M, H*d_h]    fp32, device
 *   k_cache, v_cache      both NULL, or [Bt][H][S_max][photon_kv_row_elems(d_h)]
 *                         in dt (device): receive the rotated keys and the
 *                         values of positions 0 .. M-1 (S_max >= M), zeros in
 *                         the columns past d_h, i.e. the coarse cache a decode
 *                         step continues from
 *   workspace             photon_encoder_attn_workspace_bytes(...) bytes,
 *                         device, caller-owned (0 bytes for fp32)
 * dt PHOTON_BF16: matrix-core kernel, d_h a multiple of 4 up to 64 (operand
 * rows are zero-padded to 64); q, k, v and the probabilities enter the
 * matrix cores as fp16 (11 significant bits, values saturated at 65504),
 * accumulation in fp32.
 * dt PHOTON_F32: fp32 vector kernel, d_h a multiple of 4 in [16, 64].
 * Bt*H <= 65535.  Bt == 0 or M == 0 is a no-op.  Nothing is allocated or
 * synchronised; errors are reported by status + photon_last_error().
 * -------------------------------------------------------------------------- */
PHOTON_API size_t photon_encoder_attn_workspace_bytes(int32_t Bt, int64_t M, int32_t H, int32_t d_h, photon_dtype dt);
PHOTON_API int32_t photon_encoder_attn(const float* qkv, float* out, int32_t Bt, int64_t M, int32_t H, int32_t d_h,
                                       float rope_theta, float scale, void* k_cache, void* v_cache, int64_t S_max,
                                       void* workspace, size_t workspace_bytes, photon_dtype dt, void* stream);


/* --------------------------------------------------------------------------
 * Few-row linear map with fused pre-norm and epilogue: the weight-streaming
 * building block of the decode step (every projection of the LLaMA blocks,
 * the converters, the LM head, the chunker at decode shapes).
 *     y[m, :] = rmsnorm(x[m, :]; gain, rms_eps) * W^T      (gain == NULL: y = x * W^T)
 *     epilogue 0 (plain)   : out = y + bias
 *     epilogue 1 (residual): out = res + y + bias          (out may alias res)
 *     epilogue 2 (SwiGLU)  : out = silu(y[:, 0:N]) * y[:, N:2N]   (w has 2N rows: gate, then up)
 *   x    [M, K]          fp32
 *   w    [N or 2N, K]    dt
 *   gain [K], bias [N]   fp32 or NULL;   res [M, N] fp32 (epilogue 1)
 *   out  [M, N]          fp32
 * bf16 needs K % 64 == 0 and N % 16 == 0; fp32 needs K % 4 == 0.
 * With dt = bf16 two flags may be added to `epilogue` (the decode step keeps the
 * feed-forward's hidden rows, Eq. 6-7's SwiGLU product, in bf16 this way):
 *   PHOTON_LINEAR_OUT_BF16: out holds bf16 values (the result rounded to nearest even);
 *   PHOTON_LINEAR_X_BF16  : x holds bf16 values, which enter the matrix cores as they are;
 *                           needs gain == NULL; with more than 16 rows a workgroup takes two
 *                           or four row tiles of 16, so the matrix is streamed once per 32-64 rows.
 * One kernel, no workspace; run-to-run deterministic.
 * -------------------------------------------------------------------------- */
#define PHOTON_LINEAR_X_BF16 0x10
#define PHOTON_LINEAR_OUT_BF16 0x20
PHOTON_API int32_t photon_linear(const void* x, const void* w, const float* gain, float rms_eps, const float* bias,
                                 const float* res, void* out, int32_t M, int32_t N, int32_t K, int32_t epilogue,
                                 photon_dtype dt, void* stream);

/* --------------------------------------------------------------------------
 * One recursive-generation step g -> g+1 for Bt sequences (paper Section
 * 2.3.3 steps (i)-(iii); Appendix A, Definition 2):
 *   (i)  top-down: the level-L local decoder expands X^(L)_g into C_L new
 *        level-(L-1) units; every lower level l decodes one chunk per new
 *        level-l unit, all chunks of a level batched, each chunk conditioned on
 *        the previous level-l unit (the carry for the first one); level 1 emits
 *        the prod(C) tokens of the next meta-context (greedy argmax, lowest
 *        index on ties, or the caller's forced tokens) and feeds back their
 *        decoder-side embeddings;
 *   (ii) the top chunker (Eq. 4) folds the C_L new level-(L-1) units into A-hat;
 *   (iii) STEP (Eq. 13): every layer of the top encoder appends one K/V entry
 *        and attends over the whole coarse cache; X^(L)_{g+1} is stored.
 * Block structure: pre-RMSNorm LLaMA blocks (rotary positions local to each
 * module, SwiGLU feed-forward unless d_ff == 0), one final RMSNorm per module.
 *
 * Host structs below hold DEVICE pointers.  Matrices/tables are `dt`; gains,
 * biases and all state vectors are fp32.  Arithmetic with dt = bf16: residual
 * stream, norms, softmax and every accumulation in fp32; the feed-forward's
 * hidden rows and the attention rows of the local decoders and of the prefill
 * are kept in bf16, and so are the rows entering a projection once
 * a pass holds 17 rows or more (below that they enter as a bf16 head plus a
 * bf16 remainder, i.e. with fp32 accuracy).
 * -------------------------------------------------------------------------- */
typedef struct photon_config {
  int32_t L;                     /* levels, 1..PHOTON_MAX_LEVELS */
  int32_t C[PHOTON_MAX_LEVELS];  /* C[l-1] = C_l >= 1 */
  int32_t R[PHOTON_MAX_LEVELS];  /* R[l-1] = R_l >= 1;  R_l + C_l - 1 <= PHOTON_MAX_WINDOW */
  int32_t D, H, d_h;             /* D == H * d_h; d_h a multiple of 4, at most 128 (prefill: at most 64) */
  int32_t n_layers;              /* blocks per module */
  int32_t d_ff;                  /* SwiGLU width, 0 = attention-only blocks */
  int32_t vocab;
  photon_dtype dt;               /* storage of matrices and tables */
  photon_dtype kv_dt;            /* storage of the coarse K/V caches (state and hierarchical state): equal to dt, or
                                    PHOTON_FP8_E4M3 with dt == PHOTON_BF16: entries are rounded to nearest even from their
                                    fp32 values and saturate at +-448; no scale factor (a variant beyond the paper) */
  float rms_eps;
  float rope_theta;              /* 0 disables the rotary encoding */
} photon_config;

typedef struct photon_layer_weights {
  const float* g1;   /* [D]      pre-attention norm gain */
  const void* wqkv;  /* [3D, D]  rows: Wq, then Wk, then Wv */
  const void* wo;    /* [D, D] */
  const float* g2;   /* [D]      pre-MLP norm gain       (d_ff > 0) */
  const void* wgu;   /* [2F, D]  rows: Wgate, then Wup   (d_ff > 0) */
  const void* wd;    /* [D, F]                           (d_ff > 0) */
} photon_layer_weights;

typedef struct photon_module_weights {
  const photon_layer_weights* layers; /* HOST array of n_layers entries */
  const float* g_final;               /* [D] */
} photon_module_weights;

typedef struct photon_weights {
  const void* E_dec;        /* [vocab, D] decoder-side token embedding */
  const void* W_lm;         /* [vocab, D] vocabulary projection */
  const void* chunker_w;    /* [D, C_L*D] top-level chunker */
  const float* chunker_b;   /* [D] or NULL */
  photon_module_weights top;                      /* top-level context encoder F^(L) */
  const void* conv_w[PHOTON_MAX_LEVELS];          /* conv_w[l-1]: [R_l*D, D] converter of level l */
  const float* conv_b[PHOTON_MAX_LEVELS];         /* conv_b[l-1]: [R_l*D] */
  photon_module_weights dec[PHOTON_MAX_LEVELS];   /* dec[l-1]: local decoder G^(l) */
} photon_weights;

typedef struct photon_state {
  void* k_cache;        /* [n_layers, Bt, H, S_max, photon_kv_row_elems(d_h)] kv_dt : KV^(L) */
  void* v_cache;
  int32_t* seq_len;     /* [Bt] entries cached per sequence; the step adds 1.  Must be < S_max on entry (else see status). */
  float* x_top;         /* [Bt, D]       X^(L)_g, replaced by X^(L)_{g+1} */
  float* carry;         /* [L-1, Bt, D]  carry[l-1] = last reconstructed level-l unit, updated */
  int64_t S_max;
  void* workspace;      /* photon_decode_step_workspace_bytes(); contents need no initialisation */
  size_t workspace_bytes;
  int32_t* status;      /* NULL, or a device word the step ORs photon_step_status bits into (never cleared by the library) */
  void* side_stream;    /* NULL, or a hipStream_t other than the call's stream, owned by the caller and used by one state
                           at a time: with fork_event and join_event given, the levels below the top of an L >= 2 model
                           run on it beside the top-level update (ii)-(iii) and are joined back before the call's work
                           ends (unless pipeline is set) */
  void* fork_event;     /* hipEvent_t (timing may be disabled), recorded and waited on by the step; NULL: no side stream */
  void* join_event;     /* hipEvent_t, likewise */
  void* free_event;     /* hipEvent_t, needed only for pipelined steps */
  int32_t pipeline;     /* 0: every call joins the side stream before its work ends.  1 (needs side_stream and the three
                           events; recursive generation only): the levels below the top, which turn the top-level
                           decoder's output into this step's tokens and feed nothing back into the recurrence
                           X^(L)_g -> X^(L)_{g+1}, are left running on the side stream when the call returns, so that
                           they also run beside the NEXT step's top level.  out_tokens (and the trace buffers of the
                           lower levels) of such a step are complete only after photon_decode_join(); successive
                           pipelined steps must be given distinct out_tokens buffers if all are to be read */
  int32_t lower_levels_pending;   /* maintained by the library: non-zero between a pipelined step and the join.  Set to 0 once */
} photon_state;

/* Bits of photon_state.status. */
typedef enum {
  PHOTON_STATUS_CACHE_FULL = 1,       /* a sequence had seq_len == S_max on entry: its count stays, its new K/V entry
                                         overwrites the last one and its results of the step are not valid */
  PHOTON_STATUS_BARRIER_TIMEOUT = 2   /* a grid-barrier wait of a persistent launch ran out (see photon_set_persistent):
                                         every workgroup left the kernel; the step's results are not valid */
} photon_step_status;

/* Optional outputs for inspection (each pointer may be NULL). */
typedef struct photon_trace {
  float* logits;                        /* [Bt, prod(C), vocab] */
  float* new_units[PHOTON_MAX_LEVELS];  /* new_units[l]: [Bt, C_L*...*C_{l+1}, D] new level-l units, l = 0..L-1 */
  float* a_hat;                         /* [Bt, D] chunker output */
} photon_trace;

PHOTON_API size_t photon_decode_step_workspace_bytes(const photon_config* cfg, int32_t Bt, int64_t S_max);

/* forced_tokens: device int32 [Bt, prod(C)] or NULL; out_tokens: device int32
 * [Bt, prod(C)].  cfg, w, st and trace are host structs, read during the call
 * only.  All work is enqueued on `stream` (and, between a fork and a join that
 * both happen inside the call, on st->side_stream when the caller lends one);
 * tokens stay on the device.  The library creates no stream or event, so any
 * call may be made under stream capture. */
PHOTON_API int32_t photon_decode_step(const photon_config* cfg, const photon_weights* w, photon_state* st,
                                      int32_t Bt, const int32_t* forced_tokens, int32_t* out_tokens,
                                      const photon_trace* trace, void* stream);

/* Makes `stream` wait for the lower levels that pipelined steps (photon_state.pipeline) left running on the side
 * stream; afterwards, in stream order, every out_tokens buffer of those steps is complete.  A no-op when nothing is
 * outstanding.  Must be called (under stream capture: inside the same capture) before the state is used by anything
 * but further pipelined steps. */
PHOTON_API int32_t photon_decode_join(photon_state* st, void* stream);

/* Schedule of a local decoder's module pass (all blocks of G^(l) on the rows of one decode sub-step, Eq. 6-7) when
 * it holds at most 16 rows of a bf16 configuration: on != 0 (the default) runs it as ONE persistent launch, one
 * workgroup per compute unit, whose phases meet at grid barriers (bounded waits; needs head size 64 or 128, a window
 * of at most 8 positions, at most 16 blocks per module and one of the compiled width classes, else the separate
 * launches are used); on == 0 always uses separate launches.  Process-wide; results agree to the last bit.
 * At most two persistent launches can be resident on a GPU at a time: steps of more than two states issued
 * concurrently on different streams serialise on the barrier waits (and fail with the error word set after 10 s). */
PHOTON_API int32_t photon_set_persistent(int32_t on);

/* Measurement aid for benchmarks.  While `stamps` (device memory, room for 16 * 16 values of 8 bytes) is set, workgroup
 * 0 of every persistent launch notes the device's constant 100 MHz clock at the milestones of every phase, 14 per
 * block in this order: QKV contraction done; its epilogue and stores issued; barrier passed; attention done; barrier;
 * O contraction; epilogue; barrier; gate/up contraction; epilogue; barrier; down contraction; epilogue; barrier (the
 * last block has no final barrier).  NULL switches it off.  Process-wide; the buffer is the caller's. */
PHOTON_API int32_t photon_persistent_trace(uint64_t* stamps);

/* Bound of a grid-barrier wait inside a persistent launch, in ticks of the device's constant 100 MHz clock (default
 * 10^9 = 10 s; process-wide).  A wait that runs out sets PHOTON_STATUS_BARRIER_TIMEOUT and makes every workgroup
 * leave the kernel normally.  Meant for tests of that path (a limit of a few ticks makes the first real wait run out). */
PHOTON_API int32_t photon_set_barrier_wait_limit(int64_t ticks);

/* --------------------------------------------------------------------------
 * Hierarchical prefill of a batch of prompts (paper Section 2.3.3, first
 * paragraph; encoder Eq. 3-4): embeds the tokens, runs chunker + encoder
 * module of every level bottom-up over the whole prompt (whole-sequence causal
 * attention, see photon_encoder_attn), and leaves in `st` exactly what a decode
 * step continues from: the top-level K/V cache of all M_L = T / prod(C) units,
 * seq_len = M_L, x_top = X^(L)_{M_L}, and for every level l < L the carry =
 * last reconstructed level-l unit, obtained by a teacher-forced decode of the
 * last chunk of every level l >= 2 (conditioned on the previous level-l unit,
 * or on the level's learned start latent when the prompt holds a single one).
 *   tokens  device int32 [Bt, T], T a positive multiple of prod(C),
 *           T / prod(C) <= st->S_max (strictly less if decode steps follow)
 *   ew      encoder-side parameters (host struct of device pointers)
 *   st      as for photon_decode_step, its workspace included (the carry
 *           decode runs on it); cache rows beyond M_L are left untouched
 *   workspace  photon_prefill_workspace_bytes(cfg, Bt, T) bytes, device,
 *           caller-owned, no initialisation needed
 * Levels >= 2 need C_l >= 2.  Everything is enqueued on `stream`.
 * -------------------------------------------------------------------------- */
typedef struct photon_encoder_weights {
  const void* E_enc;                            /* [vocab, D] dt: encoder-side embedding table ([vocab, D / C_1] when
                                                   chunker_w[0] is NULL) */
  const void* chunker_w[PHOTON_MAX_LEVELS];     /* index l-1: chunker of level l, [D, C_l * D] dt.  chunker_w[0] may be
                                                   NULL when L >= 2: the parameter-free concatenation of the paper's
                                                   models (Appendix tables, "Ctx Chunker (block=4, concatenate)"):
                                                   A^(1)_g is the C_1 embeddings of its tokens side by side */
  const float* chunker_b[PHOTON_MAX_LEVELS];    /* [D] fp32 or NULL */
  photon_module_weights enc[PHOTON_MAX_LEVELS]; /* index l-1: encoder module of level l (enc[L-1] = photon_weights.top) */
  const float* x0[PHOTON_MAX_LEVELS];           /* index l-1: start latent of the level-l decoder, [D] fp32 */
} photon_encoder_weights;

/* Encoder streams of the levels below the top, kept only by hierarchical
 * generation (Appendix A, Definition 1): index l-1 for level l = 1 .. L-1. */
typedef struct photon_hier_state {
  void* k_cache[PHOTON_MAX_LEVELS];     /* [n_layers, Bt, H, S_cap[l-1], photon_kv_row_elems(d_h)] kv_dt: K/V of the level-l encoder */
  void* v_cache[PHOTON_MAX_LEVELS];
  int32_t* seq_len[PHOTON_MAX_LEVELS];  /* [Bt] units cached per sequence at level l */
  int64_t S_cap[PHOTON_MAX_LEVELS];     /* capacity per sequence; a step appends prod(C_{l+1..L}) units */
} photon_hier_state;

/* hst: NULL for recursive generation; else the lower-level streams are filled
 * too (all M_l units of every level l < L, seq_len = M_l; needs M_l <= S_cap). */
PHOTON_API size_t photon_prefill_workspace_bytes(const photon_config* cfg, int32_t Bt, int64_t T);
PHOTON_API int32_t photon_prefill(const photon_config* cfg, const photon_weights* w, const photon_encoder_weights* ew,
                                  const photon_state* st, const photon_hier_state* hst, int32_t Bt,
                                  const int32_t* tokens, int64_t T, void* workspace, size_t workspace_bytes, void* stream);

/* --------------------------------------------------------------------------
 * One step of hierarchical generation (Appendix A, Definition 1), the schedule
 * recursive generation is compared with (Section 2.3.3, Table 2): (1) the same
 * top-down decode as photon_decode_step; (2) the generated tokens are
 * re-encoded bottom-up: every level l < L advances its own stream by
 * prod(C_{l+1..L}) units, one STEP (Eq. 12-13) per unit on that level's cache;
 * (3) the top chunker (Eq. 4) summarises the ENCODER-side level-(L-1) block and
 * the top stream advances.  Arguments as for photon_decode_step, plus the
 * encoder-side weights and the lower-level streams (every level must have room
 * for the units of one step).  trace->a_hat receives the encoder-side summary.
 * Runs on `stream` only.
 * -------------------------------------------------------------------------- */
PHOTON_API int32_t photon_hiergen_step(const photon_config* cfg, const photon_weights* w, const photon_encoder_weights* ew,
                                       photon_state* st, const photon_hier_state* hst, int32_t Bt,
                                       const int32_t* forced_tokens, int32_t* out_tokens, const photon_trace* trace,
                                       void* stream);

/* --------------------------------------------------------------------------
 * Bandwidth probe for benchmarks: a trivial kernel that reads `bytes` bytes of
 * `buf` once with 128-bit non-temporal loads (2048 workgroups, grid-stride) and discards
 * them.  Timing it gives the streaming-read ceiling of the machine, which the
 * attention kernels' GB/s can be set against.  sink: 4 writable device bytes.
 * -------------------------------------------------------------------------- */
PHOTON_API int32_t photon_hbm_read_probe(const void* buf, size_t bytes, void* sink, void* stream);

/* --------------------------------------------------------------------------
 * Matrix-core probe for benchmarks: 256 workgroups of 4 waves, each wave
 * issuing iters x 16 independent bf16 MFMA 32x32x16 on register operands, no
 * memory traffic.  Timing it gives the rate the matrix cores sustain on this
 * machine (the clock under matrix load depends on the operand values:
 * random_operands != 0 uses values spread like N(0,1) data, 0 small constants),
 * which the MFMA kernels' TFLOP/s can be set against.  Returns the number of
 * floating-point operations the launch performs (0.0 on error).
 * sink: 4 writable device bytes.
 * -------------------------------------------------------------------------- */
PHOTON_API double photon_mfma_probe(int32_t iters, int32_t random_operands, void* sink, void* stream);

/* --------------------------------------------------------------------------
 * Per-kernel timing for benchmarks.  While enabled, every kernel launch of the
 * library carries a pair of HIP events attached to the dispatch itself (start
 * and end of the kernel as the command processor stamps them, on the launch
 * stream); this allocates events (at most 65536 pairs between two resets, later
 * launches go untimed) and must not be used under stream capture.
 * Kernels are grouped in classes 0 .. photon_profile_num_classes()-1, named by
 * photon_profile_class_name().  photon_profile_get() waits for the recorded
 * events of a class and returns the launch count and the summed elapsed
 * milliseconds; photon_profile_reset() drops all records.  While enabled,
 * photon_decode_step keeps all its work on the caller's stream (no side stream).
 * -------------------------------------------------------------------------- */
PHOTON_API int32_t photon_profile_enable(int32_t on);
PHOTON_API int32_t photon_profile_reset(void);
PHOTON_API int32_t photon_profile_num_classes(void);
PHOTON_API const char* photon_profile_class_name(int32_t cls);
PHOTON_API int32_t photon_profile_get(int32_t cls, int64_t* launches, double* total_ms);

#ifdef __cplusplus
}
#endif
#endif /* PHOTON_H_ */
