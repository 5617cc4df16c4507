/*
 * tandem.h - C ABI of the MI355X (gfx950) Tandem Transformer hot path.
 *
 * Paper: "Tandem Transformers for Inference Efficient LLMs", Sec. 3 (Eq. (1), Eq. (2)),
 * Sec. 3.1 (Tandem + SPEED).  Notation follows the paper: M_L / M_S are the primary
 * (large) and secondary (small) model, gamma the block length, l(j) the layer assignment,
 * FF_Tandem the map from M_L's width d_L to M_S's width d_S.
 *
 * General conventions
 *   - Every pointer named "device" is GPU memory owned by the caller; the library never
 *     allocates or frees device memory, never synchronises a stream or the device, and keeps
 *     no mutable global state beyond one-time, thread-safe kernel attribute set-up (and the scratch array of
 *     tandem_draft_attn_static, which is part of the library image).  Descriptor
 *     structs and the pointer arrays inside them are host memory, read during the call only
 *     (the model handle copies what it needs).
 *   - All entry points enqueue work on the given HIP stream (a hipStream_t passed as
 *     void*, NULL = default stream) and return without synchronising.
 *   - Return value: a tandem_status.  All argument checks happen on the host before any
 *     launch; on error nothing has been enqueued.  Launch failures map to TANDEM_ERR_HIP.
 *   - Tensors are dense, row-major, last index fastest.  Linear maps are y = W x + b with
 *     W stored [out_features, in_features].
 *   - dtype TANDEM_BF16: bf16 storage, fp32 scores / softmax / accumulation, bf16 results.
 *     dtype TANDEM_F32: fp32 everywhere (correctness path for small models, not tuned).
 *   - Per-sequence lengths live in device memory (int32).  Kernels clamp them to the
 *     capacities in the descriptor, so a corrupt length cannot cause an out-of-bounds read.
 *   - Results are deterministic: identical inputs and shapes give bit-identical outputs.
 */
#ifndef TANDEM_H
#define TANDEM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#pragma GCC visibility push(default)

typedef enum {
  TANDEM_OK = 0,
  TANDEM_ERR_NULL = 1,        /* a required pointer is NULL                         */
  TANDEM_ERR_SHAPE = 2,       /* a size is non-positive, inconsistent or over limit */
  TANDEM_ERR_UNSUPPORTED = 3, /* a valid request this build has no kernel for       */
  TANDEM_ERR_WORKSPACE = 4,   /* ws_bytes is smaller than the *_workspace() answer  */
  TANDEM_ERR_HIP = 5          /* the HIP runtime reported an error                  */
} tandem_status;

typedef enum { TANDEM_F32 = 0, TANDEM_BF16 = 1 } tandem_dtype;
typedef enum { TANDEM_ACT_NONE = 0, TANDEM_ACT_GELU = 1 /* 0.5 x (1 + erf(x / sqrt 2)); the bf16 kernels evaluate erf to 1.5e-7 */, TANDEM_ACT_RELU = 2 } tandem_act;

#define TANDEM_MAX_QLEN 32 /* most query rows per sequence in one block-mode pass */
#define TANDEM_MAX_PREFILL 128 /* most prompt tokens per sequence in one tandem_prefill call */
#define TANDEM_MAX_SHARED_ROWS 256 /* most samples * q_len per prompt in tandem_block_attn_shared */

/* Shape of one attention layer's caches.
 *   caches:            [B, Hkv, T_max, dh]      (large K/V, or the large-derived K_hat/V_hat)
 *   own-block scratch: [B, Hkv, gamma_max, dh]  (K/V the small model computed for the current block)
 * Hq must be a multiple of Hkv; G = Hq/Hkv query heads share a KV head and must be 1, 2, 4 or 8
 * (other group sizes return TANDEM_ERR_UNSUPPORTED).
 * dh is 64 or 128.  scale is the score multiplier, normally 1/sqrt(dh). */
typedef struct {
  int32_t B, Hq, Hkv, dh;
  int64_t T_max;
  int32_t gamma_max;
  float scale;
  int32_t dtype; /* tandem_dtype */
} tandem_attn_desc;

/* FF_Tandem of one small layer (Eq. (2), first line).
 *   d_hidden == 0: linear form  y_hat = W1 x + b1,            W1 [d_S, d_L]   (the paper's experiments)
 *   d_hidden  > 0: MLP form     y_hat = W2 act(W1 x + b1) + b2, W1 [d_hidden, d_L], W2 [d_S, d_hidden]
 * Weights and biases are device pointers in `dtype`; b1 / b2 may be NULL (no bias). */
typedef struct {
  int32_t d_L, d_hidden, d_S;
  int32_t act;   /* tandem_act, ignored when d_hidden == 0 */
  int32_t dtype; /* tandem_dtype */
  const void *W1, *b1, *W2, *b2;
  const void *W1p, *W2p; /* optional: W1 / W2 in the packed layout written by tandem_pack_weight (device, same
                            dtype and shape), or NULL.  Used instead of W1 / W2 when the row count allows. */
} tandem_ff_desc;

/* ---- workspace sizes (bytes of device scratch a call needs; 256-byte aligned base) ---- */
size_t tandem_project_workspace(const tandem_ff_desc *ff, int64_t M);
size_t tandem_block_attn_workspace(const tandem_attn_desc *a, int32_t q_len);
size_t tandem_draft_attn_workspace(const tandem_attn_desc *a);

/* Packed weight layout (a choice of this library, not of the paper: the products of Eq. (1) / Eq. (2)
 * are unchanged, only the order of W's elements in memory).  W[N, K] row-major, bf16, is cut into
 * tiles of 32 rows x 64 columns; tile (nb, kb) starts at element (nb * (K / 64) + kb) * 2048 and holds,
 * at element ((j * 64 + 32 * h + c) * 8 + e), W[32 * nb + c][64 * kb + 32 * h + 8 * j + e]
 * (j < 4, h < 2, c < 32, e < 8).  tandem_packed_weight_bytes: size of the packed copy, 0 when the
 * shape or dtype cannot be packed (needs bf16, N % 128 == 0, K % 256 == 0).  tandem_pack_weight
 * writes it (W, Wp: device, 16-byte aligned, not overlapping; enqueued on hip_stream). */
size_t tandem_packed_weight_bytes(int64_t N, int64_t K, int32_t dtype);
int tandem_pack_weight(const void *W, int64_t N, int64_t K, int32_t dtype, void *Wp, void *hip_stream);

/* FF_Tandem: y_hat[M, d_S] = FF_Tandem(x[M, d_L])  (Eq. (2), first line; Sec. 1 "projection
 * layer").  x, y_hat: device, dtype ff->dtype.  M >= 1 rows (the gamma new rows of every
 * sequence at decode time, whole prompts at prefill time).  ws: device scratch of at least
 * tandem_project_workspace(ff, M) bytes (holds the hidden activations and split partials). */
int tandem_project(const tandem_ff_desc *ff, const void *x, void *y_hat, int64_t M, void *ws, size_t ws_bytes,
                   void *hip_stream);

/* Large-model block-mode attention (Sec. 1 step 3; Sec. 3 "Inference"; Eq. (1) restricted to
 * the q_len new rows; the SPEED verifier of Sec. 3.1).  For sequence b the K/V rows of the
 * q_len new tokens are already in the caches at [n_prefix[b], n_prefix[b] + q_len).  Query
 * row r of head h attends cache rows 0 .. n_prefix[b] + r inclusive of KV head h / G.
 *   q, out   device [B, q_len, Hq, dh]      k_cache, v_cache  device [B, Hkv, T_max, dh]
 *   n_prefix device int32 [B], requires n_prefix[b] + q_len <= T_max (clamped otherwise)
 *   1 <= q_len <= TANDEM_MAX_QLEN.  Reads the caches only; writes out and ws only.
 * Placement hint (throughput only): a workgroup streams the K and the V rows of one (sequence, KV head) side by side.
 * Where such a region (T_max * dh * element size) is a multiple of 2 MB, give v_cache a base address 1 MB out of
 * phase with k_cache's modulo 2 MB; measured at B = 32, 8 KV heads, 8192 rows of 128: 178 instead of 183 us. */
int tandem_block_attn(const tandem_attn_desc *a, const void *q, const void *k_cache, const void *v_cache,
                      const int32_t *n_prefix, int32_t q_len, void *out, void *ws, size_t ws_bytes, void *hip_stream);

/* Block-mode attention when several samples continue one prompt (the num-samples > 1 setting of Sec. 3.1,
 * measured with 4 samples in the latency evaluation of Sec. 4; the footnote of Sec. 3.1 notes that more samples
 * per prompt raise the efficiency of the attention layer too - this is where that comes from).  The prompt's
 * K/V rows are stored once per prompt and read once per prompt for all samples' query rows; each sample keeps
 * only the rows generated after the prompt.  The result equals tandem_block_attn on per-sample caches that
 * hold a copy of the prompt rows followed by the sample's own rows.  Sample s of prompt b is sequence
 * i = b * samples + s.  Query row r of sequence i attends, in ONE softmax,
 *   k_shared/v_shared[b, h/G, 0 : n_shared[b]]  and  k_own/v_own[i, h/G, 0 : n_own[i] + r + 1]
 * (the q_len new rows of sequence i are already in place at [n_own[i], n_own[i] + q_len)).
 *   q, out    device [B, samples, q_len, Hq, dh]     (B = a->B prompts)
 *   k_shared, v_shared device [B, Hkv, a->T_max, dh];  n_shared device int32 [B], clamped to [0, a->T_max]
 *   k_own, v_own       device [B * samples, Hkv, T_own, dh];  n_own device int32 [B * samples], clamped to
 *                      [0, T_own - q_len]
 *   1 <= q_len <= TANDEM_MAX_QLEN, samples * q_len <= TANDEM_MAX_SHARED_ROWS, B * samples <= 65535.
 * ws: device scratch of at least tandem_block_attn_shared_workspace(...) bytes, always needed (the two key
 * segments are merged through it).  Reads the caches only; writes out and ws only. */
size_t tandem_block_attn_shared_workspace(const tandem_attn_desc *a, int32_t samples, int64_t T_own, int32_t q_len);
int tandem_block_attn_shared(const tandem_attn_desc *a, int32_t samples, int64_t T_own, const void *q,
                             const void *k_shared, const void *v_shared, const int32_t *n_shared, const void *k_own,
                             const void *v_own, const int32_t *n_own, int32_t q_len, void *out, void *ws,
                             size_t ws_bytes, void *hip_stream);

/* tandem_draft_attn when several samples continue one prompt (Sec. 3.1, num-samples): the prompt's Khat/Vhat rows
 * are stored and read once per prompt for the queries of all its samples.  Sample s of prompt b is sequence
 * i = b * samples + s; its query attends, in ONE softmax,
 *   k_hat_shared/v_hat_shared[b, h/G, 0 : n_shared[b])   the prompt's rows (derived from M_L)
 *   k_hat_own/v_hat_own[i, h/G, 0 : n_own[i])            rows of the sample's completed blocks after the prompt
 *   k_cur/v_cur[i, h/G, 0 : n_cur[i])                    the sample's own rows of the block being drafted
 *   q, out  device [B, samples, Hq, dh]  (B = a->B prompts);  k_hat_shared, v_hat_shared device [B, Hkv, a->T_max, dh]
 *   k_hat_own, v_hat_own device [B * samples, Hkv, T_own, dh];  k_cur, v_cur device [B * samples, Hkv, a->gamma_max, dh]
 *   n_shared int32 [B]; n_own, n_cur int32 [B * samples]; all clamped to their caches
 *   samples <= TANDEM_MAX_SHARED_ROWS, B * samples <= 65535.
 * ws: at least tandem_draft_attn_shared_workspace(...) bytes, always needed.  Reads the caches only. */
size_t tandem_draft_attn_shared_workspace(const tandem_attn_desc *a, int32_t samples, int64_t T_own);
int tandem_draft_attn_shared(const tandem_attn_desc *a, int32_t samples, int64_t T_own, const void *q,
                             const void *k_hat_shared, const void *v_hat_shared, const int32_t *n_shared,
                             const void *k_hat_own, const void *v_hat_own, const int32_t *n_own, const void *k_cur,
                             const void *v_cur, const int32_t *n_cur, void *out, void *ws, size_t ws_bytes,
                             void *hip_stream);

/* Deep Tandem's large-model attention (Eq. (3)): the query at position i = n_prefix[b] + r (0-indexed) attends only
 * the rows of the blocks completed before its own block, cache rows 0 .. floor(i / gamma) * gamma - 1 (the paper's
 * keys x_{<= k gamma}, k = ceil((i - gamma) / gamma), in 1-indexed positions); queries of the first block see no key
 * and give zeros (the paper does not say).  Shapes, limits and workspace as tandem_block_attn; gamma >= 1. */
size_t tandem_block_prefix_attn_workspace(const tandem_attn_desc *a, int32_t q_len);
int tandem_block_prefix_attn(const tandem_attn_desc *a, const void *q, const void *k_cache, const void *v_cache,
                             const int32_t *n_prefix, int32_t q_len, int32_t gamma, void *out, void *ws, size_t ws_bytes,
                             void *hip_stream);

/* The small model's attention at every position of a known sequence (Eq. (2), second line, with the block
 * boundary of each query's own position; Sec. 3 "Training": the form used in training and in teacher-forced
 * scoring, where M_S processes all tokens and, inside a block, sees its own rows instead of M_L's).  One call
 * handles the q_len consecutive positions n_prefix[b] .. n_prefix[b] + q_len - 1 of every sequence.  The query
 * at position i (0-indexed), head h, attends in ONE softmax, with k = floor(i / gamma) * gamma,
 *   k_hat/v_hat[b, h/G, 0 : k)       rows derived from M_L through FF_Tandem (completed blocks)
 *   k_own/v_own[b, h/G, k : i + 1)   rows M_S computed itself (the query's own block, incl. its own row)
 *   q, out  device [B, q_len, Hq, dh]     all four caches device [B, Hkv, T_max, dh], indexed by position
 *   n_prefix device int32 [B], requires n_prefix[b] + q_len <= T_max (clamped otherwise);  gamma >= 1
 *   1 <= q_len <= TANDEM_MAX_QLEN.  ws: at least tandem_mixed_attn_workspace(a, q_len) bytes.
 * gamma = 1 is tandem_draft_attn with one own row per query; gamma > T_max is tandem_block_attn on the own
 * caches.  Reads the caches only; writes out and ws only. */
size_t tandem_mixed_attn_workspace(const tandem_attn_desc *a, int32_t q_len);
int tandem_mixed_attn(const tandem_attn_desc *a, const void *q, const void *k_hat, const void *v_hat,
                      const void *k_own, const void *v_own, const int32_t *n_prefix, int32_t q_len, int32_t gamma,
                      void *out, void *ws, size_t ws_bytes, void *hip_stream);

/* Mixed-source small-model attention (Eq. (2), second line; Sec. 3 "Training", both bullets).
 * One query per sequence and head attends, in ONE softmax, the union of
 *   k_hat/v_hat[b, h/G, 0 : n_large[b]]  rows derived from M_L through FF_Tandem (completed blocks)
 *   k_cur/v_cur[b, h/G, 0 : n_cur[b]]    rows M_S computed itself for the current block (incl. the query's own)
 *   q, out device [B, Hq, dh];  k_hat, v_hat device [B, Hkv, T_max, dh];  k_cur, v_cur device
 *   [B, Hkv, gamma_max, dh];  n_large, n_cur device int32 [B] (clamped to [0,T_max], [0,gamma_max]).
 * A sequence with n_large + n_cur == 0 gets an all-zero output row.  Never writes the caches. */
int tandem_draft_attn(const tandem_attn_desc *a, const void *q, const void *k_hat, const void *v_hat,
                      const int32_t *n_large, const void *k_cur, const void *v_cur, const int32_t *n_cur, void *out,
                      void *ws, size_t ws_bytes, void *hip_stream);

/* tandem_draft_attn for callers that cannot allocate device memory or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * tandem_draft_attn, but the split-K partials live in a device array that is part of the library image
 * (TANDEM_STATIC_SCRATCH_BYTES per GPU, held from library load to process end); the call allocates nothing.
 * Returns TANDEM_ERR_WORKSPACE when tandem_draft_attn_workspace(a) exceeds TANDEM_STATIC_SCRATCH_BYTES (nothing is
 * enqueued): the limit covers every shape with up to two query heads per KV head, and grouped shapes with few splits.  All calls on one GPU share that array: calls that may overlap on one GPU (different streams, threads
 * or processes' graphs replayed concurrently) race on it - order them.  Nothing in it needs clearing between calls. */
#define TANDEM_STATIC_SCRATCH_BYTES (1u << 20)
int tandem_draft_attn_static(const tandem_attn_desc *a, const void *q, const void *k_hat, const void *v_hat,
                             const int32_t *n_large, const void *k_cur, const void *v_cur, const int32_t *n_cur, void *out,
                             void *hip_stream);

/* ------------------------------------------------------------------ whole decode step */

/* One pre-norm decoder layer: h = x + Wo Atn(RMSNorm(x; g_attn)); x' = h + W2 gelu(W1 RMSNorm(h; g_mlp) + b1) + b2.
 * Wqkv stacks the query, key and value maps: [(Hq + 2 Hkv) dh, d] (all Hq query heads, then the
 * Hkv key heads, then the Hkv value heads).  Wo [d, Hq dh], W1 [d_ff, d], W2 [d, d_ff].
 * b1, b2 may be NULL.  All device pointers in the model dtype. */
typedef struct {
  const void *g_attn, *Wqkv, *Wo, *g_mlp, *W1, *b1, *W2, *b2;
} tandem_layer_weights;

typedef struct {
  int32_t n_layers, d, Hq, Hkv, dh, d_ff, vocab;
  const void *emb;     /* device [vocab, d]                          */
  const void *g_final; /* device [d], gain of the final RMSNorm       */
  const void *W_out;   /* device [vocab, d], untied output head        */
  const tandem_layer_weights *layers; /* host array [n_layers]        */
} tandem_decoder_desc;

typedef struct {
  tandem_decoder_desc L, S;  /* M_L and M_S                                                   */
  const int32_t *ell;        /* host [S.n_layers]; small layer j reads x^(ell[j]), the residual
                                stream after ell[j] large layers, 0 <= ell[j] <= L.n_layers    */
  const tandem_ff_desc *ff;  /* host [S.n_layers]; ff[j].d_L == L.d, ff[j].d_S == S.d          */
  float rms_eps;
  int32_t dtype;             /* tandem_dtype of every weight, cache and activation             */
  int32_t flags;             /* reserved, must be 0                                            */
} tandem_model_desc;

/* Caller-owned decoding state (all device memory except the pointer arrays themselves).
 *   KL[j], VL[j]      [B, L.Hkv, T_max, dh]     M_L's K/V cache of large layer j
 *   Khat[j], Vhat[j]  [B, S.Hkv, T_max, dh]     rows of small layer j derived from M_L via FF_Tandem
 *   Kcur[j], Vcur[j]  [B, S.Hkv, gamma_max, dh] small layer j's own rows for the current block
 *   n[b]        positions 0..n[b]-1 have rows in KL/VL and Khat/Vhat
 *   pending[b]  token at position n[b]: emitted, but not yet processed by M_L
 * Cache ownership rule (Sec. 3 "Inference", last paragraph): the draft phase writes only
 * Kcur/Vcur; KL/VL/Khat/Vhat rows [n, n+q) are written by the verify phase after the
 * small model has finished the block; rows below n[b] are never modified. */
typedef struct {
  int32_t B;
  int64_t T_max;
  int32_t gamma_max;
  void *const *KL, *const *VL;     /* host arrays [L.n_layers] */
  void *const *Khat, *const *Vhat; /* host arrays [S.n_layers] */
  void *const *Kcur, *const *Vcur; /* host arrays [S.n_layers] */
  int32_t *n, *pending;            /* device int32 [B]         */
} tandem_state_desc;

/* Optional per-step outputs, each a device pointer or NULL (q = rows M_L verifies per sequence: gamma,
 * or gamma + 1 with TANDEM_STEP_FREE_TOKEN):
 *   draft  int32 [B, gamma]  d_1..d_gamma, the small model's greedy tokens
 *   verify int32 [B, q]      M_L's greedy token after each verified row
 *   y_small  [B, gamma, S.d] final small-model representation y^(L_S) of every draft run
 *   x_large  [B, q, L.d]     final large-model representation x^(L_L) of the block rows
 *   logits_S [B, gamma, vocab], logits_L [B, q, vocab]   (model dtype)           */
typedef struct {
  int32_t *draft, *verify;
  void *y_small, *x_large, *logits_S, *logits_L;
} tandem_step_aux;

typedef struct tandem_model tandem_model; /* opaque host object: validated copy of a tandem_model_desc */

/* tandem_model_create allocates host memory only (a validated copy of the descriptor); the weights stay the
 * caller's and must outlive the handle. */
int tandem_model_create(const tandem_model_desc *desc, tandem_model **out);
void tandem_model_destroy(tandem_model *m);

/* Packed copies of the model's weights, in memory the caller owns.  Every bf16 weight matrix of the model whose shape
 * allows it (rows % 128 == 0, columns % 256 == 0) gets a second copy in the layout of tandem_pack_weight; the
 * decode-time products of every later call on this handle then read each weight as one contiguous stream.
 *   tandem_model_packed_bytes(m)  bytes the copies need (0: nothing to pack) - as much again as those matrices
 *   tandem_model_pack(m, packed, packed_bytes, hip_stream)  packed: device, 256-byte aligned, at least that many
 *     bytes, owned by the caller and kept alive and unmodified as long as the handle is used.  The packing kernels are
 *     enqueued on hip_stream; calls that use the handle must be ordered after them (same stream, or an event).
 * Not thread-safe against concurrent calls on the same handle.  Without it the row-major weights are used. */
size_t tandem_model_packed_bytes(const tandem_model *m);
int tandem_model_pack(tandem_model *m, void *packed, size_t packed_bytes, void *hip_stream);
size_t tandem_decode_step_workspace(const tandem_model *m, int32_t B, int32_t gamma);

/* tandem_decode_step flags.  TANDEM_STEP_FREE_TOKEN (Sec. 3.1, Fig. 2): M_L also processes the last
 * draft token, q = gamma + 1 rows, so its own token after the accepted prefix is always available: every
 * step emits a + 1 tokens, the last one a bonus token when all gamma drafts were right. */
#define TANDEM_STEP_FREE_TOKEN 1

/* One Tandem + SPEED decode step for every sequence (Sec. 3.1; Sec. 1 steps 2-4; one step is
 * gamma runs of M_S and one block run of M_L over q = gamma (+ 1 with the free token) rows):
 *   1. draft: M_S runs gamma times from `pending`, each run attending Khat/Vhat[0:n) and its own
 *      block rows (tandem_draft_attn per small layer), greedy token d_{r+1} after run r;
 *   2. verify: M_L processes the first q of [pending, d_1 .. d_gamma] in block mode at positions
 *      n..n+q-1 (tandem_block_attn per large layer), appending its K/V rows and giving its own greedy tokens;
 *   3. tandem_project per small layer on the q new rows of x^(ell[j]), then that layer's
 *      RMSNorm and W_K/W_V produce the new Khat/Vhat rows;
 *   4. accept: a[b] = number of leading draft tokens equal to M_L's tokens; emitted tokens are
 *      d_1..d_a followed by M_L's token after them - except that without the free token a fully accepted
 *      block (a == gamma) emits d_1..d_gamma only, M_L not having seen d_gamma;
 *      n[b] += number of emitted tokens; pending[b] = last emitted token.  Ties in argmax go to the lowest id.
 * forced: optional device int32 [B, gamma]; when given, forced[b, r] replaces d_{r+1} as the input
 *   of the following runs and everything is treated as accepted (teacher forcing / prompt ingestion):
 *   n[b] += q, emitted = forced[b, :] (+ M_L's token after them with the free token).
 * out_tokens device int32 [B, q] (emitted tokens, -1 padded), n_accepted device int32 [B] (a[b]).
 * 1 <= gamma <= gamma_max, q <= TANDEM_MAX_QLEN; requires n[b] + q <= T_max.
 * ws: at least tandem_decode_step_workspace(m, B, gamma) bytes (sized for either mode). */
int tandem_decode_step(const tandem_model *m, const tandem_state_desc *state, int32_t gamma, int32_t flags,
                       const int32_t *forced,
                       int32_t *out_tokens, int32_t *n_accepted, const tandem_step_aux *aux, void *ws, size_t ws_bytes,
                       void *hip_stream);

/* ---- several samples per prompt (Sec. 3.1, num-samples; the latency evaluation's 4 samples) ----
 * The step for state->B = prompts * samples sequences, sequence i = b * samples + s continuing prompt b.  The rows
 * of the prompts live once per prompt in the caches of `prompt` (as a tandem_prefill on a state of `prompts`
 * sequences leaves them: that state's KL / VL / Khat / Vhat and n) and are only read.  The caches of `state` hold
 * each sequence's rows AFTER its prompt: state->n[i] counts those rows, state->T_max is their capacity.  Every
 * attention call of the step runs through tandem_block_attn_shared / tandem_draft_attn_shared, so the prompt rows
 * cross HBM once per prompt; everything else, and the result, is that of tandem_decode_step on per-sequence
 * caches holding a copy of the prompt rows followed by the sequence's own (this model has no positional encoding). */
typedef struct {
  int32_t samples;
  int64_t T_prompt;              /* rows per prompt cache */
  void *const *KLp, *const *VLp; /* host arrays [L.n_layers] of device [prompts, L.Hkv, T_prompt, L.dh] */
  void *const *Khp, *const *Vhp; /* host arrays [S.n_layers] of device [prompts, S.Hkv, T_prompt, S.dh] */
  const int32_t *n_prompt;       /* device int32 [prompts] */
} tandem_prompt_desc;

size_t tandem_decode_step_shared_workspace(const tandem_model *m, int32_t B, int32_t samples, int32_t gamma);
int tandem_decode_step_shared(const tandem_model *m, const tandem_state_desc *state, const tandem_prompt_desc *prompt,
                              int32_t gamma, int32_t flags, int32_t *out_tokens, int32_t *n_accepted,
                              const tandem_step_aux *aux, void *ws, size_t ws_bytes, void *hip_stream);

/* ---- adaptive block length (Sec. 3.1 "Adaptive Block Length"; Sec. 4: threshold 0.8) ----
 * A 2-layer router MLP decides after every draft token whether M_S goes on drafting or M_L verifies now.  Its
 * input, in this order: the entropy (nats) of M_S's distribution over the vocabulary for the current token, the k
 * largest probabilities in descending order (equal logits: lowest id first), and M_S's input-embedding rows of those
 * k tokens - 1 + k + k * d numbers.  The paper fixes neither the hidden activation nor the meaning of the output;
 * here: p = sigmoid(w2 . relu(W1 f + b1) + b2) is the predicted probability that M_L accepts the current draft
 * token, and drafting continues iff p >= tau.  All device pointers in `dtype`; b1, b2 may be NULL (zero).
 *   W1 [d_hidden, 1 + k + k * d]   b1 [d_hidden]   w2 [d_hidden]   b2 [1]
 * 1 <= k <= TANDEM_ROUTER_MAX_K, (1 + k + k * d) * 4 bytes + 64 <= 64 KB (the feature vector lives in LDS). */
#define TANDEM_ROUTER_MAX_K 8
typedef struct {
  int32_t k, d_hidden;
  int32_t dtype; /* tandem_dtype; for tandem_decode_step_adaptive the model's */
  float tau;
  const void *W1, *b1, *w2, *b2;
} tandem_router_desc;

/* The router alone: p_out[i] (device fp32 [rows]) for the logits rows logits[i, :] (device [rows, vocab]) with the
 * embedding table emb (device [vocab, d]), both in r->dtype.  tau is not used. */
int tandem_router_eval(const tandem_router_desc *r, const void *logits, const void *emb, int32_t rows, int32_t vocab,
                       int32_t d, float *p_out, void *hip_stream);

/* tandem_decode_step with the adaptive block length: gamma_max is the largest block.  Sequence b stops drafting
 * after the first draft token whose router probability is below tau: g[b] tokens, 1 <= g[b] <= gamma_max.  The
 * batch still runs gamma_max draft runs and verifies q = gamma_max (+ 1) rows per sequence - a stopped sequence
 * keeps its place, its later rows are ignored, and the cache rows they write lie beyond the new n[b] and are
 * overwritten by the following steps - but its draft attention is skipped in the later runs (no cache traffic, zero
 * rows), and once EVERY sequence has stopped the kernels of the remaining draft runs return at once (bf16 models: a
 * device counter of sequences still drafting gates them; the launch sequence stays the same, so the step can still be
 * captured in a HIP graph).  Acceptance, emitted tokens, n[b] and pending[b] are those of a step with gamma = g[b]
 * (the free token, if asked for, is M_L's token after d_g[b]).
 *   n_drafted  optional device int32 [B]: g[b]
 *   router_p   optional device fp32 [B, gamma_max]: the router's p after every draft run; entries past g[b], like the
 *              aux outputs of those runs, are unspecified
 * No forced tokens.  Everything else as in tandem_decode_step, including the workspace size. */
int tandem_decode_step_adaptive(const tandem_model *m, const tandem_state_desc *state,
                                const tandem_router_desc *router, int32_t gamma_max, int32_t flags,
                                int32_t *out_tokens, int32_t *n_accepted, int32_t *n_drafted, float *router_p,
                                const tandem_step_aux *aux, void *ws, size_t ws_bytes, void *hip_stream);

/* Prompt ingestion (Sec. 1 steps 1 and 3 for tokens that are already known; Sec. 3 "Inference"): for every
 * sequence, M_L processes tokens[b, 0:q_len) at positions n[b] .. n[b]+q_len-1 in block mode, appending its
 * K/V rows, and FF_Tandem with the small layers' norm and W_K / W_V appends the Khat/Vhat rows.  M_S does not
 * run: of its own rows only those of the block being drafted are ever attended (Eq. (2) line 2).
 * n[b] += q_len.  With TANDEM_PREFILL_EMIT, pending[b] becomes M_L's greedy token after the last row (the first
 * generated token); otherwise pending is left alone (the caller keeps the last prompt token pending).
 *   tokens   device int32 [B, q_len];  1 <= q_len <= TANDEM_MAX_PREFILL: longer prompts take several calls (the
 *            dense layers run on all B * q_len rows at once; the attention of a layer is one launch for bf16 models
 *            with heads of 128, which takes the rows in passes of 128 per KV head, and runs on sub-blocks of
 *            TANDEM_MAX_QLEN rows otherwise)
 *   x_large  optional device [B, q_len, L.d]: x^(L_L) of the rows
 *   requires n[b] + q_len <= T_max;  ws: at least tandem_prefill_workspace(m, B, q_len) bytes. */
#define TANDEM_PREFILL_EMIT 1
size_t tandem_prefill_workspace(const tandem_model *m, int32_t B, int32_t q_len);
int tandem_prefill(const tandem_model *m, const tandem_state_desc *state, const int32_t *tokens, int32_t q_len,
                   int32_t flags, void *x_large, void *ws, size_t ws_bytes, void *hip_stream);

/* Teacher-forced pass of the small model over known tokens (Eq. (2) at every position; Sec. 3 "Training": the form
 * that training and the evaluation of the Tandem model's own predictions use).  For every sequence, M_S processes
 * tokens[b, 0:q_len) at positions pos[b] .. pos[b] + q_len - 1: every layer appends its own K/V rows to
 * k_own[j] / v_own[j] at those positions and attends with tandem_mixed_attn (Khat/Vhat rows below the query's block
 * boundary floor(i / gamma) * gamma, own rows from there to i).  The Khat/Vhat rows of all completed blocks below
 * pos[b] + q_len must already be in the state (tandem_prefill over the same tokens), and the own rows of the current
 * block below pos[b] in k_own / v_own (earlier calls).  The state is only read.
 *   k_own, v_own  host arrays [S.n_layers] of device [B, S.Hkv, T_max, S.dh] (caller-owned, indexed by position)
 *   pos           device int32 [B], requires pos[b] + q_len <= T_max
 *   tokens        device int32 [B, q_len];  1 <= q_len <= TANDEM_MAX_QLEN, gamma >= 1
 *   greedy        optional device int32 [B, q_len]: M_S's greedy prediction of the token after each position
 *   logits        optional device [B, q_len, vocab];  y_small optional device [B, q_len, S.d]: y^(L_S)
 * ws: at least tandem_score_workspace(m, B, q_len) bytes. */
size_t tandem_score_workspace(const tandem_model *m, int32_t B, int32_t q_len);
int tandem_score(const tandem_model *m, const tandem_state_desc *state, void *const *k_own, void *const *v_own,
                 const int32_t *pos, const int32_t *tokens, int32_t q_len, int32_t gamma, int32_t *greedy, void *logits,
                 void *y_small, void *ws, size_t ws_bytes, void *hip_stream);

/* ---- Deep Tandem (Sec. 5, Eq. (3) and Eq. (4)), teacher-forced over known tokens ----
 * M_L predicts a sketch of the next block in parallel; M_S, a plain causal decoder, adds each row's sketch to its input
 * embedding.  In 0-indexed positions (the paper's row i is row i - 1 of M_L and position i - 2 of M_S):
 *   M_L row r:   input Emb_L(token r - gamma) (a zero row when r < gamma); it attends, in every layer, the K/V rows of
 *                M_L rows [0, floor(r / gamma) * gamma) - the blocks completed before its own (no visible row: zero
 *                attention output); its final representation x^(L_L) is the sketch for M_S's position r - 1
 *   M_S pos p:   y^(0) = Emb_S(token p) + FF_DeepTandem(sketch of M_L row p + 1); causal attention over its own rows
 *                [0, p]; y^(L_S) predicts token p + 1
 * (Where the displayed formula and the sentence after it disagree about M_L's input token, the formula is taken.)
 * Caches are the caller's, indexed by row / position: KL, VL [L.n_layers] of [B, L.Hkv, T_max, dh] (M_L's rows) and
 * KS, VS [S.n_layers] of [B, S.Hkv, T_max, dh] (M_S's rows), host arrays of device pointers.
 *   tandem_deep_begin   computes M_L's row 0 (it has no token and sees nothing, but later rows attend it); once per
 *                       sequence set, before the first tandem_deep_score
 *   tandem_deep_score   one chunk: M_S positions pos[b] .. pos[b] + q_len - 1 and M_L rows pos[b] + 1 .. pos[b] + q_len;
 *                       M_L rows up to pos[b] and M_S rows below pos[b] must be in the caches (earlier calls)
 *     tokens  device int32 [B, n_tokens]: the known tokens of every sequence (positions >= n_tokens read the last one)
 *     pos     device int32 [B], pos[b] + q_len < T_max;  1 <= q_len <= TANDEM_MAX_QLEN;  gamma >= 1
 *     greedy  optional device int32 [B, q_len]; logits optional [B, q_len, vocab]; y_small optional [B, q_len, S.d];
 *     sketch  optional [B, q_len, L.d]: x^(L_L) of M_L's rows of the chunk
 *   ff_deep: FF_DeepTandem, d_L = L.d, d_S = S.d, model dtype.  ws: at least tandem_deep_score_workspace(...) bytes. */
typedef struct {
  int32_t B;
  int64_t T_max;
  void *const *KL, *const *VL; /* host arrays [L.n_layers] */
  void *const *KS, *const *VS; /* host arrays [S.n_layers] */
} tandem_deep_state_desc;
size_t tandem_deep_score_workspace(const tandem_model *m, const tandem_ff_desc *ff_deep, int32_t B, int32_t q_len);
int tandem_deep_begin(const tandem_model *m, const tandem_ff_desc *ff_deep, const tandem_deep_state_desc *st, void *ws,
                      size_t ws_bytes, void *hip_stream);
int tandem_deep_score(const tandem_model *m, const tandem_ff_desc *ff_deep, const tandem_deep_state_desc *st,
                      const int32_t *tokens, int64_t n_tokens, const int32_t *pos, int32_t q_len, int32_t gamma,
                      int32_t *greedy, void *logits, void *y_small, void *sketch, void *ws, size_t ws_bytes,
                      void *hip_stream);

/* One Deep Tandem decoding step (Sec. 5): greedy generation of the next gamma tokens of every sequence.
 * M_L's rows of a block read only tokens at least gamma positions back (Eq. (3)), so the sketches of the next gamma
 * rows are computed in ONE block pass of M_L before M_S samples any of them; M_S then runs gamma times, each run on
 * the token the run before produced plus its row's sketch (Eq. (4)).  With len[b] tokens of sequence b known:
 *   M_L rows len[b] .. len[b] + gamma - 1 (inputs: tokens len[b] - gamma .. len[b] - 1), then FF_DeepTandem of them;
 *   run t = 0 .. gamma - 1: M_S position len[b] - 1 + t reads token len[b] - 1 + t and the sketch of M_L row
 *   len[b] + t, attends its own rows [0, len[b] - 1 + t], and its highest logit (ties: lowest id) is token len[b] + t.
 * Needs M_L rows [0, len[b]) and M_S positions [0, len[b] - 1) in the caches: tandem_deep_begin, then
 * tandem_deep_score over the known tokens (pos = 0 .., the last chunk ending at position len[b] - 2) or earlier steps.
 *   tokens  device int32 [B, n_tokens], read and written: the new tokens are appended at len[b] + t
 *   len     device int32 [B], 1 <= len[b], len[b] + gamma <= min(n_tokens, T_max); advanced by gamma (never past that
 *           minimum; a sequence that would pass it gets no defined tokens, nothing is written out of bounds)
 *   out_tokens optional device int32 [B, gamma]; logits optional [B, gamma, vocab]; y_small optional [B, gamma, S.d];
 *   sketch optional [B, gamma, L.d];  1 <= gamma <= TANDEM_MAX_QLEN
 *   ws: at least tandem_deep_score_workspace(m, ff_deep, B, gamma) bytes.
 * Scoring the sequence afterwards with tandem_deep_score reproduces the tokens (the same rows are computed). */
int tandem_deep_step(const tandem_model *m, const tandem_ff_desc *ff_deep, const tandem_deep_state_desc *st,
                     int32_t *tokens, int64_t n_tokens, int32_t *len, int32_t gamma, int32_t *out_tokens, void *logits,
                     void *y_small, void *sketch, void *ws, size_t ws_bytes, void *hip_stream);

/* Measurement helper, no part of the method: reads src[0 : bytes) (device, 16-byte aligned; a multiple of 16 bytes is
 * read) once with coalesced non-temporal 16-byte loads and writes TANDEM_READ_STREAM_BLOCKS 32-bit words of folded data to
 * sink (device).  The rate this call reaches is the read ceiling of the box for kernels that stream HBM once, the
 * yardstick bench.py reports next to the datasheet peak for the attention kernels (Sec. 3.1, footnote: attention is
 * the part of decoding whose memory traffic does not amortise over the batch). */
#define TANDEM_READ_STREAM_BLOCKS 2048
int tandem_read_stream(const void *src, size_t bytes, void *sink, void *hip_stream);

const char *tandem_status_string(int status);

#pragma GCC visibility pop

#ifdef __cplusplus
}
#endif
#endif /* TANDEM_H */
