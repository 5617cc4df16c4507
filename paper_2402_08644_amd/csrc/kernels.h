// Internal launch interface between the C ABI layer and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tandem.h"

// ---------------------------------------------------------------- attention (attn_rows.hip)
// Streaming attention of query rows over a virtual key sequence that is the concatenation
// of source A (cache rows [0, nA)) and source B (own-block rows [0, nB)).
struct AttnArgs {
  const void* q;               // [B, q_len, Hq, dh]
  const void *kA, *vA;         // [B, Hkv, T_max, dh]
  const void *kB, *vB;         // [B, Hkv, gamma_max, dh] or nullptr
  const int32_t* nA;           // [B]
  const int32_t* nB;           // [B] or nullptr
  int causal;                  // 1: row r of the block sees nA[b] + r + 1 rows of A (block mode);
                               // 0: every row sees nA[b] rows of A (and nB[b] rows of B)
  int B, Hq, Hkv, dh, q_len;
  int64_t T_max;
  int gamma_max;
  float scale;
  int dtype;
  void* out;                   // [B, q_len, Hq, dh]
  float* part_ml;              // [rows, S, 2]   (m in log2 units, l)
  float* part_o;               // [rows, S, dh]  un-normalised
  int S;                       // number of context splits
  int wide;                    // 1 = workgroups of eight wavefronts (see attn_*_splits)
  // Several launches over different key segments can fill one table of partials: the launch writes slots
  // [s_off, s_off + S) of S_total per row and leaves the combine to the caller.  S_total = 0 means S_total = S,
  // s_off = 0, and the launch combines its own splits.
  int S_total, s_off;
  // MFMA block kernels only, S == 1: fold slots [0, merge_prev) (written by earlier launches on the stream)
  // into this launch's rows and write the finished rows to out - the last segment needs no combine launch.
  int merge_prev;
  // All-positions small-model attention (Eq. (2) with the query's own block boundary kb = floor(i / gamma) * gamma,
  // i = nA[b] + r).  MFMA kernels: mixed = 1 - kA/vA hold the rows derived from the large model, row r sees keys
  // [0, kb); mixed = 2 - kA/vA hold the model's own rows, row r sees [kb, i].  attn_rows kernels: mixed = 3 - kA/vA
  // as in 1, kB/vB own rows in a cache of T_max rows indexed by position, both in one launch.
  int mixed, gamma;
  // A call may cover q_len of the q_rows rows that q and out hold per sequence (q / out then point at the first
  // covered row of sequence 0): q_rows = 0 means q_len.  n_off is added to every nA[b].
  int q_rows, n_off;
  // attn_rows kernels only, optional [B]: sequences with skip[b] != 0 are not processed (zero output rows)
  const int32_t* skip;
};

// number of context splits; *wide (optional) = 1 when the workgroups should have eight wavefronts (AttnArgs::wide)
int attn_rows_splits(int B, int Hkv, int q_len, int G, int64_t T_max, int gamma_max, int* wide);
size_t attn_rows_workspace(int B, int Hq, int q_len, int dh, int S);
int launch_attn_rows(const AttnArgs& a, hipStream_t st);

// MFMA block-mode attention (attn_block.hip): bf16, dh = 128, all G*q_len rows of a KV head per workgroup.
// number of context splits; *wide (optional) = 1 when the workgroups should have eight wavefronts (AttnArgs::wide)
int attn_block_splits(int B, int Hkv, int q_len, int G, int64_t T_max, int* wide);
size_t attn_block_workspace(int B, int Hq, int q_len, int S);
bool attn_block_supported(const AttnArgs& a);
int launch_attn_block(const AttnArgs& a, hipStream_t st);

// combine of split partials (attn_rows.hip); fixed split order
// rows_per_seq / row_skip: output row (row + (row / rows_per_seq) * row_skip); 0 / 0 for a dense output
int launch_attn_combine(const float* part_ml, const float* part_o, void* out, int rows, int S, int dh, int dtype,
                        hipStream_t st, int rows_per_seq = 0, long long row_skip = 0);

// ---------------------------------------------------------------- dense (gemm.hip)
// Y[M, N] = epilogue(X[M, K] . W[N, K]^T): + bias[N], activation, + residual[M, N].
struct GemmArgs {
  const void* X;
  int64_t ldx;  // row stride of X in elements
  const void* W;
  const void* Wp;        // W in the packed tile layout (launch_pack_weights) or nullptr; used when the shape allows
  const void* bias;      // [N] or nullptr
  const void* residual;  // [M, ldr] or nullptr
  int64_t ldr;
  void* Y;
  int64_t ldy;
  int M, N, K;
  int act;    // tandem_act
  int dtype;  // tandem_dtype of X, W, bias, residual, Y
  float* ws;  // split-K partials
  size_t ws_bytes;
  int defer;  // 1: leave fp32 partial sums [splits, M, N] in ws and skip the epilogue (bf16 MFMA path only);
              //    a fused consumer kernel finishes the layer.  bias / act / residual / Y are then ignored.
  const int32_t* gate = nullptr;  // optional device flag: when *gate == 0 the kernels return at once and write nothing
                                  // (bf16 MFMA kernels and their split epilogue; the generic kernel ignores it)
};
size_t gemm_workspace(int M, int N, int K, int dtype);
bool gemm_can_defer(int M, int N, int K, int dtype, int64_t ldx);  // deferred epilogue available for this shape
size_t gemm_deferred_workspace(int M, int N, int K);
int gemm_splits(int M, int N, int K, bool packed);  // number of partials a deferred launch leaves
bool gemm_packable(int64_t N, int64_t K, int dtype);  // a packed copy of W[N, K] can be used
int launch_pack_weights(const void* W, void* Wp, int64_t N, int64_t K, hipStream_t st);
int launch_gemm(const GemmArgs& g, hipStream_t st);

// ---------------------------------------------------------------- glue (glue.hip)
int launch_rmsnorm(const void* x, const void* g, void* y, int rows, int d, float eps, int dtype, hipStream_t st);
// finishes a deferred GEMM row by row: v = sum of partials (+ bias) (+ residual); x_out = v (and x_out2 = v when
// given: a second copy that outlives the next in-place update); and, when g is given, xn_out = RMSNorm(v; g).
// residual may alias x_out.
// gate (here and below, optional): a device flag; when *gate == 0 the kernel returns at once and writes nothing.
int launch_finish_norm(const float* part, int splits, const void* bias, const void* residual, void* x_out,
                       const void* g, void* xn_out, int rows, int d, float eps, int dtype, hipStream_t st,
                       void* x_out2 = nullptr, const int32_t* gate = nullptr);
// x[row] = emb[token(row)] and, when g is given, xn[row] = RMSNorm(x[row]; g).  token(row): tokens[row * tok_stride],
// or - pending given - the token at block position r = row % q + r0 of sequence b = row / q: pending[b] for r = 0,
// follow[b * gamma + r - 1] otherwise.  init_B > 0 (rows == init_B): also ncur[r][b] = r + 1 for r < init_gamma and
// stop[b] = 0 (stop optional) - the bookkeeping the first draft run of a step needs.
int launch_embed_norm(const void* emb, const int32_t* tokens, int64_t tok_stride, const int32_t* pending,
                      const int32_t* follow, int gamma, int q, int r0, void* x, const void* g, void* xn, int rows, int d,
                      int vocab, float eps, int32_t* ncur, int32_t* stop, int init_B, int init_gamma, int dtype,
                      hipStream_t st, int32_t* active = nullptr, const int32_t* gate = nullptr);  // active: [init_gamma] counters cleared with stop
// The same gather with shifted token indices: tokens is [B, n_tokens]; row b * q + rr reads token
// (pos ? pos[b] : 0) + fixed + rr - shift of sequence b.  A negative index gives an all-zero row (x and xn), an
// index past the end is clamped.  (Deep Tandem, Eq. (3): row i of M_L reads token i - gamma.)
int launch_embed_shifted(const void* emb, const int32_t* tokens, int64_t n_tokens, const int32_t* pos, int fixed,
                         int shift, int q, void* x, const void* g, void* xn, int rows, int d, int vocab, float eps,
                         int dtype, hipStream_t st);
