// Launchers of the small decode-step kernels (glue.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tandem.h"

int launch_scatter_qkv(const void* qkv, void* q, void* kc, void* vc, const int32_t* base, int fixed, int rows, int q_len,
                       int Hq, int Hkv, int dh, int64_t cap, int q_off_cols, int kv_off_cols, int row_cols, int dtype,
                       hipStream_t st);
int launch_finish_scatter(const float* part, int splits, void* q, void* kc, void* vc, const int32_t* base, int fixed,
                          int rows, int q_len, int Hq, int Hkv, int dh, int64_t cap, int q_cols, int row_cols, int dtype,
                          hipStream_t st, const int32_t* gate = nullptr);
int launch_argmax(const void* logits, int rows, int vocab, int32_t* out, int64_t out_stride, int dtype, hipStream_t st,
                  const int32_t* gate = nullptr);
// stop (optional, [B]): sequence b drafted stop[b] tokens (0 = all gamma); n_drafted (optional) receives that number
int launch_accept(const int32_t* draft, const int32_t* verify, const int32_t* forced, const int32_t* stop,
                  int32_t* out_tokens, int32_t* n_accepted, int32_t* n_drafted, int32_t* n, int32_t* pending, int B,
                  int gamma, int q, int64_t cap, hipStream_t st);  // cap: n[b] never advances past the cache capacity
// router of the adaptive block length (router.hip)
int check_router(const tandem_router_desc* r, int d);
// active (optional, with stop): active[run] += 1 for every sequence still drafting after this run; gate as elsewhere
int launch_router(const tandem_router_desc* r, const void* logits, const void* emb, int rows, int vocab, int d, int run,
                  int32_t* stop, float* p_out, int64_t p_stride, hipStream_t st, int32_t* active = nullptr,
                  const int32_t* gate = nullptr);
int launch_advance(int32_t* n, int B, int by, int64_t cap, hipStream_t st);  // n[b] = min(n[b] + by, cap)
int launch_fill_i32(int32_t* p, int32_t v, int n, hipStream_t st);  // p[0:n) = v (a kernel: safe under graph capture)
// Deep Tandem decoding (Sec. 5): input of M_S's run t (token lookup, appending the run before's token, embedding +
// add[b, t] and the first RMSNorm), and the end of a step (last token appended, len[b] = min(len[b] + gamma, cap))
int launch_deep_input(const void* emb, int32_t* tokens, int64_t n_tokens, const int32_t* len, int t, const int32_t* prev,
                      int gamma, const void* add, void* x, const void* g, void* xn, int B, int d, int vocab, float eps,
                      int dtype, hipStream_t st);
int launch_deep_advance(int32_t* tokens, int64_t n_tokens, int32_t* len, const int32_t* prev, int B, int gamma, int64_t cap,
                        hipStream_t st);
