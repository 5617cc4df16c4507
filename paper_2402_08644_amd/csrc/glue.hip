// Small kernels between the dense layers and the attention kernels of the decode step:
// embedding gather, RMSNorm, scattering fresh K/V rows into the caches, greedy argmax and the
// SPEED acceptance rule (Sec. 3.1).  None of them moves a significant number of bytes.
#include "common.h"
#include "kernels.h"
#include "glue.h"

namespace {

__device__ __forceinline__ void store4(float* p, const float4& v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void store4(bf16_t* p, const float4& v) {
  uint2 u;
  u.x = pack_bf16x2(v.x, v.y);
  u.y = pack_bf16x2(v.z, v.w);
  *reinterpret_cast<uint2*>(p) = u;
}
__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load4(const bf16_t* p) {
  const uint2 u = *reinterpret_cast<const uint2*>(p);
  return make_float4(bf16lo_to_f32(u.x), bf16hi_to_f32(u.x), bf16lo_to_f32(u.y), bf16hi_to_f32(u.y));
}

// Token of row `row` of an embedding gather.  Plain form: tokens[row * stride].  Step form (pending != nullptr): row
// = b * q + rr stands for block position r = rr + r0 of sequence b, whose token is pending[b] for r = 0 and
// follow[b * gamma + r - 1] after that (the draft, or forced, tokens): no separate kernel has to lay the block's
// tokens out first.
// Shifted form (shift_pos or shift_mode): tokens is [B, n_tokens]; row = b * q + rr reads token index
// (shift_pos ? shift_pos[b] : 0) + fixed + rr - shift of sequence b; a negative index means "no token" (-1 is
// returned and the row is all zeros), an index past the end is clamped.
struct TokenSrc {
  const int32_t* tokens;
  long long stride;
  const int32_t *pending, *follow;
  int gamma, q, r0;
  const int32_t* shift_pos;
  int shift_mode, fixed, shift;
  long long n_tokens;
};
__device__ __forceinline__ int token_of(const TokenSrc& t, int row) {
  if (t.shift_mode) {
    const int b = row / t.q, rr = row % t.q;
    long long idx = (long long)(t.shift_pos ? t.shift_pos[b] : 0) + t.fixed + rr - t.shift;
    if (idx < 0) return -1;
    idx = idx < t.n_tokens ? idx : t.n_tokens - 1;
    return t.tokens[(long long)b * t.n_tokens + idx];
  }
  if (!t.pending) return t.tokens[(long long)row * t.stride];
  const int b = row / t.q, r = row % t.q + t.r0;
  return r == 0 ? t.pending[b] : t.follow[(long long)b * t.gamma + r - 1];
}

// x[row] = emb[token(row)]; and, when g is given, xn[row] = RMSNorm(x[row]; g) - the input of the first layer's
// first product.  One workgroup per row.  init_B > 0 (first draft run of a step, one row per sequence): the
// workgroup of sequence b also writes ncur[r][b] = r + 1 for r < init_gamma (own-block rows visible to draft run r)
// and clears stop[b] (adaptive block length: nobody has stopped).
template <typename T>
__global__ __launch_bounds__(256) void embed_norm_kernel(const T* __restrict__ emb, TokenSrc src, T* __restrict__ x,
                                                         const T* __restrict__ g, T* __restrict__ xn, int d, int vocab,
                                                         float eps, int32_t* ncur, int32_t* stop, int init_B,
                                                         int init_gamma, int32_t* active, const int32_t* gate) {
  __shared__ float red[4];
  const int row = blockIdx.x;
  if (gate && *gate == 0) return;  // the caller's flag says nobody needs this launch
  if (init_B > 0) {
    if ((int)threadIdx.x < init_gamma) ncur[(long long)threadIdx.x * init_B + row] = threadIdx.x + 1;
    if (stop && threadIdx.x == 0) stop[row] = 0;
    if (active && row == 0 && (int)threadIdx.x < init_gamma) active[threadIdx.x] = 0;
  }
  int t = token_of(src, row);
  if (src.shift_mode && t < 0) {  // a row without a token: zeros (its norm is zero as well)
    for (int i = threadIdx.x; i < d; i += 256) {
      x[(long long)row * d + i] = from_f32<T>(0.f);
      if (g) xn[(long long)row * d + i] = from_f32<T>(0.f);
    }
    return;
  }
  t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
  const T* er = emb + (long long)t * d;
  T* xr = x + (long long)row * d;
  float ss = 0.f;
  const bool vec = (d & 3) == 0;
  if (vec) {
    for (int i = threadIdx.x * 4; i < d; i += 1024) {
      const float4 v = load4(er + i);
      store4(xr + i, v);
      ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
  } else {
    for (int i = threadIdx.x; i < d; i += 256) {
      const T e = er[i];
      xr[i] = e;
      const float v = to_f32<T>(e);
      ss += v * v;
    }
  }
  if (!g) return;
  for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float inv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
  T* yr = xn + (long long)row * d;
  if (vec) {
    for (int i = threadIdx.x * 4; i < d; i += 1024) {
      const float4 v = load4(er + i), gg = load4(g + i);
      store4(yr + i, make_float4(v.x * inv * gg.x, v.y * inv * gg.y, v.z * inv * gg.z, v.w * inv * gg.w));
    }
  } else {
    for (int i = threadIdx.x; i < d; i += 256) yr[i] = from_f32<T>(to_f32<T>(er[i]) * inv * to_f32<T>(g[i]));
  }
}

template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const T* __restrict__ x, const T* __restrict__ g, T* __restrict__ y,
                                                      int d, float eps) {
  __shared__ float red[4];
  const long long row = blockIdx.x;
  const T* xr = x + row * d;
  float ss = 0.f;
  const bool vec = (d & 3) == 0;
  if (vec) {
    for (int i = threadIdx.x * 4; i < d; i += 1024) {
      const float4 v = load4(xr + i);
      ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
  } else {
    for (int i = threadIdx.x; i < d; i += 256) {
      const float v = to_f32<T>(xr[i]);
      ss += v * v;
    }
  }
  for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = red[0] + red[1] + red[2] + red[3];
  const float inv = 1.0f / sqrtf(tot / (float)d + eps);
  if (vec) {
    for (int i = threadIdx.x * 4; i < d; i += 1024) {
      const float4 v = load4(xr + i), gg = load4(g + i);
      store4(y + row * d + i, make_float4(v.x * inv * gg.x, v.y * inv * gg.y, v.z * inv * gg.z, v.w * inv * gg.w));
    }
  } else {
    for (int i = threadIdx.x; i < d; i += 256) y[row * d + i] = from_f32<T>(to_f32<T>(xr[i]) * inv * to_f32<T>(g[i]));
  }
}

// qkv rows [rows, (Hq + 2 Hkv) dh] -> q [rows, Hq dh] (contiguous) and K/V rows into a cache
// [B, Hkv, cap, dh] at position pos = base[b] (or 0) + fixed + (row % q_len).
template <typename T>
__global__ void scatter_qkv_kernel(const T* __restrict__ qkv, T* __restrict__ q, T* __restrict__ kc, T* __restrict__ vc,
                                   const int32_t* __restrict__ base, int fixed, int q_len, int Hq, int Hkv, int dh,
                                   long long cap, int q_off_cols, int kv_off_cols, int row_cols) {
  const int row = blockIdx.x;
  const int b = row / q_len, r = row % q_len;
  const T* src = qkv + (long long)row * row_cols;
  if (q) {
    T* qd = q + (long long)row * Hq * dh;
    for (int i = threadIdx.x; i < Hq * dh; i += blockDim.x) qd[i] = src[q_off_cols + i];
  }
  long long pos = (base ? base[b] : 0) + fixed + r;
  if (pos < 0 || pos >= cap) return;  // never write outside the cache
  for (int i = threadIdx.x; i < Hkv * dh; i += blockDim.x) {
    const int kvh = i / dh, e = i % dh;
    const long long dst = (((long long)b * Hkv + kvh) * cap + pos) * dh + e;
    kc[dst] = src[kv_off_cols + i];
    vc[dst] = src[kv_off_cols + Hkv * dh + i];
  }
}

// greedy token per row; ties go to the lowest id.  One workgroup of 1024 lanes per row; a lane has up to eight 8- or
// 16-byte loads of the row in flight before it compares anything (the row is read once, and a row of 32768 logits
// is only 64 KB: the kernel's time is the latency of its loads).
template <typename T>
__global__ __launch_bounds__(1024) void argmax_kernel(const T* __restrict__ logits, int vocab, int32_t* __restrict__ out,
                                                      long long out_stride, const int32_t* gate) {
  __shared__ float sv[16];
  __shared__ int si[16];
  if (gate && *gate == 0) return;  // the caller's flag says nobody needs this launch
  const long long row = blockIdx.x;
  const T* lr = logits + row * vocab;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  auto consider = [&](float v, int i) __attribute__((always_inline)) {
    if (v > best || (v == best && i < bi)) {
      best = v;
      bi = i;
    }
  };
  if ((vocab & 3) == 0) {
    for (int base = threadIdx.x * 4; base < vocab; base += 8 * 4096) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = base + u * 4096;
        v[u] = i < vocab ? load4(lr + i) : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = base + u * 4096;
        if (i < vocab) {
          consider(v[u].x, i);
          consider(v[u].y, i + 1);
          consider(v[u].z, i + 2);
          consider(v[u].w, i + 3);
        }
      }
    }
  } else {
    for (int i = threadIdx.x; i < vocab; i += 1024) consider(to_f32<T>(lr[i]), i);
  }
  for (int off = 32; off >= 1; off >>= 1) {
    const float ov = __shfl_xor(best, off);
    const int oi = __shfl_xor(bi, off);
    if (ov > best || (ov == best && oi < bi)) {
      best = ov;
      bi = oi;
    }
  }
  if ((threadIdx.x & 63) == 0) {
    sv[threadIdx.x >> 6] = best;
    si[threadIdx.x >> 6] = bi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 16; ++w)
      if (sv[w] > best || (sv[w] == best && si[w] < bi)) {
        best = sv[w];
        bi = si[w];
      }
    out[row * out_stride] = bi == 0x7fffffff ? 0 : bi;
  }
}

// Finishes a deferred GEMM for one row per workgroup: v = sum_s part[s][row][:] (+ bias) (+ residual);
// x_out = v (storage dtype; also x_out2 when given); if g: xn_out = v / sqrt(mean(v^2) + eps) * g.  Partials are summed in split
// order.  Up to 1024 threads per row, each owning NV groups of four consecutive columns held in registers,
// so the row is read once.
constexpr int FIN_NV = 4;  // column groups per thread: rows up to 1024 * 4 * FIN_NV = 16384 wide

template <typename T>
__global__ __launch_bounds__(1024) void finish_norm_kernel(const float* __restrict__ part, int splits, long long MN,
                                                           const T* __restrict__ bias, const T* residual, T* x_out,
                                                           T* __restrict__ x_out2, const T* __restrict__ g,
                                                           T* __restrict__ xn_out, int d, float eps, const int32_t* gate) {
  __shared__ float red[16];
  if (gate && *gate == 0) return;  // the caller's flag says nobody needs this launch
  const long long row = blockIdx.x;
  const float* pr = part + row * d;
  const int stride = blockDim.x * 4;
  float4 v[FIN_NV];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < FIN_NV; ++i) {
    const int c = threadIdx.x * 4 + i * stride;
    v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < d) {
      for (int s = 0; s < splits; ++s) {
        const float4 t = load4(pr + s * MN + c);
        v[i].x += t.x;
        v[i].y += t.y;
        v[i].z += t.z;
        v[i].w += t.w;
      }
      if (bias) {
        const float4 t = load4(bias + c);
        v[i].x += t.x;
        v[i].y += t.y;
        v[i].z += t.z;
        v[i].w += t.w;
      }
      if (residual) {
        const float4 t = load4(residual + row * d + c);
        v[i].x += t.x;
        v[i].y += t.y;
        v[i].z += t.z;
        v[i].w += t.w;
      }
      ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
    }
  }
  float inv = 0.f;
  if (g) {
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) tot += red[w];
    inv = 1.0f / sqrtf(tot / (float)d + eps);
  }
#pragma unroll
  for (int i = 0; i < FIN_NV; ++i) {
    const int c = threadIdx.x * 4 + i * stride;
    if (c < d) {
      store4(x_out + row * d + c, v[i]);
      if (x_out2) store4(x_out2 + row * d + c, v[i]);
      if (g) {
        const float4 gg = load4(g + c);
        store4(xn_out + row * d + c,
               make_float4(v[i].x * inv * gg.x, v[i].y * inv * gg.y, v[i].z * inv * gg.z, v[i].w * inv * gg.w));
      }
    }
  }
}

// Finishes a deferred QKV (or KV) GEMM: sums the partials of one row and writes the query part to the
// contiguous q buffer and the key / value parts into the cache rows (same addressing as scatter_qkv_kernel).
template <typename T>
__global__ __launch_bounds__(1024) void finish_scatter_kernel(const float* __restrict__ part, int splits, long long MN,
                                                             T* __restrict__ q, T* __restrict__ kc, T* __restrict__ vc,
                                                             const int32_t* __restrict__ base, int fixed, int q_len,
                                                             int Hq, int Hkv, int dh, long long cap, int q_cols,
                                                             int row_cols, const int32_t* gate) {
  if (gate && *gate == 0) return;  // the caller's flag says nobody needs this launch
  const int row = blockIdx.x;
  const int b = row / q_len, r = row % q_len;
  const float* pr = part + (long long)row * row_cols;
  const long long pos = (base ? base[b] : 0) + fixed + r;
  const bool pos_ok = pos >= 0 && pos < cap;  // never write outside the cache
  for (int c = threadIdx.x * 4; c < row_cols; c += blockDim.x * 4) {
    float4 v = *reinterpret_cast<const float4*>(pr + c);
    for (int s = 1; s < splits; ++s) {
      const float4 t = *reinterpret_cast<const float4*>(pr + s * MN + c);
      v.x += t.x;
      v.y += t.y;
      v.z += t.z;
      v.w += t.w;
    }
    T* dst;
    if (c < q_cols) {
      dst = q + (long long)row * q_cols + c;
    } else {
      if (!pos_ok) continue;
      int i = c - q_cols;
      T* cache = kc;
      if (i >= Hkv * dh) {
        i -= Hkv * dh;
        cache = vc;
      }
      const int kvh = i / dh, e = i % dh;
      dst = cache + (((long long)b * Hkv + kvh) * cap + pos) * dh + e;
    }
    store4(dst, v);
  }
}

// Sec. 3.1: first location where the draft differs from M_L's token; emit the agreed prefix and
// M_L's token there; advance n by the rows that stay valid; the last emitted token becomes pending.
// draft, forced: [B, gamma]; verify, out_tokens: [B, q] with q = gamma (M_L has not seen the last draft:
// a fully accepted block emits gamma tokens) or gamma + 1 (free token, Fig. 2: always a + 1 tokens).
// With the adaptive block length (Sec. 3.1) sequence b drafted only gb = stop[b] tokens (0 = all gamma): M_L's rows
// beyond them are ignored, and gb takes gamma's place in the rule above.
__global__ void accept_kernel(const int32_t* draft, const int32_t* verify, const int32_t* forced, const int32_t* stop,
                              int32_t* out_tokens, int32_t* n_accepted, int32_t* n_drafted, int32_t* n,
                              int32_t* pending, int B, int gamma, int q, long long cap) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const bool free_token = q > gamma;
  const int gb = stop && stop[b] > 0 && stop[b] < gamma ? stop[b] : gamma;
  if (n_drafted) n_drafted[b] = gb;
  int a = 0;
  if (forced) {
    a = gamma;
    for (int r = 0; r < gamma; ++r) out_tokens[b * q + r] = forced[b * gamma + r];
    if (free_token) out_tokens[b * q + gamma] = verify[b * q + gamma];
    pending[b] = out_tokens[b * q + q - 1];
    const long long nn = (long long)n[b] + q;
    n[b] = (int32_t)(nn < 0 ? 0 : (nn > cap ? cap : nn));  // never past the caches' capacity
  } else {
    while (a < gb && draft[b * gamma + a] == verify[b * q + a]) ++a;
    const int emit = (a < gb || free_token) ? a + 1 : gb;
    for (int r = 0; r < q; ++r) {
      int t = -1;
      if (r < a) t = draft[b * gamma + r];
      else if (r == a && r < emit) t = verify[b * q + a];
      out_tokens[b * q + r] = t;
    }
    pending[b] = out_tokens[b * q + emit - 1];
    const long long nn = (long long)n[b] + emit;
    n[b] = (int32_t)(nn < 0 ? 0 : (nn > cap ? cap : nn));
  }
  n_accepted[b] = a;
}

// Deep Tandem decoding (Sec. 5, Eq. (4)): the input of M_S's run t of a step, one workgroup per sequence b.
// The run's token is tokens[b, len[b] - 1] for t = 0 (the last known token), else prev[b * gamma + t - 1], the greedy
// token of the run before, which this kernel also appends to the sequence at tokens[b, len[b] + t - 1].
// x[b] = emb[token] + add[(b * gamma + t)] (FF_DeepTandem of the row's sketch), and, when g is given,
// xn[b] = RMSNorm(x[b]; g) from the unrounded sum.
template <typename T>
__global__ __launch_bounds__(256) void deep_input_kernel(const T* __restrict__ emb, int32_t* tokens, long long n_tokens,
                                                         const int32_t* __restrict__ len, int t,
                                                         const int32_t* __restrict__ prev, int gamma,
                                                         const T* __restrict__ add, T* __restrict__ x,
                                                         const T* __restrict__ g, T* __restrict__ xn, int d, int vocab,
                                                         float eps) {
  __shared__ float red[4];
  const int b = blockIdx.x;
  const long long at = (long long)len[b] + t - 1;  // position of the run's input token
  int tok;
  if (t == 0) {
    const long long i = at < 0 ? 0 : (at < n_tokens ? at : n_tokens - 1);
    tok = tokens[(long long)b * n_tokens + i];
  } else {
    tok = prev[(long long)b * gamma + t - 1];
    if (threadIdx.x == 0 && at >= 0 && at < n_tokens) tokens[(long long)b * n_tokens + at] = tok;
  }
  tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
  const T* er = emb + (long long)tok * d;
  const T* ar = add + ((long long)b * gamma + t) * d;
  T* xr = x + (long long)b * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float v = to_f32<T>(er[i]) + to_f32<T>(ar[i]);
    xr[i] = from_f32<T>(v);
    ss += v * v;
  }
  if (!g) return;
  for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float inv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
  T* yr = xn + (long long)b * d;
  for (int i = threadIdx.x; i < d; i += 256)
    yr[i] = from_f32<T>((to_f32<T>(er[i]) + to_f32<T>(ar[i])) * inv * to_f32<T>(g[i]));
}

// End of a Deep Tandem decoding step: the last run's token joins the sequence and len[b] advances by gamma, never
// past cap.
__global__ void deep_advance_kernel(int32_t* tokens, long long n_tokens, int32_t* len, const int32_t* prev, int B,
                                    int gamma, long long cap) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const long long at = (long long)len[b] + gamma - 1;
  if (at >= 0 && at < n_tokens) tokens[(long long)b * n_tokens + at] = prev[(long long)b * gamma + gamma - 1];
  const long long nn = (long long)len[b] + gamma;
  len[b] = (int32_t)(nn < 0 ? 0 : (nn > cap ? cap : nn));
}

__global__ void fill_i32_kernel(int32_t* p, int32_t v, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ void advance_kernel(int32_t* n, int B, int by, long long cap) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const long long nn = (long long)n[b] + by;
  n[b] = (int32_t)(nn < 0 ? 0 : (nn > cap ? cap : nn));
}

}  // namespace

int launch_fill_i32(int32_t* p, int32_t v, int n, hipStream_t st) {
  hipLaunchKernelGGL(fill_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, v, n);
  return hip_ok(hipGetLastError());
}

int launch_advance(int32_t* n, int B, int by, int64_t cap, hipStream_t st) {
  hipLaunchKernelGGL(advance_kernel, dim3((B + 63) / 64), dim3(64), 0, st, n, B, by, (long long)cap);
  return hip_ok(hipGetLastError());
}

int launch_embed_norm(const void* emb, const int32_t* tokens, int64_t tok_stride, const int32_t* pending,
                      const int32_t* follow, int gamma, int q, int r0, void* x, const void* g, void* xn, int rows, int d,
                      int vocab, float eps, int32_t* ncur, int32_t* stop, int init_B, int init_gamma, int dtype,
                      hipStream_t st, int32_t* active, const int32_t* gate) {
  if (init_gamma > 256) return TANDEM_ERR_UNSUPPORTED;
  TokenSrc src{tokens, (long long)tok_stride, pending, follow, gamma, q > 0 ? q : 1, r0, nullptr, 0, 0, 0, 0};
  if (dtype == TANDEM_BF16)
    hipLaunchKernelGGL(embed_norm_kernel<bf16_t>, dim3(rows), dim3(256), 0, st, (const bf16_t*)emb, src, (bf16_t*)x,
                       (const bf16_t*)g, (bf16_t*)xn, d, vocab, eps, ncur, stop, init_B, init_gamma, active, gate);
  else
    hipLaunchKernelGGL(embed_norm_kernel<float>, dim3(rows), dim3(256), 0, st, (const float*)emb, src, (float*)x,
                       (const float*)g, (float*)xn, d, vocab, eps, ncur, stop, init_B, init_gamma, active, gate);
  return hip_ok(hipGetLastError());
}

int launch_embed_shifted(const void* emb, const int32_t* tokens, int64_t n_tokens, const int32_t* pos, int fixed,
                         int shift, int q, void* x, const void* g, void* xn, int rows, int d, int vocab, float eps,
                         int dtype, hipStream_t st) {
  TokenSrc src{tokens, 0, nullptr, nullptr, 0, q > 0 ? q : 1, 0, pos, 1, fixed, shift, (long long)n_tokens};
  if (dtype == TANDEM_BF16)
    hipLaunchKernelGGL(embed_norm_kernel<bf16_t>, dim3(rows), dim3(256), 0, st, (const bf16_t*)emb, src, (bf16_t*)x,
                       (const bf16_t*)g, (bf16_t*)xn, d, vocab, eps, nullptr, nullptr, 0, 0, nullptr, nullptr);
  else
    hipLaunchKernelGGL(embed_norm_kernel<float>, dim3(rows), dim3(256), 0, st, (const float*)emb, src, (float*)x,
                       (const float*)g, (float*)xn, d, vocab, eps, nullptr, nullptr, 0, 0, nullptr, nullptr);
  return hip_ok(hipGetLastError());
}

int launch_deep_input(const void* emb, int32_t* tokens, int64_t n_tokens, const int32_t* len, int t, const int32_t* prev,
                      int gamma, const void* add, void* x, const void* g, void* xn, int B, int d, int vocab, float eps,
                      int dtype, hipStream_t st) {
  if (dtype == TANDEM_BF16)
    hipLaunchKernelGGL(deep_input_kernel<bf16_t>, dim3(B), dim3(256), 0, st, (const bf16_t*)emb, tokens,
                       (long long)n_tokens, len, t, prev, gamma, (const bf16_t*)add, (bf16_t*)x, (const bf16_t*)g,
                       (bf16_t*)xn, d, vocab, eps);
  else
    hipLaunchKernelGGL(deep_input_kernel<float>, dim3(B), dim3(256), 0, st, (const float*)emb, tokens,
                       (long long)n_tokens, len, t, prev, gamma, (const float*)add, (float*)x, (const float*)g, (float*)xn,
                       d, vocab, eps);
  return hip_ok(hipGetLastError());
}

int launch_deep_advance(int32_t* tokens, int64_t n_tokens, int32_t* len, const int32_t* prev, int B, int gamma, int64_t cap,
                        hipStream_t st) {
  hipLaunchKernelGGL(deep_advance_kernel, dim3((B + 63) / 64), dim3(64), 0, st, tokens, (long long)n_tokens, len, prev, B,
                     gamma, (long long)cap);
  return hip_ok(hipGetLastError());
}

int launch_rmsnorm(const void* x, const void* g, void* y, int rows, int d, float eps, int dtype, hipStream_t st) {
  if (dtype == TANDEM_BF16)
    hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, dim3(rows), dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)g,
                       (bf16_t*)y, d, eps);
  else
    hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(rows), dim3(256), 0, st, (const float*)x, (const float*)g, (float*)y,
                       d, eps);
  return hip_ok(hipGetLastError());
}

int launch_finish_norm(const float* part, int splits, const void* bias, const void* residual, void* x_out,
                       const void* g, void* xn_out, int rows, int d, float eps, int dtype, hipStream_t st, void* x_out2,
                       const int32_t* gate) {
  if (d % 4 != 0 || d > 1024 * 4 * FIN_NV) return TANDEM_ERR_UNSUPPORTED;
  const long long MN = (long long)rows * d;
  int threads = (d / 4 + 63) / 64 * 64;
  threads = threads > 1024 ? 1024 : threads;
  if (dtype == TANDEM_BF16)
    hipLaunchKernelGGL(finish_norm_kernel<bf16_t>, dim3(rows), dim3(threads), 0, st, part, splits, MN, (const bf16_t*)bias,
                       (const bf16_t*)residual, (bf16_t*)x_out, (bf16_t*)x_out2, (const bf16_t*)g, (bf16_t*)xn_out, d, eps, gate);
  else
    hipLaunchKernelGGL(finish_norm_kernel<float>, dim3(rows), dim3(threads), 0, st, part, splits, MN, (const float*)bias,
                       (const float*)residual, (float*)x_out, (float*)x_out2, (const float*)g, (float*)xn_out, d, eps, gate);
  return hip_ok(hipGetLastError());
}

int launch_finish_scatter(const float* part, int splits, void* q, void* kc, void* vc, const int32_t* base, int fixed,
                          int rows, int q_len, int Hq, int Hkv, int dh, int64_t cap, int q_cols, int row_cols, int dtype,
                          hipStream_t st, const int32_t* gate) {
  if (row_cols % 4 != 0 || q_cols % 4 != 0 || dh % 4 != 0) return TANDEM_ERR_UNSUPPORTED;
  const long long MN = (long long)rows * row_cols;
  int threads = (row_cols / 4 + 63) / 64 * 64;
  threads = threads > 1024 ? 1024 : threads;
  if (dtype == TANDEM_BF16)
    hipLaunchKernelGGL(finish_scatter_kernel<bf16_t>, dim3(rows), dim3(threads), 0, st, part, splits, MN, (bf16_t*)q,
                       (bf16_t*)kc, (bf16_t*)vc, base, fixed, q_len, Hq, Hkv, dh, (long long)cap, q_cols, row_cols, gate);
  else
    hipLaunchKernelGGL(finish_scatter_kernel<float>, dim3(rows), dim3(threads), 0, st, part, splits, MN, (float*)q,
                       (float*)kc, (float*)vc, base, fixed, q_len, Hq, Hkv, dh, (long long)cap, q_cols, row_cols, gate);
  return hip_ok(hipGetLastError());
}

int launch_scatter_qkv(const void* qkv, void* q, void* kc, void* vc, const int32_t* base, int fixed, int rows, int q_len,
                       int Hq, int Hkv, int dh, int64_t cap, int q_off_cols, int kv_off_cols, int row_cols, int dtype,
                       hipStream_t st) {
  if (dtype == TANDEM_BF16)
    hipLaunchKernelGGL(scatter_qkv_kernel<bf16_t>, dim3(rows), dim3(256), 0, st, (const bf16_t*)qkv, (bf16_t*)q,
                       (bf16_t*)kc, (bf16_t*)vc, base, fixed, q_len, Hq, Hkv, dh, (long long)cap, q_off_cols,
                       kv_off_cols, row_cols);
  else
    hipLaunchKernelGGL(scatter_qkv_kernel<float>, dim3(rows), dim3(256), 0, st, (const float*)qkv, (float*)q, (float*)kc,
                       (float*)vc, base, fixed, q_len, Hq, Hkv, dh, (long long)cap, q_off_cols, kv_off_cols, row_cols);
  return hip_ok(hipGetLastError());
}

int launch_argmax(const void* logits, int rows, int vocab, int32_t* out, int64_t out_stride, int dtype, hipStream_t st,
                  const int32_t* gate) {
  if (dtype == TANDEM_BF16)
    hipLaunchKernelGGL(argmax_kernel<bf16_t>, dim3(rows), dim3(1024), 0, st, (const bf16_t*)logits, vocab, out,
                       (long long)out_stride, gate);
  else
    hipLaunchKernelGGL(argmax_kernel<float>, dim3(rows), dim3(1024), 0, st, (const float*)logits, vocab, out,
                       (long long)out_stride, gate);
  return hip_ok(hipGetLastError());
}

int launch_accept(const int32_t* draft, const int32_t* verify, const int32_t* forced, const int32_t* stop,
                  int32_t* out_tokens, int32_t* n_accepted, int32_t* n_drafted, int32_t* n, int32_t* pending, int B,
                  int gamma, int q, int64_t cap, hipStream_t st) {
  hipLaunchKernelGGL(accept_kernel, dim3((B + 63) / 64), dim3(64), 0, st, draft, verify, forced, stop, out_tokens,
                     n_accepted, n_drafted, n, pending, B, gamma, q, (long long)cap);
  return hip_ok(hipGetLastError());
}
