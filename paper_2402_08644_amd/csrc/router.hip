// Router of the adaptive block length (Sec. 3.1 "Adaptive Block Length"; threshold tau = 0.8 in Sec. 4): after every
// draft token a 2-layer MLP looks at M_S's output distribution and decides whether M_S goes on drafting or M_L
// verifies now.  One workgroup per sequence computes, from the logits row of the current draft run,
//   * the entropy of the distribution over the vocabulary (nats),
//   * its k largest probabilities, descending, equal logits in id order,
//   * M_S's embedding rows of those k tokens,
// concatenated in this order into the feature vector f (1 + k + k d numbers, kept in LDS), then
//   p = sigmoid(w2 . relu(W1 f + b1) + b2)
// - the predicted probability that M_L accepts the token - and records the first draft run whose p is below tau.
// All arithmetic in fp32 whatever the storage type.
#include "common.h"
#include "glue.h"
#include "kernels.h"

namespace {

constexpr int RT_THREADS = 1024, RT_WAVES = RT_THREADS / 64;

__device__ __forceinline__ float wave_sum(float v) {
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// REG: the logits row (at most 32 * 1024 tokens) is read once into 32 registers per lane and all passes run from
// them; otherwise every pass re-reads the row.
template <typename T, bool REG>
__global__ __launch_bounds__(RT_THREADS) void router_kernel(const T* __restrict__ logits, const T* __restrict__ emb,
                                                            const T* __restrict__ W1, const T* __restrict__ b1,
                                                            const T* __restrict__ w2, const T* __restrict__ b2, int vocab,
                                                            int d, int k, int hidden, float tau, int run,
                                                            int32_t* __restrict__ stop, float* __restrict__ p_out,
                                                            long long p_stride, int32_t* __restrict__ active,
                                                            const int32_t* __restrict__ gate) {
  // gate: nobody drafts any more; a sequence that has stopped needs no further decision (its p is not written)
  if (gate && *gate == 0) return;
  if (stop && stop[blockIdx.x] != 0) return;
  extern __shared__ float f[];  // features
  __shared__ float red[RT_WAVES], red2[RT_WAVES];
  __shared__ int ids[TANDEM_ROUTER_MAX_K];
  __shared__ float cv[RT_WAVES * TANDEM_ROUTER_MAX_K];  // per-wavefront candidates of the top-k search
  __shared__ int ci[RT_WAVES * TANDEM_ROUTER_MAX_K];
  __shared__ float bc[2];
  constexpr int NPT = 32;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const long long row = blockIdx.x;
  const T* lr = logits + row * vocab;

  // token c * 1024 + tid is this lane's c-th value
  float vals[NPT];
  if (REG) {
#pragma unroll
    for (int c = 0; c < NPT; ++c) {
      const int i = c * RT_THREADS + tid;
      vals[c] = i < vocab ? to_f32<T>(lr[i]) : -INFINITY;
    }
  }
  const int npt = REG ? NPT : (vocab + RT_THREADS - 1) / RT_THREADS;
  auto val = [&](int c) -> float {
    if (REG) return vals[c];
    const int i = c * RT_THREADS + tid;
    return i < vocab ? to_f32<T>(lr[i]) : -INFINITY;
  };

  // largest logit
  float mx = -INFINITY;
#pragma unroll
  for (int c = 0; c < npt; ++c) mx = fmaxf(mx, val(c));
  for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  if (lane == 0) red[w] = mx;
  __syncthreads();
  if (tid == 0) {
    float m = red[0];
    for (int i = 1; i < RT_WAVES; ++i) m = fmaxf(m, red[i]);
    bc[0] = m;
  }
  __syncthreads();
  const float m = bc[0];

  // Z = sum e^(x - m),  A = sum e^(x - m) (x - m);  entropy = ln Z - A / Z
  float z = 0.f, a = 0.f;
#pragma unroll
  for (int c = 0; c < npt; ++c) {
    const float t = val(c) - m;
    const float e = expf(t);  // 0 for the padding (-inf)
    z += e;
    a += e > 0.f ? e * t : 0.f;
  }
  z = wave_sum(z);
  a = wave_sum(a);
  if (lane == 0) {
    red[w] = z;
    red2[w] = a;
  }
  __syncthreads();
  if (tid == 0) {
    float zs = 0.f, as = 0.f;
    for (int i = 0; i < RT_WAVES; ++i) {
      zs += red[i];
      as += red2[i];
    }
    bc[1] = zs;
    f[0] = logf(zs) - as / zs;  // fi(0) = 0
  }
  __syncthreads();
  const float Z = bc[1];

  // The k largest logits in two levels: every wavefront finds the k largest of its own 64 x npt values (k rounds of a
  // wavefront-wide argmax, no workgroup barrier; REG: bit c of `mine` marks this lane's c-th value as taken), then
  // wavefront 0 finds the k largest of the 16 k candidates.  Equal logits go by the lower id at both levels.
  constexpr int NONE = 0x7fffffff;
  auto wave_argmax = [&](float& best, int& bi) {
    for (int off = 32; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(best, off);
      const int oi = __shfl_xor(bi, off);
      if (oi != NONE && (bi == NONE || ov > best || (ov == best && oi < bi))) {
        best = ov;
        bi = oi;
      }
    }
  };
  uint32_t mine = 0;
  for (int t = 0; t < k; ++t) {
    float best = -INFINITY;
    int bi = NONE;
#pragma unroll
    for (int c = 0; c < npt; ++c) {
      const int i = c * RT_THREADS + tid;
      bool taken = i >= vocab;
      if (REG) {
        taken |= (mine >> c) & 1u;
      } else {
        for (int u = 0; u < t; ++u) taken |= ci[w * TANDEM_ROUTER_MAX_K + u] == i;
      }
      const float v = val(c);
      if (!taken && (bi == NONE || v > best)) {  // ids grow with c: a later equal value does not replace
        best = v;
        bi = i;
      }
    }
    wave_argmax(best, bi);
    if (lane == 0) {
      cv[w * TANDEM_ROUTER_MAX_K + t] = best;
      ci[w * TANDEM_ROUTER_MAX_K + t] = bi;
    }
    if (REG && bi != NONE && (bi & (RT_THREADS - 1)) == tid) mine |= 1u << (bi / RT_THREADS);
  }
  __syncthreads();
  if (w == 0) {
    // candidate slots lane and lane + 64 of the 16 x MAX_K table (rounds t >= k of a wavefront were not filled)
    float v0 = -INFINITY, v1 = -INFINITY;
    int i0 = NONE, i1 = NONE;
    if ((lane & (TANDEM_ROUTER_MAX_K - 1)) < k) {
      v0 = cv[lane];
      i0 = ci[lane];
      v1 = cv[lane + 64];
      i1 = ci[lane + 64];
    }
    for (int t = 0; t < k; ++t) {
      float best = v0;
      int bi = i0;
      if (i1 != NONE && (bi == NONE || v1 > best || (v1 == best && i1 < bi))) {
        best = v1;
        bi = i1;
      }
      wave_argmax(best, bi);
      if (lane == 0) {
        ids[t] = bi;
        f[((1 + t) & 7) * ((1 + k + k * d + 7) / 8 + 1) + ((1 + t) >> 3)] = expf(best - m) / Z;  // fi(1 + t)
      }
      if (i0 == bi) i0 = NONE;
      if (i1 == bi) i1 = NONE;
    }
  }
  __syncthreads();

  // Feature j lives at f[fi(j)], fi(j) = (j % 8) * FS + j / 8: lanes that take consecutive 16-byte pieces of a row
  // of W1 (8 or 4 consecutive features each) then read consecutive LDS words, whatever the row's alignment.
  const int F = 1 + k + k * d;
  const int FS = (F + 7) / 8 + 1;
  auto fi = [&](int j) { return (j & 7) * FS + (j >> 3); };
  for (int idx = tid; idx < k * d; idx += RT_THREADS)
    f[fi(1 + k + idx)] = to_f32<T>(emb[(long long)ids[idx / d] * d + idx % d]);
  __syncthreads();

  // hidden layer: unit i belongs to wavefront i % 16, eight units at a time per wavefront (eight independent rows of
  // W1 in flight per lane).  Rows 16 apart start 32 F bytes apart, a multiple of 16: all rows of a wavefront have the
  // same alignment, so they share the split into an aligned middle part read with 16-byte loads (each lane's 8 or 4
  // features read from LDS once for all eight rows) and up to 15 bytes before and after it read element by element.
  constexpr int UN = 8, VEC = 16 / (int)sizeof(T);
  int head = (int)(((16 - ((uintptr_t)(W1 + (long long)w * F) & 15)) & 15) / sizeof(T));
  head = head < F ? head : F;
  const int nvec = (F - head) / VEC;
  const int tail = head + nvec * VEC + lane;  // this lane's element after the middle part (if < F)
  float zacc = 0.f;
  for (int i0 = w; i0 < hidden; i0 += RT_WAVES * UN) {
    float dot[UN];
    const T* wr[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int i = i0 + u * RT_WAVES;
      wr[u] = W1 + (long long)(i < hidden ? i : i0) * F;  // a unit past the end re-reads a valid row, not used
      dot[u] = 0.f;
    }
    for (int v = lane; v < nvec; v += 64) {
      const int j = head + v * VEC;
      uint4 raw[UN];
#pragma unroll
      for (int u = 0; u < UN; ++u) raw[u] = *reinterpret_cast<const uint4*>(wr[u] + j);
      float fv[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) fv[e] = f[fi(j + e)];
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const uint32_t rw[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
        float acc = dot[u];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (sizeof(T) == 2) {
            acc = fmaf(bf16lo_to_f32(rw[e]), fv[(2 * e) % VEC], acc);
            acc = fmaf(bf16hi_to_f32(rw[e]), fv[(2 * e + 1) % VEC], acc);
          } else {
            acc = fmaf(__uint_as_float(rw[e]), fv[e % VEC], acc);
          }
        }
        dot[u] = acc;
      }
    }
    if (lane < head) {
      const float fl = f[fi(lane)];
#pragma unroll
      for (int u = 0; u < UN; ++u) dot[u] = fmaf(to_f32<T>(wr[u][lane]), fl, dot[u]);
    }
    if (tail < F) {
      const float ft = f[fi(tail)];
#pragma unroll
      for (int u = 0; u < UN; ++u) dot[u] = fmaf(to_f32<T>(wr[u][tail]), ft, dot[u]);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int i = i0 + u * RT_WAVES;
      const float sdot = wave_sum(dot[u]);
      if (i < hidden) {
        const float h = fmaxf(sdot + (b1 ? to_f32<T>(b1[i]) : 0.f), 0.f);
        zacc = fmaf(to_f32<T>(w2[i]), h, zacc);
      }
    }
  }
  if (lane == 0) red[w] = zacc;
  __syncthreads();
  if (tid == 0) {
    float zs = b2 ? to_f32<T>(b2[0]) : 0.f;
    for (int i = 0; i < RT_WAVES; ++i) zs += red[i];
    const float p = 1.f / (1.f + expf(-zs));
    if (p_out) p_out[row * p_stride] = p;
    if (stop && p < tau) stop[row] = run + 1;
    else if (active) atomicAdd(active + run, 1);  // still drafting after this run
  }
}

template <typename T>
void launch_router_t(const tandem_router_desc* r, const void* logits, const void* emb, int rows, int vocab, int d, int run,
                     int32_t* stop, float* p_out, int64_t p_stride, size_t lds, hipStream_t st, int32_t* active,
                     const int32_t* gate) {
  if (vocab <= 32 * RT_THREADS)
    hipLaunchKernelGGL((router_kernel<T, true>), dim3(rows), dim3(RT_THREADS), lds, st, (const T*)logits, (const T*)emb,
                       (const T*)r->W1, (const T*)r->b1, (const T*)r->w2, (const T*)r->b2, vocab, d, r->k, r->d_hidden,
                       r->tau, run, stop, p_out, (long long)p_stride, active, gate);
  else
    hipLaunchKernelGGL((router_kernel<T, false>), dim3(rows), dim3(RT_THREADS), lds, st, (const T*)logits, (const T*)emb,
                       (const T*)r->W1, (const T*)r->b1, (const T*)r->w2, (const T*)r->b2, vocab, d, r->k, r->d_hidden,
                       r->tau, run, stop, p_out, (long long)p_stride, active, gate);
}

}  // namespace

int check_router(const tandem_router_desc* r, int d) {
  if (!r) return TANDEM_ERR_NULL;
  if (!r->W1 || !r->w2) return TANDEM_ERR_NULL;
  if (r->dtype != TANDEM_F32 && r->dtype != TANDEM_BF16) return TANDEM_ERR_UNSUPPORTED;
  if (r->k < 1 || r->k > TANDEM_ROUTER_MAX_K || r->d_hidden < 1 || d < 1) return TANDEM_ERR_SHAPE;
  if (8 * ((1 + (int64_t)r->k * (d + 1) + 7) / 8 + 1) * sizeof(float) > 64 * 1024) return TANDEM_ERR_UNSUPPORTED;
  return TANDEM_OK;
}

int launch_router(const tandem_router_desc* r, const void* logits, const void* emb, int rows, int vocab, int d, int run,
                  int32_t* stop, float* p_out, int64_t p_stride, hipStream_t st, int32_t* active, const int32_t* gate) {
  const size_t lds = 8 * ((1 + (size_t)r->k * (d + 1) + 7) / 8 + 1) * sizeof(float);  // features, see fi() in the kernel
  if (r->dtype == TANDEM_BF16)
    launch_router_t<bf16_t>(r, logits, emb, rows, vocab, d, run, stop, p_out, p_stride, lds, st, active, gate);
  else
    launch_router_t<float>(r, logits, emb, rows, vocab, d, run, stop, p_out, p_stride, lds, st, active, gate);
  return hip_ok(hipGetLastError());
}

extern "C" int tandem_router_eval(const tandem_router_desc* r, const void* logits, const void* emb, int32_t rows,
                                  int32_t vocab, int32_t d, float* p_out, void* hip_stream) {
  int rc = check_router(r, d);
  if (rc != TANDEM_OK) return rc;
  if (!logits || !emb || !p_out) return TANDEM_ERR_NULL;
  if (rows < 1 || vocab < r->k) return TANDEM_ERR_SHAPE;
  return launch_router(r, logits, emb, rows, vocab, d, 0, nullptr, p_out, 1, (hipStream_t)hip_stream);
}
