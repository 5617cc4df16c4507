// Streaming softmax attention on the vector ALUs: the mixed-source small-model attention
// of Eq. (2) (second line) - one query per head over [K_hat rows of completed blocks ;
// own rows of the current block] - and the generic (fp32 / dh = 64) form of the block-mode
// pass of Eq. (1).  Arithmetic intensity is 1 flop per KV byte, so the kernel is a pure
// HBM stream: every K and V row is read exactly once, 16 lanes per 256-byte row, four rows
// (1 KiB, contiguous) per load instruction.
//
// Work split: grid (S context splits, Hkv * q_len, B); 4 wavefronts per workgroup, each
// quarter-wavefront (one DPP row of 16 lanes) owns whole key rows and keeps a private
// online-softmax state (m, l, acc), so the main loop has no cross-row communication apart
// from the 4-step DPP dot-product reduction.  States are merged once at the end: DPP rows
// inside the wavefront, wavefronts through LDS, splits through the workspace in fixed order.
#include "common.h"
#include "kernels.h"

namespace {

struct RowsParams {
  const void* q;
  const void *kA, *vA, *kB, *vB;
  const int32_t *nA, *nB;
  int causal, Hq, Hkv, q_len, gamma_max, S;
  int S_total, s_off;  // partial slots per row and this launch's first slot
  long long row_skip;  // q / out hold (q_len * Hq + row_skip) rows per sequence
  int n_off;           // added to nA[b]
  const int32_t* skip;  // optional [B]: a sequence with skip[b] != 0 is not processed, its output rows are zero
  int mixed_gamma;     // > 0: all-positions small-model attention with this block length (see below)
  long long T_max;
  float scale_log2e;
  void* out;
  float* part_ml;
  float* part_o;
};

// NW wavefronts per workgroup (4 or 8): eight put the work of two context splits into one workgroup, whose
// wavefronts merge through LDS, so that no partials leave the workgroup and no combine kernel follows.
template <typename T, int DH, int G, int U, int NW>
__global__ __launch_bounds__(64 * NW) void attn_rows_kernel(RowsParams p) {
  constexpr int EPL = DH / 16;  // elements of a row per lane
  constexpr int RB = EPL * (int)sizeof(T);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int sub = lane >> 4, t = lane & 15;
  const int s = blockIdx.x, b = blockIdx.z;
  const int kvh = blockIdx.y % p.Hkv, r = blockIdx.y / p.Hkv;

  long long nA = (long long)p.nA[b] + p.n_off;
  long long nB = 0;
  long long strideB = p.gamma_max;  // rows per (sequence, head) of source B
  if (p.mixed_gamma > 0) {
    // Eq. (2) at position i = n + r: rows [0, kb) of A (derived from the large model), rows [kb, i] of B (own rows,
    // a cache indexed by position), kb = floor(i / gamma) * gamma
    const long long nmax = p.T_max - p.q_len;
    nA = nA < 0 ? 0 : (nA > nmax ? nmax : nA);
    const long long i = nA + r;
    nA = i / p.mixed_gamma * p.mixed_gamma;
    nB = p.kB ? i + 1 - nA : 0;  // without source B: only the rows below the block boundary (Eq. (3))
    strideB = p.T_max;
  } else {
    if (p.causal) nA += r + 1;
    nA = nA < 0 ? 0 : (nA > p.T_max ? p.T_max : nA);
    if (p.nB) {
      nB = p.nB[b];
      nB = nB < 0 ? 0 : (nB > p.gamma_max ? p.gamma_max : nB);
    }
  }
  const long long total = nA + nB;
  long long per = (total + p.S - 1) / p.S;
  per = (per + 15) & ~15LL;
  const long long begin = (long long)s * per;
  const long long end = total < begin + per ? total : begin + per;

  const T* kA = (const T*)p.kA + ((long long)b * p.Hkv + kvh) * p.T_max * DH;
  const T* vA = (const T*)p.vA + ((long long)b * p.Hkv + kvh) * p.T_max * DH;
  // in the all-positions form row (row - nA) of B is cache row `row`: shift the base by nA rows
  const long long offB = ((long long)b * p.Hkv + kvh) * strideB * DH + (p.mixed_gamma > 0 ? nA * DH : 0);
  const T* kB = p.kB ? (const T*)p.kB + offB : nullptr;
  const T* vB = p.vB ? (const T*)p.vB + offB : nullptr;

  const long long row0 = ((long long)b * p.q_len + r) * p.Hq + (long long)kvh * G;  // first query row of the group
  if (p.skip && p.skip[b] != 0) {
    // (adaptive block length: the sequence has stopped drafting) nothing is read; zero rows, or neutral partials
    for (int idx = threadIdx.x; idx < G * DH; idx += 64 * NW) {
      const long long row = row0 + idx / DH;
      const int d = idx % DH;
      if (p.S_total == 1) {
        ((T*)p.out)[(row + b * p.row_skip) * DH + d] = from_f32<T>(0.f);
      } else {
        const long long ps = row * p.S_total + p.s_off + s;
        p.part_o[ps * DH + d] = 0.f;
        if (d == 0) {
          p.part_ml[ps * 2 + 0] = TANDEM_NEG_BIG;
          p.part_ml[ps * 2 + 1] = 0.f;
        }
      }
    }
    return;
  }
  float qv[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    Raw<RB> raw;
    raw.load((const T*)p.q + (row0 + b * p.row_skip + g) * DH + t * EPL);
    Unpack<T, EPL>::run(raw, qv[g]);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qv[g][e] *= p.scale_log2e;
  }

  float m[G], l[G], acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = TANDEM_NEG_BIG;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }

  // Iteration i of a wavefront covers the 4 U rows from begin + (i NW + w) 4 U.  The workgroups of a launch all
  // start at a multiple of the cache's per-head size and advance in step, so without further ado they would all
  // press on the same memory channels at the same time: every workgroup starts its walk at a different iteration
  // (a function of its position in the grid only) and wraps around.
  const long long nit = (end - begin + 4 * NW * U - 1) / (4 * NW * U);
  const long long rot = nit > 0 ? (long long)((blockIdx.z * 7 + blockIdx.y * 3 + blockIdx.x) * 5) % nit : 0;
  for (long long it = 0; it < nit; ++it) {
    long long ii = it + rot;
    ii = ii >= nit ? ii - nit : ii;
    const long long base = begin + (ii * NW + w) * (4 * U);
    Raw<RB> kr[U], vr[U];
    bool valid[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      long long row = base + u * 4 + sub;
      valid[u] = row < end;
      if (!valid[u]) row = begin;  // begin < end here: a readable row, its score is masked below
      const T *kp, *vp;
      if (row < nA) {
        kp = kA + row * DH;
        vp = vA + row * DH;
      } else {
        kp = kB + (row - nA) * DH;
        vp = vB + (row - nA) * DH;
      }
      kr[u].load_stream(kp + t * EPL);
      vr[u].load_stream(vp + t * EPL);
    }
    float sc[U][G];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPL];
      Unpack<T, EPL>::run(kr[u], kf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) d = fmaf(qv[g][e], kf[e], d);
        d = row16_sum(d);
        sc[u][g] = valid[u] ? d : -INFINITY;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mn = m[g];
#pragma unroll
      for (int u = 0; u < U; ++u) mn = fmaxf(mn, sc[u][g]);
      const float corr = fast_exp2(m[g] - mn);
      m[g] = mn;
      l[g] *= corr;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= corr;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float vf[EPL];
      Unpack<T, EPL>::run(vr[u], vf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float pw = fast_exp2(sc[u][g] - m[g]);
        l[g] += pw;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(pw, vf[e], acc[g][e]);
      }
    }
  }

  // merge the four DPP rows of the wavefront
#pragma unroll
  for (int off = 16; off <= 32; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float mo = __shfl_xor(m[g], off), lo = __shfl_xor(l[g], off);
      const float mn = fmaxf(m[g], mo);
      const float ca = fast_exp2(m[g] - mn), cb = fast_exp2(mo - mn);
      l[g] = l[g] * ca + lo * cb;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] = acc[g][e] * ca + __shfl_xor(acc[g][e], off) * cb;
      m[g] = mn;
    }
  }

  __shared__ float sm_m[NW][G], sm_l[NW][G];
  __shared__ float sm_o[NW][G][DH];
  if (sub == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      if (t == 0) {
        sm_m[w][g] = m[g];
        sm_l[w][g] = l[g];
      }
#pragma unroll
      for (int e = 0; e < EPL; ++e) sm_o[w][g][t * EPL + e] = acc[g][e];
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * DH; idx += 64 * NW) {
    const int g = idx / DH, d = idx % DH;
    float mn = sm_m[0][g];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) mn = fmaxf(mn, sm_m[ww][g]);
    float lt = 0.f, ot = 0.f;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) {
      const float c = fast_exp2(sm_m[ww][g] - mn);
      lt += sm_l[ww][g] * c;
      ot += sm_o[ww][g][d] * c;
    }
    const long long row = row0 + g;
    if (p.S_total == 1) {
      ((T*)p.out)[(row + b * p.row_skip) * DH + d] = from_f32<T>(lt > 0.f ? ot / lt : 0.f);
    } else {
      const long long ps = row * p.S_total + p.s_off + s;
      p.part_o[ps * DH + d] = ot;
      if (d == 0) {
        p.part_ml[ps * 2 + 0] = mn;
        p.part_ml[ps * 2 + 1] = lt;
      }
    }
  }
}

// out[row, :] = sum_s O_s 2^(m_s - m) / sum_s l_s 2^(m_s - m), splits visited in index order
template <typename T>
__global__ void attn_combine_kernel(const float* __restrict__ part_ml, const float* __restrict__ part_o, T* out,
                                    int S, int dh, int rows_per_seq, long long row_skip) {
  const long long row = blockIdx.x;
  const int d = threadIdx.x;
  float mn = TANDEM_NEG_BIG;
  for (int s = 0; s < S; ++s) mn = fmaxf(mn, part_ml[(row * S + s) * 2]);
  float lt = 0.f, ot = 0.f;
  for (int s = 0; s < S; ++s) {
    const float c = fast_exp2(part_ml[(row * S + s) * 2] - mn);
    lt += part_ml[(row * S + s) * 2 + 1] * c;
    ot += part_o[(row * S + s) * dh + d] * c;
  }
  const long long orow = rows_per_seq > 0 ? row + row / rows_per_seq * row_skip : row;
  out[orow * dh + d] = from_f32<T>(lt > 0.f ? ot / lt : 0.f);
}

template <typename T, int DH, int G, int NW>
int launch_rows_t(const RowsParams& p, dim3 grid, hipStream_t st) {
  hipLaunchKernelGGL((attn_rows_kernel<T, DH, G, 4, NW>), grid, dim3(64 * NW), 0, st, p);
  return hip_ok(hipGetLastError());
}

template <typename T, int DH>
int launch_rows_g(int G, bool wide, const RowsParams& p, dim3 grid, hipStream_t st) {
  switch (G) {
    case 1: return wide ? launch_rows_t<T, DH, 1, 8>(p, grid, st) : launch_rows_t<T, DH, 1, 4>(p, grid, st);
    case 2: return wide ? launch_rows_t<T, DH, 2, 8>(p, grid, st) : launch_rows_t<T, DH, 2, 4>(p, grid, st);
    case 4: return launch_rows_t<T, DH, 4, 4>(p, grid, st);
    case 8: return launch_rows_t<T, DH, 8, 4>(p, grid, st);
    default: return TANDEM_ERR_UNSUPPORTED;
  }
}

}  // namespace

// Context splits: a function of shapes only.  Measured on MI355X: about 512 workgroups in total (two
// per CU) stream best; more splits only add partials and tail effects.  At least 256 keys per split.
int attn_rows_splits(int B, int Hkv, int q_len, int G, int64_t T_max, int gamma_max, int* wide) {
  const int64_t groups = (int64_t)B * Hkv * q_len;
  const int64_t keys = T_max + gamma_max;
  int64_t want = (512 + groups - 1) / groups;
  int64_t cap = keys / 256;
  if (cap < 1) cap = 1;
  int64_t S = want < cap ? want : cap;
  if (S < 1) S = 1;
  if (S > 64) S = 64;
  // an even number of splits becomes half as many workgroups of eight wavefronts (query groups of 1 or 2 heads)
  const bool w8 = S % 2 == 0 && G <= 2;
  if (wide) *wide = w8 ? 1 : 0;
  return (int)(w8 ? S / 2 : S);
}

size_t attn_rows_workspace(int B, int Hq, int q_len, int dh, int S) {
  if (S <= 1) return 0;
  const size_t rows = (size_t)B * q_len * Hq;
  return rows * S * (dh + 2) * sizeof(float);
}

int launch_attn_combine(const float* part_ml, const float* part_o, void* out, int rows, int S, int dh, int dtype,
                        hipStream_t st, int rows_per_seq, long long row_skip) {
  if (dtype == TANDEM_BF16)
    hipLaunchKernelGGL(attn_combine_kernel<bf16_t>, dim3(rows), dim3(dh), 0, st, part_ml, part_o, (bf16_t*)out, S, dh,
                       rows_per_seq, row_skip);
  else
    hipLaunchKernelGGL(attn_combine_kernel<float>, dim3(rows), dim3(dh), 0, st, part_ml, part_o, (float*)out, S, dh,
                       rows_per_seq, row_skip);
  return hip_ok(hipGetLastError());
}

int launch_attn_rows(const AttnArgs& a, hipStream_t st) {
  RowsParams p;
  p.q = a.q;
  p.kA = a.kA;
  p.vA = a.vA;
  p.kB = a.kB;
  p.vB = a.vB;
  p.nA = a.nA;
  p.nB = a.nB;
  p.causal = a.causal;
  p.Hq = a.Hq;
  p.Hkv = a.Hkv;
  p.q_len = a.q_len;
  p.gamma_max = a.gamma_max;
  p.S = a.S;
  p.S_total = a.S_total > 0 ? a.S_total : a.S;
  p.s_off = a.S_total > 0 ? a.s_off : 0;
  p.row_skip = a.q_rows > a.q_len ? (long long)(a.q_rows - a.q_len) * a.Hq : 0;
  p.n_off = a.n_off;
  p.skip = a.skip;
  p.mixed_gamma = a.mixed == 3 ? (a.gamma > 0 ? a.gamma : 1) : 0;
  p.T_max = a.T_max;
  p.scale_log2e = a.scale * 1.4426950408889634f;
  p.out = a.out;
  p.part_ml = a.part_ml;
  p.part_o = a.part_o;
  const int G = a.Hq / a.Hkv;
  dim3 grid(a.S, a.Hkv * a.q_len, a.B);
  int rc;
  if (a.dtype == TANDEM_BF16 && a.dh == 128)
    rc = launch_rows_g<bf16_t, 128>(G, a.wide != 0, p, grid, st);
  else if (a.dtype == TANDEM_BF16 && a.dh == 64)
    rc = launch_rows_g<bf16_t, 64>(G, a.wide != 0, p, grid, st);
  else if (a.dtype == TANDEM_F32 && a.dh == 128)
    rc = launch_rows_g<float, 128>(G, a.wide != 0, p, grid, st);
  else if (a.dtype == TANDEM_F32 && a.dh == 64)
    rc = launch_rows_g<float, 64>(G, a.wide != 0, p, grid, st);
  else
    return TANDEM_ERR_UNSUPPORTED;
  if (rc != TANDEM_OK || a.S_total > 0 || a.S == 1) return rc;
  return launch_attn_combine(a.part_ml, a.part_o, a.out, a.B * a.q_len * a.Hq, a.S, a.dh, a.dtype, st, a.q_len * a.Hq,
                             p.row_skip);
}
