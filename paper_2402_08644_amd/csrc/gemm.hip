// Dense layers: Y[M, N] = epilogue(X[M, K] . W[N, K]^T), weights stored [out, in] so both
// operands have the contraction index contiguous - exactly the in-lane layout the matrix
// cores want, no transposes anywhere.  Used by FF_Tandem (Eq. (2), first line) and by every
// projection / MLP / output-head product of the decode step.
//
// gemm_skinny_kernel (bf16, M <= 128 per pass): the decode-time regime, bound by streaming
// the weights once from HBM.  A workgroup owns 32 output features for all rows; its
// wavefronts split the contraction range, each streaming its slice of W straight from
// global memory into the A-operand of v_mfma_f32_32x32x16_bf16 (each lane reads 64
// contiguous bytes of one weight row per 64-deep chunk, the two half-waves cover a
// 128-byte line) while the small, cache-resident X provides the B-operands.  Partial sums
// meet in LDS; the epilogue (bias, activation, residual, store) is fused when no split
// across workgroups is needed.
//
// gemm_tile_kernel / gemm_stream_kernel (bf16, 32 < M <= 128 per pass): the same regime with the X rows
// shared through LDS; the stream kernel reads weights re-laid out in contiguous operand tiles.
// gemm_big_kernel (bf16, thousands of rows): 256 x 256 tiles, both operands through LDS, compute-bound.
//
// gemm_generic_kernel: any dtype / shape, LDS-tiled on the vector ALUs (the fp32
// correctness path of the tiny configuration and odd shapes).
#include "common.h"
#include "kernels.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct GemmParams {
  const void* X;
  const void* W;
  const void* Wp;  // the same weights in the packed tile layout, or null
  const void* bias;
  const void* residual;
  void* Y;
  float* part;  // [splitK, M, N] fp32 partial sums
  long long ldx, ldr, ldy;
  int M, N, K, act, splitK, m_base, defer;
  int xcd_map;  // stream kernel: 1 = workgroup ids are mapped to (tile, split) so that a split stays on one XCD
  const int32_t* gate;  // optional device flag: *gate == 0 means nobody needs this product, the kernels return at once
};

__device__ __forceinline__ float apply_act(float v, int act) {
  if (act == TANDEM_ACT_GELU) return 0.5f * v * (1.f + erff(v * 0.70710678118654752f));
  if (act == TANDEM_ACT_RELU) return fmaxf(v, 0.f);
  return v;
}

template <typename T>
__device__ __forceinline__ float epilogue(float v, int m, int n, const GemmParams& p) {
  if (p.bias) v += to_f32<T>(((const T*)p.bias)[n]);
  v = apply_act(v, p.act);
  if (p.residual) v += to_f32<T>(((const T*)p.residual)[(long long)m * p.ldr + n]);
  return v;
}

// The MFMA kernels finish dozens of values per lane.  With the activation chosen at run time per value the
// unrolled epilogue was a chain of branches around inlined erff bodies, larger than the instruction cache
// (measured: 10 us per launch).  There the activation is a template argument, selected once per kernel by
// ACT_SWITCH, and the erf of GELU is the branch-free rational-times-exponential form (Abramowitz & Stegun
// 7.1.26, absolute error below 1.5e-7: three orders below bf16 resolution).
// GELU with that erf formula, erf(x) = 1 - P(t) t exp(-x^2), t = 1 / (1 + p x) for x >= 0, arranged for epilogues that
// finish hundreds of values per lane: with a = |v|, x = a / sqrt 2 and q = (P(t) t / 2) exp(-x^2) = erfc(x) / 2 it is
// gelu(v) = v Phi(v) = max(v, 0) - a q for either sign of v: 19 instruction slots instead of 25 (the reciprocal and
// the exponential count four each).
__device__ __forceinline__ float gelu_as(float v) {
  const float a = fabsf(v);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752f, a, 1.f));
  float y = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
  y = fmaf(y, t, 0.5f * 1.421413741f);
  y = fmaf(y, t, 0.5f * -0.284496736f);
  y = fmaf(y, t, 0.5f * 0.254829592f);
  const float q = y * t * fast_exp2((-0.5f * 1.4426950408889634f) * (v * v));
  return fmaf(-a, q, fmaxf(v, 0.f));
}
template <int ACT>
__device__ __forceinline__ float act_fn(float v) {
  if (ACT == TANDEM_ACT_GELU) return gelu_as(v);
  if (ACT == TANDEM_ACT_RELU) return fmaxf(v, 0.f);
  return v;
}
#define ACT_SWITCH(act, BODY)                         \
  switch (act) {                                      \
    case TANDEM_ACT_GELU: {                           \
      constexpr int ACT = TANDEM_ACT_GELU;            \
      BODY                                            \
    } break;                                          \
    case TANDEM_ACT_RELU: {                           \
      constexpr int ACT = TANDEM_ACT_RELU;            \
      BODY                                            \
    } break;                                          \
    default: {                                        \
      constexpr int ACT = TANDEM_ACT_NONE;            \
      BODY                                            \
    }                                                 \
  }

// bf16 store of one 32 x 32 MFMA result tile whose lanes hold a feature each (X rows were the A-operand):
// lane (c, h) has feature n and rows mbase + 8 * (r / 4) + 4 * h + r % 4.  Neighbouring lanes (features n,
// n ^ 1) trade one value per pair of rows, so that every lane stores two adjacent features of one row as a
// 4-byte word and a store instruction covers 64-byte row segments.  bn: bias of feature n (0 without).
template <int ACT>
__device__ __forceinline__ void store_tile_bf16(const f32x16& acc, int mbase, int n, int h, float bn, const GemmParams& p) {
  const bool odd = n & 1;
#pragma unroll
  for (int r = 0; r < 16; r += 2) {
    const int m = mbase + 8 * (r >> 2) + 4 * h + (r & 3);  // rows m (value r) and m + 1 (value r + 1)
    float v0 = act_fn<ACT>(acc[r] + bn), v1 = act_fn<ACT>(acc[r + 1] + bn);
    if (p.residual) {
      const int mc = m < p.M ? m : p.M - 1, mc1 = m + 1 < p.M ? m + 1 : p.M - 1;
      v0 += bf16_to_f32(((const bf16_t*)p.residual)[(long long)mc * p.ldr + n]);
      v1 += bf16_to_f32(((const bf16_t*)p.residual)[(long long)mc1 * p.ldr + n]);
    }
    const float got = dpp_f32<0xB1>(odd ? v0 : v1);  // from lane ^ 1
    const uint32_t word = odd ? pack_bf16x2(got, v1) : pack_bf16x2(v0, got);
    const int row = odd ? m + 1 : m;
    if (row < p.M) *reinterpret_cast<uint32_t*>((bf16_t*)p.Y + (long long)row * p.ldy + (n & ~1)) = word;
  }
}

// The same store for the big-tile kernel, whose epilogue finishes 256 values per lane: everything that does not depend
// on the value is taken out of it.  yt: the wavefront's first output row at its first column (a wave-uniform byte
// pointer); loff: this lane's byte offset inside that (row 4 h, plus 1 for odd lanes, column n & ~1); rowb: bytes per
// row; mleft: rows of the wavefront's 128 that exist (FULL: all of them, no test per store); lrow = 4 h.  dm0 = first
// row of the 32 x 32 tile inside the wavefront's 128, nofs = its first column.  No residual (products with one take
// store_tile_bf16).
template <int ACT, bool FULL>
__device__ __forceinline__ void store_tile_big(const f32x16& acc, char* yt, uint32_t loff, uint32_t rowb, int dm0, int nofs,
                                               bool odd, float bn, int mleft, int lrow) {
#pragma unroll
  for (int r = 0; r < 16; r += 2) {
    const int dm = dm0 + 8 * (r >> 2) + (r & 3);  // rows dm (value r) and dm + 1 (value r + 1), plus 4 h in loff
    const float v0 = act_fn<ACT>(acc[r] + bn), v1 = act_fn<ACT>(acc[r + 1] + bn);
    const float got = dpp_f32<0xB1>(odd ? v0 : v1);  // from lane ^ 1
    const uint32_t word = odd ? pack_bf16x2(got, v1) : pack_bf16x2(v0, got);
    if (FULL || lrow + dm + (odd ? 1 : 0) < mleft)
      *reinterpret_cast<uint32_t*>(yt + (size_t)dm * rowb + (size_t)nofs * 2 + loff) = word;
  }
}

__device__ __forceinline__ bf16x8 ldg8(const bf16_t* p) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p));
}

// ---------------------------------------------------------------- skinny bf16 MFMA kernel
// grid (N/32, splitK, ceil(M/(32*MT))); block NW*64.  Requires N % 32 == 0, K % 64 == 0.
//
// Every wavefront is independent inside the main loop (no workgroup barrier).  Per 64-deep chunk it
//   - loads its 32 weight rows straight into MFMA A-operands (each lane 64 contiguous bytes),
//   - loads the X chunk [32*MT rows, 64] with fully coalesced 16-byte loads (8 lanes = one 128-byte
//     row segment), parks it in a wavefront-private LDS tile (row pitch 144 B) and reads it back in
//     the B-operand layout with conflict-free ds_read_b128.  Coalesced loads cost the vector cache a
//     third of what operand-layout loads cost (measured), and X is read 32*MT/32 times per weight byte.
// The loads of chunk i+1 are in flight while chunk i is multiplied.
constexpr int XP = 72;  // LDS row pitch in bf16 elements (64 + 8 padding)

template <int MT, int NW>
__global__ __launch_bounds__(NW * 64) void gemm_skinny_kernel(GemmParams p) {
  if (p.gate && *p.gate == 0) return;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c32 = lane & 31, h = lane >> 5;
  const int n0 = blockIdx.x * 32;
  const int m0 = blockIdx.z * (32 * MT);
  const int chunks = p.K >> 6;
  const int per = (chunks + p.splitK - 1) / p.splitK;
  const int cb = blockIdx.y * per;
  const int ce = chunks < cb + per ? chunks : cb + per;
  bf16_t* xs = reinterpret_cast<bf16_t*>(smem) + (size_t)w * (32 * MT) * XP;  // this wavefront's X tile

  const bf16_t* wrow = (const bf16_t*)p.W + (long long)(n0 + c32) * p.K + 32 * h;
  // X staging: piece id = lane + 64*i -> row (lane>>3) + 8*i, 16-byte column lane&7
  constexpr int XL = 4 * MT;  // 16-byte pieces per lane per chunk
  const int xrow0 = lane >> 3, xcol = lane & 7;
  const bf16_t* xbase = (const bf16_t*)p.X + xcol * 8;
  bf16_t* xdst0 = xs + xrow0 * XP + xcol * 8;

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;

  // Wavefront w owns chunks cb + w, cb + w + NW, ...  Workgroups start at different points of that
  // list (rotation by block index): weight rows are a power-of-two stride apart, so workgroups that
  // all walk K in the same order would keep hitting the same memory channel at the same time.
  const int cnt = (ce - cb - w + NW - 1) / NW;  // chunks of this wavefront (<= 0: none)
  const int rot = cnt > 0 ? (int)((blockIdx.x + 3 * blockIdx.y) % cnt) : 0;
  auto k_of = [&](int i) __attribute__((always_inline)) -> long long {
    int r = i + rot;
    r = r >= cnt ? r - cnt : r;
    return (long long)(cb + w + r * NW) << 6;
  };
  bf16x8 a0[4], a1[4];
  u32x4 xr[XL];
  auto gload = [&](bf16x8* a, int i) __attribute__((always_inline)) {
    const long long k0 = k_of(i);
#pragma unroll
    for (int j = 0; j < 4; ++j) a[j] = ldg8(wrow + k0 + 8 * j);
#pragma unroll
    for (int q = 0; q < XL; ++q) {
      int m = m0 + xrow0 + 8 * q;
      m = m < p.M ? m : p.M - 1;  // rows past M re-read the last row; their results are dropped
      xr[q] = *reinterpret_cast<const u32x4*>(xbase + (long long)m * p.ldx + k0);
    }
  };
  auto xstore = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < XL; ++q) *reinterpret_cast<u32x4*>(xdst0 + q * 8 * XP) = xr[q];
  };
  auto compute = [&](const bf16x8* a) __attribute__((always_inline)) {
    const bf16_t* xb = xs + c32 * XP + 32 * h;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const bf16x8 b = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(xb + mt * 32 * XP + 8 * j));
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b, acc[mt], 0, 0, 0);
      }
  };
  if (cnt > 0) {
    gload(a0, 0);
    int i = 0;
    for (; i + 2 < cnt; i += 2) {  // steady state: no branch inside, both steps have a successor
      xstore();
      gload(a1, i + 1);
      compute(a0);
      xstore();
      gload(a0, i + 2);
      compute(a1);
    }
    if (cnt - i == 2) {
      xstore();
      gload(a1, i + 1);
      compute(a0);
      xstore();
      compute(a1);
    } else {
      xstore();
      compute(a0);
    }
  }

  // tree reduction over the wavefronts (lane-local layout) through the LDS the X tiles no longer need
  __syncthreads();
  float* red = reinterpret_cast<float*>(smem);
  auto slot = [&](int buf, int mt, int r) __attribute__((always_inline)) -> float& { return red[((buf * MT + mt) * 16 + r) * 64 + lane]; };
#pragma unroll
  for (int half = NW / 2; half >= 1; half >>= 1) {
    if (w >= half && w < 2 * half) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) slot(w - half, mt, r) = acc[mt][r];
    }
    __syncthreads();
    if (w < half) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] += slot(w, mt, r);
    }
    __syncthreads();
  }
  if (w != 0) return;

  // C layout of the 32x32 tile: lane holds column j = lane%32 (row m of X), rows i = 8*(r/4) + 4*(lane/32) + r%4 (n)
  if (p.splitK > 1 || p.defer) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = m0 + mt * 32 + c32;
      if (m >= p.M) continue;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float* dst = p.part + ((long long)blockIdx.y * p.M + m) * p.N + n0 + 8 * q + 4 * h;
        *reinterpret_cast<float4*>(dst) =
            make_float4(acc[mt][4 * q], acc[mt][4 * q + 1], acc[mt][4 * q + 2], acc[mt][4 * q + 3]);
      }
    }
    return;
  }
  ACT_SWITCH(p.act, {
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) {
      const int m = m0 + mt * 32 + c32;
      if (m >= p.M) continue;
      _Pragma("unroll") for (int q = 0; q < 4; ++q) {
        const int n = n0 + 8 * q + 4 * h;
        float v[4];
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {
          v[i] = acc[mt][4 * q + i];
          if (p.bias) v[i] += bf16_to_f32(((const bf16_t*)p.bias)[n + i]);
          v[i] = act_fn<ACT>(v[i]);
          if (p.residual) v[i] += bf16_to_f32(((const bf16_t*)p.residual)[(long long)m * p.ldr + n + i]);
        }
        uint2 u;
        u.x = pack_bf16x2(v[0], v[1]);
        u.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2*>((bf16_t*)p.Y + (long long)m * p.ldy + n) = u;
      }
    }
  })
}

// ---------------------------------------------------------------- tile bf16 MFMA kernel (32 < M <= 128 per pass)
// grid (N/128, splitK, ceil(M/(32*MT))); block 512 = 8 wavefronts = 4 feature groups x 2 contraction
// groups.  A wavefront owns 32 output features and every second 128-deep chunk of the workgroup's
// contraction range; it streams its weight rows straight from global memory into MFMA A-operands
// (each lane 128 contiguous bytes, a weight row 256 contiguous bytes per chunk: shorter runs per row
// cap the HBM stream well below what longer ones reach).  The X chunk of a contraction group is
// fetched once (coalesced), parked in a double-buffered LDS tile (row pitch 272 B, conflict-free
// 16-byte reads) and read by the group's four wavefronts in the B-operand layout: a quarter of the X
// loads and LDS writes per MFMA of the wavefront-private scheme above.  One barrier per chunk; the
// loads of chunk i+1 fly while chunk i is multiplied.
// Requires N % 128 == 0, K % 256 == 0 and an even chunk count per split.
constexpr int KC = 128;      // contraction depth of a chunk
constexpr int XPT = KC + 8;  // LDS row pitch in bf16 elements

template <int MT>
__global__ __launch_bounds__(512) void gemm_tile_kernel(GemmParams p) {
  if (p.gate && *p.gate == 0) return;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int ng = w & 3, kg = w >> 2;
  const int c32 = lane & 31, h = lane >> 5;
  const int tg = threadIdx.x & 255;  // thread index inside the contraction group
  const int n0 = blockIdx.x * 128 + ng * 32;
  const int m0 = blockIdx.z * (32 * MT);
  const int chunks = p.K / KC;
  const int per = chunks / p.splitK;  // even (launcher)
  const int cb = blockIdx.y * per;
  const int T = per >> 1;  // iterations: one chunk per contraction group each
  const int rot = (int)((blockIdx.x * 5 + blockIdx.y * 3) % T);

  constexpr int TILE = (32 * MT) * XPT;  // elements of one X tile
  constexpr int XL = 2 * MT;             // 16-byte pieces per thread per chunk
  bf16_t* xs = reinterpret_cast<bf16_t*>(smem) + (size_t)kg * 2 * TILE;  // [2][32*MT][XPT]
  const bf16_t* wrow = (const bf16_t*)p.W + (long long)(n0 + c32) * p.K + (KC / 2) * h;
  // X staging: piece id = tg + 256*q -> row (tg>>4) + 16*q, 16-byte column tg&15
  const int xrow0 = tg >> 4, xcol = tg & 15;
  const bf16_t* xbase = (const bf16_t*)p.X + xcol * 8;
  bf16_t* xdst0 = xs + xrow0 * XPT + xcol * 8;
  const bf16_t* xb0 = xs + c32 * XPT + (KC / 2) * h;

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;

  bf16x8 a0[8], a1[8];
  u32x4 xr[XL];
#define TG_K0(i, k0_)                                             \
  long long k0_;                                                  \
  {                                                               \
    int r_ = (i) < T ? (i) : T - 1; /* past the end: re-read */   \
    r_ += rot;                                                    \
    r_ = r_ >= T ? r_ - T : r_;                                   \
    k0_ = (long long)(cb + 2 * r_ + kg) * KC;                     \
  }
#define TG_XLOAD(i)                                                                           \
  {                                                                                           \
    TG_K0(i, k0_)                                                                             \
    _Pragma("unroll") for (int q = 0; q < XL; ++q) {                                          \
      int m_ = m0 + xrow0 + 16 * q;                                                           \
      m_ = m_ < p.M ? m_ : p.M - 1;                                                           \
      xr[q] = *reinterpret_cast<const u32x4*>(xbase + (long long)m_ * p.ldx + k0_);           \
    }                                                                                         \
    __builtin_amdgcn_sched_barrier(0); /* keep the issue order: loads complete in order */    \
  }
#define TG_WLOAD(a, i)                                                                        \
  {                                                                                           \
    TG_K0(i, k0_)                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                        \
    _Pragma("unroll") for (int j = 0; j < 8; ++j) a[j] = ldg8(wrow + k0_ + 8 * j);            \
    __builtin_amdgcn_sched_barrier(0);                                                        \
  }
#define TG_XSTORE(buf)                                                                                         \
  {                                                                                                            \
    _Pragma("unroll") for (int q = 0; q < XL; ++q)                                                             \
        *reinterpret_cast<u32x4*>(xdst0 + (buf) * TILE + q * 16 * XPT) = xr[q];                                \
  }
#define TG_COMPUTE(a, buf)                                                                                     \
  {                                                                                                            \
    _Pragma("unroll") for (int j = 0; j < 8; ++j) _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) {           \
      const bf16x8 b_ = __builtin_bit_cast(                                                                    \
          bf16x8, *reinterpret_cast<const u32x4*>(xb0 + (buf) * TILE + mt * 32 * XPT + 8 * j));                \
      acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b_, acc[mt], 0, 0, 0);                           \
    }                                                                                                          \
  }

  // Software pipeline, one chunk ahead.  X is requested before the weights: loads complete in issue
  // order, X comes from cache and is needed first (LDS store before the barrier), so the weight loads
  // stay in flight across the barrier.
  TG_XLOAD(0)
  TG_WLOAD(a0, 0)
  TG_XSTORE(0)
  __syncthreads();
  int i = 0;
  for (; i + 1 < T; i += 2) {  // no branch inside
    TG_XLOAD(i + 1)
    TG_WLOAD(a1, i + 1)
    TG_COMPUTE(a0, 0)
    TG_XSTORE(1)
    __syncthreads();
    TG_XLOAD(i + 2)
    TG_WLOAD(a0, i + 2)
    TG_COMPUTE(a1, 1)
    TG_XSTORE(0)
    __syncthreads();
  }
  if (i < T) TG_COMPUTE(a0, 0)
#undef TG_K0
#undef TG_XLOAD
#undef TG_WLOAD
#undef TG_XSTORE
#undef TG_COMPUTE

  // contraction group 1 hands its sums to group 0 through LDS (lane-local layout)
  __syncthreads();
  float* red = reinterpret_cast<float*>(smem);
  if (kg == 1) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) red[((ng * MT + mt) * 16 + r) * 64 + lane] = acc[mt][r];
  }
  __syncthreads();
  if (kg == 1) return;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] += red[((ng * MT + mt) * 16 + r) * 64 + lane];

  if (p.splitK > 1 || p.defer) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = m0 + mt * 32 + c32;
      if (m >= p.M) continue;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float* dst = p.part + ((long long)blockIdx.y * p.M + m) * p.N + n0 + 8 * q + 4 * h;
        *reinterpret_cast<float4*>(dst) =
            make_float4(acc[mt][4 * q], acc[mt][4 * q + 1], acc[mt][4 * q + 2], acc[mt][4 * q + 3]);
      }
    }
    return;
  }
  ACT_SWITCH(p.act, {
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) {
      const int m = m0 + mt * 32 + c32;
      if (m >= p.M) continue;
      _Pragma("unroll") for (int q = 0; q < 4; ++q) {
        const int n = n0 + 8 * q + 4 * h;
        float v[4];
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {
          v[i] = acc[mt][4 * q + i];
          if (p.bias) v[i] += bf16_to_f32(((const bf16_t*)p.bias)[n + i]);
          v[i] = act_fn<ACT>(v[i]);
          if (p.residual) v[i] += bf16_to_f32(((const bf16_t*)p.residual)[(long long)m * p.ldr + n + i]);
        }
        uint2 u;
        u.x = pack_bf16x2(v[0], v[1]);
        u.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2*>((bf16_t*)p.Y + (long long)m * p.ldy + n) = u;
      }
    }
  })
}

// ---------------------------------------------------------------- stream bf16 MFMA kernel (packed weights)
// The decode-time regime again (32 < M <= 128 rows per pass, bound by reading every weight once), for
// weights re-laid out by pack_weights_kernel: one 4 KB tile per (32 features, 64-deep stage), inside it
// [j = 0..3][lane = 0..63][8 values] with lane = 32 * h + c holding W[32 * nb + c][64 * kb + 32 * h + 8 * j ..],
// the A-operand of the j-th v_mfma_f32_32x32x16_bf16 of the stage.  Every load instruction of a wavefront
// then reads 1 KB of consecutive addresses and a wavefront walks one contiguous stream.
//
// grid (N/128, splitK, row passes), 8 wavefronts with two roles:
//   wavefronts 0-3 (multipliers) own 32 features each; their only global loads are their weight tiles, three
//     stages ahead in a ring of four register sets (contiguous per-wavefront streams reach the HBM rate with
//     one or two stages in flight: measured).
//   wavefronts 4-7 (feeders) bring the X rows of each stage into LDS for all four multipliers (coalesced
//     16-byte loads eight stages ahead, row pitch 144 B for conflict-free operand reads).
// Separate roles keep the two load streams apart: a wavefront's loads complete in issue order, so one that
// waits for cache-resident X rows also waits for every HBM weight load issued before them.  One workgroup
// barrier per stage hands an X buffer over.  X rows are the MFMA A-operand, so a lane ends up holding one
// feature for 16 rows per tile and stores cover whole row segments.
// Measured at M = 128, N = 32768, K = 4096 (268 MB of weights): the main loop runs at the HBM rate (about
// 38 us); launch, the first loads, uneven finishing times of the workgroups and the output stores add some
// 25 us.  Requires N % 128 == 0, K % 256 == 0, at least four stages per split.
constexpr int SK = 64;       // contraction depth of a stage
constexpr int XPS = SK + 8;  // LDS row pitch in bf16 elements

template <int MT>
__global__ __launch_bounds__(512) void gemm_stream_kernel(GemmParams p) {
  if (p.gate && *p.gate == 0) return;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m0 = blockIdx.z * (32 * MT);
  // (feature tile bx, contraction split by) of this workgroup.  Workgroups go to the 8 XCDs round-robin by id;
  // the split index follows the XCD, so that the workgroups sharing an XCD's L2 read the same slice of X
  // (with the plain order an XCD saw every slice, and X competed with the weight stream for its L2).
  int bx, by;
  {
    const int id = blockIdx.x, S = p.splitK, xcd = id & 7;
    if (p.xcd_map && S >= 8) {
      by = xcd + 8 * ((id >> 3) % (S >> 3));
      bx = id / S;
    } else if (p.xcd_map) {
      by = xcd % S;
      bx = (id >> 3) * (8 / S) + xcd / S;
    } else {
      bx = id % (p.N / 128);
      by = id / (p.N / 128);
    }
  }
  const int T = (p.K / SK) / p.splitK;  // stages of this workgroup
  const int sb = by * T;
  const int rot = (int)((bx * 5 + by * 3) % T);
  constexpr int TILE = (32 * MT) * XPS;  // elements of one X buffer
  bf16_t* xs = reinterpret_cast<bf16_t*>(smem);  // [2][32*MT][XPS]

  // global stage index of the i-th stage (rotated start; past the end: re-read the last)
#define SG_STAGE(i, st_)                 \
  long long st_;                         \
  {                                      \
    int r_ = (i) < T ? (i) : T - 1;      \
    r_ += rot;                           \
    r_ = r_ >= T ? r_ - T : r_;          \
    st_ = (long long)(sb + r_);          \
  }

  if (w >= 4) {
    // ---------------- feeder: X rows of stage s+1 into LDS buffer (s+1)&1 while stage s is multiplied
    const int tl = threadIdx.x - 256;
    // piece id = tl + 256*q -> row (tl>>3) + 32*q, 16-byte column tl&7
    const int xrow0 = tl >> 3, xcol = tl & 7;
    const bf16_t* xbase = (const bf16_t*)p.X + xcol * 8;
    bf16_t* xdst0 = xs + xrow0 * XPS + xcol * 8;
    u32x4 x0[MT], x1[MT], x2[MT], x3[MT], x4[MT], x5[MT], x6[MT], x7[MT];
#define SG_XLOAD(xr, i)                                                                    \
  {                                                                                        \
    SG_STAGE(i, st_)                                                                       \
    _Pragma("unroll") for (int q = 0; q < MT; ++q) {                                       \
      int m_ = m0 + xrow0 + 32 * q;                                                        \
      m_ = m_ < p.M ? m_ : p.M - 1;                                                        \
      xr[q] = *reinterpret_cast<const u32x4*>(xbase + (long long)m_ * p.ldx + st_ * SK);   \
    }                                                                                      \
    __builtin_amdgcn_sched_barrier(0);                                                     \
  }
#define SG_XSTORE(xr, buf)                                                                 \
  {                                                                                        \
    _Pragma("unroll") for (int q = 0; q < MT; ++q)                                         \
        *reinterpret_cast<u32x4*>(xdst0 + (buf) * TILE + q * 32 * XPS) = xr[q];            \
  }
    // step s: request X(s+8) into the set parked one step ago, park X(s+1)
#define SG_FEED(s, xload, xstore, buf) \
  SG_XLOAD(xload, (s) + 8)             \
  SG_XSTORE(xstore, buf)               \
  __syncthreads();
    SG_XLOAD(x0, 0)
    SG_XLOAD(x1, 1)
    SG_XLOAD(x2, 2)
    SG_XLOAD(x3, 3)
    SG_XLOAD(x4, 4)
    SG_XLOAD(x5, 5)
    SG_XLOAD(x6, 6)
    SG_XLOAD(x7, 7)
    SG_XSTORE(x0, 0)
    __syncthreads();
    int s = 0;
    for (; s + 8 <= T; s += 8) {
      SG_FEED(s, x0, x1, 1)
      SG_FEED(s + 1, x1, x2, 0)
      SG_FEED(s + 2, x2, x3, 1)
      SG_FEED(s + 3, x3, x4, 0)
      SG_FEED(s + 4, x4, x5, 1)
      SG_FEED(s + 5, x5, x6, 0)
      SG_FEED(s + 6, x6, x7, 1)
      SG_FEED(s + 7, x7, x0, 0)
    }
    if (s < T) {
      SG_FEED(s, x0, x1, 1)
      if (s + 1 < T) {
        SG_FEED(s + 1, x1, x2, 0)
        if (s + 2 < T) {
          SG_FEED(s + 2, x2, x3, 1)
          if (s + 3 < T) {
            SG_FEED(s + 3, x3, x4, 0)
            if (s + 4 < T) {
              SG_FEED(s + 4, x4, x5, 1)
              if (s + 5 < T) {
                SG_FEED(s + 5, x5, x6, 0)
                if (s + 6 < T) { SG_FEED(s + 6, x6, x7, 1) }
              }
            }
          }
        }
      }
    }
#undef SG_XLOAD
#undef SG_XSTORE
#undef SG_FEED
    return;
  }

  // ---------------- multiplier
  const int c32 = lane & 31, h = lane >> 5;
  const int n0 = bx * 128 + w * 32;
  const bf16_t* wp = (const bf16_t*)p.Wp + (long long)(n0 >> 5) * 32 * p.K + lane * 8;
  const bf16_t* xb0 = xs + c32 * XPS + 32 * h;
  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;
  bf16x8 a0[4], a1[4], a2[4], a3[4];
  bf16x8 b0[2][MT], b1[2][MT];  // B-operands of the first / second half (j = 0,1 / 2,3) of a stage
#pragma unroll
  for (int j = 0; j < 4; ++j) a3[j] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) b1[j][mt] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#define SG_WLOAD(a, i)                                                                         \
  {                                                                                            \
    SG_STAGE(i, st_)                                                                           \
    __builtin_amdgcn_sched_barrier(0);                                                         \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) a[j] = ldg8(wp + st_ * (32 * SK) + 512 * j); \
    __builtin_amdgcn_sched_barrier(0);                                                         \
  }
#define SG_READ(b, buf, half)                                                                  \
  {                                                                                            \
    _Pragma("unroll") for (int j = 0; j < 2; ++j) _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)  \
        b[j][mt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(                 \
                                                  xb0 + (buf) * TILE + mt * 32 * XPS + 8 * (2 * (half) + j))); \
    __builtin_amdgcn_sched_barrier(0);                                                         \
  }
#define SG_MMA(a, b, half)                                                                     \
  {                                                                                            \
    _Pragma("unroll") for (int j = 0; j < 2; ++j) _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)  \
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j][mt], a[2 * (half) + j], acc[mt], 0, 0, 0); \
    __builtin_amdgcn_sched_barrier(0);                                                         \
  }
  // A wavefront is alone on its SIMD and an LDS read returns 1 KB in about as many cycles as an MFMA takes,
  // so reads and MFMAs are interleaved by hand, half a stage apart: while the 8 operand reads of one half
  // return, the 8 MFMAs of the half before it run.  The second half of a stage is multiplied after the
  // barrier that ends the stage (its operands are in registers by then), under the reads of the next stage.
  // step s: aprev = weights of stage s-1 (its set is refilled with W(s+3) once its last MFMAs are issued)
#define SG_MUL(s, acur, aprev, buf)       \
  SG_READ(b0, buf, 0)                     \
  SG_MMA(aprev, b1, 1)                    \
  SG_WLOAD(aprev, (s) + 3)                \
  SG_READ(b1, buf, 1)                     \
  SG_MMA(acur, b0, 0)                     \
  __syncthreads();
  SG_WLOAD(a0, 0)
  SG_WLOAD(a1, 1)
  SG_WLOAD(a2, 2)
  __syncthreads();
  int s = 0;
  for (; s + 4 <= T; s += 4) {  // no branch inside
    SG_MUL(s, a0, a3, 0)
    SG_MUL(s + 1, a1, a0, 1)
    SG_MUL(s + 2, a2, a1, 0)
    SG_MUL(s + 3, a3, a2, 1)
  }
  if (s < T) {
    SG_MUL(s, a0, a3, 0)
    if (s + 1 < T) {
      SG_MUL(s + 1, a1, a0, 1)
      if (s + 2 < T) {
        SG_MUL(s + 2, a2, a1, 0)
        SG_MMA(a2, b1, 1)
      } else {
        SG_MMA(a1, b1, 1)
      }
    } else {
      SG_MMA(a0, b1, 1)
    }
  } else {
    SG_MMA(a3, b1, 1)
  }
#undef SG_READ
#undef SG_MMA
#undef SG_STAGE
#undef SG_WLOAD
#undef SG_MUL

  // X rows are the A-operand, so a lane holds feature n = n0 + c32 for the rows 8 * (r / 4) + 4 * h + r % 4 of
  // each 32-row tile: a store instruction covers whole 128-byte (fp32) or 64-byte (bf16) row segments.
  const int n = n0 + c32;
  if (p.splitK > 1 || p.defer) {
    // wave-uniform base + one per-lane byte offset; each store then adds a compile-time multiple of the row pitch
    char* dst = reinterpret_cast<char*>(p.part + ((long long)by * p.M + m0) * p.N + n0);
    const uint32_t rowb = (uint32_t)p.N * 4u;
    const uint32_t loff = (uint32_t)(4 * h) * rowb + (uint32_t)c32 * 4u;
    const int mleft = p.M - m0 - 4 * h;  // rows from this lane's first one to the end of the matrix
    if (p.M - m0 >= 32 * MT) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          *reinterpret_cast<float*>(dst + (size_t)(mt * 32 + 8 * (r >> 2) + (r & 3)) * rowb + loff) = acc[mt][r];
    } else {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int dm = mt * 32 + 8 * (r >> 2) + (r & 3);
          if (dm < mleft) *reinterpret_cast<float*>(dst + (size_t)dm * rowb + loff) = acc[mt][r];
        }
    }
    return;
  }
  const float bn = p.bias ? bf16_to_f32(((const bf16_t*)p.bias)[n]) : 0.f;
  if (p.residual) {
    ACT_SWITCH(p.act, {
      _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) store_tile_bf16<ACT>(acc[mt], m0 + mt * 32, n, h, bn, p);
    })
    return;
  }
  // as in the big-tile kernel: a wave-uniform base, one byte offset per lane, no address arithmetic per value
  const bool odd = c32 & 1;
  char* yt = reinterpret_cast<char*>((bf16_t*)p.Y + (long long)m0 * p.ldy + n0);
  const uint32_t rowb = (uint32_t)p.ldy * 2u;
  const uint32_t loff = (uint32_t)(4 * h + (odd ? 1 : 0)) * rowb + (uint32_t)(c32 & ~1) * 2u;
  const int mleft = p.M - m0;
  if (mleft >= 32 * MT) {
    ACT_SWITCH(p.act, {
      _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)
          (store_tile_big<ACT, true>)(acc[mt], yt, loff, rowb, mt * 32, 0, odd, bn, mleft, 4 * h);
    })
  } else {
    ACT_SWITCH(p.act, {
      _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)
          (store_tile_big<ACT, false>)(acc[mt], yt, loff, rowb, mt * 32, 0, odd, bn, mleft, 4 * h);
    })
  }
}

// Re-lays W[N, K] (bf16, row-major) out in the 4 KB tiles the stream kernel reads: one thread per 16 bytes
// of output.  Requires N % 32 == 0, K % 64 == 0.
__global__ void pack_weights_kernel(const bf16_t* __restrict__ W, bf16_t* __restrict__ Wp, long long N, long long K) {
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;  // output piece
  if (t >= N * K / 8) return;
  const int lane = (int)(t & 63), j = (int)((t >> 6) & 3);
  const long long tile = t >> 8, kbs = K / SK;
  const long long nb = tile / kbs, kb = tile - nb * kbs;
  const int c = lane & 31, h = lane >> 5;
  const uint4 v = *reinterpret_cast<const uint4*>(W + (32 * nb + c) * K + SK * kb + 32 * h + 8 * j);
  *reinterpret_cast<uint4*>(Wp + t * 8) = v;
}

// ---------------------------------------------------------------- big-tile bf16 MFMA kernel (M >= 256)
// The compute-bound regime (prompt-time FF_Tandem over whole prompts, large verify batches): 256 x 256
// output tile per workgroup, 4 wavefronts in a 2 x 2 arrangement, 128 x 128 per wavefront = 16 MFMA
// tiles of 32x32 (256 accumulator registers) so that one operand fetched from LDS feeds four MFMAs.
// Both operands reach LDS by direct global-to-LDS loads (global_load_lds_dwordx4: no staging registers, no
// LDS store instructions), 64-deep stages, double-buffered; the loads of stage s+1 are issued when stage s
// starts and must have landed at the barrier that ends it.  Such a load writes the 64 lanes' 16-byte
// pieces to consecutive LDS addresses, so rows cannot be padded; instead piece c of row r sits at position
// c ^ ((r >> 1) & 7) of the row (the lane-to-address map of the load does the permutation), which keeps
// the 16-byte operand reads of 16 consecutive rows on 16 different bank groups.
// A wavefront is alone on its SIMD, so LDS reads and MFMAs are interleaved by hand: the operands of
// contraction step k+1 are requested before the 16 MFMAs of step k are issued; the last step of a stage
// is multiplied after the barrier, under the first operand reads of the next stage.
// Workgroup ids are remapped so that the workgroups an XCD receives (round-robin by id) cover
// neighbouring tiles that share a weight tile in that XCD's L2.
// Requires N % 256 == 0, K % 128 == 0; M ragged (rows past M are clamped on load, skipped on store).
constexpr int BK = 64;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

__global__ __launch_bounds__(256, 1) void gemm_big_kernel(GemmParams p, int tiles_m, int tiles_n) {
  if (p.gate && *p.gate == 0) return;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);  // [2][256][BK], pieces permuted inside a row
  bf16_t* Bs = As + 2 * 256 * BK;                // [2][256][BK]
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = w >> 1, wn = w & 1;
  const int c32 = lane & 31, h = lane >> 5;

  // XCD-aware tile order.  A workgroup takes the tiles blockIdx.x, blockIdx.x + gridDim.x, ... (the launcher starts
  // one workgroup per compute unit when there are more tiles than that): ids go to the XCDs round-robin, so a
  // workgroup's tiles stay on its XCD.
  const int total = tiles_m * tiles_n;
#define BG_TILE(id_, m0_, n0_)                                                                          \
  {                                                                                                     \
    int id = (id_);                                                                                     \
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);                                     \
    int tn = id / tiles_m, tm = id % tiles_m;                                                           \
    if ((total & 7) == 0 && (tiles_m & 7) == 0 && (tiles_n & 3) == 0) {                                 \
      /* the 32 tiles an XCD works on at a time form an 8 x 4 block: 12 operand tiles feed 32 output tiles */ \
      const int block = id >> 5, within = id & 31, blocks_m = tiles_m >> 3;                             \
      tm = (block % blocks_m) * 8 + (within & 7);                                                       \
      tn = (block / blocks_m) * 4 + (within >> 3);                                                      \
    }                                                                                                   \
    m0_ = tm * 256;                                                                                     \
    n0_ = tn * 256;                                                                                     \
  }
  int tile = blockIdx.x, m0, n0;
  BG_TILE(tile, m0, n0)
  const int stages = (p.K / BK) / p.splitK;  // of this workgroup; even (launcher)
  const long long kbase = (long long)blockIdx.y * stages * BK;

  // Direct loads: instruction q of wavefront w fills rows 8 * (4 * q + w) .. + 8 of an operand tile (1 KB of
  // LDS); lane l lands on row l >> 3, position l & 7, so it fetches piece (l & 7) ^ ((row >> 1) & 7).
  const bf16_t* ag[8];
  const bf16_t* bg[8];
  // (the lane number is taken again from the hardware - through an opaque operand, so that the compiler neither
  // reuses nor hoists it - and everything derived from it is recomputed where the addresses are set up: the main
  // loop has no register to keep such values in, they would be spilled)
#define BG_LANE(lane_)                                                                         \
  int lane_;                                                                                   \
  {                                                                                            \
    unsigned ones_ = ~0u;                                                                      \
    asm volatile("" : "+s"(ones_));                                                            \
    lane_ = (int)__builtin_amdgcn_mbcnt_hi(ones_, __builtin_amdgcn_mbcnt_lo(ones_, 0u));       \
  }
#define BG_PTRS(m0_, n0_)                                                                      \
  {                                                                                            \
    BG_LANE(lane_)                                                                             \
    const int drow_ = lane_ >> 3;                                                              \
    const int dpiece_ = (lane_ & 7) ^ ((((w & 1) << 2) | (drow_ >> 1)) & 7);                   \
    _Pragma("unroll") for (int q = 0; q < 8; ++q) {                                            \
      const int row = 8 * (4 * q + w) + drow_;                                                 \
      int m_ = (m0_) + row;                                                                    \
      m_ = m_ < p.M ? m_ : p.M - 1;                                                            \
      ag[q] = (const bf16_t*)p.X + (long long)m_ * p.ldx + kbase + dpiece_ * 8;                \
      bg[q] = (const bf16_t*)p.W + (long long)((n0_) + row) * p.K + kbase + dpiece_ * 8;       \
    }                                                                                          \
  }
  BG_PTRS(m0, n0)
  // one direct load (1 KB): rows 8 * (4 * q + w) .. + 8 of the A (X) or B (W) tile of a stage
#define BG_DMA_A(buf, k0, q)                                                                                \
  __builtin_amdgcn_global_load_lds((global_void_ptr)(ag[q] + (k0)),                                         \
                                   (lds_void_ptr)(As + (buf) * 256 * BK + (4 * (q) + w) * 8 * BK), 16, 0, 0); \
  __builtin_amdgcn_sched_barrier(0);
#define BG_DMA_B(buf, k0, q)                                                                                \
  __builtin_amdgcn_global_load_lds((global_void_ptr)(bg[q] + (k0)),                                         \
                                   (lds_void_ptr)(Bs + (buf) * 256 * BK + (4 * (q) + w) * 8 * BK), 16, 0, 0); \
  __builtin_amdgcn_sched_barrier(0);

  f32x16 acc[4][4];

  // operand reads: row (wm | wn) * 128 + 32 * t + c32, piece 2 * ks + h, at position piece ^ ((c32 >> 1) & 7)
  const int fsw = (c32 >> 1) & 7;
  const bf16_t* a_rd = As + (wm * 128 + c32) * BK;
  const bf16_t* b_rd = Bs + (wn * 128 + c32) * BK;
  int pos[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) pos[ks] = ((2 * ks + h) ^ fsw) * 8;
  bf16x8 av0[4], bv0[4], av1[4], bv1[4];
#define BG_OPS(av, bv, buf, ks)                                                                             \
  {                                                                                                         \
    _Pragma("unroll") for (int t = 0; t < 4; ++t) {                                                         \
      av[t] = __builtin_bit_cast(                                                                           \
          bf16x8, *reinterpret_cast<const u32x4*>(a_rd + (buf) * 256 * BK + t * 32 * BK + pos[ks]));        \
      bv[t] = __builtin_bit_cast(                                                                           \
          bf16x8, *reinterpret_cast<const u32x4*>(b_rd + (buf) * 256 * BK + t * 32 * BK + pos[ks]));        \
    }                                                                                                       \
    __builtin_amdgcn_sched_barrier(0);                                                                      \
  }
#define BG_MFMA(av, bv)                                                                                     \
  {                                                                                                         \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) _Pragma("unroll") for (int j = 0; j < 4; ++j)              \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);              \
    __builtin_amdgcn_sched_barrier(0);                                                                      \
  }
#define BG_MFMA2(av, bv, i, j)                                                                             \
  acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);                   \
  acc[i][(j) + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[(j) + 1], acc[i][(j) + 1], 0, 0, 0); \
  __builtin_amdgcn_sched_barrier(0);
  // 16 MFMAs with a direct load after every second one.  Issuing such a load occupies the wavefront for
  // about 60 cycles (measured), an MFMA the matrix pipe for 32: issued in one block, the 16 loads of a
  // stage left the pipe idle for some 900 cycles per stage.
#define BG_MFMA_DMA(av, bv, DMA, buf, k0)                                    \
  BG_MFMA2(av, bv, 0, 0) DMA(buf, k0, 0) BG_MFMA2(av, bv, 0, 2) DMA(buf, k0, 1) \
  BG_MFMA2(av, bv, 1, 0) DMA(buf, k0, 2) BG_MFMA2(av, bv, 1, 2) DMA(buf, k0, 3) \
  BG_MFMA2(av, bv, 2, 0) DMA(buf, k0, 4) BG_MFMA2(av, bv, 2, 2) DMA(buf, k0, 5) \
  BG_MFMA2(av, bv, 3, 0) DMA(buf, k0, 6) BG_MFMA2(av, bv, 3, 2) DMA(buf, k0, 7)
  // BG_LDS_DONE waits for the operand reads issued before the previous group of MFMAs (long complete: the
  // group takes 512 cycles to issue).  Without it the compiler waits for ALL outstanding LDS reads right
  // before each MFMA group, i.e. also for the reads just issued for the next step.
#define BG_LDS_DONE                                                      \
  __builtin_amdgcn_s_waitcnt(0xC07F); /* lgkmcnt(0), other counters free */ \
  __builtin_amdgcn_sched_barrier(0);
  // One stage reading LDS buffer buf.  On entry av0 / bv0 are being read for its first contraction step and
  // av1 / bv1 hold the last step of the stage before, which is multiplied first, under those reads; the
  // loads of the next stage (into the buffer that stage before just left) ride on the first two groups.
#define BG_STAGE(buf, knext)                                  \
  BG_MFMA_DMA(av1, bv1, BG_DMA_A, 1 - (buf), knext)           \
  BG_LDS_DONE                                                 \
  BG_OPS(av1, bv1, buf, 1)                                    \
  BG_MFMA_DMA(av0, bv0, BG_DMA_B, 1 - (buf), knext)           \
  BG_LDS_DONE                                                 \
  BG_OPS(av0, bv0, buf, 2)                                    \
  BG_MFMA(av1, bv1)                                           \
  BG_LDS_DONE                                                 \
  BG_OPS(av1, bv1, buf, 3)                                    \
  BG_MFMA(av0, bv0)                                           \
  __syncthreads();                                            \
  BG_OPS(av0, bv0, 1 - (buf), 0)

#pragma unroll
  for (int q = 0; q < 8; ++q) {
    BG_DMA_A(0, 0, q)
    BG_DMA_B(0, 0, q)
  }
  // Tile loop.  The first stage of a workgroup's next tile is requested before the epilogue of the current one, so
  // its latency (and a workgroup launch) is off the path between two tiles.
  for (;;) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t) av1[t] = bv1[t] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};  // "last step of the stage before" of stage 0
  __syncthreads();
  BG_OPS(av0, bv0, 0, 0)
  for (int st = 0; st < stages; st += 2) {
    const long long k1 = (long long)(st + 1) * BK;                                  // st + 1 < stages
    const long long k2 = (long long)(st + 2 < stages ? st + 2 : stages - 1) * BK;   // past the end: harmless re-read
    BG_STAGE(0, k1)
    BG_STAGE(1, k2)
  }
  BG_MFMA(av1, bv1)  // last step of the last stage
  // every wavefront is past the last stage's barrier: buffer 0 holds nothing anybody needs
  const int m0c = m0, n0c = n0;  // the tile whose results are in the accumulators
  const int next = tile + (int)gridDim.x;
  const bool more = next < total;
  if (more) {
    tile = next;
    BG_TILE(tile, m0, n0)
    BG_PTRS(m0, n0)
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      BG_DMA_A(0, 0, q)
      BG_DMA_B(0, 0, q)
    }
  }

  // (lane coordinates taken afresh, see BG_LANE: everything the epilogue derives from them is computed per tile)
  BG_LANE(lane_e)
  const int c32e = lane_e & 31, he = lane_e >> 5;
  if (p.splitK > 1 || p.defer) {
    // fp32 partial sums [split, M, N]: 32 lanes = 128 contiguous bytes of a row per store
    const int mrow = m0c + wm * 128 + 4 * he;
    float* part = p.part + ((long long)blockIdx.y * p.M + mrow) * p.N + n0c + wn * 128 + c32e;
#define BG_PART(i, j)                                                                             \
  {                                                                                               \
    _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                              \
      const int dm = (i) * 32 + 8 * (r >> 2) + (r & 3);                                           \
      if (mrow + dm < p.M) part[dm * p.N + (j) * 32] = acc[i][j][r];                              \
    }                                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                            \
  }
#define BG_PART_ROW(i) BG_PART(i, 0) BG_PART(i, 1) BG_PART(i, 2) BG_PART(i, 3)
    BG_PART_ROW(0) BG_PART_ROW(1) BG_PART_ROW(2) BG_PART_ROW(3)
#undef BG_PART_ROW
#undef BG_PART
  } else
  // C layout: lane holds column j = lane % 32 (feature n), rows i = 8 * (r / 4) + 4 * (lane / 32) + r % 4 (row m).
  // Per lane 256 values: the wave-uniform and per-lane parts of the addresses, the biases and the row test are
  // computed once (an epilogue that redid them per value took 12 us of a 120 us tile).
  if (p.residual) {
    // rare at this size (no caller of the library has one): the general store
#define BG_OUT(i, j)                                                                              \
  {                                                                                               \
    const int n_ = n0c + wn * 128 + (j) * 32 + c32e;                                               \
    const float bn_ = p.bias ? bf16_to_f32(((const bf16_t*)p.bias)[n_]) : 0.f;                    \
    store_tile_bf16<ACT>(acc[i][j], m0c + wm * 128 + (i) * 32, n_, he, bn_, p);                    \
    __builtin_amdgcn_sched_barrier(0);                                                            \
  }
#define BG_OUT_ROW(i) BG_OUT(i, 0) BG_OUT(i, 1) BG_OUT(i, 2) BG_OUT(i, 3)
    ACT_SWITCH(p.act, { BG_OUT_ROW(0) BG_OUT_ROW(1) BG_OUT_ROW(2) BG_OUT_ROW(3) })
#undef BG_OUT_ROW
#undef BG_OUT
  } else {
    const int mw = m0c + wm * 128, nw = n0c + wn * 128;
    const bool odd = c32e & 1;
    char* yt = reinterpret_cast<char*>((bf16_t*)p.Y + (long long)mw * p.ldy + nw);
    const uint32_t rowb = (uint32_t)p.ldy * 2u;
    const uint32_t loff = (uint32_t)(4 * he + (odd ? 1 : 0)) * rowb + (uint32_t)(c32e & ~1) * 2u;
    const int mleft = p.M - mw, lrow = 4 * he;  // rows of this wavefront's 128 that exist; this lane's first row
    float bn[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) bn[j] = p.bias ? bf16_to_f32(((const bf16_t*)p.bias)[nw + j * 32 + c32e]) : 0.f;
#define BG_OUT(i, j)                                                                                    \
  store_tile_big<ACT, FULL>(acc[i][j], yt, loff, rowb, (i) * 32, (j) * 32, odd, bn[j], mleft, lrow);    \
  __builtin_amdgcn_sched_barrier(0);
#define BG_OUT_ROW(i) BG_OUT(i, 0) BG_OUT(i, 1) BG_OUT(i, 2) BG_OUT(i, 3)
#define BG_OUT_ALL BG_OUT_ROW(0) BG_OUT_ROW(1) BG_OUT_ROW(2) BG_OUT_ROW(3)
    if (mleft >= 128) {
      constexpr bool FULL = true;
      ACT_SWITCH(p.act, { BG_OUT_ALL })
    } else if (mleft > 0) {
      constexpr bool FULL = false;
      ACT_SWITCH(p.act, { BG_OUT_ALL })
    }
#undef BG_OUT_ALL
#undef BG_OUT_ROW
#undef BG_OUT
  }
  if (!more) break;
  // the load addresses of the new tile are computed again rather than kept in 32 registers through the epilogue
  asm volatile("" : "+s"(m0), "+s"(n0));
  BG_PTRS(m0, n0)
  }  // tile loop
#undef BG_DMA_A
#undef BG_DMA_B
#undef BG_MFMA2
#undef BG_MFMA_DMA
#undef BG_LDS_DONE
#undef BG_STAGE
#undef BG_OPS
#undef BG_MFMA
#undef BG_TILE
#undef BG_PTRS
#undef BG_LANE
}

// sums the split partials in split order, then the epilogue
template <typename T>
__global__ void gemm_splitk_epilogue_kernel(GemmParams p) {
  if (p.gate && *p.gate == 0) return;
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)p.M * p.N) return;
  const int m = (int)(idx / p.N), n = (int)(idx % p.N);
  float v = 0.f;
  for (int s = 0; s < p.splitK; ++s) v += p.part[((long long)s * p.M + m) * p.N + n];
  ((T*)p.Y)[(long long)m * p.ldy + n] = from_f32<T>(epilogue<T>(v, m, n, p));
}

// ---------------------------------------------------------------- generic LDS-tiled kernel
template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmParams p) {
  __shared__ float xs[16][17], wsm[16][17];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m = blockIdx.y * 16 + ty, n = blockIdx.x * 16 + tx;
  float acc = 0.f;
  for (int k0 = 0; k0 < p.K; k0 += 16) {
    const int mm = blockIdx.y * 16 + ty, nn = blockIdx.x * 16 + ty, kk = k0 + tx;
    xs[ty][tx] = (mm < p.M && kk < p.K) ? to_f32<T>(((const T*)p.X)[(long long)mm * p.ldx + kk]) : 0.f;
    wsm[ty][tx] = (nn < p.N && kk < p.K) ? to_f32<T>(((const T*)p.W)[(long long)nn * p.K + kk]) : 0.f;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) acc = fmaf(xs[ty][k], wsm[tx][k], acc);
    __syncthreads();
  }
  if (m < p.M && n < p.N) ((T*)p.Y)[(long long)m * p.ldy + n] = from_f32<T>(epilogue<T>(acc, m, n, p));
}

template <int MT, int NW>
int launch_skinny(const GemmParams& p, int mpasses, hipStream_t st) {
  const size_t xbytes = (size_t)NW * (32 * MT) * XP * sizeof(bf16_t);
  const size_t rbytes = (size_t)(NW / 2) * MT * 16 * 64 * sizeof(float);
  const size_t lds_bytes = xbytes > rbytes ? xbytes : rbytes;
  if (const int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(&gemm_skinny_kernel<MT, NW>), lds_bytes)) return rc;
  hipLaunchKernelGGL((gemm_skinny_kernel<MT, NW>), dim3(p.N / 32, p.splitK, mpasses), dim3(NW * 64), lds_bytes, st, p);
  return hip_ok(hipGetLastError());
}

template <int MT>
int launch_stream(const GemmParams& p, int mpasses, hipStream_t st) {
  const size_t lds_bytes = (size_t)2 * (32 * MT) * XPS * sizeof(bf16_t);
  if (const int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(&gemm_stream_kernel<MT>), lds_bytes)) return rc;
  GemmParams q = p;
  const int tiles = p.N / 128, S = p.splitK;
  q.xcd_map = (S >= 8 ? S % 8 == 0 : (8 % S == 0 && tiles % (8 / S) == 0)) ? 1 : 0;
  hipLaunchKernelGGL((gemm_stream_kernel<MT>), dim3(tiles * S, 1, mpasses), dim3(512), lds_bytes, st, q);
  return hip_ok(hipGetLastError());
}

template <int MT>
int launch_tile(const GemmParams& p, int mpasses, hipStream_t st) {
  const size_t xbytes = (size_t)2 * 2 * (32 * MT) * XPT * sizeof(bf16_t);
  const size_t rbytes = (size_t)4 * MT * 16 * 64 * sizeof(float);
  const size_t lds_bytes = xbytes > rbytes ? xbytes : rbytes;
  if (const int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(&gemm_tile_kernel<MT>), lds_bytes)) return rc;
  hipLaunchKernelGGL((gemm_tile_kernel<MT>), dim3(p.N / 128, p.splitK, mpasses), dim3(512), lds_bytes, st, p);
  return hip_ok(hipGetLastError());
}

int launch_big(const GemmParams& p, hipStream_t st) {
  const size_t lds_bytes = (size_t)2 * 2 * 256 * BK * sizeof(bf16_t);
  if (const int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(&gemm_big_kernel), lds_bytes)) return rc;
  const int tiles_m = (p.M + 255) / 256, tiles_n = p.N / 256;
  // one workgroup per compute unit, each taking every gridDim.x-th tile, when there are more tiles than units
  int grid_x = tiles_m * tiles_n;
  const int cus = compute_units();
  if (cus > 0 && grid_x * p.splitK > cus && p.splitK == 1) grid_x = cus;
  hipLaunchKernelGGL(gemm_big_kernel, dim3(grid_x, p.splitK), dim3(256), lds_bytes, st, p, tiles_m, tiles_n);
  return hip_ok(hipGetLastError());
}
// The big-tile kernel takes a product when its 256 x 256 tiles occupy at least half the CUs, or, from 1024
// rows on, when splitting the contraction across workgroups gets them there (each split keeps at least 16
// stages, an even number): below that the weight-streaming kernels in passes of 128 rows are as fast
// (measured at 512 rows) and leave no fp32 partials.  Returns the split count, 0 when the kernel does not
// apply.
int big_splits(int M, int N, int K) {
  if (M < 256 || N % 256 != 0 || N > (1 << 22) || K % (2 * BK) != 0) return 0;
  const long long tiles = (long long)((M + 255) / 256) * (N / 256);
  if (M < 1024) return tiles >= 128 ? 1 : 0;
  // From 1024 rows on, contraction splits while all workgroups still run at once (one per CU): a second round of
  // quarter-length workgroups and twice the fp32 partials cost more than they save (measured at 1024 x 6144 x 4096:
  // 4 splits of 96 tiles 104 us, 2 splits 75 us), and 128 tiles alone leave half of the chip idle.
  const int stages = K / BK;
  int s = 1;
  while (tiles * s * 2 <= 256 && s < 8 && stages % (4 * s) == 0 && stages / (2 * s) >= 16) s *= 2;
  return tiles * s >= 128 ? s : 0;
}
bool big_ok(int M, int N, int K) { return big_splits(M, N, K) > 0; }

bool skinny_ok(int M, int N, int K, int dtype, long long ldx) {
  return dtype == TANDEM_BF16 && N % 32 == 0 && K % 64 == 0 && ldx % 8 == 0 && M >= 1;
}
bool tile_ok(int M, int N, int K) { return M > 32 && N % 128 == 0 && K % (2 * KC) == 0; }
bool stream_ok(int M, int N, int K) { return M > 32 && N % 128 == 0 && K % (4 * SK) == 0; }  // = gemm_packable

// Stream kernel: contraction splits when every pass covers 128 rows: at most one workgroup per CU (a second
// round of workgroups would run alone), at least four stages each.
int stream_base_splits(int M, int N, int K) {
  const int tiles = (N / 128) * ((M + 127) / 128), stages = K / SK;
  int s = 1;
  while (tiles * s * 2 <= 256 && s < 16 && stages % (2 * s) == 0 && stages / (2 * s) >= 4) s *= 2;
  return s;
}

// Stream kernel, 64 < M <= 128: instead of s contraction splits of 128 rows, two row halves of s / 2 splits
// each (same number of workgroups).  The halves of a tile run on the same XCD at the same time and share
// the weight tile through its L2, so every weight still comes from HBM once but crosses L2 -> CU twice;
// in return half the fp32 partials are written and read back (none at all, and no epilogue kernel, when
// s was 2).  Measured: a gain unless the weights are much larger than the partials saved (a quarter of
// the weight bytes is the break-even).
bool stream_row_halves(int M, int N, int K, int s) {
  if (M <= 64 || M > 128 || s < 2) return false;
  const double saved = (double)(s / 2) * M * N * 8.0, extra = 0.25 * 2.0 * N * (double)K;
  return s == 2 || saved >= extra;
}

// Split of the contraction across workgroups (a function of the shape only): used when the feature
// tiles alone cannot occupy the 256 CUs.
int gemm_splitk(int M, int N, int K, bool packed) {
  const int mpasses = (M + 127) / 128;
  const int chunks = K / 64;
  int s = big_splits(M, N, K);
  if (s > 0) return s;
  s = 1;
  if (packed && stream_ok(M, N, K)) {
    s = stream_base_splits(M, N, K);
    if (stream_row_halves(M, N, K, s)) s /= 2;
  } else if (tile_ok(M, N, K)) {
    const int tiles = (N / 128) * mpasses, kc = K / KC;  // every split keeps an even number (>= 4) of chunks
    while (tiles * s < 200 && s < 16 && kc % (4 * s) == 0 && kc / (2 * s) >= 4) s *= 2;
  } else {
    // (from 128 workgroups on a split buys nothing: these products are launch-bound, and a split of a
    // product with an epilogue costs a second kernel)
    const int tiles = (N / 32) * mpasses;
    while (tiles * s < 128 && s * 2 * 8 <= chunks && s < 16) s *= 2;
  }
  return s;
}

}  // namespace

bool gemm_can_defer(int M, int N, int K, int dtype, int64_t ldx) { return skinny_ok(M, N, K, dtype, ldx); }
int gemm_splits(int M, int N, int K, bool packed) { return gemm_splitk(M, N, K, packed); }
size_t gemm_deferred_workspace(int M, int N, int K) {
  const int a = gemm_splitk(M, N, K, false), b = gemm_splitk(M, N, K, true);
  return (size_t)(a > b ? a : b) * M * N * sizeof(float);
}
bool gemm_packable(int64_t N, int64_t K, int dtype) { return dtype == TANDEM_BF16 && N % 128 == 0 && K % (4 * SK) == 0; }
int launch_pack_weights(const void* W, void* Wp, int64_t N, int64_t K, hipStream_t st) {
  const long long pieces = N * K / 8;
  hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, (const bf16_t*)W,
                     (bf16_t*)Wp, (long long)N, (long long)K);
  return hip_ok(hipGetLastError());
}

size_t gemm_workspace(int M, int N, int K, int dtype) {
  if (!skinny_ok(M, N, K, dtype, 8)) return 0;
  const int a = gemm_splitk(M, N, K, false), b = gemm_splitk(M, N, K, true);
  const int s = a > b ? a : b;
  return s > 1 ? (size_t)s * M * N * sizeof(float) : 0;
}

int launch_gemm(const GemmArgs& g, hipStream_t st) {
  GemmParams p;
  p.X = g.X;
  p.W = g.W;
  p.Wp = g.Wp;
  p.bias = g.bias;
  p.residual = g.residual;
  p.Y = g.Y;
  p.part = g.ws;
  p.ldx = g.ldx;
  p.ldr = g.ldr;
  p.ldy = g.ldy;
  p.M = g.M;
  p.N = g.N;
  p.K = g.K;
  p.act = g.act;
  p.splitK = 1;
  p.m_base = 0;
  p.xcd_map = 0;
  p.defer = g.defer;
  p.gate = g.gate;
  if (skinny_ok(g.M, g.N, g.K, g.dtype, g.ldx) && (reinterpret_cast<uintptr_t>(g.X) % 16 == 0) &&
      (reinterpret_cast<uintptr_t>(g.W) % 16 == 0) && (reinterpret_cast<uintptr_t>(g.Y) % 8 == 0) && g.ldy % 4 == 0) {
    const bool big = big_ok(g.M, g.N, g.K);
    const bool packed = !big && g.Wp && stream_ok(g.M, g.N, g.K);
    if (packed && reinterpret_cast<uintptr_t>(g.Wp) % 16 != 0) return TANDEM_ERR_SHAPE;
    p.splitK = gemm_splitk(g.M, g.N, g.K, packed);
    if ((p.splitK > 1 || g.defer) && (size_t)p.splitK * g.M * g.N * sizeof(float) > g.ws_bytes) return TANDEM_ERR_WORKSPACE;
    if (big) {
      const int rc = launch_big(p, st);
      if (rc != TANDEM_OK || p.splitK == 1 || g.defer) return rc;
      const long long total = (long long)g.M * g.N;
      hipLaunchKernelGGL(gemm_splitk_epilogue_kernel<bf16_t>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, p);
      return hip_ok(hipGetLastError());
    }
    int mt = g.M <= 32 ? 1 : (g.M <= 64 ? 2 : 4);
    if (packed && stream_row_halves(g.M, g.N, g.K, stream_base_splits(g.M, g.N, g.K))) mt = 2;  // two passes of 64 rows
    const int mpasses = (g.M + 32 * mt - 1) / (32 * mt);
    int rc;
    if (packed)
      rc = mt == 2 ? launch_stream<2>(p, mpasses, st) : launch_stream<4>(p, mpasses, st);
    else if (tile_ok(g.M, g.N, g.K))
      rc = mt == 2 ? launch_tile<2>(p, mpasses, st) : launch_tile<4>(p, mpasses, st);
    else if (mt == 1)
      rc = launch_skinny<1, 8>(p, mpasses, st);
    else if (mt == 2)
      rc = launch_skinny<2, 8>(p, mpasses, st);
    else
      rc = launch_skinny<4, 8>(p, mpasses, st);
    if (rc != TANDEM_OK || p.splitK == 1 || g.defer) return rc;
    const long long total = (long long)g.M * g.N;
    hipLaunchKernelGGL(gemm_splitk_epilogue_kernel<bf16_t>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, p);
    return hip_ok(hipGetLastError());
  }
  if (g.defer) return TANDEM_ERR_UNSUPPORTED;
  dim3 grid((g.N + 15) / 16, (g.M + 15) / 16);
  if (g.dtype == TANDEM_BF16)
    hipLaunchKernelGGL(gemm_generic_kernel<bf16_t>, grid, dim3(256), 0, st, p);
  else if (g.dtype == TANDEM_F32)
    hipLaunchKernelGGL(gemm_generic_kernel<float>, grid, dim3(256), 0, st, p);
  else
    return TANDEM_ERR_UNSUPPORTED;
  return hip_ok(hipGetLastError());
}
