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
// gemm_generic_kernel: any dtype / shape, LDS-tiled on the vector ALUs (the fp32
// correctness path of the tiny configuration and odd shapes).
#include "common.h"
#include "kernels.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct GemmParams {
  const void* X;
  const void* W;
  const void* bias;
  const void* residual;
  void* Y;
  float* part;  // [splitK, M, N] fp32 partial sums
  long long ldx, ldr, ldy;
  int M, N, K, act, splitK, m_base;
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

__device__ __forceinline__ bf16x8 ldg8(const bf16_t* p) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p));
}

// ---------------------------------------------------------------- skinny bf16 MFMA kernel
// grid (N/32, splitK, ceil(M/(32*MT))); block NW*64.  Requires N % 32 == 0, K % 64 == 0.
template <int MT, int NW>
__global__ __launch_bounds__(NW * 64) void gemm_skinny_kernel(GemmParams p) {
  extern __shared__ float lds[];  // [NW/2][MT][16][64]
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c32 = lane & 31, h = lane >> 5;
  const int n0 = blockIdx.x * 32;
  const int m0 = blockIdx.z * (32 * MT);
  const int chunks = p.K >> 6;
  const int per = (chunks + p.splitK - 1) / p.splitK;
  const int cb = blockIdx.y * per;
  const int ce = chunks < cb + per ? chunks : cb + per;

  const bf16_t* wrow = (const bf16_t*)p.W + (long long)(n0 + c32) * p.K + 32 * h;
  const bf16_t* xrow[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    int m = m0 + mt * 32 + c32;
    m = m < p.M ? m : p.M - 1;  // rows past M re-read the last row; their results are dropped
    xrow[mt] = (const bf16_t*)p.X + (long long)m * p.ldx + 32 * h;
  }

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;

  bf16x8 a0[4], b0[MT][4], a1[4], b1[MT][4];
  auto load = [&](bf16x8* a, bf16x8(*b)[4], int c) {
    const long long k0 = (long long)c << 6;
#pragma unroll
    for (int j = 0; j < 4; ++j) a[j] = ldg8(wrow + k0 + 8 * j);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 4; ++j) b[mt][j] = ldg8(xrow[mt] + k0 + 8 * j);
  };
  auto fma = [&](const bf16x8* a, const bf16x8(*b)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[mt][j], acc[mt], 0, 0, 0);
  };

  // Wavefront w owns chunks cb + w, cb + w + NW, ...  Workgroups start at different points of that
  // list (rotation by block index): weight rows are a power-of-two stride apart, so workgroups that
  // all walk K in the same order would keep hitting the same memory channel at the same time.
  const int cnt = (ce - cb - w + NW - 1) / NW;  // chunks of this wavefront (<= 0: none)
  const int rot = cnt > 0 ? (int)((blockIdx.x + 3 * blockIdx.y) % cnt) : 0;
  auto chunk_of = [&](int i) {
    int r = i + rot;
    r = r >= cnt ? r - cnt : r;
    return cb + w + r * NW;
  };
  int i = 0;
  if (i < cnt) load(a0, b0, chunk_of(0));
  while (i < cnt) {
    if (i + 1 < cnt) load(a1, b1, chunk_of(i + 1));
    fma(a0, b0);
    ++i;
    if (i >= cnt) break;
    if (i + 1 < cnt) load(a0, b0, chunk_of(i + 1));
    fma(a1, b1);
    ++i;
  }

  // tree reduction over the wavefronts (lane-local layout)
  auto slot = [&](int buf, int mt, int r) -> float& { return lds[((buf * MT + mt) * 16 + r) * 64 + lane]; };
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
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = m0 + mt * 32 + c32;
    if (m >= p.M) continue;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int n = n0 + 8 * q + 4 * h;
      if (p.splitK > 1) {
        float* dst = p.part + ((long long)blockIdx.y * p.M + m) * p.N + n;
        *reinterpret_cast<float4*>(dst) =
            make_float4(acc[mt][4 * q], acc[mt][4 * q + 1], acc[mt][4 * q + 2], acc[mt][4 * q + 3]);
      } else {
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = epilogue<bf16_t>(acc[mt][4 * q + i], m, n + i, p);
        uint2 u;
        u.x = pack_bf16x2(v[0], v[1]);
        u.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2*>((bf16_t*)p.Y + (long long)m * p.ldy + n) = u;
      }
    }
  }
}

// sums the split partials in split order, then the epilogue
template <typename T>
__global__ void gemm_splitk_epilogue_kernel(GemmParams p) {
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
  const size_t lds_bytes = (size_t)(NW / 2) * MT * 16 * 64 * sizeof(float);
  static bool attr_set = false;
  if (!attr_set && lds_bytes > 48 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_skinny_kernel<MT, NW>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
      return TANDEM_ERR_HIP;
    attr_set = true;
  }
  hipLaunchKernelGGL((gemm_skinny_kernel<MT, NW>), dim3(p.N / 32, p.splitK, mpasses), dim3(NW * 64), lds_bytes, st, p);
  return hip_ok(hipGetLastError());
}

bool skinny_ok(int M, int N, int K, int dtype, long long ldx) {
  return dtype == TANDEM_BF16 && N % 32 == 0 && K % 64 == 0 && ldx % 8 == 0 && M >= 1;
}

// split of the contraction across workgroups: only when the N tiles alone cannot fill the chip
int skinny_splitk(int M, int N, int K) {
  const int tiles = (N / 32) * ((M + 127) / 128);
  const int chunks = K / 64;
  int s = 1;
  while (tiles * s < 256 && s * 2 * 8 <= chunks && s < 16) s *= 2;  // keep >= 1 chunk per wavefront
  return s;
}

}  // namespace

size_t gemm_workspace(int M, int N, int K, int dtype) {
  if (!skinny_ok(M, N, K, dtype, 8)) return 0;
  const int s = skinny_splitk(M, N, K);
  return s > 1 ? (size_t)s * M * N * sizeof(float) : 0;
}

int launch_gemm(const GemmArgs& g, hipStream_t st) {
  GemmParams p;
  p.X = g.X;
  p.W = g.W;
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
  if (skinny_ok(g.M, g.N, g.K, g.dtype, g.ldx) && (reinterpret_cast<uintptr_t>(g.X) % 16 == 0) &&
      (reinterpret_cast<uintptr_t>(g.W) % 16 == 0) && (reinterpret_cast<uintptr_t>(g.Y) % 8 == 0) && g.ldy % 4 == 0) {
    p.splitK = skinny_splitk(g.M, g.N, g.K);
    if (p.splitK > 1 && (size_t)p.splitK * g.M * g.N * sizeof(float) > g.ws_bytes) return TANDEM_ERR_WORKSPACE;
    const int mt = g.M <= 32 ? 1 : (g.M <= 64 ? 2 : 4);
    const int mpasses = (g.M + 32 * mt - 1) / (32 * mt);
    int rc;
    if (mt == 1)
      rc = launch_skinny<1, 8>(p, mpasses, st);
    else if (mt == 2)
      rc = launch_skinny<2, 8>(p, mpasses, st);
    else
      rc = launch_skinny<4, 8>(p, mpasses, st);
    if (rc != TANDEM_OK || p.splitK == 1) return rc;
    const long long total = (long long)g.M * g.N;
    hipLaunchKernelGGL(gemm_splitk_epilogue_kernel<bf16_t>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, p);
    return hip_ok(hipGetLastError());
  }
  dim3 grid((g.N + 15) / 16, (g.M + 15) / 16);
  if (g.dtype == TANDEM_BF16)
    hipLaunchKernelGGL(gemm_generic_kernel<bf16_t>, grid, dim3(256), 0, st, p);
  else if (g.dtype == TANDEM_F32)
    hipLaunchKernelGGL(gemm_generic_kernel<float>, grid, dim3(256), 0, st, p);
  else
    return TANDEM_ERR_UNSUPPORTED;
  return hip_ok(hipGetLastError());
}
