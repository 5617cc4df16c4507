// C ABI entry points: argument validation on the host, then kernel launches.  Nothing is
// enqueued when a check fails.
#include <map>
#include <mutex>
#include <utility>

#include "common.h"
#include "kernels.h"

int ensure_dynamic_lds(const void* kernel, size_t bytes) {
  if (bytes <= 48 * 1024) return TANDEM_OK;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return TANDEM_ERR_HIP;
  static std::mutex mu;
  static std::map<std::pair<const void*, int>, size_t> done;  // (kernel, device) -> limit already set
  std::lock_guard<std::mutex> lock(mu);
  const auto key = std::make_pair(kernel, dev);
  const auto it = done.find(key);
  if (it != done.end() && it->second >= bytes) return TANDEM_OK;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
    return TANDEM_ERR_HIP;
  done[key] = bytes;
  return TANDEM_OK;
}

int compute_units() {
  constexpr int MAX_DEVICES = 64;
  static std::mutex mu;
  static int count[MAX_DEVICES] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return 0;
  std::lock_guard<std::mutex> lock(mu);
  if (count[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 0;
    count[dev] = n;
  }
  return count[dev];
}

// Split-K partials of tandem_draft_attn_static: device memory that exists from the moment the library is loaded, so
// that entry point never allocates.  One copy per GPU; in host code the name is only a handle for
// hipGetSymbolAddress, the kernels get the address that call returns.  (No `used` attribute: with it the compiler
// keeps the device-side symbol local, and the runtime, which finds the array by name, aborts.)
static __device__ __align__(256) unsigned char scratch[TANDEM_STATIC_SCRATCH_BYTES];

namespace {

// Plain read-only stream: every workgroup walks a contiguous piece of the buffer of its own with 16-byte loads (a
// wavefront reads 1 KB of consecutive addresses per instruction, the workgroup 4 KB), eight loads in flight per lane;
// the values are folded into one word per workgroup so that the loads cannot be dropped.  What this kernel reaches
// is the box's ceiling for any kernel that reads HBM once.
__global__ __launch_bounds__(256) void read_stream_kernel(const uint4* __restrict__ src, long long n16,
                                                          uint32_t* __restrict__ sink) {
  const long long per = (n16 + gridDim.x - 1) / gridDim.x;
  const long long begin = (long long)blockIdx.x * per;
  const long long end = begin + per < n16 ? begin + per : n16;
  long long i = begin + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 7 * 256 < end; i += 8 * 256) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = ld_stream16(src + i + u * 256);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < end; i += 256) {
    const uint4 a = ld_stream16(src + i);
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  for (int off = 32; off >= 1; off >>= 1) acc ^= __shfl_xor(acc, off);
  __shared__ uint32_t red[4];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = red[0] ^ red[1] ^ red[2] ^ red[3];
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void** out) {
  constexpr int MAX_DEVICES = 64;
  static std::mutex mu;
  static void* ptr[MAX_DEVICES] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return TANDEM_ERR_HIP;
  if (dev < 0 || dev >= MAX_DEVICES) return TANDEM_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TANDEM_ERR_HIP;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return TANDEM_OK;
}

int check_attn_desc(const tandem_attn_desc* a) {
  if (!a) return TANDEM_ERR_NULL;
  if (a->B <= 0 || a->Hq <= 0 || a->Hkv <= 0 || a->T_max <= 0 || a->gamma_max < 0) return TANDEM_ERR_SHAPE;
  if (a->Hq % a->Hkv != 0) return TANDEM_ERR_SHAPE;
  if (a->dtype != TANDEM_F32 && a->dtype != TANDEM_BF16) return TANDEM_ERR_UNSUPPORTED;
  if (a->dh != 64 && a->dh != 128) return TANDEM_ERR_UNSUPPORTED;
  const int G = a->Hq / a->Hkv;
  if (G != 1 && G != 2 && G != 4 && G != 8) return TANDEM_ERR_UNSUPPORTED;
  if (a->B > 65535 || (int64_t)a->Hkv * TANDEM_MAX_QLEN > 65535) return TANDEM_ERR_SHAPE;
  return TANDEM_OK;
}

bool block_uses_mfma(const tandem_attn_desc* a) { return a->dtype == TANDEM_BF16 && a->dh == 128; }

void carve(void* ws, size_t rows, int S, float** ml, float** o) {
  *ml = (float*)ws;
  *o = (float*)((char*)ws + align256(rows * S * 2 * sizeof(float)));
}
size_t carved_bytes(size_t rows, int S, int dh) {
  if (S <= 1) return 0;
  return align256(rows * S * 2 * sizeof(float)) + rows * S * dh * sizeof(float);
}

// Splits of the two key segments of shared-prompt attention: the prompt rows (one workgroup set per prompt, all
// samples' rows together) and each sample's own rows.
struct SharedPlan {
  int S1, wide1, S2, wide2;
};
int plan_shared(const tandem_attn_desc* a, int32_t samples, int64_t T_own, int32_t q_len, SharedPlan* pl) {
  int rc = check_attn_desc(a);
  if (rc != TANDEM_OK) return rc;
  if (samples < 1 || q_len < 1 || q_len > TANDEM_MAX_QLEN || (int64_t)samples * q_len > TANDEM_MAX_SHARED_ROWS)
    return TANDEM_ERR_SHAPE;
  if (T_own < q_len || (int64_t)a->B * samples > 65535) return TANDEM_ERR_SHAPE;
  if ((int64_t)a->Hkv * samples * q_len > 65535) return TANDEM_ERR_SHAPE;
  const int G = a->Hq / a->Hkv;
  const int rows1 = samples * q_len;
  pl->wide1 = pl->wide2 = 0;
  if (block_uses_mfma(a)) {
    pl->S1 = attn_block_splits(a->B, a->Hkv, rows1, G, a->T_max, &pl->wide1);
    pl->S2 = attn_block_splits(a->B * samples, a->Hkv, q_len, G, T_own, &pl->wide2);
  } else {
    pl->S1 = attn_rows_splits(a->B, a->Hkv, rows1, G, a->T_max, 0, &pl->wide1);
    pl->S2 = attn_rows_splits(a->B * samples, a->Hkv, q_len, G, T_own, 0, &pl->wide2);
  }
  return TANDEM_OK;
}

}  // namespace

extern "C" {

const char* tandem_status_string(int status) {
  switch (status) {
    case TANDEM_OK: return "ok";
    case TANDEM_ERR_NULL: return "required pointer is NULL";
    case TANDEM_ERR_SHAPE: return "invalid or inconsistent shape";
    case TANDEM_ERR_UNSUPPORTED: return "unsupported configuration";
    case TANDEM_ERR_WORKSPACE: return "workspace too small";
    case TANDEM_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int tandem_read_stream(const void* src, size_t bytes, void* sink, void* hip_stream) {
  if (!src || !sink) return TANDEM_ERR_NULL;
  if (bytes < 16 || reinterpret_cast<uintptr_t>(src) % 16 != 0) return TANDEM_ERR_SHAPE;
  hipLaunchKernelGGL(read_stream_kernel, dim3(TANDEM_READ_STREAM_BLOCKS), dim3(256), 0, (hipStream_t)hip_stream,
                     (const uint4*)src, (long long)(bytes / 16), (uint32_t*)sink);
  return hip_ok(hipGetLastError());
}

size_t tandem_draft_attn_workspace(const tandem_attn_desc* a) {
  if (check_attn_desc(a) != TANDEM_OK) return 0;
  const int S = attn_rows_splits(a->B, a->Hkv, 1, a->Hq / a->Hkv, a->T_max, a->gamma_max, nullptr);
  return carved_bytes((size_t)a->B * a->Hq, S, a->dh);
}

size_t tandem_block_attn_workspace(const tandem_attn_desc* a, int32_t q_len) {
  if (check_attn_desc(a) != TANDEM_OK || q_len < 1 || q_len > TANDEM_MAX_QLEN) return 0;
  const int S = block_uses_mfma(a) ? attn_block_splits(a->B, a->Hkv, q_len, a->Hq / a->Hkv, a->T_max, nullptr)
                                   : attn_rows_splits(a->B, a->Hkv, q_len, a->Hq / a->Hkv, a->T_max, 0, nullptr);
  return carved_bytes((size_t)a->B * q_len * a->Hq, S, a->dh);
}

int tandem_draft_attn(const tandem_attn_desc* a, const void* q, const void* k_hat, const void* v_hat,
                      const int32_t* n_large, const void* k_cur, const void* v_cur, const int32_t* n_cur, void* out,
                      void* ws, size_t ws_bytes, void* hip_stream) {
  int rc = check_attn_desc(a);
  if (rc != TANDEM_OK) return rc;
  if (!q || !k_hat || !v_hat || !n_large || !k_cur || !v_cur || !n_cur || !out) return TANDEM_ERR_NULL;
  if (a->gamma_max < 1) return TANDEM_ERR_SHAPE;
  const size_t need = tandem_draft_attn_workspace(a);
  if (need > 0 && !ws) return TANDEM_ERR_NULL;
  if (ws_bytes < need) return TANDEM_ERR_WORKSPACE;
  AttnArgs x{};
  x.q = q;
  x.kA = k_hat;
  x.vA = v_hat;
  x.kB = k_cur;
  x.vB = v_cur;
  x.nA = n_large;
  x.nB = n_cur;
  x.causal = 0;
  x.B = a->B;
  x.Hq = a->Hq;
  x.Hkv = a->Hkv;
  x.dh = a->dh;
  x.q_len = 1;
  x.T_max = a->T_max;
  x.gamma_max = a->gamma_max;
  x.scale = a->scale;
  x.dtype = a->dtype;
  x.out = out;
  x.S = attn_rows_splits(a->B, a->Hkv, 1, a->Hq / a->Hkv, a->T_max, a->gamma_max, &x.wide);
  if (x.S > 1) carve(ws, (size_t)a->B * a->Hq, x.S, &x.part_ml, &x.part_o);
  return launch_attn_rows(x, (hipStream_t)hip_stream);
}

int tandem_draft_attn_static(const tandem_attn_desc* a, const void* q, const void* k_hat, const void* v_hat,
                             const int32_t* n_large, const void* k_cur, const void* v_cur, const int32_t* n_cur, void* out,
                             void* hip_stream) {
  const int rc = check_attn_desc(a);
  if (rc != TANDEM_OK) return rc;
  if (tandem_draft_attn_workspace(a) > TANDEM_STATIC_SCRATCH_BYTES) return TANDEM_ERR_WORKSPACE;
  void* ws = nullptr;
  const int rs = static_scratch(&ws);
  if (rs != TANDEM_OK) return rs;
  // every partial slot the combine reads is written by this call's own launch first: nothing to clear
  return tandem_draft_attn(a, q, k_hat, v_hat, n_large, k_cur, v_cur, n_cur, out, ws, TANDEM_STATIC_SCRATCH_BYTES, hip_stream);
}

int tandem_block_attn(const tandem_attn_desc* a, const void* q, const void* k_cache, const void* v_cache,
                      const int32_t* n_prefix, int32_t q_len, void* out, void* ws, size_t ws_bytes, void* hip_stream) {
  int rc = check_attn_desc(a);
  if (rc != TANDEM_OK) return rc;
  if (!q || !k_cache || !v_cache || !n_prefix || !out) return TANDEM_ERR_NULL;
  if (q_len < 1 || q_len > TANDEM_MAX_QLEN || a->T_max < q_len) return TANDEM_ERR_SHAPE;
  const size_t need = tandem_block_attn_workspace(a, q_len);
  if (need > 0 && !ws) return TANDEM_ERR_NULL;
  if (ws_bytes < need) return TANDEM_ERR_WORKSPACE;
  AttnArgs x{};
  x.q = q;
  x.kA = k_cache;
  x.vA = v_cache;
  x.kB = nullptr;
  x.vB = nullptr;
  x.nA = n_prefix;
  x.nB = nullptr;
  x.causal = 1;
  x.B = a->B;
  x.Hq = a->Hq;
  x.Hkv = a->Hkv;
  x.dh = a->dh;
  x.q_len = q_len;
  x.T_max = a->T_max;
  x.gamma_max = 0;
  x.scale = a->scale;
  x.dtype = a->dtype;
  x.out = out;
  const bool mfma = block_uses_mfma(a);
  x.wide = 0;
  x.S = mfma ? attn_block_splits(a->B, a->Hkv, q_len, a->Hq / a->Hkv, a->T_max, &x.wide)
             : attn_rows_splits(a->B, a->Hkv, q_len, a->Hq / a->Hkv, a->T_max, 0, &x.wide);
  if (x.S > 1) carve(ws, (size_t)a->B * q_len * a->Hq, x.S, &x.part_ml, &x.part_o);
  return mfma ? launch_attn_block(x, (hipStream_t)hip_stream) : launch_attn_rows(x, (hipStream_t)hip_stream);
}

size_t tandem_block_attn_shared_workspace(const tandem_attn_desc* a, int32_t samples, int64_t T_own, int32_t q_len) {
  SharedPlan pl;
  if (plan_shared(a, samples, T_own, q_len, &pl) != TANDEM_OK) return 0;
  return carved_bytes((size_t)a->B * samples * q_len * a->Hq, pl.S1 + pl.S2, a->dh);
}

int tandem_block_attn_shared(const tandem_attn_desc* a, int32_t samples, int64_t T_own, const void* q,
                             const void* k_shared, const void* v_shared, const int32_t* n_shared, const void* k_own,
                             const void* v_own, const int32_t* n_own, int32_t q_len, void* out, void* ws,
                             size_t ws_bytes, void* hip_stream) {
  SharedPlan pl;
  int rc = plan_shared(a, samples, T_own, q_len, &pl);
  if (rc != TANDEM_OK) return rc;
  if (!q || !k_shared || !v_shared || !n_shared || !k_own || !v_own || !n_own || !out || !ws) return TANDEM_ERR_NULL;
  const size_t rows = (size_t)a->B * samples * q_len * a->Hq;
  const int S = pl.S1 + pl.S2;
  if (ws_bytes < carved_bytes(rows, S, a->dh)) return TANDEM_ERR_WORKSPACE;
  const bool mfma = block_uses_mfma(a);
  hipStream_t st = (hipStream_t)hip_stream;
  AttnArgs x{};
  x.q = q;
  x.Hq = a->Hq;
  x.Hkv = a->Hkv;
  x.dh = a->dh;
  x.scale = a->scale;
  x.dtype = a->dtype;
  x.out = out;
  x.S_total = S;
  carve(ws, rows, S, &x.part_ml, &x.part_o);
  // prompt rows: per prompt, the samples * q_len query rows form one block that sees all n_shared[b] keys
  x.kA = k_shared;
  x.vA = v_shared;
  x.nA = n_shared;
  x.causal = 0;
  x.B = a->B;
  x.q_len = samples * q_len;
  x.T_max = a->T_max;
  x.S = pl.S1;
  x.wide = pl.wide1;
  x.s_off = 0;
  rc = mfma ? launch_attn_block(x, st) : launch_attn_rows(x, st);
  if (rc != TANDEM_OK) return rc;
  // own rows: every sample is a sequence of its own, causal inside the block
  x.kA = k_own;
  x.vA = v_own;
  x.nA = n_own;
  x.causal = 1;
  x.B = a->B * samples;
  x.q_len = q_len;
  x.T_max = T_own;
  x.S = pl.S2;
  x.wide = pl.wide2;
  x.s_off = pl.S1;
  // an unsplit last segment merges the prompt segment's partials itself (matrix-core kernels)
  const bool merge = mfma && pl.S2 == 1;
  x.merge_prev = merge ? pl.S1 : 0;
  rc = mfma ? launch_attn_block(x, st) : launch_attn_rows(x, st);
  if (rc != TANDEM_OK || merge) return rc;
  return launch_attn_combine(x.part_ml, x.part_o, out, (int)rows, S, a->dh, a->dtype, st);
}

// splits of the two launches of the shared-prompt draft attention
int plan_draft_shared(const tandem_attn_desc* a, int32_t samples, int64_t T_own, SharedPlan* pl) {
  int rc = check_attn_desc(a);
  if (rc != TANDEM_OK) return rc;
  if (samples < 1 || samples > TANDEM_MAX_SHARED_ROWS || T_own < 1 || a->gamma_max < 1) return TANDEM_ERR_SHAPE;
  if ((int64_t)a->B * samples > 65535 || (int64_t)a->Hkv * samples > 65535) return TANDEM_ERR_SHAPE;
  const int G = a->Hq / a->Hkv;
  pl->wide1 = pl->wide2 = 0;
  pl->S1 = block_uses_mfma(a) ? attn_block_splits(a->B, a->Hkv, samples, G, a->T_max, &pl->wide1)
                              : attn_rows_splits(a->B, a->Hkv, samples, G, a->T_max, 0, &pl->wide1);
  pl->S2 = attn_rows_splits(a->B * samples, a->Hkv, 1, G, T_own, a->gamma_max, &pl->wide2);
  return TANDEM_OK;
}

size_t tandem_draft_attn_shared_workspace(const tandem_attn_desc* a, int32_t samples, int64_t T_own) {
  SharedPlan pl;
  if (plan_draft_shared(a, samples, T_own, &pl) != TANDEM_OK) return 0;
  return carved_bytes((size_t)a->B * samples * a->Hq, pl.S1 + pl.S2, a->dh);
}

int tandem_draft_attn_shared(const tandem_attn_desc* a, int32_t samples, int64_t T_own, const void* q,
                             const void* k_hat_shared, const void* v_hat_shared, const int32_t* n_shared,
                             const void* k_hat_own, const void* v_hat_own, const int32_t* n_own, const void* k_cur,
                             const void* v_cur, const int32_t* n_cur, void* out, void* ws, size_t ws_bytes,
                             void* hip_stream) {
  SharedPlan pl;
  int rc = plan_draft_shared(a, samples, T_own, &pl);
  if (rc != TANDEM_OK) return rc;
  if (!q || !k_hat_shared || !v_hat_shared || !n_shared || !k_hat_own || !v_hat_own || !n_own || !k_cur || !v_cur ||
      !n_cur || !out || !ws)
    return TANDEM_ERR_NULL;
  const size_t rows = (size_t)a->B * samples * a->Hq;
  const int S = pl.S1 + pl.S2;
  if (ws_bytes < carved_bytes(rows, S, a->dh)) return TANDEM_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  AttnArgs x{};
  x.q = q;
  x.Hq = a->Hq;
  x.Hkv = a->Hkv;
  x.dh = a->dh;
  x.scale = a->scale;
  x.dtype = a->dtype;
  x.out = out;
  x.causal = 0;
  x.S_total = S;
  carve(ws, rows, S, &x.part_ml, &x.part_o);
  // the prompt's rows: per prompt, the queries of its samples form one block that sees all n_shared[b] keys
  x.kA = k_hat_shared;
  x.vA = v_hat_shared;
  x.nA = n_shared;
  x.B = a->B;
  x.q_len = samples;
  x.T_max = a->T_max;
  x.gamma_max = 0;
  x.S = pl.S1;
  x.wide = pl.wide1;
  x.s_off = 0;
  rc = block_uses_mfma(a) ? launch_attn_block(x, st) : launch_attn_rows(x, st);
  if (rc != TANDEM_OK) return rc;
  // each sample's rows of completed blocks after the prompt and its rows of the block being drafted
  x.kA = k_hat_own;
  x.vA = v_hat_own;
  x.nA = n_own;
  x.kB = k_cur;
  x.vB = v_cur;
  x.nB = n_cur;
  x.B = a->B * samples;
  x.q_len = 1;
  x.T_max = T_own;
  x.gamma_max = a->gamma_max;
  x.S = pl.S2;
  x.wide = pl.wide2;
  x.s_off = pl.S1;
  rc = launch_attn_rows(x, st);
  if (rc != TANDEM_OK) return rc;
  return launch_attn_combine(x.part_ml, x.part_o, out, (int)rows, S, a->dh, a->dtype, st);
}

size_t tandem_block_prefix_attn_workspace(const tandem_attn_desc* a, int32_t q_len) {
  return tandem_block_attn_workspace(a, q_len);
}

int tandem_block_prefix_attn(const tandem_attn_desc* a, const void* q, const void* k_cache, const void* v_cache,
                             const int32_t* n_prefix, int32_t q_len, int32_t gamma, void* out, void* ws, size_t ws_bytes,
                             void* hip_stream) {
  int rc = check_attn_desc(a);
  if (rc != TANDEM_OK) return rc;
  if (!q || !k_cache || !v_cache || !n_prefix || !out) return TANDEM_ERR_NULL;
  if (q_len < 1 || q_len > TANDEM_MAX_QLEN || a->T_max < q_len || gamma < 1) return TANDEM_ERR_SHAPE;
  const size_t need = tandem_block_prefix_attn_workspace(a, q_len);
  if (need > 0 && !ws) return TANDEM_ERR_NULL;
  if (ws_bytes < need) return TANDEM_ERR_WORKSPACE;
  AttnArgs x{};
  x.q = q;
  x.kA = k_cache;
  x.vA = v_cache;
  x.nA = n_prefix;
  x.B = a->B;
  x.Hq = a->Hq;
  x.Hkv = a->Hkv;
  x.dh = a->dh;
  x.q_len = q_len;
  x.T_max = a->T_max;
  x.scale = a->scale;
  x.dtype = a->dtype;
  x.out = out;
  x.gamma = gamma;
  const bool mfma = block_uses_mfma(a);
  x.mixed = mfma ? 1 : 3;  // the first key segment of the all-positions attention, alone
  x.S = mfma ? attn_block_splits(a->B, a->Hkv, q_len, a->Hq / a->Hkv, a->T_max, &x.wide)
             : attn_rows_splits(a->B, a->Hkv, q_len, a->Hq / a->Hkv, a->T_max, 0, &x.wide);
  if (x.S > 1) carve(ws, (size_t)a->B * q_len * a->Hq, x.S, &x.part_ml, &x.part_o);
  return mfma ? launch_attn_block(x, (hipStream_t)hip_stream) : launch_attn_rows(x, (hipStream_t)hip_stream);
}

size_t tandem_mixed_attn_workspace(const tandem_attn_desc* a, int32_t q_len) {
  if (check_attn_desc(a) != TANDEM_OK || q_len < 1 || q_len > TANDEM_MAX_QLEN) return 0;
  const size_t rows = (size_t)a->B * q_len * a->Hq;
  if (block_uses_mfma(a))
    return carved_bytes(rows, attn_block_splits(a->B, a->Hkv, q_len, a->Hq / a->Hkv, a->T_max, nullptr) + 1, a->dh);
  return carved_bytes(rows, attn_rows_splits(a->B, a->Hkv, q_len, a->Hq / a->Hkv, a->T_max, 0, nullptr), a->dh);
}

int tandem_mixed_attn(const tandem_attn_desc* a, const void* q, const void* k_hat, const void* v_hat,
                      const void* k_own, const void* v_own, const int32_t* n_prefix, int32_t q_len, int32_t gamma,
                      void* out, void* ws, size_t ws_bytes, void* hip_stream) {
  int rc = check_attn_desc(a);
  if (rc != TANDEM_OK) return rc;
  if (!q || !k_hat || !v_hat || !k_own || !v_own || !n_prefix || !out) return TANDEM_ERR_NULL;
  if (q_len < 1 || q_len > TANDEM_MAX_QLEN || a->T_max < q_len || gamma < 1) return TANDEM_ERR_SHAPE;
  const size_t need = tandem_mixed_attn_workspace(a, q_len);
  if (need > 0 && !ws) return TANDEM_ERR_NULL;
  if (ws_bytes < need) return TANDEM_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t rows = (size_t)a->B * q_len * a->Hq;
  AttnArgs x{};
  x.q = q;
  x.nA = n_prefix;
  x.B = a->B;
  x.Hq = a->Hq;
  x.Hkv = a->Hkv;
  x.dh = a->dh;
  x.q_len = q_len;
  x.T_max = a->T_max;
  x.scale = a->scale;
  x.dtype = a->dtype;
  x.out = out;
  x.gamma = gamma;
  if (!block_uses_mfma(a)) {
    // generic kernel: both sources in one launch, one workgroup per query row and KV head
    x.kA = k_hat;
    x.vA = v_hat;
    x.kB = k_own;
    x.vB = v_own;
    x.mixed = 3;
    x.wide = 0;
    x.S = attn_rows_splits(a->B, a->Hkv, q_len, a->Hq / a->Hkv, a->T_max, 0, &x.wide);
    if (x.S > 1) carve(ws, rows, x.S, &x.part_ml, &x.part_o);
    return launch_attn_rows(x, st);
  }
  // matrix-core kernels: the rows derived from the large model first (split over the context), then the few own
  // rows of the blocks in flight, whose launch folds the first segment's partials in and finishes the rows
  const int S1 = attn_block_splits(a->B, a->Hkv, q_len, a->Hq / a->Hkv, a->T_max, &x.wide);
  x.S_total = S1 + 1;
  carve(ws, rows, x.S_total, &x.part_ml, &x.part_o);
  x.kA = k_hat;
  x.vA = v_hat;
  x.mixed = 1;
  x.S = S1;
  x.s_off = 0;
  rc = launch_attn_block(x, st);
  if (rc != TANDEM_OK) return rc;
  x.kA = k_own;
  x.vA = v_own;
  x.mixed = 2;
  x.wide = 0;
  x.S = 1;
  x.s_off = S1;
  x.merge_prev = S1;
  return launch_attn_block(x, st);
}

}  // extern "C"
