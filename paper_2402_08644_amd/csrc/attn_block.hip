// Block-mode attention of the large model on the matrix cores (Sec. 1 step 3, Sec. 3
// "Inference", Eq. (1) restricted to the q_len new rows; the SPEED verifier of Sec. 3.1).
// All R = G * q_len query rows that share a KV head (G query heads per KV head, q_len block
// positions) are handled by one workgroup, so each K and V row is read from HBM exactly once
// and feeds R rows: R flop per KV byte - past the vector ALUs, a few percent of MFMA peak.
//
// Each wavefront works alone on 32-key tiles (no workgroup barrier in the main loop):
//   * a tile's K and V rows come through a 16 KB piece of LDS that belongs to the wavefront: direct
//     global-to-LDS loads of whole rows (non-temporal), then 16-byte reads in the MFMA A-operand layout
//     (lane = key row l%16, the 16 bytes at dh offset 32c + 8*(l/16));
//   * S^T[key, q] = K Q^T with v_mfma_f32_16x16x32_bf16, Q^T held in registers;
//   * online softmax per query column (one column per lane, 2 cross-lane max steps per tile);
//   * the C-layout of two 16-key score tiles already IS the B-operand layout of P^T for a
//     32-deep contraction when contraction index 8g+j is mapped to key 4g+j (j<4) and
//     16+4g+j-4 (j>=4), so P never moves between lanes;
//   * V is brought into the matching A-operand layout (keys along the contraction) by
//     multiplying each 16x32 piece with a 0/1 selection matrix on the matrix cores - an
//     exact transpose that needs no barrier;
//   * O^T[d, q] += V^T P^T.
// Wavefront states are merged through LDS at the end, context splits through the workspace.
#include "common.h"
#include "kernels.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct BlockParams {
  const bf16_t *q, *k, *v;
  const int32_t* n;
  int Hq, Hkv, q_len, G, S;
  int causal;         // 1: the q_len rows are the last rows of the cache (row r sees n + r + 1 keys); 0: all see n keys
  int S_total, s_off;  // partial slots per row and this launch's first slot
  int mixed, gamma;    // attn_mrows_kernel only: 1 / 2 = first / second key segment of the all-positions small-model attention
  long long row_skip;  // q / out hold (q_len * Hq + row_skip) rows per sequence (a call on part of the rows)
  int n_off;           // added to n[b]
  int merge_prev;      // > 0 (needs S == 1): merge slots [0, merge_prev) into this launch's result and write out
  long long T_max;
  float scale_log2e;
  bf16_t* out;
  float* part_ml;
  float* part_o;
};

__device__ __forceinline__ bf16x8 ld_bf16x8(const bf16_t* p) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p));
}
// fp32 values that are bf16 values already (the transposed copies of V that come out of the selection products):
// the upper halves of two words, one byte-permute instruction per pair
__device__ __forceinline__ bf16x8 pack8_exact(const f32x4& a, const f32x4& b) {
  auto hi2 = [](float lo, float hi) {
    return __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, hi), __builtin_bit_cast(uint32_t, lo), 0x07060302u);
  };
  uint4 u;
  u.x = hi2(a[0], a[1]);
  u.y = hi2(a[2], a[3]);
  u.z = hi2(b[0], b[1]);
  u.w = hi2(b[2], b[3]);
  return __builtin_bit_cast(bf16x8, u);
}
// rounding to bf16 with the conversion instruction (round to nearest even, NaN stays NaN)
__device__ __forceinline__ bf16x8 pack8_hw(const f32x4& a, const f32x4& b) {
  uint4 u;
  u.x = pack_bf16x2(a[0], a[1]);
  u.y = pack_bf16x2(a[2], a[3]);
  u.z = pack_bf16x2(b[0], b[1]);
  u.w = pack_bf16x2(b[2], b[3]);
  return __builtin_bit_cast(bf16x8, u);
}
// maximum over the four lanes l, l ^ 16, l ^ 32, l ^ 48 with the row-swap instructions (no LDS traffic: the LDS
// pipeline is busy with the incoming tiles).  v_permlane16_swap exchanges rows 1 and 3 of its first operand with
// rows 0 and 2 of its second, v_permlane32_swap the upper half of the first with the lower half of the second:
// started from two copies of x, the two operands hold x of both partners in every lane afterwards.  Written as
// asm because the compiler's builtin hands back the first result twice; the s_nop covers the wait states the
// instruction needs after a vector write of its operands.  All lanes must be active.
__device__ __forceinline__ float max_over_rows(float x) {
  float y = x;
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(x), "+v"(y));
  x = fmaxf(x, y);
  y = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(x), "+v"(y));
  return fmaxf(x, y);
}
__device__ __forceinline__ f32x4 mfma16(const bf16x8& a, const bf16x8& b, const f32x4& c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Result of one query column (lane group c16; this lane holds output elements 16 db + 4 g4 + r4): the finished
// row when this launch sees all keys, its partial (m, l, O) otherwise.  With merge_prev the partials that earlier
// launches left for this row are folded in first, in slot order, and the row is finished here.
__device__ __forceinline__ void write_row(const BlockParams& p, long long orow, int b, int s, int g4, float m, float l,
                                          f32x4 (&acc)[8]) {
  if (p.merge_prev > 0) {
    for (int t = 0; t < p.merge_prev; ++t) {
      const long long ps = orow * p.S_total + t;
      const float mo = p.part_ml[ps * 2], lo = p.part_ml[ps * 2 + 1];
      const float mn = fmaxf(m, mo);
      const float ca = fast_exp2(m - mn), cb = fast_exp2(mo - mn);
      m = mn;
      l = l * ca + lo * cb;
      const float* op = p.part_o + ps * 128 + 4 * g4;
#pragma unroll
      for (int db = 0; db < 8; ++db) {
        const float4 o = *reinterpret_cast<const float4*>(op + 16 * db);
        acc[db][0] = acc[db][0] * ca + o.x * cb;
        acc[db][1] = acc[db][1] * ca + o.y * cb;
        acc[db][2] = acc[db][2] * ca + o.z * cb;
        acc[db][3] = acc[db][3] * ca + o.w * cb;
      }
    }
  }
  if (p.S_total == 1 || p.merge_prev > 0) {
    const float inv = l > 0.f ? 1.f / l : 0.f;
    bf16_t* op = p.out + (orow + b * p.row_skip) * 128 + 4 * g4;
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      uint2 u;
      u.x = pack_bf16x2(acc[db][0] * inv, acc[db][1] * inv);
      u.y = pack_bf16x2(acc[db][2] * inv, acc[db][3] * inv);
      *reinterpret_cast<uint2*>(op + 16 * db) = u;
    }
  } else {
    const long long ps = orow * p.S_total + p.s_off + s;
    float* op = p.part_o + ps * 128 + 4 * g4;
#pragma unroll
    for (int db = 0; db < 8; ++db)
      *reinterpret_cast<float4*>(op + 16 * db) = make_float4(acc[db][0], acc[db][1], acc[db][2], acc[db][3]);
    if (g4 == 0) {
      p.part_ml[ps * 2 + 0] = m;
      p.part_ml[ps * 2 + 1] = l;
    }
  }
}

// The same for one block of 16 output elements (db): this lane's four values o of elements 16 db + 4 g4 + r4.  Used
// by the merge of attn_block_kernel, where every wavefront finishes one such block of every row.
__device__ __forceinline__ void write_piece(const BlockParams& p, long long orow, int b, int s, int g4, int db, float m,
                                            float l, f32x4 o) {
  if (p.merge_prev > 0) {
    for (int t = 0; t < p.merge_prev; ++t) {
      const long long ps = orow * p.S_total + t;
      const float mo = p.part_ml[ps * 2], lo = p.part_ml[ps * 2 + 1];
      const float mn = fmaxf(m, mo);
      const float ca = fast_exp2(m - mn), cb = fast_exp2(mo - mn);
      m = mn;
      l = l * ca + lo * cb;
      const float4 q = *reinterpret_cast<const float4*>(p.part_o + ps * 128 + 4 * g4 + 16 * db);
      o[0] = o[0] * ca + q.x * cb;
      o[1] = o[1] * ca + q.y * cb;
      o[2] = o[2] * ca + q.z * cb;
      o[3] = o[3] * ca + q.w * cb;
    }
  }
  if (p.S_total == 1 || p.merge_prev > 0) {
    const float inv = l > 0.f ? 1.f / l : 0.f;
    uint2 u;
    u.x = pack_bf16x2(o[0] * inv, o[1] * inv);
    u.y = pack_bf16x2(o[2] * inv, o[3] * inv);
    *reinterpret_cast<uint2*>(p.out + (orow + b * p.row_skip) * 128 + 4 * g4 + 16 * db) = u;
  } else {
    const long long ps = orow * p.S_total + p.s_off + s;
    *reinterpret_cast<float4*>(p.part_o + ps * 128 + 4 * g4 + 16 * db) = make_float4(o[0], o[1], o[2], o[3]);
    if (g4 == 0 && db == 0) {
      p.part_ml[ps * 2 + 0] = m;
      p.part_ml[ps * 2 + 1] = l;
    }
  }
}

constexpr int ST_REGS = 34;  // per-lane state of one row tile: m, l, 32 accumulators

// NW wavefronts per workgroup (4 or 8): eight put the work of two context splits into one workgroup, whose
// wavefronts merge through LDS, so that no partials leave the workgroup and no combine kernel follows.
template <int RT, int NW>
__global__ __launch_bounds__(64 * NW, (RT <= 2 && NW == 4 ? 2 : 1)) void attn_block_kernel(BlockParams p) {
  extern __shared__ float lds[];  // staging pieces [NW][16 KB] inside the loop, then the states [NW][RT][ST_REGS][64]
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int g4 = lane >> 4, c16 = lane & 15;
  const int s = blockIdx.x, b = blockIdx.z;
  const int kvh = blockIdx.y % p.Hkv, pass = blockIdx.y / p.Hkv;

  long long n = (long long)p.n[b] + p.n_off;
  // mixed == 1: first key segment of the all-positions small-model attention (see attn_mrows_kernel): row r sees
  // the keys below its block boundary kb(n + r), no lower limit - the only segment form this kernel takes
  const int ext = (p.causal || p.mixed) ? p.q_len : 0;
  const long long nmax = p.T_max - ext;
  n = n < 0 ? 0 : (n > nmax ? nmax : n);
  const long long total = p.mixed ? (n + p.q_len - 1) / p.gamma * p.gamma : n + ext;
  const int R = p.G * p.q_len;

  const long long ntiles = (total + 31) >> 5;
  const long long per = (ntiles + p.S - 1) / p.S;
  const long long tile_begin = (long long)s * per;
  const long long tile_end = ntiles < tile_begin + per ? ntiles : tile_begin + per;

  const bf16_t* kbase = p.k + ((long long)b * p.Hkv + kvh) * p.T_max * 128;
  const bf16_t* vbase = p.v + ((long long)b * p.Hkv + kvh) * p.T_max * 128;

  // Q^T operands and per-lane causal limits
  bf16x8 qreg[RT][4];
  long long lim[RT];
  long long orow[RT];  // output row index of this lane's query column, -1 for padding
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int rho = (pass * RT + rt) * 16 + c16;
    if (rho < R) {
      const int r = rho / p.G, gq = rho % p.G;
      orow[rt] = ((long long)b * p.q_len + r) * p.Hq + kvh * p.G + gq;
      lim[rt] = p.mixed ? (n + r) / p.gamma * p.gamma - 1 : (p.causal ? n + r : n - 1);
      const bf16_t* qp = p.q + (orow[rt] + b * p.row_skip) * 128 + 8 * g4;
#pragma unroll
      for (int c = 0; c < 4; ++c) qreg[rt][c] = ld_bf16x8(qp + 32 * c);
    } else {
      orow[rt] = -1;
      lim[rt] = n;
      const uint4 z = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int c = 0; c < 4; ++c) qreg[rt][c] = __builtin_bit_cast(bf16x8, z);
    }
  }

  // selection matrices: sel[h][k = 8*g4 + j][col = c16] = (k == c16 + 16 h)
  bf16x8 sel[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    uint32_t wv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t lo = (8 * g4 + 2 * i == c16 + 16 * h) ? 0x3F80u : 0u;
      const uint32_t hi = (8 * g4 + 2 * i + 1 == c16 + 16 * h) ? 0x3F80u : 0u;
      wv[i] = lo | (hi << 16);
    }
    const uint4 u = {wv[0], wv[1], wv[2], wv[3]};
    sel[h] = __builtin_bit_cast(bf16x8, u);
  }

  float m[RT], l[RT];
  f32x4 acc[RT][8];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    m[rt] = TANDEM_NEG_BIG;
    l[rt] = 0.f;
#pragma unroll
    for (int db = 0; db < 8; ++db) acc[rt][db] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  // K and V tiles (32 keys, 8 KB each) reach the wavefront through a private 16 KB piece of LDS: direct
  // global-to-LDS loads of 1 KB (four whole rows per instruction, so that every instruction reads whole cache
  // lines; loading the MFMA operand layout directly touches 64 of every 128 bytes per instruction, and with
  // the non-temporal hint that halves the rate), then operand reads in the layout of the two products.  Lane
  // (r4, slot) of load i brings piece slot ^ (row & 15) of tile row 4 i + r4: the operand reads of 16 rows at
  // one piece index then fall into 16 different 16-byte bank groups.  The loads of the next tile's K (V) are
  // issued as soon as this tile's K (V) operands are in registers and fly during the arithmetic.
  unsigned char* const stg = reinterpret_cast<unsigned char*>(lds) + w * 16384;
  // (addresses: a uniform tile base plus a 32-bit lane offset; rows past the end re-read the last valid row of the
  // tile - there is one, a tile starts below `total` - and are masked below)
  auto issue = [&](const bf16_t* base, unsigned char* dst, long long ti) __attribute__((always_inline)) {
    const long long key0 = ti << 5;
    const unsigned char* tile = reinterpret_cast<const unsigned char*>(base + key0 * 128);
    asm volatile("" : "+s"(tile));  // one scalar base: the loads take it with a 32-bit lane offset
    const long long left = total - 1 - key0;
    const int last = left < 31 ? (int)left : 31;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int rl = 4 * i + g4;
      const uint32_t off = (uint32_t)(rl < last ? rl : last) * 256u + 16u * (uint32_t)(c16 ^ (rl & 15));
      __builtin_amdgcn_global_load_lds((global_void_ptr)(tile + off), (lds_void_ptr)(dst + 1024 * i), 16, 0, 2);
    }
  };
  // Loads complete in issue order and the order is K(t), V(t), K(t + NW), V(t + NW), ...: with eight loads per half
  // tile, "at most eight outstanding" means that the older half has arrived.
  if (tile_begin + w < tile_end) {
    issue(kbase, stg, tile_begin + w);
    issue(vbase, stg + 8192, tile_begin + w);
  }
  for (long long ti = tile_begin + w; ti < tile_end; ti += NW) {
    const long long key0 = ti << 5;
    const bool more = ti + NW < tile_end;
    bf16x8 kreg[2][4], vreg[2][4];
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int c = 0; c < 4; ++c)
        kreg[sub][c] = __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const uint4*>(stg + (16 * sub + c16) * 256 + 16 * ((4 * c + g4) ^ c16)));
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    f32x4 qk[RT][2];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c) a = mfma16(kreg[sub][c], qreg[rt][c], a);
        qk[rt][sub] = a;
      }
    // the K operands are consumed: the next tile's K may overwrite the staging piece
    __builtin_amdgcn_sched_barrier(0);
    if (more) issue(kbase, stg, ti + NW);
    __builtin_amdgcn_sched_barrier(0);

    bf16x8 pb[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      f32x4 sc[2];
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        f32x4 a = qk[rt][sub];
        const long long kidx = key0 + 16 * sub + 4 * g4;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) a[r4] = (kidx + r4 <= lim[rt]) ? a[r4] * p.scale_log2e : -INFINITY;
        sc[sub] = a;
      }
      float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                       fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
      mx = max_over_rows(mx);
      const float mn = fmaxf(m[rt], mx);
      const float corr = fast_exp2(m[rt] - mn);
      m[rt] = mn;
      float ps = 0.f;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          sc[sub][r4] = fast_exp2(sc[sub][r4] - mn);
          ps += sc[sub][r4];
        }
      l[rt] = l[rt] * corr + ps;
#pragma unroll
      for (int db = 0; db < 8; ++db) acc[rt][db] *= corr;
      pb[rt] = pack8_hw(sc[0], sc[1]);
    }

    if (more)
      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int c = 0; c < 4; ++c)
        vreg[sub][c] = __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const uint4*>(stg + 8192 + (16 * sub + c16) * 256 + 16 * ((4 * c + g4) ^ c16)));
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    bf16x8 vt[8];
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      const f32x4 z = {0.f, 0.f, 0.f, 0.f};
      const f32x4 t0 = mfma16(vreg[0][db >> 1], sel[db & 1], z);
      const f32x4 t1 = mfma16(vreg[1][db >> 1], sel[db & 1], z);
      vt[db] = pack8_exact(t0, t1);
    }
    // likewise for V, once its transposed copies are in registers
    __builtin_amdgcn_sched_barrier(0);
    if (more) issue(vbase, stg + 8192, ti + NW);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int db = 0; db < 8; ++db)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) acc[rt][db] = mfma16(vt[db], pb[rt], acc[rt][db]);
  }

  // row sums: lanes l, l^16, l^32, l^48 hold partial sums of the same query column
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    l[rt] += __shfl_xor(l[rt], 16);
    l[rt] += __shfl_xor(l[rt], 32);
  }

  // Merge of the wavefronts through LDS (lane-local: all waves use the same layout), in one step: every wavefront
  // parks its state, then wavefront w finishes the output elements 16 db .. 16 db + 15 of every row for db = w, w + NW,
  // ...: it combines the NW states in wavefront order (a fixed order: results do not depend on timing) and writes
  // its piece.  (A tree of pairwise merges took three to six barriers and left the writing to one wavefront.)
  auto slot = [&](int wv, int rt, int reg) -> float& { return lds[((wv * RT + rt) * ST_REGS + reg) * 64 + lane]; };
  __syncthreads();  // the states take the place of the staging pieces: every wavefront has left its loop
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    slot(w, rt, 0) = m[rt];
    slot(w, rt, 1) = l[rt];
#pragma unroll
    for (int db = 0; db < 8; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) slot(w, rt, 2 + db * 4 + r4) = acc[rt][db][r4];
  }
  __syncthreads();
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    float mi[NW], mm = TANDEM_NEG_BIG;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      mi[i] = slot(i, rt, 0);
      mm = fmaxf(mm, mi[i]);
    }
    float ll = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      mi[i] = fast_exp2(mi[i] - mm);  // weight of state i
      ll += slot(i, rt, 1) * mi[i];
    }
    for (int db = w; db < 8; db += NW) {
      f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < NW; ++i)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) o[r4] += slot(i, rt, 2 + db * 4 + r4) * mi[i];
      if (orow[rt] >= 0) write_piece(p, orow[rt], b, s, g4, db, mm, ll, o);
    }
  }
}

// Many query rows per KV head (G * q_len > 32: long prompt blocks, several samples per prompt).  Splitting the
// keys over the wavefronts, as above, would need one pass over K and V per 32 rows; here the wavefronts split
// the ROWS instead - wavefront w owns row tile w (16 query columns) for the whole key range of the workgroup,
// so no merge between wavefronts is needed - and every 32-key tile is fetched from HBM once per workgroup and
// handed to all wavefronts through LDS, already in the operand layouts of the two products:
//   * chunks 0..7:  K operand pieces (sub, c), a plain copy of what each lane would have loaded itself;
//   * chunks 8..15: V^T operand pieces db, transposed once per workgroup on the matrix cores (selection
//     matrices, as above).
// The eight staging units of a tile (4 of K, 4 of V) are dealt round-robin to the wavefronts; their global loads
// for tile t + 1 are in flight while tile t is multiplied.  One barrier per tile, two LDS buffers.
// MIXED = false compiles the per-row lower key limit and the segment logic out (they cost registers: 121 -> 134 at
// five wavefronts, one wavefront per SIMD less).
template <int NW, int D, bool MIXED>
__global__ __launch_bounds__(64 * NW) void attn_mrows_kernel(BlockParams p) {
  __shared__ uint4 buf[2][16][64];
  constexpr int NU = (8 + NW - 1) / NW;  // staging units per wavefront
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int g4 = lane >> 4, c16 = lane & 15;
  const int s = blockIdx.x, b = blockIdx.z;
  const int kvh = blockIdx.y % p.Hkv, pass = blockIdx.y / p.Hkv;

  // Key range and per-row visibility.  Ordinary block (mixed == 0): keys [0, total), row r sees keys <= lim.
  // All-positions small-model attention (Eq. (2) with the query's own block boundary kb(i) = floor(i / gamma)
  // * gamma, i = n + r): segment 1 reads the rows derived from the large model, keys [0, kb(i)); segment 2 the
  // model's own rows, keys [kb(i), i].
  long long n = (long long)p.n[b] + p.n_off;
  const int mixed = MIXED ? p.mixed : 0;
  const int ext = (p.causal || mixed) ? p.q_len : 0;
  const long long nmax = p.T_max - ext;
  n = n < 0 ? 0 : (n > nmax ? nmax : n);
  auto kb = [&](long long i) { return i / p.gamma * p.gamma; };
  const long long total = mixed == 1 ? kb(n + p.q_len - 1) : n + ext;
  const long long first = mixed == 2 ? kb(n) >> 5 : 0;  // first tile that any row can see
  const int R = p.G * p.q_len;

  const long long ntiles = ((total + 31) >> 5) - first;
  const long long per = (ntiles + p.S - 1) / p.S;
  const long long tile_begin = first + (long long)s * per;
  const long long tile_end = first + (ntiles < (s + 1) * per ? ntiles : (s + 1) * per);

  const bf16_t* kbase = p.k + ((long long)b * p.Hkv + kvh) * p.T_max * 128;
  const bf16_t* vbase = p.v + ((long long)b * p.Hkv + kvh) * p.T_max * 128;

  // scores are taken as (+-Q K) * |scale|: a negative scale is moved into Q's sign bits (exact)
  const float absl = fabsf(p.scale_log2e);
  const uint32_t flip = p.scale_log2e < 0.f ? 0x80008000u : 0u;
  bf16x8 qreg[4];
  long long lim, lo = 0, orow;  // this lane's query column sees keys lo .. lim
  {
    const int rho = (pass * NW + w) * 16 + c16;
    if (rho < R) {
      const int r = rho / p.G, gq = rho % p.G;
      orow = ((long long)b * p.q_len + r) * p.Hq + kvh * p.G + gq;
      if (mixed == 1) {
        lim = kb(n + r) - 1;
      } else if (mixed == 2) {
        lim = n + r;
        lo = kb(n + r);
      } else {
        lim = p.causal ? n + r : n - 1;
      }
      const bf16_t* qp = p.q + (orow + b * p.row_skip) * 128 + 8 * g4;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        uint4 u = *reinterpret_cast<const uint4*>(qp + 32 * c);
        u.x ^= flip, u.y ^= flip, u.z ^= flip, u.w ^= flip;
        qreg[c] = __builtin_bit_cast(bf16x8, u);
      }
    } else {
      orow = -1;
      lim = total;  // padding columns: Q = 0, everything visible, never written
      const uint4 z = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int c = 0; c < 4; ++c) qreg[c] = __builtin_bit_cast(bf16x8, z);
    }
  }
  long long lim_min = lim, lo_max = lo;  // tightest limits among the wavefront's rows
#pragma unroll
  for (int off = 1; off < 16; off <<= 1) {
    const long long o = __shfl_xor(lim_min, off), u = __shfl_xor(lo_max, off);
    lim_min = o < lim_min ? o : lim_min;
    lo_max = u > lo_max ? u : lo_max;
  }

  bf16x8 sel[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    uint32_t wv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t lo = (8 * g4 + 2 * i == c16 + 16 * h) ? 0x3F80u : 0u;
      const uint32_t hi = (8 * g4 + 2 * i + 1 == c16 + 16 * h) ? 0x3F80u : 0u;
      wv[i] = lo | (hi << 16);
    }
    const uint4 u = {wv[0], wv[1], wv[2], wv[3]};
    sel[h] = __builtin_bit_cast(bf16x8, u);
  }

  float m = TANDEM_NEG_BIG, l = 0.f;
  f32x4 acc[8];
#pragma unroll
  for (int db = 0; db < 8; ++db) acc[db] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // staging unit u of a tile: u < 4 - V columns [32u, 32u + 32) of its 32 rows; u >= 4 - the same of K
  // D tiles ahead are in flight in registers
  uint4 raw[D][NU][2];
  auto issue = [&](int j, long long ti) {
#pragma unroll
    for (int i = 0; i < NU; ++i) {
      const int u = w + i * NW;
      if (u < 8) {
        const bf16_t* base = (u >= 4 ? kbase : vbase) + 32 * (u & 3) + 8 * g4;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
          long long row = (ti << 5) + 16 * sub + c16;
          row = row < total ? row : total - 1;  // rows past the end are re-reads of a valid row, masked below
          raw[j][i][sub] = *reinterpret_cast<const uint4*>(base + row * 128);
        }
      }
    }
  };
  auto stage = [&](int j, int bi) {
#pragma unroll
    for (int i = 0; i < NU; ++i) {
      const int u = w + i * NW;
      if (u >= 8) continue;
      const int c = u & 3;
      if (u >= 4) {
        buf[bi][c][lane] = raw[j][i][0];
        buf[bi][4 + c][lane] = raw[j][i][1];
      } else {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        const bf16x8 v0 = __builtin_bit_cast(bf16x8, raw[j][i][0]), v1 = __builtin_bit_cast(bf16x8, raw[j][i][1]);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const f32x4 t0 = mfma16(v0, sel[h], z);
          const f32x4 t1 = mfma16(v1, sel[h], z);
          buf[bi][8 + 2 * c + h][lane] = __builtin_bit_cast(uint4, pack8_hw(t0, t1));
        }
      }
    }
  };

#pragma unroll
  for (int j = 0; j < D; ++j)
    if (tile_begin + j < tile_end) issue(j, tile_begin + j);
  for (long long t0 = tile_begin; t0 < tile_end; t0 += D) {
#pragma unroll
  for (int j = 0; j < D; ++j) {
    const long long ti = t0 + j;
    if (ti >= tile_end) break;
    const int bi = (int)(ti - tile_begin) & 1;
    stage(j, bi);
    if (ti + D < tile_end) issue(j, ti + D);
    __syncthreads();  // tile ti is complete in buf[bi]; buf[1 - bi] is free again (everyone finished tile ti - 1)

    const long long key0 = ti << 5;
    f32x4 sc[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < 4; ++c) a = mfma16(__builtin_bit_cast(bf16x8, buf[bi][4 * sub + c][lane]), qreg[c], a);
      sc[sub] = a;
    }
    // wave-uniform: some key of this tile is hidden from some row
    const bool edge = key0 + 31 > lim_min || (MIXED && key0 < lo_max);
    uint32_t seen = 0xffu;  // bit 4 sub + r4: this lane's score is of a visible key
    if (edge) {
      seen = 0;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const long long kidx = key0 + 16 * sub + 4 * g4;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const bool ok = kidx + r4 <= lim && (!MIXED || kidx + r4 >= lo);
          seen |= ok ? 1u << (4 * sub + r4) : 0u;
          sc[sub][r4] = ok ? sc[sub][r4] : -INFINITY;
        }
      }
    }
    float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                     fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));  // (LDS shuffles: this kernel is bound by its vector instructions, and the
    mx = fmaxf(mx, __shfl_xor(mx, 32));  // row-swap form costs more of them: 438 against 422 us per prompt layer)
    mx *= absl;
    // The running maximum m is only raised when some row's scores pass it by more than 2^8 (weights stay
    // below 256, exact in the fp32 sums; the result does not depend on which m is subtracted), so the
    // rescaling of the 32 accumulators is skipped for almost every tile.
    if (__builtin_amdgcn_ballot_w64(mx > m + 8.f) != 0) {
      const float mn = fmaxf(m, mx);
      const float corr = fast_exp2(m - mn);
      m = mn;
      l *= corr;
#pragma unroll
      for (int db = 0; db < 8; ++db) acc[db] *= corr;
    }
    float ps = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const float e = fast_exp2(fmaf(sc[sub][r4], absl, -m));
        sc[sub][r4] = (seen >> (4 * sub + r4)) & 1u ? e : 0.f;  // (-inf * 0 is not a number when the scale is 0)
        ps += sc[sub][r4];
      }
    l += ps;
    const bf16x8 pb = pack8_hw(sc[0], sc[1]);
#pragma unroll
    for (int db = 0; db < 8; ++db)
      acc[db] = mfma16(__builtin_bit_cast(bf16x8, buf[bi][8 + db][lane]), pb, acc[db]);
  }
  }

  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  if (orow >= 0) write_row(p, orow, b, s, g4, m, l, acc);
}

template <int NW>
int launch_mrows(const BlockParams& p, int passes, int B, hipStream_t st) {
  if (p.mixed)
    hipLaunchKernelGGL((attn_mrows_kernel<NW, 1, true>), dim3(p.S, p.Hkv * passes, B), dim3(64 * NW), 0, st, p);
  else
    hipLaunchKernelGGL((attn_mrows_kernel<NW, 1, false>), dim3(p.S, p.Hkv * passes, B), dim3(64 * NW), 0, st, p);
  return hip_ok(hipGetLastError());
}

template <int RT, int NW>
int launch_rt(const BlockParams& p, int passes, int B, hipStream_t st) {
  const size_t state_bytes = (size_t)NW * RT * ST_REGS * 64 * sizeof(float), stage_bytes = (size_t)NW * 16384;
  const size_t lds_bytes = state_bytes > stage_bytes ? state_bytes : stage_bytes;
  if (const int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(&attn_block_kernel<RT, NW>), lds_bytes)) return rc;
  hipLaunchKernelGGL((attn_block_kernel<RT, NW>), dim3(p.S, p.Hkv * passes, B), dim3(64 * NW), lds_bytes, st, p);
  return hip_ok(hipGetLastError());
}

}  // namespace

bool attn_block_supported(const AttnArgs& a) { return a.dtype == TANDEM_BF16 && a.dh == 128 && !a.kB; }

// Context splits: a function of shapes only.  Measured on MI355X: about 512 workgroups in total (two
// per CU) stream best; more splits only add partials and tail effects.  At least 8 tiles (256 keys) each.
int attn_block_splits(int B, int Hkv, int q_len, int G, int64_t T_max, int* wide) {
  // more than 32 query rows per KV head run as row passes of up to 128 rows, each a workgroup of its own
  const int tiles = (G * q_len + 15) / 16;
  const int64_t groups = (int64_t)B * Hkv * (tiles > 2 ? (tiles + 7) / 8 : 1);
  int64_t want = (512 + groups - 1) / groups;
  int64_t cap = T_max / 256;
  if (cap < 1) cap = 1;
  int64_t S = want < cap ? want : cap;
  if (S < 1) S = 1;
  if (S > 64) S = 64;
  // an even number of splits becomes half as many workgroups of eight wavefronts (up to 32 query rows)
  const bool w8 = S % 2 == 0 && G * q_len <= 32;
  if (wide) *wide = w8 ? 1 : 0;
  return (int)(w8 ? S / 2 : S);
}

size_t attn_block_workspace(int B, int Hq, int q_len, int S) {
  if (S <= 1) return 0;
  return (size_t)B * q_len * Hq * S * (128 + 2) * sizeof(float);
}

int launch_attn_block(const AttnArgs& a, hipStream_t st) {
  BlockParams p;
  p.q = (const bf16_t*)a.q;
  p.k = (const bf16_t*)a.kA;
  p.v = (const bf16_t*)a.vA;
  p.n = a.nA;
  p.Hq = a.Hq;
  p.Hkv = a.Hkv;
  p.q_len = a.q_len;
  p.G = a.Hq / a.Hkv;
  p.S = a.S;
  p.causal = a.causal;
  p.S_total = a.S_total > 0 ? a.S_total : a.S;
  p.s_off = a.S_total > 0 ? a.s_off : 0;
  p.merge_prev = a.S_total > 0 && a.S == 1 ? a.merge_prev : 0;
  p.mixed = a.mixed;
  p.row_skip = a.q_rows > a.q_len ? (long long)(a.q_rows - a.q_len) * a.Hq : 0;
  p.n_off = a.n_off;
  p.gamma = a.gamma > 0 ? a.gamma : 1;
  p.T_max = a.T_max;
  p.scale_log2e = a.scale * 1.4426950408889634f;
  p.out = (bf16_t*)a.out;
  p.part_ml = a.part_ml;
  p.part_o = a.part_o;
  const int R = p.G * a.q_len;
  const int tiles = (R + 15) / 16;
  int rc;
  if (a.mixed == 2 || (a.mixed == 1 && tiles > 2)) {
    // per-row key ranges with a lower end exist in the row-split kernel only
    const int passes = (tiles + 7) / 8;
    switch ((tiles + passes - 1) / passes) {
      case 1: rc = launch_mrows<1>(p, passes, a.B, st); break;
      case 2: rc = launch_mrows<2>(p, passes, a.B, st); break;
      case 3: rc = launch_mrows<3>(p, passes, a.B, st); break;
      case 4: rc = launch_mrows<4>(p, passes, a.B, st); break;
      case 5: rc = launch_mrows<5>(p, passes, a.B, st); break;
      case 6: rc = launch_mrows<6>(p, passes, a.B, st); break;
      case 7: rc = launch_mrows<7>(p, passes, a.B, st); break;
      default: rc = launch_mrows<8>(p, passes, a.B, st); break;
    }
  } else if (tiles == 1)
    rc = a.wide ? launch_rt<1, 8>(p, 1, a.B, st) : launch_rt<1, 4>(p, 1, a.B, st);
  else if (tiles == 2)
    rc = a.wide ? launch_rt<2, 8>(p, 1, a.B, st) : launch_rt<2, 4>(p, 1, a.B, st);
  else {
    // more than 32 rows: the wavefronts split the rows, up to 128 rows per pass over K and V
    const int passes = (tiles + 7) / 8;
    const int nw = (tiles + passes - 1) / passes;
    switch (nw) {
      case 3: rc = launch_mrows<3>(p, passes, a.B, st); break;
      case 4: rc = launch_mrows<4>(p, passes, a.B, st); break;
      case 5: rc = launch_mrows<5>(p, passes, a.B, st); break;
      case 6: rc = launch_mrows<6>(p, passes, a.B, st); break;
      case 7: rc = launch_mrows<7>(p, passes, a.B, st); break;
      default: rc = launch_mrows<8>(p, passes, a.B, st); break;
    }
  }
  if (rc != TANDEM_OK || a.S_total > 0 || a.S == 1) return rc;
  return launch_attn_combine(a.part_ml, a.part_o, a.out, a.B * a.q_len * a.Hq, a.S, 128, a.dtype, st, a.q_len * a.Hq,
                             p.row_skip);
}
