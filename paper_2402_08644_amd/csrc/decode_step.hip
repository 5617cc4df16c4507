// tandem_project and tandem_decode_step: host-side orchestration of the kernels for one
// Tandem + SPEED step (Sec. 3.1; Sec. 1 steps 2-4).  Everything is enqueued on one stream;
// lengths, tokens and the acceptance decision stay on the device, so the step never
// synchronises with the host.
#include <new>
#include <unordered_map>
#include <vector>

#include "common.h"
#include "glue.h"
#include "kernels.h"

namespace {

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline size_t elsize(int dtype) { return dtype == TANDEM_BF16 ? 2 : 4; }
inline size_t maxz(size_t a, size_t b) { return a > b ? a : b; }

int check_ff(const tandem_ff_desc* ff) {
  if (!ff) return TANDEM_ERR_NULL;
  if (ff->d_L <= 0 || ff->d_S <= 0 || ff->d_hidden < 0) return TANDEM_ERR_SHAPE;
  if (ff->dtype != TANDEM_F32 && ff->dtype != TANDEM_BF16) return TANDEM_ERR_UNSUPPORTED;
  if (!ff->W1) return TANDEM_ERR_NULL;
  if (ff->d_hidden > 0) {
    if (!ff->W2) return TANDEM_ERR_NULL;
    if (ff->act != TANDEM_ACT_NONE && ff->act != TANDEM_ACT_GELU && ff->act != TANDEM_ACT_RELU)
      return TANDEM_ERR_UNSUPPORTED;
  }
  return TANDEM_OK;
}

size_t project_ws(const tandem_ff_desc* ff, int64_t M) {
  if (ff->d_hidden == 0) return align256(gemm_workspace((int)M, ff->d_S, ff->d_L, ff->dtype));
  const size_t hidden = align256((size_t)M * ff->d_hidden * elsize(ff->dtype));
  const size_t g = maxz(gemm_workspace((int)M, ff->d_hidden, ff->d_L, ff->dtype),
                        gemm_workspace((int)M, ff->d_S, ff->d_hidden, ff->dtype));
  return hidden + align256(g);
}

int gemm(const void* X, int64_t ldx, const void* W, const void* Wp, const void* bias, const void* residual, int64_t ldr, void* Y,
         int64_t ldy, int M, int N, int K, int act, int dtype, void* ws, size_t ws_bytes, hipStream_t st,
         const int32_t* gate = nullptr) {
  GemmArgs g;
  g.gate = gate;
  g.X = X;
  g.ldx = ldx;
  g.W = W;
  g.Wp = Wp;
  g.bias = bias;
  g.residual = residual;
  g.ldr = ldr;
  g.Y = Y;
  g.ldy = ldy;
  g.M = M;
  g.N = N;
  g.K = K;
  g.act = act;
  g.dtype = dtype;
  g.ws = (float*)ws;
  g.ws_bytes = ws_bytes;
  g.defer = 0;
  return launch_gemm(g, st);
}

// X . W^T left as fp32 partial sums in ws (see GemmArgs::defer)
int gemm_deferred(const void* X, int64_t ldx, const void* W, const void* Wp, int M, int N, int K, int dtype, void* ws, size_t ws_bytes,
                  hipStream_t st, const int32_t* gate = nullptr) {
  GemmArgs g{};
  g.gate = gate;
  g.X = X;
  g.ldx = ldx;
  g.W = W;
  g.Wp = Wp;
  g.M = M;
  g.N = N;
  g.K = K;
  g.act = TANDEM_ACT_NONE;
  g.dtype = dtype;
  g.ws = (float*)ws;
  g.ws_bytes = ws_bytes;
  g.defer = 1;
  return launch_gemm(g, st);
}

// y_hat = FF_Tandem(x)   (Eq. (2), first line)
// residual (optional, [M, d_S], may alias y): added to the result
int run_project(const tandem_ff_desc* ff, const void* x, void* y, int64_t M, void* ws, size_t ws_bytes, hipStream_t st,
                const void* residual = nullptr) {
  if (ff->d_hidden == 0)
    return gemm(x, ff->d_L, ff->W1, ff->W1p, ff->b1, residual, ff->d_S, y, ff->d_S, (int)M, ff->d_S, ff->d_L, TANDEM_ACT_NONE,
                ff->dtype, ws, ws_bytes, st);
  const size_t hidden = align256((size_t)M * ff->d_hidden * elsize(ff->dtype));
  void* hbuf = ws;
  void* gws = (char*)ws + hidden;
  const size_t gws_bytes = ws_bytes - hidden;
  int rc = gemm(x, ff->d_L, ff->W1, ff->W1p, ff->b1, nullptr, 0, hbuf, ff->d_hidden, (int)M, ff->d_hidden, ff->d_L, ff->act,
                ff->dtype, gws, gws_bytes, st);
  if (rc != TANDEM_OK) return rc;
  return gemm(hbuf, ff->d_hidden, ff->W2, ff->W2p, ff->b2, residual, ff->d_S, y, ff->d_S, (int)M, ff->d_S, ff->d_hidden,
              TANDEM_ACT_NONE, ff->dtype, gws, gws_bytes, st);
}

int check_decoder(const tandem_decoder_desc& d) {
  if (d.n_layers <= 0 || d.d <= 0 || d.Hq <= 0 || d.Hkv <= 0 || d.d_ff <= 0 || d.vocab <= 0) return TANDEM_ERR_SHAPE;
  if (d.Hq % d.Hkv != 0) return TANDEM_ERR_SHAPE;
  if (d.dh != 64 && d.dh != 128) return TANDEM_ERR_UNSUPPORTED;
  const int G = d.Hq / d.Hkv;
  if (G != 1 && G != 2 && G != 4 && G != 8) return TANDEM_ERR_UNSUPPORTED;
  if (!d.emb || !d.g_final || !d.W_out || !d.layers) return TANDEM_ERR_NULL;
  for (int j = 0; j < d.n_layers; ++j) {
    const tandem_layer_weights& l = d.layers[j];
    if (!l.g_attn || !l.Wqkv || !l.Wo || !l.g_mlp || !l.W1 || !l.W2) return TANDEM_ERR_NULL;
  }
  return TANDEM_OK;
}

}  // namespace

struct tandem_model {
  tandem_model_desc d;
  std::vector<tandem_layer_weights> L_layers, S_layers;
  std::vector<int32_t> ell;
  std::vector<tandem_ff_desc> ff;
  std::unordered_map<const void*, const void*> packed;     // caller's weight pointer -> packed copy (caller's buffer)
  const void* pk(const void* W) const {
    auto it = packed.find(W);
    return it == packed.end() ? nullptr : it->second;
  }
};

namespace {

// The weight matrices of the model that have a packed form (the layout the stream GEMM kernel reads), each once.
struct PackItem {
  const void* W;
  int64_t N, K;
};
std::vector<PackItem> pack_items(const tandem_model* m) {
  std::vector<PackItem> items;
  std::unordered_map<const void*, int> seen;
  const int dt = m->d.dtype;
  auto add = [&](const void* W, int64_t N, int64_t K) {
    if (W && gemm_packable(N, K, dt) && reinterpret_cast<uintptr_t>(W) % 16 == 0 && !seen.count(W)) {
      items.push_back({W, N, K});
      seen[W] = 1;
    }
  };
  auto add_decoder = [&](const tandem_decoder_desc& D) {
    for (int j = 0; j < D.n_layers; ++j) {
      const tandem_layer_weights& l = D.layers[j];
      add(l.Wqkv, (int64_t)(D.Hq + 2 * D.Hkv) * D.dh, D.d);
      add(l.Wo, D.d, (int64_t)D.Hq * D.dh);
      add(l.W1, D.d_ff, D.d);
      add(l.W2, D.d, D.d_ff);
    }
    add(D.W_out, D.vocab, D.d);
  };
  add_decoder(m->d.L);
  add_decoder(m->d.S);
  for (const tandem_ff_desc& f : m->ff) {
    if (f.d_hidden > 0) {
      add(f.W1, f.d_hidden, f.d_L);
      add(f.W2, f.d_S, f.d_hidden);
    } else {
      add(f.W1, f.d_S, f.d_L);
    }
  }
  return items;
}

// Workspace layout of one step, a pure function of (model, B, gamma, T_max, gamma_max).
struct StepPlan {
  size_t x, xn, qkv, q, att, h, logits, yhat, kv, keep, ints, attn_ws, gemm_ws, total;
  size_t attn_ws_bytes, gemm_ws_bytes, keep_stride;
  int32_t n_keep;
  bool fused;  // bf16 path with deferred GEMM epilogues finished by fused row kernels
};

// score: the small model also runs on all B * gamma rows (teacher-forced pass), with the all-positions attention
// samples > 0: the step of several samples per prompt (attention through the shared-prompt entry points)
StepPlan make_plan(const tandem_model* m, int B, int gamma, int64_t T_max, int gamma_max, bool score = false,
                   int samples = 0, int64_t T_prompt = 0) {
  const tandem_decoder_desc &L = m->d.L, &S = m->d.S;
  const size_t es = elsize(m->d.dtype);
  const size_t M = (size_t)B * gamma;
  const size_t dmax = maxz(L.d, S.d);
  const size_t qkvmax = maxz((size_t)(L.Hq + 2 * L.Hkv) * L.dh, (size_t)(S.Hq + 2 * S.Hkv) * S.dh);
  const size_t qmax = maxz((size_t)L.Hq * L.dh, (size_t)S.Hq * S.dh);
  size_t ffmax = maxz(L.d_ff, S.d_ff);
  for (int j = 0; j < S.n_layers; ++j) ffmax = maxz(ffmax, (size_t)m->ff[j].d_hidden);
  const size_t vmax = maxz(L.vocab, S.vocab);
  StepPlan p{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t o = off;
    off += align256(bytes);
    return o;
  };
  p.x = take(M * dmax * es);
  p.xn = take(M * dmax * es);
  p.qkv = take(M * qkvmax * es);
  p.q = take(M * qmax * es);
  p.att = take(M * qmax * es);
  p.h = take(M * ffmax * es);
  p.logits = take(M * vmax * es);
  p.yhat = take(M * S.d * es);
  p.kv = take(M * 2 * S.Hkv * S.dh * es);
  p.n_keep = S.n_layers;
  p.keep_stride = align256(M * L.d * es);
  p.keep = take(p.keep_stride * S.n_layers);
  // ints: ncur[gamma][B] (2 M reserved), draft[B*gamma], verify[B*nq], stop[B], active[gamma]
  p.ints = take(sizeof(int32_t) * (4 * M + B + TANDEM_MAX_QLEN));  // + stop[B], active[gamma] of the adaptive block length
  // Attention scratch: the larger of the draft and the block call, for ANY cache capacity.  The number of context
  // splits a launch uses depends on the capacity (at most one split per 256 keys; an even count becomes half as many
  // wide workgroups, an odd one does not), and not monotonically - so the table of partials is sized for the
  // largest count any capacity can give: min(ceil(512 / groups), 64) slots per row.
  {
    auto smax = [](int64_t groups) -> int {
      const int64_t w = (512 + groups - 1) / groups;
      return (int)(w < 1 ? 1 : (w > 64 ? 64 : w));
    };
    auto carved = [](size_t rows, int S, int dh) -> size_t {
      return S > 1 ? align256(rows * S * 2 * 4) + rows * S * dh * 4 : 0;
    };
    (void)T_max;
    (void)T_prompt;
    (void)gamma_max;
    int Sd = smax((int64_t)B * S.Hkv);
    if (Sd < 4) Sd = 4;  // the adaptive step cuts the draft attention in at least four (see attn_call)
    size_t a = carved((size_t)B * S.Hq, Sd, S.dh);
    const bool mfma = m->d.dtype == TANDEM_BF16 && L.dh == 128;
    // block calls cover at most TANDEM_MAX_QLEN rows per sequence (longer prompt chunks run in sub-blocks)
    auto blk_ws = [&](int q) -> size_t {
      return carved((size_t)B * q * L.Hq, smax(mfma ? (int64_t)B * L.Hkv : (int64_t)B * L.Hkv * q), L.dh);
    };
    // the matrix-core kernels take up to TANDEM_MAX_PREFILL rows per call (row passes inside one launch)
    const int sub = mfma ? TANDEM_MAX_PREFILL : TANDEM_MAX_QLEN;
    size_t b = blk_ws(gamma < sub ? gamma : sub);
    if (gamma > sub && gamma % sub) b = maxz(b, blk_ws(gamma % sub));
    p.attn_ws_bytes = maxz(a, b);
    if (score) {
      // tandem_mixed_attn: the K_hat segment's splits plus one slot for the own-row segment (matrix-core kernels)
      const bool smf = m->d.dtype == TANDEM_BF16 && S.dh == 128;
      const int Ss = smf ? smax((int64_t)B * S.Hkv) + 1 : smax((int64_t)B * S.Hkv * gamma);
      p.attn_ws_bytes = maxz(p.attn_ws_bytes, carved((size_t)B * gamma * S.Hq, Ss, S.dh));
    }
    if (samples > 0) {
      // shared-prompt calls: the prompt segment (per prompt) and the own segment (per sequence) share one table
      const int P = B / samples;
      const bool smf = m->d.dtype == TANDEM_BF16 && S.dh == 128;
      const int Sb = (mfma ? smax((int64_t)P * L.Hkv) : smax((int64_t)P * L.Hkv * samples * gamma)) +
                     (mfma ? smax((int64_t)B * L.Hkv) : smax((int64_t)B * L.Hkv * gamma));
      const int Sdr = (smf ? smax((int64_t)P * S.Hkv) : smax((int64_t)P * S.Hkv * samples)) + smax((int64_t)B * S.Hkv);
      p.attn_ws_bytes = maxz(p.attn_ws_bytes, carved((size_t)B * gamma * L.Hq, Sb, L.dh));
      p.attn_ws_bytes = maxz(p.attn_ws_bytes, carved((size_t)B * S.Hq, Sdr, S.dh));
    }
    p.attn_ws = take(p.attn_ws_bytes);
  }
  {
    const int dt = m->d.dtype;
    size_t g = 0;
    auto need = [&](size_t rows, int N, int K) { g = maxz(g, gemm_workspace((int)rows, N, K, dt)); };
    auto need_decoder = [&](const tandem_decoder_desc& D, size_t rows) {
      need(rows, (D.Hq + 2 * D.Hkv) * D.dh, D.d);
      need(rows, D.d, D.Hq * D.dh);
      need(rows, D.d_ff, D.d);
      need(rows, D.d, D.d_ff);
      need(rows, D.vocab, D.d);
    };
    need_decoder(S, score ? M : (size_t)B);
    need_decoder(L, M);
    need(M, 2 * S.Hkv * S.dh, S.d);
    // deferred epilogues: every product of the step must be able to leave partials
    p.fused = dt == TANDEM_BF16 && L.d % 4 == 0 && S.d % 4 == 0 && L.d <= 16384 && S.d <= 16384;
    auto dneed = [&](size_t rows, int N, int K) {
      if (!gemm_can_defer((int)rows, N, K, dt, K)) p.fused = false;
      else g = maxz(g, gemm_deferred_workspace((int)rows, N, K));
    };
    auto dneed_decoder = [&](const tandem_decoder_desc& D, size_t rows) {
      dneed(rows, (D.Hq + 2 * D.Hkv) * D.dh, D.d);
      dneed(rows, D.d, D.Hq * D.dh);
      dneed(rows, D.d, D.d_ff);
    };
    dneed_decoder(S, score ? M : (size_t)B);
    dneed_decoder(L, M);
    dneed(M, 2 * S.Hkv * S.dh, S.d);
    for (int j = 0; j < S.n_layers; ++j) {
      const tandem_ff_desc& f = m->ff[j];
      if (f.d_hidden > 0) dneed(M, f.d_S, f.d_hidden);
      else dneed(M, f.d_S, f.d_L);
    }
    size_t pj = 0;
    for (int j = 0; j < S.n_layers; ++j) pj = maxz(pj, project_ws(&m->ff[j], (int64_t)M));
    p.gemm_ws_bytes = maxz(align256(g), pj);
    p.gemm_ws = take(p.gemm_ws_bytes);
  }
  p.total = off;
  return p;
}

struct Ctx {
  const tandem_model* m;
  const tandem_state_desc* st;
  StepPlan plan;
  char* ws;
  hipStream_t stream;
  int dtype;
  float eps;
  const tandem_prompt_desc* pr = nullptr;  // several samples per prompt: the prompts' caches
  const int32_t* gate = nullptr;  // device flag of the current draft run (adaptive block length): 0 = every sequence
                                  // has stopped drafting, the run's kernels return at once
  template <typename T = void> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
  const void* pk(const void* W) const { return m->pk(W); }
};

#define TRY(expr)                     \
  do {                                \
    const int rc_ = (expr);           \
    if (rc_ != TANDEM_OK) return rc_; \
  } while (0)

// row0 / q_rows: the call covers rows row0 .. row0 + q_len - 1 of the q_rows rows that q and out hold per sequence
// (block mode: those rows sit at positions nA[b] + row0 ..)
// prefix_gamma > 0 (instead of causal): row r at position i = nA[b] + n_extra + row0 + r sees only the rows of the blocks
// completed before its own, keys [0, floor(i / prefix_gamma) * prefix_gamma) (Deep Tandem, Eq. (3)).
int attn_call(const Ctx& c, const tandem_decoder_desc& D, const void* q, const void* kA, const void* vA, const int32_t* nA,
              const void* kB, const void* vB, const int32_t* nB, int causal, int q_len, void* out, int row0 = 0,
              int q_rows = 0, const void* kP = nullptr, const void* vP = nullptr, const int32_t* skip = nullptr,
              int prefix_gamma = 0, int n_extra = 0) {
  if (c.pr) {
    // several samples per prompt: kP / vP hold the prompts' rows of this layer, kA / vA each sample's later rows
    tandem_attn_desc d{c.st->B / c.pr->samples, D.Hq, D.Hkv, D.dh, c.pr->T_prompt, causal ? 0 : c.st->gamma_max,
                       1.0f / sqrtf((float)D.dh), c.dtype};
    void* aws = c.at<>(c.plan.attn_ws);
    if (causal)
      return tandem_block_attn_shared(&d, c.pr->samples, c.st->T_max, q, kP, vP, c.pr->n_prompt, kA, vA, nA, q_len, out, aws,
                                      c.plan.attn_ws_bytes, c.stream);
    return tandem_draft_attn_shared(&d, c.pr->samples, c.st->T_max, q, kP, vP, c.pr->n_prompt, kA, vA, nA, kB, vB, nB, out,
                                    aws, c.plan.attn_ws_bytes, c.stream);
  }
  AttnArgs a{};
  const size_t row0_bytes = (size_t)row0 * D.Hq * D.dh * elsize(c.dtype);
  q = (const char*)q + row0_bytes;
  out = (char*)out + row0_bytes;
  a.q_rows = q_rows;
  a.n_off = row0 + n_extra;
  a.skip = skip;
  a.q = q;
  a.kA = kA;
  a.vA = vA;
  a.kB = kB;
  a.vB = vB;
  a.nA = nA;
  a.nB = nB;
  a.causal = causal;
  a.B = c.st->B;
  a.Hq = D.Hq;
  a.Hkv = D.Hkv;
  a.dh = D.dh;
  a.q_len = q_len;
  a.T_max = c.st->T_max;
  a.gamma_max = causal ? 0 : c.st->gamma_max;
  a.scale = 1.0f / sqrtf((float)D.dh);
  a.dtype = c.dtype;
  a.out = out;
  const bool mfma = (causal || prefix_gamma > 0) && attn_block_supported(a);
  if (prefix_gamma > 0) {
    a.mixed = mfma ? 1 : 3;
    a.gamma = prefix_gamma;
  }
  a.S = mfma ? attn_block_splits(a.B, a.Hkv, q_len, a.Hq / a.Hkv, a.T_max, &a.wide)
             : attn_rows_splits(a.B, a.Hkv, q_len, a.Hq / a.Hkv, a.T_max, causal ? 0 : c.st->gamma_max, &a.wide);
  if (skip && !mfma && a.S * (a.wide ? 2 : 1) < 4) {
    // Sequences may drop out of this call (adaptive block length): with one workgroup per sequence and KV head the
    // remaining ones would stream no faster (a single compute unit pulls about 25 GB/s), so the context is cut in
    // four and the time follows the number of sequences still drafting.
    a.S = 4;
    a.wide = 0;
  }
  if (a.S > 1) {
    const size_t rows = (size_t)a.B * q_len * a.Hq;
    a.part_ml = c.at<float>(c.plan.attn_ws);
    a.part_o = reinterpret_cast<float*>(c.ws + c.plan.attn_ws + align256(rows * a.S * 2 * sizeof(float)));
  }
  return mfma ? launch_attn_block(a, c.stream) : launch_attn_rows(a, c.stream);
}

// One pre-norm decoder layer on `rows` rows of the residual stream c.x (in place).
// attn: callable doing scatter + attention, reading c.qkv and writing c.att.
template <typename AttnFn>
int decoder_layer(const Ctx& c, const tandem_decoder_desc& D, const tandem_layer_weights& w, int rows, AttnFn attn) {
  void *x = c.at<>(c.plan.x), *xn = c.at<>(c.plan.xn), *qkv = c.at<>(c.plan.qkv), *att = c.at<>(c.plan.att),
       *h = c.at<>(c.plan.h), *gws = c.at<>(c.plan.gemm_ws);
  const int nqkv = (D.Hq + 2 * D.Hkv) * D.dh, nq = D.Hq * D.dh;
  TRY(launch_rmsnorm(x, w.g_attn, xn, rows, D.d, c.eps, c.dtype, c.stream));
  TRY(gemm(xn, D.d, w.Wqkv, c.pk(w.Wqkv), nullptr, nullptr, 0, qkv, nqkv, rows, nqkv, D.d, TANDEM_ACT_NONE, c.dtype, gws,
           c.plan.gemm_ws_bytes, c.stream));
  TRY(attn());
  TRY(gemm(att, nq, w.Wo, c.pk(w.Wo), nullptr, x, D.d, x, D.d, rows, D.d, nq, TANDEM_ACT_NONE, c.dtype, gws, c.plan.gemm_ws_bytes,
           c.stream));
  TRY(launch_rmsnorm(x, w.g_mlp, xn, rows, D.d, c.eps, c.dtype, c.stream));
  TRY(gemm(xn, D.d, w.W1, c.pk(w.W1), w.b1, nullptr, 0, h, D.d_ff, rows, D.d_ff, D.d, TANDEM_ACT_GELU, c.dtype, gws,
           c.plan.gemm_ws_bytes, c.stream));
  TRY(gemm(h, D.d_ff, w.W2, c.pk(w.W2), w.b2, x, D.d, x, D.d, rows, D.d, D.d_ff, TANDEM_ACT_NONE, c.dtype, gws, c.plan.gemm_ws_bytes,
           c.stream));
  return TANDEM_OK;
}

// Fused form of one decoder layer (bf16): the QKV, O and second MLP products leave fp32 partials that row
// kernels finish together with what follows them (cache scatter; residual + next RMSNorm), so a layer is
// 10 launches instead of 13.  On entry c.xn holds RMSNorm(x; w.g_attn); on exit RMSNorm(x'; g_next).
// x_keep (optional): receives a second copy of x' (the residual stream after this layer).
template <typename ScatterFn, typename AttnFn>
int decoder_layer_fused(const Ctx& c, const tandem_decoder_desc& D, const tandem_layer_weights& w, int rows,
                        const void* g_next, ScatterFn finish_qkv, AttnFn attn, void* x_keep = nullptr) {
  void *x = c.at<>(c.plan.x), *xn = c.at<>(c.plan.xn), *att = c.at<>(c.plan.att), *h = c.at<>(c.plan.h);
  float* gws = c.at<float>(c.plan.gemm_ws);
  const size_t gwb = c.plan.gemm_ws_bytes;
  const int nqkv = (D.Hq + 2 * D.Hkv) * D.dh, nq = D.Hq * D.dh;
  TRY(gemm_deferred(xn, D.d, w.Wqkv, c.pk(w.Wqkv), rows, nqkv, D.d, c.dtype, gws, gwb, c.stream, c.gate));
  TRY(finish_qkv(gws, gemm_splits(rows, nqkv, D.d, c.pk(w.Wqkv) != nullptr)));
  TRY(attn());
  TRY(gemm_deferred(att, nq, w.Wo, c.pk(w.Wo), rows, D.d, nq, c.dtype, gws, gwb, c.stream, c.gate));
  TRY(launch_finish_norm(gws, gemm_splits(rows, D.d, nq, c.pk(w.Wo) != nullptr), nullptr, x, x, w.g_mlp, xn, rows, D.d, c.eps, c.dtype,
                         c.stream, nullptr, c.gate));
  TRY(gemm(xn, D.d, w.W1, c.pk(w.W1), w.b1, nullptr, 0, h, D.d_ff, rows, D.d_ff, D.d, TANDEM_ACT_GELU, c.dtype, gws, gwb, c.stream,
           c.gate));
  TRY(gemm_deferred(h, D.d_ff, w.W2, c.pk(w.W2), rows, D.d, D.d_ff, c.dtype, gws, gwb, c.stream, c.gate));
  TRY(launch_finish_norm(gws, gemm_splits(rows, D.d, D.d_ff, c.pk(w.W2) != nullptr), w.b2, x, x, g_next, xn, rows, D.d, c.eps, c.dtype,
                         c.stream, x_keep, c.gate));
  return TANDEM_OK;
}

// logits and greedy token when c.xn already holds RMSNorm(x; g_final)
int head_normed(const Ctx& c, const tandem_decoder_desc& D, int rows, int32_t* tok_out, int64_t tok_stride) {
  void *xn = c.at<>(c.plan.xn), *lg = c.at<>(c.plan.logits);
  TRY(gemm(xn, D.d, D.W_out, c.pk(D.W_out), nullptr, nullptr, 0, lg, D.vocab, rows, D.vocab, D.d, TANDEM_ACT_NONE, c.dtype,
           c.at<>(c.plan.gemm_ws), c.plan.gemm_ws_bytes, c.stream, c.gate));
  return launch_argmax(lg, rows, D.vocab, tok_out, tok_stride, c.dtype, c.stream, c.gate);
}

int head(const Ctx& c, const tandem_decoder_desc& D, int rows, int32_t* tok_out, int64_t tok_stride) {
  void *x = c.at<>(c.plan.x), *xn = c.at<>(c.plan.xn), *lg = c.at<>(c.plan.logits);
  TRY(launch_rmsnorm(x, D.g_final, xn, rows, D.d, c.eps, c.dtype, c.stream));
  TRY(gemm(xn, D.d, D.W_out, c.pk(D.W_out), nullptr, nullptr, 0, lg, D.vocab, rows, D.vocab, D.d, TANDEM_ACT_NONE, c.dtype,
           c.at<>(c.plan.gemm_ws), c.plan.gemm_ws_bytes, c.stream));
  return launch_argmax(lg, rows, D.vocab, tok_out, tok_stride, c.dtype, c.stream);
}

int copy2d(void* dst, size_t dpitch, const void* src, size_t spitch, size_t width, size_t height, hipStream_t st) {
  return hip_ok(hipMemcpy2DAsync(dst, dpitch, src, spitch, width, height, hipMemcpyDeviceToDevice, st));
}

// M_L in block mode on the block's tokens [B, nq] at positions n .. n+nq-1 (Eq. (1) on the new rows: appends its K/V
// rows, tandem_block_attn per layer), then, per small layer, FF_Tandem on x^(ell[j]) of those rows and that
// layer's RMSNorm and W_K / W_V, which append the K_hat / V_hat rows (Eq. (2) line 1).  verify (optional):
// M_L's greedy token after every row.  Reads state->n, does not change it.
// Tokens of the rows: tokens[B, nq], or - tokens == nullptr - pending[b] followed by the first nq - 1 of follow[b, :gamma].
int large_block_pass(const Ctx& c, const int32_t* tokens, const int32_t* follow, int gamma, int nq,
                     const tandem_step_aux* aux, int32_t* verify) {
  const tandem_model* m = c.m;
  const tandem_state_desc* state = c.st;
  const tandem_decoder_desc &L = m->d.L, &S = m->d.S;
  const int B = state->B, M = B * nq;
  const size_t es = elsize(c.dtype);
  void *x = c.at<>(c.plan.x), *qkv = c.at<>(c.plan.qkv), *q = c.at<>(c.plan.q), *att = c.at<>(c.plan.att);
  TRY(launch_embed_norm(L.emb, tokens, 1, tokens ? nullptr : state->pending, follow, gamma, nq, 0, x,
                        c.plan.fused ? L.layers[0].g_attn : nullptr, c.at<>(c.plan.xn), M, L.d, L.vocab, c.eps, nullptr,
                        nullptr, 0, 0, c.dtype, c.stream));
  // x^(depth) for every small layer that reads it; the first skip_first of them already have their copy
  auto keep = [&](int depth, int skip_first) -> int {
    int seen = 0;
    for (int j = 0; j < S.n_layers; ++j)
      if (m->ell[j] == depth && seen++ >= skip_first)
        TRY(hip_ok(hipMemcpyAsync(c.ws + c.plan.keep + j * c.plan.keep_stride, x, (size_t)M * L.d * es,
                                  hipMemcpyDeviceToDevice, c.stream)));
    return TANDEM_OK;
  };
  TRY(keep(0, 0));
  for (int j = 0; j < L.n_layers; ++j) {
    auto attn_only = [&]() -> int {
      // long prompt chunks: the matrix-core kernels take up to TANDEM_MAX_PREFILL rows per sequence in one launch (row
      // passes inside it), the generic ones TANDEM_MAX_QLEN per launch; all K/V rows are already in the cache
      const int sub = c.dtype == TANDEM_BF16 && L.dh == 128 && !c.pr ? TANDEM_MAX_PREFILL : TANDEM_MAX_QLEN;
      for (int r0 = 0; r0 < nq; r0 += sub) {
        const int rows = nq - r0 < sub ? nq - r0 : sub;
        TRY(attn_call(c, L, q, state->KL[j], state->VL[j], state->n, nullptr, nullptr, nullptr, 1, rows, att, r0, nq,
                      c.pr ? c.pr->KLp[j] : nullptr, c.pr ? c.pr->VLp[j] : nullptr));
      }
      return TANDEM_OK;
    };
    if (c.plan.fused) {
      auto finish_qkv = [&](const float* part, int splits) -> int {
        return launch_finish_scatter(part, splits, q, state->KL[j], state->VL[j], state->n, 0, M, nq, L.Hq, L.Hkv,
                                     L.dh, state->T_max, L.Hq * L.dh, (L.Hq + 2 * L.Hkv) * L.dh, c.dtype, c.stream);
      };
      const void* g_next = j + 1 < L.n_layers ? L.layers[j + 1].g_attn : L.g_final;
      // the first small layer that reads x^(j+1) gets its copy from the kernel that finishes this layer
      void* x_keep = nullptr;
      for (int t = S.n_layers - 1; t >= 0; --t)
        if (m->ell[t] == j + 1) x_keep = c.ws + c.plan.keep + t * c.plan.keep_stride;
      TRY(decoder_layer_fused(c, L, L.layers[j], M, g_next, finish_qkv, attn_only, x_keep));
      TRY(keep(j + 1, 1));
    } else {
      auto attn = [&]() -> int {
        TRY(launch_scatter_qkv(qkv, q, state->KL[j], state->VL[j], state->n, 0, M, nq, L.Hq, L.Hkv, L.dh,
                               state->T_max, 0, L.Hq * L.dh, (L.Hq + 2 * L.Hkv) * L.dh, c.dtype, c.stream));
        return attn_only();
      };
      TRY(decoder_layer(c, L, L.layers[j], M, attn));
      TRY(keep(j + 1, 0));
    }
  }
  if (aux && aux->x_large)
    TRY(hip_ok(hipMemcpyAsync(aux->x_large, x, (size_t)M * L.d * es, hipMemcpyDeviceToDevice, c.stream)));
  if (verify) {
    TRY(c.plan.fused ? head_normed(c, L, M, verify, 1) : head(c, L, M, verify, 1));
    if (aux && aux->logits_L)
      TRY(hip_ok(hipMemcpyAsync(aux->logits_L, c.at<>(c.plan.logits), (size_t)M * L.vocab * es, hipMemcpyDeviceToDevice,
                                c.stream)));
  }

  // ---- 3. FF_Tandem on the new rows, then the small layer's norm and W_K / W_V ---------
  for (int j = 0; j < S.n_layers; ++j) {
    void *yhat = c.at<>(c.plan.yhat), *xn = c.at<>(c.plan.xn), *kv = c.at<>(c.plan.kv), *gws = c.at<>(c.plan.gemm_ws);
    const void* xk = c.ws + c.plan.keep + j * c.plan.keep_stride;
    const void* Wkv = (const char*)S.layers[j].Wqkv + (size_t)S.Hq * S.dh * S.d * es;
    const void* Wq_p = c.pk(S.layers[j].Wqkv);  // packed tiles hold 32 rows each: the K/V rows start on a tile
    const void* Wkv_p = Wq_p && (S.Hq * S.dh) % 32 == 0 ? (const char*)Wq_p + (size_t)S.Hq * S.dh * S.d * es : nullptr;
    const int nkv = 2 * S.Hkv * S.dh;
    if (c.plan.fused) {
      const tandem_ff_desc& f = m->ff[j];
      float* part = (float*)gws;
      if (f.d_hidden > 0) {
        void* hb = c.at<>(c.plan.h);
        TRY(gemm(xk, f.d_L, f.W1, f.W1p, f.b1, nullptr, 0, hb, f.d_hidden, M, f.d_hidden, f.d_L, f.act, c.dtype, gws,
                 c.plan.gemm_ws_bytes, c.stream));
        TRY(gemm_deferred(hb, f.d_hidden, f.W2, f.W2p, M, f.d_S, f.d_hidden, c.dtype, gws, c.plan.gemm_ws_bytes, c.stream));
        TRY(launch_finish_norm(part, gemm_splits(M, f.d_S, f.d_hidden, f.W2p != nullptr), f.b2, nullptr, yhat, S.layers[j].g_attn, xn, M,
                               S.d, c.eps, c.dtype, c.stream));
      } else {
        TRY(gemm_deferred(xk, f.d_L, f.W1, f.W1p, M, f.d_S, f.d_L, c.dtype, gws, c.plan.gemm_ws_bytes, c.stream));
        TRY(launch_finish_norm(part, gemm_splits(M, f.d_S, f.d_L, f.W1p != nullptr), f.b1, nullptr, yhat, S.layers[j].g_attn, xn, M, S.d,
                               c.eps, c.dtype, c.stream));
      }
      TRY(gemm_deferred(xn, S.d, Wkv, Wkv_p, M, nkv, S.d, c.dtype, gws, c.plan.gemm_ws_bytes, c.stream));
      TRY(launch_finish_scatter(part, gemm_splits(M, nkv, S.d, Wkv_p != nullptr), nullptr, state->Khat[j], state->Vhat[j], state->n, 0, M,
                                nq, S.Hq, S.Hkv, S.dh, state->T_max, 0, nkv, c.dtype, c.stream));
    } else {
      TRY(run_project(&m->ff[j], xk, yhat, M, gws, c.plan.gemm_ws_bytes, c.stream));
      TRY(launch_rmsnorm(yhat, S.layers[j].g_attn, xn, M, S.d, c.eps, c.dtype, c.stream));
      TRY(gemm(xn, S.d, Wkv, Wkv_p, nullptr, nullptr, 0, kv, nkv, M, nkv, S.d, TANDEM_ACT_NONE, c.dtype, gws,
               c.plan.gemm_ws_bytes, c.stream));
      TRY(launch_scatter_qkv(kv, nullptr, state->Khat[j], state->Vhat[j], state->n, 0, M, nq, S.Hq, S.Hkv, S.dh,
                             state->T_max, 0, 0, nkv, c.dtype, c.stream));
    }
  }

  return TANDEM_OK;
}

}  // namespace

extern "C" {

size_t tandem_project_workspace(const tandem_ff_desc* ff, int64_t M) {
  if (check_ff(ff) != TANDEM_OK || M < 1) return 0;
  return project_ws(ff, M);
}

int tandem_project(const tandem_ff_desc* ff, const void* x, void* y_hat, int64_t M, void* ws, size_t ws_bytes,
                   void* hip_stream) {
  int rc = check_ff(ff);
  if (rc != TANDEM_OK) return rc;
  if (!x || !y_hat) return TANDEM_ERR_NULL;
  if (M < 1 || M > (1 << 24)) return TANDEM_ERR_SHAPE;
  const size_t need = project_ws(ff, M);
  if (need > 0 && !ws) return TANDEM_ERR_NULL;
  if (ws_bytes < need) return TANDEM_ERR_WORKSPACE;
  return run_project(ff, x, y_hat, M, ws, ws_bytes, (hipStream_t)hip_stream);
}

int tandem_model_create(const tandem_model_desc* desc, tandem_model** out) {
  if (!desc || !out) return TANDEM_ERR_NULL;
  *out = nullptr;
  if (desc->dtype != TANDEM_F32 && desc->dtype != TANDEM_BF16) return TANDEM_ERR_UNSUPPORTED;
  if (desc->flags != 0) return TANDEM_ERR_UNSUPPORTED;
  int rc = check_decoder(desc->L);
  if (rc != TANDEM_OK) return rc;
  rc = check_decoder(desc->S);
  if (rc != TANDEM_OK) return rc;
  if (!desc->ell || !desc->ff) return TANDEM_ERR_NULL;
  if (!(desc->rms_eps >= 0.f)) return TANDEM_ERR_SHAPE;
  for (int j = 0; j < desc->S.n_layers; ++j) {
    if (desc->ell[j] < 0 || desc->ell[j] > desc->L.n_layers) return TANDEM_ERR_SHAPE;
    rc = check_ff(&desc->ff[j]);
    if (rc != TANDEM_OK) return rc;
    if (desc->ff[j].d_L != desc->L.d || desc->ff[j].d_S != desc->S.d || desc->ff[j].dtype != desc->dtype)
      return TANDEM_ERR_SHAPE;
  }
  tandem_model* m = new (std::nothrow) tandem_model();
  if (!m) return TANDEM_ERR_HIP;
  m->d = *desc;
  m->L_layers.assign(desc->L.layers, desc->L.layers + desc->L.n_layers);
  m->S_layers.assign(desc->S.layers, desc->S.layers + desc->S.n_layers);
  m->ell.assign(desc->ell, desc->ell + desc->S.n_layers);
  m->ff.assign(desc->ff, desc->ff + desc->S.n_layers);
  m->d.L.layers = m->L_layers.data();
  m->d.S.layers = m->S_layers.data();
  m->d.ell = m->ell.data();
  m->d.ff = m->ff.data();
  for (auto& f : m->ff) f.W1p = f.W2p = nullptr;  // packed copies come from tandem_model_pack only
  *out = m;
  return TANDEM_OK;
}

void tandem_model_destroy(tandem_model* m) { delete m; }

size_t tandem_model_packed_bytes(const tandem_model* m) {
  if (!m) return 0;
  size_t total = 0;
  for (const PackItem& it : pack_items(m)) total += align256((size_t)it.N * it.K * elsize(m->d.dtype));
  return total;
}

int tandem_model_pack(tandem_model* m, void* packed, size_t packed_bytes, void* hip_stream) {
  if (!m) return TANDEM_ERR_NULL;
  const std::vector<PackItem> items = pack_items(m);
  if (items.empty()) return TANDEM_OK;
  if (!packed) return TANDEM_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(packed) % 256 != 0) return TANDEM_ERR_SHAPE;
  if (packed_bytes < tandem_model_packed_bytes(m)) return TANDEM_ERR_WORKSPACE;
  size_t off = 0;
  for (const PackItem& it : items) {
    void* dst = (char*)packed + off;
    const int rc = launch_pack_weights(it.W, dst, it.N, it.K, (hipStream_t)hip_stream);
    if (rc != TANDEM_OK) {
      m->packed.clear();
      for (tandem_ff_desc& f : m->ff) f.W1p = f.W2p = nullptr;
      return rc;
    }
    m->packed[it.W] = dst;
    off += align256((size_t)it.N * it.K * elsize(m->d.dtype));
  }
  for (tandem_ff_desc& f : m->ff) {
    f.W1p = m->pk(f.W1);
    f.W2p = f.d_hidden > 0 ? m->pk(f.W2) : nullptr;
  }
  return TANDEM_OK;
}

size_t tandem_packed_weight_bytes(int64_t N, int64_t K, int32_t dtype) {
  if (N < 1 || K < 1 || !gemm_packable(N, K, dtype)) return 0;
  return (size_t)N * K * elsize(dtype);
}

int tandem_pack_weight(const void* W, int64_t N, int64_t K, int32_t dtype, void* Wp, void* hip_stream) {
  if (!W || !Wp) return TANDEM_ERR_NULL;
  if (N < 1 || K < 1) return TANDEM_ERR_SHAPE;
  if (!gemm_packable(N, K, dtype)) return TANDEM_ERR_UNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(W) % 16 != 0 || reinterpret_cast<uintptr_t>(Wp) % 16 != 0) return TANDEM_ERR_SHAPE;
  return launch_pack_weights(W, Wp, N, K, (hipStream_t)hip_stream);
}

size_t tandem_decode_step_workspace(const tandem_model* m, int32_t B, int32_t gamma) {
  if (!m || B < 1 || gamma < 1 || gamma > TANDEM_MAX_QLEN) return 0;
  // T_max only scales the split-K scratch, which is capped at 64 splits: size for the cap.  The larger of the
  // plain mode and the free-token mode (gamma + 1 verified rows): more rows can mean fewer contraction splits
  // and hence less scratch, so neither covers the other.
  size_t total = make_plan(m, B, gamma, (int64_t)1 << 40, gamma).total;
  if (gamma < TANDEM_MAX_QLEN) total = maxz(total, make_plan(m, B, gamma + 1, (int64_t)1 << 40, gamma).total);
  return total;
}

namespace {
int decode_step_impl(const tandem_model* m, const tandem_state_desc* state, const tandem_router_desc* router,
                     const tandem_prompt_desc* pr, int32_t gamma, int32_t flags, const int32_t* forced, int32_t* out_tokens, int32_t* n_accepted,
                     int32_t* n_drafted, float* router_p, const tandem_step_aux* aux, void* ws, size_t ws_bytes,
                     void* hip_stream) {
  if (!m || !state || !out_tokens || !n_accepted || !ws) return TANDEM_ERR_NULL;
  if (!state->KL || !state->VL || !state->Khat || !state->Vhat || !state->Kcur || !state->Vcur || !state->n ||
      !state->pending)
    return TANDEM_ERR_NULL;
  const tandem_decoder_desc &L = m->d.L, &S = m->d.S;
  const int B = state->B;
  if (B < 1 || B > 65535 || state->T_max < 1 || state->gamma_max < 1) return TANDEM_ERR_SHAPE;
  if (flags & ~TANDEM_STEP_FREE_TOKEN) return TANDEM_ERR_UNSUPPORTED;
  // rows M_L verifies per sequence: the block [pending, d_1 .. d_{gamma-1}], plus d_gamma for the free token
  const int nq = gamma + ((flags & TANDEM_STEP_FREE_TOKEN) ? 1 : 0);
  if (gamma < 1 || nq > TANDEM_MAX_QLEN || gamma > state->gamma_max || nq > state->T_max) return TANDEM_ERR_SHAPE;
  for (int j = 0; j < L.n_layers; ++j)
    if (!state->KL[j] || !state->VL[j]) return TANDEM_ERR_NULL;
  for (int j = 0; j < S.n_layers; ++j)
    if (!state->Khat[j] || !state->Vhat[j] || !state->Kcur[j] || !state->Vcur[j]) return TANDEM_ERR_NULL;
  if (pr) {
    if (!pr->KLp || !pr->VLp || !pr->Khp || !pr->Vhp || !pr->n_prompt) return TANDEM_ERR_NULL;
    if (pr->samples < 1 || B % pr->samples != 0 || pr->T_prompt < 1) return TANDEM_ERR_SHAPE;
    for (int j = 0; j < L.n_layers; ++j)
      if (!pr->KLp[j] || !pr->VLp[j]) return TANDEM_ERR_NULL;
    for (int j = 0; j < S.n_layers; ++j)
      if (!pr->Khp[j] || !pr->Vhp[j]) return TANDEM_ERR_NULL;
  } else if (ws_bytes < tandem_decode_step_workspace(m, B, gamma)) {
    return TANDEM_ERR_WORKSPACE;
  }

  Ctx c;
  c.m = m;
  c.st = state;
  c.pr = pr;
  c.plan = make_plan(m, B, nq, state->T_max, state->gamma_max, false, pr ? pr->samples : 0, pr ? pr->T_prompt : 0);
  if (c.plan.total > ws_bytes) return TANDEM_ERR_WORKSPACE;
  c.ws = (char*)ws;
  c.stream = (hipStream_t)hip_stream;
  c.dtype = m->d.dtype;
  c.eps = m->d.rms_eps;
  const size_t es = elsize(c.dtype);
  const int M = B * nq;  // rows of the verify pass and of everything derived from it

  int32_t* ncur = c.at<int32_t>(c.plan.ints);        // [gamma][B], ncur[r][b] = r + 1
  int32_t* draft = aux && aux->draft ? aux->draft : ncur + 2 * (size_t)M;    // [B, gamma]
  int32_t* verify = aux && aux->verify ? aux->verify : ncur + 3 * (size_t)M;  // [B, nq]
  int32_t* stop = router ? ncur + 4 * (size_t)M : nullptr;                    // [B], see accept_kernel
  // [gamma]: sequences still drafting after run r; run r + 1 is gated on it (bf16 path: when every sequence has
  // stopped, the kernels of the remaining runs return at once)
  int32_t* active = router && c.plan.fused ? stop + B : nullptr;
  void *x = c.at<>(c.plan.x), *qkv = c.at<>(c.plan.qkv), *q = c.at<>(c.plan.q), *att = c.at<>(c.plan.att);


  // ---- 1. draft: gamma autoregressive runs of M_S --------------------------------------
  for (int r = 0; r < gamma; ++r) {
    // input of run r: the pending token, then the draft (or forced) token of the run before; the first run's kernel
    // also sets up ncur (own-block rows visible to each run) and clears the router's stop marks
    c.gate = active && r > 0 ? active + r - 1 : nullptr;
    TRY(launch_embed_norm(S.emb, nullptr, 1, state->pending, forced ? forced : draft, gamma, 1, r, x,
                          c.plan.fused ? S.layers[0].g_attn : nullptr, c.at<>(c.plan.xn), B, S.d, S.vocab, c.eps, ncur, stop,
                          r == 0 ? B : 0, gamma, c.dtype, c.stream, r == 0 ? active : nullptr, c.gate));
    for (int j = 0; j < S.n_layers; ++j) {
      auto attn_only = [&]() -> int {
        return attn_call(c, S, q, state->Khat[j], state->Vhat[j], state->n, state->Kcur[j], state->Vcur[j],
                         ncur + (size_t)r * B, 0, 1, att, 0, 0, c.pr ? c.pr->Khp[j] : nullptr, c.pr ? c.pr->Vhp[j] : nullptr,
                         stop);  // a sequence the router has stopped costs no attention traffic in the later runs
      };
      if (c.plan.fused) {
        auto finish_qkv = [&](const float* part, int splits) -> int {
          return launch_finish_scatter(part, splits, q, state->Kcur[j], state->Vcur[j], nullptr, r, B, 1, S.Hq, S.Hkv,
                                       S.dh, state->gamma_max, S.Hq * S.dh, (S.Hq + 2 * S.Hkv) * S.dh, c.dtype, c.stream,
                                       c.gate);
        };
        const void* g_next = j + 1 < S.n_layers ? S.layers[j + 1].g_attn : S.g_final;
        TRY(decoder_layer_fused(c, S, S.layers[j], B, g_next, finish_qkv, attn_only));
      } else {
        auto attn = [&]() -> int {
          TRY(launch_scatter_qkv(qkv, q, state->Kcur[j], state->Vcur[j], nullptr, r, B, 1, S.Hq, S.Hkv, S.dh,
                                 state->gamma_max, 0, S.Hq * S.dh, (S.Hq + 2 * S.Hkv) * S.dh, c.dtype, c.stream));
          return attn_only();
        };
        TRY(decoder_layer(c, S, S.layers[j], B, attn));
      }
    }
    if (aux && aux->y_small)
      TRY(copy2d((char*)aux->y_small + (size_t)r * S.d * es, (size_t)gamma * S.d * es, x, S.d * es, S.d * es, B, c.stream));
    TRY(c.plan.fused ? head_normed(c, S, B, draft + r, gamma) : head(c, S, B, draft + r, gamma));
    if (aux && aux->logits_S)
      TRY(copy2d((char*)aux->logits_S + (size_t)r * S.vocab * es, (size_t)gamma * S.vocab * es, c.at<>(c.plan.logits),
                 S.vocab * es, S.vocab * es, B, c.stream));
    // adaptive block length (Sec. 3.1): the router sees this run's distribution; a sequence it stops keeps its
    // place in the batch (the later runs skip its attention and compute rows that nobody reads) and is verified on
    // its shorter block
    if (router)
      TRY(launch_router(router, c.at<>(c.plan.logits), S.emb, B, S.vocab, S.d, r, stop, router_p ? router_p + r : nullptr,
                        gamma, c.stream, active, c.gate));
  }
  c.gate = nullptr;

  // ---- 2. verify: M_L in block mode on the first nq of [pending, d_1 .. d_gamma]; 3. new K_hat / V_hat rows
  TRY(large_block_pass(c, nullptr, forced ? forced : draft, gamma, nq, aux, verify));

  // ---- 4. accept ------------------------------------------------------------------------
  return launch_accept(draft, verify, forced, stop, out_tokens, n_accepted, n_drafted, state->n, state->pending, B, gamma,
                       nq, state->T_max, c.stream);
}
}  // namespace

int tandem_decode_step(const tandem_model* m, const tandem_state_desc* state, int32_t gamma, int32_t flags,
                       const int32_t* forced, int32_t* out_tokens, int32_t* n_accepted, const tandem_step_aux* aux,
                       void* ws, size_t ws_bytes, void* hip_stream) {
  return decode_step_impl(m, state, nullptr, nullptr, gamma, flags, forced, out_tokens, n_accepted, nullptr, nullptr, aux, ws,
                          ws_bytes, hip_stream);
}

size_t tandem_decode_step_shared_workspace(const tandem_model* m, int32_t B, int32_t samples, int32_t gamma) {
  if (!m || B < 1 || samples < 1 || B % samples != 0 || gamma < 1 || gamma > TANDEM_MAX_QLEN) return 0;
  const int64_t big = (int64_t)1 << 40;
  size_t total = make_plan(m, B, gamma, big, gamma, false, samples, big).total;
  if (gamma < TANDEM_MAX_QLEN) total = maxz(total, make_plan(m, B, gamma + 1, big, gamma, false, samples, big).total);
  return total;
}

int tandem_decode_step_shared(const tandem_model* m, const tandem_state_desc* state, const tandem_prompt_desc* prompt,
                              int32_t gamma, int32_t flags, int32_t* out_tokens, int32_t* n_accepted,
                              const tandem_step_aux* aux, void* ws, size_t ws_bytes, void* hip_stream) {
  if (!prompt) return TANDEM_ERR_NULL;
  return decode_step_impl(m, state, nullptr, prompt, gamma, flags, nullptr, out_tokens, n_accepted, nullptr, nullptr, aux, ws,
                          ws_bytes, hip_stream);
}

int tandem_decode_step_adaptive(const tandem_model* m, const tandem_state_desc* state, const tandem_router_desc* router,
                                int32_t gamma_max, int32_t flags, int32_t* out_tokens, int32_t* n_accepted,
                                int32_t* n_drafted, float* router_p, const tandem_step_aux* aux, void* ws,
                                size_t ws_bytes, void* hip_stream) {
  if (!m || !router) return TANDEM_ERR_NULL;
  int rc = check_router(router, m->d.S.d);
  if (rc != TANDEM_OK) return rc;
  if (router->dtype != m->d.dtype || m->d.S.vocab < router->k) return TANDEM_ERR_UNSUPPORTED;
  return decode_step_impl(m, state, router, nullptr, gamma_max, flags, nullptr, out_tokens, n_accepted, n_drafted, router_p, aux,
                          ws, ws_bytes, hip_stream);
}

size_t tandem_prefill_workspace(const tandem_model* m, int32_t B, int32_t q_len) {
  if (!m || B < 1 || q_len < 1 || q_len > TANDEM_MAX_PREFILL) return 0;
  return make_plan(m, B, q_len, (int64_t)1 << 40, 1).total;
}

int tandem_prefill(const tandem_model* m, const tandem_state_desc* state, const int32_t* tokens, int32_t q_len,
                   int32_t flags, void* x_large, void* ws, size_t ws_bytes, void* hip_stream) {
  if (!m || !state || !tokens || !ws) return TANDEM_ERR_NULL;
  if (!state->KL || !state->VL || !state->Khat || !state->Vhat || !state->n || !state->pending) return TANDEM_ERR_NULL;
  if (flags & ~TANDEM_PREFILL_EMIT) return TANDEM_ERR_UNSUPPORTED;
  const tandem_decoder_desc &L = m->d.L, &S = m->d.S;
  const int B = state->B;
  if (B < 1 || B > 65535 || state->T_max < 1) return TANDEM_ERR_SHAPE;
  if (q_len < 1 || q_len > TANDEM_MAX_PREFILL || q_len > state->T_max) return TANDEM_ERR_SHAPE;
  for (int j = 0; j < L.n_layers; ++j)
    if (!state->KL[j] || !state->VL[j]) return TANDEM_ERR_NULL;
  for (int j = 0; j < S.n_layers; ++j)
    if (!state->Khat[j] || !state->Vhat[j]) return TANDEM_ERR_NULL;
  Ctx c;
  c.m = m;
  c.st = state;
  c.plan = make_plan(m, B, q_len, state->T_max, state->gamma_max > 0 ? state->gamma_max : 1);
  if (c.plan.total > ws_bytes) return TANDEM_ERR_WORKSPACE;
  c.ws = (char*)ws;
  c.stream = (hipStream_t)hip_stream;
  c.dtype = m->d.dtype;
  c.eps = m->d.rms_eps;
  const size_t es = elsize(c.dtype);
  tandem_step_aux aux{};
  aux.x_large = x_large;
  TRY(large_block_pass(c, tokens, nullptr, 0, q_len, x_large ? &aux : nullptr, nullptr));
  if (flags & TANDEM_PREFILL_EMIT) {
    // M_L's greedy token after the last row of every sequence: gather those rows of the residual stream to
    // the front of x (through a buffer that step 3 no longer needs) and run the head on B rows
    void* x = c.at<>(c.plan.x);
    if (q_len > 1) {
      void* tmp = c.ws + c.plan.keep;
      TRY(copy2d(tmp, (size_t)L.d * es, (const char*)x + (size_t)(q_len - 1) * L.d * es, (size_t)q_len * L.d * es,
                 (size_t)L.d * es, B, c.stream));
      TRY(hip_ok(hipMemcpyAsync(x, tmp, (size_t)B * L.d * es, hipMemcpyDeviceToDevice, c.stream)));
    }
    TRY(head(c, L, B, state->pending, 1));
  }
  return launch_advance(state->n, B, q_len, state->T_max, c.stream);
}

size_t tandem_score_workspace(const tandem_model* m, int32_t B, int32_t q_len) {
  if (!m || B < 1 || q_len < 1 || q_len > TANDEM_MAX_QLEN) return 0;
  return make_plan(m, B, q_len, (int64_t)1 << 40, 1, true).total;
}

int tandem_score(const tandem_model* m, const tandem_state_desc* state, void* const* k_own, void* const* v_own,
                 const int32_t* pos, const int32_t* tokens, int32_t q_len, int32_t gamma, int32_t* greedy, void* logits,
                 void* y_small, void* ws, size_t ws_bytes, void* hip_stream) {
  if (!m || !state || !k_own || !v_own || !pos || !tokens || !ws) return TANDEM_ERR_NULL;
  if (!state->Khat || !state->Vhat) return TANDEM_ERR_NULL;
  const tandem_decoder_desc& S = m->d.S;
  const int B = state->B;
  if (B < 1 || B > 65535 || state->T_max < 1) return TANDEM_ERR_SHAPE;
  if (q_len < 1 || q_len > TANDEM_MAX_QLEN || q_len > state->T_max || gamma < 1) return TANDEM_ERR_SHAPE;
  for (int j = 0; j < S.n_layers; ++j)
    if (!state->Khat[j] || !state->Vhat[j] || !k_own[j] || !v_own[j]) return TANDEM_ERR_NULL;
  Ctx c;
  c.m = m;
  c.st = state;
  c.plan = make_plan(m, B, q_len, state->T_max, state->gamma_max > 0 ? state->gamma_max : 1, true);
  if (c.plan.total > ws_bytes) return TANDEM_ERR_WORKSPACE;
  c.ws = (char*)ws;
  c.stream = (hipStream_t)hip_stream;
  c.dtype = m->d.dtype;
  c.eps = m->d.rms_eps;
  const size_t es = elsize(c.dtype);
  const int M = B * q_len;
  void *x = c.at<>(c.plan.x), *qkv = c.at<>(c.plan.qkv), *q = c.at<>(c.plan.q), *att = c.at<>(c.plan.att);
  int32_t* tok_scratch = c.at<int32_t>(c.plan.ints);  // greedy tokens when the caller does not want them
  tandem_attn_desc ad{B, S.Hq, S.Hkv, S.dh, state->T_max, 0, 1.0f / sqrtf((float)S.dh), c.dtype};

  TRY(launch_embed_norm(S.emb, tokens, 1, nullptr, nullptr, 0, 1, 0, x, c.plan.fused ? S.layers[0].g_attn : nullptr,
                        c.at<>(c.plan.xn), M, S.d, S.vocab, c.eps, nullptr, nullptr, 0, 0, c.dtype, c.stream));
  for (int j = 0; j < S.n_layers; ++j) {
    auto attn_only = [&]() -> int {
      return tandem_mixed_attn(&ad, q, state->Khat[j], state->Vhat[j], k_own[j], v_own[j], pos, q_len, gamma, att,
                               c.at<>(c.plan.attn_ws), c.plan.attn_ws_bytes, c.stream);
    };
    if (c.plan.fused) {
      auto finish_qkv = [&](const float* part, int splits) -> int {
        return launch_finish_scatter(part, splits, q, k_own[j], v_own[j], pos, 0, M, q_len, S.Hq, S.Hkv, S.dh,
                                     state->T_max, S.Hq * S.dh, (S.Hq + 2 * S.Hkv) * S.dh, c.dtype, c.stream);
      };
      const void* g_next = j + 1 < S.n_layers ? S.layers[j + 1].g_attn : S.g_final;
      TRY(decoder_layer_fused(c, S, S.layers[j], M, g_next, finish_qkv, attn_only));
    } else {
      auto attn = [&]() -> int {
        TRY(launch_scatter_qkv(qkv, q, k_own[j], v_own[j], pos, 0, M, q_len, S.Hq, S.Hkv, S.dh, state->T_max, 0,
                               S.Hq * S.dh, (S.Hq + 2 * S.Hkv) * S.dh, c.dtype, c.stream));
        return attn_only();
      };
      TRY(decoder_layer(c, S, S.layers[j], M, attn));
    }
  }
  if (y_small) TRY(hip_ok(hipMemcpyAsync(y_small, x, (size_t)M * S.d * es, hipMemcpyDeviceToDevice, c.stream)));
  int32_t* tok = greedy ? greedy : tok_scratch;
  TRY(c.plan.fused ? head_normed(c, S, M, tok, 1) : head(c, S, M, tok, 1));
  if (logits)
    TRY(hip_ok(hipMemcpyAsync(logits, c.at<>(c.plan.logits), (size_t)M * S.vocab * es, hipMemcpyDeviceToDevice, c.stream)));
  return TANDEM_OK;
}

// ---------------------------------------------------------------- Deep Tandem (Sec. 5)
namespace {

struct DeepCtx {
  Ctx c;
  tandem_state_desc st;  // B and T_max for attn_call; the cache arrays are passed explicitly
};

int deep_setup(DeepCtx& dc, const tandem_model* m, const tandem_ff_desc* ff, const tandem_deep_state_desc* st, int q_len,
               void* ws, size_t ws_bytes, void* hip_stream, size_t* ff_ws_off, size_t* ff_ws_bytes) {
  if (!m || !ff || !st || !ws) return TANDEM_ERR_NULL;
  if (!st->KL || !st->VL || !st->KS || !st->VS) return TANDEM_ERR_NULL;
  const tandem_decoder_desc &L = m->d.L, &S = m->d.S;
  int rc = check_ff(ff);
  if (rc != TANDEM_OK) return rc;
  if (ff->d_L != L.d || ff->d_S != S.d || ff->dtype != m->d.dtype) return TANDEM_ERR_SHAPE;
  if (st->B < 1 || st->B > 65535 || st->T_max < 1) return TANDEM_ERR_SHAPE;
  if (q_len < 1 || q_len > TANDEM_MAX_QLEN || q_len >= st->T_max) return TANDEM_ERR_SHAPE;
  for (int j = 0; j < L.n_layers; ++j)
    if (!st->KL[j] || !st->VL[j]) return TANDEM_ERR_NULL;
  for (int j = 0; j < S.n_layers; ++j)
    if (!st->KS[j] || !st->VS[j]) return TANDEM_ERR_NULL;
  dc.st = tandem_state_desc{};
  dc.st.B = st->B;
  dc.st.T_max = st->T_max;
  dc.st.gamma_max = 1;
  Ctx& c = dc.c;
  c.m = m;
  c.st = &dc.st;
  c.plan = make_plan(m, st->B, q_len, st->T_max, 1, true);
  *ff_ws_off = c.plan.total;
  *ff_ws_bytes = align256(project_ws(ff, (int64_t)st->B * q_len));
  if (c.plan.total + *ff_ws_bytes > ws_bytes) return TANDEM_ERR_WORKSPACE;
  c.ws = (char*)ws;
  c.stream = (hipStream_t)hip_stream;
  c.dtype = m->d.dtype;
  c.eps = m->d.rms_eps;
  return TANDEM_OK;
}

// M_L's rows r = (pos ? pos[b] : 0) + fixed + rr, rr < q_len, of Eq. (3): input = embedding of token r - gamma (zero
// without one), every layer's K/V rows appended at row r, attention over the rows of the blocks completed before the
// row's own.  Leaves x^(L_L) of the rows in the plan's x buffer.
int deep_large_rows(const Ctx& c, const tandem_deep_state_desc* st, const int32_t* tokens, int64_t n_tokens,
                    const int32_t* pos, int fixed, int q_len, int gamma) {
  const tandem_decoder_desc& L = c.m->d.L;
  const int M = st->B * q_len;
  void *x = c.at<>(c.plan.x), *qkv = c.at<>(c.plan.qkv), *q = c.at<>(c.plan.q), *att = c.at<>(c.plan.att);
  TRY(launch_embed_shifted(L.emb, tokens, n_tokens, pos, fixed, gamma, q_len, x, c.plan.fused ? L.layers[0].g_attn : nullptr,
                           c.at<>(c.plan.xn), M, L.d, L.vocab, c.eps, c.dtype, c.stream));
  for (int j = 0; j < L.n_layers; ++j) {
    auto attn_only = [&]() -> int {
      return attn_call(c, L, q, st->KL[j], st->VL[j], pos, nullptr, nullptr, nullptr, 0, q_len, att, 0, 0, nullptr, nullptr,
                       nullptr, gamma, fixed);
    };
    if (c.plan.fused) {
      auto finish_qkv = [&](const float* part, int splits) -> int {
        return launch_finish_scatter(part, splits, q, st->KL[j], st->VL[j], pos, fixed, M, q_len, L.Hq, L.Hkv, L.dh,
                                     st->T_max, L.Hq * L.dh, (L.Hq + 2 * L.Hkv) * L.dh, c.dtype, c.stream);
      };
      const void* g_next = j + 1 < L.n_layers ? L.layers[j + 1].g_attn : L.g_final;
      TRY(decoder_layer_fused(c, L, L.layers[j], M, g_next, finish_qkv, attn_only));
    } else {
      auto attn = [&]() -> int {
        TRY(launch_scatter_qkv(qkv, q, st->KL[j], st->VL[j], pos, fixed, M, q_len, L.Hq, L.Hkv, L.dh, st->T_max, 0,
                               L.Hq * L.dh, (L.Hq + 2 * L.Hkv) * L.dh, c.dtype, c.stream));
        return attn_only();
      };
      TRY(decoder_layer(c, L, L.layers[j], M, attn));
    }
  }
  return TANDEM_OK;
}

}  // namespace

size_t tandem_deep_score_workspace(const tandem_model* m, const tandem_ff_desc* ff_deep, int32_t B, int32_t q_len) {
  if (!m || !ff_deep || check_ff(ff_deep) != TANDEM_OK || B < 1 || q_len < 1 || q_len > TANDEM_MAX_QLEN) return 0;
  return make_plan(m, B, q_len, (int64_t)1 << 40, 1, true).total + align256(project_ws(ff_deep, (int64_t)B * q_len));
}

int tandem_deep_begin(const tandem_model* m, const tandem_ff_desc* ff_deep, const tandem_deep_state_desc* st, void* ws,
                      size_t ws_bytes, void* hip_stream) {
  DeepCtx dc;
  size_t fo = 0, fb = 0;
  TRY(deep_setup(dc, m, ff_deep, st, 1, ws, ws_bytes, hip_stream, &fo, &fb));
  // row 0 of M_L: no input token, no visible key (any block length gives that; 1 is passed)
  int32_t* zero = dc.c.at<int32_t>(dc.c.plan.ints);
  TRY(launch_fill_i32(zero, 0, st->B, dc.c.stream));
  return deep_large_rows(dc.c, st, nullptr, 0, zero, 0, 1, 1);
}

int tandem_deep_score(const tandem_model* m, const tandem_ff_desc* ff_deep, const tandem_deep_state_desc* st,
                      const int32_t* tokens, int64_t n_tokens, const int32_t* pos, int32_t q_len, int32_t gamma,
                      int32_t* greedy, void* logits, void* y_small, void* sketch, void* ws, size_t ws_bytes,
                      void* hip_stream) {
  if (!tokens || !pos) return TANDEM_ERR_NULL;
  if (gamma < 1 || n_tokens < 1) return TANDEM_ERR_SHAPE;
  DeepCtx dc;
  size_t fo = 0, fb = 0;
  TRY(deep_setup(dc, m, ff_deep, st, q_len, ws, ws_bytes, hip_stream, &fo, &fb));
  const Ctx& c = dc.c;
  const tandem_decoder_desc &L = m->d.L, &S = m->d.S;
  const int B = st->B, M = B * q_len;
  const size_t es = elsize(c.dtype);
  // ---- Eq. (3): M_L's rows pos + 1 .. pos + q_len (row p + 1 is the sketch M_S's position p reads)
  TRY(deep_large_rows(c, st, tokens, n_tokens, pos, 1, q_len, gamma));
  void* keep = c.ws + c.plan.keep;  // x^(L_L) of the rows; the step's keep buffers are free here
  TRY(hip_ok(hipMemcpyAsync(keep, c.at<>(c.plan.x), (size_t)M * L.d * es, hipMemcpyDeviceToDevice, c.stream)));
  if (sketch) TRY(hip_ok(hipMemcpyAsync(sketch, keep, (size_t)M * L.d * es, hipMemcpyDeviceToDevice, c.stream)));
  // ---- Eq. (4): y^(0) = Emb_S(token at p) + FF_DeepTandem(sketch), then M_S as a plain causal decoder on its own rows
  void *x = c.at<>(c.plan.x), *qkv = c.at<>(c.plan.qkv), *q = c.at<>(c.plan.q), *att = c.at<>(c.plan.att);
  TRY(launch_embed_shifted(S.emb, tokens, n_tokens, pos, 0, 0, q_len, x, nullptr, nullptr, M, S.d, S.vocab, c.eps, c.dtype,
                           c.stream));
  TRY(run_project(ff_deep, keep, x, M, c.ws + fo, fb, c.stream, x));
  if (c.plan.fused) TRY(launch_rmsnorm(x, S.layers[0].g_attn, c.at<>(c.plan.xn), M, S.d, c.eps, c.dtype, c.stream));
  for (int j = 0; j < S.n_layers; ++j) {
    auto attn_only = [&]() -> int {
      return attn_call(c, S, q, st->KS[j], st->VS[j], pos, nullptr, nullptr, nullptr, 1, q_len, att);
    };
    if (c.plan.fused) {
      auto finish_qkv = [&](const float* part, int splits) -> int {
        return launch_finish_scatter(part, splits, q, st->KS[j], st->VS[j], pos, 0, M, q_len, S.Hq, S.Hkv, S.dh, st->T_max,
                                     S.Hq * S.dh, (S.Hq + 2 * S.Hkv) * S.dh, c.dtype, c.stream);
      };
      const void* g_next = j + 1 < S.n_layers ? S.layers[j + 1].g_attn : S.g_final;
      TRY(decoder_layer_fused(c, S, S.layers[j], M, g_next, finish_qkv, attn_only));
    } else {
      auto attn = [&]() -> int {
        TRY(launch_scatter_qkv(qkv, q, st->KS[j], st->VS[j], pos, 0, M, q_len, S.Hq, S.Hkv, S.dh, st->T_max, 0, S.Hq * S.dh,
                               (S.Hq + 2 * S.Hkv) * S.dh, c.dtype, c.stream));
        return attn_only();
      };
      TRY(decoder_layer(c, S, S.layers[j], M, attn));
    }
  }
  if (y_small) TRY(hip_ok(hipMemcpyAsync(y_small, x, (size_t)M * S.d * es, hipMemcpyDeviceToDevice, c.stream)));
  int32_t* tok = greedy ? greedy : c.at<int32_t>(c.plan.ints);
  TRY(c.plan.fused ? head_normed(c, S, M, tok, 1) : head(c, S, M, tok, 1));
  if (logits)
    TRY(hip_ok(hipMemcpyAsync(logits, c.at<>(c.plan.logits), (size_t)M * S.vocab * es, hipMemcpyDeviceToDevice, c.stream)));
  return TANDEM_OK;
}

int tandem_deep_step(const tandem_model* m, const tandem_ff_desc* ff_deep, const tandem_deep_state_desc* st,
                     int32_t* tokens, int64_t n_tokens, int32_t* len, int32_t gamma, int32_t* out_tokens, void* logits,
                     void* y_small, void* sketch, void* ws, size_t ws_bytes, void* hip_stream) {
  if (!tokens || !len) return TANDEM_ERR_NULL;
  if (gamma < 1 || n_tokens < 1) return TANDEM_ERR_SHAPE;
  DeepCtx dc;
  size_t fo = 0, fb = 0;
  TRY(deep_setup(dc, m, ff_deep, st, gamma, ws, ws_bytes, hip_stream, &fo, &fb));
  const Ctx& c = dc.c;
  const tandem_decoder_desc &L = m->d.L, &S = m->d.S;
  const int B = st->B, M = B * gamma;
  const size_t es = elsize(c.dtype);
  // ---- Eq. (3): the sketch of the next gamma rows in one block pass of M_L.  Row len + rr reads token len + rr - gamma,
  // which is known, and the rows of the blocks completed before its own.
  TRY(deep_large_rows(c, st, tokens, n_tokens, len, 0, gamma, gamma));
  if (sketch) TRY(hip_ok(hipMemcpyAsync(sketch, c.at<>(c.plan.x), (size_t)M * L.d * es, hipMemcpyDeviceToDevice, c.stream)));
  void* ffs = c.at<>(c.plan.yhat);  // FF_DeepTandem of the gamma sketches, [B, gamma, d_S]
  TRY(run_project(ff_deep, c.at<>(c.plan.x), ffs, M, c.ws + fo, fb, c.stream));
  // ---- Eq. (4): gamma runs of M_S, each on the token the run before produced
  void *x = c.at<>(c.plan.x), *qkv = c.at<>(c.plan.qkv), *q = c.at<>(c.plan.q), *att = c.at<>(c.plan.att);
  int32_t* out = out_tokens ? out_tokens : c.at<int32_t>(c.plan.ints);  // [B, gamma]
  for (int t = 0; t < gamma; ++t) {
    TRY(launch_deep_input(S.emb, tokens, n_tokens, len, t, out, gamma, ffs, x, c.plan.fused ? S.layers[0].g_attn : nullptr,
                          c.at<>(c.plan.xn), B, S.d, S.vocab, c.eps, c.dtype, c.stream));
    for (int j = 0; j < S.n_layers; ++j) {
      // position len - 1 + t attends its own rows [0, len - 1 + t]: len + t rows of the position-indexed cache
      auto attn_only = [&]() -> int {
        return attn_call(c, S, q, st->KS[j], st->VS[j], len, nullptr, nullptr, nullptr, 0, 1, att, 0, 0, nullptr, nullptr,
                         nullptr, 0, t);
      };
      if (c.plan.fused) {
        auto finish_qkv = [&](const float* part, int splits) -> int {
          return launch_finish_scatter(part, splits, q, st->KS[j], st->VS[j], len, t - 1, B, 1, S.Hq, S.Hkv, S.dh, st->T_max,
                                       S.Hq * S.dh, (S.Hq + 2 * S.Hkv) * S.dh, c.dtype, c.stream);
        };
        const void* g_next = j + 1 < S.n_layers ? S.layers[j + 1].g_attn : S.g_final;
        TRY(decoder_layer_fused(c, S, S.layers[j], B, g_next, finish_qkv, attn_only));
      } else {
        auto attn = [&]() -> int {
          TRY(launch_scatter_qkv(qkv, q, st->KS[j], st->VS[j], len, t - 1, B, 1, S.Hq, S.Hkv, S.dh, st->T_max, 0, S.Hq * S.dh,
                                 (S.Hq + 2 * S.Hkv) * S.dh, c.dtype, c.stream));
          return attn_only();
        };
        TRY(decoder_layer(c, S, S.layers[j], B, attn));
      }
    }
    if (y_small)
      TRY(copy2d((char*)y_small + (size_t)t * S.d * es, (size_t)gamma * S.d * es, x, S.d * es, S.d * es, B, c.stream));
    TRY(c.plan.fused ? head_normed(c, S, B, out + t, gamma) : head(c, S, B, out + t, gamma));
    if (logits)
      TRY(copy2d((char*)logits + (size_t)t * S.vocab * es, (size_t)gamma * S.vocab * es, c.at<>(c.plan.logits), S.vocab * es,
                 S.vocab * es, B, c.stream));
  }
  const int64_t cap = n_tokens < st->T_max ? n_tokens : st->T_max;
  return launch_deep_advance(tokens, n_tokens, len, out, B, gamma, cap, c.stream);
}

}  // extern "C"
