// Host side of libptdp: argument checks, stash / workspace layout, layer and chunk composition,
// pipeline order of one device, profiling.  Every exported function is declared in include/ptdp.h.
#include <new>
#include <cmath>
#include <mutex>
#include <vector>

#include "common.h"

namespace ptdp {

// ---------------------------------------------------------------- profiling / launch bookkeeping
struct ProfRecord {
  int family;
  double work;
  hipEvent_t start, stop;
};
static std::atomic<bool> g_prof_on{false};
static std::mutex g_prof_mu;                // guards the three containers below
static std::vector<ProfRecord> g_open;      // recorded, not yet collected
static std::vector<hipEvent_t> g_free_events;
static ptdp_prof_entry g_totals[PTDP_K_NFAMILIES];

static bool get_event(hipEvent_t* e) {
  if (!g_free_events.empty()) {
    *e = g_free_events.back();
    g_free_events.pop_back();
    return true;
  }
  return hipEventCreate(e) == hipSuccess;
}

bool profiling_enabled() { return g_prof_on.load(std::memory_order_relaxed); }

Launch::Launch(int family, double work, hipStream_t stream) : stream_(stream), slot_(-1), status_(PTDP_OK), closed_(false) {
  (void)hipGetLastError();  // do not inherit a stale error
  if (!g_prof_on.load(std::memory_order_relaxed)) return;
  std::lock_guard<std::mutex> lock(g_prof_mu);
  ProfRecord r;
  r.family = family;
  r.work = work;
  if (!get_event(&r.start)) { status_ = PTDP_E_HIP; return; }
  if (!get_event(&r.stop)) { g_free_events.push_back(r.start); status_ = PTDP_E_HIP; return; }
  if (hipEventRecord(r.start, stream) != hipSuccess) status_ = PTDP_E_HIP;
  g_open.push_back(r);
  slot_ = (int)g_open.size() - 1;
}

int Launch::status() {
  if (!closed_) {
    closed_ = true;
    if (hipGetLastError() != hipSuccess) status_ = PTDP_E_HIP;
    if (slot_ >= 0) {
      std::lock_guard<std::mutex> lock(g_prof_mu);
      // (a collect between the two halves of a launch has already retired the record: nothing to stop)
      if (slot_ < (int)g_open.size() && hipEventRecord(g_open[slot_].stop, stream_) != hipSuccess) status_ = PTDP_E_HIP;
    }
  }
  return status_;
}

Launch::~Launch() { (void)status(); }

// ---------------------------------------------------------------- configuration
struct Dims {
  int64_t T, h, hp, fp, dh, al;
  size_t esz;
};

static int validate(const ptdp_layer_cfg* c) {
  if (!c) return PTDP_E_NULL_PTR;
  if (c->struct_size != sizeof(ptdp_layer_cfg)) return PTDP_E_INVALID_ARG;
  if (c->h <= 0 || c->a <= 0 || c->t <= 0 || c->s <= 0 || c->b <= 0) return PTDP_E_INVALID_ARG;
  if (c->h % c->a != 0 || c->a % c->t != 0 || (4ll * c->h) % c->t != 0) return PTDP_E_INVALID_ARG;
  if (c->dtype != PTDP_F32 && c->dtype != PTDP_BF16) return PTDP_E_INVALID_ARG;
  if (c->gelu_mode != PTDP_GELU_ERF && c->gelu_mode != PTDP_GELU_TANH) return PTDP_E_INVALID_ARG;
  if (!(c->p_hidden >= 0.f && c->p_hidden < 1.f)) return PTDP_E_INVALID_ARG;
  if (!(c->ln_eps > 0.f)) return PTDP_E_INVALID_ARG;
  if (c->causal != 0 && c->causal != 1) return PTDP_E_INVALID_ARG;
  const int dh = c->h / c->a;
  if (dh % 8 != 0 || c->h % 8 != 0) return PTDP_E_INVALID_ARG;
  if ((int64_t)c->s * c->b > (1ll << 30)) return PTDP_E_INVALID_ARG;
  if (!attn_dh_supported(c->dtype, dh)) return PTDP_E_UNSUPPORTED;
  // LayerNorm keeps a row in registers: at most 8 vectors x 512 threads
  const int64_t per_vec = c->dtype == PTDP_BF16 ? 8 : 4;
  if (c->h > 8 * 512 * per_vec) return PTDP_E_UNSUPPORTED;
  if (c->dtype == PTDP_BF16) {
    // the bf16 GEMM addresses each operand through a 31-bit byte offset: refuse up front what a GEMM
    // in the middle of a layer would refuse (the largest operands are w_1 / w_2 and the [T, 4h/t] activations)
    const int64_t lim = 0x7fffffffll, T = (int64_t)c->s * c->b, fp = 4ll * c->h / c->t, qp = 3ll * c->h / c->t;
    const int64_t wide = fp > qp ? fp : qp, big = wide > c->h ? wide : c->h;
    if (2 * (int64_t)c->h * wide >= lim || 2 * T * big >= lim) return PTDP_E_UNSUPPORTED;
  }
  return PTDP_OK;
}

static Dims dims_of(const ptdp_layer_cfg* c) {
  Dims d;
  d.T = (int64_t)c->s * c->b;
  d.h = c->h;
  d.hp = c->h / c->t;
  d.fp = 4ll * c->h / c->t;
  d.dh = c->h / c->a;
  d.al = c->a / c->t;
  d.esz = c->dtype == PTDP_BF16 ? 2 : 4;
  return d;
}

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct StashLayout {
  size_t off[PTDP_STASH_NFIELDS];
  size_t total;
};
static StashLayout stash_layout(const ptdp_layer_cfg* c) {
  const Dims d = dims_of(c);
  size_t sz[PTDP_STASH_NFIELDS];
  sz[PTDP_STASH_X] = d.T * d.h * d.esz;
  sz[PTDP_STASH_U] = d.T * d.h * d.esz;
  sz[PTDP_STASH_QKV] = d.T * 3 * d.hp * d.esz;
  sz[PTDP_STASH_CTX] = d.T * d.hp * d.esz;
  sz[PTDP_STASH_X1] = d.T * d.h * d.esz;
  sz[PTDP_STASH_U2] = d.T * d.h * d.esz;
  sz[PTDP_STASH_Z] = d.T * d.fp * d.esz;
  sz[PTDP_STASH_G] = d.T * d.fp * d.esz;
  sz[PTDP_STASH_MU1] = sz[PTDP_STASH_RSTD1] = sz[PTDP_STASH_MU2] = sz[PTDP_STASH_RSTD2] = d.T * sizeof(float);
  sz[PTDP_STASH_LSE] = (size_t)c->b * d.al * c->s * sizeof(float);
  StashLayout L;
  size_t o = 0;
  for (int i = 0; i < PTDP_STASH_NFIELDS; ++i) {
    L.off[i] = o;
    o += align256(sz[i]);
  }
  L.total = o;
  return L;
}

// workspace fields
enum { WS_H1 = 0, WS_H2, WS_X1, WS_CHAIN, WS_BIG, WS_CTX, WS_QKV, WS_DMO, WS_DELTA, WS_COLSUM, WS_SPLITK, WS_N };
struct WsLayout {
  size_t off[WS_N];
  size_t total;
};
// scratch regions of WS_COLSUM, in the order the backward uses them: b_2, b_1, LayerNorm-2, b_o, b_qkv, LayerNorm-1
constexpr int kColsumRegions = 6;
static size_t colsum_region_bytes(const Dims& d, int i) {
  size_t b = 0;
  switch (i) {
    case 0: case 3: b = colsum_scratch_bytes((int)d.T, (int)d.h); break;
    case 1: b = colsum_scratch_bytes((int)d.T, (int)d.fp); break;
    case 4: b = colsum_scratch_bytes((int)d.T, (int)(3 * d.hp)); break;
    default: b = layernorm_bwd_scratch_bytes((int)d.T, (int)d.h); break;
  }
  return align256(b);
}

static WsLayout ws_layout(const ptdp_layer_cfg* c) {
  const Dims d = dims_of(c);
  size_t sz[WS_N];
  sz[WS_H1] = sz[WS_H2] = sz[WS_X1] = sz[WS_CHAIN] = sz[WS_DMO] = d.T * d.h * d.esz;
  sz[WS_BIG] = d.T * d.fp * d.esz;
  sz[WS_CTX] = d.T * d.hp * d.esz;
  sz[WS_QKV] = d.T * 3 * d.hp * d.esz;
  sz[WS_DELTA] = (size_t)c->b * d.al * c->s * sizeof(float);
  // the six column-sum producers of a layer's backward keep their partial sums until one launch finishes them all
  size_t cs = 0;
  for (int i = 0; i < kColsumRegions; ++i) cs += colsum_region_bytes(d, i);
  sz[WS_COLSUM] = cs;
  // partial tiles of GEMMs whose last, incomplete round of tiles is split along k
  sz[WS_SPLITK] = c->dtype == PTDP_BF16 ? gemm_workspace_bytes() : 0;
  WsLayout L;
  size_t o = 0;
  for (int i = 0; i < WS_N; ++i) {
    L.off[i] = o;
    o += align256(sz[i]);
  }
  L.total = o;
  return L;
}

static inline size_t ws_field_bytes(const WsLayout& L, int f) {
  return (f + 1 < WS_N ? L.off[f + 1] : L.total) - L.off[f];
}

}  // namespace ptdp

using namespace ptdp;

struct ptdp_chunk {
  ptdp_layer_cfg cfg;
  int n_layers;
  int first_layer;
  std::vector<ptdp_layer_params> params;
  std::vector<ptdp_layer_grads> grads;
  std::vector<char> have_params, have_grads;
  const uint8_t* mask = nullptr;   // general attention mask [b, s, s] (dev, borrowed); used when cfg.causal == 0
  StashLayout sl;
  WsLayout wl;
};

extern "C" {

const char* ptdp_status_string(int status) {
  switch (status) {
    case PTDP_OK: return "ok";
    case PTDP_E_INVALID_ARG: return "invalid argument";
    case PTDP_E_UNSUPPORTED: return "unsupported configuration";
    case PTDP_E_NULL_PTR: return "null pointer";
    case PTDP_E_TOO_SMALL: return "buffer or capacity too small";
    case PTDP_E_HIP: return "HIP runtime error";
    case PTDP_E_STATE: return "object not ready";
    default: return "unknown status";
  }
}

int ptdp_cfg_validate(const ptdp_layer_cfg* cfg) { return validate(cfg); }

size_t ptdp_layer_stash_bytes(const ptdp_layer_cfg* cfg) {
  if (validate(cfg) != PTDP_OK) return 0;
  return stash_layout(cfg).total;
}

size_t ptdp_stash_offset(const ptdp_layer_cfg* cfg, int field) {
  if (validate(cfg) != PTDP_OK || field < 0 || field >= PTDP_STASH_NFIELDS) return (size_t)-1;
  return stash_layout(cfg).off[field];
}

size_t ptdp_workspace_bytes(const ptdp_layer_cfg* cfg) {
  if (validate(cfg) != PTDP_OK) return 0;
  return ws_layout(cfg).total;
}

size_t ptdp_workspace_offset(const ptdp_layer_cfg* cfg, int field) {
  static_assert(PTDP_WS_DO == WS_H1 && PTDP_WS_DU == WS_H2 && PTDP_WS_DX1 == WS_X1 && PTDP_WS_CHAIN == WS_CHAIN &&
                    PTDP_WS_DZ == WS_BIG && PTDP_WS_DCTX == WS_CTX && PTDP_WS_DQKV == WS_QKV && PTDP_WS_DMO == WS_DMO,
                "public workspace fields are the first internal ones, in order");
  if (validate(cfg) != PTDP_OK || field < 0 || field >= PTDP_WS_NFIELDS) return (size_t)-1;
  return ws_layout(cfg).off[field];
}

int64_t ptdp_layer_flops_fwd(const ptdp_layer_cfg* cfg) {
  if (validate(cfg) != PTDP_OK) return -1;
  const int64_t b = cfg->b, s = cfg->s, h = cfg->h;
  return (24 * b * s * h * h + 4 * b * s * s * h) / cfg->t;
}

double ptdp_batch_time(int64_t b_prime, int64_t b, int p, double t_fwd, double t_bwd) {
  if (b_prime < 1 || b < 1 || p < 1 || b_prime % b != 0 || !(t_fwd >= 0.0) || !(t_bwd >= 0.0) || std::isinf(t_fwd) ||
      std::isinf(t_bwd))
    return std::nan("");
  return (double)(b_prime / b + p - 1) * (t_fwd + t_bwd);
}

uint64_t ptdp_hash(uint64_t seed, uint32_t layer, uint32_t site, uint64_t microbatch, uint64_t group) {
  return mix64(dropout_key(seed, layer, site, microbatch) + kGolden * group);
}

// ------------------------------------------------------------------------------------- chunks
int ptdp_chunk_create(const ptdp_layer_cfg* cfg, int n_layers, int first_global_layer, ptdp_chunk** out) {
  if (!out) return PTDP_E_NULL_PTR;
  *out = nullptr;
  const int rc = validate(cfg);
  if (rc != PTDP_OK) return rc;
  if (n_layers <= 0 || n_layers > 65536 || first_global_layer < 0) return PTDP_E_INVALID_ARG;
  ptdp_chunk* c = new (std::nothrow) ptdp_chunk();
  if (!c) return PTDP_E_TOO_SMALL;
  c->cfg = *cfg;
  c->n_layers = n_layers;
  c->first_layer = first_global_layer;
  c->params.resize(n_layers);
  c->grads.resize(n_layers);
  c->have_params.assign(n_layers, 0);
  c->have_grads.assign(n_layers, 0);
  c->sl = stash_layout(cfg);
  c->wl = ws_layout(cfg);
  *out = c;
  return PTDP_OK;
}

void ptdp_chunk_destroy(ptdp_chunk* chunk) { delete chunk; }

int ptdp_chunk_n_layers(const ptdp_chunk* chunk) { return chunk ? chunk->n_layers : PTDP_E_NULL_PTR; }

int ptdp_chunk_bind_params(ptdp_chunk* chunk, int layer, const ptdp_layer_params* p) {
  if (!chunk || !p) return PTDP_E_NULL_PTR;
  if (layer < 0 || layer >= chunk->n_layers) return PTDP_E_INVALID_ARG;
  const void* const* q = reinterpret_cast<const void* const*>(p);
  for (int i = 0; i < 12; ++i)
    if (!q[i]) return PTDP_E_NULL_PTR;
  chunk->params[layer] = *p;
  chunk->have_params[layer] = 1;
  return PTDP_OK;
}

int ptdp_chunk_set_mask(ptdp_chunk* chunk, const uint8_t* mask) {
  if (!chunk) return PTDP_E_NULL_PTR;
  if ((chunk->cfg.causal != 0 && mask) || ((uintptr_t)mask & 3)) return PTDP_E_INVALID_ARG;
  chunk->mask = mask;
  return PTDP_OK;
}

int ptdp_chunk_bind_grads(ptdp_chunk* chunk, int layer, const ptdp_layer_grads* g) {
  if (!chunk || !g) return PTDP_E_NULL_PTR;
  if (layer < 0 || layer >= chunk->n_layers) return PTDP_E_INVALID_ARG;
  float* const* q = reinterpret_cast<float* const*>(g);
  for (int i = 0; i < 12; ++i)
    if (!q[i]) return PTDP_E_NULL_PTR;
  chunk->grads[layer] = *g;
  chunk->have_grads[layer] = 1;
  return PTDP_OK;
}

#define PTDP_TRY(expr)            \
  do {                            \
    const int rc__ = (expr);      \
    if (rc__ != PTDP_OK) return rc__; \
  } while (0)

int ptdp_layer_forward(ptdp_chunk* ch, int layer, int64_t microbatch, const void* x, void* y, void* stash,
                       void* workspace, void* stream) {
  if (!ch || !x || !y || !stash || !workspace) return PTDP_E_NULL_PTR;
  if (layer < 0 || layer >= ch->n_layers || microbatch < 0 || x == y) return PTDP_E_INVALID_ARG;
  if (!ch->have_params[layer]) return PTDP_E_STATE;
  const ptdp_layer_cfg& c = ch->cfg;
  const ptdp_layer_params& P = ch->params[layer];
  const Dims d = dims_of(&c);
  hipStream_t st = (hipStream_t)stream;
  char* S = (char*)stash;
  char* W = (char*)workspace;
  auto sf = [&](int f) { return (void*)(S + ch->sl.off[f]); };
  const int T = (int)d.T, h = (int)d.h, hp = (int)d.hp, fp = (int)d.fp;
  const uint32_t gl = (uint32_t)(ch->first_layer + layer);
  void* o = W + ch->wl.off[WS_H1];
  void* sk = W + ch->wl.off[WS_SPLITK];
  const size_t skb = ws_field_bytes(ch->wl, WS_SPLITK);
  void* x_copy = (x == sf(PTDP_STASH_X)) ? nullptr : sf(PTDP_STASH_X);

  PTDP_TRY(launch_layernorm_fwd(c.dtype, x, P.ln1_g, P.ln1_b, sf(PTDP_STASH_U), (float*)sf(PTDP_STASH_MU1),
                                (float*)sf(PTDP_STASH_RSTD1), x_copy, T, h, c.ln_eps, st));
  PTDP_TRY(launch_gemm(c.dtype, PTDP_GEMM_NN, sf(PTDP_STASH_U), P.w_qkv, sf(PTDP_STASH_QKV), P.b_qkv, T, 3 * hp, h, 0,
                       0, sk, skb, st));
  PTDP_TRY(launch_attn_fwd(c.dtype, sf(PTDP_STASH_QKV), sf(PTDP_STASH_CTX), (float*)sf(PTDP_STASH_LSE), c.s, c.b,
                           (int)d.al, (int)d.dh, ch->mask, c.causal, st));
  PTDP_TRY(launch_gemm(c.dtype, PTDP_GEMM_NN, sf(PTDP_STASH_CTX), P.w_o, o, nullptr, T, h, hp, 0, 0, sk, skb, st));
  PTDP_TRY(launch_bda_fwd(c.dtype, o, P.b_o, x, sf(PTDP_STASH_X1), T, h, c.p_hidden,
                          dropout_key(c.seed, gl, 0, (uint64_t)microbatch), st));
  PTDP_TRY(launch_layernorm_fwd(c.dtype, sf(PTDP_STASH_X1), P.ln2_g, P.ln2_b, sf(PTDP_STASH_U2),
                                (float*)sf(PTDP_STASH_MU2), (float*)sf(PTDP_STASH_RSTD2), nullptr, T, h, c.ln_eps,
                                st));
  PTDP_TRY(launch_gemm(c.dtype, PTDP_GEMM_NN, sf(PTDP_STASH_U2), P.w_1, sf(PTDP_STASH_Z), nullptr, T, fp, h, 0, 0, sk, skb, st));
  PTDP_TRY(launch_bias_gelu_fwd(c.dtype, c.gelu_mode, sf(PTDP_STASH_Z), P.b_1, sf(PTDP_STASH_G), T, fp, st));
  PTDP_TRY(launch_gemm(c.dtype, PTDP_GEMM_NN, sf(PTDP_STASH_G), P.w_2, o, nullptr, T, h, fp, 0, 0, sk, skb, st));
  PTDP_TRY(launch_bda_fwd(c.dtype, o, P.b_2, sf(PTDP_STASH_X1), y, T, h, c.p_hidden,
                          dropout_key(c.seed, gl, 1, (uint64_t)microbatch), st));
  return PTDP_OK;
}

int ptdp_layer_backward(ptdp_chunk* ch, int layer, int64_t microbatch, const void* dy, void* dx, const void* stash,
                        void* workspace, void* stream) {
  if (!ch || !dy || !dx || !stash || !workspace) return PTDP_E_NULL_PTR;
  if (layer < 0 || layer >= ch->n_layers || microbatch < 0) return PTDP_E_INVALID_ARG;
  if (!ch->have_params[layer] || !ch->have_grads[layer]) return PTDP_E_STATE;
  const ptdp_layer_cfg& c = ch->cfg;
  const ptdp_layer_params& P = ch->params[layer];
  const ptdp_layer_grads& G = ch->grads[layer];
  const Dims d = dims_of(&c);
  hipStream_t st = (hipStream_t)stream;
  const char* S = (const char*)stash;
  char* W = (char*)workspace;
  auto sf = [&](int f) { return (const void*)(S + ch->sl.off[f]); };
  auto wf = [&](int f) { return (void*)(W + ch->wl.off[f]); };
  const int T = (int)d.T, h = (int)d.h, hp = (int)d.hp, fp = (int)d.fp;
  const uint32_t gl = (uint32_t)(ch->first_layer + layer);
  const int dt = c.dtype;
  char* cs0 = (char*)wf(WS_COLSUM);
  void* csr[kColsumRegions];
  for (int i = 0; i < kColsumRegions; ++i) {
    csr[i] = cs0;
    cs0 += colsum_region_bytes(d, i);
  }
  ColsumBatch sums;   // the six second stages run as one launch at the end
  void* sk = wf(WS_SPLITK);
  const size_t skb = ws_field_bytes(ch->wl, WS_SPLITK);

  // MLP block.  The four weight gradients of the layer wait until all their inputs are there and run as one
  // launch at the end (each one's tiles fill the last, partial round of the ones before it); until then G, U2,
  // CTX, U and the gradients d(mo) [WS_DMO], dz [WS_BIG], do [WS_H1], dqkv [WS_QKV] stay untouched.
  PTDP_TRY(launch_bda_bwd(dt, dy, wf(WS_DMO), G.b_2, csr[0], T, h, c.p_hidden,
                          dropout_key(c.seed, gl, 1, (uint64_t)microbatch), st, &sums));
  PTDP_TRY(launch_gemm(dt, PTDP_GEMM_NT, wf(WS_DMO), P.w_2, wf(WS_BIG), nullptr, T, fp, h, 0, 0, sk, skb, st));
  PTDP_TRY(launch_bias_gelu_bwd(dt, c.gelu_mode, wf(WS_BIG), sf(PTDP_STASH_Z), P.b_1, wf(WS_BIG), G.b_1, csr[1], T, fp, st, &sums));
  PTDP_TRY(launch_gemm(dt, PTDP_GEMM_NT, wf(WS_BIG), P.w_1, wf(WS_H2), nullptr, T, h, fp, 0, 0, sk, skb, st));
  PTDP_TRY(launch_layernorm_bwd(dt, wf(WS_H2), sf(PTDP_STASH_X1), P.ln2_g, (const float*)sf(PTDP_STASH_MU2),
                                (const float*)sf(PTDP_STASH_RSTD2), dy, wf(WS_X1), G.ln2_g, G.ln2_b, csr[2], T, h, st, &sums));
  // attention block
  PTDP_TRY(launch_bda_bwd(dt, wf(WS_X1), wf(WS_H1), G.b_o, csr[3], T, h, c.p_hidden,
                          dropout_key(c.seed, gl, 0, (uint64_t)microbatch), st, &sums));
  PTDP_TRY(launch_gemm(dt, PTDP_GEMM_NT, wf(WS_H1), P.w_o, wf(WS_CTX), nullptr, T, hp, h, 0, 0, sk, skb, st));
  PTDP_TRY(launch_attn_bwd(dt, sf(PTDP_STASH_QKV), sf(PTDP_STASH_CTX), (const float*)sf(PTDP_STASH_LSE), wf(WS_CTX),
                           wf(WS_QKV), (float*)wf(WS_DELTA), c.s, c.b, (int)d.al, (int)d.dh, ch->mask, c.causal, st));
  PTDP_TRY(launch_colsum(dt, wf(WS_QKV), G.b_qkv, csr[4], T, 3 * hp, st, &sums));
  PTDP_TRY(launch_gemm(dt, PTDP_GEMM_NT, wf(WS_QKV), P.w_qkv, wf(WS_H2), nullptr, T, h, 3 * hp, 0, 0, sk, skb, st));
  {
    const void* A[4] = {sf(PTDP_STASH_G), sf(PTDP_STASH_U2), sf(PTDP_STASH_U), sf(PTDP_STASH_CTX)};
    const void* B[4] = {wf(WS_DMO), wf(WS_BIG), wf(WS_QKV), wf(WS_H1)};
    float* C[4] = {G.w_2, G.w_1, G.w_qkv, G.w_o};
    const int M[4] = {fp, h, h, hp}, N[4] = {h, fp, 3 * hp, h};
    PTDP_TRY(launch_gemm_tn_multi(dt, 4, A, B, C, M, N, T, st));
  }
  PTDP_TRY(launch_layernorm_bwd(dt, wf(WS_H2), sf(PTDP_STASH_X), P.ln1_g, (const float*)sf(PTDP_STASH_MU1),
                                (const float*)sf(PTDP_STASH_RSTD1), wf(WS_X1), dx, G.ln1_g, G.ln1_b, csr[5], T, h, st, &sums));
  PTDP_TRY(launch_colsum_batch(sums, st));
  return PTDP_OK;
}

int ptdp_chunk_forward(ptdp_chunk* ch, int64_t microbatch, const void* x, void* y, void* stash, void* workspace,
                       void* stream) {
  if (!ch || !x || !y || !stash || !workspace) return PTDP_E_NULL_PTR;
  if (microbatch < 0 || x == y) return PTDP_E_INVALID_ARG;
  for (int l = 0; l < ch->n_layers; ++l)
    if (!ch->have_params[l]) return PTDP_E_STATE;
  char* S = (char*)stash;
  const void* cur = x;
  for (int l = 0; l < ch->n_layers; ++l) {
    // a layer's output is written straight into the next layer's stash slot for X
    void* out = (l + 1 < ch->n_layers) ? (void*)(S + (size_t)(l + 1) * ch->sl.total + ch->sl.off[PTDP_STASH_X]) : y;
    PTDP_TRY(ptdp_layer_forward(ch, l, microbatch, cur, out, S + (size_t)l * ch->sl.total, workspace, stream));
    cur = out;
  }
  return PTDP_OK;
}

int ptdp_chunk_backward(ptdp_chunk* ch, int64_t microbatch, const void* dy, void* dx, const void* stash,
                        void* workspace, void* stream) {
  if (!ch || !dy || !dx || !stash || !workspace) return PTDP_E_NULL_PTR;
  if (microbatch < 0) return PTDP_E_INVALID_ARG;
  for (int l = 0; l < ch->n_layers; ++l)
    if (!ch->have_params[l] || !ch->have_grads[l]) return PTDP_E_STATE;
  const char* S = (const char*)stash;
  void* chain = (char*)workspace + ch->wl.off[WS_CHAIN];
  const void* cur = dy;
  for (int l = ch->n_layers - 1; l >= 0; --l) {
    void* out = l > 0 ? chain : dx;
    PTDP_TRY(ptdp_layer_backward(ch, l, microbatch, cur, out, S + (size_t)l * ch->sl.total, workspace, stream));
    cur = out;
  }
  return PTDP_OK;
}

// ------------------------------------------------------------------------ activation recomputation
size_t ptdp_checkpoint_bytes(const ptdp_layer_cfg* cfg) {
  if (validate(cfg) != PTDP_OK) return 0;
  const Dims d = dims_of(cfg);
  const size_t esz = cfg->dtype == PTDP_BF16 ? 2 : 4;
  return ((size_t)d.T * d.h * esz + 255) / 256 * 256;
}

int ptdp_chunk_n_checkpoints(const ptdp_chunk* ch, int seg_layers) {
  if (!ch) return PTDP_E_NULL_PTR;
  if (seg_layers < 1 || seg_layers > ch->n_layers) return PTDP_E_INVALID_ARG;
  return (ch->n_layers + seg_layers - 1) / seg_layers;
}

// Forward of layers [l0, l1) of a chunk with layer l's stash at seg_stash slot (l - l0).  The
// segment's output goes to `out`.
static int segment_forward(ptdp_chunk* ch, int l0, int l1, int64_t mb, const void* x, void* out, char* seg_stash,
                           void* workspace, void* stream) {
  const void* cur = x;
  for (int l = l0; l < l1; ++l) {
    void* y = (l + 1 < l1) ? (void*)(seg_stash + (size_t)(l + 1 - l0) * ch->sl.total + ch->sl.off[PTDP_STASH_X]) : out;
    PTDP_TRY(ptdp_layer_forward(ch, l, mb, cur, y, seg_stash + (size_t)(l - l0) * ch->sl.total, workspace, stream));
    cur = y;
  }
  return PTDP_OK;
}

int ptdp_chunk_forward_ckpt(ptdp_chunk* ch, int64_t microbatch, const void* x, void* y, void* ckpt, int seg_layers,
                            void* seg_stash, void* workspace, void* stream) {
  if (!ch || !x || !y || !ckpt || !seg_stash || !workspace) return PTDP_E_NULL_PTR;
  if (microbatch < 0 || x == y || x == ckpt || seg_layers < 1 || seg_layers > ch->n_layers) return PTDP_E_INVALID_ARG;
  for (int l = 0; l < ch->n_layers; ++l)
    if (!ch->have_params[l]) return PTDP_E_STATE;
  const size_t cb = ptdp_checkpoint_bytes(&ch->cfg);
  const Dims d = dims_of(&ch->cfg);
  const size_t act = (size_t)d.T * d.h * (ch->cfg.dtype == PTDP_BF16 ? 2 : 4);
  if (hipMemcpyAsync(ckpt, x, act, hipMemcpyDeviceToDevice, (hipStream_t)stream) != hipSuccess) return PTDP_E_HIP;
  const int n = ch->n_layers;
  for (int l0 = 0, sg = 0; l0 < n; l0 += seg_layers, ++sg) {
    const int l1 = l0 + seg_layers < n ? l0 + seg_layers : n;
    // a segment's output is the next segment's checkpoint
    void* out = l1 < n ? (void*)((char*)ckpt + (size_t)(sg + 1) * cb) : y;
    PTDP_TRY(segment_forward(ch, l0, l1, microbatch, (char*)ckpt + (size_t)sg * cb, out, (char*)seg_stash, workspace,
                             stream));
  }
  return PTDP_OK;
}

int ptdp_chunk_backward_ckpt(ptdp_chunk* ch, int64_t microbatch, const void* dy, void* dx, const void* ckpt,
                             int seg_layers, void* seg_stash, void* workspace, void* stream) {
  if (!ch || !dy || !dx || !ckpt || !seg_stash || !workspace) return PTDP_E_NULL_PTR;
  if (microbatch < 0 || seg_layers < 1 || seg_layers > ch->n_layers) return PTDP_E_INVALID_ARG;
  for (int l = 0; l < ch->n_layers; ++l)
    if (!ch->have_params[l] || !ch->have_grads[l]) return PTDP_E_STATE;
  const size_t cb = ptdp_checkpoint_bytes(&ch->cfg);
  const int n = ch->n_layers, n_seg = (n + seg_layers - 1) / seg_layers;
  char* S = (char*)seg_stash;
  void* chain = (char*)workspace + ch->wl.off[WS_CHAIN];
  const void* cur = dy;
  for (int sg = n_seg - 1; sg >= 0; --sg) {
    const int l0 = sg * seg_layers, l1 = l0 + seg_layers < n ? l0 + seg_layers : n;
    // Rerun the segment.  Its output is not needed again: the last segment's goes to the gradient
    // chain buffer (idle until the first backward), an inner segment's rewrites the next checkpoint
    // with the bits it already holds.
    void* out = l1 < n ? (void*)((char*)ckpt + (size_t)(sg + 1) * cb) : chain;
    PTDP_TRY(segment_forward(ch, l0, l1, microbatch, (const char*)ckpt + (size_t)sg * cb, out, S, workspace, stream));
    for (int l = l1 - 1; l >= l0; --l) {
      void* o = l > 0 ? chain : dx;
      PTDP_TRY(ptdp_layer_backward(ch, l, microbatch, cur, o, S + (size_t)(l - l0) * ch->sl.total, workspace, stream));
      cur = o;
    }
  }
  return PTDP_OK;
}

// ------------------------------------------------------------------------------------ schedule
static int sched_check(int p, int v, int m, int rank) {
  if (p < 1 || v < 1 || m < 1 || rank < 0 || rank >= p) return PTDP_E_INVALID_ARG;
  if (v > 1 && m % p != 0) return PTDP_E_INVALID_ARG;
  if ((int64_t)m * v > (1 << 28)) return PTDP_E_INVALID_ARG;
  return PTDP_OK;
}

// k-th forward (backward) pass of a device: microbatches go in groups of p; within a group the
// device runs the group on chunk 0, then chunk 1, ... (backward: last chunk first).
static inline void sched_slot(int k, int p, int v, bool backward, int* chunk, int* mb) {
  const int group = k / (p * v), within = k % (p * v);
  const int c = within / p;
  *chunk = backward ? v - 1 - c : c;
  *mb = group * p + within % p;
}

static int sched_warmup(int p, int v, int m, int rank) {
  const int64_t total = (int64_t)m * v;
  const int64_t w = (v == 1) ? (p - rank - 1) : ((int64_t)(v - 1) * p + 2ll * (p - rank - 1));
  return (int)(w < total ? w : total);
}

int ptdp_schedule_build(int p, int v, int m, int rank, ptdp_step* out, int cap, int* n_out) {
  PTDP_TRY(sched_check(p, v, m, rank));
  if (!n_out) return PTDP_E_NULL_PTR;
  const int total = m * v;
  *n_out = 2 * total;
  if (!out) return cap == 0 ? PTDP_OK : PTDP_E_NULL_PTR;
  if (cap < 2 * total) return PTDP_E_TOO_SMALL;
  const int w = sched_warmup(p, v, m, rank);
  int n = 0;
  auto emit = [&](int k, bool bwd) {
    out[n].kind = bwd ? 1 : 0;
    sched_slot(k, p, v, bwd, &out[n].chunk, &out[n].microbatch);
    ++n;
  };
  for (int k = 0; k < w; ++k) emit(k, false);
  for (int k = 0; k < total - w; ++k) {
    emit(w + k, false);
    emit(k, true);
  }
  for (int k = total - w; k < total; ++k) emit(k, true);
  return PTDP_OK;
}

int ptdp_schedule_peak_inflight(int p, int v, int m, int rank) {
  PTDP_TRY(sched_check(p, v, m, rank));
  // forwards lead backwards by the warm-up count, plus one during the steady 1F1B phase
  const int total = m * v, w = sched_warmup(p, v, m, rank);
  return w < total ? w + 1 : w;
}

// seg_layers == 0: full stashes in the pool; > 0: checkpoints in the pool, seg_stash as scratch.
static int schedule_run_impl(ptdp_chunk* const* chunks, int v, int m, const ptdp_step* steps, int n_steps,
                             const void* const* stage_in, void* const* stage_out, const void* const* stage_dout,
                             void* const* stage_din, void* stash_pool, size_t slot_bytes, int n_slots, int seg_layers,
                             void* seg_stash, void* workspace, void* stream) {
  if (!chunks || !steps || !stage_in || !stage_out || !stage_dout || !stage_din || !stash_pool || !workspace)
    return PTDP_E_NULL_PTR;
  if (seg_layers > 0 && !seg_stash) return PTDP_E_NULL_PTR;
  if (v < 1 || m < 1 || n_steps < 0 || n_slots < 0) return PTDP_E_INVALID_ARG;
  for (int c = 0; c < v; ++c) {
    if (!chunks[c]) return PTDP_E_NULL_PTR;
    if (seg_layers > 0) {
      const int nc = ptdp_chunk_n_checkpoints(chunks[c], seg_layers);
      if (nc < 0) return nc;
      if (slot_bytes < (size_t)nc * ptdp_checkpoint_bytes(&chunks[c]->cfg)) return PTDP_E_TOO_SMALL;
      if (chunks[c]->sl.total > chunks[0]->sl.total) return PTDP_E_INVALID_ARG;  // one seg_stash serves all
    } else if (slot_bytes < (size_t)chunks[c]->n_layers * chunks[c]->sl.total) {
      return PTDP_E_TOO_SMALL;
    }
    if (ws_layout(&chunks[c]->cfg).total > ws_layout(&chunks[0]->cfg).total) return PTDP_E_INVALID_ARG;
  }
  // dry run on the host: slot assignment, order validity, capacity
  std::vector<int> slot_of((size_t)v * m, -1), done_b((size_t)v * m, 0), assigned(n_steps, -1);
  std::vector<int> free_slots;
  for (int i = n_slots - 1; i >= 0; --i) free_slots.push_back(i);
  for (int i = 0; i < n_steps; ++i) {
    const ptdp_step& s = steps[i];
    if (s.chunk < 0 || s.chunk >= v || s.microbatch < 0 || s.microbatch >= m || (s.kind != 0 && s.kind != 1))
      return PTDP_E_INVALID_ARG;
    const size_t id = (size_t)s.chunk * m + s.microbatch;
    if (!stage_in[id] || !stage_out[id] || !stage_dout[id] || !stage_din[id]) return PTDP_E_NULL_PTR;
    if (s.kind == 0) {
      if (slot_of[id] != -1 || done_b[id]) return PTDP_E_INVALID_ARG;  // forwarded twice
      if (free_slots.empty()) return PTDP_E_TOO_SMALL;
      slot_of[id] = free_slots.back();
      free_slots.pop_back();
      assigned[i] = slot_of[id];
    } else {
      if (slot_of[id] < 0) return PTDP_E_INVALID_ARG;  // backward without its forward
      assigned[i] = slot_of[id];
      free_slots.push_back(slot_of[id]);
      slot_of[id] = -1;
      done_b[id] = 1;
    }
  }
  for (int i = 0; i < n_steps; ++i) {
    const ptdp_step& s = steps[i];
    const size_t id = (size_t)s.chunk * m + s.microbatch;
    char* slot = (char*)stash_pool + (size_t)assigned[i] * slot_bytes;
    ptdp_chunk* ch = chunks[s.chunk];
    if (seg_layers > 0) {
      if (s.kind == 0)
        PTDP_TRY(ptdp_chunk_forward_ckpt(ch, s.microbatch, stage_in[id], stage_out[id], slot, seg_layers, seg_stash,
                                         workspace, stream));
      else
        PTDP_TRY(ptdp_chunk_backward_ckpt(ch, s.microbatch, stage_dout[id], stage_din[id], slot, seg_layers,
                                          seg_stash, workspace, stream));
    } else if (s.kind == 0) {
      PTDP_TRY(ptdp_chunk_forward(ch, s.microbatch, stage_in[id], stage_out[id], slot, workspace, stream));
    } else {
      PTDP_TRY(ptdp_chunk_backward(ch, s.microbatch, stage_dout[id], stage_din[id], slot, workspace, stream));
    }
  }
  return PTDP_OK;
}

int ptdp_schedule_run(ptdp_chunk* const* chunks, int v, int m, const ptdp_step* steps, int n_steps,
                      const void* const* stage_in, void* const* stage_out, const void* const* stage_dout,
                      void* const* stage_din, void* stash_pool, size_t slot_bytes, int n_slots, void* workspace,
                      void* stream) {
  return schedule_run_impl(chunks, v, m, steps, n_steps, stage_in, stage_out, stage_dout, stage_din, stash_pool,
                           slot_bytes, n_slots, 0, nullptr, workspace, stream);
}

int ptdp_schedule_run_ckpt(ptdp_chunk* const* chunks, int v, int m, const ptdp_step* steps, int n_steps,
                           const void* const* stage_in, void* const* stage_out, const void* const* stage_dout,
                           void* const* stage_din, void* ckpt_pool, size_t slot_bytes, int n_slots, int seg_layers,
                           void* seg_stash, void* workspace, void* stream) {
  if (seg_layers < 1) return PTDP_E_INVALID_ARG;
  return schedule_run_impl(chunks, v, m, steps, n_steps, stage_in, stage_out, stage_dout, stage_din, ckpt_pool,
                           slot_bytes, n_slots, seg_layers, seg_stash, workspace, stream);
}

// --------------------------------------------------------------------- first / last stage extras
namespace {
enum { LM_U = 0, LM_MU, LM_RSTD, LM_LOGITS, LM_DU, LM_COLSUM, LM_SPLITK, LM_N };
struct LmLayout {
  size_t off[LM_N];
  size_t total;
};
LmLayout lm_layout(const ptdp_layer_cfg* c, int vrows) {
  const Dims d = dims_of(c);
  size_t sz[LM_N];
  sz[LM_U] = sz[LM_DU] = d.T * d.h * d.esz;   // LM_DU doubles as the masked gradient of the embedding backward
  sz[LM_MU] = sz[LM_RSTD] = d.T * sizeof(float);
  sz[LM_LOGITS] = (size_t)d.T * vrows * d.esz;
  sz[LM_COLSUM] = layernorm_bwd_scratch_bytes((int)d.T, (int)d.h);
  sz[LM_SPLITK] = c->dtype == PTDP_BF16 ? gemm_workspace_bytes() : 0;
  LmLayout L;
  size_t o = 0;
  for (int i = 0; i < LM_N; ++i) {
    L.off[i] = o;
    o += align256(sz[i]);
  }
  L.total = o;
  return L;
}
int lm_check(const ptdp_layer_cfg* cfg, int v0, int vrows) {
  const int rc = validate(cfg);
  if (rc != PTDP_OK) return rc;
  if (v0 < 0 || vrows <= 0 || vrows % 8 != 0 || (int64_t)v0 + vrows > 0x7fffffffll) return PTDP_E_INVALID_ARG;
  return PTDP_OK;
}
}  // namespace

size_t ptdp_lm_workspace_bytes(const ptdp_layer_cfg* cfg, int vocab_rows) {
  if (lm_check(cfg, 0, vocab_rows) != PTDP_OK) return 0;
  return lm_layout(cfg, vocab_rows).total;
}

int64_t ptdp_logit_flops_fwd(const ptdp_layer_cfg* cfg, int vocab_rows) {
  if (lm_check(cfg, 0, vocab_rows) != PTDP_OK) return -1;
  return 2ll * cfg->b * cfg->s * cfg->h * vocab_rows;
}

int ptdp_embedding_forward(const ptdp_layer_cfg* cfg, int vocab_first, int vocab_rows, const int32_t* tokens,
                           const void* e_word, const void* e_pos, void* x, int64_t microbatch, void* stream) {
  PTDP_TRY(lm_check(cfg, vocab_first, vocab_rows));
  if (!tokens || !e_word || !e_pos || !x) return PTDP_E_NULL_PTR;
  if (microbatch < 0) return PTDP_E_INVALID_ARG;
  return launch_embed_fwd(cfg->dtype, tokens, e_word, e_pos, x, cfg->s, cfg->b, cfg->h, vocab_first, vocab_rows,
                          cfg->p_hidden, dropout_key(cfg->seed, PTDP_EMBED_LAYER, 0, (uint64_t)microbatch),
                          (hipStream_t)stream);
}

int ptdp_embedding_backward(const ptdp_layer_cfg* cfg, int vocab_first, int vocab_rows, const int32_t* tokens,
                            const void* dx, float* d_e_word, float* d_e_pos, void* workspace, int64_t microbatch,
                            void* stream) {
  PTDP_TRY(lm_check(cfg, vocab_first, vocab_rows));
  if (!tokens || !dx || !d_e_word || !d_e_pos || !workspace) return PTDP_E_NULL_PTR;
  if (microbatch < 0) return PTDP_E_INVALID_ARG;
  const LmLayout L = lm_layout(cfg, vocab_rows);
  return launch_embed_bwd(cfg->dtype, tokens, dx, (char*)workspace + L.off[LM_DU], d_e_word, d_e_pos, cfg->s, cfg->b,
                          cfg->h, vocab_first, vocab_rows, cfg->p_hidden,
                          dropout_key(cfg->seed, PTDP_EMBED_LAYER, 0, (uint64_t)microbatch), (hipStream_t)stream);
}

int ptdp_lm_head_step(const ptdp_layer_cfg* cfg, int vocab_first, int vocab_rows, const void* y, const void* lnf_g,
                      const void* lnf_b, const void* e_word, const int32_t* targets, float loss_scale, float* loss,
                      float* token_loss, void* dy, float* d_lnf_g, float* d_lnf_b, float* d_e_word, void* workspace,
                      void* stream) {
  PTDP_TRY(lm_check(cfg, vocab_first, vocab_rows));
  if (!y || !lnf_g || !lnf_b || !e_word || !targets || !loss || !token_loss || !dy || !d_lnf_g || !d_lnf_b ||
      !d_e_word || !workspace)
    return PTDP_E_NULL_PTR;
  if (!(loss_scale == loss_scale) || std::isinf(loss_scale)) return PTDP_E_INVALID_ARG;
  const Dims d = dims_of(cfg);
  if (d.h > 8 * 512 * (cfg->dtype == PTDP_BF16 ? 8 : 4)) return PTDP_E_UNSUPPORTED;
  const LmLayout L = lm_layout(cfg, vocab_rows);
  char* W = (char*)workspace;
  auto wf = [&](int f) { return (void*)(W + L.off[f]); };
  hipStream_t st = (hipStream_t)stream;
  const int T = (int)d.T, h = (int)d.h, dt = cfg->dtype;
  void* sk = wf(LM_SPLITK);
  const size_t skb = L.total - L.off[LM_SPLITK];
  PTDP_TRY(launch_layernorm_fwd(dt, y, lnf_g, lnf_b, wf(LM_U), (float*)wf(LM_MU), (float*)wf(LM_RSTD), nullptr, T, h,
                                cfg->ln_eps, st));
  PTDP_TRY(launch_gemm(dt, PTDP_GEMM_NT, wf(LM_U), e_word, wf(LM_LOGITS), nullptr, T, vocab_rows, h, 0, 0, sk, skb, st));
  PTDP_TRY(launch_xent(dt, wf(LM_LOGITS), targets, token_loss, loss, T, vocab_rows, vocab_first, loss_scale / (float)T,
                       st));
  PTDP_TRY(launch_gemm(dt, PTDP_GEMM_NN, wf(LM_LOGITS), e_word, wf(LM_DU), nullptr, T, h, vocab_rows, 0, 0, sk, skb, st));
  PTDP_TRY(launch_gemm(dt, PTDP_GEMM_TN, wf(LM_LOGITS), wf(LM_U), d_e_word, nullptr, vocab_rows, h, T, 1, 1, sk, skb, st));
  PTDP_TRY(launch_layernorm_bwd(dt, wf(LM_DU), y, lnf_g, (const float*)wf(LM_MU), (const float*)wf(LM_RSTD), nullptr, dy,
                                d_lnf_g, d_lnf_b, wf(LM_COLSUM), T, h, st));
  return PTDP_OK;
}

// ------------------------------------------------------------------------- single-kernel exports
static int check_dtype(int dtype) { return (dtype == PTDP_F32 || dtype == PTDP_BF16) ? PTDP_OK : PTDP_E_INVALID_ARG; }
static int check_rw(int dtype, int rows, int width) {
  PTDP_TRY(check_dtype(dtype));
  if (rows < 0 || width <= 0 || width % 8 != 0) return PTDP_E_INVALID_ARG;
  return PTDP_OK;
}
static int check_ln_width(int dtype, int width) {
  return width > 8 * 512 * (dtype == PTDP_BF16 ? 8 : 4) ? PTDP_E_UNSUPPORTED : PTDP_OK;
}

int ptdp_layernorm_fwd(int dtype, const void* x, const void* gain, const void* bias, void* u, float* mu, float* rstd,
                       void* x_copy, int rows, int width, float eps, void* stream) {
  PTDP_TRY(check_rw(dtype, rows, width));
  PTDP_TRY(check_ln_width(dtype, width));
  if (!(eps > 0.f)) return PTDP_E_INVALID_ARG;
  if (!x || !gain || !bias || !u || !mu || !rstd) return PTDP_E_NULL_PTR;
  return launch_layernorm_fwd(dtype, x, gain, bias, u, mu, rstd, x_copy, rows, width, eps, (hipStream_t)stream);
}

int ptdp_layernorm_bwd(int dtype, const void* du, const void* x, const void* gain, const float* mu, const float* rstd,
                       const void* resid, void* dx, float* dgain, float* dbias, void* scratch, int rows, int width,
                       void* stream) {
  PTDP_TRY(check_rw(dtype, rows, width));
  PTDP_TRY(check_ln_width(dtype, width));
  if (!du || !x || !gain || !mu || !rstd || !dx || !dgain || !dbias || !scratch) return PTDP_E_NULL_PTR;
  return launch_layernorm_bwd(dtype, du, x, gain, mu, rstd, resid, dx, dgain, dbias, scratch, rows, width,
                              (hipStream_t)stream);
}

int ptdp_bias_gelu_fwd(int dtype, int gelu_mode, const void* z, const void* bias, void* g, int rows, int width,
                       void* stream) {
  PTDP_TRY(check_rw(dtype, rows, width));
  if (gelu_mode != PTDP_GELU_ERF && gelu_mode != PTDP_GELU_TANH) return PTDP_E_INVALID_ARG;
  if (!z || !bias || !g) return PTDP_E_NULL_PTR;
  return launch_bias_gelu_fwd(dtype, gelu_mode, z, bias, g, rows, width, (hipStream_t)stream);
}

int ptdp_bias_gelu_bwd(int dtype, int gelu_mode, const void* dg, const void* z, const void* bias, void* dz,
                       float* dbias, void* scratch, int rows, int width, void* stream) {
  PTDP_TRY(check_rw(dtype, rows, width));
  if (gelu_mode != PTDP_GELU_ERF && gelu_mode != PTDP_GELU_TANH) return PTDP_E_INVALID_ARG;
  if (!dg || !z || !bias || !dz || !dbias || !scratch) return PTDP_E_NULL_PTR;
  return launch_bias_gelu_bwd(dtype, gelu_mode, dg, z, bias, dz, dbias, scratch, rows, width, (hipStream_t)stream);
}

int ptdp_bias_dropout_add_fwd(int dtype, const void* in, const void* bias, const void* resid, void* out, int rows,
                              int width, float p, uint64_t seed, uint32_t layer, uint32_t site, uint64_t microbatch,
                              void* stream) {
  PTDP_TRY(check_rw(dtype, rows, width));
  if (!(p >= 0.f && p < 1.f) || site > 1) return PTDP_E_INVALID_ARG;
  if (!in || !bias || !resid || !out) return PTDP_E_NULL_PTR;
  return launch_bda_fwd(dtype, in, bias, resid, out, rows, width, p, dropout_key(seed, layer, site, microbatch),
                        (hipStream_t)stream);
}

int ptdp_bias_dropout_add_bwd(int dtype, const void* dout, void* din, float* dbias, void* scratch, int rows, int width,
                              float p, uint64_t seed, uint32_t layer, uint32_t site, uint64_t microbatch,
                              void* stream) {
  PTDP_TRY(check_rw(dtype, rows, width));
  if (!(p >= 0.f && p < 1.f) || site > 1 || dout == din) return PTDP_E_INVALID_ARG;
  if (!dout || !din || !dbias || !scratch) return PTDP_E_NULL_PTR;
  return launch_bda_bwd(dtype, dout, din, dbias, scratch, rows, width, p, dropout_key(seed, layer, site, microbatch),
                        (hipStream_t)stream);
}

int ptdp_bias_dropout_add_bwd_noalloc(int dtype, const void* dout, void* din, float* dbias, int rows, int width,
                                      float p, uint64_t seed, uint32_t layer, uint32_t site, uint64_t microbatch,
                                      void* stream) {
  PTDP_TRY(check_rw(dtype, rows, width));
  if (!(p >= 0.f && p < 1.f) || site > 1 || dout == din) return PTDP_E_INVALID_ARG;
  if (!dout || !din || !dbias) return PTDP_E_NULL_PTR;
  if (profiling_enabled()) return PTDP_E_STATE;   // profiling creates events: not for callers that may not allocate
  return launch_bda_bwd_static(dtype, dout, din, dbias, rows, width, p, dropout_key(seed, layer, site, microbatch),
                               (hipStream_t)stream);
}

size_t ptdp_noalloc_scratch_bytes(void) { return kStaticScratchBytes; }

size_t ptdp_colsum_scratch_bytes(int rows, int width) { return colsum_scratch_bytes(rows, width); }

size_t ptdp_layernorm_bwd_scratch_bytes(int rows, int width) { return layernorm_bwd_scratch_bytes(rows, width); }

size_t ptdp_gemm_workspace_bytes(void) { return gemm_workspace_bytes(); }

int ptdp_gemm_plan(int M, int N, int K, int out_f32, int accumulate, int has_bias, size_t workspace_bytes,
                   int* dp_columns, int* n_groups, int* group_tiles, int* group_parts) {
  if (!dp_columns || !n_groups || !group_tiles || !group_parts) return PTDP_E_NULL_PTR;
  if (M <= 0 || N <= 0 || K <= 0 || M % 8 || N % 8 || K % 8) return PTDP_E_INVALID_ARG;
  int cols = 0;
  gemm_plan_query(M, N, K, out_f32, accumulate, has_bias, workspace_bytes, &cols, n_groups, group_tiles, group_parts);
  *dp_columns = cols < (N + 255) / 256 ? cols * 256 : N;
  return PTDP_OK;
}

int ptdp_dropout_mask(uint8_t* keep, int64_t n, float p, uint64_t seed, uint32_t layer, uint32_t site,
                      uint64_t microbatch, void* stream) {
  if (n < 0 || !(p >= 0.f && p < 1.f) || site > 1) return PTDP_E_INVALID_ARG;
  if (!keep && n > 0) return PTDP_E_NULL_PTR;
  return launch_dropout_mask(keep, n, p, dropout_key(seed, layer, site, microbatch), (hipStream_t)stream);
}

int ptdp_gemm(int dtype, int mode, const void* A, const void* B, void* C, const void* bias, int M, int N, int K,
              int out_f32, int accumulate, void* workspace, size_t workspace_bytes, void* stream) {
  PTDP_TRY(check_dtype(dtype));
  if (mode != PTDP_GEMM_NN && mode != PTDP_GEMM_NT && mode != PTDP_GEMM_TN) return PTDP_E_INVALID_ARG;
  if (M < 0 || N < 0 || K < 0) return PTDP_E_INVALID_ARG;
  if (dtype == PTDP_BF16 && (M % 8 || N % 8 || K % 8)) return PTDP_E_INVALID_ARG;
  if (dtype == PTDP_BF16 && accumulate && !out_f32) return PTDP_E_INVALID_ARG;
  if (!A || !B || !C) return PTDP_E_NULL_PTR;
  if (!workspace) workspace_bytes = 0;
  return launch_gemm(dtype, mode, A, B, C, bias, M, N, K, out_f32, accumulate, workspace, workspace_bytes,
                     (hipStream_t)stream);
}

int ptdp_attn_fwd(int dtype, const void* qkv, void* ctx, float* lse, int s, int b, int heads, int dh, void* stream) {
  PTDP_TRY(check_dtype(dtype));
  if (s < 0 || b < 0 || heads < 0 || dh <= 0 || dh % 8 != 0) return PTDP_E_INVALID_ARG;
  if (!attn_dh_supported(dtype, dh)) return PTDP_E_UNSUPPORTED;
  if (!qkv || !ctx || !lse) return PTDP_E_NULL_PTR;
  return launch_attn_fwd(dtype, qkv, ctx, lse, s, b, heads, dh, nullptr, 1, (hipStream_t)stream);
}

int ptdp_attn_masked_fwd(int dtype, const void* qkv, const uint8_t* mask, void* ctx, float* lse, int s, int b, int heads,
                         int dh, void* stream) {
  PTDP_TRY(check_dtype(dtype));
  if (s < 0 || b < 0 || heads < 0 || dh <= 0 || dh % 8 != 0) return PTDP_E_INVALID_ARG;
  if (!attn_dh_supported(dtype, dh)) return PTDP_E_UNSUPPORTED;
  if (!qkv || !ctx || !lse) return PTDP_E_NULL_PTR;
  if (mask && ((uintptr_t)mask & 3)) return PTDP_E_INVALID_ARG;
  return launch_attn_fwd(dtype, qkv, ctx, lse, s, b, heads, dh, mask, 0, (hipStream_t)stream);
}

int ptdp_attn_bwd(int dtype, const void* qkv, const void* ctx, const float* lse, const void* dctx, void* dqkv,
                  float* delta, int s, int b, int heads, int dh, void* stream) {
  PTDP_TRY(check_dtype(dtype));
  if (s < 0 || b < 0 || heads < 0 || dh <= 0 || dh % 8 != 0) return PTDP_E_INVALID_ARG;
  if (!attn_dh_supported(dtype, dh)) return PTDP_E_UNSUPPORTED;
  if (!qkv || !ctx || !lse || !dctx || !dqkv || !delta) return PTDP_E_NULL_PTR;
  return launch_attn_bwd(dtype, qkv, ctx, lse, dctx, dqkv, delta, s, b, heads, dh, nullptr, 1, (hipStream_t)stream);
}

int ptdp_attn_masked_bwd(int dtype, const void* qkv, const uint8_t* mask, const void* ctx, const float* lse,
                         const void* dctx, void* dqkv, float* delta, int s, int b, int heads, int dh, void* stream) {
  PTDP_TRY(check_dtype(dtype));
  if (s < 0 || b < 0 || heads < 0 || dh <= 0 || dh % 8 != 0) return PTDP_E_INVALID_ARG;
  if (!attn_dh_supported(dtype, dh)) return PTDP_E_UNSUPPORTED;
  if (!qkv || !ctx || !lse || !dctx || !dqkv || !delta) return PTDP_E_NULL_PTR;
  if (mask && ((uintptr_t)mask & 3)) return PTDP_E_INVALID_ARG;
  return launch_attn_bwd(dtype, qkv, ctx, lse, dctx, dqkv, delta, s, b, heads, dh, mask, 0, (hipStream_t)stream);
}

// ----------------------------------------------------------------------------------- profiling
int ptdp_prof_enable(int on) {
  std::lock_guard<std::mutex> lock(g_prof_mu);
  if (on) {
    for (int i = 0; i < PTDP_K_NFAMILIES; ++i) g_totals[i] = ptdp_prof_entry{0.0, 0.0, 0};
    for (auto& r : g_open) {
      g_free_events.push_back(r.start);
      g_free_events.push_back(r.stop);
    }
    g_open.clear();
  }
  g_prof_on.store(on != 0, std::memory_order_relaxed);
  return PTDP_OK;
}

int ptdp_prof_collect(ptdp_prof_entry* out) {
  if (!out) return PTDP_E_NULL_PTR;
  std::lock_guard<std::mutex> lock(g_prof_mu);
  int rc = PTDP_OK;
  for (auto& r : g_open) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess)
      rc = PTDP_E_HIP;
    else {
      g_totals[r.family].ms += ms;
      g_totals[r.family].work += r.work;
      g_totals[r.family].launches += 1;
    }
    g_free_events.push_back(r.start);
    g_free_events.push_back(r.stop);
  }
  g_open.clear();
  for (int i = 0; i < PTDP_K_NFAMILIES; ++i) out[i] = g_totals[i];
  return rc;
}

const char* ptdp_prof_family_name(int family) {
  static const char* names[PTDP_K_NFAMILIES] = {"gemm_nn", "gemm_nt", "gemm_tn", "attn_fwd", "attn_bwd",
                                                "layernorm_fwd", "layernorm_bwd", "bias_gelu_fwd", "bias_gelu_bwd",
                                                "bias_dropout_add_fwd", "bias_dropout_add_bwd", "colsum", "other",
                                                "embedding", "loss"};
  return (family >= 0 && family < PTDP_K_NFAMILIES) ? names[family] : "?";
}

}  // extern "C"
