// C ABI of libcada: argument checking, workspace layout, initialisation and the per-step
// launch sequence of Algorithm 1 (declared and documented in cada.h).
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <new>
#include <vector>

#include "cada_internal.h"

namespace cada {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int ring_finalize(Ctx *c);

struct Prof {
  std::vector<hipEvent_t> ev;
  int64_t max_steps = 0;
  size_t used = 0;
};

void prof_mark(Ctx *c) {
  Prof *p = static_cast<Prof *>(c->prof);
  if (!p || p->used >= p->ev.size()) return;
  if (hipEventRecord(p->ev[p->used], c->stream) == hipSuccess) p->used += 1;
}

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Walks the workspace; with base == nullptr only sizes are computed.
struct Carver {
  char *base;
  size_t off = 0;
  template <typename T> T *take(size_t n) {
    T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
    off = align_up(off + n * sizeof(T));
    return p;
  }
};

struct Geometry {
  int vec;
  int n_col_chunks;
  int64_t chunk_cols;
  int n_lhs_part;
  int lhs_cap;              // slots reserved per worker (the single-pass logistic kernel needs 4 per workgroup)
  int n_ring_part, ring_cap;
  int64_t total_rows;
};

bool check_config(const cada_config *cfg, Geometry *g) {
  if (!cfg) { set_error("cfg is NULL"); return false; }
  if (cfg->M < 1 || cfg->M > 65535) { set_error("M must be in [1, 65535] (got %d)", cfg->M); return false; }
  if (cfg->p < 1) { set_error("p must be >= 1"); return false; }
  if (cfg->B < 1 || cfg->B > CADA_MAX_B) { set_error("B must be in [1, %d] (got %d)", CADA_MAX_B, cfg->B); return false; }
  if (cfg->d_max < 1 || cfg->d_max > CADA_MAX_DMAX) { set_error("d_max must be in [1, %d]", CADA_MAX_DMAX); return false; }
  if (cfg->D < 1) { set_error("D must be >= 1"); return false; }
  if (!(cfg->c >= 0.0)) { set_error("c must be >= 0"); return false; }
  if (!(cfg->beta1 >= 0.0 && cfg->beta1 < 1.0 && cfg->beta2 >= 0.0 && cfg->beta2 < 1.0)) { set_error("beta1, beta2 must be in [0, 1)"); return false; }
  if (!(cfg->eps >= 0.0)) { set_error("eps must be >= 0"); return false; }
  if (cfg->alpha_K0 < 0) { set_error("alpha_K0 must be >= 0"); return false; }
  if (cfg->rule < CADA_RULE_ALWAYS || cfg->rule > CADA_RULE_LAG) { set_error("rule must be one of CADA_RULE_* (got %d)", cfg->rule); return false; }
  if (cfg->server != CADA_SERVER_AMSGRAD && cfg->server != CADA_SERVER_SGD) { set_error("server must be one of CADA_SERVER_* (got %d)", cfg->server); return false; }
  if (cfg->model != CADA_MODEL_LOGREG && cfg->model != CADA_MODEL_MLP) { set_error("unknown model %d", cfg->model); return false; }
  if (cfg->path < CADA_PATH_AUTO || cfg->path > CADA_PATH_WHOLE_STEPS) { set_error("path must be one of CADA_PATH_* (got %d)", cfg->path); return false; }
  if (cfg->gradient_store != CADA_STORE_F32 && cfg->gradient_store != CADA_STORE_BF16) { set_error("gradient_store must be one of CADA_STORE_* (got %d)", cfg->gradient_store); return false; }
  if (cfg->single_pass_rows < 0 || cfg->single_pass_rows > 1 || cfg->single_pass_clusters < 0 || cfg->two_pass_group < 0) { set_error("negative tuning field"); return false; }
  if (!cfg->layer_dims) { set_error("layer_dims is NULL"); return false; }
  if (!cfg->n_samples) { set_error("n_samples is NULL"); return false; }
  if (cfg->trace_steps < 0) { set_error("trace_steps must be >= 0"); return false; }
  if (cfg->n_layers < 1 || cfg->n_layers > CADA_MAX_LAYERS) { set_error("n_layers must be in [1, %d]", CADA_MAX_LAYERS); return false; }
  int64_t p = 0;
  if (cfg->model == CADA_MODEL_LOGREG) {
    if (cfg->n_layers != 1) { set_error("LOGREG needs n_layers == 1"); return false; }
    p = cfg->layer_dims[0];
  } else {
    for (int l = 0; l < cfg->n_layers; ++l) {
      if (cfg->layer_dims[l] < 1 || cfg->layer_dims[l + 1] < 1) { set_error("layer_dims must be positive"); return false; }
      p += (int64_t)cfg->layer_dims[l] * cfg->layer_dims[l + 1] + cfg->layer_dims[l + 1];
    }
  }
  if (p != cfg->p) { set_error("p = %lld does not match the model (%lld parameters)", (long long)cfg->p, (long long)p); return false; }
  int64_t rows = 0;
  for (int m = 0; m < cfg->M; ++m) {
    if (cfg->n_samples[m] < 1) { set_error("n_samples[%d] must be >= 1", m); return false; }
    rows += cfg->n_samples[m];
  }
  g->total_rows = rows;
  // float4 access needs every row start, every p-vector and every chunk start 16-byte aligned.
  g->vec = (cfg->p % 4 == 0) ? 4 : 1;
  // pass 1: one column chunk per block, at most 8192 columns (8 iterations of 256 float4 lanes)
  g->chunk_cols = 8192;
  g->n_col_chunks = (int)((cfg->p + g->chunk_cols - 1) / g->chunk_cols);
  const int64_t per_block = (int64_t)kBlock * g->vec;
  g->n_lhs_part = (int)((cfg->p + per_block - 1) / per_block);
  // server kernel: one block per 256 coordinates, see cada_server.hip (the multi-step kernel of
  // cada_logreg_small.hip writes one partial per worker instead: room for either)
  g->n_ring_part = (int)((cfg->p + 255) / 256);
  g->ring_cap = g->n_ring_part > cfg->M ? g->n_ring_part : cfg->M;
  if (cfg->model == CADA_MODEL_MLP) g->n_lhs_part = mlp_lhs_slots(cfg);
  const int fused_slots = kFusedWaves * (int)((cfg->p + 2047) / 2048);
  g->lhs_cap = g->n_lhs_part > fused_slots ? g->n_lhs_part : fused_slots;
  return true;
}

// Lays out the common state.  Returns bytes used so far.
void carve_common(Carver &w, const cada_config *cfg, const Geometry &g, DevState *s, Ctx *c) {
  const size_t p = (size_t)cfg->p, M = (size_t)cfg->M;
  float *theta = w.take<float>(p), *theta_lo = w.take<float>(p), *h = w.take<float>(p), *v = w.take<float>(p);
  float *vhat = w.take<float>(p), *nabla = w.take<float>(p);
  // rows of the per-worker stores: the MLP path pads them to 16 bytes (its p is rarely a multiple of 4)
  const bool mlp = cfg->model == CADA_MODEL_MLP;
  const size_t ps = mlp ? (p + 3) / 4 * 4 : p, ps16 = (p + 7) / 8 * 8;
  float *gbuf = nullptr;
  uint16_t *gbuf16 = nullptr;
  if (cfg->gradient_store == CADA_STORE_BF16) gbuf16 = w.take<uint16_t>(2 * M * ps16);
  else gbuf = w.take<float>(2 * M * ps);
  float *hist = nullptr, *hist_lo = nullptr, *snap = nullptr, *snap_lo = nullptr, *dtl = nullptr;
  uint16_t *dtl16 = nullptr;
  if (cfg->rule == CADA_RULE_CADA2) {
    hist = w.take<float>((size_t)(cfg->D + 1) * ps);
    hist_lo = w.take<float>((size_t)(cfg->D + 1) * ps);
  } else if (cfg->rule == CADA_RULE_CADA1) {
    snap = w.take<float>(p);
    snap_lo = w.take<float>(p);
    if (mlp) dtl16 = w.take<uint16_t>(2 * M * ps16);
    else dtl = w.take<float>(2 * M * ps);
  }
  int32_t *tau = w.take<int32_t>(M), *sel = w.take<int32_t>(M);
  float *lhs = w.take<float>(M);
  float *lhs_part = w.take<float>(M * (size_t)g.lhs_cap);
  uint8_t *mask = w.take<uint8_t>(M);
  float *ring = w.take<float>((size_t)cfg->d_max);
  float *ring_part = w.take<float>((size_t)g.ring_cap);
  uint64_t *uploads = w.take<uint64_t>(1);
  uint32_t *n_up = w.take<uint32_t>(2);
  uint32_t *err = w.take<uint32_t>(1);
  int64_t *row_off = w.take<int64_t>(M + 1);
  const size_t T = (size_t)cfg->trace_steps;
  uint8_t *t_mask = w.take<uint8_t>(T * M), *t_own = w.take<uint8_t>(T * M);
  float *t_lhs = w.take<float>(T * M), *t_rhs = w.take<float>(T);
  int32_t *t_tau = w.take<int32_t>(T * M);
  double *eval_part = w.take<double>(M * (size_t)kEvalBlocks * 2), *eval_acc = w.take<double>(M * 2);
  int32_t *eval_idx = w.take<int32_t>(M * (size_t)cfg->B);
  float *zpart = nullptr;
  unsigned long long *post = nullptr;
  float *tail = nullptr;
  uint32_t *small_bar = nullptr;
  unsigned char *small_args = nullptr;
  if (cfg->model == CADA_MODEL_LOGREG) {
    zpart = w.take<float>(M * (size_t)cfg->B * (size_t)g.n_col_chunks * 2);
    post = w.take<unsigned long long>(kFusedPostWords);
    if (cfg->p >= 8192 && cfg->p % 4 == 0) tail = w.take<float>(kFusedTailFloatsPerP * (size_t)cfg->p);   // (shapes the single-pass kernel serves)
    small_bar = w.take<uint32_t>(64 + 2 * M);      // (a cache line kept free,) then the tagged decision words of the last two steps [2][M]
    small_args = w.take<unsigned char>(kSmallArgsBytes);
  }
  if (!s) return;
  c->fused_post = post;
  c->fused_tail = tail;
  c->eval_part = eval_part; c->eval_acc = eval_acc; c->eval_idx = eval_idx;
  c->small_bar = small_bar;
  c->small_args = small_args;
  s->theta = theta; s->theta_lo = theta_lo; s->hist_lo = hist_lo; s->snap_lo = snap_lo; s->h = h; s->v = v; s->vhat = vhat; s->nabla = nabla;
  s->gbuf = gbuf; s->gbuf16 = gbuf16; s->hist = hist; s->snap = snap; s->dtl = dtl; s->dtl16 = dtl16;
  s->ps = (int64_t)ps; s->ps16 = (int64_t)ps16;
  s->tau = tau; s->sel = sel; s->lhs = lhs; s->lhs_part = lhs_part; s->mask = mask;
  s->ring = ring; s->ring_part = ring_part; s->uploads = uploads; s->n_up = n_up; s->err = err;
  s->row_off = row_off;
  s->t_mask = t_mask; s->t_own = t_own; s->t_lhs = t_lhs; s->t_rhs = t_rhs; s->t_tau = t_tau;
  s->trace_steps = cfg->trace_steps;
  c->zpart = zpart;
}

__global__ void k_fill_i32(int32_t *p, int32_t v, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// dst[r][i] = src[i] for r < reps, rows `stride` floats apart
__global__ void k_broadcast_rows(float *dst, const float *src, int64_t p, int64_t reps, int64_t stride) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= p) return;
  const float v = src[i];
  for (int64_t r = 0; r < reps; ++r) dst[r * stride + i] = v;
}

// out[m][i] = gbuf[sel[m]][m][i] (as float32, whatever the store holds)
__global__ void k_gather_stored(const DevState s, float *out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int m = blockIdx.y;
  if (i >= s.p) return;
  if (s.gbuf16) out[(int64_t)m * s.p + i] = bf2f(s.gbuf16[((int64_t)s.sel[m] * s.M + m) * s.ps16 + i]);
  else out[(int64_t)m * s.p + i] = s.gbuf[((int64_t)s.sel[m] * s.M + m) * s.ps + i];
}

// cada_set_state, [p]-sized part: iterate, moments, and the reference point that is one vector
// (CADA1: the snapshot; CADA2: slot k mod R of the retained iterates holds theta^k itself).
struct SetStateArgs {
  DevState s;
  cada_state_in in;
};

__global__ __launch_bounds__(kBlock) void k_set_vectors(const SetStateArgs a) {
  const DevState &s = a.s;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < s.p; i += (int64_t)gridDim.x * kBlock) {
    const float th = a.in.theta[i], tl = a.in.theta_lo ? a.in.theta_lo[i] : 0.f;
    s.theta[i] = th; s.theta_lo[i] = tl;
    s.h[i] = a.in.h[i]; s.vhat[i] = a.in.vhat[i]; s.v[i] = a.in.vhat[i];
    if (s.rule == CADA_RULE_CADA2) {
      const int64_t slot = a.in.k % s.R;
      s.hist[slot * s.ps + i] = th; s.hist_lo[slot * s.ps + i] = tl;
    } else if (s.rule == CADA_RULE_CADA1) {
      s.snap[i] = a.in.reference[i];
      s.snap_lo[i] = a.in.reference_lo ? a.in.reference_lo[i] : 0.f;
    }
  }
}

// cada_set_state, [M, p]-sized part; grid (blocks, M).  Stored gradients (and CADA1's stored
// innovations) go to buffer 0 of worker m, which the small kernel below makes the selected one.
// CADA2: theta-hat_m goes to the slot of theta^{k - tau_m}; among workers with the same delay
// the first one writes it.
__global__ __launch_bounds__(kBlock) void k_set_rows(const SetStateArgs a) {
  const DevState &s = a.s;
  __shared__ int dup;
  const int m = blockIdx.y;
  const int64_t row = (int64_t)m * s.p;
  int64_t slot = -1;
  if (s.rule == CADA_RULE_CADA2) {
    const int32_t tau_m = min(max(a.in.tau[m], 1), s.D);
    if (threadIdx.x == 0) dup = 0;
    __syncthreads();
    for (int j = threadIdx.x; j < m; j += kBlock)
      if (min(max(a.in.tau[j], 1), s.D) == tau_m) dup = 1;       // (every writer writes the same value)
    __syncthreads();
    if (!dup) {
      slot = (a.in.k - tau_m) % s.R;
      if (slot < 0) slot += s.R;
    }
  }
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < s.p; i += (int64_t)gridDim.x * kBlock) {
    if (s.gbuf16) s.gbuf16[(int64_t)m * s.ps16 + i] = f2bf(a.in.stored_gradients[row + i]);
    else s.gbuf[(int64_t)m * s.ps + i] = a.in.stored_gradients[row + i];
    if (s.rule == CADA_RULE_CADA1) {
      if (s.dtl16) s.dtl16[(int64_t)m * s.ps16 + i] = f2bf(a.in.stored_innovations[row + i]);
      else s.dtl[(int64_t)m * s.ps + i] = a.in.stored_innovations[row + i];
    }
    if (slot >= 0) {
      s.hist[slot * s.ps + i] = a.in.reference[row + i];
      s.hist_lo[slot * s.ps + i] = a.in.reference_lo ? a.in.reference_lo[row + i] : 0.f;
    }
  }
}

// cada_set_state, the small pieces: delays, buffer selectors, the squared steps (the newest one
// is kept as partial sums that the next rule evaluation adds up: all of it goes to the first), counters.
__global__ __launch_bounds__(kBlock) void k_set_small(const SetStateArgs a, int n_ring_cap) {
  const DevState &s = a.s;
  for (int m = threadIdx.x; m < s.M; m += kBlock) {
    const int32_t t = a.in.tau[m];
    if (t < 1 || t > s.D) atomicOr(s.err, 4u);
    s.tau[m] = min(max(t, 1), s.D);
    s.sel[m] = 0;
  }
  for (int j = threadIdx.x; j < s.d_max; j += kBlock) s.ring[j] = a.in.ring[j];
  const float newest = a.in.k > 0 ? a.in.ring[(a.in.k - 1) % s.d_max] : 0.f;
  for (int i = threadIdx.x; i < n_ring_cap; i += kBlock) s.ring_part[i] = i == 0 ? newest : 0.f;
  if (threadIdx.x == 0) { *s.uploads = a.in.uploads_total; s.n_up[0] = 0u; s.n_up[1] = 0u; }
}

#define HIP_TRY(expr)                                                        \
  do {                                                                       \
    hipError_t e_ = (expr);                                                  \
    if (e_ != hipSuccess) {                                                  \
      set_error("%s failed: %s", #expr, hipGetErrorString(e_));              \
      return CADA_EHIP;                                                      \
    }                                                                        \
  } while (0)

}  // namespace
}  // namespace cada

using namespace cada;

// The bf16 gradient store exists on the MLP path, for the rules whose left-hand side does not read the store.
static bool store_supported(const cada_config *cfg) {
  if (cfg->gradient_store == CADA_STORE_F32) return true;
  if (cfg->model != CADA_MODEL_MLP) { set_error("gradient_store = CADA_STORE_BF16 is implemented for the MLP model only"); return false; }
  if (cfg->rule == CADA_RULE_LAG) { set_error("gradient_store = CADA_STORE_BF16: the stochastic LAG rule compares stored gradients themselves and keeps them in float32"); return false; }
  return true;
}

struct cada_ctx {
  Ctx c;
  std::vector<int64_t> row_off_host;
};

extern "C" {

const char *cada_last_error(void) { return g_err; }

size_t cada_workspace_bytes(const cada_config *cfg) {
  Geometry g;
  if (!check_config(cfg, &g) || !store_supported(cfg)) return 0;
  Carver w{nullptr};
  carve_common(w, cfg, g, nullptr, nullptr);
  size_t total = w.off;
  if (cfg->model == CADA_MODEL_MLP) {
    const size_t extra = mlp_workspace_bytes(cfg, g.total_rows);
    if (extra == 0) return 0;
    total += extra;
  }
  return total;
}

int cada_init(const cada_config *cfg, const float *theta0, cada_ctx **out) {
  if (!out) { set_error("out is NULL"); return CADA_EINVAL; }
  *out = nullptr;
  Geometry g;
  if (!check_config(cfg, &g)) return CADA_EINVAL;
  if (!store_supported(cfg)) return CADA_EUNSUPPORTED;
  if (!theta0) { set_error("theta0 is NULL"); return CADA_EINVAL; }
  if (!cfg->X || !cfg->y) { set_error("X and y must be device pointers"); return CADA_EINVAL; }
  if (!cfg->workspace) { set_error("workspace is NULL"); return CADA_EWORKSPACE; }
  if (reinterpret_cast<uintptr_t>(cfg->workspace) % kAlign != 0) { set_error("workspace must be %zu-byte aligned", kAlign); return CADA_EWORKSPACE; }
  if (g.vec == 4 && reinterpret_cast<uintptr_t>(cfg->X) % 16 != 0) g.vec = 1;
  if (cfg->model == CADA_MODEL_MLP) g.vec = 4;      // (its rows are padded to 16 bytes; X is read through copies of its own)
  const size_t need = cada_workspace_bytes(cfg);
  if (need == 0) return CADA_EINVAL;
  if (cfg->workspace_bytes < need) {
    set_error("workspace too small: %zu bytes given, %zu needed", cfg->workspace_bytes, need);
    return CADA_EWORKSPACE;
  }
  cada_ctx *h = new (std::nothrow) cada_ctx();
  if (!h) { set_error("out of host memory"); return CADA_EINVAL; }
  Ctx *c = &h->c;
  memset(c, 0, sizeof(Ctx));
  DevState &s = c->s;
  c->stream = static_cast<hipStream_t>(cfg->stream);
  c->model = cfg->model;
  c->gemm_dtype = cfg->gemm_dtype;
  c->n_layers = cfg->n_layers;
  for (int l = 0; l <= cfg->n_layers; ++l) c->dims[l] = cfg->layer_dims[l];
  c->vec = g.vec;
  c->n_col_chunks = g.n_col_chunks;
  c->chunk_cols = g.chunk_cols;
  c->ws_bytes = need;
  c->ring_cap = g.ring_cap;
  c->force_resum = 1;
  c->ws_base = cfg->workspace;
  c->logreg_group = cfg->two_pass_group > 0 ? cfg->two_pass_group : 0;
  Carver w{static_cast<char *>(cfg->workspace)};
  carve_common(w, cfg, g, &s, c);
  s.X = cfg->X; s.y = cfg->y;
  s.M = cfg->M; s.B = cfg->B; s.d_max = cfg->d_max; s.D = cfg->D; s.R = cfg->D + 1; s.rule = cfg->rule; s.server_sgd = cfg->server == CADA_SERVER_SGD;
  s.n_lhs_part = g.n_lhs_part; s.n_ring_part = g.n_ring_part;
  s.p = cfg->p; s.k = 0;
  s.alpha0 = cfg->alpha; s.alpha_K0 = cfg->alpha_K0;
  s.alpha = (float)cfg->alpha; s.beta1 = (float)cfg->beta1; s.beta2 = (float)cfg->beta2;
  s.omb1 = (float)(1.0 - cfg->beta1); s.omb2 = (float)(1.0 - cfg->beta2);
  s.eps = (float)cfg->eps; s.lam = (float)cfg->lambda_l2; s.c = cfg->c;
  if (cfg->model == CADA_MODEL_LOGREG) {
    // the requested path first; a request that the shape does not allow falls back to the others
    if (cfg->path == CADA_PATH_WHOLE_STEPS && small_plan(c, cfg)) s.n_ring_part = cfg->M;
    else if (cfg->path != CADA_PATH_TWO_PASS && fused_plan(c, cfg)) s.n_lhs_part = kFusedWaves * c->fused_Q;
    else if (cfg->path == CADA_PATH_AUTO && small_plan(c, cfg)) s.n_ring_part = cfg->M;
    if (c->small) {
      c->n_phases = 1; c->phase_names[0] = "logreg_whole_steps";
    } else if (c->fused && c->fused_tail_f > 0) {
      c->n_phases = 4; c->phase_names[0] = "logreg_single_pass"; c->phase_names[1] = "logreg_split_round_sum";
      c->phase_names[2] = "rule"; c->phase_names[3] = "server_update";
    } else if (c->fused) {
      c->n_phases = 3; c->phase_names[0] = "logreg_single_pass"; c->phase_names[1] = "rule"; c->phase_names[2] = "server_update";
    } else {
      // (the two passes of a group of workers follow each other, group after group: one phase)
      c->n_phases = 3; c->phase_names[0] = "logreg_two_pass"; c->phase_names[1] = "rule"; c->phase_names[2] = "server_update";
    }
  }
  if (cfg->model == CADA_MODEL_MLP) {
    size_t off = w.off;
    const int rc = mlp_plan(c, cfg, static_cast<char *>(cfg->workspace), &off, g.total_rows);
    if (rc != CADA_OK) { delete h; return rc; }
  }

  h->row_off_host.resize((size_t)cfg->M + 1);
  h->row_off_host[0] = 0;
  for (int m = 0; m < cfg->M; ++m) h->row_off_host[m + 1] = h->row_off_host[m] + cfg->n_samples[m];

  hipStream_t st = c->stream;
  const size_t p = (size_t)s.p, M = (size_t)s.M;
  auto fail = [&](hipError_t e, const char *what) {
    set_error("%s failed: %s", what, hipGetErrorString(e));
    mlp_free(c);
    small_free(c);
    delete h;
    return CADA_EHIP;
  };
  hipError_t e;
  // whole workspace to zero, then the non-zero pieces
  if ((e = hipMemsetAsync(cfg->workspace, 0, need, st)) != hipSuccess) return fail(e, "hipMemsetAsync(workspace)");
  if ((e = hipMemcpyAsync(s.theta, theta0, p * sizeof(float), hipMemcpyDeviceToDevice, st)) != hipSuccess) return fail(e, "copy theta0");
  if ((e = hipMemcpyAsync(const_cast<int64_t *>(s.row_off), h->row_off_host.data(), (M + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st)) != hipSuccess) return fail(e, "copy row offsets");
  const int tb = 256;
  hipLaunchKernelGGL(k_fill_i32, dim3((unsigned)((M + tb - 1) / tb)), dim3(tb), 0, st, s.tau, (int32_t)s.D, (int64_t)M);
  const unsigned pb = (unsigned)((p + tb - 1) / tb);
  if (s.rule == CADA_RULE_CADA2)
    hipLaunchKernelGGL(k_broadcast_rows, dim3(pb), dim3(tb), 0, st, s.hist, theta0, (int64_t)p, (int64_t)s.R, s.ps);
  else if (s.rule == CADA_RULE_CADA1)
    hipLaunchKernelGGL(k_broadcast_rows, dim3(pb), dim3(tb), 0, st, s.snap, theta0, (int64_t)p, (int64_t)1, (int64_t)p);
  if ((e = hipGetLastError()) != hipSuccess) return fail(e, "init kernels");
  if (cfg->model == CADA_MODEL_MLP) {
    const int rc = mlp_init_state(c, theta0);
    if (rc != CADA_OK) { mlp_free(c); delete h; return rc; }
  } else {
    int rc = logreg_init(c);
    if (rc == CADA_OK) rc = eval_scratch_init();
    if (rc == CADA_OK) rc = small_publish_args(c);
    if (rc != CADA_OK) { small_free(c); delete h; return rc; }
  }
  *out = h;
  return CADA_OK;
}

int cada_step(cada_ctx *ctx, const int32_t *idx, const uint8_t *replay) {
  if (!ctx) { set_error("ctx is NULL"); return CADA_EINVAL; }
  if (!idx) { set_error("idx is NULL"); return CADA_EINVAL; }
  Ctx *c = &ctx->c;
  if (c->small) {
    const int rs = small_steps(c, idx, replay, 1);
    if (rs == CADA_OK) c->k += 1;
    return rs;
  }
  int rc = (c->model != CADA_MODEL_LOGREG) ? mlp_gradients(c, idx)
           : (c->fused ? logreg_gradients_fused(c, idx) : logreg_gradients(c, idx));
  if (rc != CADA_OK) return rc;
  rc = rule_and_server(c, replay);
  if (rc != CADA_OK) return rc;
  c->k += 1;
  return CADA_OK;
}

int cada_run(cada_ctx *ctx, const int32_t *idx_sched, const uint8_t *replay_sched, int64_t n_steps) {
  if (!ctx) { set_error("ctx is NULL"); return CADA_EINVAL; }
  if (n_steps < 0) { set_error("n_steps must be >= 0"); return CADA_EINVAL; }
  if (n_steps > 0 && !idx_sched) { set_error("idx_sched is NULL"); return CADA_EINVAL; }
  const int64_t M = ctx->c.s.M, B = ctx->c.s.B;
  if (ctx->c.small && n_steps > 0) {      // all n_steps iterations in one launch
    const int rs = small_steps(&ctx->c, idx_sched, replay_sched, n_steps);
    if (rs == CADA_OK) ctx->c.k += n_steps;
    return rs;
  }
  for (int64_t i = 0; i < n_steps; ++i) {
    const int rc = cada_step(ctx, idx_sched + i * M * B, replay_sched ? replay_sched + i * M : nullptr);
    if (rc != CADA_OK) return rc;
  }
  return CADA_OK;
}

int cada_run_replicas(cada_ctx *const *ctxs, int32_t n_replicas, const int32_t *const *idx_scheds,
                      const uint8_t *const *replay_scheds, int64_t n_steps) {
  if (!ctxs || !idx_scheds) { set_error("ctxs/idx_scheds is NULL"); return CADA_EINVAL; }
  if (n_replicas < 1 || n_replicas > CADA_MAX_REPLICAS) { set_error("n_replicas must be 1..%d", CADA_MAX_REPLICAS); return CADA_EINVAL; }
  if (n_steps < 0) { set_error("n_steps must be >= 0"); return CADA_EINVAL; }
  if (n_steps == 0) return CADA_OK;
  Ctx *cs[CADA_MAX_REPLICAS];
  for (int r = 0; r < n_replicas; ++r) {
    if (!ctxs[r] || !idx_scheds[r]) { set_error("replica %d: ctx or idx_sched is NULL", r); return CADA_EINVAL; }
    cs[r] = &ctxs[r]->c;
    for (int q = 0; q < r; ++q)
      if (cs[q] == cs[r]) { set_error("replica %d: the same context twice", r); return CADA_EINVAL; }
    if (!cs[r]->small) { set_error("replica %d does not run whole iterations in one launch (initialise a logistic workload with path = CADA_PATH_WHOLE_STEPS)", r); return CADA_EUNSUPPORTED; }
    const DevState &a = cs[0]->s, &b = cs[r]->s;
    if (a.M != b.M || a.p != b.p || a.B != b.B || a.rule != b.rule || cs[0]->stream != cs[r]->stream) {
      set_error("replica %d differs from replica 0 in M, p, B, rule or stream", r);
      return CADA_EINVAL;
    }
  }
  const int rc = small_steps_replicas(cs, n_replicas, idx_scheds, replay_scheds, n_steps);
  if (rc == CADA_OK)
    for (int r = 0; r < n_replicas; ++r) cs[r]->k += n_steps;
  return rc;
}

int cada_get_state(cada_ctx *ctx, cada_state *out) {
  if (!ctx || !out) { set_error("ctx/out is NULL"); return CADA_EINVAL; }
  Ctx *c = &ctx->c;
  const int rc = ring_finalize(c);   // fold the last step's squared step into the ring
  if (rc != CADA_OK) return rc;
  const DevState &s = c->s;
  out->theta = s.theta; out->theta_lo = s.theta_lo; out->h = s.h; out->v = s.v; out->vhat = s.vhat; out->nabla = s.nabla;
  out->tau = s.tau; out->ring = s.ring; out->mask = s.mask; out->lhs = s.lhs;
  out->uploads_total = s.uploads; out->error_flags = s.err;
  out->k = c->k; out->trace_steps = s.trace_steps;
  out->trace_mask = s.t_mask; out->trace_own_mask = s.t_own; out->trace_lhs = s.t_lhs;
  out->trace_rhs = s.t_rhs; out->trace_tau = s.t_tau;
  return CADA_OK;
}

int cada_copy_stored_gradients(cada_ctx *ctx, float *out) {
  if (!ctx || !out) { set_error("ctx/out is NULL"); return CADA_EINVAL; }
  Ctx *c = &ctx->c;
  const int tb = 256;
  hipLaunchKernelGGL(k_gather_stored, dim3((unsigned)((c->s.p + tb - 1) / tb), c->s.M), dim3(tb), 0, c->stream, c->s, out);
  HIP_TRY(hipGetLastError());
  return CADA_OK;
}

int cada_set_state(cada_ctx *ctx, const cada_state_in *in) {
  if (!ctx || !in) { set_error("ctx/in is NULL"); return CADA_EINVAL; }
  Ctx *c = &ctx->c;
  const DevState &s = c->s;
  if (in->k < 0) { set_error("cada_set_state: k must be >= 0"); return CADA_EINVAL; }
  if (!in->theta || !in->h || !in->vhat || !in->stored_gradients || !in->tau || !in->ring) {
    set_error("cada_set_state: theta, h, vhat, stored_gradients, tau and ring are required");
    return CADA_EINVAL;
  }
  if ((s.rule == CADA_RULE_CADA1 || s.rule == CADA_RULE_CADA2) && !in->reference) {
    set_error("cada_set_state: reference is required for the CADA rules");
    return CADA_EINVAL;
  }
  if (s.rule == CADA_RULE_CADA1 && !in->stored_innovations) {
    set_error("cada_set_state: stored_innovations is required for CADA1");
    return CADA_EINVAL;
  }
  SetStateArgs a;
  a.s = s;
  a.in = *in;
  const unsigned pb = (unsigned)std::min<int64_t>((s.p + kBlock - 1) / kBlock, 4096);
  hipLaunchKernelGGL(k_set_vectors, dim3(pb), dim3(kBlock), 0, c->stream, a);
  hipLaunchKernelGGL(k_set_rows, dim3(std::min(pb, 1024u), (unsigned)s.M), dim3(kBlock), 0, c->stream, a);
  hipLaunchKernelGGL(k_set_small, dim3(1), dim3(kBlock), 0, c->stream, a, c->ring_cap);
  HIP_TRY(hipGetLastError());
  c->k = in->k;
  c->force_resum = 1;       // (the aggregate of the step before is not part of the state handed over)
  return CADA_OK;
}

int cada_eval(cada_ctx *ctx, double *out) {
  if (!ctx || !out) { set_error("ctx/out is NULL"); return CADA_EINVAL; }
  Ctx *c = &ctx->c;
  return c->model == CADA_MODEL_LOGREG ? logreg_eval(c, out) : mlp_eval(c, out);
}

int cada_eval_noalloc(cada_ctx *ctx, double *out) {
  if (!ctx || !out) { set_error("ctx/out is NULL"); return CADA_EINVAL; }
  Ctx *c = &ctx->c;
  if (c->model != CADA_MODEL_LOGREG) {
    set_error("cada_eval_noalloc serves the logistic model: the MLP evaluation stages a chunk's activations, far more than its fixed scratch array");
    return CADA_EUNSUPPORTED;
  }
  return logreg_eval_noalloc(c, out);
}

namespace {
struct CheckpointHeader {          // in front of the workspace image
  uint64_t magic, ws_bytes;
  int64_t k, p;
  int32_t M, B, rule, model, D, d_max, server_sgd;
  uint32_t fused_seq, small_seq;
  int32_t force_resum;
};
static_assert(sizeof(CheckpointHeader) <= 128, "checkpoint header");
constexpr uint64_t kCheckpointMagic = 0x43414441434b5031ull;   // "CADACKP1"
constexpr size_t kCheckpointHeaderBytes = 128;

CheckpointHeader header_of(const Ctx *c) {
  CheckpointHeader h{};
  h.magic = kCheckpointMagic; h.ws_bytes = c->ws_bytes; h.k = c->k; h.p = c->s.p;
  h.M = c->s.M; h.B = c->s.B; h.rule = c->s.rule; h.model = c->model; h.D = c->s.D; h.d_max = c->s.d_max;
  h.server_sgd = c->s.server_sgd; h.fused_seq = c->fused_seq; h.small_seq = c->small_seq;
  h.force_resum = c->force_resum;
  return h;
}
}  // namespace

size_t cada_checkpoint_bytes(cada_ctx *ctx) { return ctx ? kCheckpointHeaderBytes + ctx->c.ws_bytes : 0; }

int cada_checkpoint_save(cada_ctx *ctx, void *dst) {
  if (!ctx || !dst) { set_error("ctx/dst is NULL"); return CADA_EINVAL; }
  Ctx *c = &ctx->c;
  const CheckpointHeader h = header_of(c);
  HIP_TRY(hipMemcpyAsync(static_cast<char *>(dst) + kCheckpointHeaderBytes, c->ws_base, c->ws_bytes, hipMemcpyDeviceToDevice, c->stream));
  HIP_TRY(hipMemcpyAsync(dst, &h, sizeof(h), hipMemcpyHostToDevice, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));     // h lives on this frame
  return CADA_OK;
}

int cada_checkpoint_load(cada_ctx *ctx, const void *src) {
  if (!ctx || !src) { set_error("ctx/src is NULL"); return CADA_EINVAL; }
  Ctx *c = &ctx->c;
  CheckpointHeader h{};
  HIP_TRY(hipMemcpyAsync(&h, src, sizeof(h), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));
  const CheckpointHeader mine = header_of(c);
  if (h.magic != kCheckpointMagic) { set_error("not a checkpoint block"); return CADA_EINVAL; }
  if (h.ws_bytes != mine.ws_bytes || h.p != mine.p || h.M != mine.M || h.B != mine.B || h.rule != mine.rule ||
      h.model != mine.model || h.D != mine.D || h.d_max != mine.d_max || h.server_sgd != mine.server_sgd) {
    set_error("checkpoint was saved with a different configuration");
    return CADA_EINVAL;
  }
  HIP_TRY(hipMemcpyAsync(c->ws_base, static_cast<const char *>(src) + kCheckpointHeaderBytes, c->ws_bytes, hipMemcpyDeviceToDevice, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));
  c->k = h.k;
  c->fused_seq = h.fused_seq;
  c->small_seq = h.small_seq;
  c->force_resum = h.force_resum;
  // (the image holds the saving context's launch arguments, which point into its workspace)
  const int rc = small_publish_args(c);
  if (rc != CADA_OK) return rc;
  HIP_TRY(hipStreamSynchronize(c->stream));
  return CADA_OK;
}

int cada_profile_phases(cada_ctx *ctx) { return ctx ? ctx->c.n_phases : 0; }

const char *cada_profile_phase_name(cada_ctx *ctx, int phase) {
  if (!ctx || phase < 0 || phase >= ctx->c.n_phases) return "";
  return ctx->c.phase_names[phase];
}

static void prof_drop(Ctx *c) {
  Prof *p = static_cast<Prof *>(c->prof);
  if (!p) return;
  for (hipEvent_t e : p->ev) (void)hipEventDestroy(e);
  delete p;
  c->prof = nullptr;
}

int cada_profile_begin(cada_ctx *ctx, int64_t max_steps) {
  if (!ctx || max_steps < 1 || max_steps > (1 << 20)) { set_error("cada_profile_begin: bad arguments"); return CADA_EINVAL; }
  Ctx *c = &ctx->c;
  prof_drop(c);
  Prof *p = new (std::nothrow) Prof();
  if (!p) { set_error("out of host memory"); return CADA_EINVAL; }
  p->max_steps = max_steps;
  p->ev.resize((size_t)max_steps * (size_t)(c->n_phases + 1));
  for (size_t i = 0; i < p->ev.size(); ++i) {
    const hipError_t e = hipEventCreate(&p->ev[i]);
    if (e != hipSuccess) {
      p->ev.resize(i);
      c->prof = p;
      prof_drop(c);
      set_error("hipEventCreate failed: %s", hipGetErrorString(e));
      return CADA_EHIP;
    }
  }
  c->prof = p;
  return CADA_OK;
}

int cada_profile_end(cada_ctx *ctx, double *ms_out, int n_out, int64_t *steps_out) {
  if (!ctx || !ms_out || !steps_out) { set_error("cada_profile_end: NULL argument"); return CADA_EINVAL; }
  Ctx *c = &ctx->c;
  Prof *p = static_cast<Prof *>(c->prof);
  if (!p) { set_error("profiling is not active"); return CADA_EINVAL; }
  if (n_out < c->n_phases) { set_error("ms_out too small"); return CADA_EINVAL; }
  const size_t per = (size_t)c->n_phases + 1;
  const size_t steps = p->used / per;
  for (int i = 0; i < n_out; ++i) ms_out[i] = 0.0;
  int rc = CADA_OK;
  if (steps > 0) {
    hipError_t e = hipEventSynchronize(p->ev[steps * per - 1]);
    for (size_t s = 0; s < steps && e == hipSuccess; ++s)
      for (int ph = 0; ph < c->n_phases && e == hipSuccess; ++ph) {
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, p->ev[s * per + ph], p->ev[s * per + ph + 1]);
        ms_out[ph] += ms;
      }
    if (e != hipSuccess) { set_error("profiling events: %s", hipGetErrorString(e)); rc = CADA_EHIP; }
  }
  *steps_out = (int64_t)steps;
  prof_drop(c);
  return rc;
}

void cada_destroy(cada_ctx *ctx) {
  if (!ctx) return;
  prof_drop(&ctx->c);
  mlp_free(&ctx->c);
  small_free(&ctx->c);
  delete ctx;
}

}  // extern "C"
