// Host side of the C ABI declared in include/ls.h: argument validation, workspace layout,
// program set-up and launches of the persistent kernel.  No device memory is allocated here;
// everything lives in the caller's workspace.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/ls.h"
#include "ls_internal.h"

extern "C" int ls_launch_program(const LsKParams* p, int dtype_is_bf16, int grid, hipStream_t stream);
extern "C" int ls_kernel_setup(int dtype_is_bf16, int hd, int* max_blocks_per_cu);
extern "C" int ls_launch_copy(const void* src, void* dst, size_t bytes, hipStream_t stream);
extern "C" int ls_launch_read(const void* src, size_t bytes, void* sink, int workgroups, hipStream_t stream);
extern "C" int ls_prefill_layers(const LsPfParams* p, const LsLayerW* host_layers, int pos0, int M, hipStream_t s);
extern "C" int ls_prefill_finish(const LsPfParams* p, int last_row, hipStream_t s);
extern "C" int ls_static_scratch_ptr(void** ptr);

namespace {

struct Layout {
  size_t layers, rope_cos, rope_sin, kcache, vcache, xbuf, ssq, qbuf, obuf, actbuf, attn_part, attn_cnt, cand, bar,
      state, x_pf, a_pf, q_pf, o_pf, act_pf, total;
  int pf_rows;
};

constexpr int kMaxGrid = 1024;
constexpr int kPrefillRows = 2048;   // prompt rows the GEMM prefill handles per chunk
constexpr int kPrefillMinRows = 32;  // shorter prompts take the 16-row passes of the decode kernel

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool config_ok(const ls_config* c) {
  if (!c) return false;
  if (c->dtype != LS_F32 && c->dtype != LS_BF16) return false;
  if (c->n_layers < 1 || c->n_layers > 4096) return false;
  if (c->head_dim != 64 && c->head_dim != 128) return false;
  if (c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads) return false;
  if (c->n_q_heads / c->n_kv_heads > 4) return false;
  if (c->d_model < 16 || c->d_model % 16 || c->ffn_dim < 16 || c->ffn_dim % 16) return false;
  if (c->vocab < 16 || c->vocab % 16) return false;
  // (the kernels split a stage's rows over the workgroups with 32-bit products of row units and workgroup ids)
  if (c->d_model > (1 << 20) || c->ffn_dim > (1 << 22) || c->vocab > (1 << 22) || c->n_q_heads > 4096) return false;
  if (c->max_draft < 1 || c->max_draft > LS_MAX_ROWS - 1) return false;
  if (c->max_seq < 2 || c->max_seq > 32768) return false;
  if (!(c->rms_eps > 0.f) || !(c->rope_base > 1.f)) return false;
  return true;
}

Layout make_layout(const ls_config* c) {
  Layout L{};
  const size_t esz = c->dtype == LS_BF16 ? 2 : 4;
  const size_t qd = (size_t)c->n_q_heads * c->head_dim, kvd = (size_t)c->n_kv_heads * c->head_dim;
  const size_t max_tiles = ((size_t)c->max_seq + LS_ATTN_TILE - 1) / LS_ATTN_TILE;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  L.layers = take(sizeof(LsLayerW) * c->n_layers);
  L.rope_cos = take(sizeof(float) * c->max_seq * (c->head_dim / 2));
  L.rope_sin = take(sizeof(float) * c->max_seq * (c->head_dim / 2));
  L.kcache = take(esz * c->n_layers * kvd * c->max_seq);
  L.vcache = take(esz * c->n_layers * kvd * c->max_seq);
  L.xbuf = take(sizeof(float) * LS_ROWS * c->d_model);
  L.ssq = take(sizeof(float) * LS_ROWS * kMaxGrid);           // sums of squares of the rows, one per workgroup
  L.qbuf = take(esz * LS_ROWS * qd);
  L.obuf = take(esz * LS_ROWS * qd);
  L.actbuf = take(esz * LS_ROWS * c->ffn_dim);
  L.attn_part = take(sizeof(float) * c->n_kv_heads * max_tiles * 64 * (c->head_dim + 2));
  L.attn_cnt = take(sizeof(uint32_t) * c->n_kv_heads);
  L.cand = take(sizeof(float) * 4 * LS_ROWS * kMaxGrid);
  L.bar = take(4096);
  L.state = take(sizeof(LsState));
  L.pf_rows = c->max_seq < kPrefillRows ? c->max_seq : kPrefillRows;
  L.x_pf = take(sizeof(float) * L.pf_rows * c->d_model);
  L.a_pf = take(esz * L.pf_rows * c->d_model);
  L.q_pf = take(esz * L.pf_rows * qd);
  L.o_pf = take(esz * L.pf_rows * qd);
  L.act_pf = take(esz * L.pf_rows * c->ffn_dim);
  L.total = off;
  return L;
}

}  // namespace

struct ls_ctx {
  ls_config cfg;
  Layout lay;
  char* ws;
  LsKParams base;   // model + workspace part of the kernel parameters
  int n_cu, max_wg_per_cu, wg_per_cu, grid;
  bool prefilled, drafted;
  bool poisoned;    // the device reported an error: exchange bookkeeping is rebuilt before the next prompt
  int draft_E, draft_d;
  int pos_bound;    // upper bound of the device-side position, for capacity checks
  hipEvent_t ev[3];
  bool owns_events;
  float* capture;
  unsigned long long* prof;
  int prof_cap, prof_wg;
  std::vector<LsLayerW> host_layers;
  LsPfParams pf;
  bool gemm_prefill;
  int kv_policy;   // 0: settled K/V tiles through the caches when the KV cache is small; 1: always; 2: never
};

namespace {

void set_decomposition(ls_ctx* c) {
  const ls_config& g = c->cfg;
  // Every matrix product splits its output rows evenly over the workgroups in units of four (the
  // kernel's part_of); here only what the kernel needs up front: one sum-of-squares slot per
  // workgroup and residual row, and the most 16-row tiles a workgroup gets in the O / down
  // projections (at least four units per active workgroup there).
  c->base.ssq_nt = c->grid;
  const int units = g.d_model / 4;
  int nwg = units / 4;
  nwg = nwg < 1 ? 1 : (nwg > c->grid ? c->grid : nwg);
  const int most_units = (units + nwg - 1) / nwg;
  c->base.x_tiles = (most_units + 3) / 4;
  // attention work items: (kv head, C consecutive 64-position tiles), C the smallest count for
  // which a full cache gives at most one item per workgroup
  const int max_tiles = (g.max_seq + LS_ATTN_TILE - 1) / LS_ATTN_TILE;
  int C = 1;
  while (g.n_kv_heads * ((max_tiles + C - 1) / C) > c->grid && C < max_tiles) ++C;
  c->base.attn_ctiles = C;
  // Settled K/V tiles: through the caches when the whole KV cache can stay in the 256 MB memory-side cache
  // between two passes (short contexts, small models: the tiles then come back from a cache, measured 1 us
  // per layer faster on the 1.5B and 8B shapes); with coherent loads otherwise (a large cache is streamed
  // once per pass, and coherent requests were 1 us per layer faster on the 13B shape).  Same bytes, same
  // arithmetic either way.
  const size_t kv_bytes = 2 * (size_t)g.n_layers * g.max_seq * g.n_kv_heads * g.head_dim * (g.dtype == LS_BF16 ? 2 : 4);
  c->base.kv_through_caches = c->kv_policy == 0 ? kv_bytes <= ((size_t)192 << 20) : c->kv_policy == 1;
}

int launch(ls_ctx* c, LsKParams& p, hipStream_t s) {
  if (hipMemsetAsync(p.bar, 0, 4096, s) != hipSuccess) return LS_E_HIP;
  if (ls_launch_program(&p, c->cfg.dtype == LS_BF16, c->grid, s) != 0) return LS_E_HIP;
  return LS_OK;
}

LsKParams program(const ls_ctx* c, int kind) {
  LsKParams p = c->base;
  p.kind = kind;
  p.E = 0; p.d = 0; p.E_low = 0; p.tau = 0.f; p.out_exits = nullptr; p.max_new = 0x7fffffff; p.eos = -1; p.n_tokens = 0; p.layers_used = c->cfg.n_layers;
  p.tokens = nullptr; p.out_tokens = nullptr; p.out_margin = nullptr;
  p.capture = c->capture;
  p.prof = c->prof; p.prof_cap = c->prof_cap; p.prof_wg = c->prof_wg;
  return p;
}

int read_state(ls_ctx* c, LsState* st, hipStream_t s) {
  if (hipMemcpyAsync(st, c->base.state, sizeof(LsState), hipMemcpyDeviceToHost, s) != hipSuccess) return LS_E_HIP;
  if (hipStreamSynchronize(s) != hipSuccess) return LS_E_HIP;
  if (st->error) c->poisoned = true;
  return LS_OK;
}

// After a device-side error the counters and the error flag are unreliable: start them over (row
// buffers, counters and state are contiguous in the workspace).
int recover(ls_ctx* c, hipStream_t s) {
  if (!c->poisoned) return LS_OK;
  if (hipMemsetAsync(c->ws + c->lay.xbuf, 0, c->lay.x_pf - c->lay.xbuf, s) != hipSuccess) return LS_E_HIP;
  c->poisoned = false;
  c->prefilled = c->drafted = false;
  return LS_OK;
}

}  // namespace

extern "C" {

size_t ls_workspace_bytes(const ls_config* cfg) {
  if (!config_ok(cfg)) return 0;
  return make_layout(cfg).total;
}

// Validates the configuration, the weight pointers and the workspace, then fills *c: uploads the
// layer pointer table and the rotary table into the workspace and zeroes counters and state.
// `events`: three timing events the context uses but does not own, or null to create its own.
static int init_ctx(ls_ctx* c, const ls_config* cfg, const ls_weights* w, void* dev_workspace, size_t workspace_bytes,
                    const hipEvent_t* events) {
  if (!config_ok(cfg) || !w || !dev_workspace) return LS_E_ARG;
  if ((uintptr_t)dev_workspace % 256) return LS_E_ARG;
  if (!w->embed || !w->final_norm || !w->lm_head || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_gate || !w->w_up ||
      !w->w_down || !w->attn_norm || !w->ffn_norm)
    return LS_E_ARG;
  auto bad = [](const void* p) { return p == nullptr || ((uintptr_t)p % 16) != 0; };
  if (bad(w->embed) || bad(w->final_norm) || bad(w->lm_head)) return LS_E_ARG;
  for (int l = 0; l < cfg->n_layers; ++l)
    if (bad(w->wq[l]) || bad(w->wk[l]) || bad(w->wv[l]) || bad(w->wo[l]) || bad(w->w_gate[l]) || bad(w->w_up[l]) ||
        bad(w->w_down[l]) || bad(w->attn_norm[l]) || bad(w->ffn_norm[l]))
      return LS_E_ARG;
  const Layout lay = make_layout(cfg);
  if (workspace_bytes < lay.total) return LS_E_CAPACITY;

  c->cfg = *cfg;
  c->lay = lay;
  c->ws = static_cast<char*>(dev_workspace);
  c->capture = nullptr;
  c->prof = nullptr; c->prof_cap = 0; c->prof_wg = 0;
  c->prefilled = c->drafted = false;
c->kv_policy = 0;
  c->poisoned = false;
  c->pos_bound = 0;

  hipDeviceProp_t prop;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return LS_E_HIP;
  c->n_cu = prop.multiProcessorCount;
  int nb = 0;
  if (ls_kernel_setup(cfg->dtype == LS_BF16, cfg->head_dim, &nb) != 0 || nb < 1) return LS_E_HIP;
  c->max_wg_per_cu = nb > 2 ? 2 : nb;
  c->wg_per_cu = c->max_wg_per_cu;
  c->grid = c->n_cu * c->wg_per_cu;
  if (c->grid > kMaxGrid) c->grid = kMaxGrid;

  // layer pointer table and rotary table
  std::vector<LsLayerW> lw(cfg->n_layers);
  for (int l = 0; l < cfg->n_layers; ++l)
    lw[l] = LsLayerW{w->wq[l], w->wk[l], w->wv[l], w->wo[l], w->w_gate[l], w->w_up[l], w->w_down[l],
                     w->attn_norm[l], w->ffn_norm[l]};
  const int half = cfg->head_dim / 2;
  std::vector<float> cs((size_t)cfg->max_seq * half), sn((size_t)cfg->max_seq * half);
  for (int j = 0; j < half; ++j) {
    const double inv_freq = std::pow((double)cfg->rope_base, -2.0 * j / cfg->head_dim);
    for (int t = 0; t < cfg->max_seq; ++t) {
      const double a = (double)t * inv_freq;
      cs[(size_t)t * half + j] = (float)std::cos(a);
      sn[(size_t)t * half + j] = (float)std::sin(a);
    }
  }
  bool okc = hipMemcpy(c->ws + lay.layers, lw.data(), sizeof(LsLayerW) * lw.size(), hipMemcpyHostToDevice) == hipSuccess;
  okc = okc && hipMemcpy(c->ws + lay.rope_cos, cs.data(), sizeof(float) * cs.size(), hipMemcpyHostToDevice) == hipSuccess;
  okc = okc && hipMemcpy(c->ws + lay.rope_sin, sn.data(), sizeof(float) * sn.size(), hipMemcpyHostToDevice) == hipSuccess;
  okc = okc && hipMemset(c->ws + lay.xbuf, 0, lay.x_pf - lay.xbuf) == hipSuccess;
  okc = okc && hipDeviceSynchronize() == hipSuccess;
  c->owns_events = events == nullptr;
  for (int i = 0; i < 3 && okc; ++i) {
    if (events) c->ev[i] = events[i];
    else okc = hipEventCreate(&c->ev[i]) == hipSuccess;
  }
  if (!okc) return LS_E_HIP;

  LsKParams& p = c->base;
  memset(&p, 0, sizeof(p));
  p.L = cfg->n_layers; p.dm = cfg->d_model; p.nq = cfg->n_q_heads; p.nkv = cfg->n_kv_heads; p.hd = cfg->head_dim;
  p.ffn = cfg->ffn_dim; p.vocab = cfg->vocab; p.qd = cfg->n_q_heads * cfg->head_dim;
  p.kvd = cfg->n_kv_heads * cfg->head_dim; p.G = cfg->n_q_heads / cfg->n_kv_heads; p.max_seq = cfg->max_seq;
  p.eps = cfg->rms_eps;
  p.attn_scale = (float)(1.0 / std::sqrt((double)cfg->head_dim));
  p.layers = reinterpret_cast<const LsLayerW*>(c->ws + lay.layers);
  p.embed = w->embed; p.final_norm = w->final_norm; p.lm_head = w->lm_head;
  p.rope_cos = reinterpret_cast<const float*>(c->ws + lay.rope_cos);
  p.rope_sin = reinterpret_cast<const float*>(c->ws + lay.rope_sin);
  p.kcache = c->ws + lay.kcache; p.vcache = c->ws + lay.vcache;
  p.xbuf = reinterpret_cast<float*>(c->ws + lay.xbuf);
  p.ssq = reinterpret_cast<float*>(c->ws + lay.ssq);
  p.qbuf = c->ws + lay.qbuf; p.obuf = c->ws + lay.obuf; p.actbuf = c->ws + lay.actbuf;
  p.attn_part = reinterpret_cast<float*>(c->ws + lay.attn_part);
  p.attn_cnt = reinterpret_cast<uint32_t*>(c->ws + lay.attn_cnt);
  p.max_tiles = (cfg->max_seq + LS_ATTN_TILE - 1) / LS_ATTN_TILE;
  p.cand = reinterpret_cast<float*>(c->ws + lay.cand);
  p.bar = reinterpret_cast<uint32_t*>(c->ws + lay.bar);
  p.state = reinterpret_cast<LsState*>(c->ws + lay.state);
  p.spin_limit = 1 << 22;
  set_decomposition(c);
  c->host_layers = lw;
  LsPfParams& f = c->pf;
  memset(&f, 0, sizeof(f));
  f.is_bf16 = cfg->dtype == LS_BF16; f.dm = p.dm; f.qd = p.qd; f.kvd = p.kvd; f.ffn = p.ffn; f.vocab = p.vocab;
  f.hd = p.hd; f.nkv = p.nkv; f.max_seq = p.max_seq; f.layers_used = p.L; f.eps = p.eps;
  f.embed = w->embed; f.rope_cos = p.rope_cos; f.rope_sin = p.rope_sin; f.kcache = p.kcache; f.vcache = p.vcache;
  f.x_pf = reinterpret_cast<float*>(c->ws + lay.x_pf); f.a_pf = c->ws + lay.a_pf; f.q_pf = c->ws + lay.q_pf;
  f.o_pf = c->ws + lay.o_pf; f.act_pf = c->ws + lay.act_pf; f.xbuf = p.xbuf; f.ssq = p.ssq;
  c->gemm_prefill = true;
  return LS_OK;
}

int ls_load_weights(const ls_config* cfg, const ls_weights* w, void* dev_workspace, size_t workspace_bytes,
                    ls_ctx** out) {
  if (!out) return LS_E_ARG;
  *out = nullptr;
  ls_ctx* c = new (std::nothrow) ls_ctx();
  if (!c) return LS_E_ARG;
  const int rc = init_ctx(c, cfg, w, dev_workspace, workspace_bytes, nullptr);
  if (rc != LS_OK) { delete c; return rc; }
  *out = c;
  return LS_OK;
}

int ls_set_prompt_tiles(ls_ctx* c, int32_t rows) {
  if (!c) return LS_E_ARG;
  if (rows != 0 && rows != 16 && rows != 32 && rows != 64 && rows != 128 && rows != 160) return LS_E_RANGE;
  c->gemm_prefill = rows != 16;
  c->pf.tile_rows = rows == 16 ? 0 : rows;
  return LS_OK;
}

int ls_debug_spin_limit(ls_ctx* c, int32_t polls) {
  if (!c) return LS_E_ARG;
  if (polls < 0) return LS_E_RANGE;
  c->base.spin_limit = polls == 0 ? (1 << 22) : polls;
  return LS_OK;
}

int ls_debug_kv_policy(ls_ctx* c, int32_t policy) {
  if (!c) return LS_E_ARG;
  if (policy < 0 || policy > 2) return LS_E_RANGE;
  c->kv_policy = policy;
  set_decomposition(c);
  return LS_OK;
}

int ls_set_launch(ls_ctx* c, int32_t wg_per_cu) {
  if (!c) return LS_E_ARG;
  if (wg_per_cu < 0 || wg_per_cu > c->max_wg_per_cu) return LS_E_RANGE;
  c->wg_per_cu = wg_per_cu == 0 ? c->max_wg_per_cu : wg_per_cu;
  c->grid = c->n_cu * c->wg_per_cu;
  if (c->grid > kMaxGrid) c->grid = kMaxGrid;
  set_decomposition(c);
  return c->grid;
}

// The prompt pass: GEMM path for prompts of kPrefillMinRows rows or more (in chunks of pf_rows),
// else the 16-row passes of the decode kernel.  Ends with the decoding state of a finished prefill.
static int enqueue_prefill(ls_ctx* c, const int32_t* dev_prompt, int32_t n_prompt, int32_t layers_used,
                           int32_t* dev_out, int32_t eos, int32_t max_new, hipStream_t s) {
  if (!c->gemm_prefill || n_prompt < kPrefillMinRows) {
    LsKParams p = program(c, LS_PROG_PREFILL);
    p.tokens = dev_prompt; p.n_tokens = n_prompt; p.out_tokens = dev_out; p.eos = eos; p.max_new = max_new;
    p.layers_used = layers_used;
    return launch(c, p, s);
  }
  LsPfParams f = c->pf;
  f.ssq_nt = c->base.ssq_nt;
  f.tokens = dev_prompt; f.layers_used = layers_used; f.capture = c->capture;
  int last_rows = 0;
  for (int pos0 = 0; pos0 < n_prompt; pos0 += c->lay.pf_rows) {
    const int M = n_prompt - pos0 < c->lay.pf_rows ? n_prompt - pos0 : c->lay.pf_rows;
    if (ls_prefill_layers(&f, c->host_layers.data(), pos0, M, s) != 0) return LS_E_HIP;
    last_rows = M;
  }
  if (ls_prefill_finish(&f, last_rows - 1, s) != 0) return LS_E_HIP;
  LsKParams p = program(c, LS_PROG_PF_FINISH);
  p.n_tokens = n_prompt; p.out_tokens = dev_out; p.eos = eos; p.max_new = max_new;
  return launch(c, p, s);
}

int ls_prefill(ls_ctx* c, const int32_t* dev_prompt, int32_t n_prompt, void* stream) {
  if (!c || !dev_prompt) return LS_E_ARG;
  if (n_prompt < 1) return LS_E_RANGE;
  if (n_prompt + 1 > c->cfg.max_seq) return LS_E_CAPACITY;
  int rc = recover(c, static_cast<hipStream_t>(stream));
  if (rc != LS_OK) return rc;
  rc = enqueue_prefill(c, dev_prompt, n_prompt, c->cfg.n_layers, nullptr, -1, 0x7fffffff,
                       static_cast<hipStream_t>(stream));
  if (rc != LS_OK) return rc;
  c->prefilled = true; c->drafted = false; c->pos_bound = n_prompt;
  return LS_OK;
}

int ls_draft(ls_ctx* c, int32_t E, int32_t d, void* stream) {
  if (!c) return LS_E_ARG;
  if (E < 1 || E > c->cfg.n_layers || d < 1 || d > c->cfg.max_draft) return LS_E_RANGE;
  if (!c->prefilled) return LS_E_STATE;
  if (c->pos_bound + d + 1 > c->cfg.max_seq) return LS_E_CAPACITY;
  LsKParams p = program(c, LS_PROG_DRAFT);
  p.E = E; p.d = d;
  const int rc = launch(c, p, static_cast<hipStream_t>(stream));
  if (rc != LS_OK) return rc;
  c->drafted = true; c->draft_E = E; c->draft_d = d;
  return LS_OK;
}

int ls_verify(ls_ctx* c, int32_t E, int32_t d, void* stream) {
  if (!c) return LS_E_ARG;
  if (E < 1 || E > c->cfg.n_layers || d < 1 || d > c->cfg.max_draft) return LS_E_RANGE;
  if (!c->prefilled || !c->drafted || c->draft_E != E || c->draft_d != d) return LS_E_STATE;
  LsKParams p = program(c, LS_PROG_VERIFY);
  p.E = E; p.d = d;
  const int rc = launch(c, p, static_cast<hipStream_t>(stream));
  if (rc != LS_OK) return rc;
  c->drafted = false;
  c->pos_bound += d + 1;
  return LS_OK;
}

struct DynamicExit {      // per-token exit layer (ls_generate_dynamic)
  int32_t E_low = 0;
  float tau = 0.f;
  int32_t* dev_exits = nullptr;
  int64_t* low_exits = nullptr;
};

static int generate_impl(ls_ctx* c, const int32_t* dev_prompt, int32_t n_prompt, int32_t max_new, int32_t E, int32_t d,
                         int32_t eos, int32_t layers_used, int32_t* dev_out, ls_stats* stats, void* stream,
                         bool no_reuse = false, const DynamicExit* dyn = nullptr) {
  if (!c || !dev_prompt || !dev_out) return LS_E_ARG;
  if (n_prompt < 1 || max_new < 1) return LS_E_RANGE;
  if (d < 0 || d > c->cfg.max_draft) return LS_E_RANGE;
  if (d > 0 && (E < 1 || E > c->cfg.n_layers)) return LS_E_RANGE;
  if (layers_used < 1 || layers_used > c->cfg.n_layers) return LS_E_RANGE;
  if ((long)n_prompt + max_new + d + 1 > c->cfg.max_seq) return LS_E_CAPACITY;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int rc = recover(c, s);
  if (rc != LS_OK) return rc;
  if (hipMemsetAsync(dev_out, 0xFF, sizeof(int32_t) * max_new, s) != hipSuccess) return LS_E_HIP;
  if (hipEventRecord(c->ev[0], s) != hipSuccess) return LS_E_HIP;
  rc = enqueue_prefill(c, dev_prompt, n_prompt, layers_used, dev_out, eos, max_new, s);
  if (rc != LS_OK) return rc;
  if (hipEventRecord(c->ev[1], s) != hipSuccess) return LS_E_HIP;
  LsKParams g = program(c, LS_PROG_GENERATE);
  g.E = E; g.d = d; g.max_new = max_new; g.eos = eos; g.out_tokens = dev_out; g.layers_used = layers_used;
  g.no_reuse = no_reuse ? 1 : 0;
  if (dyn) { g.E_low = dyn->E_low; g.tau = dyn->tau; g.out_exits = dyn->dev_exits; }
  rc = launch(c, g, s);
  if (rc != LS_OK) return rc;
  if (hipEventRecord(c->ev[2], s) != hipSuccess) return LS_E_HIP;
  LsState st;
  rc = read_state(c, &st, s);
  if (rc != LS_OK) return rc;
  c->prefilled = true; c->drafted = false; c->pos_bound = st.pos;
  if (dyn && dyn->low_exits) *dyn->low_exits = st.low_exits;
  if (stats) {
    stats->rounds = st.rounds; stats->drafted = st.drafted; stats->accepted = st.accepted; stats->generated = st.n_gen;
    stats->ms_prefill = stats->ms_decode = 0.f;
    (void)hipEventElapsedTime(&stats->ms_prefill, c->ev[0], c->ev[1]);
    (void)hipEventElapsedTime(&stats->ms_decode, c->ev[1], c->ev[2]);
  }
  return st.error ? LS_E_DEVICE : LS_OK;
}

int ls_generate(ls_ctx* c, const int32_t* dev_prompt, int32_t n_prompt, int32_t max_new, int32_t E, int32_t d,
                int32_t eos, int32_t* dev_out, ls_stats* stats, void* stream) {
  if (!c) return LS_E_ARG;
  return generate_impl(c, dev_prompt, n_prompt, max_new, E, d, eos, c->cfg.n_layers, dev_out, stats, stream);
}

int ls_generate_no_reuse(ls_ctx* c, const int32_t* dev_prompt, int32_t n_prompt, int32_t max_new, int32_t E, int32_t d,
                         int32_t eos, int32_t* dev_out, ls_stats* stats, void* stream) {
  if (!c) return LS_E_ARG;
  if (d < 1) return LS_E_RANGE;
  return generate_impl(c, dev_prompt, n_prompt, max_new, E, d, eos, c->cfg.n_layers, dev_out, stats, stream, true);
}

int ls_generate_dynamic(ls_ctx* c, const int32_t* dev_prompt, int32_t n_prompt, int32_t max_new, int32_t E_low,
                        int32_t E_high, int32_t d, float tau, int32_t eos, int32_t* dev_out, int32_t* dev_exit_layers,
                        ls_stats* stats, int64_t* host_low_exits, void* stream) {
  if (!c) return LS_E_ARG;
  if (d < 1 || E_low < 1 || E_low >= E_high || E_high > c->cfg.n_layers || tau != tau) return LS_E_RANGE;
  DynamicExit dyn;
  dyn.E_low = E_low; dyn.tau = tau; dyn.dev_exits = dev_exit_layers; dyn.low_exits = host_low_exits;
  return generate_impl(c, dev_prompt, n_prompt, max_new, E_high, d, eos, c->cfg.n_layers, dev_out, stats, stream, false, &dyn);
}

int ls_generate_early_exit(ls_ctx* c, const int32_t* dev_prompt, int32_t n_prompt, int32_t max_new, int32_t E,
                           int32_t* dev_out, ls_stats* stats, void* stream) {
  if (!c) return LS_E_ARG;
  if (E < 1 || E > c->cfg.n_layers) return LS_E_RANGE;
  return generate_impl(c, dev_prompt, n_prompt, max_new, E, 0, -1, E, dev_out, stats, stream);
}

static int score_impl(ls_ctx* c, const int32_t* dev_tokens, int32_t n, int32_t layers_used, int32_t* dev_argmax,
                      float* dev_margin, void* stream, bool probe) {
  if (!c || !dev_tokens || !dev_argmax) return LS_E_ARG;
  if (n < 1 || layers_used < 1 || layers_used > c->cfg.n_layers) return LS_E_RANGE;
  if (n > c->cfg.max_seq) return LS_E_CAPACITY;
  hipStream_t s = static_cast<hipStream_t>(stream);
  LsKParams p = program(c, LS_PROG_SCORE);
  p.probe = probe ? 1 : 0;
  p.tokens = dev_tokens; p.n_tokens = n; p.layers_used = layers_used; p.out_tokens = dev_argmax; p.out_margin = dev_margin;
  int rc = launch(c, p, s);
  if (rc != LS_OK) return rc;
  c->prefilled = false; c->drafted = false;
  LsState st;
  rc = read_state(c, &st, s);
  if (rc != LS_OK) return rc;
  return st.error ? LS_E_DEVICE : LS_OK;
}

int ls_score(ls_ctx* c, const int32_t* dev_tokens, int32_t n, int32_t layers_used, int32_t* dev_argmax,
             float* dev_margin, void* stream) {
  return score_impl(c, dev_tokens, n, layers_used, dev_argmax, dev_margin, stream, false);
}

int ls_probe_layers(ls_ctx* c, const int32_t* dev_tokens, int32_t n, int32_t* dev_argmax, float* dev_margin,
                    void* stream) {
  if (!c) return LS_E_ARG;
  return score_impl(c, dev_tokens, n, c->cfg.n_layers, dev_argmax, dev_margin, stream, true);
}

int ls_get_state(ls_ctx* c, int32_t* pos, int32_t* last, int32_t* n_gen, void* stream) {
  if (!c) return LS_E_ARG;
  LsState st;
  const int rc = read_state(c, &st, static_cast<hipStream_t>(stream));
  if (rc != LS_OK) return rc;
  if (pos) *pos = st.pos;
  if (last) *last = st.last;
  if (n_gen) *n_gen = st.n_gen;
  c->pos_bound = st.pos;
  return st.error ? LS_E_DEVICE : LS_OK;
}

int ls_peek_round(ls_ctx* c, int32_t* hd, int32_t* hv, float* hdm, float* hvm, int32_t* n_accept, void* stream) {
  if (!c) return LS_E_ARG;
  LsState st;
  const int rc = read_state(c, &st, static_cast<hipStream_t>(stream));
  if (rc != LS_OK) return rc;
  const int d = st.draft_valid ? st.draft_d : c->draft_d;
  if (d < 1 || d > LS_ROWS - 1) return LS_E_STATE;
  if (hd) memcpy(hd, st.D, sizeof(int32_t) * d);
  if (hv) memcpy(hv, st.V, sizeof(int32_t) * (d + 1));
  if (hdm) memcpy(hdm, st.dmargin, sizeof(float) * d);
  if (hvm) memcpy(hvm, st.vmargin, sizeof(float) * (d + 1));
  if (n_accept) *n_accept = st.n_acc;
  return st.error ? LS_E_DEVICE : LS_OK;
}

int ls_debug_capture(ls_ctx* c, float* dev_hidden) {
  if (!c) return LS_E_ARG;
  c->capture = dev_hidden;
  return LS_OK;
}

int ls_debug_timeline(ls_ctx* c, unsigned long long* dev_events, int32_t capacity, int32_t workgroup) {
  if (!c) return LS_E_ARG;
  if (dev_events != nullptr && (capacity < 1 || workgroup < 0 || workgroup >= c->grid)) return LS_E_RANGE;
  c->prof = dev_events; c->prof_cap = dev_events ? capacity : 0; c->prof_wg = workgroup;
  return LS_OK;
}

int ls_debug_copy(void* dev_dst, const void* dev_src, size_t bytes, void* stream) {
  if (!dev_dst || !dev_src || bytes == 0 || bytes % 16 || ((uintptr_t)dev_dst | (uintptr_t)dev_src) % 16) return LS_E_ARG;
  return ls_launch_copy(dev_src, dev_dst, bytes, static_cast<hipStream_t>(stream)) == 0 ? LS_OK : LS_E_HIP;
}

int ls_debug_read(const void* dev_src, size_t bytes, void* dev_sink, int32_t workgroups, void* stream) {
  if (!dev_src || !dev_sink || workgroups < 1 || workgroups > 4096 || ((uintptr_t)dev_src | (uintptr_t)dev_sink) % 16) return LS_E_ARG;
  if (bytes == 0 || bytes % ((size_t)workgroups * 256 * 16 * 16)) return LS_E_ARG;
  return ls_launch_read(dev_src, bytes, dev_sink, workgroups, static_cast<hipStream_t>(stream)) == 0 ? LS_OK : LS_E_HIP;
}

const char* ls_strerror(int code) {
  switch (code) {
    case LS_OK: return "ok";
    case LS_E_ARG: return "invalid argument (null pointer, unsupported shape, dtype or alignment)";
    case LS_E_RANGE: return "value out of range (exit layer, draft length or count)";
    case LS_E_CAPACITY: return "capacity exceeded (workspace or max_seq)";
    case LS_E_STATE: return "call out of order (prefill -> draft -> verify)";
    case LS_E_HIP: return "HIP runtime call failed";
    case LS_E_DEVICE: return "device reported an error (bounded wait expired or cache capacity)";
    default: return "unknown error";
  }
}

void ls_destroy(ls_ctx* c) {
  if (!c) return;
  if (c->owns_events)
    for (int i = 0; i < 3; ++i) (void)hipEventDestroy(c->ev[i]);
  delete c;
}

size_t ls_static_workspace_limit(void) { return LS_STATIC_SCRATCH_BYTES; }

int ls_generate_static(const ls_config* cfg, const ls_weights* w, const int32_t* dev_prompt, int32_t n_prompt,
                       int32_t max_new, int32_t E, int32_t d, int32_t eos, int32_t* dev_out, ls_stats* stats,
                       void* stream) {
  if (!config_ok(cfg)) return LS_E_ARG;
  // sizes beyond the fixed array are refused before anything touches the device
  if (make_layout(cfg).total > (size_t)LS_STATIC_SCRATCH_BYTES) return LS_E_CAPACITY;
  // set-up, once per device with that device current: the address of this device's copy of the array
  // (never the array's name: in host code that is not a device address) and the timing events
  constexpr int kMaxDev = 64;
  struct PerDevice { hipEvent_t ev[3]; bool ready; };
  static PerDevice per_dev[kMaxDev];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return LS_E_HIP;
  void* scratch = nullptr;
  if (ls_static_scratch_ptr(&scratch) != 0) return LS_E_HIP;
  PerDevice& pd = per_dev[dev];
  if (!pd.ready) {
    for (int i = 0; i < 3; ++i)
      if (hipEventCreate(&pd.ev[i]) != hipSuccess) return LS_E_HIP;
    pd.ready = true;
  }
  // The array keeps the previous call's contents: init_ctx uploads the tables again and zeroes every
  // counter, flag and state word of this configuration's layout; stale cache rows and stage buffers are
  // overwritten before they are read.
  ls_ctx c{};
  int rc = init_ctx(&c, cfg, w, scratch, LS_STATIC_SCRATCH_BYTES, pd.ev);
  if (rc != LS_OK) return rc;
  return generate_impl(&c, dev_prompt, n_prompt, max_new, E, d, eos, cfg->n_layers, dev_out, stats, stream);
}

}  // extern "C"
