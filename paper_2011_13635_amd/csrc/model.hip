// Host logic of the MSLT stage-step library: tensor table, arena layout, the launch sequence of
// one stage step (frozen prefix forward-only, trainable top layers and head forward + backward),
// gradient read-back and the optimizer update over the trainable tensors only (paper Section
// 3.2).  Every arithmetic step runs in the HIP kernels of the sibling files; this file only
// validates, lays out memory and enqueues.
#include "../../include/mslt.h"
#include "common.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

using namespace mslt;

static thread_local std::string g_err;
static int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}
#define HIP_TRY(expr)                                                                       \
  do {                                                                                      \
    hipError_t e__ = (expr);                                                                \
    if (e__ != hipSuccess) return fail(MSLT_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e__)); \
  } while (0)

static inline size_t rup(size_t x, size_t a) { return (x + a - 1) / a * a; }

enum { T_WORD = 0, T_POS, T_TYPE, T_ELN_G, T_ELN_B, N_EMB };
enum { L_WQ = 0, L_WK, L_WV, L_BQ, L_BK, L_BV, L_WO, L_BO, L_LN1G, L_LN1B, L_W1, L_B1, L_W2, L_B2, L_LN2G, L_LN2B, N_LAYER_T };
enum { H_WT = 0, H_BT, H_LNG, H_LNB, H_BOUT, N_HEAD };
// next-sentence head, after the masked-LM head when the model has one
enum { P_W = N_HEAD, P_B, C_W, C_B, N_HEAD_NSP };

// Optional per-kernel-class timing with HIP events on the model's stream (off by default).
enum ProfClass { PC_GEMM_NT = 0, PC_GEMM_NN, PC_GEMM_TN, PC_GEMM_SIMT, PC_ATTN_FWD, PC_ATTN_BWD, PC_LN_FWD, PC_LN_BWD,
                 PC_COLSUM, PC_EMBED, PC_HEAD_MISC, PC_CE, PC_EMBED_BWD, PC_OPT, PC_REDUCE, PC_COUNT };
static const char* kProfNames[PC_COUNT] = {"gemm_mfma_nt", "gemm_mfma_nn", "gemm_mfma_tn", "gemm_simt", "attention_fwd",
                                           "attention_bwd", "layernorm_fwd", "layernorm_bwd", "bias_colsum", "embed_fwd",
                                           "head_gather_scatter", "cross_entropy", "embed_bwd", "optimizer", "gradient_sums"};
static int pick_splitk(int M, int N, int K);
// Tile of the grouped weight-gradient launch of one layer (index into kGroupTile), or -1 when the products go
// out one by one.  cnt[c]: tiles of all the products together at shape c; ok[c]: every product fits shape c.
// 256x256 moves half the bytes per FLOP of 128x128 and 256x128 three quarters, but one such workgroup fills a
// compute unit, so a large tile is taken when its tiles keep at least 160 of the 256 compute units busy in every
// round; with fewer than 256 small tiles splitting k fills the chip better than grouping.
static const int kGroupTile[3][2] = {{256, 256}, {256, 128}, {128, 128}};
static int group_tile_pick(const int (&cnt)[3], const bool (&ok)[3]) {
  constexpr int BIG_MIN = 160;
  for (int c = 0; c < 2; ++c) {
    const int rounds = (cnt[c] + 255) / 256;
    if (ok[c] && cnt[c] >= BIG_MIN * rounds) return c;
  }
  return ok[2] && cnt[2] >= 256 ? 2 : -1;
}
struct ProfSpan {
  hipEvent_t a, b;
  int cls;
  double flops, bytes;
};
struct Profiler {
  bool on = false;
  std::vector<ProfSpan> spans;    // spans of the steps since the last read
  std::vector<hipEvent_t> pool;   // recycled events
  hipEvent_t get() {
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    hipEventCreate(&e);
    return e;
  }
};

struct LayerStash {
  // ctx32: unrounded fp32 copy of the attention context (bf16 mode only), from which the backward takes delta
  // u holds GELU'(FFN pre-activation): the forward epilogue computes it next to the GELU value, so
  // the backward pass multiplies instead of evaluating erf and exp again
  void *xout, *qkv, *ctx, *xhat1, *x1, *u, *g, *xhat2;
  float *lse, *rstd1, *rstd2, *ctx32;
};

struct mslt_model {
  mslt_config cfg;
  int dtype;        // 0 fp32, 1 bf16
  size_t esz;       // bytes per activation element
  bool mfma;        // bf16 MFMA GEMMs with padded row counts
  hipStream_t stream;
  int H, F, V, Vp, nh, dh, L, Tp, Mp, cap;
  int nsp;          // next-sentence head present (pooler + two-way classifier)
  void *n_xc, *n_p, *n_dz, *n_dp, *n_du, *n_dx;   // its batch-many rows: first tokens, pooled, and gradients
  float* n_z;       // its logits [max_batch, 2]
  int lpg, Lp;      // layers per parameter-sharing group (1: every layer has its own set), number of sets = L / lpg
  int acc_now;      // the layer whose backward is being queued adds to its set's gradients (not the first of its group)
  std::vector<mslt_tensor_desc> table;
  std::vector<size_t> alloc_count;  // elements reserved per tensor (>= count)
  size_t arena_elems, packed_count;
  float *param, *grad, *mom1, *mom2;
  char* ws;
  size_t ws_bytes;
  // workspace carve-up
  bf16* shadow;
  void *x0, *xhat0; float* rstd0;
  void *xa, *xb;                       // frozen-prefix ping-pong
  void *s_qkv, *s_ctx, *s_x1, *s_g, *s_y;  // scratch of the forward-only path (+ s_y: pre-LN GEMM output)
  std::vector<LayerStash> stash;       // one per layer that can train in one step (n_stash); layer l of a step uses stash[l - frozen]
  int n_stash, stash_base;             // stash_base: frozen layer count of the step being queued / of the last step
  void *dxa, *dxb, *d_d, *d_u, *d_x1, *d_z1, *d_c, *d_qkv, *d_z0;
  // bf16 mode: the residual branch of the backward pass (layer-output gradient, dz2 and dz1 as addends, dx1) is
  // carried in fp32, so that its rounding does not pile up from layer to layer; the GEMM operands stay bf16
  bool wide;
  float *d_d32, *d_z1_32;
  float *delta;
  int32_t *pos, *lab, *inv, *counters;
  void *xm, *ut, *gt, *xhat_t, *hm, *dz, *d_hm, *d_gt, *d_ut, *d_xm;
  void *c_g, *c_u, *c_du;              // compacted FFN rows of the top layer [Mp, F]
  float *rstd_t, *logits, *row_loss, *lse_t, *loss;
  float *red_scratch; size_t red_floats;
  float *splitk; size_t splitk_floats;
  // side stream: weight-gradient products and bias column sums overlap the data-gradient chain
  hipStream_t side; hipEvent_t ev_fork, ev_join; bool side_forked;
  // the gradient buffers the side stream reads exist twice and alternate by layer, so a layer's
  // side work only has to finish before the layer two below starts
  struct GradSet { void *d_d, *d_u, *d_z1, *d_qkv, *d_dm, *d_z1m; } gset[2];   // d_dm, d_z1m: dropout-masked dz2, dz1
  hipEvent_t ev_set[2]; bool set_busy[2];
  hipEvent_t ev_scan;      // batch check done and its verdict copied to the host
  // dropout (off unless mslt_set_dropout was called with p > 0)
  uint64_t drop_seed = 0, drop_step = 0;
  uint32_t drop_thr = 0;
  float drop_scale = 1.f;
  void *d_dm, *d_z1m;      // masked dz2 / dz1 of the current layer's set
  void *c_dz2m, *c_dz1m;   // the same for the compacted top layer
  void *c_xhat2, *c_dz2, *c_dc;   // compacted top layer: rows of xhat2, dz2 and dC (buffers of their own: the side
                                  // stream may still be reading the head's when the top layer starts)
  float *splitk2, *red2;
  // Sums of partial results that only the optimizer reads (parameter gradients: LayerNorm and bias column
  // sums, split-k partial products of the weight gradients) are not launched one by one: their partials go
  // to an arena of their own, the jobs are listed here and one launch at the end of the step adds them all.
  // Off when layers share parameters (a shared tensor is then written by one layer and added to by others,
  // which the order of single launches keeps and one batch would not).
  // Inside a layer's backward the weight-gradient products and bias column sums are collected and queued on
  // the side stream together when the layer is done (one fork; the products as one grouped launch).
  struct SideColsum { const void* dY; int ld, rows, N; float* out; int accumulate; };
  std::vector<GemmDesc> side_dw;
  std::vector<SideColsum> side_cs;
  bool side_collect = false;
  std::vector<ReduceJob> later;
  float* later_arena = nullptr; size_t later_floats = 0, later_used = 0;
  bool later_on = false;
  int32_t *e_rank, *e_cnt, *e_start, *e_order, *e_blockcnt;
  float* e_partial;                    // [Tp, H] run sums of the embedding backward
  OptTensor* o_tensors; int32_t* o_chunk_tensor; int32_t* o_tsteps; float* o_chunk_norms; float* o_ratio;
  std::vector<int> first_chunk;  // per tensor, plus total at the end
  float* static_scratch;   // this device's copy of the file-scope scratch array (see mslt_apply_update_static)
  // pinned host scalars
  int32_t* h_counters; float* h_loss;
  // last step
  bool have_grads;
  int last_f, last_k, last_emb, last_B, last_S, last_M;
  const void* last_prefix;
  Profiler prof;
};

// ---- scratch for the entry point that must not allocate ----------------------------------------
// mslt_apply_update_static keeps the only scratch the update needs (LAMB's per-chunk partial sums of
// |w|^2 and |u|^2 and the per-tensor ratios) in this file-scope device array instead of the caller's
// workspace.  Every GPU the library runs on holds its own copy until the process ends.  The array's
// name is only a host-side handle: its device address is looked up once per device (with that
// device current) and that address is what kernels and copies get.
constexpr int STATIC_MAX_CHUNKS = 32768;     // 16384-element optimizer chunks: models up to 536 M parameters
constexpr int STATIC_MAX_TENSORS = 1024;
constexpr size_t STATIC_SCRATCH_FLOATS = (size_t)2 * STATIC_MAX_CHUNKS + STATIC_MAX_TENSORS;   // 266 240 bytes
static __device__ __align__(256) float scratch[STATIC_SCRATCH_FLOATS];
constexpr int MAX_DEVICES = 64;
static float* g_scratch_ptr[MAX_DEVICES];    // device address of `scratch` per device id, null until looked up
// Address of this device's copy of the scratch array (looked up on first use; the caller's current device is restored).
static int static_scratch_for(int dev, float** out) {
  if (dev < 0 || dev >= MAX_DEVICES) return fail(MSLT_ERR_ARG, "device id %d outside 0..%d", dev, MAX_DEVICES - 1);
  if (!g_scratch_ptr[dev]) {
    int cur = -1;
    HIP_TRY(hipGetDevice(&cur));
    if (cur != dev) HIP_TRY(hipSetDevice(dev));
    void* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (cur != dev) hipSetDevice(cur);
    if (e != hipSuccess || !ptr) return fail(MSLT_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = static_cast<float*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return MSLT_OK;
}

// ---- tensor table ---------------------------------------------------------------------------
static void add_tensor(mslt_model* m, const char* name, int layer, int rows, int cols, int decays, size_t reserve,
                       bool align, size_t& off) {
  mslt_tensor_desc d;
  memset(&d, 0, sizeof d);
  snprintf(d.name, sizeof d.name, "%s", name);
  d.layer = layer;
  d.rows = rows;
  d.cols = cols;
  d.decays = decays;
  d.count = (size_t)rows * cols;
  if (align) off = rup(off, 64);
  d.offset = off;
  off += reserve ? reserve : d.count;
  m->table.push_back(d);
  m->alloc_count.push_back(reserve ? reserve : d.count);
}

static void build_table(mslt_model* m) {
  const int H = m->H, F = m->F, V = m->V, Vp = m->Vp;
  size_t off = 0;
  add_tensor(m, "emb.word", -1, V, H, 1, (size_t)Vp * H, true, off);
  add_tensor(m, "emb.pos", -1, m->cfg.max_pos, H, 1, 0, true, off);
  add_tensor(m, "emb.type", -1, m->cfg.type_vocab, H, 1, 0, true, off);
  add_tensor(m, "emb.ln_g", -1, H, 1, 0, 0, true, off);
  add_tensor(m, "emb.ln_b", -1, H, 1, 0, 0, true, off);
  static const char* ln[N_LAYER_T] = {"wq", "wk", "wv", "bq", "bk", "bv", "wo", "bo", "ln1_g", "ln1_b",
                                      "w1", "b1", "w2", "b2", "ln2_g", "ln2_b"};
  for (int l = 0; l < m->Lp; ++l) {
    char nm[32];
    for (int j = 0; j < N_LAYER_T; ++j) {
      snprintf(nm, sizeof nm, "layer%d.%s", l, ln[j]);
      int rows = H, cols = 1, dec = 0;
      switch (j) {
        case L_WQ: case L_WK: case L_WV: case L_WO: rows = H; cols = H; dec = 1; break;
        case L_W1: rows = F; cols = H; dec = 1; break;
        case L_W2: rows = H; cols = F; dec = 1; break;
        case L_B1: rows = F; break;
        default: break;
      }
      // wq|wk|wv and bq|bk|bv stay contiguous: they are read as one [3H,H] matrix and one [3H] bias
      bool align = !(j == L_WK || j == L_WV || j == L_BK || j == L_BV);
      add_tensor(m, nm, l, rows, cols, dec, 0, align, off);
    }
  }
  add_tensor(m, "head.wt", -2, H, H, 1, 0, true, off);
  add_tensor(m, "head.bt", -2, H, 1, 0, 0, true, off);
  add_tensor(m, "head.ln_g", -2, H, 1, 0, 0, true, off);
  add_tensor(m, "head.ln_b", -2, H, 1, 0, 0, true, off);
  add_tensor(m, "head.b_out", -2, V, 1, 0, (size_t)Vp, true, off);
  if (m->nsp) {
    add_tensor(m, "pooler.w", -2, H, H, 1, 0, true, off);
    add_tensor(m, "pooler.b", -2, H, 1, 0, 0, true, off);
    add_tensor(m, "nsp.w", -2, 2, H, 1, 0, true, off);
    add_tensor(m, "nsp.b", -2, 2, 1, 0, 0, true, off);
  }
  m->arena_elems = rup(off, 64);
  m->packed_count = 0;
  for (auto& d : m->table) m->packed_count += d.count;
  // optimizer chunks
  m->first_chunk.clear();
  int c = 0;
  for (auto& d : m->table) {
    m->first_chunk.push_back(c);
    c += (int)((d.count + OPT_CHUNK - 1) / OPT_CHUNK);
  }
  m->first_chunk.push_back(c);
}
static inline int t_emb(int j) { return j; }
static inline int t_layer(int l, int j) { return N_EMB + l * N_LAYER_T + j; }
static inline int t_head(const mslt_model* m, int j) { return N_EMB + m->Lp * N_LAYER_T + j; }
// tensor j of the parameter set that applied layer l uses (layers of a group share one set)
static inline int t_app(const mslt_model* m, int l, int j) { return t_layer(l / m->lpg, j); }
static inline float* Wf(const mslt_model* m, int t) { return m->param + m->table[t].offset; }
static inline float* Gf(const mslt_model* m, int t) { return m->grad + m->table[t].offset; }
// GEMM operand view of a weight matrix: bf16 shadow in bf16 mode, the master itself in fp32 mode
static inline const void* Wg(const mslt_model* m, int t) {
  return m->dtype ? (const void*)(m->shadow + m->table[t].offset) : (const void*)(m->param + m->table[t].offset);
}

struct ProfScope {   // brackets the launches of one kernel class with two events
  mslt_model* m;
  ProfSpan sp;
  bool active;
  ProfScope(mslt_model* m_, int cls, double flops, double bytes) : m(m_), active(m_->prof.on) {
    if (!active) return;
    sp.a = m->prof.get(); sp.b = m->prof.get(); sp.cls = cls; sp.flops = flops; sp.bytes = bytes;
    hipEventRecord(sp.a, m->stream);
  }
  ~ProfScope() {
    if (!active) return;
    hipEventRecord(sp.b, m->stream);
    m->prof.spans.push_back(sp);
  }
};

// ---- workspace ------------------------------------------------------------------------------
struct Bump {
  char* base;
  size_t off;
  template <typename T>
  T* take(size_t bytes) {
    off = rup(off, 256);
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += bytes;
    return p;
  }
};

static size_t carve(mslt_model* m, char* base) {
  Bump b{base, 0};
  const size_t e = m->esz, H = m->H, F = m->F, Tp = m->Tp, Mp = m->Mp, Vp = m->Vp;
  const size_t TH = Tp * H * e, TF = Tp * F * e, MH = Mp * H * e;
  m->shadow = m->dtype ? b.take<bf16>(m->arena_elems * 2) : nullptr;
  m->x0 = b.take<void>(TH); m->xhat0 = b.take<void>(TH); m->rstd0 = b.take<float>(Tp * 4);
  m->xa = b.take<void>(TH); m->xb = b.take<void>(TH);
  m->s_qkv = b.take<void>(3 * TH); m->s_ctx = b.take<void>(TH); m->s_x1 = b.take<void>(TH);
  m->s_g = b.take<void>(TF); m->s_y = b.take<void>(TH);
  m->stash.resize(m->n_stash);
  size_t lse_bytes = (size_t)m->cfg.max_batch * m->nh * m->cfg.max_seq * 4;
  for (int l = 0; l < m->n_stash; ++l) {
    LayerStash& s = m->stash[l];
    s.xout = b.take<void>(TH); s.qkv = b.take<void>(3 * TH); s.ctx = b.take<void>(TH);
    s.xhat1 = b.take<void>(TH); s.x1 = b.take<void>(TH); s.u = b.take<void>(TF); s.g = b.take<void>(TF);
    s.xhat2 = b.take<void>(TH);
    s.lse = b.take<float>(lse_bytes); s.rstd1 = b.take<float>(Tp * 4); s.rstd2 = b.take<float>(Tp * 4);
    s.ctx32 = m->dtype ? b.take<float>(Tp * H * 4) : nullptr;
  }
  const size_t TH32 = m->wide ? Tp * H * 4 : TH;
  m->dxa = b.take<void>(TH32); m->dxb = b.take<void>(TH32);
  for (int i = 0; i < 2; ++i) {
    m->gset[i].d_d = b.take<void>(TH); m->gset[i].d_u = b.take<void>(TF);
    m->gset[i].d_z1 = b.take<void>(TH); m->gset[i].d_qkv = b.take<void>(3 * TH);
    m->gset[i].d_dm = b.take<void>(TH); m->gset[i].d_z1m = b.take<void>(TH);
  }
  m->d_d = m->gset[0].d_d; m->d_u = m->gset[0].d_u; m->d_z1 = m->gset[0].d_z1; m->d_qkv = m->gset[0].d_qkv;
  m->d_dm = m->gset[0].d_dm; m->d_z1m = m->gset[0].d_z1m;
  m->d_x1 = b.take<void>(TH32); m->d_c = b.take<void>(TH);
  m->d_d32 = m->wide ? b.take<float>(TH32) : nullptr;
  m->d_z1_32 = m->wide ? b.take<float>(TH32) : nullptr;
  m->d_z0 = b.take<void>(TH);
  m->delta = b.take<float>(lse_bytes);
  m->pos = b.take<int32_t>((size_t)m->cap * 4); m->lab = b.take<int32_t>((size_t)m->cap * 4);
  m->inv = b.take<int32_t>(Tp * 4); m->counters = b.take<int32_t>(64);
  m->xm = b.take<void>(MH); m->ut = b.take<void>(MH); m->gt = b.take<void>(MH); m->xhat_t = b.take<void>(MH);
  m->hm = b.take<void>(MH); m->d_hm = b.take<void>(MH); m->d_gt = b.take<void>(MH);
  m->d_ut = b.take<void>(MH); m->d_xm = b.take<void>(MH);
  m->c_g = b.take<void>(Mp * F * e); m->c_u = b.take<void>(Mp * F * e); m->c_du = b.take<void>(Mp * F * e);
  m->c_dz2m = b.take<void>(MH); m->c_dz1m = b.take<void>(MH);
  m->c_xhat2 = b.take<void>(MH); m->c_dz2 = b.take<void>(MH); m->c_dc = b.take<void>(MH);
  m->rstd_t = b.take<float>(Mp * 4); m->logits = b.take<float>(Mp * Vp * 4); m->dz = m->logits;   // dZ overwrites the logits in place
  m->row_loss = b.take<float>(Mp * 4);
  m->lse_t = b.take<float>(Mp * 4); m->loss = b.take<float>(64);
  {
    const size_t BH = rup((size_t)m->cfg.max_batch, 128) * H * e;
    m->n_xc = b.take<void>(BH); m->n_p = b.take<void>(BH); m->n_dp = b.take<void>(BH); m->n_du = b.take<void>(BH);
    m->n_dx = b.take<void>(BH);
    m->n_dz = b.take<void>(rup((size_t)m->cfg.max_batch, 128) * 2 * e);
    m->n_z = b.take<float>(rup((size_t)m->cfg.max_batch, 128) * 2 * 4);
  }
  // reduction scratch: the largest of LayerNorm-backward partials, column-sum partials, token-type partials
  size_t rows = Tp > Mp ? Tp : Mp;
  size_t maxN = 3 * H > F ? 3 * H : F;
  if (Vp > maxN) maxN = Vp;
  size_t red = ln_bwd_scratch_floats((int)rows, (int)H);
  size_t cs = colsum_scratch_floats((int)Tp, (int)(3 * H > F ? 3 * H : F));
  size_t cv = colsum_scratch_floats((int)Mp, (int)Vp);
  size_t ct = colsum_scratch_floats((int)Tp, (int)(m->cfg.type_vocab * H));
  if (cs > red) red = cs;
  if (cv > red) red = cv;
  if (ct > red) red = ct;
  m->red_floats = red;
  m->red_scratch = b.take<float>(red * 4);
  m->splitk_floats = m->mfma ? (size_t)1024 * 128 * 128 : 0;
  m->splitk = b.take<float>(m->splitk_floats * 4);
  m->splitk2 = b.take<float>(m->splitk_floats * 4);
  m->red2 = b.take<float>(red * 4);
  {
    // room for one step's partials with every stashed layer trainable at full batch size
    auto dw = [&](size_t Mo, size_t No, size_t rowsK) -> size_t {
      if (!m->mfma || Mo % 128 || No % 128 || rowsK % 64) return 0;
      int sk = pick_splitk((int)Mo, (int)No, (int)rowsK);
      return sk > 1 ? (size_t)sk * Mo * No : 0;
    };
    // (a layer whose four weight-gradient products go out as one grouped launch splits none of them)
    const size_t mn[4][2] = {{3 * H, H}, {H, H}, {F, H}, {H, F}};
    int cnt[3] = {0, 0, 0};
    bool ok[3] = {m->mfma, m->mfma, m->mfma};
    for (auto& q : mn)
      for (int c = 0; c < 3; ++c) {
        ok[c] = ok[c] && q[0] % kGroupTile[c][0] == 0 && q[1] % kGroupTile[c][1] == 0;
        cnt[c] += (int)((q[0] / kGroupTile[c][0]) * (q[1] / kGroupTile[c][1]));
      }
    const bool layers_grouped = group_tile_pick(cnt, ok) >= 0;
    size_t layer = 2 * ln_bwd_scratch_floats((int)Tp, (int)H) + colsum_scratch_floats((int)Tp, (int)(3 * H + F + 2 * H)) +
                   (layers_grouped ? 0 : dw(3 * H, H, Tp) + dw(H, H, Tp) + dw(F, H, Tp) + dw(H, F, Tp));
    size_t head = 2 * ln_bwd_scratch_floats((int)rows, (int)H) + colsum_scratch_floats((int)Mp, (int)(Vp + 2 * H)) +
                  dw(H, H, Mp) + (layers_grouped ? 0 : 2 * (dw(3 * H, H, Mp) + dw(H, H, Mp) + dw(F, H, Mp) + dw(H, F, Mp)));
    m->later_floats = rup((size_t)m->n_stash * layer + head, 64);
    const size_t cap = (size_t)1 << 30;      // 4 GiB; what does not fit is summed at once, as without the arena
    if (m->later_floats > cap) m->later_floats = cap;
    m->later_arena = b.take<float>(m->later_floats * 4);
  }
  m->e_rank = b.take<int32_t>(Tp * 4); m->e_order = b.take<int32_t>(Tp * 4);
  m->e_cnt = b.take<int32_t>(rup(m->V, 4) * 4); m->e_start = b.take<int32_t>(rup(m->V, 4) * 4);
  m->e_partial = b.take<float>(Tp * H * 4);
  m->e_blockcnt = b.take<int32_t>(rup(embed_bwd_int_scratch((int)Tp, m->V), 4) * 4);
  size_t nt = m->table.size();
  size_t nchunks = (size_t)m->first_chunk.back();
  m->o_tensors = b.take<OptTensor>(nt * sizeof(OptTensor));
  m->o_chunk_tensor = b.take<int32_t>(nchunks * 4);
  m->o_tsteps = b.take<int32_t>(nt * 4);
  m->o_chunk_norms = b.take<float>(nchunks * 8);
  m->o_ratio = b.take<float>(nt * 4);
  return rup(b.off, 256);
}

static int check_config(const mslt_config* c) {
  if (!c) return fail(MSLT_ERR_ARG, "config is null");
  if (c->n_layers_max < 1 || c->hidden < 4 || c->n_heads < 1 || c->ffn < 4 || c->vocab < 2 || c->max_pos < 1 ||
      c->type_vocab < 1 || c->max_batch < 1 || c->max_seq < 1 || c->max_predictions < 0 || c->max_trainable_layers < 0)
    return fail(MSLT_ERR_ARG, "config: non-positive dimension");
  if (c->hidden % 4 || c->ffn % 4) return fail(MSLT_ERR_ARG, "config: hidden and ffn must be multiples of 4");
  if (c->hidden > 2048) return fail(MSLT_ERR_ARG, "config: hidden above 2048 is not supported");
  if (c->hidden % c->n_heads) return fail(MSLT_ERR_ARG, "config: hidden is not a multiple of n_heads");
  if (c->hidden / c->n_heads > 128) return fail(MSLT_ERR_ARG, "config: head width above 128 is not supported");
  if (c->type_vocab > 4) return fail(MSLT_ERR_ARG, "config: type_vocab above 4 is not supported");
  if (c->max_seq > c->max_pos) return fail(MSLT_ERR_ARG, "config: max_seq exceeds max_pos");
  if ((long long)c->max_batch * c->max_seq > (1 << 22)) return fail(MSLT_ERR_ARG, "config: max_batch*max_seq too large");
  if (c->precision != 0 && c->precision != 1) return fail(MSLT_ERR_ARG, "config: precision must be 0 or 1");
  if (!(c->ln_eps >= 0.f)) return fail(MSLT_ERR_ARG, "config: ln_eps must be >= 0");
  if (c->layers_per_group < 0 || (c->layers_per_group > 1 && c->n_layers_max % c->layers_per_group))
    return fail(MSLT_ERR_ARG, "config: n_layers_max must be a multiple of layers_per_group");
  if (c->layers_per_group > 1 && c->max_trainable_layers % c->layers_per_group)
    return fail(MSLT_ERR_ARG, "config: max_trainable_layers must be a multiple of layers_per_group");
  return MSLT_OK;
}

static void setup_dims(mslt_model* m, const mslt_config* cfg) {
  m->cfg = *cfg;
  m->dtype = cfg->precision;
  m->esz = cfg->precision ? 2 : 4;
  m->H = cfg->hidden; m->F = cfg->ffn; m->V = cfg->vocab; m->nh = cfg->n_heads; m->dh = cfg->hidden / cfg->n_heads;
  m->L = cfg->n_layers_max;
  m->nsp = cfg->with_nsp != 0;
  m->lpg = cfg->layers_per_group > 1 ? cfg->layers_per_group : 1;
  m->Lp = m->L / m->lpg;
  m->Vp = (int)rup(cfg->vocab, 128);
  // frozen layers keep nothing (Section 3.2): the stash is sized by how many layers one step may train
  m->n_stash = cfg->max_trainable_layers > 0 && cfg->max_trainable_layers < m->L ? cfg->max_trainable_layers : m->L;
  m->stash_base = 0;
  int T = cfg->max_batch * cfg->max_seq;
  m->cap = cfg->max_predictions > 0 && cfg->max_predictions < T ? cfg->max_predictions : T;
  m->Tp = (int)rup(T, 128);
  m->Mp = (int)rup(m->cap, 128);
  m->mfma = cfg->precision == 1 && cfg->hidden % 128 == 0 && cfg->ffn % 128 == 0;
  m->wide = cfg->precision == 1;
  build_table(m);
}

extern "C" int mslt_query_sizes(const mslt_config* cfg, size_t* param_bytes, size_t* grad_bytes, size_t* opt_state_bytes,
                                size_t* workspace_bytes) {
  int rc = check_config(cfg);
  if (rc) return rc;
  mslt_model m{};
  setup_dims(&m, cfg);
  size_t ws = carve(&m, nullptr);
  if (param_bytes) *param_bytes = m.arena_elems * 4;
  if (grad_bytes) *grad_bytes = m.arena_elems * 4;
  if (opt_state_bytes) *opt_state_bytes = m.arena_elems * 8;
  if (workspace_bytes) *workspace_bytes = ws;
  return MSLT_OK;
}

extern "C" int mslt_init_model(const mslt_config* cfg, void* param_arena, void* grad_arena, void* opt_arena,
                               void* workspace, void* hip_stream, mslt_model** out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!param_arena || !grad_arena || !opt_arena || !workspace || !out) return fail(MSLT_ERR_ARG, "null arena or out");
  for (void* p : {param_arena, grad_arena, opt_arena, workspace})
    if (reinterpret_cast<uintptr_t>(p) % 256) return fail(MSLT_ERR_ARG, "arena not 256-byte aligned");
  mslt_model* m = new mslt_model{};
  setup_dims(m, cfg);
  m->stream = reinterpret_cast<hipStream_t>(hip_stream);
  m->param = (float*)param_arena;
  m->grad = (float*)grad_arena;
  m->mom1 = (float*)opt_arena;
  m->mom2 = m->mom1 + m->arena_elems;
  m->ws = (char*)workspace;
  m->ws_bytes = carve(m, m->ws);
  m->have_grads = false;
  m->last_prefix = nullptr;
  {
    // the device that holds the arenas is the one whose scratch copy this model uses
    hipPointerAttribute_t at;
    hipError_t pe = hipPointerGetAttributes(&at, param_arena);
    if (pe != hipSuccess) { delete m; return fail(MSLT_ERR_HIP, "hipPointerGetAttributes(param_arena): %s", hipGetErrorString(pe)); }
    int prc = static_scratch_for(at.device, &m->static_scratch);
    if (prc) { delete m; return prc; }
  }
  hipError_t e;
#define INIT_TRY(expr)                                                                  \
  if ((e = (expr)) != hipSuccess) {                                                     \
    delete m;                                                                           \
    return fail(MSLT_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e));                   \
  }
  INIT_TRY(hipHostMalloc((void**)&m->h_counters, 64, hipHostMallocDefault));
  INIT_TRY(hipStreamCreateWithFlags(&m->side, hipStreamNonBlocking));
  INIT_TRY(hipEventCreateWithFlags(&m->ev_fork, hipEventDisableTiming));
  INIT_TRY(hipEventCreateWithFlags(&m->ev_join, hipEventDisableTiming));
  m->side_forked = false;
  INIT_TRY(hipEventCreateWithFlags(&m->ev_scan, hipEventDisableTiming));
  for (int i = 0; i < 2; ++i) {
    INIT_TRY(hipEventCreateWithFlags(&m->ev_set[i], hipEventDisableTiming));
    m->set_busy[i] = false;
  }
  m->h_loss = reinterpret_cast<float*>(m->h_counters + 8);
  INIT_TRY(fill_zero(m->param, m->arena_elems * 4, m->stream));
  INIT_TRY(fill_zero(m->grad, m->arena_elems * 4, m->stream));
  INIT_TRY(fill_zero(m->mom1, m->arena_elems * 8, m->stream));
  INIT_TRY(fill_zero(m->ws, m->ws_bytes, m->stream));
  // optimizer tables
  std::vector<OptTensor> ot(m->table.size());
  std::vector<int32_t> ct((size_t)m->first_chunk.back());
  for (size_t i = 0; i < m->table.size(); ++i) {
    ot[i].offset = m->table[i].offset;
    ot[i].count = m->table[i].count;
    ot[i].decays = m->table[i].decays;
    ot[i].first_chunk = m->first_chunk[i];
    ot[i].n_chunks = m->first_chunk[i + 1] - m->first_chunk[i];
    ot[i].pad_ = 0;
    for (int c = m->first_chunk[i]; c < m->first_chunk[i + 1]; ++c) ct[c] = (int32_t)i;
  }
  INIT_TRY(hipMemcpyAsync(m->o_tensors, ot.data(), ot.size() * sizeof(OptTensor), hipMemcpyHostToDevice, m->stream));
  INIT_TRY(hipMemcpyAsync(m->o_chunk_tensor, ct.data(), ct.size() * 4, hipMemcpyHostToDevice, m->stream));
  INIT_TRY(hipStreamSynchronize(m->stream));
#undef INIT_TRY
  *out = m;
  return MSLT_OK;
}

extern "C" int mslt_destroy(mslt_model* m) {
  if (!m) return MSLT_OK;
  hipStreamSynchronize(m->stream);
  if (m->side) { hipStreamSynchronize(m->side); hipStreamDestroy(m->side); }
  if (m->ev_fork) hipEventDestroy(m->ev_fork);
  if (m->ev_join) hipEventDestroy(m->ev_join);
  if (m->ev_scan) hipEventDestroy(m->ev_scan);
  for (int i = 0; i < 2; ++i)
    if (m->ev_set[i]) hipEventDestroy(m->ev_set[i]);
  if (m->h_counters) hipHostFree(m->h_counters);
  for (auto& sp : m->prof.spans) { hipEventDestroy(sp.a); hipEventDestroy(sp.b); }
  for (auto e : m->prof.pool) hipEventDestroy(e);
  delete m;
  return MSLT_OK;
}

extern "C" const char* mslt_last_error(void) { return g_err.c_str(); }

extern "C" int mslt_sync(const mslt_model* m) {
  if (!m) return fail(MSLT_ERR_ARG, "model is null");
  HIP_TRY(hipStreamSynchronize(m->stream));
  return MSLT_OK;
}

extern "C" int mslt_tensor_table(const mslt_model* m, int* n, const mslt_tensor_desc** out) {
  if (!m || !n || !out) return fail(MSLT_ERR_ARG, "null argument");
  *n = (int)m->table.size();
  *out = m->table.data();
  return MSLT_OK;
}

static int refresh_shadow(mslt_model* m, size_t off, size_t count) {
  if (!m->dtype) return MSLT_OK;
  HIP_TRY(cast_f32_to_bf16(m->param + off, m->shadow + off, count, m->stream));
  return MSLT_OK;
}

extern "C" int mslt_load_params(mslt_model* m, const float* host, size_t n_floats) {
  if (!m || !host) return fail(MSLT_ERR_ARG, "null argument");
  if (n_floats != m->packed_count)
    return fail(MSLT_ERR_ARG, "load_params: expected %zu floats, got %zu", m->packed_count, n_floats);
  size_t o = 0;
  for (auto& d : m->table) {
    HIP_TRY(hipMemcpyAsync(m->param + d.offset, host + o, d.count * 4, hipMemcpyHostToDevice, m->stream));
    o += d.count;
  }
  int rc = refresh_shadow(m, 0, m->arena_elems);
  if (rc) return rc;
  HIP_TRY(hipStreamSynchronize(m->stream));
  return MSLT_OK;
}

extern "C" int mslt_get_params(const mslt_model* m, float* host, size_t n_floats) {
  if (!m || !host) return fail(MSLT_ERR_ARG, "null argument");
  if (n_floats != m->packed_count)
    return fail(MSLT_ERR_ARG, "get_params: expected %zu floats, got %zu", m->packed_count, n_floats);
  size_t o = 0;
  for (auto& d : m->table) {
    HIP_TRY(hipMemcpyAsync(host + o, m->param + d.offset, d.count * 4, hipMemcpyDeviceToHost, m->stream));
    o += d.count;
  }
  HIP_TRY(hipStreamSynchronize(m->stream));
  return MSLT_OK;
}

// ---- GEMM dispatch --------------------------------------------------------------------------
// space for partial sums that are added at the end of the step, or null when the arena is used up or off
static float* later_take(mslt_model* m, size_t floats) {
  floats = rup(floats, 64);
  if (!m->later_on || m->later_used + floats > m->later_floats) return nullptr;
  float* p = m->later_arena + m->later_used;
  m->later_used += floats;
  return p;
}
static int later_flush(mslt_model* m) {
  if (m->later.empty()) return MSLT_OK;
  double bytes = 0.0;
  for (const ReduceJob& j : m->later) bytes += 4.0 * j.N * (j.n_partials + 1.0);
  ProfScope ps(m, PC_REDUCE, 0.0, bytes);
  HIP_TRY(reduce_batch(m->later.data(), (int)m->later.size(), m->stream));
  m->later.clear();
  return MSLT_OK;
}
static int pick_splitk(int M, int N, int K) {
  // Few output tiles and a long contraction: split k.  The factor minimises a small cost model
  // fitted to measured launches (microseconds): one 64-wide k tile of a 128x128 workgroup takes
  // about 0.65 us while a CU holds one workgroup (up to 256 workgroups) and 0.95 us once it holds
  // two (up to 512); workgroups beyond 512 run as a second round; the fp32 partials cost their
  // write plus read at about 5 TB/s (they stay in the last-level cache) and the summing kernel a
  // fixed 5 us.
  const int tiles = (M / 128) * (N / 128), nkt = K / 64;
  if (nkt < 16) return 1;
  double best = 0.0;
  int pick = 1;
  for (int s = 1; s <= 16 && nkt / s >= 4; ++s) {
    const int wgs = tiles * s;
    const double it = (double)((nkt + s - 1) / s);
    const int full = wgs / 512, rem = wgs % 512;
    double t;
    if (full == 0) t = it * (rem <= 256 ? 0.65 : 0.95);
    else t = it * 0.95 * full + (rem ? it * (rem <= 256 ? 0.65 : 0.95) : 0.0);
    if (s > 1) t += 5.0 + (double)s * M * N * 8.0 / 5.0e6;
    if (s == 1 || t < best) { best = t; pick = s; }
  }
  return pick;
}
// Weight-gradient products and bias column sums only consume what the main stream has already
// produced and write tensors nothing else touches, so they run on a side stream next to the
// data-gradient chain (which is what the layer below waits for).  side_fork makes the side stream
// see the main stream's work so far; side_join makes the main stream wait for the side stream and
// is called before any buffer the side work reads is overwritten.  Off while event profiling.
// again: nothing the side work reads was produced on the main stream since the previous fork, so
// that fork's event still covers it (recording an event costs the recording stream about 6 us).
static int side_fork(mslt_model* m, hipStream_t* st, float** partials, float** red, bool again = false) {
  *st = m->stream; *partials = m->splitk; *red = m->red_scratch;
  if (m->prof.on) return MSLT_OK;
  if (!(again && m->side_forked)) {
    HIP_TRY(hipEventRecord(m->ev_fork, m->stream));
    HIP_TRY(hipStreamWaitEvent(m->side, m->ev_fork, 0));
  }
  m->side_forked = true;
  *st = m->side; *partials = m->splitk2; *red = m->red2;
  return MSLT_OK;
}
static int side_join(mslt_model* m) {
  if (!m->side_forked) return MSLT_OK;
  HIP_TRY(hipEventRecord(m->ev_join, m->side));
  HIP_TRY(hipStreamWaitEvent(m->stream, m->ev_join, 0));
  m->side_forked = false;
  m->set_busy[0] = m->set_busy[1] = false;
  return MSLT_OK;
}
// Layer l's backward uses gradient-buffer set l & 1: wait for the side work of layer l + 2, the
// last reader of that set, before anything is written there.
static int layer_backward_begin(mslt_model* m, int l) {
  const int p = l & 1;
  // the top layer of a group is the first to run backward and writes its set's gradients; the
  // layers of the group below it add theirs (the two streams keep the order per tensor)
  m->acc_now = (l % m->lpg) != m->lpg - 1;
  if (m->set_busy[p]) {
    HIP_TRY(hipStreamWaitEvent(m->stream, m->ev_set[p], 0));
    m->set_busy[p] = false;
  }
  m->d_d = m->gset[p].d_d; m->d_u = m->gset[p].d_u; m->d_z1 = m->gset[p].d_z1; m->d_qkv = m->gset[p].d_qkv;
  m->d_dm = m->gset[p].d_dm; m->d_z1m = m->gset[p].d_z1m;
  m->side_collect = true;
  return MSLT_OK;
}
static int side_flush(mslt_model* m);
static int layer_backward_end(mslt_model* m, int l) {
  if (int rc = side_flush(m)) return rc;
  m->acc_now = 0;
  if (!m->side_forked) return MSLT_OK;
  HIP_TRY(hipEventRecord(m->ev_set[l & 1], m->side));
  m->set_busy[l & 1] = true;
  return MSLT_OK;
}

// Tile shape and split factor of the large-tile kernel for one product, or false when the 128-wide
// kernel should take it.  One workgroup occupies a compute unit, so what counts is how full the rounds
// of 256 workgroups are: a 256x256 tile moves the fewest bytes per FLOP (relative rate 1), the two
// half-size tiles about 0.88 of it (measured on the step's shapes), and splitting k costs the partial
// sums and a second launch (factor 0.9).
struct RingPlan { int tm, tn, rk, sk; };
static bool ring_plan(const GemmDesc& d, bool allow_splitk, size_t partial_floats, RingPlan* out) {
  static const int cand[3][2] = {{256, 256}, {128, 256}, {256, 128}};
  const int rk = 64;
  if (d.K % rk) return false;
  double best = 0.0;
  for (auto& c : cand) {
    if (!gemm_ring_supported(d, c[0], c[1], rk)) continue;
    const int tiles = (d.M / c[0]) * (d.N / c[1]), nk = d.K / rk;
    int sk = 1;
    if (allow_splitk && tiles < 192) {
      sk = 256 / tiles;
      if (sk > 8) sk = 8;
      if (sk > nk / 4) sk = nk / 4;
      while (sk > 1 && (size_t)sk * d.M * d.N > partial_floats) --sk;
      if (sk < 1) sk = 1;
    }
    const int wgs = tiles * sk, rounds = (wgs + 255) / 256;
    double score = (c[0] == 256 && c[1] == 256 ? 1.0 : 0.88) * wgs / (rounds * 256.0) * (sk > 1 ? 0.9 : 1.0);
    if (score > best) { best = score; *out = RingPlan{c[0], c[1], rk, sk}; }
  }
  return best > 0.0;
}

// sum_later: the result is a parameter gradient nothing reads before the optimizer, so a split product may
// leave its partial sums for the batch at the end of the step
static int run_gemm(mslt_model* m, const GemmDesc& d, bool allow_splitk = false, hipStream_t st = nullptr,
                    float* partials = nullptr, bool sum_later = false) {
  if (!st) { st = m->stream; partials = m->splitk; }
  const bool use_mfma = m->mfma && gemm_mfma_supported(d);
  const double out_esz = d.epi.out_f32 ? 4.0 : (double)m->esz;
  ProfScope ps(m, !use_mfma ? PC_GEMM_SIMT : (d.a_kcontig ? (d.b_kcontig ? PC_GEMM_NT : PC_GEMM_NN) : PC_GEMM_TN),
               2.0 * d.M * d.N * d.K, ((double)d.M * d.K + (double)d.N * d.K) * m->esz + (double)d.M * d.N * out_esz);
  // Which kernel takes which product was settled by measuring whole steps (two kernel chains run side by
  // side there, so a kernel's footprint counts as much as its own speed): forward-type products (both
  // operands k-contiguous) go to the large-tile kernel; weight-gradient products (both operands k-strided)
  // to its 128x128 form, two workgroups per compute unit, fed by direct loads and transposing LDS reads;
  // data-gradient products stay on the 128-wide register-staged kernel, except the one with a wide output (the
  // gradient of the feed-forward layer's hidden activation), which gains on the large tiles in the step as well.
  RingPlan rp;
  const bool nt = d.a_kcontig && d.b_kcontig, tn = !d.a_kcontig && !d.b_kcontig;
  const bool nn_wide = d.a_kcontig && !d.b_kcontig && d.N >= 2048 && d.M >= 4096;
  if (use_mfma && tn && gemm_ring_supported(d, 128, 128, 64)) {
    int sk = allow_splitk ? pick_splitk(d.M, d.N, d.K) : 1;
    float* kept = nullptr;
    if (sk > 1 && sum_later && d.epi.out_f32 && d.epi.ldo == d.N && !d.epi.bias && d.epi.act == EPI_NONE && !d.epi.drop.thr &&
        !d.epi.out2)
      kept = later_take(m, (size_t)sk * d.M * d.N);
    if (kept) {
      HIP_TRY(gemm_ring(d, 128, 128, 64, sk, kept, st, true));
      m->later.push_back(reduce_job(kept, (float*)d.epi.out, sk, (size_t)d.M * d.N, d.epi.accumulate != 0, true));
    } else {
      while (sk > 1 && (size_t)sk * d.M * d.N > m->splitk_floats) --sk;
      HIP_TRY(gemm_ring(d, 128, 128, 64, sk, partials, st));
    }
  } else if (use_mfma && (nt || nn_wide) && ring_plan(d, allow_splitk, m->splitk_floats, &rp)) {
    HIP_TRY(gemm_ring(d, rp.tm, rp.tn, rp.rk, rp.sk, partials, st));
  } else if (use_mfma) {
    int sk = allow_splitk ? pick_splitk(d.M, d.N, d.K) : 1;
    while (sk > 1 && (size_t)sk * d.M * d.N > m->splitk_floats) --sk;
    HIP_TRY(gemm_mfma(d, sk, partials, st));
  } else {
    HIP_TRY(gemm_simt(m->dtype, d, st));
  }
  return MSLT_OK;
}
#define RC(expr)          \
  do {                    \
    int rc__ = (expr);    \
    if (rc__) return rc__; \
  } while (0)

// keep decisions of one dropout site of one layer in the current step (thr 0 = dropout off)
// first_elem: index, in the whole tensor, of the element the kernel will call element 0 (a multiple
// of 4).  The decision of quad q comes from mix64(key + q * DROP_GOLDEN), so an offset folds into the key.
static DropSpec dspec(const mslt_model* m, int layer, int site, uint64_t first_elem = 0) {
  DropSpec d;
  if (m->drop_thr) {
    d.key = drop_key(m->drop_seed, m->drop_step, layer, site) + (first_elem >> 2) * DROP_GOLDEN;
    d.thr = m->drop_thr;
    d.scale = m->drop_scale;
  }
  return d;
}

// Y[rows,N] = X[rows,K] W[N,K]^T + bias, optional GELU (gelu_grad_out then receives GELU' of the pre-activation),
// optional dropout of the result
static int linear_fwd(mslt_model* m, const void* X, int rows, int K, const void* W, int N, const float* bias, void* Y,
                      int out_f32, int ldo, int act, void* gelu_grad_out, const DropSpec& drop = DropSpec(),
                      hipStream_t st = nullptr) {
  GemmDesc d;
  d.epi.drop = drop; d.epi.drop_ld = N;
  d.A = X; d.lda = K; d.a_kcontig = 1; d.M = rows;
  d.B = W; d.ldb = K; d.b_kcontig = 1; d.N = N; d.K = K;
  d.epi.out = Y; d.epi.ldo = ldo; d.epi.out_f32 = out_f32; d.epi.bias = bias; d.epi.act = act; d.epi.out2 = gelu_grad_out;
  return run_gemm(m, d, false, st);
}
// dX[rows,K] = dY[rows,N] W[N,K]  (+ addend | * gelu'(U))
// aux_f32 / out_f32: the addend / the result is fp32 whatever the activation type (wide residual gradients)
static int linear_bwd_input(mslt_model* m, const void* dY, int rows, int N, int ldy, const void* W, int K, void* dX,
                            int act, const void* aux, bool allow_splitk = true, int aux_f32 = 0, int out_f32 = 0) {
  GemmDesc d;
  d.A = dY; d.lda = ldy; d.a_kcontig = 1; d.M = rows;
  d.B = W; d.ldb = K; d.b_kcontig = 0; d.N = K; d.K = N;
  d.epi.out = dX; d.epi.ldo = K; d.epi.act = act; d.epi.aux = aux; d.epi.ldaux = K;
  d.epi.aux_f32 = aux_f32; d.epi.out_f32 = out_f32;
  return run_gemm(m, d, allow_splitk);
}
// dW[N,K] = dY[rows,N]^T X[rows,K]   (fp32 out, contraction over rows)
// sum_later = false for a tensor that something else writes or adds to later in the same step
static int linear_bwd_weight(mslt_model* m, const void* dY, int rows, int N, int ldy, const void* X, int K, float* dW,
                             bool again = false, bool sum_later = true) {
  GemmDesc d;
  d.A = dY; d.lda = ldy; d.a_kcontig = 0; d.M = N;
  d.B = X; d.ldb = K; d.b_kcontig = 0; d.N = K; d.K = rows;
  d.epi.out = dW; d.epi.ldo = K; d.epi.out_f32 = 1; d.epi.accumulate = m->acc_now;
  if (m->side_collect) {
    m->side_dw.push_back(d);
    return MSLT_OK;
  }
  hipStream_t st; float *partials, *red;
  RC(side_fork(m, &st, &partials, &red, again));
  return run_gemm(m, d, true, st, partials, sum_later);
}

static int ln_forward(mslt_model* m, const void* a, const void* r, const float* g, const float* b, void* out, LnStash st,
                      int rows, hipStream_t stream = nullptr) {
  ProfScope ps(m, PC_LN_FWD, 0.0, (double)rows * m->H * m->esz * (2.0 + (r ? 1.0 : 0.0) + (st.xhat ? 1.0 : 0.0)));
  HIP_TRY(add_ln_fwd(m->dtype, a, r, g, b, m->cfg.ln_eps, out, st, rows, m->H, stream ? stream : m->stream));
  return MSLT_OK;
}

// ---- one encoder layer ----------------------------------------------------------------------
// Every kernel of the forward pass works on token rows (or whole sequences) independently of the
// other rows, so a layer can run on a range of the batch's sequences: FwdPart names the range and
// the stream.  Without a part the layer runs on all Tr rows on the main stream.
struct FwdPart {
  int b0, nb;        // sequences [b0, b0 + nb)
  hipStream_t st;
};
static int layer_forward(mslt_model* m, int l, const mslt_batch* bt, int Tr, const void* Xin, void* Xout,
                         const LayerStash* st, const FwdPart* part = nullptr) {
  const int H = m->H, F = m->F, S = bt->seq;
  const int nb = part ? part->nb : bt->batch;
  const size_t r0 = part ? (size_t)part->b0 * S : 0;          // first token row
  const int rows = part ? nb * S : Tr;
  hipStream_t s = part ? part->st : m->stream;
  auto at = [&](const void* p, size_t width_bytes) -> void* {   // row r0 of a [rows, width] array (null stays null)
    return p ? (void*)((char*)p + r0 * width_bytes) : nullptr;
  };
  const size_t e = m->esz;
  void* qkv = at(st ? st->qkv : m->s_qkv, 3 * H * e);
  void* ctx = at(st ? st->ctx : m->s_ctx, H * e);
  void* x1 = at(st ? st->x1 : m->s_x1, H * e);
  void* g = at(st ? st->g : m->s_g, F * e);
  void* y = at(m->s_y, H * e);
  const void* xin = at(Xin, H * e);
  void* xout = at(Xout, H * e);
  RC(linear_fwd(m, xin, rows, H, Wg(m, t_app(m, l, L_WQ)), 3 * H, Wf(m, t_app(m, l, L_BQ)), qkv, 0, 3 * H, EPI_NONE, nullptr,
                DropSpec(), s));
  AttnDesc a{qkv, ctx, st ? (float*)at(st->lse, (size_t)m->nh * 4) : nullptr, bt->attn_mask + r0, nb, S, m->nh, m->dh,
             m->cfg.mask_bias, dspec(m, l, SITE_ATTN_PROBS, r0 * m->nh * S), st ? (float*)at(st->ctx32, H * 4) : nullptr};
  {
    const double TS = (double)nb * S;
    ProfScope ps(m, PC_ATTN_FWD, 4.0 * TS * S * H, 4.0 * TS * H * m->esz);
    if (m->dtype == 1 && attention_mfma_supported(S, m->dh))
      HIP_TRY(attention_fwd_mfma(a, s));
    else
      HIP_TRY(attention_fwd_simple(m->dtype, a, s));
  }
  RC(linear_fwd(m, ctx, rows, H, Wg(m, t_app(m, l, L_WO)), H, Wf(m, t_app(m, l, L_BO)), y, 0, H, EPI_NONE, nullptr,
                dspec(m, l, SITE_ATTN_OUT, r0 * H), s));
  LnStash s1, s2;
  if (st) {
    s1.xhat = at(st->xhat1, H * e); s1.rstd = (float*)at(st->rstd1, 4);
    s2.xhat = at(st->xhat2, H * e); s2.rstd = (float*)at(st->rstd2, 4);
  }
  RC(ln_forward(m, y, xin, Wf(m, t_app(m, l, L_LN1G)), Wf(m, t_app(m, l, L_LN1B)), x1, s1, rows, s));
  RC(linear_fwd(m, x1, rows, H, Wg(m, t_app(m, l, L_W1)), F, Wf(m, t_app(m, l, L_B1)), g, 0, F, EPI_GELU,
                st ? at(st->u, F * e) : nullptr, DropSpec(), s));
  RC(linear_fwd(m, g, rows, F, Wg(m, t_app(m, l, L_W2)), H, Wf(m, t_app(m, l, L_B2)), y, 0, H, EPI_NONE, nullptr,
                dspec(m, l, SITE_FFN_OUT, r0 * H), s));
  RC(ln_forward(m, y, x1, Wf(m, t_app(m, l, L_LN2G)), Wf(m, t_app(m, l, L_LN2B)), xout, s2, rows, s));
  return MSLT_OK;
}

static int bias_grad(mslt_model* m, const void* dY, int ld, int rows, int N, float* out, bool again = false) {
  if (m->side_collect) {
    m->side_cs.push_back({dY, ld, rows, N, out, m->acc_now});
    return MSLT_OK;
  }
  ProfScope ps(m, PC_COLSUM, (double)rows * N, (double)rows * N * m->esz);
  hipStream_t st; float *partials, *red;
  RC(side_fork(m, &st, &partials, &red, again));
  if (float* kept = later_take(m, colsum_scratch_floats(rows, N))) {
    ReduceJob j;
    HIP_TRY(colsum(m->dtype, dY, ld, rows, N, out, kept, st, m->acc_now, &j));
    m->later.push_back(j);
    return MSLT_OK;
  }
  HIP_TRY(colsum(m->dtype, dY, ld, rows, N, out, red, st, m->acc_now));
  return MSLT_OK;
}
// dzsum (may be null): column sums of dz = bias gradient of the linear layer feeding this LayerNorm
// dy_f32: dy is fp32; dz32 (or null): fp32 copy of dz (both only in bf16 mode, see mslt_model::wide)
static int ln_backward(mslt_model* m, const void* dy, const void* xhat, const float* rstd, const float* g, void* dz,
                       float* dg, float* db, float* dzsum, int rows, const LnBwdDrop& dd_in = LnBwdDrop(), int dy_f32 = 0,
                       float* dz32 = nullptr) {
  ProfScope ps(m, PC_LN_BWD, 0.0, ((dd_in.out.thr ? 3.0 : 2.0) * m->esz + (dy_f32 ? 4.0 : (double)m->esz) + (dz32 ? 4.0 : 0.0)) *
                                      rows * m->H);
  LnBwdDrop dd = dd_in;
  dd.accumulate = m->acc_now;
  if (float* kept = later_take(m, ln_bwd_scratch_floats(rows, m->H))) {
    ReduceJob j[3];
    int n = 0;
    HIP_TRY(ln_bwd(m->dtype, dy, xhat, rstd, g, dz, dg, db, dzsum, kept, rows, m->H, dd, m->stream, dy_f32, dz32, j, &n));
    m->later.insert(m->later.end(), j, j + n);
    return MSLT_OK;
  }
  HIP_TRY(ln_bwd(m->dtype, dy, xhat, rstd, g, dz, dg, db, dzsum, m->red_scratch, rows, m->H, dd, m->stream, dy_f32, dz32));
  return MSLT_OK;
}

// Queues what a layer's backward has collected.  The weight-gradient products go out as grouped launches of
// the large-tile kernel's 128x128 form when every one of them fits it (together they fill the chip, so none
// splits its contraction and no partial sums travel through memory), one by one otherwise.
static int side_flush(mslt_model* m) {
  m->side_collect = false;
  if (m->side_dw.empty() && m->side_cs.empty()) return MSLT_OK;
  const int acc_keep = m->acc_now;
  bool grouped = m->mfma && !m->side_dw.empty();
  int cnt[3] = {0, 0, 0};
  bool ok[3] = {true, true, true};
  for (const GemmDesc& d : m->side_dw) {
    grouped = grouped && gemm_mfma_supported(d);
    for (int c = 0; c < 3; ++c) {
      ok[c] = ok[c] && gemm_ring_supported(d, kGroupTile[c][0], kGroupTile[c][1], 64);
      cnt[c] += (d.M / kGroupTile[c][0]) * (d.N / kGroupTile[c][1]);
    }
  }
  const int pick = grouped ? group_tile_pick(cnt, ok) : -1;
  grouped = pick >= 0;
  bool forked = false;
  hipStream_t st; float *partials, *red;
  if (grouped) {
    RC(side_fork(m, &st, &partials, &red));
    forked = true;
    const int gmax = gemm_ring_group_max();
    for (size_t at = 0; at < m->side_dw.size(); at += gmax) {
      const int n = (int)std::min((size_t)gmax, m->side_dw.size() - at);
      double flops = 0.0, bytes = 0.0;
      for (int i = 0; i < n; ++i) {
        const GemmDesc& d = m->side_dw[at + i];
        flops += 2.0 * d.M * d.N * d.K;
        bytes += ((double)d.M * d.K + (double)d.N * d.K) * m->esz + (double)d.M * d.N * 4.0;
      }
      ProfScope ps(m, PC_GEMM_TN, flops, bytes);
      HIP_TRY(gemm_ring_grouped_tn(&m->side_dw[at], n, kGroupTile[pick][0], kGroupTile[pick][1], st));
    }
  } else {
    for (const GemmDesc& d : m->side_dw) {
      RC(side_fork(m, &st, &partials, &red, forked));
      forked = true;
      RC(run_gemm(m, d, true, st, partials, true));
    }
  }
  for (const auto& c : m->side_cs) {
    RC(side_fork(m, &st, &partials, &red, forked));
    forked = true;
    m->acc_now = c.accumulate;
    ProfScope ps(m, PC_COLSUM, (double)c.rows * c.N, (double)c.rows * c.N * m->esz);
    if (float* kept = later_take(m, colsum_scratch_floats(c.rows, c.N))) {
      ReduceJob j;
      HIP_TRY(colsum(m->dtype, c.dY, c.ld, c.rows, c.N, c.out, kept, st, c.accumulate, &j));
      m->later.push_back(j);
    } else {
      HIP_TRY(colsum(m->dtype, c.dY, c.ld, c.rows, c.N, c.out, red, st, c.accumulate));
    }
  }
  m->acc_now = acc_keep;
  m->side_dw.clear();
  m->side_cs.clear();
  return MSLT_OK;
}

// Backward of the row-local upper part of a layer (LayerNorm 2, FFN, LayerNorm 1, output
// projection), on `rows` rows.  Used on all token rows, or on the compacted predicted rows of the
// top layer (see layer_backward_top).
struct UpperRows {
  const void *xhat2, *g, *u, *x1, *xhat1, *ctx;  // stash rows
  const float *rstd2, *rstd1;
  void *dz2, *du, *dx1, *dz1, *dc;               // gradient buffers
  int rows;
  void *dz2m, *dz1m;                             // dz2, dz1 times the dropout keep factors (used when dropout is on)
  const int32_t* rowmap;                         // token row of each compacted row, or null
  int n_mapped;
  // wide residual branch (dense rows in bf16 mode): dXout and dx1 are fp32, dz2_32 / dz1_32 receive fp32 copies
  int wide;
  float *dz2_32, *dz1_32;
};
static int layer_backward_upper(mslt_model* m, int l, const void* dXout, const UpperRows& r) {
  const int H = m->H, F = m->F, R = r.rows;
  // With dropout the gradient of a dropped linear output (dy2, dy1) is dz times the keep factors,
  // while the residual branch takes dz itself; without it they are the same buffer.
  LnBwdDrop d2, d1;
  d2.out = dspec(m, l, SITE_FFN_OUT); d2.dzm = r.dz2m; d2.rowmap = r.rowmap; d2.n_mapped = r.n_mapped;
  d1.out = dspec(m, l, SITE_ATTN_OUT); d1.dzm = r.dz1m; d1.rowmap = r.rowmap; d1.n_mapped = r.n_mapped;
  const void* dy2 = d2.out.thr ? r.dz2m : r.dz2;
  const void* dy1 = d1.out.thr ? r.dz1m : r.dz1;
  RC(ln_backward(m, dXout, r.xhat2, r.rstd2, Wf(m, t_app(m, l, L_LN2G)), r.dz2, Gf(m, t_app(m, l, L_LN2G)),
                 Gf(m, t_app(m, l, L_LN2B)), Gf(m, t_app(m, l, L_B2)), R, d2, r.wide, r.dz2_32));
  // one fork for the three side products of the feed-forward part (W2's waits for the data gradient
  // of the second linear layer: the side stream has a backlog anyway, and every fork stalls this stream)
  RC(linear_bwd_input(m, dy2, R, H, H, Wg(m, t_app(m, l, L_W2)), F, r.du, EPI_MUL, r.u));
  RC(linear_bwd_weight(m, dy2, R, H, H, r.g, F, Gf(m, t_app(m, l, L_W2))));
  RC(linear_bwd_weight(m, r.du, R, F, F, r.x1, H, Gf(m, t_app(m, l, L_W1)), true));
  RC(bias_grad(m, r.du, F, R, F, Gf(m, t_app(m, l, L_B1)), true));
  RC(linear_bwd_input(m, r.du, R, F, F, Wg(m, t_app(m, l, L_W1)), H, r.dx1, EPI_ADD, r.wide ? (const void*)r.dz2_32 : r.dz2, true,
                      r.wide, r.wide));
  RC(ln_backward(m, r.dx1, r.xhat1, r.rstd1, Wf(m, t_app(m, l, L_LN1G)), r.dz1, Gf(m, t_app(m, l, L_LN1G)),
                 Gf(m, t_app(m, l, L_LN1B)), Gf(m, t_app(m, l, L_BO)), R, d1, r.wide, r.dz1_32));
  RC(linear_bwd_weight(m, dy1, R, H, H, r.ctx, H, Gf(m, t_app(m, l, L_WO))));
  RC(linear_bwd_input(m, dy1, R, H, H, Wg(m, t_app(m, l, L_WO)), H, r.dc, EPI_NONE, nullptr));
  return MSLT_OK;
}
// Attention backward and the QKV projection backward, from dC and dz1 (both [Tr, H], all token rows).
// dXin: where to put the gradient w.r.t. the layer input, or null when nothing below needs it
// (the block below is frozen: Section 3.1).
// resid: dz1, the residual addend of dXin (fp32 if resid_f32); dXin itself is fp32 in bf16 mode (mslt_model::wide).
static int layer_backward_lower(mslt_model* m, int l, const mslt_batch* bt, int T, int Tr, const void* Xin, void* dXin,
                                const void* resid, int resid_f32) {
  const int H = m->H;
  const LayerStash& st = m->stash[l - m->stash_base];
  hipStream_t s = m->stream;
  AttnBwdDesc a{st.qkv, st.ctx, m->d_c, st.lse, m->delta, m->d_qkv, bt->attn_mask, bt->batch, bt->seq, m->nh, m->dh,
                m->cfg.mask_bias, dspec(m, l, SITE_ATTN_PROBS), st.ctx32};
  {
    const double TS = (double)bt->batch * bt->seq;
    ProfScope ps(m, PC_ATTN_BWD, 10.0 * TS * bt->seq * H, 8.0 * TS * H * m->esz);
    if (m->dtype == 1 && attention_mfma_supported(bt->seq, m->dh))
      HIP_TRY(attention_bwd_mfma(a, s));
    else
      HIP_TRY(attention_bwd_simple(m->dtype, a, s));
    if (Tr > T)  // padded token rows must contribute nothing to the weight gradients
      HIP_TRY(fill_zero((char*)m->d_qkv + (size_t)T * 3 * H * m->esz, (size_t)(Tr - T) * 3 * H * m->esz, s));
  }
  RC(linear_bwd_weight(m, m->d_qkv, Tr, 3 * H, 3 * H, Xin, H, Gf(m, t_app(m, l, L_WQ))));
  RC(bias_grad(m, m->d_qkv, 3 * H, Tr, 3 * H, Gf(m, t_app(m, l, L_BQ)), true));
  if (dXin)
    RC(linear_bwd_input(m, m->d_qkv, Tr, 3 * H, 3 * H, Wg(m, t_app(m, l, L_WQ)), H, dXin, EPI_ADD, resid, true, resid_f32, m->wide));
  return layer_backward_end(m, l);
}
// dXout: gradient w.r.t. the layer output on all token rows.
static int layer_backward(mslt_model* m, int l, const mslt_batch* bt, int T, int Tr, const void* Xin, const void* dXout,
                          void* dXin) {
  const LayerStash& st = m->stash[l - m->stash_base];
  RC(layer_backward_begin(m, l));
  UpperRows r{st.xhat2, st.g, st.u, st.x1, st.xhat1, st.ctx, st.rstd2, st.rstd1, m->d_d, m->d_u, m->d_x1, m->d_z1, m->d_c, Tr,
              m->d_dm, m->d_z1m, nullptr, 0, m->wide, m->d_d32, m->d_z1_32};
  RC(layer_backward_upper(m, l, dXout, r));
  return layer_backward_lower(m, l, bt, T, Tr, Xin, dXin, m->wide ? (const void*)m->d_z1_32 : m->d_z1, m->wide);
}
// Top trainable layer: the gradient of its output is non-zero only in the M predicted rows, and
// everything above the attention is row-local, so that part runs on the compacted rows (exact, not
// an approximation); dC and dz1 are scattered back to token rows for the attention and QKV backward.
static int layer_backward_top(mslt_model* m, int l, const mslt_batch* bt, int T, int Tr, int M, int Mr, const void* Xin,
                              const void* dXm, void* dXin) {
  const int H = m->H, F = m->F;
  const LayerStash& st = m->stash[l - m->stash_base];
  hipStream_t s = m->stream;
  RC(layer_backward_begin(m, l));
  {
    ProfScope ps(m, PC_HEAD_MISC, 0.0, 2.0 * Mr * (4.0 * H + 2.0 * F) * m->esz);
    const int hb = H * (int)m->esz, fb = F * (int)m->esz;
    const GatherDesc g[8] = {{st.xhat2, m->c_xhat2, hb}, {st.x1, m->ut, hb}, {st.xhat1, m->gt, hb}, {st.ctx, m->xhat_t, hb},
                             {st.g, m->c_g, fb},    {st.u, m->c_u, fb}, {st.rstd2, m->rstd_t, 4}, {st.rstd1, m->lse_t, 4}};
    HIP_TRY(gather_rows_multi(g, 8, m->pos, M, Mr, s));
  }
  UpperRows r{m->c_xhat2, m->c_g, m->c_u, m->ut, m->gt, m->xhat_t, m->rstd_t, m->lse_t,
              m->c_dz2, m->c_du, m->d_hm, m->d_gt, m->c_dc, Mr, m->c_dz2m, m->c_dz1m, m->pos, M, 0, nullptr, nullptr};
  RC(layer_backward_upper(m, l, dXm, r));
  {
    ProfScope ps(m, PC_HEAD_MISC, 0.0, 2.0 * ((double)Tr + M) * H * m->esz);
    HIP_TRY(scatter_rows(m->dtype, m->c_dc, m->inv, Tr, T, H, m->d_c, s));
    HIP_TRY(scatter_rows(m->dtype, m->d_gt, m->inv, Tr, T, H, m->d_z1, s));
  }
  return layer_backward_lower(m, l, bt, T, Tr, Xin, dXin, m->d_z1, 0);
}

// ---- the stage step -------------------------------------------------------------------------
// Queues one whole stage step (everything but the final wait) on the model's streams.
static int stage_step_enqueue(mslt_model* m, int f, int k, int train_emb, const mslt_batch* bt) {
  if (!m || !bt) return fail(MSLT_ERR_ARG, "null argument");
  if (k < 1 || f < 0 || f + k > m->L)
    return fail(MSLT_ERR_ARG, "stage_step: bad layer split frozen=%d trainable=%d (layers %d)", f, k, m->L);
  if (k > m->n_stash)
    return fail(MSLT_ERR_ARG, "stage_step: %d trainable layers exceed max_trainable_layers %d of the configuration", k, m->n_stash);
  if (train_emb != 0 && train_emb != 1) return fail(MSLT_ERR_ARG, "stage_step: train_embeddings must be 0 or 1");
  if (train_emb && f != 0) return fail(MSLT_ERR_ARG, "stage_step: embeddings train only when nothing is frozen");
  if (f % m->lpg || k % m->lpg)
    return fail(MSLT_ERR_ARG, "stage_step: frozen and trainable layer counts must be whole groups of %d layers", m->lpg);
  if (!bt->input_ids || !bt->token_type_ids || !bt->attn_mask || !bt->labels)
    return fail(MSLT_ERR_ARG, "stage_step: null batch pointer");
  if (m->nsp && !bt->nsp_labels) return fail(MSLT_ERR_ARG, "stage_step: the model has a next-sentence head but nsp_labels is null");
  if (bt->batch < 1 || bt->batch > m->cfg.max_batch || bt->seq < 1 || bt->seq > m->cfg.max_seq)
    return fail(MSLT_ERR_ARG, "stage_step: batch %dx%d outside 1..%dx1..%d", bt->batch, bt->seq, m->cfg.max_batch,
                m->cfg.max_seq);
  RC(side_join(m));      // only pending after a step that failed half-way
  hipStream_t s = m->stream;
  const int H = m->H, B = bt->batch, S = bt->seq, T = B * S;
  m->have_grads = false;
  m->acc_now = 0;
  m->stash_base = f;
  m->side_dw.clear(); m->side_cs.clear(); m->side_collect = false;
  m->later.clear();          // (a step that failed half-way may have left jobs behind)
  m->later_used = 0;
  m->later_on = m->lpg == 1;

  // S0: batch check and compaction of the predicted positions (only index scratch is written)
  HIP_TRY(batch_scan(bt->input_ids, bt->token_type_ids, bt->attn_mask, bt->labels, T, m->V, m->cfg.type_vocab, m->cap,
                     m->pos, m->lab, m->inv, m->counters, m->nsp ? S : 0, m->nsp ? bt->nsp_labels : nullptr, B, s));
  HIP_TRY(hipMemcpyAsync(m->h_counters, m->counters, 12, hipMemcpyDeviceToHost, s));
  HIP_TRY(hipEventRecord(m->ev_scan, s));
  const int Tr = m->mfma ? (int)rup(T, 128) : T;
  const int Vr = m->mfma ? m->Vp : m->V;

  // The encoder forward does not depend on the verdict of the batch check (the embedding lookup
  // clamps its indices), so it is queued before the host waits for that verdict: the device then
  // has work while the host reads the count of predicted positions the head is sized by.
  // S1: embeddings + LayerNorm
  LnStash e0;
  if (train_emb) { e0.xhat = m->xhat0; e0.rstd = m->rstd0; }
  {
    ProfScope ps(m, PC_EMBED, 0.0, (double)T * H * (4.0 + m->esz * (train_emb ? 2.0 : 1.0)));
    HIP_TRY(embed_ln_fwd(m->dtype, bt->input_ids, bt->token_type_ids, S, Wf(m, T_WORD), Wf(m, T_POS), Wf(m, T_TYPE),
                         Wf(m, T_ELN_G), Wf(m, T_ELN_B), m->cfg.ln_eps, m->x0, e0, T, H, m->V, m->cfg.type_vocab,
                         dspec(m, 0, SITE_EMBEDDING), s));
  }
  // The two halves of the batch go through the encoder as two independent chains of kernels, one per
  // stream: where a kernel of one chain leaves compute units idle (a last, partly filled round of
  // workgroups, its ramp-up and its drain) kernels of the other chain take them.  Measured: 2-5 %
  // of the step; four chains on four streams were slower.  Dropout indexes its decisions by position
  // in the whole batch: the second half's kernels get keys that carry its offset (S even keeps the
  // offset of the attention probabilities a multiple of 4).  Off while event profiling.
  const bool halves = !m->prof.on && m->dtype == 1 && m->mfma && B % 2 == 0 && (T / 2) % 128 == 0 && Tr == T && S % 2 == 0;
  const FwdPart parts[2] = {{0, B / 2, s}, {B / 2, B / 2, m->side}};
  if (halves) {
    HIP_TRY(hipEventRecord(m->ev_fork, s));
    HIP_TRY(hipStreamWaitEvent(m->side, m->ev_fork, 0));
    m->side_forked = true;     // a step that fails half-way is joined at the start of the next one
  }
  auto forward = [&](int l, const void* xin, void* xo, const LayerStash* st) -> int {
    if (!halves) return layer_forward(m, l, bt, Tr, xin, xo, st);
    RC(layer_forward(m, l, bt, Tr, xin, xo, st, &parts[0]));
    return layer_forward(m, l, bt, Tr, xin, xo, st, &parts[1]);
  };
  // S2: frozen prefix, forward only, two ping-pong buffers, nothing kept
  const void* x = m->x0;
  for (int l = 0; l < f; ++l) {
    void* xo = (l & 1) ? m->xb : m->xa;
    RC(forward(l, x, xo, nullptr));
    x = xo;
  }
  m->last_prefix = x;
  // S3: trainable layers, with stash
  for (int l = f; l < f + k; ++l) {
    RC(forward(l, x, m->stash[l - f].xout, &m->stash[l - f]));
    x = m->stash[l - f].xout;
  }
  if (halves) RC(side_join(m));
  HIP_TRY(hipEventSynchronize(m->ev_scan));
  // M: compacted rows (predicted positions, plus every first token when there is a next-sentence head);
  // Mn: those of them that carry a masked-LM label
  const int M = m->h_counters[0], bad = m->h_counters[1], Mn = m->h_counters[2];
  if (bad || Mn < 1 || M > m->cap) {
    m->last_prefix = nullptr;           // the workspace now holds the rejected batch's activations
    HIP_TRY(hipStreamSynchronize(s));   // let the queued forward drain before reporting
    if (bad)
      return fail(MSLT_ERR_DATA, "stage_step: batch content out of range (bits %d: 1 id, 2 type, 4 label, 8 mask, 16 nsp label)", bad);
    if (Mn < 1) return fail(MSLT_ERR_DATA, "stage_step: no predicted position in the batch");
    return fail(MSLT_ERR_DATA, "stage_step: %d predicted positions exceed max_predictions %d", M, m->cap);
  }
  const int Mr = m->mfma ? (int)rup(M, 128) : M;
  // S4-S6: head forward and loss
  const int th = t_head(m, 0);
  {
    ProfScope ps(m, PC_HEAD_MISC, 0.0, 2.0 * Mr * H * m->esz);
    const GatherDesc g{x, m->xm, H * (int)m->esz};
    HIP_TRY(gather_rows_multi(&g, 1, m->pos, M, Mr, s));
  }
  RC(linear_fwd(m, m->xm, Mr, H, Wg(m, th + H_WT), H, Wf(m, th + H_BT), m->gt, 0, H, EPI_GELU, m->ut));
  LnStash sh{m->xhat_t, m->rstd_t};
  RC(ln_forward(m, m->gt, nullptr, Wf(m, th + H_LNG), Wf(m, th + H_LNB), m->hm, sh, Mr));
  RC(linear_fwd(m, m->hm, Mr, H, Wg(m, T_WORD), Vr, Wf(m, th + H_BOUT), m->logits, 0, m->Vp, EPI_NONE, nullptr));
  {
    ProfScope ps(m, PC_CE, 0.0, (double)M * m->V * m->esz + (double)Mr * m->Vp * m->esz);
    HIP_TRY(ce_fwd_bwd(m->dtype, m->logits, m->Vp, m->lab, M, Mn, Mr, m->V, m->dz, m->row_loss, m->lse_t, m->loss, s));
  }
  if (m->nsp) {
    // next-sentence head (the second objective is added to the loss): pooled = tanh(X_first Wp^T + bp),
    // logits = pooled Wc^T + bc, mean two-way cross-entropy over the batch
    HIP_TRY(gather_first_tokens(m->dtype, x, S, H, B, m->n_xc, s));
    RC(linear_fwd(m, m->n_xc, B, H, Wg(m, th + P_W), H, Wf(m, th + P_B), m->n_p, 0, H, EPI_NONE, nullptr));
    HIP_TRY(tanh_inplace(m->dtype, m->n_p, (size_t)B * H, s));
    RC(linear_fwd(m, m->n_p, B, H, Wg(m, th + C_W), 2, Wf(m, th + C_B), m->n_z, 1, 2, EPI_NONE, nullptr));
    HIP_TRY(nsp_ce(m->dtype, m->n_z, bt->nsp_labels, B, m->n_dz, m->loss, s));
  }
  HIP_TRY(hipMemcpyAsync(m->h_loss, m->loss, 4, hipMemcpyDeviceToHost, s));
  // S7: head backward
  // over the padded vocabulary (the padded columns of dZ are zero and the output bias reserves them)
  RC(bias_grad(m, m->dz, m->Vp, Mr, m->Vp, Gf(m, th + H_BOUT)));
  // (the embedding backward adds the lookup's gradient to the same tensor later in this step)
  if (train_emb) RC(linear_bwd_weight(m, m->dz, Mr, Vr, m->Vp, m->hm, H, Gf(m, T_WORD), true, false));
  // few output tiles, contraction over the whole vocabulary: split it
  RC(linear_bwd_input(m, m->dz, Mr, Vr, m->Vp, Wg(m, T_WORD), H, m->d_hm, EPI_NONE, nullptr, true));
  RC(ln_backward(m, m->d_hm, m->xhat_t, m->rstd_t, Wf(m, th + H_LNG), m->d_gt, Gf(m, th + H_LNG), Gf(m, th + H_LNB), nullptr, Mr));
  {
    ProfScope ps(m, PC_HEAD_MISC, 0.0, 3.0 * Mr * H * m->esz);
    HIP_TRY(mul_dgelu(m->dtype, m->d_gt, m->ut, m->d_ut, (size_t)Mr * H, s));
  }
  RC(linear_bwd_weight(m, m->d_ut, Mr, H, H, m->xm, H, Gf(m, th + H_WT)));
  RC(bias_grad(m, m->d_ut, H, Mr, H, Gf(m, th + H_BT), true));
  RC(linear_bwd_input(m, m->d_ut, Mr, H, H, Wg(m, th + H_WT), H, m->d_xm, EPI_NONE, nullptr));
  if (m->nsp) {
    // backward of the next-sentence head; its input gradient joins the compacted rows of the first tokens
    RC(linear_bwd_weight(m, m->n_dz, B, 2, 2, m->n_p, H, Gf(m, th + C_W)));
    RC(bias_grad(m, m->n_dz, 2, B, 2, Gf(m, th + C_B), true));
    RC(linear_bwd_input(m, m->n_dz, B, 2, 2, Wg(m, th + C_W), H, m->n_dp, EPI_NONE, nullptr, false));
    HIP_TRY(tanh_bwd(m->dtype, m->n_dp, m->n_p, m->n_du, (size_t)B * H, s));
    RC(linear_bwd_weight(m, m->n_du, B, H, H, m->n_xc, H, Gf(m, th + P_W)));
    RC(bias_grad(m, m->n_du, H, B, H, Gf(m, th + P_B), true));
    RC(linear_bwd_input(m, m->n_du, B, H, H, Wg(m, th + P_W), H, m->n_dx, EPI_NONE, nullptr, false));
    HIP_TRY(add_first_token_rows(m->dtype, m->n_dx, m->inv, S, H, B, m->d_xm, s));
  }
  // (no join here: the top layer's compacted rows have buffers of their own, so the side stream may still be
  //  working on the head's weight gradients while the main stream goes on)
  // S8/S9: trainable layers backward, top down.  The top layer works on the compacted predicted rows
  // and scatters inside; the layers below get dense gradients.
  void* dx = m->dxa;
  for (int l = f + k - 1; l >= f; --l) {
    const void* xin = (l == f) ? m->last_prefix : m->stash[l - 1 - f].xout;
    bool need_dx = (l > f) || train_emb;
    void* dxin = need_dx ? (dx == m->dxa ? m->dxb : m->dxa) : nullptr;
    if (l == f + k - 1)
      RC(layer_backward_top(m, l, bt, T, Tr, M, Mr, xin, m->d_xm, dxin));
    else
      RC(layer_backward(m, l, bt, T, Tr, xin, dx, dxin));
    if (dxin) dx = dxin;
  }
  RC(side_join(m));      // all weight gradients are complete when the step returns
  // S10: embedding backward (first stage / retraining)
  if (train_emb) {
    LnBwdDrop de;
    de.in = dspec(m, 0, SITE_EMBEDDING);
    RC(ln_backward(m, dx, m->xhat0, m->rstd0, Wf(m, T_ELN_G), m->d_z0, Gf(m, T_ELN_G), Gf(m, T_ELN_B), nullptr, T, de, m->wide));
    ProfScope ps(m, PC_EMBED_BWD, 0.0, (double)T * H * (m->esz + 8.0));
    HIP_TRY(embed_bwd(m->dtype, m->d_z0, bt->input_ids, bt->token_type_ids, B, S, H, m->V, m->cfg.type_vocab,
                      Gf(m, T_WORD), Gf(m, T_POS), Gf(m, T_TYPE), m->e_rank, m->e_cnt, m->e_start, m->e_order, m->e_blockcnt,
                      m->cfg.max_pos, m->red_scratch, m->e_partial, s));
  }
  RC(later_flush(m));
  m->last_f = f; m->last_k = k; m->last_emb = train_emb; m->last_B = B; m->last_S = S; m->last_M = M;
  return MSLT_OK;
}
// Waits for the queued step and hands out its loss.
static int stage_step_finish(mslt_model* m, float* loss_out) {
  HIP_TRY(hipStreamSynchronize(m->stream));
  *loss_out = *m->h_loss;
  if (!std::isfinite(*loss_out)) return fail(MSLT_ERR_NONFINITE, "stage_step: loss is not finite");
  return MSLT_OK;
}

extern "C" int mslt_stage_step(mslt_model* m, int f, int k, int train_emb, const mslt_batch* bt, float* loss_out) {
  if (!loss_out) return fail(MSLT_ERR_ARG, "null argument");
  RC(stage_step_enqueue(m, f, k, train_emb, bt));
  m->have_grads = true;     // the gradients are well defined even when the loss turns out non-finite
  return stage_step_finish(m, loss_out);
}

// trainable tensor ranges of the last step, as [first, last) index pairs in table order
static int trainable_ranges(const mslt_model* m, int (*r)[2]) {
  int n = 0;
  if (m->last_emb) { r[n][0] = 0; r[n][1] = N_EMB; ++n; }
  r[n][0] = t_layer(m->last_f / m->lpg, 0); r[n][1] = t_layer((m->last_f + m->last_k) / m->lpg, 0); ++n;
  r[n][0] = t_head(m, 0); r[n][1] = t_head(m, 0) + (m->nsp ? N_HEAD_NSP : N_HEAD); ++n;
  // merge adjacent ranges
  int out = 0;
  for (int i = 0; i < n; ++i) {
    if (out && r[out - 1][1] == r[i][0]) r[out - 1][1] = r[i][1];
    else { r[out][0] = r[i][0]; r[out][1] = r[i][1]; ++out; }
  }
  return out;
}

extern "C" int mslt_grad_count(const mslt_model* m, size_t* n_floats) {
  if (!m || !n_floats) return fail(MSLT_ERR_ARG, "null argument");
  if (!m->have_grads) return fail(MSLT_ERR_STATE, "no gradients: run a successful stage_step first");
  int r[3][2];
  int n = trainable_ranges(m, r);
  size_t c = 0;
  for (int i = 0; i < n; ++i)
    for (int t = r[i][0]; t < r[i][1]; ++t) c += m->table[t].count;
  *n_floats = c;
  return MSLT_OK;
}

extern "C" int mslt_get_grads(const mslt_model* m, float* host, size_t n_floats) {
  if (!m || !host) return fail(MSLT_ERR_ARG, "null argument");
  size_t need;
  int rc = mslt_grad_count(m, &need);
  if (rc) return rc;
  if (need != n_floats) return fail(MSLT_ERR_ARG, "get_grads: expected %zu floats, got %zu", need, n_floats);
  int r[3][2];
  int n = trainable_ranges(m, r);
  size_t o = 0;
  for (int i = 0; i < n; ++i)
    for (int t = r[i][0]; t < r[i][1]; ++t) {
      HIP_TRY(hipMemcpyAsync(host + o, m->grad + m->table[t].offset, m->table[t].count * 4, hipMemcpyDeviceToHost,
                             m->stream));
      o += m->table[t].count;
    }
  HIP_TRY(hipStreamSynchronize(m->stream));
  return MSLT_OK;
}

static int check_opt(const mslt_opt* opt, const char* who) {
  if (opt->kind != 0 && opt->kind != 1) return fail(MSLT_ERR_ARG, "%s: kind must be 0 (Adam) or 1 (LAMB)", who);
  if (!(opt->beta1 >= 0.f && opt->beta1 < 1.f && opt->beta2 >= 0.f && opt->beta2 < 1.f && opt->eps >= 0.f))
    return fail(MSLT_ERR_ARG, "%s: bad beta or eps", who);
  return MSLT_OK;
}
// Queues the update of the tensors the last step trained; gate: see OptHyper::gate.
static int update_enqueue(mslt_model* m, const mslt_opt* opt, const float* gate, float* chunk_norms = nullptr,
                          float* ratio = nullptr) {
  if (!chunk_norms) { chunk_norms = m->o_chunk_norms; ratio = m->o_ratio; }
  OptHyper h{opt->kind, opt->lr, opt->beta1, opt->beta2, opt->eps, opt->weight_decay, opt->bias_correction, gate};
  int r[3][2];
  int n = trainable_ranges(m, r);
  for (int i = 0; i < n; ++i) {
    int t0 = r[i][0], nt = r[i][1] - r[i][0];
    int c0 = m->first_chunk[t0], nc = m->first_chunk[r[i][1]] - c0;
    size_t n_elems = 0;
    for (int t = t0; t < r[i][1]; ++t) n_elems += m->table[t].count;
    ProfScope ps(m, PC_OPT, 0.0, (double)n_elems * ((opt->kind ? 40.0 : 28.0) + (m->dtype ? 2.0 : 0.0)));
    HIP_TRY(bump_steps(m->o_tsteps, t0, nt, gate, m->stream));
    HIP_TRY(optimizer_step(h, m->o_tensors, m->o_tsteps, t0, nt, m->o_chunk_tensor, c0, nc, m->param, m->grad, m->mom1,
                           m->mom2, m->shadow, chunk_norms, ratio, m->stream));
  }
  return MSLT_OK;
}

extern "C" int mslt_apply_update(mslt_model* m, const mslt_opt* opt) {
  if (!m || !opt) return fail(MSLT_ERR_ARG, "null argument");
  if (!m->have_grads) return fail(MSLT_ERR_STATE, "apply_update: no gradients from a preceding stage_step");
  RC(check_opt(opt, "apply_update"));
  // gated on the device by the loss of the step whose gradients these are: after a step that returned
  // MSLT_ERR_NONFINITE the update kernels do nothing, as in mslt_train_step
  RC(update_enqueue(m, opt, m->loss));
  m->have_grads = false;
  return MSLT_OK;
}

extern "C" int mslt_apply_update_static(mslt_model* m, const mslt_opt* opt) {
  if (!m || !opt) return fail(MSLT_ERR_ARG, "null argument");
  if (!m->have_grads) return fail(MSLT_ERR_STATE, "apply_update_static: no gradients from a preceding stage_step");
  RC(check_opt(opt, "apply_update_static"));
  if (m->first_chunk.back() > STATIC_MAX_CHUNKS || (int)m->table.size() > STATIC_MAX_TENSORS)
    return fail(MSLT_ERR_ARG, "apply_update_static: model has %d optimizer chunks and %d tensors, the static scratch holds %d and %d",
                m->first_chunk.back(), (int)m->table.size(), STATIC_MAX_CHUNKS, STATIC_MAX_TENSORS);
  // every chunk sum and ratio the update reads is written earlier in the same call: nothing to clear
  RC(update_enqueue(m, opt, m->loss, m->static_scratch, m->static_scratch + (size_t)2 * STATIC_MAX_CHUNKS));
  m->have_grads = false;
  return MSLT_OK;
}

extern "C" int mslt_train_step(mslt_model* m, int f, int k, int train_emb, const mslt_batch* bt, const mslt_opt* opt,
                               float* loss_out) {
  if (!m || !opt || !loss_out) return fail(MSLT_ERR_ARG, "null argument");
  RC(check_opt(opt, "train_step"));
  RC(stage_step_enqueue(m, f, k, train_emb, bt));
  // the update goes in right behind the step; on the device it does nothing if the loss is not finite
  RC(update_enqueue(m, opt, m->loss));
  m->have_grads = false;
  return stage_step_finish(m, loss_out);
}

extern "C" int mslt_set_dropout(mslt_model* m, float p, uint64_t seed, uint64_t step) {
  if (!m) return fail(MSLT_ERR_ARG, "model is null");
  if (!(p >= 0.f && p < 1.f)) return fail(MSLT_ERR_ARG, "set_dropout: probability %g outside [0, 1)", (double)p);
  if (step >> 44) return fail(MSLT_ERR_ARG, "set_dropout: step number too large");
  if (m->H % 4) return fail(MSLT_ERR_ARG, "set_dropout: hidden size must be a multiple of 4");
  m->drop_thr = (uint32_t)lrintf(p * 65536.0f);
  m->drop_scale = 1.0f / (1.0f - p);
  m->drop_seed = seed;
  m->drop_step = step;
  return MSLT_OK;
}

extern "C" int mslt_debug_masked(const mslt_model* m, int32_t* pos_out, int32_t* label_out, int* m_out) {
  if (!m || !pos_out || !label_out || !m_out) return fail(MSLT_ERR_ARG, "null argument");
  if (!m->last_prefix) return fail(MSLT_ERR_STATE, "debug_masked: no step has run");
  HIP_TRY(hipMemcpyAsync(pos_out, m->pos, (size_t)m->last_M * 4, hipMemcpyDeviceToHost, m->stream));
  HIP_TRY(hipMemcpyAsync(label_out, m->lab, (size_t)m->last_M * 4, hipMemcpyDeviceToHost, m->stream));
  HIP_TRY(hipStreamSynchronize(m->stream));
  int n = 0;               // rows that are only there for the next-sentence head carry no label: leave them out
  for (int i = 0; i < m->last_M; ++i)
    if (label_out[i] >= 0) { pos_out[n] = pos_out[i]; label_out[n] = label_out[i]; ++n; }
  *m_out = n;
  return MSLT_OK;
}

extern "C" int mslt_debug_prefix_output(const mslt_model* m, float* host, size_t n_floats) {
  if (!m || !host) return fail(MSLT_ERR_ARG, "null argument");
  if (!m->last_prefix) return fail(MSLT_ERR_STATE, "debug_prefix_output: no step has run");
  size_t need = (size_t)m->last_B * m->last_S * m->H;
  if (n_floats != need) return fail(MSLT_ERR_ARG, "debug_prefix_output: expected %zu floats, got %zu", need, n_floats);
  if (m->dtype == 0) {
    HIP_TRY(hipMemcpyAsync(host, m->last_prefix, need * 4, hipMemcpyDeviceToHost, m->stream));
  } else {
    // widen on the device into the logits buffer (free between steps), then copy
    if (need > (size_t)m->Mp * m->Vp) return fail(MSLT_ERR_ARG, "debug_prefix_output: scratch too small");
    HIP_TRY(widen_to_f32(1, m->last_prefix, m->logits, need, m->stream));
    HIP_TRY(hipMemcpyAsync(host, m->logits, need * 4, hipMemcpyDeviceToHost, m->stream));
  }
  HIP_TRY(hipStreamSynchronize(m->stream));
  return MSLT_OK;
}

extern "C" int mslt_grow(mslt_model* m, int n_present, int n_new) {
  if (!m) return fail(MSLT_ERR_ARG, "model is null");
  if (n_new < 1 || n_present < n_new || n_present + n_new > m->L)
    return fail(MSLT_ERR_ARG, "grow: bad layer counts present=%d new=%d (layers %d)", n_present, n_new, m->L);
  if (n_present % m->lpg || n_new % m->lpg)
    return fail(MSLT_ERR_ARG, "grow: layer counts must be whole groups of %d layers", m->lpg);
  n_present /= m->lpg;      // from here on in parameter sets
  n_new /= m->lpg;
  for (int i = 0; i < n_new; ++i) {
    int src = n_present - n_new + i, dst = n_present + i;
    for (int j = 0; j < N_LAYER_T; ++j) {
      const mslt_tensor_desc& a = m->table[t_layer(src, j)];
      const mslt_tensor_desc& b = m->table[t_layer(dst, j)];
      HIP_TRY(hipMemcpyAsync(m->param + b.offset, m->param + a.offset, a.count * 4, hipMemcpyDeviceToDevice, m->stream));
      if (m->dtype)
        HIP_TRY(hipMemcpyAsync(m->shadow + b.offset, m->shadow + a.offset, a.count * 2, hipMemcpyDeviceToDevice,
                               m->stream));
    }
    // moments of the new layer restart from zero (its tensors are one contiguous block)
    size_t lo = m->table[t_layer(dst, 0)].offset;
    size_t hi = m->table[t_layer(dst, N_LAYER_T - 1)].offset + m->table[t_layer(dst, N_LAYER_T - 1)].count;
    hi = rup(hi, 4);
    HIP_TRY(fill_zero(m->mom1 + lo, (hi - lo) * 4, m->stream));
    HIP_TRY(fill_zero(m->mom2 + lo, (hi - lo) * 4, m->stream));
  }
  // step counts of the new layers back to 0: 16 ints per layer are contiguous in the table
  std::vector<int32_t> z((size_t)n_new * N_LAYER_T, 0);
  HIP_TRY(hipMemcpyAsync(m->o_tsteps + t_layer(n_present, 0), z.data(), z.size() * 4, hipMemcpyHostToDevice, m->stream));
  HIP_TRY(hipStreamSynchronize(m->stream));
  m->have_grads = false;
  return MSLT_OK;
}

extern "C" int mslt_debug_gemm(void* hip_stream, const void* A, const void* B, void* C, int M, int N, int K, int a_kcontig,
                               int b_kcontig, int out_f32, int kernel, int tile_m, int tile_n, int tile_k, int splitk,
                               void* partials, size_t partial_bytes) {
  if (!A || !B || !C) return fail(MSLT_ERR_ARG, "debug_gemm: null operand");
  if (M < 1 || N < 1 || K < 1) return fail(MSLT_ERR_ARG, "debug_gemm: non-positive size");
  if (splitk < 1) return fail(MSLT_ERR_ARG, "debug_gemm: splitk must be at least 1");
  if (splitk > 1 && (kernel == 0 || !partials || partial_bytes < (size_t)splitk * M * N * 4))
    return fail(MSLT_ERR_ARG, "debug_gemm: split-k needs kernel 1 or 2 and %zu bytes of partials", (size_t)splitk * M * N * 4);
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  GemmDesc d;
  d.A = A; d.B = B; d.M = M; d.N = N; d.K = K;
  d.a_kcontig = a_kcontig != 0; d.b_kcontig = b_kcontig != 0;
  d.lda = d.a_kcontig ? K : M; d.ldb = d.b_kcontig ? K : N;
  d.epi.out = C; d.epi.ldo = N; d.epi.out_f32 = out_f32 != 0;
  if (kernel == 0) {
    HIP_TRY(gemm_simt(1, d, st));
  } else if (kernel == 1) {
    if (!gemm_mfma_supported(d) || (tile_m != 0 && tile_m != 128 && tile_m != 256) || (tile_m && M % tile_m) || splitk > K / 64)
      return fail(MSLT_ERR_ARG, "debug_gemm: shape %dx%dx%d (tile_m %d, splitk %d) not taken by the 128-wide kernel", M, N, K,
                  tile_m, splitk);
    HIP_TRY(gemm_mfma(d, splitk, (float*)partials, st, tile_m));
  } else if (kernel == 2) {
    if (!gemm_ring_supported(d, tile_m, tile_n, tile_k) || splitk > K / tile_k)
      return fail(MSLT_ERR_ARG, "debug_gemm: shape %dx%dx%d not taken by the large-tile kernel with tile %dx%dx%d, splitk %d", M, N,
                  K, tile_m, tile_n, tile_k, splitk);
    HIP_TRY(gemm_ring(d, tile_m, tile_n, tile_k, splitk, (float*)partials, st));
  } else {
    return fail(MSLT_ERR_ARG, "debug_gemm: kernel must be 0, 1 or 2");
  }
  return MSLT_OK;
}

extern "C" int mslt_profile_enable(mslt_model* m, int on) {
  if (!m) return fail(MSLT_ERR_ARG, "model is null");
  HIP_TRY(hipStreamSynchronize(m->stream));
  for (auto& sp : m->prof.spans) { m->prof.pool.push_back(sp.a); m->prof.pool.push_back(sp.b); }
  m->prof.spans.clear();
  m->prof.on = on != 0;
  return MSLT_OK;
}

extern "C" int mslt_profile_read(mslt_model* m, mslt_profile_entry* out, int cap, int* n) {
  if (!m || !out || !n) return fail(MSLT_ERR_ARG, "null argument");
  if (cap < PC_COUNT) return fail(MSLT_ERR_ARG, "profile_read: need room for %d entries", (int)PC_COUNT);
  HIP_TRY(hipStreamSynchronize(m->stream));
  for (int c = 0; c < PC_COUNT; ++c) {
    memset(&out[c], 0, sizeof out[c]);
    snprintf(out[c].name, sizeof out[c].name, "%s", kProfNames[c]);
  }
  for (auto& sp : m->prof.spans) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, sp.a, sp.b));
    out[sp.cls].launches += 1;
    out[sp.cls].ms += ms;
    out[sp.cls].flops += sp.flops;
    out[sp.cls].bytes += sp.bytes;
    m->prof.pool.push_back(sp.a);
    m->prof.pool.push_back(sp.b);
  }
  m->prof.spans.clear();
  *n = PC_COUNT;
  return MSLT_OK;
}
