// Host runtime behind the C ABI: module registry with per-module contiguous buffers, route table,
// use counters n_j, per-step workspace, and the launch sequence of one routed training step
// (Algorithm 1: forward through the task's modules in order, gradients only for those modules,
// renormalisation by n_j folded into the update).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "../../include/mammoth_hip.h"
#include "mm_kernels.h"

using namespace mm;

// Segment table of mm_apply_update_noalloc, which may not allocate: one array per GPU the library
// runs on, held until the process ends.  In host code the name stands for the symbol only; the
// device address is looked up once per device (scratch_address) and that pointer is what copies
// and kernels receive.  All contexts of one GPU share the array.  (The compiler gives a static
// device variable that host code names a visible symbol in the code object, which the lookup
// needs; forcing its emission with the "used" attribute happens before that and leaves it local.)
constexpr int NOALLOC_MAX_MODULES = MM_NOALLOC_MAX_MODULES;
static __device__ __align__(256) unsigned char scratch[NOALLOC_MAX_MODULES * sizeof(AdamSegment)];

namespace {

constexpr int64_t ALIGN_ELEMS = 64;
inline int64_t round_up(int64_t n, int64_t a) { return (n + a - 1) / a * a; }

struct TensorInfo { int64_t off; int rows, cols, role; };

struct Module {
  int kind = 0, position = 0, n_layers = 0, owns_final_norm = 0, adapter_dim = 0, adapter_stack = 0;
  std::string name;
  std::vector<TensorInfo> tensors;
  int64_t P = 0;
  float *theta = nullptr, *m = nullptr, *v = nullptr, *g = nullptr;
  bf16_t* w16 = nullptr;
  int touched = 0;
  int64_t t = 0;
  bool t_on_trust = false;   // t was raised by an update enqueued behind a step whose outcome was not known yet
};

struct Route { std::vector<int> ids; int src = -1, tgt = -1, gen = -1, ad_enc = -1, ad_dec = -1; std::vector<int> enc, dec; };

struct Arena {
  char* base = nullptr;
  size_t cap = 0, off = 0, high = 0;
  bool measuring = false;
  void reset(bool measure) { off = 0; high = 0; measuring = measure; }
  void* take(size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    void* p = measuring ? nullptr : (void*)(base + off);
    off += bytes;
    if (off > high) high = off;
    return p;
  }
};

// One timed launch: the event recorded right after it.  cls < 0: a mark that starts a new chain
// (the beginning of a call); a launch's time is the distance from the previous event of its chain.
struct ProfRec { int cls; hipEvent_t e; hipEvent_t s; };   // s: the kernel's own start time, where the launcher provides it
constexpr int MAX_GROUPED_C = 1024;

}  // namespace

struct mm_ctx {
  mm_config cfg{};
  Dtype dt = F32;
  hipStream_t st = nullptr;
  bool plan_only = false;
  std::vector<Module> mods;
  std::vector<Route> routes;
  std::string err;
  // device-side constants and per-step metadata
  float* pe = nullptr;                       // [max_len, d]
  int32_t* meta = nullptr;                   // cu_s, cu_u, lens, src_tok, src_pos, dec_tok, dec_pos, label
  int32_t *cu_s = nullptr, *cu_u = nullptr, *lens = nullptr, *src_tok = nullptr, *src_pos = nullptr,
          *dec_tok = nullptr, *dec_pos = nullptr, *label = nullptr;
  uint32_t* sort_keys = nullptr;              // [2][16384]: sorted (token,row) keys of source / decoder rows
  hipStream_t aux = nullptr;                  // side stream: the token sorts run beside the forward pass
  hipEvent_t ev_packed = nullptr, ev_sorted = nullptr;
  int32_t* flag = nullptr;                   // device: id-check result of the step
  float* loss_dev = nullptr;
  int32_t* ids_dev = nullptr; size_t ids_dev_cap = 0;      // staged copies of host ids
  int32_t* stage = nullptr; size_t stage_cap = 0;          // pinned host staging
  float* result_host = nullptr;              // pinned: [0] loss, [1] flag (as int bits)
  hipEvent_t ev_stage = nullptr, ev_done = nullptr;
  AdamSegment* seg_host = nullptr; AdamSegment* seg_dev = nullptr; int seg_cap = 0;
  hipEvent_t ev_seg = nullptr;
  // mm_apply_update_noalloc: pinned table of fixed size (allocated at creation) and this device's
  // address of the library's static device array
  AdamSegment* seg_static_host = nullptr; AdamSegment* seg_static_dev = nullptr;
  hipEvent_t ev_seg_static = nullptr;
  // table of the step's deferred weight-gradient products (pinned host copy, device copy)
  // (one pinned block and one device block: product table, first-tile table and the LayerNorm
  // reduction jobs are packed back to back and travel in one copy)
  unsigned char* tab_host = nullptr; unsigned char* tab_dev = nullptr;
  hipEvent_t ev_gtab = nullptr;
  Arena ws;
  // last step
  int B = 0, S_max = 0, T_max = 0, S = 0, U = 0;
  // test hook (mm_debug_attention): the forward attention launches of the last training step and
  // host copies of its prefix sums
  struct AttnLog { AttnParams p; int kind; };
  std::vector<AttnLog> attn_log;
  std::vector<int32_t> h_cu_s, h_cu_u;
  bool pending = false; int pending_task = -1;
  float last_loss = 0.f; mm_status last_status = MM_OK;
  // profiling
  bool prof = false;
  std::vector<ProfRec> prof_recs; std::vector<hipEvent_t> ev_pool;
  double prof_ms[MM_K_COUNT] = {}; int64_t prof_n[MM_K_COUNT] = {}; double prof_work[MM_K_COUNT] = {};
};

namespace {

mm_status fail(mm_ctx* c, mm_status s, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf;
  return s;
}

#define HIP_TRY(c, call)                                                                       \
  do {                                                                                         \
    hipError_t e_ = (call);                                                                    \
    if (e_ != hipSuccess)                                                                      \
      return fail(c, e_ == hipErrorOutOfMemory ? MM_ENOMEM : MM_EHIP, "%s: %s", #call,         \
                  hipGetErrorString(e_));                                                      \
  } while (0)

// ---------------------------------------------------------------------------------------------
// bucket layout: tensor order and 64-element alignment (the ABI's "bucket layout")
// ---------------------------------------------------------------------------------------------
void build_layout(const mm_config& cfg, Module& m) {
  const int d = cfg.d_model, F = cfg.d_ff, V = cfg.vocab, r = m.adapter_dim;
  int64_t cur = 0;
  auto add = [&](int rows, int cols, int role) {
    cur = round_up(cur, ALIGN_ELEMS);
    m.tensors.push_back({cur, rows, cols, role});
    cur += (int64_t)rows * cols;
  };
  auto ln = [&] { add(1, d, MM_T_GAMMA); add(1, d, MM_T_BETA); };
  auto attn = [&] { for (int i = 0; i < 4; ++i) { add(d, d, MM_T_MATRIX); add(1, d, MM_T_BIAS); } };
  auto ffn = [&] { add(d, F, MM_T_MATRIX); add(1, F, MM_T_BIAS); add(F, d, MM_T_MATRIX); add(1, d, MM_T_BIAS); };
  switch (m.kind) {
    case MM_SRC_EMB: case MM_TGT_EMB: add(V, d, MM_T_EMBED); break;
    case MM_ENC_STACK:
      for (int i = 0; i < m.n_layers; ++i) { ln(); attn(); ln(); ffn(); }
      if (m.owns_final_norm) ln();
      break;
    case MM_DEC_STACK:
      for (int i = 0; i < m.n_layers; ++i) { ln(); attn(); ln(); attn(); ln(); ffn(); }
      if (m.owns_final_norm) ln();
      break;
    case MM_GENERATOR: add(d, V, MM_T_MATRIX); add(1, V, MM_T_BIAS); break;
    case MM_ADAPTER:
      for (int i = 0; i < m.n_layers; ++i) {
        ln(); add(d, r, MM_T_MATRIX); add(1, r, MM_T_BIAS); add(r, d, MM_T_MATRIX); add(1, d, MM_T_BIAS);
      }
      break;
  }
  m.P = round_up(cur, ALIGN_ELEMS);
}

constexpr int ENC_T = 16, DEC_T = 26, ADP_T = 6;
constexpr int MAX_GROUPED = 1024;

// ---------------------------------------------------------------------------------------------
// launch wrappers: skip in the measuring pass, bracket with events when profiling
// ---------------------------------------------------------------------------------------------
struct Run {
  mm_ctx* c;
  bool dry;
  hipEvent_t get_event() {
    if (!c->ev_pool.empty()) { hipEvent_t e = c->ev_pool.back(); c->ev_pool.pop_back(); return e; }
    hipEvent_t e; hipEventCreate(&e); return e;
  }
  // Timing: one event after every launch and one at the start of each call; a launch is charged
  // the time since the previous event on the stream.  (A pair of events around each launch would
  // add two markers per launch to the queue and time the gaps they create.)
  int open_cls = -1;
  void mark() {
    if (!c->prof) return;
    ProfRec r{-1, get_event(), nullptr};
    hipEventRecord(r.e, c->st);
    c->prof_recs.push_back(r);
  }
  void begin(int cls, double work) {
    if (!c->prof) return;
    open_cls = cls;
    c->prof_n[cls] += 1;
    c->prof_work[cls] += work;
  }
  void end() {
    if (!c->prof) return;
    ProfRec r{open_cls, get_event(), nullptr};
    hipEventRecord(r.e, c->st);
    c->prof_recs.push_back(r);
  }
  // GEMM launches carry their own start/stop timestamps instead
  LaunchEvents begin_timed(int cls, double work) {
    LaunchEvents ev;
    if (!c->prof) return ev;
    c->prof_n[cls] += 1;
    c->prof_work[cls] += work;
    ev.start = get_event(); ev.stop = get_event();
    c->prof_recs.push_back(ProfRec{cls, ev.stop, ev.start});
    return ev;
  }
  size_t esz() const { return c->dt == BF16 ? 2 : 4; }

  void gemm(const GemmParams& p) {
    if (dry) return;
    launch_gemm(c->st, c->dt, p, begin_timed(MM_K_GEMM, 2.0 * p.M * p.N * p.K));
  }
  // Independent products of one kind: one launch for up to GEMM_MULTI_MAX of them where the
  // kernel allows it, else one by one.
  void gemm_set(const std::vector<GemmParams>& ps) {
    if (dry) return;
    for (size_t i0 = 0; i0 < ps.size(); i0 += GEMM_MULTI_MAX) {
      const int n = (int)std::min(ps.size() - i0, (size_t)GEMM_MULTI_MAX);
      double flops = 0;
      for (int i = 0; i < n; ++i) flops += 2.0 * ps[i0 + i].M * ps[i0 + i].N * ps[i0 + i].K;
      if (n > 1 && c->dt == BF16) {
        LaunchEvents ev = begin_timed(MM_K_GEMM, flops);
        if (launch_gemm_multi(c->st, c->dt, ps.data() + i0, n, ev)) continue;
        // not taken: hand the timing slot to the first single launch instead
        launch_gemm(c->st, c->dt, ps[i0], ev);
        for (int i = 1; i < n; ++i) gemm(ps[i0 + i]);
        continue;
      }
      for (int i = 0; i < n; ++i) gemm(ps[i0 + i]);
    }
  }
  void ln_fwd(const float* x, const float* g, const float* b, void* y, float* mean, float* rstd, int rows) {
    if (dry) return;
    const int d = c->cfg.d_model;
    launch_layernorm_fwd(c->st, c->dt, x, g, b, y, mean, rstd, rows, d, c->cfg.ln_eps,
                         begin_timed(MM_K_LAYERNORM_FWD, (double)rows * d * 2 * esz()));
  }
  // The gain/shift gradient sums of all LayerNorms of the step are reduced in one launch at the end.
  std::vector<LnReduceJob>* ln_jobs = nullptr;
  void ln_bwd(const float* dy, const float* x, const float* mean, const float* rstd, const float* g,
              const float* dres, float* dx, void* dxT, float* gg, float* gb, int rows, bool fresh, int dy_parts = 1,
              int64_t dy_part_stride = 0) {
    const int d = c->cfg.d_model;
    const int n_partial = ln_bwd_partial_rows(rows);
    float* partial = (float*)c->ws.take((size_t)n_partial * 2 * d * sizeof(float));
    if (dry) return;
    launch_layernorm_bwd(c->st, c->dt, dy, x, mean, rstd, g, dres, dx, c->dt == BF16 ? dxT : nullptr, partial, rows, d,
                         begin_timed(MM_K_LAYERNORM_BWD, (double)rows * d * 3 * esz()),
                         dy_parts, dy_part_stride);
    LnReduceJob jb;
    jb.partial = partial; jb.dgamma = gg; jb.dbeta = gb; jb.n_partial = n_partial; jb.d = d;
    jb.first_block = 0; jb.overwrite = fresh;
    ln_jobs->push_back(jb);
  }
  void colsum(const void* Y, int y_f32, int64_t ldy, int M, int N, float* partial, float* dst, int split,
              int64_t seg, bool overwrite) {
    if (dry) return;
    begin(MM_K_COLSUM, (double)M * N * (y_f32 ? 4 : esz()));
    launch_colsum(c->st, c->dt, Y, y_f32, ldy, M, N, partial, dst, split, seg, overwrite);
    end();
  }
  void attn_fwd(const AttnParams& p, double flops) {
    if (dry) return;
    launch_attn_fwd(c->st, c->dt, p, begin_timed(MM_K_ATTN_FWD, flops));
  }
  void attn_bwd(const AttnParams& p, double flops) {
    if (dry) return;
    launch_attn_bwd(c->st, c->dt, p, begin_timed(MM_K_ATTN_BWD, flops));
  }
};

// Buckets of modules whose every element receives a gradient in every step that uses the module
// (stacks, generator, adapters) are not zeroed by the update: the first step after an update
// overwrites them and later steps add.  Embedding tables get gradient rows for the batch's tokens
// only, so the update zeroes their buckets and every step adds.
inline bool bucket_overwrites(int kind) { return kind != MM_SRC_EMB && kind != MM_TGT_EMB; }

// parameter views of one layer ------------------------------------------------------------------
struct PV {
  mm_ctx* c; Module* m; int base;
  int64_t off(int i) const { return m->tensors[base + i].off; }
  const void* W(int i) const {  // working-dtype matrix
    return c->dt == BF16 ? (const void*)(m->w16 + off(i)) : (const void*)(m->theta + off(i));
  }
  const float* V(int i) const { return m->theta + off(i); }  // fp32 vector (bias, gamma, beta)
  float* G(int i) const { return m->g + off(i); }
  // First use of the module's bucket since its last update: gradients are written, not added
  // (see bucket_overwrites).
  bool fresh() const { return bucket_overwrites(m->kind) && m->touched == 0; }
};

struct LnSave { float* mean; float* rstd; };
struct FfnSave { float* x_in; LnSave ln; void* a; void* h; float* x_out; };
struct SelfSave { float* x_in; LnSave ln; void* a; void* qkv; float* lse; void* o; float* x_out; };
struct CrossSave { float* x_in; LnSave ln; void* a; void* q; void* kv; float* lse; void* o; float* x_out; };
struct LayerSave {
  PV pv; SelfSave self; CrossSave cross; FfnSave ffn; bool has_adapter = false; PV apv; FfnSave ad;
};

struct Step {
  mm_ctx* c; Run run; const Route* rt;
  int d, H, F, V, dh, S, U, B;
  int max_s, max_u;
  double sum_ss = 0, sum_uu = 0, sum_us = 0;  // sum over sentences of len products (flop tallies)
  size_t esz;
  Arena& ws() { return c->ws; }
  float* f32(size_t n) { return (float*)ws().take(n * 4); }
  void* act(size_t n) { return ws().take(n * esz); }

  GemmParams gp(const void* A, int64_t lda, const void* B_, int64_t ldb, void* C, int64_t ldc, int M, int N, int K) {
    GemmParams p;
    memset(&p, 0, sizeof p);
    p.A = A; p.B = B_; p.C = C; p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    return p;
  }
  // dX[R,K] = dY[R,N] * W^T, W stored [K,N]
  GemmParams gp_dgrad(const void* dY, int64_t ldy, const void* W, int K, int N, void* dX, int R) {
    GemmParams p = gp(dY, ldy, W, N, dX, K, R, K, N);
    p.transB = 1;
    return p;
  }
  // G[K,N] += X^T[K,R] * dY[R,N]
  GemmParams gp_wgrad(const void* X, int64_t ldx, const void* dY, int64_t ldy, float* G, int K, int N, int R) {
    GemmParams p = gp(X, ldx, dY, ldy, G, N, K, N, R);
    p.transA = 1; p.out_f32 = 1; p.residual = G; p.ldr = N;
    return p;
  }

  AttnParams ap(const void* q, int64_t ldq, const void* k, const void* v, int64_t ldkv, void* o, float* lse,
                bool q_is_dec, bool k_is_dec, int causal) {
    AttnParams a;
    memset(&a, 0, sizeof a);
    a.q = q; a.k = k; a.v = v; a.o = o; a.ldq = ldq; a.ldk = ldkv; a.ldv = ldkv; a.ldo = d; a.lse = lse;
    a.cu_q = q_is_dec ? c->cu_u : c->cu_s; a.cu_k = k_is_dec ? c->cu_u : c->cu_s;
    a.B = B; a.H = H; a.dh = dh; a.causal = causal; a.rows_q = q_is_dec ? U : S;
    a.max_lq = q_is_dec ? max_u : max_s; a.max_lk = k_is_dec ? max_u : max_s;
    return a;
  }
  double pair_sum(bool q_is_dec, bool k_is_dec) const { return q_is_dec ? (k_is_dec ? sum_uu : sum_us) : sum_ss; }

  // ---- forward blocks -------------------------------------------------------------------------
  // x_out = x_in + W2 relu(W1 LN(x_in) + b1) + b2 ; tensors at pv.base + t0: ln.g ln.b W1 b1 W2 b2
  FfnSave ffn_fwd(const PV& pv, int t0, float* x_in, int R, int hidden) {
    FfnSave s;
    s.x_in = x_in; s.ln.mean = f32(R); s.ln.rstd = f32(R);
    s.a = act((size_t)R * d); s.h = act((size_t)R * hidden); s.x_out = f32((size_t)R * d);
    run.ln_fwd(x_in, pv.V(t0), pv.V(t0 + 1), s.a, s.ln.mean, s.ln.rstd, R);
    GemmParams p = gp(s.a, d, pv.W(t0 + 2), hidden, s.h, hidden, R, hidden, d);
    p.bias = pv.V(t0 + 3); p.relu = 1;
    run.gemm(p);
    p = gp(s.h, hidden, pv.W(t0 + 4), d, s.x_out, d, R, d, hidden);
    p.bias = pv.V(t0 + 5); p.residual = x_in; p.ldr = d; p.out_f32 = 1;
    run.gemm(p);
    return s;
  }
  // tensors at t0: ln.g ln.b Wq bq Wk bk Wv bv Wo bo
  SelfSave self_fwd(const PV& pv, int t0, float* x_in, int R, bool is_dec) {
    SelfSave s;
    s.x_in = x_in; s.ln.mean = f32(R); s.ln.rstd = f32(R);
    s.a = act((size_t)R * d); s.qkv = act((size_t)R * 3 * d); s.lse = f32((size_t)H * R);
    s.o = act((size_t)R * d); s.x_out = f32((size_t)R * d);
    run.ln_fwd(x_in, pv.V(t0), pv.V(t0 + 1), s.a, s.ln.mean, s.ln.rstd, R);
    const int64_t seg = pv.off(t0 + 4) - pv.off(t0 + 2);
    GemmParams p = gp(s.a, d, pv.W(t0 + 2), d, s.qkv, 3 * d, R, 3 * d, d);
    p.b_split = d; p.b_seg_stride = seg; p.bias = pv.V(t0 + 3); p.bias_split = d; p.bias_seg_stride = seg;
    run.gemm(p);
    const char* qkv = (const char*)s.qkv;
    AttnParams a = ap(qkv, 3 * d, dry() ? nullptr : qkv + (size_t)d * esz, dry() ? nullptr : qkv + (size_t)2 * d * esz,
                      3 * d, s.o, s.lse, is_dec, is_dec, is_dec ? 1 : 0);
    run.attn_fwd(a, 4.0 * pair_sum(is_dec, is_dec) * d);
    if (!dry()) c->attn_log.push_back({a, is_dec ? 1 : 0});
    p = gp(s.o, d, pv.W(t0 + 8), d, s.x_out, d, R, d, d);
    p.bias = pv.V(t0 + 9); p.residual = x_in; p.ldr = d; p.out_f32 = 1;
    run.gemm(p);
    return s;
  }
  // The key/value projection of the encoder output, [S, 2d], for one decoder layer.
  GemmParams gp_cross_kv(const PV& pv, int t0, const void* mem, void* kv) {
    const int64_t seg = pv.off(t0 + 6) - pv.off(t0 + 4);
    GemmParams p = gp(mem, d, pv.W(t0 + 4), d, kv, 2 * d, S, 2 * d, d);
    p.b_split = d; p.b_seg_stride = seg; p.bias = pv.V(t0 + 5); p.bias_split = d; p.bias_seg_stride = seg;
    return p;
  }
  // kv: the layer's key/value projection, computed beforehand (all layers' in one launch)
  CrossSave cross_fwd(const PV& pv, int t0, float* x_in, void* kv_ready) {
    CrossSave s;
    s.x_in = x_in; s.ln.mean = f32(U); s.ln.rstd = f32(U);
    s.a = act((size_t)U * d); s.q = act((size_t)U * d); s.kv = kv_ready;
    s.lse = f32((size_t)H * U); s.o = act((size_t)U * d); s.x_out = f32((size_t)U * d);
    run.ln_fwd(x_in, pv.V(t0), pv.V(t0 + 1), s.a, s.ln.mean, s.ln.rstd, U);
    GemmParams p = gp(s.a, d, pv.W(t0 + 2), d, s.q, d, U, d, d);
    p.bias = pv.V(t0 + 3);
    run.gemm(p);
    const char* kv = (const char*)s.kv;
    AttnParams a = ap(s.q, d, kv, dry() ? nullptr : kv + (size_t)d * esz, 2 * d, s.o, s.lse, true, false, 0);
    run.attn_fwd(a, 4.0 * sum_us * d);
    if (!dry()) c->attn_log.push_back({a, 2});
    p = gp(s.o, d, pv.W(t0 + 8), d, s.x_out, d, U, d, d);
    p.bias = pv.V(t0 + 9); p.residual = x_in; p.ldr = d; p.out_f32 = 1;
    run.gemm(p);
    return s;
  }
  bool dry() const { return run.dry; }

  // ---- backward blocks --------------------------------------------------------------------------
  // In: dx (fp32) and dxT (working dtype copy) w.r.t. the block output.  Out: same w.r.t. its input.
  struct Grad { float* dx; void* dxT; };

  float* partial = nullptr;  // scratch for column-sum / LayerNorm partials

  // Weight-gradient products are independent of everything later in the step (their operands are
  // saved activations and gradients that stay in the workspace), and each alone has too few
  // output tiles for 256 compute units: they are collected and run as one grouped launch.
  std::vector<GemmParams> deferred;
  // p: the weight-gradient product dW += X^T dY.  gb: the bias gradient that goes with it
  // (db += column sums of dY, segmented like dW); Yf32: an fp32 version of dY if one exists.
  // fresh: the bucket holds nothing yet (PV::fresh): both results replace what is there.
  void wgrad(GemmParams p, float* gb, const float* Yf32, bool fresh) {
    if (dry()) return;
    if (fresh) p.residual = nullptr;
    if ((int)deferred.size() < MAX_GROUPED && gemm_groupable(c->dt, p)) {
      p.colsum_dst = gb;
      p.colsum_overwrite = fresh;
      deferred.push_back(p);
      return;
    }
    run.gemm(p);
    if (Yf32) run.colsum(Yf32, 1, p.ldb, p.K, p.N, partial, gb, p.c_split, p.c_seg_stride, fresh);
    else run.colsum(p.B, 0, p.ldb, p.K, p.N, partial, gb, p.c_split, p.c_seg_stride, fresh);
  }
  // End of the step: the deferred weight-gradient products as one grouped launch, then the
  // LayerNorm gain/shift partial sums as one launch.  Their tables go up in a single copy.
  void flush_deferred() {
    if (dry()) return;
    std::vector<LnReduceJob>& jobs = *run.ln_jobs;
    const size_t ng = deferred.size();
    const size_t nl = jobs.size() < (size_t)MAX_GROUPED_C ? jobs.size() : (size_t)MAX_GROUPED_C;
    if (!ng && !nl) return;
    hipEventSynchronize(c->ev_gtab);  // the previous step's upload has left the pinned block
    const size_t off_start = (ng * sizeof(GemmParams) + 15) & ~(size_t)15;
    const size_t off_jobs = (off_start + ng * sizeof(int32_t) + 15) & ~(size_t)15;
    const size_t total = off_jobs + nl * sizeof(LnReduceJob);
    GemmParams* gtab = reinterpret_cast<GemmParams*>(c->tab_host);
    int32_t* gstart = reinterpret_cast<int32_t*>(c->tab_host + off_start);
    LnReduceJob* ljob = reinterpret_cast<LnReduceJob*>(c->tab_host + off_jobs);
    int tiles = 0, blocks = 0;
    double flops = 0;
    std::vector<int> ntile(ng), order(ng);
    for (size_t i = 0; i < ng; ++i) ntile[i] = gemm_grouped_tiles(deferred[i]);
    gemm_grouped_order(ntile.data(), (int)ng, order.data());
    for (size_t i = 0; i < ng; ++i) {
      GemmParams& p = deferred[order[i]];
      gemm_prepare_grouped(p);
      gtab[i] = p;
      gstart[i] = tiles;
      tiles += ntile[order[i]];
      flops += 2.0 * p.M * p.N * p.K;
    }
    for (size_t i = 0; i < nl; ++i) {
      jobs[i].first_block = blocks;
      blocks += (2 * jobs[i].d + 63) / 64;
      ljob[i] = jobs[i];
    }
    launch_upload_words(c->st, c->tab_host, c->tab_dev, total, nullptr);
    hipEventRecord(c->ev_gtab, c->st);
    if (ng)
      launch_gemm_grouped_tn(c->st, reinterpret_cast<const GemmParams*>(c->tab_dev),
                             reinterpret_cast<const int32_t*>(c->tab_dev + off_start), (int)ng, tiles,
                             run.begin_timed(MM_K_GEMM, flops));
    if (nl) {
      run.begin(MM_K_LAYERNORM_BWD, 0.0);
      launch_ln_reduce_grouped(c->st, reinterpret_cast<const LnReduceJob*>(c->tab_dev + off_jobs), (int)nl, blocks);
      run.end();
    }
    deferred.clear();
    jobs.clear();
  }

  Grad ffn_bwd(const PV& pv, int t0, const FfnSave& s, Grad g, int R, int hidden) {
    void* dh = act((size_t)R * hidden);
    float* da = f32((size_t)R * d);
    Grad out{f32((size_t)R * d), c->dt == BF16 ? act((size_t)R * d) : nullptr};
    // d hidden = (dx W2^T) masked by relu
    GemmParams p = gp_dgrad(g.dxT, d, pv.W(t0 + 4), hidden, d, dh, R);
    p.relu_mask = s.h; p.ldm = hidden;
    run.gemm(p);
    wgrad(gp_wgrad(s.h, hidden, g.dxT, d, pv.G(t0 + 4), hidden, d, R), pv.G(t0 + 5), g.dx, pv.fresh());
    p = gp_dgrad(dh, hidden, pv.W(t0 + 2), d, hidden, da, R);
    p.out_f32 = 1;
    run.gemm(p);
    wgrad(gp_wgrad(s.a, d, dh, hidden, pv.G(t0 + 2), d, hidden, R), pv.G(t0 + 3), nullptr, pv.fresh());
    run.ln_bwd(da, s.x_in, s.ln.mean, s.ln.rstd, pv.V(t0), g.dx, out.dx, out.dxT, pv.G(t0), pv.G(t0 + 1), R, pv.fresh());
    if (c->dt != BF16) out.dxT = out.dx;
    return out;
  }

  Grad self_bwd(const PV& pv, int t0, const SelfSave& s, Grad g, int R, bool is_dec) {
    void* d_o = act((size_t)R * d);
    void* dqkv = act((size_t)R * 3 * d);
    float* da = f32((size_t)R * d);
    Grad out{f32((size_t)R * d), c->dt == BF16 ? act((size_t)R * d) : nullptr};
    run.gemm(gp_dgrad(g.dxT, d, pv.W(t0 + 8), d, d, d_o, R));
    wgrad(gp_wgrad(s.o, d, g.dxT, d, pv.G(t0 + 8), d, d, R), pv.G(t0 + 9), g.dx, pv.fresh());
    const char* qkv = (const char*)s.qkv;
    char* dq = (char*)dqkv;
    AttnParams a = ap(qkv, 3 * d, dry() ? nullptr : qkv + (size_t)d * esz, dry() ? nullptr : qkv + (size_t)2 * d * esz,
                      3 * d, s.o, s.lse, is_dec, is_dec, is_dec ? 1 : 0);
    a.d_o = d_o; a.lddo = d;
    a.dq = dq; a.dk = dry() ? nullptr : dq + (size_t)d * esz; a.dv = dry() ? nullptr : dq + (size_t)2 * d * esz;
    a.lddq = a.lddk = a.lddv = 3 * d;
    run.attn_bwd(a, 10.0 * pair_sum(is_dec, is_dec) * d);
    const int64_t seg = pv.off(t0 + 4) - pv.off(t0 + 2);
    GemmParams p = gp_dgrad(dqkv, 3 * d, pv.W(t0 + 2), d, 3 * d, da, R);
    p.ldb = d; p.b_split = d; p.b_split_on_k = 1; p.b_seg_stride = seg; p.out_f32 = 1;
    run.gemm(p);
    p = gp_wgrad(s.a, d, dqkv, 3 * d, pv.G(t0 + 2), d, 3 * d, R);
    p.ldc = d; p.ldr = d; p.c_split = d; p.c_seg_stride = seg;
    wgrad(p, pv.G(t0 + 3), nullptr, pv.fresh());
    run.ln_bwd(da, s.x_in, s.ln.mean, s.ln.rstd, pv.V(t0), g.dx, out.dx, out.dxT, pv.G(t0), pv.G(t0 + 1), R, pv.fresh());
    if (c->dt != BF16) out.dxT = out.dx;
    return out;
  }

  // dmem_part: this layer's own fp32 part of the gradient w.r.t. the encoder output; its product is
  // appended to dmem_jobs and launched with the other layers' once the decoder's backward is done.
  Grad cross_bwd(const PV& pv, int t0, const CrossSave& s, Grad g, const void* mem, float* dmem_part,
                 std::vector<GemmParams>& dmem_jobs) {
    void* d_o = act((size_t)U * d);
    void* dq = act((size_t)U * d);
    void* dkv = act((size_t)S * 2 * d);
    float* da = f32((size_t)U * d);
    Grad out{f32((size_t)U * d), c->dt == BF16 ? act((size_t)U * d) : nullptr};
    run.gemm(gp_dgrad(g.dxT, d, pv.W(t0 + 8), d, d, d_o, U));
    wgrad(gp_wgrad(s.o, d, g.dxT, d, pv.G(t0 + 8), d, d, U), pv.G(t0 + 9), g.dx, pv.fresh());
    const char* kv = (const char*)s.kv;
    char* dkvc = (char*)dkv;
    AttnParams a = ap(s.q, d, kv, dry() ? nullptr : kv + (size_t)d * esz, 2 * d, s.o, s.lse, true, false, 0);
    a.d_o = d_o; a.lddo = d; a.dq = dq; a.lddq = d;
    a.dk = dkvc; a.dv = dry() ? nullptr : dkvc + (size_t)d * esz; a.lddk = a.lddv = 2 * d;
    run.attn_bwd(a, 10.0 * sum_us * d);
    // query side
    GemmParams p = gp_dgrad(dq, d, pv.W(t0 + 2), d, d, da, U);
    p.out_f32 = 1;
    run.gemm(p);
    wgrad(gp_wgrad(s.a, d, dq, d, pv.G(t0 + 2), d, d, U), pv.G(t0 + 3), nullptr, pv.fresh());
    // memory side: this layer's part of d mem = dkv [Wk|Wv]^T
    const int64_t seg = pv.off(t0 + 6) - pv.off(t0 + 4);
    p = gp_dgrad(dkv, 2 * d, pv.W(t0 + 4), d, 2 * d, dmem_part, S);
    p.ldb = d; p.b_split = d; p.b_split_on_k = 1; p.b_seg_stride = seg; p.out_f32 = 1;
    dmem_jobs.push_back(p);
    p = gp_wgrad(mem, d, dkv, 2 * d, pv.G(t0 + 4), d, 2 * d, S);
    p.ldc = d; p.ldr = d; p.c_split = d; p.c_seg_stride = seg;
    wgrad(p, pv.G(t0 + 5), nullptr, pv.fresh());
    run.ln_bwd(da, s.x_in, s.ln.mean, s.ln.rstd, pv.V(t0), g.dx, out.dx, out.dxT, pv.G(t0), pv.G(t0 + 1), U, pv.fresh());
    if (c->dt != BF16) out.dxT = out.dx;
    return out;
  }
};

// per parameter: g, theta, m, v read (16 B); theta, m, v written (12 B); bf16 copy (2 B).  An
// embedding table is tallied with the 16 B of reads only: rows that never received a gradient
// (g = m = v = 0, most rows under a Zipf law) are left alone by the kernel, how many is not known
// on the host, and the zeroing of the bucket touches only the pieces that held a gradient.
double work_bytes_adam(const mm_ctx* c, int64_t n, bool table) {
  return (double)n * (table ? 16.0 : c->dt == BF16 ? 30.0 : 28.0);
}

mm_status collect_profile(mm_ctx* c) {
  if (c->prof_recs.empty()) return MM_OK;
  HIP_TRY(c, hipStreamSynchronize(c->st));
  hipEvent_t prev = nullptr;
  for (auto& r : c->prof_recs) {
    float ms = 0.f;
    hipEvent_t from = r.s ? r.s : prev;
    if (r.cls >= 0 && from && hipEventElapsedTime(&ms, from, r.e) == hipSuccess) c->prof_ms[r.cls] += ms;
    prev = r.e;
  }
  for (auto& r : c->prof_recs) { c->ev_pool.push_back(r.e); if (r.s) c->ev_pool.push_back(r.s); }
  c->prof_recs.clear();
  return MM_OK;
}

// Resolves the outcome of the most recent step (waits for it).
mm_status resolve_pending(mm_ctx* c) {
  if (!c->pending) return c->last_status;
  HIP_TRY(c, hipEventSynchronize(c->ev_done));
  c->pending = false;
  c->last_loss = c->result_host[0];
  int32_t flag;
  memcpy(&flag, &c->result_host[1], 4);
  if (flag != 0) {
    // the step counted for nothing.  A module that an update enqueued behind it was to change on
    // this step's account alone was left alone by the kernel: its update count goes back too.
    for (int j : c->routes[c->pending_task].ids) {
      Module& m = c->mods[j];
      if (m.t_on_trust) { m.t -= 1; m.t_on_trust = false; }
      else if (m.touched > 0) m.touched -= 1;
    }
    c->last_status = fail(c, MM_ERANGE, flag & 1 ? "token id outside [0, vocab) (found on the device); step had no effect"
                                                 : "non-pad id after the end of a sentence (found on the device); step had no effect");
    return c->last_status;
  }
  for (int j : c->routes[c->pending_task].ids) c->mods[j].t_on_trust = false;
  if (!std::isfinite(c->last_loss)) {
    c->last_status = fail(c, MM_ENONFINITE, "loss is not finite");
    return c->last_status;
  }
  c->last_status = MM_OK;
  return MM_OK;
}

// Before an update: settles the step in flight if it has finished (no wait).  Returns true if it
// is still running; the update is then enqueued behind it and decides on the device
// (AdamSegment::n_uses_alt), so that the host does not have to wait for the step's end.
bool step_still_running(mm_ctx* c) {
  if (!c->pending) return false;
  if (hipEventQuery(c->ev_done) != hipSuccess) {
    (void)hipGetLastError();   // "not ready" is an answer, not an error
    return true;
  }
  resolve_pending(c);
  return false;
}

mm_status ensure_stage(mm_ctx* c, size_t n_ints) {
  if (n_ints <= c->stage_cap) return MM_OK;
  HIP_TRY(c, hipStreamSynchronize(c->st));
  if (c->stage) hipHostFree(c->stage);
  c->stage = nullptr; c->stage_cap = 0;
  const size_t cap = n_ints + n_ints / 2 + 1024;
  HIP_TRY(c, hipHostMalloc((void**)&c->stage, cap * sizeof(int32_t), hipHostMallocDefault));
  c->stage_cap = cap;
  return MM_OK;
}

mm_status ensure_ids_dev(mm_ctx* c, size_t n_ints) {
  if (n_ints <= c->ids_dev_cap) return MM_OK;
  HIP_TRY(c, hipStreamSynchronize(c->st));
  if (c->ids_dev) hipFree(c->ids_dev);
  c->ids_dev = nullptr; c->ids_dev_cap = 0;
  const size_t cap = n_ints + n_ints / 2 + 1024;
  HIP_TRY(c, hipMalloc((void**)&c->ids_dev, cap * sizeof(int32_t)));
  c->ids_dev_cap = cap;
  return MM_OK;
}

mm_status ensure_ws(mm_ctx* c, size_t bytes) {
  if (bytes <= c->ws.cap) return MM_OK;
  HIP_TRY(c, hipStreamSynchronize(c->st));
  if (c->ws.base) hipFree(c->ws.base);
  c->ws.base = nullptr; c->ws.cap = 0;
  const size_t cap = bytes + bytes / 8 + (1 << 20);
  HIP_TRY(c, hipMalloc((void**)&c->ws.base, cap));
  c->ws.cap = cap;
  return MM_OK;
}

// The whole step as a launch sequence.  Runs twice: once measuring workspace, once for real.
void run_step(mm_ctx* c, const Route& rt, bool dry, const int32_t* lens_host) {
  Step s;
  s.c = c; s.run = Run{c, dry}; s.rt = &rt;
  s.d = c->cfg.d_model; s.H = c->cfg.n_heads; s.F = c->cfg.d_ff; s.V = c->cfg.vocab; s.dh = s.d / s.H;
  s.S = c->S; s.U = c->U; s.B = c->B; s.esz = c->dt == BF16 ? 2 : 4;
  s.max_s = 0; s.max_u = 0;
  for (int b = 0; b < c->B; ++b) {
    const double sl = lens_host[2 * b], ul = lens_host[2 * b + 1] - 1;
    s.sum_ss += sl * sl; s.sum_uu += ul * ul; s.sum_us += ul * sl;
    if (sl > s.max_s) s.max_s = (int)sl;
    if (ul > s.max_u) s.max_u = (int)ul;
  }
  const int d = s.d, S = s.S, U = s.U, V = s.V;
  Run& run = s.run;
  if (!dry) { run.mark(); c->attn_log.clear(); }
  std::vector<LnReduceJob> ln_jobs;
  run.ln_jobs = &ln_jobs;
  c->ws.reset(dry);
  const int Rmax = S > U ? S : U;
  {
    size_t pn = 0;
    const int widest = std::max(std::max(3 * d, s.F), V);
    const size_t pc = (size_t)colsum_partial_rows(Rmax) * widest;
    s.partial = s.f32(pn > pc ? pn : pc);
  }
  const float sqrt_d = sqrtf((float)d);
  Module& m_src = c->mods[rt.src];
  Module& m_tgt = c->mods[rt.tgt];
  Module& m_gen = c->mods[rt.gen];
  auto emb_w = [&](Module& m) -> const void* { return c->dt == BF16 ? (const void*)m.w16 : (const void*)m.theta; };

  // ---------------- forward: encoder ----------------
  float* x = s.f32((size_t)S * d);
  if (!dry) {
    run.begin(MM_K_EMBED, (double)S * d * (s.esz + 4));
    launch_embed_fwd(c->st, c->dt, emb_w(m_src), c->pe, c->src_tok, c->src_pos, x, S, d, sqrt_d);
    run.end();
  }
  std::vector<LayerSave> enc_saves, dec_saves;
  int li = 0;
  for (int mid : rt.enc) {
    Module& m = c->mods[mid];
    for (int l = 0; l < m.n_layers; ++l, ++li) {
      LayerSave ls;
      ls.pv = PV{c, &m, l * ENC_T};
      ls.self = s.self_fwd(ls.pv, 0, x, S, false);
      ls.ffn = s.ffn_fwd(ls.pv, 10, ls.self.x_out, S, s.F);
      x = ls.ffn.x_out;
      if (rt.ad_enc >= 0) {
        ls.has_adapter = true;
        ls.apv = PV{c, &c->mods[rt.ad_enc], li * ADP_T};
        ls.ad = s.ffn_fwd(ls.apv, 0, x, S, c->mods[rt.ad_enc].adapter_dim);
        x = ls.ad.x_out;
      }
      enc_saves.push_back(ls);
    }
  }
  Module& m_enc_last = c->mods[rt.enc.back()];
  PV pv_encf{c, &m_enc_last, m_enc_last.n_layers * ENC_T};
  float* x_enc_top = x;
  LnSave ln_encf{s.f32(S), s.f32(S)};
  void* mem = s.act((size_t)S * d);
  run.ln_fwd(x, pv_encf.V(0), pv_encf.V(1), mem, ln_encf.mean, ln_encf.rstd, S);

  // ---------------- forward: decoder ----------------
  float* y = s.f32((size_t)U * d);
  if (!dry) {
    run.begin(MM_K_EMBED, (double)U * d * (s.esz + 4));
    launch_embed_fwd(c->st, c->dt, emb_w(m_tgt), c->pe, c->dec_tok, c->dec_pos, y, U, d, sqrt_d);
    run.end();
  }
  // every decoder layer's key/value projection of the encoder output depends on `mem` only:
  // all of them in one launch, ahead of the decoder
  std::vector<void*> kv_all;
  {
    std::vector<GemmParams> kv_jobs;
    for (int mid : rt.dec) {
      Module& m = c->mods[mid];
      for (int l = 0; l < m.n_layers; ++l) {
        kv_all.push_back(s.act((size_t)S * 2 * d));
        kv_jobs.push_back(s.gp_cross_kv(PV{c, &m, l * DEC_T}, 10, mem, kv_all.back()));
      }
    }
    run.gemm_set(kv_jobs);
  }
  li = 0;
  for (int mid : rt.dec) {
    Module& m = c->mods[mid];
    for (int l = 0; l < m.n_layers; ++l, ++li) {
      LayerSave ls;
      ls.pv = PV{c, &m, l * DEC_T};
      ls.self = s.self_fwd(ls.pv, 0, y, U, true);
      ls.cross = s.cross_fwd(ls.pv, 10, ls.self.x_out, kv_all[li]);
      ls.ffn = s.ffn_fwd(ls.pv, 20, ls.cross.x_out, U, s.F);
      y = ls.ffn.x_out;
      if (rt.ad_dec >= 0) {
        ls.has_adapter = true;
        ls.apv = PV{c, &c->mods[rt.ad_dec], li * ADP_T};
        ls.ad = s.ffn_fwd(ls.apv, 0, y, U, c->mods[rt.ad_dec].adapter_dim);
        y = ls.ad.x_out;
      }
      dec_saves.push_back(ls);
    }
  }
  Module& m_dec_last = c->mods[rt.dec.back()];
  PV pv_decf{c, &m_dec_last, m_dec_last.n_layers * DEC_T};
  float* y_dec_top = y;
  LnSave ln_decf{s.f32(U), s.f32(U)};
  void* h = s.act((size_t)U * d);
  run.ln_fwd(y, pv_decf.V(0), pv_decf.V(1), h, ln_decf.mean, ln_decf.rstd, U);

  // ---------------- generator + loss ----------------
  PV pv_gen{c, &m_gen, 0};
  void* z = s.act((size_t)U * V);
  float* loss_rows = s.f32(U);
  {
    GemmParams p = s.gp(h, d, pv_gen.W(0), V, z, V, U, V, d);
    p.bias = pv_gen.V(1);
    run.gemm(p);
  }
  if (!dry) {
    launch_ce(c->st, c->dt, z, c->label, loss_rows, U, V, c->cfg.label_smoothing, 1.0f / (float)U, c->flag,
              run.begin_timed(MM_K_CE, (double)U * V * s.esz * 2));
    run.begin(MM_K_OTHER, (double)U * 4);
    launch_sum_scaled(c->st, loss_rows, U, 1.0f / (float)U, c->loss_dev, c->result_host, c->flag);   // loss and flag go to the host from here
    run.end();
  }

  // ---------------- backward: generator, decoder ----------------
  // The generator's input gradient reduces over the vocabulary into only U x d outputs: its K range
  // is split over several workgroups per tile, each writing its own partial sum, and the
  // LayerNorm backward that consumes dh adds the parts.
  int dh_parts = 4;   // measured best of 1, 2, 4, 8 at V = 32000
  float* dh = s.f32((size_t)U * d * dh_parts);   // (sized before the decision below: same in the measuring pass)
  {
    GemmParams p = s.gp_dgrad(z, V, pv_gen.W(0), d, V, dh, U);
    p.out_f32 = 1;
    p.k_splits = dh_parts;
    p.k_chunk = (((V + dh_parts - 1) / dh_parts) + 127) / 128 * 128;   // whole pairs of K steps
    p.c_part_stride = (int64_t)U * d;
    if (dh_parts < 2 || !gemm_can_split_k(c->dt, p)) { p.k_splits = 0; dh_parts = 1; }
    run.gemm(p);
    s.wgrad(s.gp_wgrad(h, d, z, V, pv_gen.G(0), d, V, U), pv_gen.G(1), nullptr, pv_gen.fresh());
  }
  Step::Grad g{s.f32((size_t)U * d), c->dt == BF16 ? s.act((size_t)U * d) : nullptr};
  run.ln_bwd(dh, y_dec_top, ln_decf.mean, ln_decf.rstd, pv_decf.V(0), nullptr, g.dx, g.dxT,
             pv_decf.G(0), pv_decf.G(1), U, pv_decf.fresh(), dh_parts, (int64_t)U * d);
  if (c->dt != BF16) g.dxT = g.dx;
  // The gradient w.r.t. the encoder output is the sum of one product per decoder layer.  Each
  // writes its own part; the products run as one launch after the decoder's backward and the
  // encoder's closing LayerNorm backward adds the parts.
  const int n_dec_layers = (int)dec_saves.size();
  float* dmem = s.f32((size_t)S * d * n_dec_layers);
  std::vector<GemmParams> dmem_jobs;
  for (int i = n_dec_layers - 1; i >= 0; --i) {
    LayerSave& ls = dec_saves[i];
    if (ls.has_adapter) g = s.ffn_bwd(ls.apv, 0, ls.ad, g, U, c->mods[rt.ad_dec].adapter_dim);
    g = s.ffn_bwd(ls.pv, 20, ls.ffn, g, U, s.F);
    g = s.cross_bwd(ls.pv, 10, ls.cross, g, mem, dry ? nullptr : dmem + (size_t)i * S * d, dmem_jobs);
    g = s.self_bwd(ls.pv, 0, ls.self, g, U, true);
  }
  run.gemm_set(dmem_jobs);
  float* eg_partial = s.f32((size_t)Rmax * d);
  if (!dry) {
    hipStreamWaitEvent(c->st, c->ev_sorted, 0);  // the side stream's token sorts
    run.begin(MM_K_EMBED_GRAD, (double)U * d * 12);
    launch_embed_grad(c->st, c->sort_keys + 16384, g.dx, m_tgt.g, eg_partial, U, d, sqrt_d);
    run.end();
  }

  // ---------------- backward: encoder ----------------
  Step::Grad ge{s.f32((size_t)S * d), c->dt == BF16 ? s.act((size_t)S * d) : nullptr};
  run.ln_bwd(dmem, x_enc_top, ln_encf.mean, ln_encf.rstd, pv_encf.V(0), nullptr, ge.dx, ge.dxT,
             pv_encf.G(0), pv_encf.G(1), S, pv_encf.fresh(), n_dec_layers, (int64_t)S * d);
  if (c->dt != BF16) ge.dxT = ge.dx;
  for (int i = (int)enc_saves.size() - 1; i >= 0; --i) {
    LayerSave& ls = enc_saves[i];
    if (ls.has_adapter) ge = s.ffn_bwd(ls.apv, 0, ls.ad, ge, S, c->mods[rt.ad_enc].adapter_dim);
    ge = s.ffn_bwd(ls.pv, 10, ls.ffn, ge, S, s.F);
    ge = s.self_bwd(ls.pv, 0, ls.self, ge, S, false);
  }
  if (!dry) {
    run.begin(MM_K_EMBED_GRAD, (double)S * d * 12);
    launch_embed_grad(c->st, c->sort_keys, ge.dx, m_src.g, eg_partial, S, d, sqrt_d);
    run.end();
  }
  s.flush_deferred();
}

bool valid_module(mm_ctx* c, int id) { return id >= 0 && id < (int)c->mods.size(); }

// This device's copy of the static array `scratch` (each GPU has its own, at its own address).
constexpr int MAX_DEVICES = 64;
void* g_scratch_addr[MAX_DEVICES] = {};
std::mutex g_scratch_mu;
mm_status scratch_address(mm_ctx* c, void** out) {
  int dev = -1;
  HIP_TRY(c, hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(c, MM_EHIP, "device index %d outside [0, %d)", dev, MAX_DEVICES);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_addr[dev]) {
    void* p = nullptr;
    HIP_TRY(c, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(c, MM_EHIP, "hipGetSymbolAddress returned a null address");
    g_scratch_addr[dev] = p;
  }
  *out = g_scratch_addr[dev];
  return MM_OK;
}

// ---------------------------------------------------------------------------------------------
// Greedy translation of one batch of one task (section 3.2: only the task's own modules are
// read).  The encoder runs once; each decoder layer keeps the q|k|v rows of the tokens written
// so far ([B][max_new][3d]) and the key/value projection of the encoder output, so a step
// works on one new row per sentence.  Runs twice like the training step: measuring, then real.
// ---------------------------------------------------------------------------------------------
struct TranslateOut {
  int32_t* ids; int32_t* len;                       // greedy search: produced ids [B][max_new], counts [B]
  // beam search: per step and row the token and the row of the step before it continues; the final
  // scores (best hypothesis of sentence b in row b * beam); number of steps taken
  int32_t* hist_tok; int32_t* hist_parent; float* score; int steps;
};

// beam == 0: greedy search (arg-max of the logits).  beam >= 1: beam search over summed
// log-probabilities with beam rows per sentence.
mm_status run_translate(mm_ctx* c, const Route& rt, bool dry, const int32_t* src_lens, int max_new,
                        TranslateOut& out, int beam) {
  Step s;
  s.c = c; s.run = Run{c, dry}; s.rt = &rt;
  s.d = c->cfg.d_model; s.H = c->cfg.n_heads; s.F = c->cfg.d_ff; s.V = c->cfg.vocab; s.dh = s.d / s.H;
  s.S = c->S; s.U = c->B; s.B = c->B; s.esz = c->dt == BF16 ? 2 : 4;
  s.max_s = 0; s.max_u = 1;
  for (int b = 0; b < c->B; ++b) {
    const double sl = src_lens[b];
    s.sum_ss += sl * sl; s.sum_us += sl; s.sum_uu += 1;
    if (sl > s.max_s) s.max_s = (int)sl;
  }
  const int d = s.d, S = s.S, V = s.V, H = s.H, dh = s.dh;
  const int n_sent = s.B;                     // sentences
  const int kb = beam > 0 ? beam : 1;         // decoder rows per sentence
  const int B = n_sent * kb;                  // decoder rows (the name the decoding code below uses)
  const size_t esz = s.esz;
  Run& run = s.run;
  if (!dry) run.mark();
  c->ws.reset(dry);
  const float sqrt_d = sqrtf((float)d);
  Module& m_src = c->mods[rt.src];
  Module& m_tgt = c->mods[rt.tgt];
  Module& m_gen = c->mods[rt.gen];
  auto emb_w = [&](Module& m) -> const void* { return c->dt == BF16 ? (const void*)m.w16 : (const void*)m.theta; };

  // ---------------- encoder, once ----------------
  float* x = s.f32((size_t)S * d);
  if (!dry) launch_embed_fwd(c->st, c->dt, emb_w(m_src), c->pe, c->src_tok, c->src_pos, x, S, d, sqrt_d);
  int li = 0;
  for (int mid : rt.enc) {
    Module& m = c->mods[mid];
    for (int l = 0; l < m.n_layers; ++l, ++li) {
      PV pv{c, &m, l * ENC_T};
      x = s.self_fwd(pv, 0, x, S, false).x_out;
      x = s.ffn_fwd(pv, 10, x, S, s.F).x_out;
      if (rt.ad_enc >= 0) x = s.ffn_fwd(PV{c, &c->mods[rt.ad_enc], li * ADP_T}, 0, x, S, c->mods[rt.ad_enc].adapter_dim).x_out;
    }
  }
  Module& m_enc_last = c->mods[rt.enc.back()];
  PV pv_encf{c, &m_enc_last, m_enc_last.n_layers * ENC_T};
  void* mem = s.act((size_t)S * d);
  run.ln_fwd(x, pv_encf.V(0), pv_encf.V(1), mem, s.f32(S), s.f32(S), S);

  // ---------------- per decoder layer: key/value projection of the encoder output, token cache ----
  struct DecLayer { PV pv; bool has_adapter; PV apv; char* kv_mem; char* cache; char* cache_alt; };
  std::vector<DecLayer> layers;
  std::vector<GemmParams> kv_jobs;
  li = 0;
  for (int mid : rt.dec) {
    Module& m = c->mods[mid];
    for (int l = 0; l < m.n_layers; ++l, ++li) {
      DecLayer L;
      L.pv = PV{c, &m, l * DEC_T};
      L.has_adapter = rt.ad_dec >= 0;
      if (L.has_adapter) L.apv = PV{c, &c->mods[rt.ad_dec], li * ADP_T};
      L.kv_mem = (char*)s.act((size_t)S * 2 * d);
      L.cache = (char*)s.act((size_t)B * max_new * 3 * d);
      L.cache_alt = beam > 0 ? (char*)s.act((size_t)B * max_new * 3 * d) : nullptr;   // hypotheses move between rows
      kv_jobs.push_back(s.gp_cross_kv(L.pv, 10, mem, L.kv_mem));
      layers.push_back(L);
    }
  }
  run.gemm_set(kv_jobs);
  Module& m_dec_last = c->mods[rt.dec.back()];
  PV pv_decf{c, &m_dec_last, m_dec_last.n_layers * DEC_T};
  PV pv_gen{c, &m_gen, 0};

  // ---------------- decoding state ----------------
  int32_t* state = (int32_t*)c->ws.take(((size_t)3 * B + 1 + (size_t)B * max_new) * 4);
  int32_t* cur_tok = state;            // next decoder input (BOS first)
  int32_t* done = state + B;
  out.len = state + 2 * B;
  int32_t* n_done = state + 3 * B;
  out.ids = n_done + 1;
  if (!dry) {
    launch_fill_i32(c->st, cur_tok, B, 1 /* BOS */);
    launch_fill_i32(c->st, done, 2 * (size_t)B + 1 + (size_t)B * max_new, 0);   // done, len, n_done, ids
  }
  // beam search state: scores and finished flags in two copies (a step reads one and writes the
  // other), the row each new row continues, and the per-step history the host walks back at the end
  float* score[2] = {nullptr, nullptr};
  int32_t* bdone[2] = {nullptr, nullptr};
  int32_t* parent = nullptr; int32_t* n_fin = nullptr;
  if (beam > 0) {
    if ((int)layers.size() > BEAM_LAYERS_MAX) return fail(c, MM_EINVAL, "beam search supports at most %d decoder layers", BEAM_LAYERS_MAX);
    char* bs = (char*)c->ws.take(((size_t)5 * B + max_new + 2 * (size_t)B * max_new) * 4);
    score[0] = (float*)bs; score[1] = score[0] + B;
    bdone[0] = (int32_t*)(score[1] + B); bdone[1] = bdone[0] + B;
    parent = bdone[1] + B;
    n_fin = parent + B;
    out.hist_tok = n_fin + max_new;
    out.hist_parent = out.hist_tok + (size_t)B * max_new;
    if (!dry) {
      launch_beam_init(c->st, score[0], B, kb);
      launch_fill_i32(c->st, bdone[0], (size_t)3 * B + max_new + 2 * (size_t)B * max_new, 0);
    }
  }
  int32_t* n_done_host = (int32_t*)c->result_host + 8;
  const int64_t row3 = (int64_t)3 * d;                 // one cached row: q | k | v
  const int64_t seq3 = row3 * max_new;                 // one sentence's cache
  // One row per sentence leaves few tiles per product, so the products that write the residual
  // stream (d outputs from d or d_ff inputs) split their K range over several workgroups per
  // tile; the LayerNorm that reads the stream next adds the partial sums (and keeps the sum).
  struct Res { float* x; int parts; };
  const int64_t part_stride = (int64_t)B * d;
  constexpr int MAX_PARTS = 8;
  auto ln_in = [&](Res r, const float* g, const float* bta, float*& x_full) -> void* {
    void* a = s.act((size_t)B * d);
    x_full = r.parts > 1 ? s.f32((size_t)B * d) : r.x;
    float* mean = s.f32(B);
    float* rstd = s.f32(B);
    if (!dry)
      launch_layernorm_fwd(c->st, c->dt, r.x, g, bta, a, mean, rstd, B, d, c->cfg.ln_eps,
                           run.begin_timed(MM_K_LAYERNORM_FWD, (double)B * d * (4 * r.parts + esz)), r.parts,
                           part_stride, r.parts > 1 ? x_full : nullptr);
    return a;
  };
  // resid + A[B,K] W[K,d] + bias
  auto proj_out = [&](const void* A, int K, const void* W, const float* bias, const float* resid) -> Res {
    Res r{s.f32((size_t)B * d * MAX_PARTS), 1};
    GemmParams p = s.gp(A, K, W, d, r.x, d, B, d, K);
    p.bias = bias; p.residual = resid; p.ldr = d; p.out_f32 = 1;
    const int want = K >= 2048 ? 8 : K >= 512 ? 4 : 1;
    if (want > 1) {
      p.k_splits = want;
      p.k_chunk = (((K + want - 1) / want) + 63) / 64 * 64;
      p.c_part_stride = part_stride;
      if (gemm_can_split_k(c->dt, p)) r.parts = want; else p.k_splits = 0;
    }
    run.gemm(p);
    return r;
  };
  auto ffn_block = [&](const PV& pv, int t0, Res in, int hidden) -> Res {
    float* x_full;
    void* a = ln_in(in, pv.V(t0), pv.V(t0 + 1), x_full);
    void* hbuf = s.act((size_t)B * hidden);
    GemmParams p = s.gp(a, d, pv.W(t0 + 2), hidden, hbuf, hidden, B, hidden, d);
    p.bias = pv.V(t0 + 3); p.relu = 1;
    run.gemm(p);
    return proj_out(hbuf, hidden, pv.W(t0 + 4), pv.V(t0 + 5), x_full);
  };
  const size_t step_mark = c->ws.off;
  for (int t = 0; t < max_new; ++t) {
    c->ws.off = step_mark;                             // every step reuses the same buffers
    Res y{s.f32((size_t)B * d), 1};
    if (!dry) launch_embed_fwd(c->st, c->dt, emb_w(m_tgt), c->pe, cur_tok, nullptr, y.x, B, d, sqrt_d, t);
    for (DecLayer& L : layers) {
      const PV& pv = L.pv;
      // self-attention over the tokens so far (row t of the cache is written by the projection)
      float* x_full;
      void* a = ln_in(y, pv.V(0), pv.V(1), x_full);
      char* row_t = L.cache + (size_t)t * row3 * esz;
      const int64_t seg = pv.off(4) - pv.off(2);
      GemmParams p = s.gp(a, d, pv.W(2), d, row_t, seq3, B, 3 * d, d);
      p.b_split = d; p.b_seg_stride = seg; p.bias = pv.V(3); p.bias_split = d; p.bias_seg_stride = seg;
      run.gemm(p);
      void* o = s.act((size_t)B * d);
      if (!dry && !launch_attn_decode(c->st, c->dt, row_t, seq3, L.cache + (size_t)d * esz, L.cache + (size_t)2 * d * esz,
                                      row3, nullptr, max_new, t + 1, max_new, o, d, B, H, dh))
        return fail(c, MM_EINVAL, "decoding attention does not support head size %d", dh);
      y = proj_out(o, d, pv.W(8), pv.V(9), x_full);
      // attention over the encoder output
      a = ln_in(y, pv.V(10), pv.V(11), x_full);
      void* q = s.act((size_t)B * d);
      p = s.gp(a, d, pv.W(12), d, q, d, B, d, d);
      p.bias = pv.V(13);
      run.gemm(p);
      o = s.act((size_t)B * d);
      if (!dry && !launch_attn_decode(c->st, c->dt, q, d, L.kv_mem, L.kv_mem + (size_t)d * esz, 2 * d, c->cu_s, 0, 0,
                                      s.max_s, o, d, B, H, dh, kb))
        return fail(c, MM_EINVAL, "decoding attention does not support head size %d", dh);
      y = proj_out(o, d, pv.W(18), pv.V(19), x_full);
      y = ffn_block(pv, 20, y, s.F);
      if (L.has_adapter) y = ffn_block(L.apv, 0, y, c->mods[rt.ad_dec].adapter_dim);
    }
    float* x_full;
    void* h = ln_in(y, pv_decf.V(0), pv_decf.V(1), x_full);
    void* z = s.act((size_t)B * V);
    GemmParams p = s.gp(h, d, pv_gen.W(0), V, z, V, B, V, d);
    p.bias = pv_gen.V(1);
    run.gemm(p);
    if (dry) break;                                    // one step measures them all
    if (beam > 0) {
      const int cur = t & 1, nxt = cur ^ 1;
      if (!launch_beam_select(c->st, c->dt, z, n_sent, V, kb, t, 2 /* EOS */, score[cur], bdone[cur], score[nxt], bdone[nxt],
                              cur_tok, parent, out.hist_tok, out.hist_parent, n_fin))
        return fail(c, MM_EINVAL, "beam width %d is not supported", kb);
      out.score = score[nxt];
      out.steps = t + 1;
      if (t + 1 < max_new) {                           // the caches follow their hypotheses
        const char* src[BEAM_LAYERS_MAX]; char* dst[BEAM_LAYERS_MAX];
        for (size_t l = 0; l < layers.size(); ++l) { src[l] = layers[l].cache; dst[l] = layers[l].cache_alt; }
        if (!launch_cache_gather(c->st, src, dst, (int)layers.size(), parent, B, seq3 * (int64_t)esz,
                                 (int64_t)(t + 1) * row3 * (int64_t)esz))
          return fail(c, MM_EINVAL, "token cache rows are not multiples of 16 bytes");
        for (DecLayer& L : layers) std::swap(L.cache, L.cache_alt);
      }
      if ((t & 7) == 7 && t + 1 < max_new) {           // now and then: is every beam finished?
        HIP_TRY(c, hipMemcpyAsync(n_done_host, n_fin + t, 4, hipMemcpyDeviceToHost, c->st));
        HIP_TRY(c, hipStreamSynchronize(c->st));
        if (*n_done_host >= n_sent) break;
      }
      continue;
    }
    launch_greedy_pick(c->st, c->dt, z, B, V, t, max_new, 2 /* EOS */, cur_tok, done, out.ids, out.len, n_done);
    if ((t & 7) == 7 && t + 1 < max_new) {             // now and then: has every sentence finished?
      HIP_TRY(c, hipMemcpyAsync(n_done_host, n_done, 4, hipMemcpyDeviceToHost, c->st));
      HIP_TRY(c, hipStreamSynchronize(c->st));
      if (*n_done_host >= B) break;
    }
  }
  return MM_OK;
}

mm_status parse_route(mm_ctx* c, const int32_t* ids, int n, Route& r) {
  for (int i = 0; i < n; ++i)
    if (!valid_module(c, ids[i])) return fail(c, MM_EINVAL, "route names unknown module id %d", ids[i]);
  for (int i = 0; i < n; ++i)
    for (int j = i + 1; j < n; ++j)
      if (ids[i] == ids[j]) return fail(c, MM_EINVAL, "module %d appears twice in the route", ids[i]);
  int k = 0;
  auto kind = [&](int i) { return c->mods[ids[i]].kind; };
  r.ids.assign(ids, ids + n);
  if (k < n && kind(k) == MM_SRC_EMB) r.src = ids[k++];
  while (k < n && kind(k) == MM_ENC_STACK) r.enc.push_back(ids[k++]);
  if (k < n && kind(k) == MM_TGT_EMB) r.tgt = ids[k++];
  while (k < n && kind(k) == MM_DEC_STACK) r.dec.push_back(ids[k++]);
  if (k < n && kind(k) == MM_GENERATOR) r.gen = ids[k++];
  while (k < n && kind(k) == MM_ADAPTER) {
    Module& m = c->mods[ids[k]];
    int& slot = m.adapter_stack == 0 ? r.ad_enc : r.ad_dec;
    if (slot >= 0) return fail(c, MM_EINVAL, "more than one adapter for one stack");
    slot = ids[k++];
  }
  if (k != n || r.src < 0 || r.tgt < 0 || r.gen < 0 || r.enc.empty() || r.dec.empty())
    return fail(c, MM_EINVAL, "route must be src_emb, enc.., tgt_emb, dec.., generator, adapters..");
  for (auto* stack : {&r.enc, &r.dec}) {
    for (size_t pos = 0; pos < stack->size(); ++pos) {
      Module& m = c->mods[(*stack)[pos]];
      if (m.position != (int)pos)
        return fail(c, MM_EINVAL, "module %d is defined for position %d, used at position %zu", (*stack)[pos], m.position, pos);
      if ((m.owns_final_norm != 0) != (pos + 1 == stack->size()))
        return fail(c, MM_EINVAL, "exactly the last position of a stack must own the final norm");
    }
  }
  for (int which = 0; which < 2; ++which) {
    const int a = which == 0 ? r.ad_enc : r.ad_dec;
    if (a < 0) continue;
    int layers = 0;
    for (int id : (which == 0 ? r.enc : r.dec)) layers += c->mods[id].n_layers;
    if (c->mods[a].n_layers != layers) return fail(c, MM_EINVAL, "adapter must cover every layer of its stack");
  }
  return MM_OK;
}

mm_status check_module(mm_ctx* c, int module, int64_t n) {
  if (!c) return MM_EINVAL;
  if (!valid_module(c, module)) return fail(c, MM_EINVAL, "unknown module id %d", module);
  if (n != c->mods[module].P) return fail(c, MM_EINVAL, "length %lld does not match the bucket length %lld", (long long)n, (long long)c->mods[module].P);
  if (c->plan_only) return fail(c, MM_ESTATE, "plan-only context holds no device memory");
  return MM_OK;
}

}  // namespace

// =================================================================================================
// C ABI
// =================================================================================================
extern "C" {

mm_status mm_create(const mm_config* cfg, mm_ctx** out) {
  if (!cfg || !out) return MM_EINVAL;
  *out = nullptr;
  const int d = cfg->d_model, H = cfg->n_heads;
  if (d <= 0 || H <= 0 || d % H != 0 || d % 16 != 0 || cfg->d_ff <= 0 || cfg->d_ff % 16 != 0) return MM_EINVAL;
  const int dh = d / H;
  if (dh != 16 && dh != 32 && dh != 64) return MM_EINVAL;
  if (cfg->vocab < 8 || cfg->vocab % 8 != 0 || cfg->vocab > (1 << 17)) return MM_EINVAL;
  if (cfg->dtype != MM_F32 && cfg->dtype != MM_BF16) return MM_EINVAL;
  if (cfg->max_len < 1 || cfg->max_len > 256) return MM_EINVAL;
  if (cfg->max_batch_tokens < 1 || cfg->max_batch_tokens > 16384) return MM_EINVAL;
  if (!(cfg->label_smoothing >= 0.f && cfg->label_smoothing < 1.f)) return MM_EINVAL;
  mm_ctx* c = new (std::nothrow) mm_ctx();
  if (!c) return MM_ENOMEM;
  c->cfg = *cfg;
  c->dt = cfg->dtype == MM_BF16 ? BF16 : F32;
  c->st = (hipStream_t)cfg->hip_stream;
  c->plan_only = cfg->plan_only != 0;
  *out = c;
  if (c->plan_only) return MM_OK;
  if (attn_lds_bytes(c->dt, dh, cfg->max_len, cfg->max_len, true) > 160 * 1024) {
    fail(c, MM_EINVAL, "max_len %d does not fit the attention kernels' LDS budget for this dtype", cfg->max_len);
    return MM_EINVAL;
  }
  // sinusoidal position table: PE[p,2k] = sin(p * 10000^(-2k/d)), PE[p,2k+1] = cos(same)
  std::vector<float> pe((size_t)cfg->max_len * d);
  for (int p = 0; p < cfg->max_len; ++p)
    for (int k = 0; k < d / 2; ++k) {
      const double ang = (double)p * std::pow(10000.0, -2.0 * k / (double)d);
      pe[(size_t)p * d + 2 * k] = (float)std::sin(ang);
      pe[(size_t)p * d + 2 * k + 1] = (float)std::cos(ang);
    }
  const int T = cfg->max_batch_tokens;
  const size_t meta_ints = 2 * (size_t)(T + 1) + 2 * (size_t)T + 5 * (size_t)T + 64;
  mm_status s = MM_OK;
  auto guard = [&](hipError_t e, const char* what) {
    if (e != hipSuccess && s == MM_OK) s = fail(c, e == hipErrorOutOfMemory ? MM_ENOMEM : MM_EHIP, "%s: %s", what, hipGetErrorString(e));
  };
  guard(hipMalloc((void**)&c->pe, pe.size() * 4), "hipMalloc(pe)");
  guard(hipMalloc((void**)&c->meta, meta_ints * 4), "hipMalloc(meta)");
  guard(hipMalloc((void**)&c->sort_keys, 2 * 16384 * 4), "hipMalloc(sort keys)");
  guard(hipStreamCreateWithFlags(&c->aux, hipStreamNonBlocking), "hipStreamCreate");
  guard(hipEventCreateWithFlags(&c->ev_packed, hipEventDisableTiming), "hipEventCreate");
  guard(hipEventCreateWithFlags(&c->ev_sorted, hipEventDisableTiming), "hipEventCreate");
  guard(hipMalloc((void**)&c->loss_dev, 64), "hipMalloc(loss)");
  guard(hipHostMalloc((void**)&c->result_host, 64, hipHostMallocDefault), "hipHostMalloc(result)");
  guard(hipEventCreateWithFlags(&c->ev_stage, hipEventDisableTiming), "hipEventCreate");
  guard(hipEventCreateWithFlags(&c->ev_done, hipEventDisableTiming), "hipEventCreate");
  guard(hipEventCreateWithFlags(&c->ev_seg, hipEventDisableTiming), "hipEventCreate");
  guard(hipEventCreateWithFlags(&c->ev_gtab, hipEventDisableTiming), "hipEventCreate");
  const size_t tab_bytes = MAX_GROUPED * (sizeof(GemmParams) + sizeof(int32_t)) + MAX_GROUPED_C * sizeof(LnReduceJob) + 64;
  guard(hipHostMalloc((void**)&c->tab_host, tab_bytes, hipHostMallocDefault), "hipHostMalloc(table)");
  guard(hipMalloc((void**)&c->tab_dev, tab_bytes), "hipMalloc(table)");
  guard(hipHostMalloc((void**)&c->seg_static_host, NOALLOC_MAX_MODULES * sizeof(AdamSegment), hipHostMallocDefault), "hipHostMalloc(static table)");
  guard(hipEventCreateWithFlags(&c->ev_seg_static, hipEventDisableTiming), "hipEventCreate");
  if (s != MM_OK) return s;
  {
    void* addr = nullptr;
    s = scratch_address(c, &addr);
    if (s != MM_OK) return s;
    c->seg_static_dev = static_cast<AdamSegment*>(addr);
  }
  guard(hipMemcpy(c->pe, pe.data(), pe.size() * 4, hipMemcpyHostToDevice), "hipMemcpy(pe)");
  c->flag = reinterpret_cast<int32_t*>(c->loss_dev + 1);   // loss and id-check flag leave in one copy
  guard(hipMemset(c->loss_dev, 0, 64), "hipMemset");
  if (s != MM_OK) return s;
  int32_t* p = c->meta;
  c->cu_s = p; p += T + 1; c->cu_u = p; p += T + 1; c->lens = p; p += 2 * T;
  c->src_tok = p; p += T; c->src_pos = p; p += T; c->dec_tok = p; p += T; c->dec_pos = p; p += T; c->label = p;
  return MM_OK;
}

mm_status mm_destroy(mm_ctx* c) {
  if (!c) return MM_EINVAL;
  if (!c->plan_only) {
    hipStreamSynchronize(c->st);
    for (auto& m : c->mods) { hipFree(m.theta); hipFree(m.m); hipFree(m.v); hipFree(m.g); if (m.w16) hipFree(m.w16); }
    hipFree(c->pe); hipFree(c->meta); hipFree(c->sort_keys); hipFree(c->loss_dev);
    if (c->ids_dev) hipFree(c->ids_dev);
    if (c->stage) hipHostFree(c->stage);
    if (c->result_host) hipHostFree(c->result_host);
    if (c->seg_host) hipHostFree(c->seg_host);
    if (c->seg_dev) hipFree(c->seg_dev);
    if (c->seg_static_host) hipHostFree(c->seg_static_host);
    if (c->ev_seg_static) hipEventDestroy(c->ev_seg_static);
    if (c->ws.base) hipFree(c->ws.base);
    for (auto& r : c->prof_recs) { hipEventDestroy(r.e); if (r.s) hipEventDestroy(r.s); }
    for (auto e : c->ev_pool) hipEventDestroy(e);
    if (c->ev_stage) hipEventDestroy(c->ev_stage);
    if (c->ev_done) hipEventDestroy(c->ev_done);
    if (c->ev_seg) hipEventDestroy(c->ev_seg);
    if (c->ev_gtab) hipEventDestroy(c->ev_gtab);
    if (c->aux) { hipStreamSynchronize(c->aux); hipStreamDestroy(c->aux); }
    if (c->ev_packed) hipEventDestroy(c->ev_packed);
    if (c->ev_sorted) hipEventDestroy(c->ev_sorted);
    if (c->tab_host) hipHostFree(c->tab_host);
    if (c->tab_dev) hipFree(c->tab_dev);
  }
  delete c;
  return MM_OK;
}

mm_status mm_register_module(mm_ctx* c, const mm_module_desc* desc, const float* init, int64_t n_params, int32_t* out_id) {
  if (!c || !desc || !out_id) return MM_EINVAL;
  if (desc->kind < MM_SRC_EMB || desc->kind > MM_ADAPTER) return fail(c, MM_EINVAL, "unknown module kind %d", desc->kind);
  Module m;
  m.kind = desc->kind; m.position = desc->position; m.n_layers = desc->n_layers;
  m.owns_final_norm = desc->owns_final_norm; m.adapter_dim = desc->adapter_dim; m.adapter_stack = desc->adapter_stack;
  m.name = desc->name ? desc->name : "";
  const bool stack = m.kind == MM_ENC_STACK || m.kind == MM_DEC_STACK;
  if ((stack || m.kind == MM_ADAPTER) && m.n_layers < 1) return fail(c, MM_EINVAL, "n_layers must be >= 1");
  if (stack && m.position < 0) return fail(c, MM_EINVAL, "negative position");
  if (m.kind == MM_ADAPTER && (m.adapter_dim < 16 || m.adapter_dim % 16 != 0 || (m.adapter_stack != 0 && m.adapter_stack != 1)))
    return fail(c, MM_EINVAL, "adapter needs adapter_dim (multiple of 16) and adapter_stack 0/1");
  if (c->plan_only && m.kind == MM_ADAPTER && m.adapter_dim % 8 == 0) { /* fine */ }
  build_layout(c->cfg, m);
  if (init && n_params != m.P)
    return fail(c, MM_EINVAL, "n_params %lld does not match the bucket length %lld", (long long)n_params, (long long)m.P);
  if (!c->plan_only) {
    const size_t bytes = (size_t)m.P * 4;
    mm_status s = MM_OK;
    auto guard = [&](hipError_t e, const char* what) {
      if (e != hipSuccess && s == MM_OK) s = fail(c, e == hipErrorOutOfMemory ? MM_ENOMEM : MM_EHIP, "%s: %s", what, hipGetErrorString(e));
    };
    guard(hipMalloc((void**)&m.theta, bytes), "hipMalloc(theta)");
    guard(hipMalloc((void**)&m.m, bytes), "hipMalloc(m)");
    guard(hipMalloc((void**)&m.v, bytes), "hipMalloc(v)");
    guard(hipMalloc((void**)&m.g, bytes), "hipMalloc(bucket)");
    if (c->dt == BF16) guard(hipMalloc((void**)&m.w16, (size_t)m.P * 2), "hipMalloc(working copy)");
    if (s == MM_OK) {
      guard(hipStreamSynchronize(c->st), "hipStreamSynchronize");
      if (init) guard(hipMemcpy(m.theta, init, bytes, hipMemcpyHostToDevice), "hipMemcpy(theta)");
      else guard(hipMemset(m.theta, 0, bytes), "hipMemset(theta)");
      guard(hipMemset(m.m, 0, bytes), "hipMemset"); guard(hipMemset(m.v, 0, bytes), "hipMemset");
      guard(hipMemset(m.g, 0, bytes), "hipMemset");
      guard(hipDeviceSynchronize(), "hipDeviceSynchronize");
      if (s == MM_OK && c->dt == BF16) {
        launch_to_bf16(c->st, m.theta, m.w16, m.P);
        guard(hipStreamSynchronize(c->st), "to_bf16");
      }
    }
    if (s != MM_OK) {
      hipFree(m.theta); hipFree(m.m); hipFree(m.v); hipFree(m.g); if (m.w16) hipFree(m.w16);
      return s;
    }
  }
  c->mods.push_back(std::move(m));
  *out_id = (int32_t)c->mods.size() - 1;
  return MM_OK;
}

mm_status mm_route_task(mm_ctx* c, const int32_t* ids, int32_t n, int32_t* out_task) {
  if (!c || !ids || !out_task || n < 5) return c ? fail(c, MM_EINVAL, "route needs at least five modules") : MM_EINVAL;
  Route r;
  mm_status s = parse_route(c, ids, n, r);
  if (s != MM_OK) return s;
  if (!c->routes.empty() && (int)c->routes[0].ids.size() != n)
    return fail(c, MM_EINVAL, "all tasks must involve the same number of modules (%zu), got %d", c->routes[0].ids.size(), n);
  c->routes.push_back(std::move(r));
  *out_task = (int32_t)c->routes.size() - 1;
  return MM_OK;
}

mm_status mm_train_step(mm_ctx* c, int32_t task, const int32_t* src_ids, const int32_t* tgt_ids, const int32_t* lengths,
                        int32_t B, int32_t S_max, int32_t T_max, int32_t ids_mem, float* out_loss) {
  if (!c) return MM_EINVAL;
  if (!src_ids || !tgt_ids || !lengths) return fail(c, MM_EINVAL, "null batch pointer");
  if (task < 0 || task >= (int)c->routes.size()) return fail(c, MM_EINVAL, "unknown task %d", task);
  if (ids_mem != MM_HOST && ids_mem != MM_DEVICE) return fail(c, MM_EINVAL, "ids_mem must be MM_HOST or MM_DEVICE");
  if (B < 1 || S_max < 1 || T_max < 2) return fail(c, MM_EINVAL, "empty batch");
  if (S_max > c->cfg.max_len || T_max - 1 > c->cfg.max_len)
    return fail(c, MM_ERANGE, "padded width exceeds max_len %d", c->cfg.max_len);
  int64_t S = 0, U = 0;
  for (int b = 0; b < B; ++b) {
    const int s = lengths[2 * b], t = lengths[2 * b + 1];
    if (s < 1 || s > S_max || t < 2 || t > T_max)
      return fail(c, MM_ERANGE, "sentence %d has lengths (%d, %d) outside [1,%d] x [2,%d]", b, s, t, S_max, T_max);
    S += s; U += t - 1;
  }
  if (S > c->cfg.max_batch_tokens || U > c->cfg.max_batch_tokens)
    return fail(c, MM_ERANGE, "batch holds %lld source / %lld target tokens, limit %d", (long long)S, (long long)U, c->cfg.max_batch_tokens);
  if (ids_mem == MM_HOST) {
    const int V = c->cfg.vocab;
    for (int b = 0; b < B; ++b) {
      const int s = lengths[2 * b], t = lengths[2 * b + 1];
      for (int i = 0; i < S_max; ++i) {
        const int id = src_ids[(size_t)b * S_max + i];
        if (i < s ? (id < 0 || id >= V) : id != 0)
          return fail(c, MM_ERANGE, "source id %d at sentence %d position %d", id, b, i);
      }
      for (int i = 0; i < T_max; ++i) {
        const int id = tgt_ids[(size_t)b * T_max + i];
        if (i < t ? (id < 0 || id >= V) : id != 0)
          return fail(c, MM_ERANGE, "target id %d at sentence %d position %d", id, b, i);
      }
    }
  }
  if (c->plan_only) return fail(c, MM_ESTATE, "plan-only context cannot compute");
  resolve_pending(c);  // settle the previous step's bookkeeping (no-op when it was read already)

  // stage lengths and prefix sums (and host ids) through pinned memory
  const size_t n_meta = (size_t)2 * B + 2 * ((size_t)B + 1);
  const size_t n_ids = ids_mem == MM_HOST ? (size_t)B * S_max + (size_t)B * T_max : 0;
  HIP_TRY(c, hipEventSynchronize(c->ev_stage));
  mm_status s = ensure_stage(c, n_meta + n_ids);
  if (s != MM_OK) return s;
  int32_t* st_lens = c->stage;
  int32_t* st_cu_s = st_lens + 2 * B;
  int32_t* st_cu_u = st_cu_s + B + 1;
  int32_t* st_ids = st_cu_u + B + 1;
  memcpy(st_lens, lengths, (size_t)2 * B * 4);
  st_cu_s[0] = 0; st_cu_u[0] = 0;
  for (int b = 0; b < B; ++b) {
    st_cu_s[b + 1] = st_cu_s[b] + lengths[2 * b];
    st_cu_u[b + 1] = st_cu_u[b] + lengths[2 * b + 1] - 1;
  }
  const int32_t* src_dev = src_ids;
  const int32_t* tgt_dev = tgt_ids;
  if (ids_mem == MM_HOST) {
    s = ensure_ids_dev(c, n_ids);
    if (s != MM_OK) return s;
    memcpy(st_ids, src_ids, (size_t)B * S_max * 4);
    memcpy(st_ids + (size_t)B * S_max, tgt_ids, (size_t)B * T_max * 4);
    HIP_TRY(c, hipMemcpyAsync(c->ids_dev, st_ids, n_ids * 4, hipMemcpyHostToDevice, c->st));
    src_dev = c->ids_dev;
    tgt_dev = c->ids_dev + (size_t)B * S_max;
  }
  c->B = B; c->S_max = S_max; c->T_max = T_max; c->S = (int)S; c->U = (int)U;
  c->h_cu_s.assign(st_cu_s, st_cu_s + B + 1);
  c->h_cu_u.assign(st_cu_u, st_cu_u + B + 1);
  const Route& rt = c->routes[task];
  run_step(c, rt, true, lengths);
  s = ensure_ws(c, c->ws.high);
  if (s != MM_OK) return s;

  // lengths and both prefix sums lie back to back in the staging block and travel in one copy
  c->lens = c->meta; c->cu_s = c->meta + 2 * B; c->cu_u = c->cu_s + B + 1;
  launch_upload_words(c->st, st_lens, c->meta, n_meta * 4, c->flag);   // (also clears the id-check flag)
  HIP_TRY(c, hipEventRecord(c->ev_stage, c->st));
  launch_pack_ids(c->st, src_dev, tgt_dev, c->lens, c->cu_s, c->cu_u, B, S_max, T_max, c->cfg.vocab, c->src_tok,
                  c->src_pos, c->dec_tok, c->dec_pos, c->label, c->flag);
  // the two token sorts need only the packed ids: they run on the side stream during the forward pass
  HIP_TRY(c, hipEventRecord(c->ev_packed, c->st));
  HIP_TRY(c, hipStreamWaitEvent(c->aux, c->ev_packed, 0));
  launch_sort_tokens(c->aux, c->src_tok, (int)S, c->sort_keys);
  launch_sort_tokens(c->aux, c->dec_tok, (int)U, c->sort_keys + 16384);
  HIP_TRY(c, hipEventRecord(c->ev_sorted, c->aux));
  run_step(c, rt, false, lengths);
  HIP_TRY(c, hipGetLastError());
  HIP_TRY(c, hipEventRecord(c->ev_done, c->st));
  for (int j : rt.ids) c->mods[j].touched += 1;
  c->pending = true; c->pending_task = task;
  if (c->prof && c->prof_recs.size() > 8192) collect_profile(c);
  if (out_loss) {
    s = resolve_pending(c);
    *out_loss = c->last_loss;
    return s;
  }
  return MM_OK;
}

}  // extern "C"

namespace {
// Which of the listed modules (null: all) take an update: those with n_j > 0, each once, in the
// order given.  use holds up to cap ids; more than that is an error (the caller's table is full).
mm_status select_updates(mm_ctx* c, const int32_t* module_ids, int n, int* use, int cap, int* n_use) {
  *n_use = 0;
  if (module_ids && n < 0) return fail(c, MM_EINVAL, "negative count");
  const int count = module_ids ? n : (int)c->mods.size();
  for (int i = 0; i < count; ++i) {
    const int j = module_ids ? module_ids[i] : i;
    if (!valid_module(c, j)) return fail(c, MM_EINVAL, "unknown module id %d", j);
    if (c->mods[j].touched <= 0) continue;
    bool dup = false;
    for (int k = 0; k < *n_use; ++k) dup |= (use[k] == j);
    if (dup) continue;
    if (*n_use >= cap)
      return fail(c, MM_ERANGE, "more than %d modules to update in one call", cap);
    use[(*n_use)++] = j;
  }
  return MM_OK;
}

// Renormalise-and-Adam over the selected modules (Algorithm 1's division by n_j, then the
// optimiser): fills the segment table in host_tab (pinned), uploads it to dev_tab and launches
// one kernel over all segments.  ev guards host_tab against being refilled before its previous
// upload has left it.  A step whose ids turned out bad on the device had no effect (its gradients
// are exact zeros) and counts for nothing.  If the step in flight has been settled (running ==
// false) its use counts were taken back already and modules left without a use were not selected.
// If it is still running, every segment also carries the count without that step and the kernel
// picks one of the two from the step's flag word; resolve_pending() later repairs the host's
// bookkeeping the same way.
mm_status update_launch(mm_ctx* c, const int* use, int n_use, float lr, AdamSegment* host_tab, AdamSegment* dev_tab,
                        hipEvent_t ev, bool timed, bool running) {
  HIP_TRY(c, hipEventSynchronize(ev));
  int chunks = 0;
  double work = 0;
  for (int i = 0; i < n_use; ++i) {
    Module& m = c->mods[use[i]];
    m.t += 1;
    AdamSegment& sg = host_tab[i];
    sg.theta = m.theta; sg.m = m.m; sg.v = m.v; sg.g = m.g; sg.w16 = m.w16; sg.len = m.P;
    sg.n_uses = (float)m.touched;
    int without = m.touched;
    if (running)
      for (int j : c->routes[c->pending_task].ids) without -= (j == use[i]);
    sg.n_uses_alt = (float)(without > 0 ? without : 0);
    m.t_on_trust = running && without <= 0;
    sg.bc1 = (float)(1.0 - std::pow((double)c->cfg.adam_beta1, (double)m.t));
    sg.bc2 = (float)(1.0 - std::pow((double)c->cfg.adam_beta2, (double)m.t));
    sg.first_chunk = chunks; sg.keep_g = bucket_overwrites(m.kind);
    chunks += (int)((m.P + ADAM_CHUNK - 1) / ADAM_CHUNK);
    work += work_bytes_adam(c, m.P, !bucket_overwrites(m.kind));
    m.touched = 0;
  }
  launch_upload_words(c->st, host_tab, dev_tab, (size_t)n_use * sizeof(AdamSegment), nullptr);
  HIP_TRY(c, hipEventRecord(ev, c->st));
  LaunchEvents le;
  if (timed) {   // (timing takes events from a pool that may grow: not for the allocation-free entry point)
    Run run{c, false};
    run.mark();
    le = run.begin_timed(MM_K_ADAM, work);
  }
  launch_adam(c->st, dev_tab, n_use, chunks, lr, c->cfg.adam_beta1, c->cfg.adam_beta2, c->cfg.adam_eps,
              running ? c->flag : nullptr, le);
  HIP_TRY(c, hipGetLastError());
  return MM_OK;
}
}  // namespace

namespace {
// Both searches: beam == 0 greedy, beam >= 1 beam search (out_scores may be NULL).
mm_status translate_impl(mm_ctx* c, int32_t task, const int32_t* src_ids, const int32_t* src_lengths, int32_t B,
                         int32_t S_max, int32_t max_new, int32_t ids_mem, int beam, int32_t* out_ids,
                         int32_t* out_lengths, float* out_scores) {
  if (!c) return MM_EINVAL;
  if (!src_ids || !src_lengths || !out_ids || !out_lengths) return fail(c, MM_EINVAL, "null pointer");
  if (beam < 0 || beam > 8) return fail(c, MM_EINVAL, "beam width %d outside [1, 8]", beam);
  if (task < 0 || task >= (int)c->routes.size()) return fail(c, MM_EINVAL, "unknown task %d", task);
  if (ids_mem != MM_HOST && ids_mem != MM_DEVICE) return fail(c, MM_EINVAL, "ids_mem must be MM_HOST or MM_DEVICE");
  if (B < 1 || S_max < 1 || max_new < 1) return fail(c, MM_EINVAL, "empty batch");
  if (S_max > c->cfg.max_len || max_new > c->cfg.max_len)
    return fail(c, MM_ERANGE, "padded width or output limit exceeds max_len %d", c->cfg.max_len);
  int64_t S = 0;
  for (int b = 0; b < B; ++b) {
    const int sl = src_lengths[b];
    if (sl < 1 || sl > S_max) return fail(c, MM_ERANGE, "sentence %d has length %d outside [1,%d]", b, sl, S_max);
    S += sl;
  }
  if (S > c->cfg.max_batch_tokens || (int64_t)B * (beam > 0 ? beam : 1) > c->cfg.max_batch_tokens)
    return fail(c, MM_ERANGE, "batch holds %lld source tokens and %lld decoder rows, limit %d", (long long)S,
                (long long)B * (beam > 0 ? beam : 1), c->cfg.max_batch_tokens);
  if (ids_mem == MM_HOST) {
    const int V = c->cfg.vocab;
    for (int b = 0; b < B; ++b)
      for (int i = 0; i < S_max; ++i) {
        const int id = src_ids[(size_t)b * S_max + i];
        if (i < src_lengths[b] ? (id < 0 || id >= V) : id != 0)
          return fail(c, MM_ERANGE, "source id %d at sentence %d position %d", id, b, i);
      }
  }
  if (c->plan_only) return fail(c, MM_ESTATE, "plan-only context cannot compute");
  resolve_pending(c);   // a training step still in flight owns the workspace and the id tables

  // The packing kernel of the training step is reused with a two-token target (BOS EOS) per
  // sentence: one decoder row each, whose token it sets to BOS.
  const size_t n_meta = (size_t)2 * B + 2 * ((size_t)B + 1);
  const size_t n_src = ids_mem == MM_HOST ? (size_t)B * S_max : 0;
  const size_t n_ids = n_src + (size_t)2 * B;
  HIP_TRY(c, hipEventSynchronize(c->ev_stage));
  mm_status s = ensure_stage(c, n_meta + n_ids);
  if (s != MM_OK) return s;
  s = ensure_ids_dev(c, n_ids);
  if (s != MM_OK) return s;
  int32_t* st_lens = c->stage;
  int32_t* st_cu_s = st_lens + 2 * B;
  int32_t* st_cu_u = st_cu_s + B + 1;
  int32_t* st_ids = st_cu_u + B + 1;
  st_cu_s[0] = 0; st_cu_u[0] = 0;
  for (int b = 0; b < B; ++b) {
    st_lens[2 * b] = src_lengths[b]; st_lens[2 * b + 1] = 2;
    st_cu_s[b + 1] = st_cu_s[b] + src_lengths[b];
    st_cu_u[b + 1] = b + 1;
    st_ids[n_src + 2 * b] = 1; st_ids[n_src + 2 * b + 1] = 2;
  }
  if (ids_mem == MM_HOST) memcpy(st_ids, src_ids, n_src * 4);
  HIP_TRY(c, hipMemcpyAsync(c->ids_dev, st_ids, n_ids * 4, hipMemcpyHostToDevice, c->st));
  const int32_t* src_dev = ids_mem == MM_HOST ? c->ids_dev : src_ids;
  const int32_t* tgt_dev = c->ids_dev + n_src;
  c->B = B; c->S_max = S_max; c->T_max = 2; c->S = (int)S; c->U = B;
  const Route& rt = c->routes[task];
  TranslateOut out{nullptr, nullptr, nullptr, nullptr, nullptr, 0};
  c->attn_log.clear(); c->h_cu_s.clear(); c->h_cu_u.clear();   // the workspace of the last training step is reused
  run_translate(c, rt, true, src_lengths, max_new, out, beam);
  s = ensure_ws(c, c->ws.high);
  if (s != MM_OK) return s;
  // lengths and both prefix sums lie back to back in the staging block and travel in one copy
  c->lens = c->meta; c->cu_s = c->meta + 2 * B; c->cu_u = c->cu_s + B + 1;
  HIP_TRY(c, hipMemcpyAsync(c->meta, st_lens, n_meta * 4, hipMemcpyHostToDevice, c->st));
  HIP_TRY(c, hipEventRecord(c->ev_stage, c->st));
  launch_fill_i32(c->st, c->flag, 1, 0);
  launch_pack_ids(c->st, src_dev, tgt_dev, c->lens, c->cu_s, c->cu_u, B, S_max, 2, c->cfg.vocab, c->src_tok,
                  c->src_pos, c->dec_tok, c->dec_pos, c->label, c->flag);
  s = run_translate(c, rt, false, src_lengths, max_new, out, beam);
  if (s != MM_OK) return s;
  HIP_TRY(c, hipGetLastError());
  int32_t* flag_host = (int32_t*)c->result_host + 9;
  HIP_TRY(c, hipMemcpyAsync(flag_host, c->flag, 4, hipMemcpyDeviceToHost, c->st));
  if (beam == 0) {
    HIP_TRY(c, hipMemcpyAsync(out_ids, out.ids, (size_t)B * max_new * 4, hipMemcpyDeviceToHost, c->st));
    HIP_TRY(c, hipMemcpyAsync(out_lengths, out.len, (size_t)B * 4, hipMemcpyDeviceToHost, c->st));
    HIP_TRY(c, hipStreamSynchronize(c->st));
  } else {
    // Walk the best hypothesis of every sentence (row b * beam of the last beam) back through the
    // steps: each step stored, per row, its token and the row of the step before that it continues.
    const size_t R = (size_t)B * beam, n_hist = R * (size_t)out.steps;
    std::vector<int32_t> tok(n_hist), par(n_hist);
    std::vector<float> sc(R);
    HIP_TRY(c, hipMemcpyAsync(tok.data(), out.hist_tok, n_hist * 4, hipMemcpyDeviceToHost, c->st));
    HIP_TRY(c, hipMemcpyAsync(par.data(), out.hist_parent, n_hist * 4, hipMemcpyDeviceToHost, c->st));
    HIP_TRY(c, hipMemcpyAsync(sc.data(), out.score, R * 4, hipMemcpyDeviceToHost, c->st));
    HIP_TRY(c, hipStreamSynchronize(c->st));
    std::vector<int32_t> seq(out.steps);
    for (int b = 0; b < B; ++b) {
      int r = b * beam;
      for (int t = out.steps - 1; t >= 0; --t) {
        if (r < b * beam || r >= (b + 1) * beam) return fail(c, MM_EHIP, "beam history leaves its sentence");
        seq[t] = tok[(size_t)t * R + r];
        r = par[(size_t)t * R + r];
      }
      int n = 0;
      while (n < out.steps) { ++n; if (seq[n - 1] == 2 /* EOS */) break; }   // carried steps follow the EOS
      for (int t = 0; t < max_new; ++t) out_ids[(size_t)b * max_new + t] = t < n ? seq[t] : 0;
      out_lengths[b] = n;
      if (out_scores) out_scores[b] = sc[(size_t)b * beam];
    }
  }
  if (c->prof && c->prof_recs.size() > 8192) collect_profile(c);
  if (*flag_host != 0)
    return fail(c, MM_ERANGE, *flag_host & 1 ? "token id outside [0, vocab) (found on the device); output is meaningless"
                                             : "non-pad id after the end of a sentence (found on the device); output is meaningless");
  return MM_OK;
}
}  // namespace

extern "C" {

mm_status mm_translate_greedy(mm_ctx* c, int32_t task, const int32_t* src_ids, const int32_t* src_lengths, int32_t B,
                              int32_t S_max, int32_t max_new, int32_t ids_mem, int32_t* out_ids, int32_t* out_lengths) {
  return translate_impl(c, task, src_ids, src_lengths, B, S_max, max_new, ids_mem, 0, out_ids, out_lengths, nullptr);
}

mm_status mm_translate_beam(mm_ctx* c, int32_t task, const int32_t* src_ids, const int32_t* src_lengths, int32_t B,
                            int32_t S_max, int32_t max_new, int32_t beam, int32_t ids_mem, int32_t* out_ids,
                            int32_t* out_lengths, float* out_scores) {
  if (c && beam < 1) return fail(c, MM_EINVAL, "beam width %d outside [1, 8]", beam);
  return translate_impl(c, task, src_ids, src_lengths, B, S_max, max_new, ids_mem, beam, out_ids, out_lengths, out_scores);
}

mm_status mm_last_loss(mm_ctx* c, float* out_loss) {
  if (!c) return MM_EINVAL;
  if (c->plan_only) return fail(c, MM_ESTATE, "plan-only context cannot compute");
  mm_status s = resolve_pending(c);
  if (out_loss) *out_loss = c->last_loss;
  return s;
}

mm_status mm_apply_update(mm_ctx* c, const int32_t* module_ids, int32_t n, float lr) {
  if (!c) return MM_EINVAL;
  if (c->plan_only) return fail(c, MM_ESTATE, "plan-only context cannot compute");
  const bool running = step_still_running(c);   // see update_launch
  std::vector<int> use(c->mods.size() + 1);
  int n_use = 0;
  mm_status s = select_updates(c, module_ids, n, use.data(), (int)c->mods.size(), &n_use);
  if (s != MM_OK || n_use == 0) return s;
  if (n_use > c->seg_cap) {
    HIP_TRY(c, hipStreamSynchronize(c->st));
    if (c->seg_host) hipHostFree(c->seg_host);
    if (c->seg_dev) hipFree(c->seg_dev);
    c->seg_host = nullptr; c->seg_dev = nullptr; c->seg_cap = 0;
    const int cap = n_use + 32;
    HIP_TRY(c, hipHostMalloc((void**)&c->seg_host, cap * sizeof(AdamSegment), hipHostMallocDefault));
    HIP_TRY(c, hipMalloc((void**)&c->seg_dev, cap * sizeof(AdamSegment)));
    c->seg_cap = cap;
  }
  return update_launch(c, use.data(), n_use, lr, c->seg_host, c->seg_dev, c->ev_seg, true, running);
}

mm_status mm_apply_update_noalloc(mm_ctx* c, const int32_t* module_ids, int32_t n, float lr) {
  if (!c) return MM_EINVAL;
  if (c->plan_only) return fail(c, MM_ESTATE, "plan-only context cannot compute");
  if (!c->seg_static_dev || !c->seg_static_host) return fail(c, MM_ESTATE, "the static segment table was not set up at creation");
  // With a step still running the selection may hold modules that a settled bad step would have
  // dropped; if the table cannot take them all, wait for the step and select again.
  bool running = step_still_running(c);
  if (running && (int64_t)c->mods.size() > NOALLOC_MAX_MODULES) { resolve_pending(c); running = false; }
  int use[NOALLOC_MAX_MODULES + 1];
  int n_use = 0;
  mm_status s = select_updates(c, module_ids, n, use, NOALLOC_MAX_MODULES, &n_use);
  if (s != MM_OK || n_use == 0) return s;
  return update_launch(c, use, n_use, lr, c->seg_static_host, c->seg_static_dev, c->ev_seg_static, false, running);
}

// ---- introspection -----------------------------------------------------------------------------
mm_status mm_num_modules(mm_ctx* c, int32_t* out_n) {
  if (!c || !out_n) return MM_EINVAL;
  *out_n = (int32_t)c->mods.size();
  return MM_OK;
}

mm_status mm_get_route(mm_ctx* c, int32_t task, int32_t* ids, int32_t* n) {
  if (!c || !n) return MM_EINVAL;
  if (task < 0 || task >= (int)c->routes.size()) return fail(c, MM_EINVAL, "unknown task %d", task);
  const auto& r = c->routes[task].ids;
  if (ids) {
    if (*n < (int)r.size()) return fail(c, MM_EINVAL, "capacity %d < %zu", *n, r.size());
    for (size_t i = 0; i < r.size(); ++i) ids[i] = r[i];
  }
  *n = (int32_t)r.size();
  return MM_OK;
}

mm_status mm_get_touched(mm_ctx* c, int32_t* counts, int32_t capacity) {
  if (!c || !counts) return MM_EINVAL;
  if (capacity < (int)c->mods.size()) return fail(c, MM_EINVAL, "capacity %d < %zu", capacity, c->mods.size());
  if (!c->plan_only) resolve_pending(c);
  for (size_t j = 0; j < c->mods.size(); ++j) counts[j] = c->mods[j].touched;
  return MM_OK;
}

mm_status mm_get_layout(mm_ctx* c, int32_t module, int64_t* offsets, int32_t* rows, int32_t* cols, int32_t* roles,
                        int32_t* n_tensors, int64_t* bucket_len) {
  if (!c || !n_tensors) return MM_EINVAL;
  if (!valid_module(c, module)) return fail(c, MM_EINVAL, "unknown module id %d", module);
  const Module& m = c->mods[module];
  const int nt = (int)m.tensors.size();
  if (offsets || rows || cols || roles) {
    if (*n_tensors < nt) return fail(c, MM_EINVAL, "capacity %d < %d tensors", *n_tensors, nt);
    for (int i = 0; i < nt; ++i) {
      if (offsets) offsets[i] = m.tensors[i].off;
      if (rows) rows[i] = m.tensors[i].rows;
      if (cols) cols[i] = m.tensors[i].cols;
      if (roles) roles[i] = m.tensors[i].role;
    }
  }
  *n_tensors = nt;
  if (bucket_len) *bucket_len = m.P;
  return MM_OK;
}

static mm_status copy_out(mm_ctx* c, const float* dev, float* dst, int64_t n) {
  HIP_TRY(c, hipStreamSynchronize(c->st));
  HIP_TRY(c, hipMemcpy(dst, dev, (size_t)n * 4, hipMemcpyDeviceToHost));
  return MM_OK;
}

mm_status mm_get_params(mm_ctx* c, int32_t module, float* dst, int64_t n) {
  mm_status s = check_module(c, module, n);
  if (s != MM_OK) return s;
  if (!dst) return fail(c, MM_EINVAL, "null destination");
  return copy_out(c, c->mods[module].theta, dst, n);
}

mm_status mm_get_grads(mm_ctx* c, int32_t module, float* dst, int64_t n) {
  mm_status s = check_module(c, module, n);
  if (s != MM_OK) return s;
  if (!dst) return fail(c, MM_EINVAL, "null destination");
  resolve_pending(c);
  if (c->mods[module].touched == 0) {   // an unused bucket is empty, whatever its memory still holds
    memset(dst, 0, (size_t)n * sizeof(float));
    return MM_OK;
  }
  return copy_out(c, c->mods[module].g, dst, n);
}

mm_status mm_get_bucket_memory(mm_ctx* c, int32_t module, float* dst, int64_t n) {
  mm_status s = check_module(c, module, n);
  if (s != MM_OK) return s;
  if (!dst) return fail(c, MM_EINVAL, "null destination");
  return copy_out(c, c->mods[module].g, dst, n);
}

mm_status mm_get_adam(mm_ctx* c, int32_t module, float* m, float* v, int64_t n, int64_t* t_j) {
  mm_status s = check_module(c, module, n);
  if (s != MM_OK) return s;
  if (m) { s = copy_out(c, c->mods[module].m, m, n); if (s != MM_OK) return s; }
  if (v) { s = copy_out(c, c->mods[module].v, v, n); if (s != MM_OK) return s; }
  if (t_j) { resolve_pending(c); *t_j = c->mods[module].t; }
  return MM_OK;
}

mm_status mm_get_working(mm_ctx* c, int32_t module, float* dst, int64_t n) {
  mm_status s = check_module(c, module, n);
  if (s != MM_OK) return s;
  if (!dst) return fail(c, MM_EINVAL, "null destination");
  Module& m = c->mods[module];
  if (c->dt != BF16) return copy_out(c, m.theta, dst, n);
  std::vector<bf16_t> tmp((size_t)n);
  HIP_TRY(c, hipStreamSynchronize(c->st));
  HIP_TRY(c, hipMemcpy(tmp.data(), m.w16, (size_t)n * 2, hipMemcpyDeviceToHost));
  for (int64_t i = 0; i < n; ++i) dst[i] = bf16_to_f32(tmp[(size_t)i]);
  return MM_OK;
}

mm_status mm_set_params(mm_ctx* c, int32_t module, const float* src, int64_t n) {
  mm_status s = check_module(c, module, n);
  if (s != MM_OK) return s;
  if (!src) return fail(c, MM_EINVAL, "null source");
  Module& m = c->mods[module];
  HIP_TRY(c, hipStreamSynchronize(c->st));
  HIP_TRY(c, hipMemcpy(m.theta, src, (size_t)n * 4, hipMemcpyHostToDevice));
  if (c->dt == BF16) {
    launch_to_bf16(c->st, m.theta, m.w16, m.P);
    HIP_TRY(c, hipStreamSynchronize(c->st));
  }
  return MM_OK;
}

mm_status mm_set_grads(mm_ctx* c, int32_t module, const float* src, int64_t n, int32_t n_uses) {
  mm_status s = check_module(c, module, n);
  if (s != MM_OK) return s;
  if (!src || n_uses < 0) return fail(c, MM_EINVAL, "null source or negative use count");
  resolve_pending(c);
  HIP_TRY(c, hipStreamSynchronize(c->st));
  HIP_TRY(c, hipMemcpy(c->mods[module].g, src, (size_t)n * 4, hipMemcpyHostToDevice));
  c->mods[module].touched = n_uses;
  return MM_OK;
}

mm_status mm_debug_dump(mm_ctx* c, int32_t what, void* dst, int64_t* nbytes) {
  if (!c || !nbytes) return MM_EINVAL;
  if (c->plan_only) return fail(c, MM_ESTATE, "plan-only context holds no device memory");
  if (c->B == 0) return fail(c, MM_ESTATE, "no step has run yet");
  const int B = c->B, Lu = c->T_max - 1, Ls = c->S_max;
  const void* src = nullptr;
  int64_t need = 0;
  bool mask = false;
  int mode = 0, Lq = 0, Lk = 0;
  const int32_t *cu_q = nullptr, *cu_k = nullptr;
  switch (what) {
    case MM_DUMP_CU_SRC: src = c->cu_s; need = ((int64_t)B + 1) * 4; break;
    case MM_DUMP_CU_DEC: src = c->cu_u; need = ((int64_t)B + 1) * 4; break;
    case MM_DUMP_SRC_TOK: src = c->src_tok; need = (int64_t)c->S * 4; break;
    case MM_DUMP_SRC_POS: src = c->src_pos; need = (int64_t)c->S * 4; break;
    case MM_DUMP_DEC_TOK: src = c->dec_tok; need = (int64_t)c->U * 4; break;
    case MM_DUMP_DEC_POS: src = c->dec_pos; need = (int64_t)c->U * 4; break;
    case MM_DUMP_LABEL: src = c->label; need = (int64_t)c->U * 4; break;
    case MM_DUMP_MASK_ENC: mask = true; mode = 0; Lq = Ls; Lk = Ls; cu_q = c->cu_s; cu_k = c->cu_s; break;
    case MM_DUMP_MASK_DEC: mask = true; mode = 1; Lq = Lu; Lk = Lu; cu_q = c->cu_u; cu_k = c->cu_u; break;
    case MM_DUMP_MASK_CROSS: mask = true; mode = 0; Lq = Lu; Lk = Ls; cu_q = c->cu_u; cu_k = c->cu_s; break;
    default: return fail(c, MM_EINVAL, "unknown dump selector %d", what);
  }
  if (mask) need = (int64_t)B * Lq * Lk;
  if (!dst) { *nbytes = need; return MM_OK; }
  if (*nbytes < need) return fail(c, MM_EINVAL, "capacity %lld < %lld bytes", (long long)*nbytes, (long long)need);
  HIP_TRY(c, hipStreamSynchronize(c->st));
  if (mask) {
    uint8_t* tmp = nullptr;
    HIP_TRY(c, hipMalloc((void**)&tmp, (size_t)need));
    launch_mask_dump(c->st, cu_q, cu_k, B, Lq, Lk, mode, tmp);
    hipError_t e = hipStreamSynchronize(c->st);
    if (e == hipSuccess) e = hipMemcpy(dst, tmp, (size_t)need, hipMemcpyDeviceToHost);
    hipFree(tmp);
    HIP_TRY(c, e);
  } else {
    HIP_TRY(c, hipMemcpy(dst, src, (size_t)need, hipMemcpyDeviceToHost));
  }
  *nbytes = need;
  return MM_OK;
}

mm_status mm_debug_attention(mm_ctx* c, int32_t kind, int32_t layer, float* probs, int64_t* n_floats) {
  if (!c || !n_floats) return MM_EINVAL;
  if (c->plan_only) return fail(c, MM_ESTATE, "plan-only context holds no device memory");
  if (kind < 0 || kind > 2 || layer < 0) return fail(c, MM_EINVAL, "kind must be 0, 1 or 2 and layer >= 0");
  mm_status st0 = resolve_pending(c);
  (void)st0;
  if (c->attn_log.empty() || c->h_cu_s.empty()) return fail(c, MM_ESTATE, "no training step's attention launches are on record");
  const mm_ctx::AttnLog* hit = nullptr;
  int seen = 0;
  for (const auto& e : c->attn_log)
    if (e.kind == kind && seen++ == layer) { hit = &e; break; }
  if (!hit) return fail(c, MM_EINVAL, "the last step ran no attention block of kind %d with index %d", kind, layer);
  const AttnParams& ap0 = hit->p;
  const int B = c->B, H = ap0.H, dh = ap0.dh, d = H * dh;
  const int Lq = kind == 0 ? c->S_max : c->T_max - 1, Lk = kind == 1 ? c->T_max - 1 : c->S_max;
  const std::vector<int32_t>& cu_q = kind == 0 ? c->h_cu_s : c->h_cu_u;
  const std::vector<int32_t>& cu_k = kind == 1 ? c->h_cu_u : c->h_cu_s;
  const int64_t need = (int64_t)B * H * Lq * Lk;
  if (!probs) { *n_floats = need; return MM_OK; }
  if (*n_floats < need) return fail(c, MM_EINVAL, "capacity %lld < %lld floats", (long long)*n_floats, (long long)need);
  const int rows_q = cu_q[B], rows_k = cu_k[B];
  const size_t esz = c->dt == BF16 ? 2 : 4;
  HIP_TRY(c, hipStreamSynchronize(c->st));
  char* v_tmp = nullptr; char* o_tmp = nullptr; float* lse_tmp = nullptr;
  mm_status s = MM_OK;
  auto guard = [&](hipError_t e, const char* what) {
    if (e != hipSuccess && s == MM_OK) s = fail(c, e == hipErrorOutOfMemory ? MM_ENOMEM : MM_EHIP, "%s: %s", what, hipGetErrorString(e));
  };
  guard(hipMalloc((void**)&v_tmp, (size_t)rows_k * d * esz), "hipMalloc(values)");
  guard(hipMalloc((void**)&o_tmp, (size_t)rows_q * d * esz), "hipMalloc(outputs)");
  guard(hipMalloc((void**)&lse_tmp, (size_t)H * rows_q * sizeof(float)), "hipMalloc(lse)");
  std::vector<unsigned char> v_host((size_t)rows_k * d * esz), o_host((size_t)rows_q * d * esz);
  memset(probs, 0, (size_t)need * sizeof(float));
  const int passes = (ap0.max_lk + dh - 1) / dh;
  for (int pass = 0; pass < passes && s == MM_OK; ++pass) {
    // value row of key j (position within its sentence) = unit vector j - pass * dh in every head
    memset(v_host.data(), 0, v_host.size());
    for (int b = 0; b < B; ++b)
      for (int r = cu_k[b]; r < cu_k[b + 1]; ++r) {
        const int e = (r - cu_k[b]) - pass * dh;
        if (e < 0 || e >= dh) continue;
        for (int h = 0; h < H; ++h) {
          const size_t idx = (size_t)r * d + (size_t)h * dh + e;
          if (c->dt == BF16) reinterpret_cast<bf16_t*>(v_host.data())[idx] = 0x3f80;   // 1.0
          else reinterpret_cast<float*>(v_host.data())[idx] = 1.0f;
        }
      }
    guard(hipMemcpy(v_tmp, v_host.data(), v_host.size(), hipMemcpyHostToDevice), "hipMemcpy(values)");
    if (s != MM_OK) break;
    AttnParams ap = ap0;
    ap.v = v_tmp; ap.ldv = d; ap.o = o_tmp; ap.ldo = d; ap.lse = lse_tmp;
    launch_attn_fwd(c->st, c->dt, ap);
    guard(hipGetLastError(), "attention launch");
    guard(hipStreamSynchronize(c->st), "hipStreamSynchronize");
    guard(hipMemcpy(o_host.data(), o_tmp, o_host.size(), hipMemcpyDeviceToHost), "hipMemcpy(outputs)");
    if (s != MM_OK) break;
    for (int b = 0; b < B; ++b)
      for (int r = cu_q[b]; r < cu_q[b + 1]; ++r)
        for (int h = 0; h < H; ++h)
          for (int e = 0; e < dh; ++e) {
            const int j = pass * dh + e;
            if (j >= Lk) break;
            const size_t idx = (size_t)r * d + (size_t)h * dh + e;
            const float v = c->dt == BF16 ? bf16_to_f32(reinterpret_cast<const bf16_t*>(o_host.data())[idx])
                                          : reinterpret_cast<const float*>(o_host.data())[idx];
            probs[(((int64_t)b * H + h) * Lq + (r - cu_q[b])) * Lk + j] = v;
          }
  }
  hipFree(v_tmp); hipFree(o_tmp); hipFree(lse_tmp);
  if (s != MM_OK) return s;
  *n_floats = need;
  return MM_OK;
}

mm_status mm_profile(mm_ctx* c, int32_t enable) {
  if (!c) return MM_EINVAL;
  if (c->plan_only) return fail(c, MM_ESTATE, "plan-only context cannot compute");
  mm_status s = collect_profile(c);
  if (s != MM_OK) return s;
  if (enable) {
    for (int i = 0; i < MM_K_COUNT; ++i) { c->prof_ms[i] = 0; c->prof_n[i] = 0; c->prof_work[i] = 0; }
  }
  c->prof = enable != 0;
  return MM_OK;
}

mm_status mm_profile_read(mm_ctx* c, double* ms, int64_t* launches, double* work) {
  if (!c) return MM_EINVAL;
  if (c->plan_only) return fail(c, MM_ESTATE, "plan-only context cannot compute");
  mm_status s = collect_profile(c);
  if (s != MM_OK) return s;
  for (int i = 0; i < MM_K_COUNT; ++i) {
    if (ms) ms[i] = c->prof_ms[i];
    if (launches) launches[i] = c->prof_n[i];
    if (work) work[i] = c->prof_work[i];
  }
  return MM_OK;
}

const char* mm_last_error(mm_ctx* c) { return c ? c->err.c_str() : "null context"; }

}  // extern "C"
