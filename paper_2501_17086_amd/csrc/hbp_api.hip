// C ABI of libhbp (see include/hbp.h): validation, workspace carving and the
// launch sequences of the forward pass, Highway-BP, exact BP and the parameter
// gradients.  Everything is enqueued on the caller's stream; nothing here
// allocates or synchronises.
#include "../../include/hbp.h"
#include "hbp_common.h"

#include <cmath>
#include <mutex>
#include <vector>

using namespace hbp;

// Scratch of hbp_initial_estimate_static, the entry point that allocates nothing and takes no workspace: the
// chunked scan's per-chunk partial results (B, the state entering each chunk, the products A, the old state above
// each chunk) live here instead of in a caller's workspace.  One copy per GPU the library's code object is loaded
// on, held until the process ends.  In host code the name below is a stand-in, not a device address: host code
// uses the pointer hipGetSymbolAddress returns for the current device (static_scratch()).
static __device__ __align__(256) unsigned char scratch[HBP_STATIC_SCRATCH_BYTES];

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t esize(const hbp_desc* d) { return d->dtype == HBP_F32 ? 4 : 2; }
inline bool cell(const hbp_desc* d) { return d->kind == HBP_GATED || d->kind == HBP_LSTM || d->kind == HBP_GRU; }
inline bool gru(const hbp_desc* d) { return d->kind == HBP_GRU; }
inline bool recurrent(const hbp_desc* d) { return d->kind == HBP_RNN || cell(d); }
// A cell's weights act on the hidden part of the state: all of it (GATED), or the second half of [c | h] (LSTM).
inline long hidden_w(const hbp_desc* d) { return d->kind == HBP_LSTM ? d->d / 2 : d->d; }
inline long hidden_off(const hbp_desc* d) { return d->kind == HBP_LSTM ? d->d / 2 : 0; }
inline bool shared_w(const hbp_desc* d) { return recurrent(d); }
// The alternating attention / MLP stack: weight sets and inner-state rows are counted per layer (L / 2).
inline bool tfm(const hbp_desc* d) { return d->kind == HBP_TRANSFORMER; }
inline long head_w(const hbp_desc* d) { return d->d / d->heads; }

struct Workspace {
  size_t off_v, off_da, off_part, off_scan, off_wt, off_pre, off_m, off_tmp, off_dqkv, off_dsum, total;
};

// split-K factor for a parameter-gradient GEMM with `tiles` output tiles and a
// contraction of length K: enough workgroups to fill the 256 CUs, at least 2048
// rows of the contraction each.  Few tiles (up to 32): once, which halves the
// partial sums to write and add up.  More: twice, so that each XCD (an eighth of
// the workgroups, sharing one L2) works on whole shares of the contraction, whose
// tiles share operand panels (measured: 64 tiles at 4 shares are 25 % slower than
// at 8).
int pick_split(long tiles, long K) {
  long want = ((tiles <= 32 ? 256 : 512) + tiles - 1) / tiles;
  long cap = K / 2048;
  if (cap < 1) cap = 1;
  if (want > cap) want = cap;
  if (want > 64) want = 64;
  if (want < 1) want = 1;
  // the aligned kernel needs every share of the contraction to be a whole number of 32-row slices:
  // take the largest such factor below the wanted one when there is one
  if (K % 32 == 0)
    for (long s = want; s >= 1; --s)
      if ((K / 32) % s == 0) return (int)s;
  return (int)want;
}

long tiles_of(long M, long N) { return ((M + 255) / 256) * ((N + 255) / 256); }

struct Splits { int s_w2, s_w1, s_u, s_qkv, s_o; };

Splits param_splits(const hbp_desc* d) {
  Splits s{1, 1, 1, 1, 1};
  if (tfm(d)) {
    const long nb = d->L / 2;
    s.s_w2 = s.s_w1 = pick_split(tiles_of(d->d, d->d_ff) * nb, d->N);
    s.s_qkv = pick_split(tiles_of(3 * d->d, d->d) * nb, d->N);
    s.s_o = pick_split(tiles_of(d->d, d->d) * nb, d->N);
    return s;
  }
  const long nb = shared_w(d) ? 1 : d->L;
  const long K = shared_w(d) ? d->L * d->N : d->N;
  s.s_w2 = pick_split(tiles_of(d->d, d->d_ff) * nb, K);
  s.s_w1 = s.s_w2;
  if (recurrent(d)) s.s_u = pick_split(tiles_of(d->d_ff, d->d_in), K);
  return s;
}

Workspace carve(const hbp_desc* d) {
  Workspace w{};
  const size_t es = esize(d);
  size_t o = 0;
  w.off_v = o;  o = align_up(o + (size_t)d->L * d->N * d->d * es, 256);
  // da [L,N,d_ff] in the storage type; the RNN forward also keeps U.xin here as fp32
  size_t da_bytes = (size_t)(tfm(d) ? d->L / 2 : d->L) * d->N * d->d_ff * (recurrent(d) ? 4 : es);
  w.off_da = o; o = align_up(o + da_bytes, 256);
  Splits sp = param_splits(d);
  const size_t nb = shared_w(d) ? 1 : tfm(d) ? (size_t)d->L / 2 : (size_t)d->L;
  size_t part = 0;
  if (sp.s_w2 > 1) part = (size_t)sp.s_w2 * nb * d->d * d->d_ff * 4;
  if (tfm(d)) {
    if (sp.s_qkv > 1 && (size_t)sp.s_qkv * nb * 3 * d->d * d->d * 4 > part) part = (size_t)sp.s_qkv * nb * 3 * d->d * d->d * 4;
    if (sp.s_o > 1 && (size_t)sp.s_o * nb * d->d * d->d * 4 > part) part = (size_t)sp.s_o * nb * d->d * d->d * 4;
  }
  if (sp.s_u > 1) {
    size_t pu = (size_t)sp.s_u * d->d_ff * d->d_in * 4;
    if (pu > part) part = pu;
  }
  w.off_part = o; o = align_up(o + part, 256);
  w.off_scan = o; o = align_up(o + scan_chunk_ws_bytes(d->L, d->N, d->d, d->norm == HBP_NORM_RMS), 256);
  // transposed copies of the shared weights for step-by-step backpropagation through time
  w.off_wt = o;
  if (recurrent(d) && d->dtype == HBP_BF16) o = align_up(o + 2 * (size_t)d->d * d->d_ff * es, 256);
  // one step's pre-activations of the gated cell, fp32 [N, 2H]
  w.off_pre = o;
  if (cell(d)) o = align_up(o + (size_t)d->N * d->d_ff * 4, 256);
  // post-norm: mean(G (.) x) per (layer, token) of the previous and of the current estimate
  w.off_m = o;
  if (d->post == HBP_POST_RMS) o = align_up(o + 2 * (size_t)d->L * d->N * 4, 256);
  // the standard GRU: what comes back through the candidate's product, [L,N,H] in the storage type
  w.off_tmp = o;
  if (gru(d)) o = align_up(o + (size_t)d->L * d->N * d->d * es, 256);
  // the attention sub-blocks: the gradient of the attention's output (in tmp), of [q | k | v], and rowsum(do (.) o)
  if (tfm(d)) o = align_up(o + (size_t)(d->L / 2) * d->N * d->d * es, 256);
  w.off_dqkv = o;
  if (tfm(d)) o = align_up(o + (size_t)(d->L / 2) * d->N * 3 * d->d * es, 256);
  w.off_dsum = o;
  if (tfm(d)) o = align_up(o + (size_t)(d->L / 2) * d->N * d->heads * 4, 256);
  w.total = o;
  return w;
}

// One step of the recurrence at a time, few rows: the few-row kernel with transposed weights.
inline bool step_skinny(const hbp_desc* d) {
  if (gru(d)) return d->dtype == HBP_BF16 && skinny_ok(d->N, d->d, d->d);   // products H x H and H x 2H, 2H x H
  return recurrent(d) && d->dtype == HBP_BF16 && skinny_ok(d->N, d->d_ff, hidden_w(d)) &&
         skinny_ok(d->N, hidden_w(d), d->d_ff);
}

hbp_status check_desc(const hbp_desc* d) {
  if (!d) return HBP_E_NULL;
  if (d->struct_size != sizeof(hbp_desc)) return HBP_E_INVALID_ARG;
  if (d->kind < HBP_MLP || d->kind > HBP_TRANSFORMER) return HBP_E_INVALID_ARG;
  if (d->dtype != HBP_F32 && d->dtype != HBP_BF16) return HBP_E_INVALID_ARG;
  if (d->act < HBP_ACT_GELU_ERF || d->act > HBP_ACT_IDENTITY) return HBP_E_INVALID_ARG;
  if (d->norm != HBP_NORM_NONE && d->norm != HBP_NORM_RMS) return HBP_E_INVALID_ARG;
  if (d->lambda_kind < HBP_LAMBDA_ONE || d->lambda_kind > HBP_LAMBDA_TOKEN) return HBP_E_INVALID_ARG;
  if (d->loss_every_state != 0 && d->loss_every_state != 1) return HBP_E_INVALID_ARG;
  if (d->L <= 0 || d->N <= 0 || d->d <= 0 || d->d_ff <= 0 || d->d_in < 0) return HBP_E_INVALID_ARG;
  if (recurrent(d) && d->d_in <= 0) return HBP_E_INVALID_ARG;
  if (cell(d) && (d->act != HBP_ACT_TANH || d->norm != HBP_NORM_NONE || d->lambda_kind != HBP_LAMBDA_TOKEN ||
                  d->d_ff != (gru(d) ? 3 : 2) * d->d))
    return HBP_E_INVALID_ARG;
  if (d->kind == HBP_LSTM && d->d % 16) return HBP_E_UNSUPPORTED;   // both halves of [c | h] in 16-byte vectors
  if ((d->kind == HBP_MLP || tfm(d)) && d->d_in != 0) return HBP_E_INVALID_ARG;
  if (tfm(d)) {
    if (d->L % 2 || d->heads <= 0 || d->seq_len <= 0 || (d->causal != 0 && d->causal != 1)) return HBP_E_INVALID_ARG;
    if (d->N % d->seq_len || d->d % d->heads) return HBP_E_INVALID_ARG;
    if (d->post == HBP_POST_RELU || head_w(d) % 8) return HBP_E_UNSUPPORTED;
    if (!attn_supported(d->dtype, d->seq_len, (int)head_w(d))) return HBP_E_UNSUPPORTED;
  }
  if (d->norm == HBP_NORM_RMS && !(d->eps >= 0.f)) return HBP_E_INVALID_ARG;
  if (d->d % 8 || d->d_ff % 8 || d->d_in % 8) return HBP_E_UNSUPPORTED;
  if (d->norm == HBP_NORM_RMS && d->d > 4096) return HBP_E_UNSUPPORTED;
  if (!(d->gamma >= 0.f && d->gamma <= 1.f)) return HBP_E_INVALID_ARG;
  if (d->post < HBP_POST_NONE || d->post > HBP_POST_RMS) return HBP_E_INVALID_ARG;
  if (d->post != HBP_POST_NONE && d->kind != HBP_MLP && !(tfm(d) && d->post == HBP_POST_RMS)) return HBP_E_UNSUPPORTED;
  if (d->post == HBP_POST_RELU && d->gamma != 0.f) return HBP_E_UNSUPPORTED;
  if (d->post == HBP_POST_RMS && (d->norm != HBP_NORM_NONE || d->lambda_kind == HBP_LAMBDA_TOKEN || d->d > 4096 ||
                                  (d->gamma != 0.f && d->d > 2048)))
    return HBP_E_UNSUPPORTED;
  if (d->gamma != 0.f && d->norm == HBP_NORM_RMS && d->d > 2048) return HBP_E_UNSUPPORTED;
  if (d->L > (1 << 20) || d->N > (1L << 24) || d->d > (1 << 20) || d->d_ff > (1 << 20)) return HBP_E_UNSUPPORTED;
  return HBP_OK;
}

enum Need { NEED_FWD = 1, NEED_BWD = 2, NEED_PG = 4 };

hbp_status check_bufs(const hbp_desc* d, const hbp_buffers* b, int need) {
  if (!b) return HBP_E_NULL;
  if (b->struct_size != sizeof(hbp_buffers)) return HBP_E_INVALID_ARG;
  if (!b->W1 || (!b->W2 && !cell(d))) return HBP_E_NULL;
  if (recurrent(d) && (need & (NEED_FWD | NEED_PG)) && (!b->U || !b->xin)) return HBP_E_NULL;
  if (d->lambda_kind != HBP_LAMBDA_ONE && !b->lambda) return HBP_E_NULL;
  if (d->norm == HBP_NORM_RMS && (!b->y || !b->rinv)) return HBP_E_NULL;
  if (d->norm == HBP_NORM_NONE && !b->x) return HBP_E_NULL;
  if ((need & NEED_FWD) && !b->x) return HBP_E_NULL;
  if (!b->z) return HBP_E_NULL;
  if (tfm(d) && (!b->Wqkv || !b->Wo || !b->qkv || !b->attn_o || !b->lse)) return HBP_E_NULL;
  if (tfm(d) && (need & NEED_PG) && (!b->dWqkv || !b->dWo)) return HBP_E_NULL;
  if (d->act == HBP_ACT_GELU_ERF && !b->dphi) return HBP_E_NULL;
  if (d->post == HBP_POST_RELU && (need & (NEED_FWD | NEED_BWD)) && !b->mask) return HBP_E_NULL;
  if (d->post == HBP_POST_RMS && (need & (NEED_FWD | NEED_BWD)) && !b->rinv) return HBP_E_NULL;
  if (need & (NEED_BWD | NEED_PG)) {
    if (!b->g) return HBP_E_NULL;
  }
  if ((need & NEED_BWD) && !b->e) return HBP_E_NULL;
  if (need & NEED_PG) {
    if (!b->dW1 || (!b->dW2 && !cell(d))) return HBP_E_NULL;
    if (recurrent(d) && !b->dU) return HBP_E_NULL;
  }
  Workspace w = carve(d);
  if (!b->workspace || b->workspace_bytes < w.total) return HBP_E_WORKSPACE;
  return HBP_OK;
}

#define HBP_TRY(expr)                          \
  do {                                         \
    hipError_t _e = (expr);                    \
    if (_e != hipSuccess) return HBP_E_DEVICE; \
  } while (0)

// ---- optional per-kernel-class timing with HIP events (off by default) ----
struct ProfRec { hipEvent_t a, b; int cls; };
struct ProfState {
  bool on = false;
  std::vector<ProfRec> recs;      // events in flight since the last read
  std::vector<hipEvent_t> pool;   // recycled events
  std::mutex mu;
};
ProfState& prof() { static ProfState p; return p; }

struct ProfScope {
  hipStream_t s; hipEvent_t a = nullptr, b = nullptr; int cls; bool live = false;
  ProfScope(int cls_, hipStream_t s_) : s(s_), cls(cls_) {
    ProfState& p = prof();
    if (!p.on) return;
    std::lock_guard<std::mutex> lk(p.mu);
    for (hipEvent_t* e : {&a, &b}) {
      if (!p.pool.empty()) { *e = p.pool.back(); p.pool.pop_back(); }
      else if (hipEventCreate(e) != hipSuccess) { *e = nullptr; return; }
    }
    live = hipEventRecord(a, s) == hipSuccess;
  }
  ~ProfScope() {
    if (!live) return;
    (void)hipEventRecord(b, s);
    ProfState& p = prof();
    std::lock_guard<std::mutex> lk(p.mu);
    p.recs.push_back({a, b, cls});
  }
};

hbp_status run_gemm(const hbp_desc* d, const GemmArgs& ga, hipStream_t s, int cls) {
  ProfScope ps(cls, s);
  hipError_t err = hipSuccess;
  if (d->dtype == HBP_BF16 && launch_gemm_mfma(ga, s, &err)) {
    return err == hipSuccess ? HBP_OK : HBP_E_DEVICE;
  }
  HBP_TRY(launch_gemm_generic(d->dtype, ga, s));
  return HBP_OK;
}

#define HBP_RUN(expr)                \
  do {                               \
    hbp_status _s = (expr);          \
    if (_s != HBP_OK) return _s;     \
  } while (0)

inline char* at(void* p, size_t bytes) { return reinterpret_cast<char*>(p) + bytes; }
inline const char* at(const void* p, size_t bytes) { return reinterpret_cast<const char*>(p) + bytes; }

// With a loss at every state and no norm between the block and the residual
// path, e_l is added to v_l by the second contraction's epilogue.
inline bool e_in_vjp(const hbp_desc* d) { return d->loss_every_state && d->norm == HBP_NORM_NONE; }

// ---- the alternating attention / MLP stack: step (i) for blocks l_lo..l_hi-1, each kind of sub-block batched over
// its own blocks (attention: even l = 2j; MLP: odd l = 2j+1; state-shaped arrays then have a batch stride of two
// states, inner arrays and weights of one layer) ----
AttnArgs attn_args(const hbp_desc* d, const hbp_buffers* b, const Workspace& w, long j_lo, long j_hi) {
  const size_t es = esize(d);
  const long N = d->N, D = d->d;
  AttnArgs a{};
  a.qkv = at((const void*)b->qkv, (size_t)j_lo * N * 3 * D * es);
  a.o = at(b->attn_o, (size_t)j_lo * N * D * es);
  a.lse = b->lse + j_lo * N * d->heads;
  a.dout = at((const void*)b->workspace, w.off_tmp + (size_t)j_lo * N * D * es);
  a.dqkv = at(b->workspace, w.off_dqkv + (size_t)j_lo * N * 3 * D * es);
  a.dsum = reinterpret_cast<float*>(at(b->workspace, w.off_dsum)) + j_lo * N * d->heads;
  a.seqs = (j_hi - j_lo) * (N / d->seq_len);
  a.T = d->seq_len;
  a.heads = d->heads;
  a.dh = (int)head_w(d);
  a.causal = d->causal;
  a.scale = 1.0f / sqrtf((float)head_w(d));
  return a;
}

// first half: da_j = (g[2j+2] W2_j) (.) act' for the MLP sub-blocks; do_j = g[2j+1] Wo_j and, through the attention,
// the gradient of [q | k | v] for the attention sub-blocks
hbp_status tfm_stage1(const hbp_desc* d, const hbp_buffers* b, const Workspace& w, long l_lo, long l_hi, hipStream_t s) {
  const size_t es = esize(d);
  const long N = d->N, D = d->d, F = d->d_ff;
  const long ja_lo = (l_lo + 1) / 2, ja_hi = (l_hi + 1) / 2;
  const long jm_lo = l_lo / 2, jm_hi = l_hi / 2;
  if (jm_hi > jm_lo) {
    GemmArgs ga{};
    ga.A = at(b->g, (size_t)(2 * jm_lo + 2) * N * D * es);
    ga.B = at(b->W2, (size_t)jm_lo * D * F * es);
    ga.C = at(b->workspace, w.off_da + (size_t)jm_lo * N * F * es);
    ga.M = N; ga.N = F; ga.K = D;
    ga.a_sm = D; ga.a_sk = 1;
    ga.b_sk = F; ga.b_sn = 1;
    ga.ldc = F;
    ga.batch = jm_hi - jm_lo;
    ga.a_sb = 2 * N * D; ga.b_sb = D * F; ga.c_sb = N * F;
    ga.split_k = 1;
    if (d->act == HBP_ACT_GELU_ERF) { ga.mode = EPI_MUL_AUX; ga.aux = at(b->dphi, (size_t)jm_lo * N * F * es); }
    else if (d->act == HBP_ACT_TANH) { ga.mode = EPI_MUL_1MZ2; ga.aux = at(b->z, (size_t)jm_lo * N * F * es); }
    else ga.mode = EPI_STORE;
    ga.aux_sb = N * F;
    HBP_RUN(run_gemm(d, ga, s, HBP_PROF_VJP1));
  }
  if (ja_hi > ja_lo) {
    GemmArgs ga{};
    ga.A = at(b->g, (size_t)(2 * ja_lo + 1) * N * D * es);
    ga.B = at(b->Wo, (size_t)ja_lo * D * D * es);
    ga.C = at(b->workspace, w.off_tmp + (size_t)ja_lo * N * D * es);
    ga.M = N; ga.N = D; ga.K = D;
    ga.a_sm = D; ga.a_sk = 1;
    ga.b_sk = D; ga.b_sn = 1;
    ga.ldc = D;
    ga.batch = ja_hi - ja_lo;
    ga.a_sb = 2 * N * D; ga.b_sb = D * D; ga.c_sb = N * D;
    ga.split_k = 1;
    ga.mode = EPI_STORE;
    HBP_RUN(run_gemm(d, ga, s, HBP_PROF_VJP1));
    ProfScope ps(HBP_PROF_ATTN, s);
    HBP_TRY(launch_attn_bwd(d->dtype, attn_args(d, b, w, ja_lo, ja_hi), s));
  }
  return HBP_OK;
}

// second half: dn = da_j W1_j into v[2j+1], dn = dqkv_j Wqkv_j into v[2j] (+ e where the scan has no norm to apply first)
hbp_status tfm_stage2(const hbp_desc* d, const hbp_buffers* b, const Workspace& w, long l_lo, long l_hi, hipStream_t s) {
  const size_t es = esize(d);
  const long N = d->N, D = d->d, F = d->d_ff;
  const long ja_lo = (l_lo + 1) / 2, ja_hi = (l_hi + 1) / 2;
  const long jm_lo = l_lo / 2, jm_hi = l_hi / 2;
  for (int attn = 0; attn < 2; ++attn) {
    const long j_lo = attn ? ja_lo : jm_lo, j_hi = attn ? ja_hi : jm_hi;
    if (j_hi <= j_lo) continue;
    const long l0 = attn ? 2 * j_lo : 2 * j_lo + 1;        // first block of this kind in the range
    const long kk = attn ? 3 * D : F;
    GemmArgs ga{};
    ga.A = attn ? at(b->workspace, w.off_dqkv + (size_t)j_lo * N * kk * es) : at(b->workspace, w.off_da + (size_t)j_lo * N * kk * es);
    ga.B = attn ? at(b->Wqkv, (size_t)j_lo * kk * D * es) : at(b->W1, (size_t)j_lo * kk * D * es);
    ga.C = at(b->workspace, w.off_v + (size_t)l0 * N * D * es);
    ga.M = N; ga.N = D; ga.K = kk;
    ga.a_sm = kk; ga.a_sk = 1;
    ga.b_sk = D; ga.b_sn = 1;
    ga.ldc = D;
    ga.batch = j_hi - j_lo;
    ga.a_sb = N * kk; ga.b_sb = kk * D; ga.c_sb = 2 * N * D;
    ga.split_k = 1;
    ga.mode = EPI_STORE;
    if (e_in_vjp(d)) {
      ga.mode = EPI_ADD_AUX;
      ga.aux = at(b->e, (size_t)l0 * N * D * es);
      ga.aux_sb = 2 * N * D;
    }
    HBP_RUN(run_gemm(d, ga, s, HBP_PROF_VJP2));
  }
  return HBP_OK;
}

// da[l] = (g[l+1] . W2_l) (.) act'(a_l) for blocks l_lo..l_hi-1
hbp_status vjp_stage1(const hbp_desc* d, const hbp_buffers* b, const Workspace& w, long l_lo, long l_hi,
                      hipStream_t s, bool skinny = false, void* rx_out = nullptr) {
  if (tfm(d)) return tfm_stage1(d, b, w, l_lo, l_hi, s);
  const size_t es = esize(d);
  const long nl = l_hi - l_lo;
  if (gru(d)) {
    // dL/dz and dL/dn elementwise; what comes back through the candidate's product, tmp = dn W_n; then dL/dr and the
    // state's direct share tmp (.) r (+ e), which the second contraction's epilogue adds to its product
    const long H = d->d, rows = nl * d->N;
    const size_t so = (size_t)l_lo * d->N * H * es, fo = (size_t)l_lo * d->N * d->d_ff * es;
    void* da = at(b->workspace, w.off_da + fo);
    void* tmp = at(b->workspace, w.off_tmp + so);
    ProfScope ps(HBP_PROF_VJP1, s);
    HBP_TRY(launch_gru_vjp1(d->dtype, at(b->g, so + (size_t)d->N * H * es), at((const void*)b->x, so),
                            at((const void*)b->z, fo), da, rows, H, s));
    if (skinny) {     // W_n^T [H,H] sits after [W_z; W_r]^T [H,2H] in the transposed-weight region
      SkinnyArgs k{};
      k.A = at((const void*)da, (size_t)2 * H * es); k.lda = d->d_ff;
      k.Bt = at(b->workspace, w.off_wt + (size_t)2 * H * H * es); k.ldbt = H;
      k.C = tmp; k.ldc = H;
      k.M = rows; k.N = H; k.K = H;
      k.mode = EPI_STORE;
      HBP_TRY(launch_gemm_skinny(k, s));
    } else {
      GemmArgs ga{};
      ga.A = at((const void*)da, (size_t)2 * H * es);
      ga.B = at(b->W1, (size_t)2 * H * H * es);
      ga.C = tmp;
      ga.M = rows; ga.N = H; ga.K = H;
      ga.a_sm = d->d_ff; ga.a_sk = 1;
      ga.b_sk = H; ga.b_sn = 1;
      ga.ldc = H; ga.batch = 1; ga.split_k = 1;
      ga.mode = EPI_STORE;
      hipError_t err = hipSuccess;
      if (!(d->dtype == HBP_BF16 && launch_gemm_mfma(ga, s, &err))) err = launch_gemm_generic(d->dtype, ga, s);
      if (err != hipSuccess) return HBP_E_DEVICE;
    }
    HBP_TRY(launch_gru_vjp2(d->dtype, tmp, at((const void*)b->x, so), at((const void*)b->z, fo),
                            e_in_vjp(d) ? at(b->e, so) : nullptr, da, rx_out, rows, H, s));
    return HBP_OK;
  }
  if (d->kind == HBP_GATED) {   // no first contraction: dL/du and dL/dc through sigmoid' and tanh', elementwise
    ProfScope ps(HBP_PROF_VJP1, s);
    HBP_TRY(launch_gated_vjp(d->dtype, at(b->g, (size_t)(l_lo + 1) * d->N * d->d * es),
                             at((const void*)b->x, (size_t)l_lo * d->N * d->d * es),
                             at((const void*)b->z, (size_t)l_lo * d->N * d->d_ff * es),
                             at(b->workspace, w.off_da + (size_t)l_lo * d->N * d->d_ff * es), nl * d->N, d->d, s));
    return HBP_OK;
  }
  if (d->kind == HBP_LSTM) {   // likewise; also writes the cell half of v (and adds e's cell half when the second
    ProfScope ps(HBP_PROF_VJP1, s);   // contraction's epilogue adds the hidden half)
    const size_t so = (size_t)l_lo * d->N * d->d * es;
    HBP_TRY(launch_lstm_vjp(d->dtype, at(b->g, so + (size_t)d->N * d->d * es), at((const void*)b->x, so),
                            at((const void*)b->x, so + (size_t)d->N * d->d * es),
                            at((const void*)b->z, (size_t)l_lo * d->N * d->d_ff * es),
                            e_in_vjp(d) ? at(b->e, so) : nullptr,
                            at(b->workspace, w.off_da + (size_t)l_lo * d->N * d->d_ff * es),
                            at(b->workspace, w.off_v + so), nl * d->N, d->d / 2, s));
    return HBP_OK;
  }
  if (skinny) {   // one step; W2^T [d_ff,d] sits first in the transposed-weight region
    SkinnyArgs k{};
    k.A = at(b->g, (size_t)(l_lo + 1) * d->N * d->d * es); k.lda = d->d;
    k.Bt = at(b->workspace, w.off_wt); k.ldbt = d->d;
    k.C = at(b->workspace, w.off_da + (size_t)l_lo * d->N * d->d_ff * es); k.ldc = d->d_ff;
    k.M = d->N; k.N = d->d_ff; k.K = d->d;
    k.ldaux = d->d_ff;
    if (d->act == HBP_ACT_GELU_ERF) { k.mode = EPI_MUL_AUX; k.aux = at(b->dphi, (size_t)l_lo * d->N * d->d_ff * es); }
    else if (d->act == HBP_ACT_TANH) { k.mode = EPI_MUL_1MZ2; k.aux = at(b->z, (size_t)l_lo * d->N * d->d_ff * es); }
    else k.mode = EPI_STORE;
    ProfScope ps(HBP_PROF_VJP1, s);
    HBP_TRY(launch_gemm_skinny(k, s));
    return HBP_OK;
  }
  GemmArgs ga{};
  const bool sh = shared_w(d);
  ga.A = at(b->g, (size_t)(l_lo + 1) * d->N * d->d * es);
  ga.B = sh ? b->W2 : at(b->W2, (size_t)l_lo * d->d * d->d_ff * es);
  ga.C = at(b->workspace, w.off_da + (size_t)l_lo * d->N * d->d_ff * es);
  ga.M = sh ? nl * d->N : d->N;
  ga.N = d->d_ff;
  ga.K = d->d;
  ga.a_sm = d->d; ga.a_sk = 1;
  ga.b_sk = d->d_ff; ga.b_sn = 1;
  ga.ldc = d->d_ff;
  ga.batch = sh ? 1 : nl;
  ga.a_sb = d->N * d->d; ga.b_sb = d->d * d->d_ff; ga.c_sb = d->N * d->d_ff;
  ga.split_k = 1;
  if (d->act == HBP_ACT_GELU_ERF) {
    ga.mode = EPI_MUL_AUX;
    ga.aux = at(b->dphi, (size_t)l_lo * d->N * d->d_ff * es);
  } else if (d->act == HBP_ACT_TANH) {
    ga.mode = EPI_MUL_1MZ2;
    ga.aux = at(b->z, (size_t)l_lo * d->N * d->d_ff * es);
  } else {
    ga.mode = EPI_STORE;
  }
  ga.aux_sb = d->N * d->d_ff;
  return run_gemm(d, ga, s, HBP_PROF_VJP1);
}

// dn[l] = da[l] . W1_l  (into the v buffer)
hbp_status vjp_stage2(const hbp_desc* d, const hbp_buffers* b, const Workspace& w, long l_lo, long l_hi,
                      hipStream_t s, bool skinny = false, bool fuse_scan = false) {
  if (tfm(d)) return tfm_stage2(d, b, w, l_lo, l_hi, s);
  const size_t es = esize(d);
  const long nl = l_hi - l_lo;
  const bool sh = shared_w(d);
  // The product lands in the hidden part of v (all of it, except for the LSTM's [c | h]: there the cell half was
  // written by the elementwise kernel and W1 is [d_ff, H]).
  const long hw = hidden_w(d);
  const size_t ho = (size_t)hidden_off(d) * es;
  // the standard GRU: the product runs over the two gates' 2H columns of da against [W_z; W_r], and the state's
  // direct share (with e already in it) comes in from the buffer the first stage left
  const long kk = gru(d) ? 2 * d->d : d->d_ff;
  const void* gru_aux = gru(d) ? at((const void*)b->workspace, w.off_tmp + (size_t)l_lo * d->N * d->d * es) : nullptr;
  if (skinny) {   // W1^T [hw,d_ff] follows W2^T (GRU: [W_z; W_r]^T [H,2H] comes first)
    SkinnyArgs k{};
    k.A = at(b->workspace, w.off_da + (size_t)l_lo * d->N * d->d_ff * es); k.lda = d->d_ff;
    k.Bt = at(b->workspace, w.off_wt + (gru(d) ? 0 : (size_t)d->d * d->d_ff * es)); k.ldbt = kk;
    k.C = at(b->workspace, w.off_v + (size_t)l_lo * d->N * d->d * es + ho); k.ldc = d->d;
    k.M = d->N; k.N = hw; k.K = kk;
    k.mode = EPI_STORE;
    if (gru(d)) { k.mode = EPI_ADD_AUX; k.aux = gru_aux; k.ldaux = d->d; }
    else if (e_in_vjp(d)) { k.mode = EPI_ADD_AUX; k.aux = at(b->e, (size_t)l_lo * d->N * d->d * es + ho); k.ldaux = d->d; }
    if (fuse_scan) {   // g_l = v_l (+ e_l) + lambda_l (.) g_{l+1} written straight into g
      k.C = at(b->g, (size_t)l_lo * d->N * d->d * es);
      k.next = at(b->g, (size_t)(l_lo + 1) * d->N * d->d * es);
      k.mode = EPI_RESID;
      if (d->lambda_kind == HBP_LAMBDA_CHANNEL) k.lambda = reinterpret_cast<const float*>(b->lambda) + l_lo * d->d;
      if (d->lambda_kind == HBP_LAMBDA_TOKEN) k.lambda_mn = at(b->lambda, (size_t)l_lo * d->N * d->d * es);
    }
    ProfScope ps(HBP_PROF_VJP2, s);
    HBP_TRY(launch_gemm_skinny(k, s));
    return HBP_OK;
  }
  GemmArgs ga{};
  ga.A = at(b->workspace, w.off_da + (size_t)l_lo * d->N * d->d_ff * es);
  ga.B = sh ? b->W1 : at(b->W1, (size_t)l_lo * d->d * d->d_ff * es);
  ga.C = at(b->workspace, w.off_v + (size_t)l_lo * d->N * d->d * es + ho);
  ga.M = sh ? nl * d->N : d->N;
  ga.N = hw;
  ga.K = kk;
  ga.a_sm = d->d_ff; ga.a_sk = 1;
  ga.b_sk = hw; ga.b_sn = 1;
  ga.ldc = d->d;
  ga.batch = sh ? 1 : nl;
  ga.a_sb = d->N * d->d_ff; ga.b_sb = d->d * d->d_ff; ga.c_sb = d->N * d->d;
  ga.split_k = 1;
  ga.mode = EPI_STORE;
  if (gru(d)) {
    ga.mode = EPI_ADD_AUX;
    ga.aux = gru_aux;
    ga.aux_sb = d->N * d->d;
  } else if (e_in_vjp(d)) {   // v_l + e_l in the epilogue: the scan then reads one stream less
    ga.mode = EPI_ADD_AUX;
    ga.aux = at(b->e, (size_t)l_lo * d->N * d->d * es + ho);
    ga.aux_sb = d->N * d->d;
  }
  return run_gemm(d, ga, s, HBP_PROF_VJP2);
}

// gamma: 0 for the exact recurrence; in the iterations of hbp_backward the descriptor's
hbp_status scan_stage(const hbp_desc* d, const hbp_buffers* b, const Workspace& w, long l_lo, long l_hi,
                      bool has_v, hipStream_t s, float gamma = 0.f, int force = 0, int m_parity = 0,
                      bool exact_step = false) {
  if (d->post == HBP_POST_RMS) {
    // the whole chain from the top (an iteration, or w^0), or one layer of exact backpropagation
    const bool whole = !exact_step;
    if (whole && (l_lo != 0 || l_hi != d->L)) return HBP_E_INVALID_ARG;
    PostScanArgs pa{};
    pa.g = b->g;
    pa.dn = has_v ? at(b->workspace, w.off_v) : nullptr;
    pa.e = (d->loss_every_state && !(has_v && e_in_vjp(d))) ? b->e : nullptr;
    pa.e_top = d->loss_every_state ? at(b->e, (size_t)d->L * d->N * d->d * esize(d)) : b->e;
    pa.x = b->x;
    pa.lambda = d->lambda_kind == HBP_LAMBDA_CHANNEL ? reinterpret_cast<const float*>(b->lambda) : nullptr;
    pa.rho = b->rinv;
    float* m0 = reinterpret_cast<float*>(at(b->workspace, w.off_m));
    float* m1 = m0 + d->L * d->N;
    pa.m_old = m_parity ? m1 : m0;      // reads the set the previous scan wrote, writes the other
    pa.m_new = m_parity ? m0 : m1;
    pa.N = d->N; pa.d = d->d;
    pa.l_lo = l_lo; pa.l_hi = l_hi;
    pa.mode = whole ? 0 : 1;
    pa.gamma = whole ? gamma : 0.f;
    pa.blk_gamma = (whole && has_v) ? gamma : 0.f;   // w^0 has no block term: only the residual path is rescaled
    ProfScope ps(HBP_PROF_SCAN, s);
    HBP_TRY(launch_scan_post(d->dtype, pa, s));
    return HBP_OK;
  }
  ScanArgs sa{};
  sa.force = force;
  sa.res_scale = 1.f - gamma;
  sa.blk_gamma = has_v ? gamma : 0.f;   // w^0 has no block term: only the residual path is rescaled
  sa.g = b->g;
  sa.dn = has_v ? at(b->workspace, w.off_v) : nullptr;
  sa.y = b->y;
  sa.rinv = b->rinv;
  sa.e = (d->loss_every_state && !(has_v && e_in_vjp(d))) ? b->e : nullptr;
  sa.chunk_ws = (force >= 2 || scan_chunk_ws_bytes(d->L, d->N, d->d, d->norm == HBP_NORM_RMS))
                    ? reinterpret_cast<float*>(at(b->workspace, force >= 2 ? 0 : w.off_scan)) : nullptr;
  sa.lambda = d->lambda_kind == HBP_LAMBDA_CHANNEL ? reinterpret_cast<const float*>(b->lambda) : nullptr;
  sa.lambda_tok = d->lambda_kind == HBP_LAMBDA_TOKEN ? b->lambda : nullptr;
  sa.N = d->N; sa.d = d->d;
  sa.l_lo = l_lo; sa.l_hi = l_hi;
  sa.norm_rms = d->norm == HBP_NORM_RMS;
  sa.mask = d->post == HBP_POST_RELU ? b->mask : nullptr;
  ProfScope ps(HBP_PROF_SCAN, s);
  HBP_TRY(launch_scan(d->dtype, sa, s));
  return HBP_OK;
}

// g[L] := e_L
hbp_status seed_top(const hbp_desc* d, const hbp_buffers* b, hipStream_t s) {
  if (d->post == HBP_POST_RMS) return HBP_OK;   // the post-norm scan seeds g[L] itself (through the last norm)
  const size_t es = esize(d);
  const size_t row = (size_t)d->N * d->d * es;
  const void* src = d->loss_every_state ? at(b->e, (size_t)d->L * row) : b->e;
  ProfScope ps(HBP_PROF_OTHER, s);
  HBP_TRY(hipMemcpyAsync(at(b->g, (size_t)d->L * row), src, row, hipMemcpyDeviceToDevice, s));
  if (d->post == HBP_POST_RELU)   // g[L] is kept taken through the ReLU that made x_L, like every g[l >= 1]
    HBP_TRY(launch_mask_apply(d->dtype, at(b->g, (size_t)d->L * row), b->mask + (size_t)(d->L - 1) * d->N * d->d / 8,
                              d->N * d->d, s));
  return HBP_OK;
}

// C[b] (fp32 [M,N]) = sum over `K` rows of A[b](k,m) * B[b](k,n), rows K-major
hbp_status tn_gemm(const hbp_desc* d, const void* A, long lda, long a_sb, const void* B, long ldb, long b_sb,
                   float* C, long M, long N, long K, long batch, int split, void* part, hipStream_t s) {
  GemmArgs ga{};
  ga.A = A; ga.B = B;
  ga.M = M; ga.N = N; ga.K = K;
  ga.a_sm = 1; ga.a_sk = lda;
  ga.b_sk = ldb; ga.b_sn = 1;
  ga.ldc = N;
  ga.batch = batch;
  ga.a_sb = a_sb; ga.b_sb = b_sb; ga.c_sb = M * N;
  ga.split_k = split;
  ga.mode = EPI_STORE;
  ga.c_is_f32 = 1;
  ga.C = split > 1 ? part : (void*)C;
  HBP_RUN(run_gemm(d, ga, s, HBP_PROF_DW));
  if (split > 1) {
    ProfScope ps(HBP_PROF_OTHER, s);
    HBP_TRY(launch_splitk_reduce((const float*)part, C, batch * M * N, split, s));
  }
  return HBP_OK;
}

}  // namespace

extern "C" {

const char* hbp_status_string(hbp_status s) {
  switch (s) {
    case HBP_OK: return "ok";
    case HBP_E_INVALID_ARG: return "invalid argument";
    case HBP_E_UNSUPPORTED: return "unsupported size";
    case HBP_E_WORKSPACE: return "workspace missing or too small";
    case HBP_E_NULL: return "required pointer is NULL";
    case HBP_E_DEVICE: return "HIP launch failed";
  }
  return "unknown status";
}

hbp_status hbp_profile_enable(int on) {
  ProfState& p = prof();
  std::lock_guard<std::mutex> lk(p.mu);
  p.on = on != 0;
  return HBP_OK;
}

hbp_status hbp_profile_read(double* ms, int64_t* launches) {
  if (!ms || !launches) return HBP_E_NULL;
  ProfState& p = prof();
  std::lock_guard<std::mutex> lk(p.mu);
  for (int c = 0; c < HBP_PROF_CLASSES; ++c) { ms[c] = 0.0; launches[c] = 0; }
  hbp_status st = HBP_OK;
  for (ProfRec& r : p.recs) {
    float t = 0.f;
    if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&t, r.a, r.b) != hipSuccess) st = HBP_E_DEVICE;
    ms[r.cls] += t;
    launches[r.cls] += 1;
    p.pool.push_back(r.a);
    p.pool.push_back(r.b);
  }
  p.recs.clear();
  return st;
}

hbp_status hbp_workspace_size(const hbp_desc* desc, size_t* bytes) {
  if (!bytes) return HBP_E_NULL;
  HBP_RUN(check_desc(desc));
  *bytes = carve(desc).total;
  return HBP_OK;
}

hbp_status hbp_check(const hbp_desc* desc, const hbp_buffers* bufs) {
  HBP_RUN(check_desc(desc));
  if (bufs) HBP_RUN(check_bufs(desc, bufs, NEED_BWD));
  return HBP_OK;
}

hbp_status hbp_forward(const hbp_desc* d, hbp_buffers* b, void* stream) {
  HBP_RUN(check_desc(d));
  HBP_RUN(check_bufs(d, b, NEED_FWD));
  hipStream_t s = (hipStream_t)stream;
  const Workspace w = carve(d);
  const size_t es = esize(d);
  const bool sh = shared_w(d);
  const bool rms = d->norm == HBP_NORM_RMS;
  float* ux = reinterpret_cast<float*>(at(b->workspace, w.off_da));
  const bool skinny = step_skinny(d) && d->act != HBP_ACT_GELU_ERF;
  if (recurrent(d)) {  // U . xin for every step at once
    GemmArgs ga{};
    ga.A = b->xin; ga.B = b->U; ga.C = ux;
    ga.M = d->L * d->N; ga.N = d->d_ff; ga.K = d->d_in;
    ga.a_sm = d->d_in; ga.a_sk = 1;
    ga.b_sk = 1; ga.b_sn = d->d_in;
    ga.ldc = d->d_ff; ga.batch = 1; ga.split_k = 1;
    ga.mode = EPI_STORE; ga.c_is_f32 = 1;
    HBP_RUN(run_gemm(d, ga, s, HBP_PROF_FORWARD));
  }
  for (long l = 0; l < d->L; ++l) {
    const long wl = tfm(d) ? l / 2 : l;          // weight set and inner-state row of this block
    const size_t xo = (size_t)l * d->N * d->d * es;
    const size_t fo = (size_t)wl * d->N * d->d_ff * es;
    const void* yl = at((const void*)b->x, xo);
    if (rms) {
      ProfScope ps(HBP_PROF_FORWARD, s);
      HBP_TRY(launch_rmsnorm_fwd(d->dtype, at((const void*)b->x, xo), at(b->y, xo), b->rinv + l * d->N, d->N, d->d,
                                 d->eps, s));
      yl = at((const void*)b->y, xo);
    }
    if (tfm(d) && l % 2 == 0) {     // attention sub-block: [q | k | v] = y Wqkv^T, attention, x_{l+1} = lambda (.) x_l + o Wo^T
      const long N = d->N, D = d->d;
      {
        GemmArgs ga{};
        ga.A = yl;
        ga.B = at(b->Wqkv, (size_t)wl * 3 * D * D * es);
        ga.C = at(b->qkv, (size_t)wl * N * 3 * D * es);
        ga.M = N; ga.N = 3 * D; ga.K = D;
        ga.a_sm = D; ga.a_sk = 1;
        ga.b_sk = 1; ga.b_sn = D;
        ga.ldc = 3 * D; ga.batch = 1; ga.split_k = 1;
        ga.mode = EPI_STORE;
        HBP_RUN(run_gemm(d, ga, s, HBP_PROF_FORWARD));
      }
      {
        ProfScope ps(HBP_PROF_ATTN, s);
        HBP_TRY(launch_attn_fwd(d->dtype, attn_args(d, b, w, wl, wl + 1), s));
      }
      GemmArgs ga{};
      ga.A = at((const void*)b->attn_o, (size_t)wl * N * D * es);
      ga.B = at(b->Wo, (size_t)wl * D * D * es);
      ga.C = at(b->x, xo + (size_t)N * D * es);
      ga.M = N; ga.N = D; ga.K = D;
      ga.a_sm = D; ga.a_sk = 1;
      ga.b_sk = 1; ga.b_sn = D;
      ga.ldc = D; ga.batch = 1; ga.split_k = 1;
      ga.mode = EPI_RESID;
      ga.aux = at((const void*)b->x, xo);
      ga.lambda = d->lambda_kind == HBP_LAMBDA_CHANNEL ? reinterpret_cast<const float*>(b->lambda) + l * D : nullptr;
      ga.lambda_mn = d->lambda_kind == HBP_LAMBDA_TOKEN ? at(b->lambda, xo) : nullptr;
      HBP_RUN(run_gemm(d, ga, s, HBP_PROF_FORWARD));
      if (d->post == HBP_POST_RMS) {     // post-norm: the norm after the residual sum, as for the MLP sub-blocks below
        ProfScope ps(HBP_PROF_FORWARD, s);
        HBP_TRY(launch_rmsnorm_inplace(d->dtype, at(b->x, xo + (size_t)N * D * es), b->rinv + l * N, N, D, d->eps, s));
      }
      continue;
    }
    if (gru(d)) {
      // two dependent products per step: the gates z, r from x; then the candidate from r (.) x
      float* pre = reinterpret_cast<float*>(at(b->workspace, w.off_pre));
      void* rx = at(b->workspace, w.off_tmp);
      const long H = d->d;
      const float* uxl = ux + l * d->N * d->d_ff;
      auto product = [&](const void* A, long n_out, long col0) -> hbp_status {   // pre[:, col0 .. col0 + n_out) = A W^T + ux
        const void* Wp = at(b->W1, (size_t)col0 * H * es);
        if (skinny) {
          SkinnyArgs k{};
          k.A = A; k.lda = H;
          k.Bt = Wp; k.ldbt = H;
          k.C = pre + col0; k.ldc = d->d_ff; k.c_is_f32 = 1;
          k.M = d->N; k.N = n_out; k.K = H;
          k.mode = EPI_STORE;
          k.addf = uxl + col0;
          ProfScope ps(HBP_PROF_FORWARD, s);
          HBP_TRY(launch_gemm_skinny(k, s));
          return HBP_OK;
        }
        GemmArgs ga{};
        ga.A = A; ga.B = Wp; ga.C = pre + col0;
        ga.M = d->N; ga.N = n_out; ga.K = H;
        ga.a_sm = H; ga.a_sk = 1;
        ga.b_sk = 1; ga.b_sn = H;
        ga.ldc = d->d_ff; ga.batch = 1; ga.split_k = 1;
        ga.mode = EPI_STORE; ga.c_is_f32 = 1;
        ga.addf = uxl + col0;
        return run_gemm(d, ga, s, HBP_PROF_FORWARD);
      };
      HBP_RUN(product(yl, 2 * H, 0));
      {
        ProfScope ps(HBP_PROF_FORWARD, s);
        HBP_TRY(launch_gru_fwd1(d->dtype, pre, yl, at(b->z, fo), rx, d->N, H, s));
      }
      HBP_RUN(product(rx, H, 2 * H));
      ProfScope ps(HBP_PROF_FORWARD, s);
      HBP_TRY(launch_gru_fwd2(d->dtype, pre, yl, at(b->z, fo), at(b->lambda, xo), at(b->x, xo + (size_t)d->N * H * es),
                              d->N, H, s));
      continue;
    }
    if (cell(d)) {
      // pre = h W1^T + U xin (fp32), then the cell elementwise: z[l] = the gates, lambda[l] = the residual
      // coefficient, x[l+1]
      float* pre = reinterpret_cast<float*>(at(b->workspace, w.off_pre));
      const long hw = hidden_w(d);
      const void* hl = at(yl, (size_t)hidden_off(d) * es);
      if (skinny) {
        SkinnyArgs k{};
        k.A = hl; k.lda = d->d;
        k.Bt = b->W1; k.ldbt = hw;
        k.C = pre; k.ldc = d->d_ff; k.c_is_f32 = 1;
        k.M = d->N; k.N = d->d_ff; k.K = hw;
        k.mode = EPI_STORE;
        k.addf = ux + l * d->N * d->d_ff;
        ProfScope ps(HBP_PROF_FORWARD, s);
        HBP_TRY(launch_gemm_skinny(k, s));
      } else {
        GemmArgs ga{};
        ga.A = hl; ga.B = b->W1; ga.C = pre;
        ga.M = d->N; ga.N = d->d_ff; ga.K = hw;
        ga.a_sm = d->d; ga.a_sk = 1;
        ga.b_sk = 1; ga.b_sn = hw;
        ga.ldc = d->d_ff; ga.batch = 1; ga.split_k = 1;
        ga.mode = EPI_STORE; ga.c_is_f32 = 1;
        ga.addf = ux + l * d->N * d->d_ff;
        HBP_RUN(run_gemm(d, ga, s, HBP_PROF_FORWARD));
      }
      ProfScope ps(HBP_PROF_FORWARD, s);
      if (d->kind == HBP_GATED)
        HBP_TRY(launch_gated_fwd(d->dtype, pre, yl, at(b->z, fo), at(b->lambda, xo),
                                 at(b->x, xo + (size_t)d->N * d->d * es), d->N, d->d, s));
      else
        HBP_TRY(launch_lstm_fwd(d->dtype, pre, yl, at(b->z, fo), at(b->lambda, xo),
                                at(b->x, xo + (size_t)d->N * d->d * es), d->N, d->d / 2, s));
      continue;
    }
    if (skinny) {   // one step of the recurrence, few rows; the weights as stored are already K-contiguous
      SkinnyArgs k{};
      k.A = yl; k.lda = d->d;
      k.Bt = b->W1; k.ldbt = d->d;
      k.C = at(b->z, fo); k.ldc = d->d_ff;
      k.M = d->N; k.N = d->d_ff; k.K = d->d;
      k.mode = d->act == HBP_ACT_TANH ? EPI_ACT_TANH : EPI_STORE;
      k.addf = ux + l * d->N * d->d_ff;
      {
        ProfScope ps(HBP_PROF_FORWARD, s);
        HBP_TRY(launch_gemm_skinny(k, s));
      }
      SkinnyArgs r{};
      r.A = at((const void*)b->z, fo); r.lda = d->d_ff;
      r.Bt = b->W2; r.ldbt = d->d_ff;
      r.C = at(b->x, xo + (size_t)d->N * d->d * es); r.ldc = d->d;
      r.M = d->N; r.N = d->d; r.K = d->d_ff;
      r.mode = EPI_RESID;
      r.next = at((const void*)b->x, xo);
      r.lambda = d->lambda_kind == HBP_LAMBDA_CHANNEL ? reinterpret_cast<const float*>(b->lambda) + l * d->d : nullptr;
      r.lambda_mn = d->lambda_kind == HBP_LAMBDA_TOKEN ? at(b->lambda, xo) : nullptr;
      ProfScope ps(HBP_PROF_FORWARD, s);
      HBP_TRY(launch_gemm_skinny(r, s));
      continue;
    }
    {  // a = y W1^T (+ U xin); z = act(a); dphi = act'(a)
      GemmArgs ga{};
      ga.A = yl;
      ga.B = sh ? b->W1 : at(b->W1, (size_t)wl * d->d * d->d_ff * es);
      ga.C = at(b->z, fo);
      ga.M = d->N; ga.N = d->d_ff; ga.K = d->d;
      ga.a_sm = d->d; ga.a_sk = 1;
      ga.b_sk = 1; ga.b_sn = d->d;
      ga.ldc = d->d_ff; ga.batch = 1; ga.split_k = 1;
      if (d->act == HBP_ACT_GELU_ERF) { ga.mode = EPI_ACT_GELU; ga.out2 = at(b->dphi, fo); }
      else if (d->act == HBP_ACT_TANH) ga.mode = EPI_ACT_TANH;
      else ga.mode = EPI_STORE;
      if (d->kind == HBP_RNN) ga.addf = ux + l * d->N * d->d_ff;
      HBP_RUN(run_gemm(d, ga, s, HBP_PROF_FORWARD));
    }
    {  // x_{l+1} = lambda (.) x_l + z W2^T
      GemmArgs ga{};
      ga.A = at((const void*)b->z, fo);
      ga.B = sh ? b->W2 : at(b->W2, (size_t)wl * d->d * d->d_ff * es);
      ga.C = at(b->x, xo + (size_t)d->N * d->d * es);
      ga.M = d->N; ga.N = d->d; ga.K = d->d_ff;
      ga.a_sm = d->d_ff; ga.a_sk = 1;
      ga.b_sk = 1; ga.b_sn = d->d_ff;
      ga.ldc = d->d; ga.batch = 1; ga.split_k = 1;
      ga.mode = EPI_RESID;
      ga.aux = at((const void*)b->x, xo);
      ga.lambda = d->lambda_kind == HBP_LAMBDA_CHANNEL ? reinterpret_cast<const float*>(b->lambda) + l * d->d : nullptr;
      ga.lambda_mn = d->lambda_kind == HBP_LAMBDA_TOKEN ? at(b->lambda, xo) : nullptr;
      HBP_RUN(run_gemm(d, ga, s, HBP_PROF_FORWARD));
    }
    if (d->post == HBP_POST_RMS) {
      ProfScope ps(HBP_PROF_FORWARD, s);
      HBP_TRY(launch_rmsnorm_inplace(d->dtype, at(b->x, xo + (size_t)d->N * d->d * es), b->rinv + l * d->N, d->N, d->d,
                                     d->eps, s));
    }
    if (d->post == HBP_POST_RELU) {
      ProfScope ps(HBP_PROF_FORWARD, s);
      HBP_TRY(launch_relu_mask(d->dtype, at(b->x, xo + (size_t)d->N * d->d * es), b->mask + (size_t)l * d->N * d->d / 8,
                               d->N * d->d, s));
    }
  }
  return HBP_OK;
}

hbp_status hbp_backward(const hbp_desc* d, int k, hbp_buffers* b, void* stream) {
  HBP_RUN(check_desc(d));
  if (k < 0) return HBP_E_INVALID_ARG;
  HBP_RUN(check_bufs(d, b, NEED_BWD));
  hipStream_t s = (hipStream_t)stream;
  const Workspace w = carve(d);
  // y aliases x when there is no norm
  hbp_buffers bb = *b;
  if (d->norm == HBP_NORM_NONE) bb.y = bb.x;
  HBP_RUN(seed_top(d, &bb, s));
  // w^0: the residual path alone
  HBP_RUN(scan_stage(d, &bb, w, 0, d->L, false, s, d->gamma));
  // More than L iterations change nothing (Theorem 2: exact for k >= L - i).
  const long iters = k > d->L ? d->L : k;
  for (long it = 1; it <= iters; ++it) {
    // After it-2 iterations the states l+1 >= L-it+2 are already exact (and
    // bit-identical from then on), so v_l of blocks l >= L-it+1 left by the
    // previous iteration is still valid: recompute only the blocks below.
    long l_hi = d->L - it + 1;
    if (recurrent(d)) {
      // One contraction covers all rows (l_hi * N): where re-doing a few of the final blocks keeps
      // the row count a multiple of the 256-row GEMM tile, do that (same values, aligned kernel).
      long step = 256;
      for (long a = d->N, b2 = 256; b2 != 0;) { const long r = a % b2; a = b2; b2 = r; step = 256 / a; }
      const long padded = (l_hi + step - 1) / step * step;
      if (padded <= d->L) l_hi = padded;
    }
    HBP_RUN(vjp_stage1(d, &bb, w, 0, l_hi, s));
    HBP_RUN(vjp_stage2(d, &bb, w, 0, l_hi, s));
    HBP_RUN(scan_stage(d, &bb, w, 0, d->L, true, s, d->gamma, 0, (int)(it & 1)));
  }
  return HBP_OK;
}

hbp_status hbp_scan_workspace_size(const hbp_desc* d, int algorithm, size_t* bytes) {
  if (!bytes) return HBP_E_NULL;
  HBP_RUN(check_desc(d));
  // a ReLU's mask or a norm after the sum is applied by the direct forms only
  if (d->post != HBP_POST_NONE && (algorithm == HBP_SCAN_CHUNKED || algorithm == HBP_SCAN_HILLIS_STEELE ||
                                   algorithm == HBP_SCAN_SINGLE_PASS))
    return HBP_E_UNSUPPORTED;
  if (algorithm == HBP_SCAN_SINGLE_PASS && d->dtype != HBP_BF16) return HBP_E_UNSUPPORTED;
  switch (algorithm) {
    case HBP_SCAN_AUTO: case HBP_SCAN_SEQUENTIAL: *bytes = carve(d).total; break;
    case HBP_SCAN_CHUNKED: *bytes = scan_chunk_ws_bytes_forced(d->L, d->N, d->d); break;
    case HBP_SCAN_SINGLE_PASS: *bytes = scan_sp_ws_bytes(d->L, d->N, d->d, d->lambda_kind == HBP_LAMBDA_TOKEN); break;
    case HBP_SCAN_HILLIS_STEELE: *bytes = hs_ws_bytes(d->L, d->N, d->d, d->lambda_kind); break;
    default: return HBP_E_INVALID_ARG;
  }
  return HBP_OK;
}

hbp_status hbp_initial_estimate(const hbp_desc* d, int algorithm, hbp_buffers* b, void* stream) {
  size_t need = 0;
  HBP_RUN(hbp_scan_workspace_size(d, algorithm, &need));
  if (!b) return HBP_E_NULL;
  if (b->struct_size != sizeof(hbp_buffers)) return HBP_E_INVALID_ARG;
  if (!b->e || !b->g) return HBP_E_NULL;
  if (d->lambda_kind != HBP_LAMBDA_ONE && !b->lambda) return HBP_E_NULL;
  if (!b->workspace || b->workspace_bytes < need) return HBP_E_WORKSPACE;
  if (d->post == HBP_POST_RELU && !b->mask) return HBP_E_NULL;
  if (d->post == HBP_POST_RMS && (!b->x || !b->rinv)) return HBP_E_NULL;
  hipStream_t s = (hipStream_t)stream;
  if (algorithm == HBP_SCAN_HILLIS_STEELE) {
    HsArgs a{};
    a.g = b->g; a.e = b->e; a.every_state = d->loss_every_state;
    a.lambda = d->lambda_kind == HBP_LAMBDA_CHANNEL ? reinterpret_cast<const float*>(b->lambda) : nullptr;
    a.lambda_tok = d->lambda_kind == HBP_LAMBDA_TOKEN ? b->lambda : nullptr;
    a.res_scale = 1.f - d->gamma;
    a.L = d->L; a.N = d->N; a.d = d->d;
    a.ws = reinterpret_cast<float*>(b->workspace);
    ProfScope ps(HBP_PROF_SCAN, s);
    HBP_TRY(launch_scan_hillis_steele(d->dtype, a, s));
    return HBP_OK;
  }
  const Workspace w = carve(d);
  HBP_RUN(seed_top(d, b, s));
  return scan_stage(d, b, w, 0, d->L, false, s, d->gamma,
                    algorithm == HBP_SCAN_SEQUENTIAL ? 1 : algorithm == HBP_SCAN_CHUNKED ? 2 :
                    algorithm == HBP_SCAN_SINGLE_PASS ? 3 : 0);
}

namespace {
// The device address of `scratch` on the current device, looked up once per device.
hbp_status static_scratch(float** out) {
  constexpr int MAX_DEV = 64;
  static std::mutex mu;
  static void* ptr[MAX_DEV] = {};
  int dev = 0;
  HBP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEV) return HBP_E_DEVICE;
  std::lock_guard<std::mutex> lk(mu);
  if (!ptr[dev]) {
    void* q = nullptr;
    HBP_TRY(hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)));
    if (!q) return HBP_E_DEVICE;
    ptr[dev] = q;
  }
  *out = reinterpret_cast<float*>(ptr[dev]);
  return HBP_OK;
}
}  // namespace

hbp_status hbp_initial_estimate_static(const hbp_desc* d, hbp_buffers* b, void* stream) {
  HBP_RUN(check_desc(d));
  if (d->post != HBP_POST_NONE) return HBP_E_UNSUPPORTED;   // as for HBP_SCAN_CHUNKED
  if (scan_chunk_ws_bytes_forced(d->L, d->N, d->d) > (size_t)HBP_STATIC_SCRATCH_BYTES) return HBP_E_WORKSPACE;
  if (!b) return HBP_E_NULL;
  if (b->struct_size != sizeof(hbp_buffers)) return HBP_E_INVALID_ARG;
  if (!b->e || !b->g) return HBP_E_NULL;
  if (d->lambda_kind != HBP_LAMBDA_ONE && !b->lambda) return HBP_E_NULL;
  hipStream_t s = (hipStream_t)stream;
  float* ws = nullptr;
  HBP_RUN(static_scratch(&ws));
  HBP_RUN(seed_top(d, b, s));
  // Every part of the scratch the passes read is written earlier in the same call (the reduce pass writes B, A and
  // the old state above each chunk, the combine pass the state entering each chunk): nothing has to start at zero.
  ScanArgs sa{};
  sa.force = 2;
  sa.res_scale = 1.f - d->gamma;
  sa.g = b->g;
  sa.e = d->loss_every_state ? b->e : nullptr;
  sa.chunk_ws = ws;
  sa.lambda = d->lambda_kind == HBP_LAMBDA_CHANNEL ? reinterpret_cast<const float*>(b->lambda) : nullptr;
  sa.lambda_tok = d->lambda_kind == HBP_LAMBDA_TOKEN ? b->lambda : nullptr;
  sa.N = d->N; sa.d = d->d;
  sa.l_lo = 0; sa.l_hi = d->L;
  ProfScope ps(HBP_PROF_SCAN, s);
  HBP_TRY(launch_scan(d->dtype, sa, s));
  return HBP_OK;
}

hbp_status hbp_exact_backward(const hbp_desc* d, hbp_buffers* b, void* stream) {
  HBP_RUN(check_desc(d));
  HBP_RUN(check_bufs(d, b, NEED_BWD));
  hipStream_t s = (hipStream_t)stream;
  const Workspace w = carve(d);
  hbp_buffers bb = *b;
  if (d->norm == HBP_NORM_NONE) bb.y = bb.x;
  HBP_RUN(seed_top(d, &bb, s));
  if (d->post == HBP_POST_RMS) {   // g[L] = e_L taken through the last norm
    PostScanArgs pa{};
    pa.g = bb.g; pa.x = bb.x; pa.rho = bb.rinv;
    pa.e_top = d->loss_every_state ? at(bb.e, (size_t)d->L * d->N * d->d * esize(d)) : bb.e;
    pa.m_new = reinterpret_cast<float*>(at(bb.workspace, w.off_m));
    pa.N = d->N; pa.d = d->d; pa.l_lo = d->L; pa.l_hi = d->L; pa.mode = 2;
    ProfScope ps(HBP_PROF_SCAN, s);
    HBP_TRY(launch_scan_post(d->dtype, pa, s));
  }
  const bool skinny = step_skinny(d);
  // the step along the residual path in the same kernel (not for the LSTM, whose cell half is not a product)
  const bool fuse = skinny && d->norm == HBP_NORM_NONE && d->kind != HBP_LSTM;
  if (skinny && gru(d)) {   // [W_z; W_r]^T [H,2H], then W_n^T [H,H]
    ProfScope ps(HBP_PROF_OTHER, s);
    const long H = d->d;
    HBP_TRY(launch_transpose_bf16(bb.W1, at(bb.workspace, w.off_wt), (int)(2 * H), (int)H, s));
    HBP_TRY(launch_transpose_bf16(at(bb.W1, (size_t)2 * H * H * esize(d)),
                                  at(bb.workspace, w.off_wt + (size_t)2 * H * H * esize(d)), (int)H, (int)H, s));
  } else if (skinny) {
    ProfScope ps(HBP_PROF_OTHER, s);
    if (!cell(d))
      HBP_TRY(launch_transpose_bf16(bb.W2, at(bb.workspace, w.off_wt), (int)d->d, (int)d->d_ff, s));
    HBP_TRY(launch_transpose_bf16(bb.W1, at(bb.workspace, w.off_wt + (size_t)d->d * d->d_ff * esize(d)), (int)d->d_ff,
                                  (int)hidden_w(d), s));
  }
  for (long l = d->L - 1; l >= 0; --l) {
    HBP_RUN(vjp_stage1(d, &bb, w, l, l + 1, s, skinny));
    HBP_RUN(vjp_stage2(d, &bb, w, l, l + 1, s, skinny, fuse));
    if (!fuse) HBP_RUN(scan_stage(d, &bb, w, l, l + 1, true, s, 0.f, 0, 0, true));
  }
  return HBP_OK;
}

hbp_status hbp_param_grads(const hbp_desc* d, hbp_buffers* b, void* stream) {
  HBP_RUN(check_desc(d));
  HBP_RUN(check_bufs(d, b, NEED_PG));
  hipStream_t s = (hipStream_t)stream;
  const Workspace w = carve(d);
  const size_t es = esize(d);
  const bool sh = shared_w(d);
  hbp_buffers bb = *b;
  if (d->norm == HBP_NORM_NONE) bb.y = bb.x;
  const Splits sp = param_splits(d);
  // da from the final estimate (the standard GRU also leaves r (.) x, the candidate weights' operand, in the v buffer)
  HBP_RUN(vjp_stage1(d, &bb, w, 0, d->L, s, false, gru(d) ? at(b->workspace, w.off_v) : nullptr));
  const long K = sh ? d->L * d->N : d->N;
  const long nb = sh ? 1 : d->L;
  void* part = at(b->workspace, w.off_part);
  const void* g1 = at((const void*)bb.g, (size_t)d->N * d->d * es);
  const void* da = at((const void*)b->workspace, w.off_da);
  if (tfm(d)) {
    // MLP sub-blocks (odd l = 2j+1): dW2_j = g[2j+2]^T z_j, dW1_j = da_j^T y[2j+1]; attention sub-blocks (even l = 2j):
    // dWo_j = g[2j+1]^T o_j, dWqkv_j = dqkv_j^T y[2j]
    const long N = d->N, D = d->d, F = d->d_ff, Lh = d->L / 2;
    const void* g2 = at((const void*)bb.g, (size_t)2 * N * D * es);
    const void* y1 = at((const void*)bb.y, (size_t)N * D * es);
    HBP_RUN(tn_gemm(d, g2, D, 2 * N * D, bb.z, F, N * F, bb.dW2, D, F, N, Lh, sp.s_w2, part, s));
    HBP_RUN(tn_gemm(d, da, F, N * F, y1, D, 2 * N * D, bb.dW1, F, D, N, Lh, sp.s_w1, part, s));
    HBP_RUN(tn_gemm(d, g1, D, 2 * N * D, bb.attn_o, D, N * D, bb.dWo, D, D, N, Lh, sp.s_o, part, s));
    HBP_RUN(tn_gemm(d, at((const void*)b->workspace, w.off_dqkv), 3 * D, 3 * N * D, bb.y, D, 2 * N * D, bb.dWqkv, 3 * D, D,
                    N, Lh, sp.s_qkv, part, s));
    return HBP_OK;
  }
  // dW2[c,j] = sum_n g_{l+1}[n,c] z_l[n,j]   (the gated cell has no second weight)
  if (!cell(d))
    HBP_RUN(tn_gemm(d, g1, d->d, d->N * d->d, bb.z, d->d_ff, d->N * d->d_ff, bb.dW2, d->d, d->d_ff, K, nb, sp.s_w2,
                    part, s));
  // dW1[j,c] = sum_n da_l[n,j] y_l[n,c]   (a cell: over the hidden part of the state)
  if (gru(d)) {      // rows of the two gates against x, rows of the candidate against r (.) x
    const long H = d->d;
    HBP_RUN(tn_gemm(d, da, d->d_ff, 0, bb.y, H, 0, bb.dW1, 2 * H, H, K, 1, sp.s_w1, part, s));
    HBP_RUN(tn_gemm(d, at(da, (size_t)2 * H * es), d->d_ff, 0, at((const void*)b->workspace, w.off_v), H, 0,
                    bb.dW1 + 2 * H * H, H, H, K, 1, sp.s_w1, part, s));
  } else
  HBP_RUN(tn_gemm(d, da, d->d_ff, d->N * d->d_ff, at((const void*)bb.y, (size_t)hidden_off(d) * es), d->d,
                  d->N * d->d, bb.dW1, d->d_ff, hidden_w(d), K, nb, sp.s_w1, part, s));
  if (recurrent(d)) {
    // dU[j,i] = sum da[n,j] xin[n,i]
    HBP_RUN(tn_gemm(d, da, d->d_ff, 0, bb.xin, d->d_in, 0, bb.dU, d->d_ff, d->d_in, K, 1, sp.s_u, part, s));
  }
  return HBP_OK;
}

namespace {
struct ParamSizes { long n1, n2, nu, nq, no; };
ParamSizes param_sizes(const hbp_desc* d) {
  const long nb = shared_w(d) ? 1 : tfm(d) ? d->L / 2 : d->L;
  ParamSizes p{};
  p.nq = tfm(d) ? nb * 3 * d->d * d->d : 0;
  p.no = tfm(d) ? nb * d->d * d->d : 0;
  p.n1 = nb * d->d_ff * hidden_w(d);
  p.n2 = cell(d) ? 0 : nb * d->d * d->d_ff;
  p.nu = recurrent(d) ? d->d_ff * d->d_in : 0;
  return p;
}
}  // namespace

hbp_status hbp_train_scratch_size(size_t* bytes) {
  if (!bytes) return HBP_E_NULL;
  *bytes = train_scratch_floats() * sizeof(float);
  return HBP_OK;
}

hbp_status hbp_loss_mse(const hbp_desc* d, const hbp_buffers* b, const void* target, void* e_out, float* loss_out,
                        float* scratch, size_t scratch_bytes, void* stream) {
  HBP_RUN(check_desc(d));
  if (!b) return HBP_E_NULL;
  if (b->struct_size != sizeof(hbp_buffers)) return HBP_E_INVALID_ARG;
  if (!b->x || !target || !e_out || !loss_out) return HBP_E_NULL;
  if (!scratch || scratch_bytes < train_scratch_floats() * sizeof(float)) return HBP_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const size_t es = esize(d);
  const long layer = d->N * d->d;
  const float inv_n = 1.0f / (float)d->N;
  ProfScope ps(HBP_PROF_OTHER, s);
  if (d->loss_every_state) {      // states 1..L; e[0] = 0
    HBP_TRY(launch_zero(d->dtype, e_out, layer, s));
    HBP_TRY(launch_mse_loss_grad(d->dtype, at((const void*)b->x, (size_t)layer * es), at(target, (size_t)layer * es),
                                 at(e_out, (size_t)layer * es), d->L * layer, inv_n, scratch, loss_out, s));
  } else {
    HBP_TRY(launch_mse_loss_grad(d->dtype, at((const void*)b->x, (size_t)d->L * layer * es), target, e_out, layer, inv_n,
                                 scratch, loss_out, s));
  }
  return HBP_OK;
}

hbp_status hbp_optimizer_step(const hbp_desc* d, hbp_buffers* b, const hbp_optim* o, hbp_optim_state* st, void* stream) {
  HBP_RUN(check_desc(d));
  if (!b || !o || !st) return HBP_E_NULL;
  if (b->struct_size != sizeof(hbp_buffers) || o->struct_size != sizeof(hbp_optim) ||
      st->struct_size != sizeof(hbp_optim_state))
    return HBP_E_INVALID_ARG;
  if (o->kind != HBP_OPT_SGD && o->kind != HBP_OPT_ADAMW) return HBP_E_INVALID_ARG;
  const bool adamw = o->kind == HBP_OPT_ADAMW;
  if (!(o->lr >= 0.f) || !(o->beta1 >= 0.f && o->beta1 < 1.f) || !(o->weight_decay >= 0.f) || !(o->clip_norm >= 0.f))
    return HBP_E_INVALID_ARG;
  if (adamw && (!(o->beta2 >= 0.f && o->beta2 < 1.f) || !(o->eps >= 0.f) || o->step < 1)) return HBP_E_INVALID_ARG;
  const ParamSizes ps = param_sizes(d);
  struct T3 { void* w; float* master; const float* g; float* m; float* v; long n; };
  T3 t[5] = {{const_cast<void*>(b->W1), st->master1, b->dW1, st->m1, st->v1, ps.n1},
             {const_cast<void*>(b->W2), st->master2, b->dW2, st->m2, st->v2, ps.n2},
             {const_cast<void*>(b->U), st->masterU, b->dU, st->mU, st->vU, ps.nu},
             {const_cast<void*>(b->Wqkv), st->masterQ, b->dWqkv, st->mQ, st->vQ, ps.nq},
             {const_cast<void*>(b->Wo), st->masterO, b->dWo, st->mO, st->vO, ps.no}};
  for (const T3& x : t) {
    if (x.n == 0) continue;
    if (!x.w || !x.g || !x.m || (adamw && !x.v)) return HBP_E_NULL;
  }
  if (o->clip_norm > 0.f && (!st->scratch || st->scratch_bytes < train_scratch_floats() * sizeof(float)))
    return HBP_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  ProfScope pscope(HBP_PROF_OTHER, s);
  const float* clip = nullptr;
  if (o->clip_norm > 0.f) {
    const float* gs[5]; long ns[5]; int cnt = 0;
    for (const T3& x : t) if (x.n) { gs[cnt] = x.g; ns[cnt] = x.n; ++cnt; }
    float* factor = st->scratch + train_scratch_floats() - 8;
    HBP_TRY(launch_clip_factor(gs, ns, cnt, o->clip_norm, st->scratch, factor, s));
    clip = factor;
  }
  OptimArgs a{};
  a.lr = o->lr; a.beta1 = o->beta1; a.beta2 = o->beta2; a.eps = o->eps; a.weight_decay = o->weight_decay;
  if (adamw) {
    a.inv_bias1 = (float)(1.0 / (1.0 - pow((double)o->beta1, (double)o->step)));
    a.inv_bias2 = (float)(1.0 / (1.0 - pow((double)o->beta2, (double)o->step)));
  }
  for (const T3& x : t)
    if (x.n) HBP_TRY(launch_optim(d->dtype, adamw ? 1 : 0, x.w, x.master, x.g, x.m, x.v, x.n, clip, a, s));
  return HBP_OK;
}

hbp_status hbp_train_step(const hbp_desc* d, int k, hbp_buffers* b, const void* target, float* loss_out,
                          const hbp_optim* o, hbp_optim_state* st, void* stream) {
  if (!b || !st) return HBP_E_NULL;
  if (st->struct_size != sizeof(hbp_optim_state)) return HBP_E_INVALID_ARG;
  HBP_RUN(hbp_forward(d, b, stream));
  HBP_RUN(hbp_loss_mse(d, b, target, const_cast<void*>(b->e), loss_out, st->scratch, st->scratch_bytes, stream));
  if (k < 0) HBP_RUN(hbp_exact_backward(d, b, stream));
  else HBP_RUN(hbp_backward(d, k, b, stream));
  HBP_RUN(hbp_param_grads(d, b, stream));
  return hbp_optimizer_step(d, b, o, st, stream);
}

}  // extern "C"
