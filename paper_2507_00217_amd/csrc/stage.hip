// Host side of the pipeline-stage engine: configuration checks, parameter and
// stash layout, the microbatch state machine / schedule validator, the stash
// slot allocator with its cap, and the executor that turns F / B / W ops into
// kernel launches on one stream (no host synchronisation inside a schedule).
//
// Block decomposition: paper section 3.1 and Appendix B.  Stash lifetime
// (cached in F, released after B and W): section 3.2.  Cap on live stashes:
// the on-device memory constraint of section 4.1.
#include "../../include/stage.h"
#include "common.h"

#include <memory>
#include <new>
#include <vector>

using namespace stg;

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

struct Dims {
  int L, d, h, hkv, hd, da, dkv, dq, f, fin, s, b, T, n_mb, cap, n_sub;   // da = h*hd: width of the attention output
  int rope;              // rotary position embedding on
  int bias;              // linear maps carry biases
  int recompute, hcap;   // layer-wise recomputation on; cap on microbatches holding a rebuilt stash (B started, W not finished)
  size_t es;  // bytes per element of the compute dtype
};

bool make_dims(const stage_config_t* c, Dims* o) {
  if (!c) return false;
  if (c->n_layers < 1 || c->hidden < 64 || c->n_heads < 1 || c->n_kv_heads < 1 || c->ffn < 64 || c->seq < 1 ||
      c->mb_size < 1 || c->n_microbatches < 1)
    return false;
  if (c->hidden % 64 || c->ffn % 64 || c->n_heads % c->n_kv_heads) return false;
  if (c->head_dim < 0 || (c->head_dim == 0 && c->hidden % c->n_heads)) return false;
  const int hd = c->head_dim ? c->head_dim : c->hidden / c->n_heads;
  if (hd != 64 && hd != 128) return false;
  if ((int64_t)c->n_heads * hd > (1 << 20)) return false;
  if (c->norm != STAGE_NORM_LAYERNORM && c->norm != STAGE_NORM_RMSNORM) return false;
  if (c->act != STAGE_ACT_GELU && c->act != STAGE_ACT_SWIGLU) return false;
  if (c->dtype != STAGE_DTYPE_FP32 && c->dtype != STAGE_DTYPE_BF16) return false;
  if (c->causal != 0 && c->causal != 1) return false;
  if (c->stash_cap < 0 || c->stash_cap > c->n_microbatches) return false;
  if (!(c->norm_eps >= 0.f) || !(c->rope_theta >= 0.f)) return false;
  if (c->n_sub < 0 || c->n_sub > 32 || (c->n_sub > 0 && c->n_layers % c->n_sub)) return false;
  if ((c->recompute != 0 && c->recompute != 1) || c->recompute_cap < 0 || c->recompute_cap > c->n_microbatches) return false;
  if (!c->recompute && c->recompute_cap) return false;
  if (c->bias != 0 && c->bias != 1) return false;
  const size_t es = c->dtype == STAGE_DTYPE_FP32 ? 4 : 2;
  if (c->hidden > 256 * 4 * (int)(16 / es)) return false;  // one norm row must fit a workgroup's registers
  if ((int64_t)c->seq * c->mb_size > (1 << 20) || c->seq > 65536) return false;
  o->L = c->n_layers; o->d = c->hidden; o->h = c->n_heads; o->hkv = c->n_kv_heads; o->hd = hd;
  o->da = c->n_heads * hd; o->dkv = c->n_kv_heads * hd; o->dq = o->da + 2 * o->dkv; o->f = c->ffn;
  o->fin = c->act == STAGE_ACT_SWIGLU ? 2 * c->ffn : c->ffn;
  o->s = c->seq; o->b = c->mb_size; o->T = c->seq * c->mb_size; o->n_mb = c->n_microbatches;
  o->cap = c->stash_cap ? c->stash_cap : c->n_microbatches;
  o->n_sub = c->n_sub > 0 ? c->n_sub : 1;
  o->rope = c->rope_theta > 0.f;
  o->bias = c->bias;
  o->recompute = c->recompute;
  o->hcap = !c->recompute ? 0 : (c->recompute_cap ? c->recompute_cap : o->cap);
  if (o->hcap > o->cap) return false;   // a microbatch with a rebuilt stash is also live
  o->es = es;
  return true;
}

// --- parameter layout (elements) -------------------------------------------
void param_dims(const Dims& D, int norm, int pid, int64_t* rows, int64_t* cols) {
  switch (pid) {
    case STAGE_P_NORM1_GAMMA: case STAGE_P_NORM2_GAMMA: *rows = 1; *cols = D.d; break;
    case STAGE_P_NORM1_BETA: case STAGE_P_NORM2_BETA:
      if (norm == STAGE_NORM_LAYERNORM) { *rows = 1; *cols = D.d; } else { *rows = 0; *cols = 0; }
      break;
    case STAGE_P_WQKV: *rows = D.d; *cols = D.dq; break;
    case STAGE_P_WO: *rows = D.da; *cols = D.d; break;
    case STAGE_P_WIN: *rows = D.d; *cols = D.fin; break;
    case STAGE_P_WOUT: *rows = D.f; *cols = D.d; break;
    case STAGE_P_BQKV: *rows = D.bias; *cols = D.bias ? D.dq : 0; break;
    case STAGE_P_BO: case STAGE_P_BOUT: *rows = D.bias; *cols = D.bias ? D.d : 0; break;
    case STAGE_P_BIN: *rows = D.bias; *cols = D.bias ? D.fin : 0; break;
    default: *rows = 0; *cols = 0;
  }
}

size_t layer_param_elems(const Dims& D, int norm) {
  size_t n = 0;
  for (int p = 0; p < STAGE_P_COUNT; ++p) { int64_t r, c; param_dims(D, norm, p, &r, &c); n += (size_t)(r * c); }
  return n;
}

size_t param_offset(const Dims& D, int norm, int layer, int pid) {
  size_t off = (size_t)layer * layer_param_elems(D, norm);
  for (int p = 0; p < pid; ++p) { int64_t r, c; param_dims(D, norm, p, &r, &c); off += (size_t)(r * c); }
  return off;
}

// --- stash slot layout (bytes) ----------------------------------------------
// The residual stream (x, x1 going forward; dx1, dx coming back, written in place over them) is kept in fp32
// whatever the compute dtype: in bf16 it would be rounded twice per layer in each direction and those roundings
// dominate the stage's error.  GEMM operands derived from it (dyb, dx1b) are stored in the compute dtype.
//
// Without recomputation a slot is L such layer records and lives from F to W.  With layer-wise recomputation
// (section 7.2, Case 2) the layer inputs x live apart, in a small slot of L fp32 [T, d] tensors held from F to W;
// everything else is a layer record without x: F runs every layer through one such record in the workspace and
// keeps nothing of it, B rebuilds it layer by layer (forward again, minus the last GEMM, whose output is the
// next layer's stashed x) into a big slot that is held from the microbatch's first B sub-block to its last W.
struct LayerOff { size_t x, n1, qkv, dqkv, o, x1, n2, z, a, dyb, dx1b, st1, st2, lse, end; };

LayerOff layer_off(const Dims& D, size_t base, bool with_x = true) {
  LayerOff o; size_t p = base;
  const size_t T = D.T;
  auto take = [&](size_t bytes) { size_t r = p; p += up(bytes); return r; };
  o.x = take(with_x ? T * D.d * sizeof(float) : 0);
  o.n1 = take(T * D.d * D.es);
  o.qkv = take(T * D.dq * D.es);
  o.dqkv = take(T * D.dq * D.es);
  o.o = take(T * D.da * D.es);
  o.x1 = take(T * D.d * sizeof(float));
  o.n2 = take(T * D.d * D.es);
  o.z = take(T * D.fin * D.es);
  o.a = take(T * D.f * D.es);
  o.dyb = take(T * D.d * D.es);
  o.dx1b = take(T * D.d * D.es);
  o.st1 = take(T * 2 * sizeof(float));
  o.st2 = take(T * 2 * sizeof(float));
  o.lse = take((size_t)D.b * D.h * D.s * sizeof(float));
  o.end = p;
  return o;
}

size_t x_bytes(const Dims& D) { return up((size_t)D.T * D.d * sizeof(float)); }
size_t rec_bytes(const Dims& D) { return layer_off(D, 0, !D.recompute).end; }        // one layer record
// slot held from F to W, and (recomputation only) the slot held from B to W
size_t slot_bytes(const Dims& D) { return (D.recompute ? x_bytes(D) : rec_bytes(D)) * D.L; }
size_t big_slot_bytes(const Dims& D) { return D.recompute ? rec_bytes(D) * D.L : 0; }
size_t stash_bytes(const Dims& D) { return slot_bytes(D) * D.cap + big_slot_bytes(D) * D.hcap; }

struct WsOff { size_t da, dn, delta, partial, rec, dkvp, rope, bpart, end; };
WsOff ws_off(const Dims& D) {
  WsOff w; size_t p = 0;
  auto take = [&](size_t bytes) { size_t r = p; p += up(bytes); return r; };
  w.da = take((size_t)D.T * D.f * D.es);
  w.dn = take((size_t)D.T * (D.d > D.da ? D.d : D.da) * D.es);
  w.delta = take((size_t)D.b * D.h * D.s * sizeof(float));
  w.partial = take((size_t)norm_partial_rows() * 2 * D.d * sizeof(float));
  w.rec = take(D.recompute ? rec_bytes(D) : 0);       // the layer record F works in under recomputation
  w.dkvp = take(D.es == 2 ? attn_bwd_part_bytes(D.b, D.s, D.h, D.hkv, D.hd) : 0);   // grouped-query dK/dV partials
  w.rope = take(D.rope ? (size_t)D.s * (D.hd / 2) * 2 * sizeof(float) : 0);          // (cos, sin) per position and pair
  w.bpart = take(D.bias ? bias_grad_partial_bytes(D.fin > D.dq ? (D.fin > D.d ? D.fin : D.d) : (D.dq > D.d ? D.dq : D.d)) : 0);
  w.end = p;
  return w;
}

// --- microbatch state machine ------------------------------------------------
struct Tracker {
  // per microbatch: forward sub-blocks done (0..n_sub, in layer order), backward-input sub-blocks done (0..n_sub, in
  // reverse layer order), and a bit per sub-block whose weight gradients are done
  std::vector<int8_t> nf, nb;
  std::vector<uint32_t> wmask;
  int n_sub = 1;
  int live = 0, peak = 0;
  int hlive = 0, hpeak = 0;       // microbatches between their first B sub-block and their last W
  std::vector<int> last;          // [kind][sub] -> last microbatch that ran it in this iteration
  int cap = 0, hcap = 0, enforce = 0;   // hcap 0: no limit on hlive (no recomputation)
  int ext_live = 0, ext_hlive = 0;      // live microbatches of the other model chunks that share this stash
  size_t slot_b = 0, big_b = 0, peak_b = 0;   // bytes per slot of either kind, peak bytes in use

  void init(const Dims& D, int enforce_) {
    nf.assign(D.n_mb, 0); nb.assign(D.n_mb, 0); wmask.assign(D.n_mb, 0);
    n_sub = D.n_sub; cap = D.cap; hcap = D.hcap; enforce = enforce_; live = peak = hlive = hpeak = 0;
    slot_b = slot_bytes(D); big_b = big_slot_bytes(D); peak_b = 0;
    last.assign(3 * n_sub, -1);
  }
  void note_bytes() { const size_t b = (live + ext_live) * slot_b + (hlive + ext_hlive) * big_b; if (b > peak_b) peak_b = b; }
  bool waits(int m, int kind, int sub) const {       // microbatch m could run (kind, sub) right now
    if (kind == STAGE_B) return nf[m] == n_sub && sub == n_sub - 1 - nb[m];
    if (kind == STAGE_W) return sub >= n_sub - nb[m] && !(wmask[m] >> sub & 1);
    return false;
  }
  // One sub-block op. Returns STAGE_OK and applies it, or an error and leaves the state unchanged.
  //   F(mb,s): s-th group of layers, s = 0,1,..  in order; the first one takes a stash slot
  //   B(mb,s): after every F of mb; s = n_sub-1 down to 0; under recomputation the first one takes a big slot
  //   W(mb,s): after B(mb,s); any order; the last one releases the slot
  int step_sub(int kind, int mb, int sub) {
    if (kind < STAGE_F || kind > STAGE_W || mb < 0 || mb >= (int)nf.size() || sub < 0 || sub >= n_sub) return STAGE_E_INVAL;
    if (kind == STAGE_F) { if (sub != nf[mb] || nb[mb] != 0 || wmask[mb] != 0) return STAGE_E_ORDER; }
    else if (!waits(mb, kind, sub)) return STAGE_E_ORDER;
    if (enforce) {   // same (kind, sub) in increasing microbatch index: none skipped, none out of order
      if (mb <= last[kind * n_sub + sub]) return STAGE_E_ORDER;
      if (kind != STAGE_F)
        for (int m = 0; m < mb; ++m)
          if (waits(m, kind, sub)) return STAGE_E_ORDER;
    }
    if (kind == STAGE_F && sub == 0 && live + ext_live >= cap) return STAGE_E_STASH_FULL;
    if (kind == STAGE_B && nb[mb] == 0 && hcap > 0 && hlive + ext_hlive >= hcap) return STAGE_E_STASH_FULL;
    last[kind * n_sub + sub] = mb;
    if (kind == STAGE_F) { if (sub == 0) { ++live; if (live > peak) peak = live; note_bytes(); } ++nf[mb]; }
    else if (kind == STAGE_B) { if (nb[mb] == 0) { ++hlive; if (hlive > hpeak) hpeak = hlive; note_bytes(); } ++nb[mb]; }
    else {
      wmask[mb] |= 1u << sub;
      if (wmask[mb] == (n_sub >= 32 ? 0xFFFFFFFFu : (1u << n_sub) - 1)) {          // microbatch complete: back to EMPTY
        nf[mb] = nb[mb] = 0; wmask[mb] = 0;
        --hlive;
        if (--live == 0) std::fill(last.begin(), last.end(), -1);                    // iteration boundary
      }
    }
    return STAGE_OK;
  }
  // A whole op = its sub-blocks in their natural order, all or nothing.
  int step(int kind, int mb) {
    if (n_sub == 1) return step_sub(kind, mb, 0);
    Tracker t = *this;
    for (int i = 0; i < n_sub; ++i) {
      const int rc = t.step_sub(kind, mb, kind == STAGE_B ? n_sub - 1 - i : i);
      if (rc != STAGE_OK) return rc;
    }
    *this = t;
    return STAGE_OK;
  }
  bool slot_held(int mb) const { return nf[mb] > 0; }
  bool big_held(int mb) const { return nb[mb] > 0; }
};

}  // namespace

// Slot allocator and occupancy of one stash, shared by the model chunks that live on it.
struct StashPool {
  std::vector<int> free_slots, free_big;
  int live = 0, hlive = 0, peak = 0;
  size_t peak_b = 0;
};

struct stage {
  stage_config_t cfg;
  Dims D;
  DType dt;
  char* weights; float* grads; char* stash; char* ws;
  hipStream_t stream;
  size_t slot_sz, big_sz, n_param_elems;
  Tracker tr;
  std::vector<int> slot_of, big_of;      // microbatch -> slot index of either kind, -1 if none
  std::shared_ptr<StashPool> pool;
  int sticky = STAGE_OK;
  int kernel_set = 0;
  // optional per-launch timing (HIP events on the stage's stream), by kernel class
  struct ProfRec { int cls; hipEvent_t t0, t1; double work; };
  bool profiling = false;
  std::vector<ProfRec> prof;
  std::vector<hipEvent_t> event_pool;
};

namespace {

struct LayerW { const char *g1, *b1, *wqkv, *wo, *g2, *b2, *win, *wout, *bqkv, *bo, *bin, *bout; float *G[STAGE_P_COUNT]; };

LayerW layer_weights(const stage* st, int l) {
  LayerW w;
  const char** slots[STAGE_P_COUNT] = {&w.g1, &w.b1, &w.wqkv, &w.wo, &w.g2, &w.b2, &w.win, &w.wout, &w.bqkv, &w.bo, &w.bin, &w.bout};
  for (int p = 0; p < STAGE_P_COUNT; ++p) {
    int64_t r, c; param_dims(st->D, st->cfg.norm, p, &r, &c);
    const size_t off = param_offset(st->D, st->cfg.norm, l, p);
    *slots[p] = (r * c) ? st->weights + off * st->D.es : nullptr;
    w.G[p] = (r * c) ? st->grads + off : nullptr;
  }
  return w;
}

struct ProfScope {
  stage* st; size_t idx; bool on;
  ProfScope(stage* s, int cls, double work) : st(s), idx(0), on(s->profiling) {
    if (!on) return;
    auto get = [&]() { hipEvent_t e; if (st->event_pool.empty()) { if (hipEventCreate(&e) != hipSuccess) e = nullptr; } else { e = st->event_pool.back(); st->event_pool.pop_back(); } return e; };
    stage::ProfRec r{cls, get(), get(), work};
    if (!r.t0 || !r.t1) { on = false; return; }
    (void)hipEventRecord(r.t0, st->stream);
    idx = st->prof.size();
    st->prof.push_back(r);
  }
  ~ProfScope() { if (on) (void)hipEventRecord(st->prof[idx].t1, st->stream); }
};

#define HIPCHK(expr) do { hipError_t e__ = (expr); if (e__ != hipSuccess) { st->sticky = STAGE_E_HIP; return STAGE_E_HIP; } } while (0)

double act_bytes_fwd(const stage* st) { return (double)st->D.T * (st->D.fin + st->D.f) * st->D.es; }
// bytes moved by a norm kernel: fp32 (residual-stream) tensors and compute-dtype tensors it reads or writes
double norm_bytes(const stage* st, int n_f32, int n_lp) { return (double)st->D.T * st->D.d * (4.0 * n_f32 + (double)st->D.es * n_lp); }
double attn_flops(const stage* st, bool bwd) {
  const Dims& D = st->D;
  const double dense = 4.0 * D.b * (double)D.s * D.s * D.da;
  return (st->cfg.causal ? 0.5 : 1.0) * dense * (bwd ? 2.5 : 1.0);
}

int do_gemm(stage* st, int mode, int M, int N, int K, const void* A, int64_t lda, const void* B, int64_t ldb,
            void* C, int64_t ldc, const void* R, int64_t ldr, int acc, int r_f32 = 0, int c_f32 = 0, const void* bias = nullptr) {
  GemmArgs g{mode, M, N, K, A, lda, B, ldb, C, ldc, R, ldr, acc, r_f32, c_f32};
  g.bias = bias;
  ProfScope ps(st, STAGE_K_GEMM_NN + mode, 2.0 * M * N * K);
  if (st->kernel_set == 0 && st->dt == DT_BF16 && gemm_mfma_supported(g)) HIPCHK(gemm_mfma(g, st->stream));
  else HIPCHK(gemm_ref(st->dt, g, st->stream));
  return STAGE_OK;
}

// FFN-in product with the activation fused into its epilogue: z = A.W and a = act(z) from the fp32 accumulators, in
// one kernel.  Returns false (nothing enqueued) when the tuned kernel does not take the shape or is switched off; the
// caller then runs the product and the activation kernel one after the other.
bool try_gemm_act(stage* st, int* rc, int M, int f, int K, const void* A, const void* W, const void* bias, void* z, void* a) {
  const int fin = st->cfg.act == STAGE_ACT_SWIGLU ? 2 * f : f;
  GemmArgs g{GEMM_NN, M, fin, K, A, (int64_t)K, W, (int64_t)fin, z, (int64_t)fin, nullptr, 0, 0, 0, 0};
  g.act = st->cfg.act == STAGE_ACT_SWIGLU ? 2 : 1; g.C2 = a; g.ldc2 = f; g.bias = bias;
  if (st->kernel_set != 0 || st->dt != DT_BF16 || !gemm_mfma_supported(g)) return false;
  ProfScope ps(st, STAGE_K_GEMM_NN, 2.0 * M * fin * K);
  *rc = STAGE_OK;
  if (gemm_mfma(g, st->stream) != hipSuccess) { st->sticky = STAGE_E_HIP; *rc = STAGE_E_HIP; }
  return true;
}

// The FFN-out map's input-gradient product with the activation backward fused into its epilogue: z becomes dz in place
// and da = dy.Wout^T never reaches memory.  False (nothing enqueued) when the tuned kernel does not apply.
bool try_gemm_act_bwd(stage* st, int* rc, int M, int f, int K, const void* dy, const void* W, void* z) {
  const int nop = st->cfg.act == STAGE_ACT_SWIGLU ? 2 : 1;
  GemmArgs g{GEMM_NT, M, f, K, dy, (int64_t)K, W, (int64_t)K, nullptr, (int64_t)f, nullptr, 0, 0, 0, 0};
  g.act_bwd = nop; g.Z = z; g.ldz = (int64_t)nop * f;
  if (st->kernel_set != 0 || st->dt != DT_BF16 || !gemm_mfma_supported(g)) return false;
  ProfScope ps(st, STAGE_K_GEMM_NT, 2.0 * M * f * K);
  *rc = STAGE_OK;
  if (gemm_mfma(g, st->stream) != hipSuccess) { st->sticky = STAGE_E_HIP; *rc = STAGE_E_HIP; }
  return true;
}

// Where one layer's tensors of one microbatch live.
struct LayerBuf { char *x, *n1, *qkv, *dqkv, *o, *x1, *n2, *z, *a, *dyb, *dx1b; float *st1, *st2, *lse; };

enum { REC_SLOT = 0, REC_WORKSPACE = 1 };

// `where`: REC_SLOT = the microbatch's stash (its big slot under recomputation); REC_WORKSPACE = the single
// layer record in the workspace that F uses under recomputation.  x always comes from the F-to-W slot.
LayerBuf layer_buf(const stage* st, int mb, int l, int where = REC_SLOT) {
  const Dims& D = st->D;
  char* slot = st->stash + (size_t)st->slot_of[mb] * st->slot_sz;
  char* rec;
  LayerBuf b;
  if (!D.recompute) {
    rec = slot + rec_bytes(D) * l;
    b.x = rec;
  } else {
    b.x = slot + x_bytes(D) * l;
    rec = where == REC_WORKSPACE ? st->ws + ws_off(D).rec
                                 : st->stash + st->slot_sz * D.cap + (size_t)st->big_of[mb] * st->big_sz + rec_bytes(D) * l;
  }
  const LayerOff o = layer_off(D, 0, !D.recompute);
  b.n1 = rec + o.n1; b.qkv = rec + o.qkv; b.dqkv = rec + o.dqkv; b.o = rec + o.o; b.x1 = rec + o.x1; b.n2 = rec + o.n2;
  b.z = rec + o.z; b.a = rec + o.a; b.dyb = rec + o.dyb; b.dx1b = rec + o.dx1b;
  b.st1 = (float*)(rec + o.st1); b.st2 = (float*)(rec + o.st2); b.lse = (float*)(rec + o.lse);
  return b;
}

AttnArgs attn_args(const stage* st, const LayerBuf& o, const void* dout, const WsOff& w) {
  const Dims& D = st->D;
  AttnArgs a{};
  a.b = D.b; a.s = D.s; a.h = D.h; a.hkv = D.hkv; a.hd = D.hd; a.causal = st->cfg.causal;
  a.qkv = o.qkv; a.ld = D.dq; a.o = o.o; a.lse = o.lse;
  a.dout = dout; a.dqkv = o.dqkv; a.delta = (float*)(st->ws + w.delta);
  a.dkv_part = w.dkvp != w.rope ? (float*)(st->ws + w.dkvp) : nullptr;
  return a;
}

// Forward of layer l through the record `o`.  y_l: where the layer's output goes (fp32 unless `y_lp`); nullptr
// skips the last GEMM, which is what rebuilding a record for B needs.
int forward_layer(stage* st, int l, const LayerBuf& o, void* y_l, bool y_lp) {
  const Dims& D = st->D;
  const LayerW W = layer_weights(st, l);
  const WsOff w = ws_off(D);
  NormArgs n{}; n.kind = st->cfg.norm; n.rows = D.T; n.d = D.d; n.eps = st->cfg.norm_eps; n.x_f32 = 1;
  n.x = o.x; n.gamma = W.g1; n.beta = W.b1; n.out = o.n1; n.stats = o.st1;
  { ProfScope ps(st, STAGE_K_NORM_FWD, norm_bytes(st, 1, 1)); HIPCHK(norm_fwd(st->dt, n, st->stream)); }
  int rc = do_gemm(st, GEMM_NN, D.T, D.dq, D.d, o.n1, D.d, W.wqkv, D.dq, o.qkv, D.dq, nullptr, 0, 0, 0, 0, W.bqkv);
  if (rc) return rc;
  if (D.rope) {      // q and k of the stash are the rotated ones: attention forward and backward both want those
    ProfScope ps(st, STAGE_K_ROPE, 2.0 * D.T * (D.da + D.dkv) * D.es);
    HIPCHK(rope_apply(st->dt, o.qkv, D.dq, D.T, D.s, D.h + D.hkv, D.hd, (const float*)(st->ws + w.rope), 0, st->stream));
  }
  AttnArgs a = attn_args(st, o, nullptr, w);
  {
    ProfScope ps(st, STAGE_K_ATTN_FWD, attn_flops(st, false));
    if (st->kernel_set == 0 && st->dt == DT_BF16 && attn_mfma_supported(a)) HIPCHK(attn_fwd_mfma(a, st->stream));
    else HIPCHK(attn_fwd_ref(st->dt, a, st->stream));
  }
  rc = do_gemm(st, GEMM_NN, D.T, D.d, D.da, o.o, D.da, W.wo, D.d, o.x1, D.d, o.x, D.d, 0, 1, 1, W.bo);
  if (rc) return rc;
  n.x = o.x1; n.gamma = W.g2; n.beta = W.b2; n.out = o.n2; n.stats = o.st2;
  { ProfScope ps(st, STAGE_K_NORM_FWD, norm_bytes(st, 1, 1)); HIPCHK(norm_fwd(st->dt, n, st->stream)); }
  if (try_gemm_act(st, &rc, D.T, D.f, D.d, o.n2, W.win, W.bin, o.z, o.a)) {
    if (rc) return rc;
  } else {
    rc = do_gemm(st, GEMM_NN, D.T, D.fin, D.d, o.n2, D.d, W.win, D.fin, o.z, D.fin, nullptr, 0, 0, 0, 0, W.bin);
    if (rc) return rc;
    ActArgs ac{}; ac.kind = st->cfg.act; ac.rows = D.T; ac.f = D.f; ac.z = o.z; ac.a = o.a;
    { ProfScope ps(st, STAGE_K_ACT_FWD, act_bytes_fwd(st)); HIPCHK(act_fwd(st->dt, ac, st->stream)); }
  }
  if (!y_l) return STAGE_OK;
  return do_gemm(st, GEMM_NN, D.T, D.d, D.f, o.a, D.f, W.wout, D.d, y_l, D.d, o.x1, D.d, 0, 1, y_lp ? 0 : 1, W.bout);
}

// layers [l0, l1): x is read when l0 == 0, y is written when l1 == L
int exec_forward(stage* st, int mb, const void* x, void* y, int l0, int l1) {
  const Dims& D = st->D;
  const size_t n_act = (size_t)D.T * D.d;
  if (l0 == 0) {
    ProfScope ps(st, STAGE_K_COPY, (double)n_act * (D.es + sizeof(float)));
    HIPCHK(widen_to_f32(st->dt, (float*)layer_buf(st, mb, 0, REC_WORKSPACE).x, x, n_act, st->stream));
  }
  for (int l = l0; l < l1; ++l) {
    const bool last = l + 1 == D.L;
    // the output is the next layer's fp32 x, or the caller's Y
    void* y_l = last ? y : (void*)layer_buf(st, mb, l + 1, REC_WORKSPACE).x;
    const int rc = forward_layer(st, l, layer_buf(st, mb, l, REC_WORKSPACE), y_l, last);
    if (rc) return rc;
  }
  return STAGE_OK;
}

// layers [l0, l1) in reverse: dy is read when l1 == L, dx is written when l0 == 0
int exec_backward_input(stage* st, int mb, const void* dy, void* dx, int l0, int l1) {
  const Dims& D = st->D;
  const WsOff w = ws_off(D);
  const size_t act_bytes = (size_t)D.T * D.d * D.es;
  if (l1 == D.L) {
    ProfScope ps(st, STAGE_K_COPY, 2.0 * act_bytes);
    HIPCHK(copy_bytes(layer_buf(st, mb, D.L - 1).dyb, dy, act_bytes, st->stream));
  }
  void* da = st->ws + w.da;
  void* dn = st->ws + w.dn;
  for (int l = l1 - 1; l >= l0; --l) {
    const LayerBuf o = layer_buf(st, mb, l);
    const LayerW W = layer_weights(st, l);
    const bool last = l + 1 == D.L;
    int rc;
    if (D.recompute && (rc = forward_layer(st, l, o, nullptr, false))) return rc;
    // gradient arriving at this layer's output: GEMM operand copy in the compute dtype, and the residual-branch
    // term, which is the fp32 dx the layer above left in its x region (the caller's dY for the last layer)
    const void* dy_op = o.dyb;
    const void* dy_res = last ? dy_op : (const void*)layer_buf(st, mb, l + 1).x;
    // bias gradients: column sums of the four dZ tensors, as each becomes available
    float* bpart = (float*)(st->ws + w.bpart);
    auto dbias = [&](const void* dz, int n, int pid) -> int {
      if (!D.bias) return STAGE_OK;
      ProfScope ps(st, STAGE_K_COPY, (double)D.T * n * D.es);
      HIPCHK(bias_grad(st->dt, dz, n, D.T, n, bpart, W.G[pid], st->stream));
      return STAGE_OK;
    };
    if ((rc = dbias(dy_op, D.d, STAGE_P_BOUT))) return rc;
    // FFN: da = dy.Wout^T ; dz = act'(z) * da (in place over z) ; dn2 = dz.Win^T
    if (try_gemm_act_bwd(st, &rc, D.T, D.f, D.d, dy_op, W.wout, o.z)) {
      if (rc) return rc;
    } else {
      rc = do_gemm(st, GEMM_NT, D.T, D.f, D.d, dy_op, D.d, W.wout, D.d, da, D.f, nullptr, 0, 0);
      if (rc) return rc;
      ActArgs ac{}; ac.kind = st->cfg.act; ac.rows = D.T; ac.f = D.f; ac.z = o.z; ac.da = da;
      { ProfScope ps(st, STAGE_K_ACT_BWD, (double)D.T * (2.0 * D.fin + D.f) * D.es); HIPCHK(act_bwd(st->dt, ac, st->stream)); }
    }
    if ((rc = dbias(o.z, D.fin, STAGE_P_BIN))) return rc;
    rc = do_gemm(st, GEMM_NT, D.T, D.d, D.fin, o.z, D.fin, W.win, D.fin, dn, D.d, nullptr, 0, 0);
    if (rc) return rc;
    // dx1 = dy + norm2'(dn2): fp32 in place over x1, plus a compute-dtype copy for the two GEMMs that read it
    NormArgs n{}; n.kind = st->cfg.norm; n.rows = D.T; n.d = D.d; n.eps = st->cfg.norm_eps;
    n.x = o.x1; n.x_f32 = 1; n.gamma = W.g2; n.out = o.x1; n.out_f32 = 1; n.out_lp = o.dx1b;
    n.stats = o.st2; n.dout = dn; n.resid = dy_res; n.resid_f32 = last ? 0 : 1;
    n.dgamma = W.G[STAGE_P_NORM2_GAMMA]; n.dbeta = W.G[STAGE_P_NORM2_BETA]; n.partial = (float*)(st->ws + w.partial);
    { ProfScope ps(st, STAGE_K_NORM_BWD, norm_bytes(st, last ? 2 : 3, last ? 3 : 2)); HIPCHK(norm_bwd(st->dt, n, st->stream)); }
    // attention: do = dx1.Wo^T ; (dq,dk,dv) ; dn1 = dqkv.Wqkv^T
    if ((rc = dbias(o.dx1b, D.d, STAGE_P_BO))) return rc;
    rc = do_gemm(st, GEMM_NT, D.T, D.da, D.d, o.dx1b, D.d, W.wo, D.d, dn, D.da, nullptr, 0, 0);
    if (rc) return rc;
    AttnArgs a = attn_args(st, o, dn, w);
    {
      ProfScope ps(st, STAGE_K_ATTN_BWD, attn_flops(st, true));
      if (st->kernel_set == 0 && st->dt == DT_BF16 && attn_mfma_supported(a)) HIPCHK(attn_bwd_mfma(a, st->stream));
      else HIPCHK(attn_bwd_ref(st->dt, a, st->stream));
    }
    if (D.rope) {    // gradients with respect to the unrotated q and k: the transposed rotation
      ProfScope ps(st, STAGE_K_ROPE, 2.0 * D.T * (D.da + D.dkv) * D.es);
      HIPCHK(rope_apply(st->dt, o.dqkv, D.dq, D.T, D.s, D.h + D.hkv, D.hd, (const float*)(st->ws + w.rope), 1, st->stream));
    }
    if ((rc = dbias(o.dqkv, D.dq, STAGE_P_BQKV))) return rc;
    rc = do_gemm(st, GEMM_NT, D.T, D.d, D.dq, o.dqkv, D.dq, W.wqkv, D.dq, dn, D.d, nullptr, 0, 0);
    if (rc) return rc;
    // dx = dx1 + norm1'(dn1): layer 0 hands it to the caller; otherwise fp32 in place over x (the residual term of
    // the layer below) plus the compute-dtype copy the layer below uses as its dy operand
    n.x = o.x; n.gamma = W.g1; n.stats = o.st1; n.dout = dn; n.resid = o.x1; n.resid_f32 = 1;
    n.dgamma = W.G[STAGE_P_NORM1_GAMMA]; n.dbeta = W.G[STAGE_P_NORM1_BETA];
    if (l == 0) { n.out = dx; n.out_f32 = 0; n.out_lp = nullptr; }
    else { n.out = o.x; n.out_f32 = 1; n.out_lp = layer_buf(st, mb, l - 1).dyb; }
    { ProfScope ps(st, STAGE_K_NORM_BWD, norm_bytes(st, l == 0 ? 2 : 3, 2)); HIPCHK(norm_bwd(st->dt, n, st->stream)); }
  }
  return STAGE_OK;
}

// A list of weight-gradient products, each reducing over nseg operand pairs in turn (pair s = the list's A and B
// moved by seg_delta[s] bytes): one launch of persistent workgroups when the tuned kernel takes all of them, else
// product by product and pair by pair -- the same accumulation order, hence the same bits.
hipError_t wgrad_list(DType dt, int kernel_set, const GemmArgs* list, int n, int nseg, const int64_t* seg_delta, hipStream_t s) {
  if (n == 0) return hipSuccess;
  if (kernel_set == 0 && dt == DT_BF16 && gemm_mfma_wgrad_group_supported(list, n, nseg, seg_delta))
    return gemm_mfma_wgrad_group(list, n, nseg, seg_delta, s);
  for (int sg = 0; sg < nseg; ++sg)
    for (int i = 0; i < n; ++i) {
      GemmArgs g = list[i];
      if (sg > 0) { g.A = (const char*)g.A + seg_delta[sg]; g.B = (const char*)g.B + seg_delta[sg]; }
      hipError_t e = (kernel_set == 0 && dt == DT_BF16 && gemm_mfma_supported(g)) ? gemm_mfma(g, s) : gemm_ref(dt, g, s);
      if (e != hipSuccess) return e;
    }
  return hipSuccess;
}

// W of layers [l0, l1) for the microbatches mbs[0..n_mb), in that order.  The four weight-gradient products of every
// layer do not depend on each other and go out as one list; the same product of successive microbatches becomes one
// reduction over their operand pairs (every tensor of a microbatch sits at the same offset inside its stash slot, so
// one byte offset per microbatch places all its operands), which reads and writes the fp32 gradients once.
int exec_backward_weight(stage* st, const int* mbs, int n_mb, int l0, int l1) {
  const Dims& D = st->D;
  std::vector<GemmArgs> list;
  list.reserve((size_t)4 * (l1 - l0));
  double flops = 0.0;
  auto add = [&](int M, int N, const void* A, int64_t lda, const void* B, int64_t ldb, float* C) {
    list.push_back(GemmArgs{GEMM_TN, M, N, D.T, A, lda, B, ldb, C, (int64_t)N, nullptr, 0, 1, 0, 0});
    flops += 2.0 * M * N * D.T * n_mb;
  };
  for (int l = l0; l < l1; ++l) {
    const LayerBuf o = layer_buf(st, mbs[0], l);
    const LayerW W = layer_weights(st, l);
    add(D.d, D.dq, o.n1, D.d, o.dqkv, D.dq, W.G[STAGE_P_WQKV]);
    add(D.da, D.d, o.o, D.da, o.dx1b, D.d, W.G[STAGE_P_WO]);
    add(D.d, D.fin, o.n2, D.d, o.z, D.fin, W.G[STAGE_P_WIN]);
    add(D.f, D.d, o.a, D.f, o.dyb, D.d, W.G[STAGE_P_WOUT]);
  }
  int64_t delta[GEMM_MAX_SEG] = {0};
  for (int i = 1; i < n_mb; ++i) delta[i] = layer_buf(st, mbs[i], l0).n1 - layer_buf(st, mbs[0], l0).n1;
  ProfScope ps(st, STAGE_K_GEMM_TN, flops);
  HIPCHK(wgrad_list(st->dt, st->kernel_set, list.data(), (int)list.size(), n_mb, delta, st->stream));
  return STAGE_OK;
}

void release_slots(stage* st, int mb) {
  st->pool->free_slots.push_back(st->slot_of[mb]);
  st->slot_of[mb] = -1;
  if (st->big_of[mb] >= 0) { st->pool->free_big.push_back(st->big_of[mb]); st->big_of[mb] = -1; }
}

// Applies one already-validated op (sub < 0: the whole op, every sub-block): allocator bookkeeping + launches.
// `had_slot` / `holds_slot`: whether the microbatch held a stash slot before / holds one after the op.
int apply_op(stage* st, int kind, int mb, int sub, bool had_slot, bool holds_slot, const void* in, void* out) {
  const int per = st->D.L / st->D.n_sub;
  const int l0 = sub < 0 ? 0 : sub * per, l1 = sub < 0 ? st->D.L : (sub + 1) * per;
  int rc = STAGE_OK;
  if (kind == STAGE_F) {
    if (!had_slot) {
      st->slot_of[mb] = st->pool->free_slots.back();
      st->pool->free_slots.pop_back();
    }
    rc = exec_forward(st, mb, in, out, l0, l1);
  } else if (kind == STAGE_B) {
    if (st->D.recompute && st->big_of[mb] < 0) {
      st->big_of[mb] = st->pool->free_big.back();
      st->pool->free_big.pop_back();
    }
    rc = exec_backward_input(st, mb, in, out, l0, l1);
  } else {
    rc = exec_backward_weight(st, &mb, 1, l0, l1);
    if (!holds_slot) release_slots(st, mb);
  }
  return rc;
}

// The tracker counts its own chunk; what the other chunks on the same stash hold comes from the pool.
void pull_pool(stage* st, Tracker& t) {
  t.ext_live = st->pool->live - st->tr.live;
  t.ext_hlive = st->pool->hlive - st->tr.hlive;
  if (st->pool->peak_b > t.peak_b) t.peak_b = st->pool->peak_b;
}
void push_pool(stage* st) {
  StashPool& p = *st->pool;
  p.live = st->tr.live + st->tr.ext_live;
  p.hlive = st->tr.hlive + st->tr.ext_hlive;
  if (p.live > p.peak) p.peak = p.live;
  if (st->tr.peak_b > p.peak_b) p.peak_b = st->tr.peak_b;
}
int step_tracked(stage* st, int kind, int mb, int sub) {
  pull_pool(st, st->tr);
  const int rc = sub < 0 ? st->tr.step(kind, mb) : st->tr.step_sub(kind, mb, sub);
  if (rc == STAGE_OK) push_pool(st);
  return rc;
}

// validate + apply one op against the stage's tracker
int run_one(stage* st, int kind, int mb, int sub, const void* in, void* out) {
  if (mb < 0 || mb >= st->D.n_mb) return STAGE_E_INVAL;
  const bool had = st->tr.slot_held(mb);
  const int rc = step_tracked(st, kind, mb, sub);
  if (rc != STAGE_OK) return rc;
  return apply_op(st, kind, mb, sub, had, st->tr.slot_held(mb), in, out);
}

// shared body of the two schedule runners: op i is (kind(i), mb(i), sub(i)), sub < 0 meaning a whole op
// Probes a list spread over the model chunks of one stash: every chunk's tracker is stepped on a copy, with the
// other chunks' live counts kept up to date, so caps that the chunks share are checked across them.
// get(i, chunk, kind, mb, sub); returns the first error and its position.
template <typename GetOp>
int probe_list(stage* const* chunks, int n_chunks, int n_ops, GetOp get, int* bad) {
  std::vector<Tracker> probe(n_chunks);
  int live = chunks[0]->pool->live, hlive = chunks[0]->pool->hlive;
  for (int c = 0; c < n_chunks; ++c) probe[c] = chunks[c]->tr;
  for (int i = 0; i < n_ops; ++i) {
    int c, kind, mb, sub; get(i, c, kind, mb, sub);
    if (bad) *bad = i;
    if (c < 0 || c >= n_chunks) return STAGE_E_INVAL;
    Tracker& t = probe[c];
    t.ext_live = live - t.live; t.ext_hlive = hlive - t.hlive;
    const int rc = sub < 0 ? t.step(kind, mb) : t.step_sub(kind, mb, sub);
    if (rc != STAGE_OK) return rc;
    live = t.live + t.ext_live; hlive = t.hlive + t.ext_hlive;
  }
  if (bad) *bad = -1;
  return STAGE_OK;
}

// Shared body of the schedule runners: op i is (chunk(i), kind(i), mb(i), sub(i)), sub < 0 meaning a whole op; chunk c
// reads and writes the boundary tensors x_all[c] ... dx_all[c].
template <typename GetOp>
int run_list(stage* const* chunks, int n_chunks, int n_ops, GetOp get, const void* const* x_all, const void* const* dy_all,
             void* const* y_all, void* const* dx_all) {
  // validate the whole list before enqueuing anything
  for (int i = 0; i < n_ops; ++i) {
    int c, kind, mb, sub; get(i, c, kind, mb, sub);
    if (c < 0 || c >= n_chunks) return STAGE_E_INVAL;
    const int ns = chunks[c]->D.n_sub;
    if (kind == STAGE_F && ((sub <= 0 && !x_all[c]) || ((sub < 0 || sub == ns - 1) && !y_all[c]))) return STAGE_E_INVAL;
    if (kind == STAGE_B && (((sub < 0 || sub == ns - 1) && !dy_all[c]) || (sub <= 0 && !dx_all[c]))) return STAGE_E_INVAL;
  }
  { const int rc = probe_list(chunks, n_chunks, n_ops, get, nullptr); if (rc != STAGE_OK) return rc; }
  // Adjacent W ops on the same layers of the same chunk (same sub-block, or whole ops) are enqueued as one: their
  // microbatches, in list order, become the K segments of one set of weight-gradient products.  The tracker still sees
  // them one by one; the stash slots are handed back when the merged launch has been enqueued.
  stage* run_st = nullptr;
  int run_mb[GEMM_MAX_SEG], run_n = 0, run_sub = 0;
  bool run_release[GEMM_MAX_SEG];
  auto flush = [&]() -> int {
    if (run_n == 0) return STAGE_OK;
    const int per = run_st->D.L / run_st->D.n_sub;
    const int l0 = run_sub < 0 ? 0 : run_sub * per, l1 = run_sub < 0 ? run_st->D.L : (run_sub + 1) * per;
    const int rc = exec_backward_weight(run_st, run_mb, run_n, l0, l1);
    for (int i = 0; i < run_n; ++i)
      if (run_release[i]) release_slots(run_st, run_mb[i]);
    run_n = 0;
    return rc;
  };
  for (int i = 0; i < n_ops; ++i) {
    int c, kind, mb, sub; get(i, c, kind, mb, sub);
    stage* st = chunks[c];
    if (kind == STAGE_W) {
      if (run_n > 0 && (st != run_st || sub != run_sub || run_n == GEMM_MAX_SEG)) { const int rc = flush(); if (rc != STAGE_OK) return rc; }
      const int rc = step_tracked(st, kind, mb, sub);
      if (rc != STAGE_OK) { flush(); return rc; }
      run_st = st; run_sub = sub; run_mb[run_n] = mb; run_release[run_n] = !st->tr.slot_held(mb); ++run_n;
      continue;
    }
    { const int rc = flush(); if (rc != STAGE_OK) return rc; }
    const size_t mb_bytes = (size_t)st->D.T * st->D.d * st->D.es;
    const void* in = kind == STAGE_F ? (const char*)x_all[c] + mb_bytes * mb : (const char*)dy_all[c] + mb_bytes * mb;
    void* out = kind == STAGE_F ? (char*)y_all[c] + mb_bytes * mb : (char*)dx_all[c] + mb_bytes * mb;
    const int rc = run_one(st, kind, mb, sub, in, out);
    if (rc != STAGE_OK) return rc;
  }
  return flush();
}

int init_stage(const stage_config_t* cfg, void* weights_dev, void* grads_dev, void* stash_dev, void* workspace_dev,
               void* hip_stream, stage* share_with, stage_t** out) {
  Dims D;
  if (!out) return STAGE_E_INVAL;
  *out = nullptr;
  if (!make_dims(cfg, &D) || !weights_dev || !grads_dev || !stash_dev || !workspace_dev) return STAGE_E_INVAL;
  if (((uintptr_t)weights_dev | (uintptr_t)grads_dev | (uintptr_t)stash_dev | (uintptr_t)workspace_dev) % ALIGN)
    return STAGE_E_INVAL;
  if (share_with) {   // chunks of one stash: same slot geometry and caps
    const Dims& S = share_with->D;
    if (slot_bytes(D) != slot_bytes(S) || big_slot_bytes(D) != big_slot_bytes(S) || D.cap != S.cap || D.hcap != S.hcap ||
        D.recompute != S.recompute)
      return STAGE_E_INVAL;
    // A workspace may be common to the chunks only if this chunk fits into it and finds the same rotary table there
    // (it is written at init): same offsets, same table.  A chunk of another shape brings its own workspace.
    if (workspace_dev == (void*)share_with->ws &&
        (ws_off(D).end > ws_off(S).end || ws_off(D).rope != ws_off(S).rope || D.rope != S.rope || D.s != S.s || D.hd != S.hd ||
         cfg->rope_theta != share_with->cfg.rope_theta))
      return STAGE_E_INVAL;
  }
  stage* st = new (std::nothrow) stage();
  if (!st) return STAGE_E_INVAL;
  st->cfg = *cfg; st->D = D; st->dt = cfg->dtype == STAGE_DTYPE_FP32 ? DT_F32 : DT_BF16;
  st->weights = (char*)weights_dev; st->grads = (float*)grads_dev; st->stash = (char*)stash_dev; st->ws = (char*)workspace_dev;
  st->stream = (hipStream_t)hip_stream;
  st->slot_sz = slot_bytes(D); st->big_sz = big_slot_bytes(D);
  st->n_param_elems = layer_param_elems(D, cfg->norm) * D.L;
  st->tr.init(D, cfg->enforce_mb_order);
  st->slot_of.assign(D.n_mb, -1); st->big_of.assign(D.n_mb, -1);
  if (share_with) {
    st->pool = share_with->pool;
  } else {
    st->pool = std::make_shared<StashPool>();
    for (int i = D.cap - 1; i >= 0; --i) st->pool->free_slots.push_back(i);
    for (int i = D.hcap - 1; i >= 0; --i) st->pool->free_big.push_back(i);
  }
  if (fill_zero_f32(st->grads, st->n_param_elems, st->stream) != hipSuccess) { delete st; return STAGE_E_HIP; }
  if (D.rope && rope_table((float*)(st->ws + ws_off(D).rope), D.s, D.hd, (double)cfg->rope_theta, st->stream) != hipSuccess) {
    delete st;
    return STAGE_E_HIP;
  }
  *out = st;
  return STAGE_OK;
}

}  // namespace

extern "C" {

int stage_query_sizes(const stage_config_t* cfg, stage_sizes_t* out) {
  Dims D;
  if (!out || !make_dims(cfg, &D)) return STAGE_E_INVAL;
  const size_t n = layer_param_elems(D, cfg->norm) * D.L;
  out->weights = up(n * D.es);
  out->grads = up(n * sizeof(float));
  out->stash = stash_bytes(D);
  out->workspace = ws_off(D).end;
  return STAGE_OK;
}

int stage_validate_schedule(const stage_config_t* cfg, const stage_op_t* ops, int n_ops, int* first_bad_index,
                            int* peak_live) {
  Dims D;
  if (first_bad_index) *first_bad_index = -1;
  if (peak_live) *peak_live = 0;
  if (!make_dims(cfg, &D) || n_ops < 0 || (n_ops > 0 && !ops)) return STAGE_E_INVAL;
  Tracker t; t.init(D, cfg->enforce_mb_order);
  for (int i = 0; i < n_ops; ++i) {
    const int rc = t.step(ops[i].kind, ops[i].mb);
    if (rc != STAGE_OK) {
      if (first_bad_index) *first_bad_index = i;
      if (peak_live) *peak_live = t.peak;
      return rc;
    }
  }
  if (peak_live) *peak_live = t.peak;
  return STAGE_OK;
}

int stage_param_layout(const stage_config_t* cfg, int layer, int param_id, size_t* offset_elems, int64_t* rows,
                       int64_t* cols) {
  Dims D;
  if (!make_dims(cfg, &D) || layer < 0 || layer >= D.L || param_id < 0 || param_id >= STAGE_P_COUNT || !offset_elems ||
      !rows || !cols)
    return STAGE_E_INVAL;
  param_dims(D, cfg->norm, param_id, rows, cols);
  *offset_elems = param_offset(D, cfg->norm, layer, param_id);
  return STAGE_OK;
}

int stage_init(const stage_config_t* cfg, void* weights_dev, void* grads_dev, void* stash_dev, void* workspace_dev,
               void* hip_stream, stage_t** out) {
  return init_stage(cfg, weights_dev, grads_dev, stash_dev, workspace_dev, hip_stream, nullptr, out);
}

int stage_init_chunk(const stage_config_t* cfg, void* weights_dev, void* grads_dev, void* workspace_dev, stage_t* share_with,
                     stage_t** out) {
  if (!share_with) { if (out) *out = nullptr; return STAGE_E_INVAL; }
  return init_stage(cfg, weights_dev, grads_dev, share_with->stash, workspace_dev, (void*)share_with->stream, share_with, out);
}

static int single_op(stage_t* st, int kind, int mb, int sub, const void* in, void* out) {
  if (!st) return STAGE_E_INVAL;
  if (st->sticky) return st->sticky;
  const int ns = st->D.n_sub;
  const bool needs_in = kind == STAGE_F ? (sub <= 0) : kind == STAGE_B ? (sub < 0 || sub == ns - 1) : false;
  const bool needs_out = kind == STAGE_F ? (sub < 0 || sub == ns - 1) : kind == STAGE_B ? (sub <= 0) : false;
  if ((needs_in && !in) || (needs_out && !out)) return STAGE_E_INVAL;
  return run_one(st, kind, mb, sub, in, out);
}

int stage_forward(stage_t* st, int mb, const void* x_dev, void* y_dev) { return single_op(st, STAGE_F, mb, -1, x_dev, y_dev); }
int stage_backward_input(stage_t* st, int mb, const void* dy_dev, void* dx_dev) { return single_op(st, STAGE_B, mb, -1, dy_dev, dx_dev); }
int stage_backward_weight(stage_t* st, int mb) { return single_op(st, STAGE_W, mb, -1, nullptr, nullptr); }

static bool sub_ok(const stage_t* st, int sub) { return st && sub >= 0 && sub < st->D.n_sub; }
int stage_forward_sub(stage_t* st, int mb, int sub, const void* x_dev, void* y_dev) {
  return sub_ok(st, sub) ? single_op(st, STAGE_F, mb, sub, x_dev, y_dev) : STAGE_E_INVAL;
}
int stage_backward_input_sub(stage_t* st, int mb, int sub, const void* dy_dev, void* dx_dev) {
  return sub_ok(st, sub) ? single_op(st, STAGE_B, mb, sub, dy_dev, dx_dev) : STAGE_E_INVAL;
}
int stage_backward_weight_sub(stage_t* st, int mb, int sub) {
  return sub_ok(st, sub) ? single_op(st, STAGE_W, mb, sub, nullptr, nullptr) : STAGE_E_INVAL;
}

int stage_run_schedule(stage_t* st, const stage_op_t* ops, int n_ops, const void* x_all_dev, const void* dy_all_dev,
                       void* y_all_dev, void* dx_all_dev) {
  if (!st || n_ops < 0 || (n_ops > 0 && !ops)) return STAGE_E_INVAL;
  if (st->sticky) return st->sticky;
  return run_list(&st, 1, n_ops, [&](int i, int& c, int& k, int& m, int& s) { c = 0; k = ops[i].kind; m = ops[i].mb; s = -1; },
                  &x_all_dev, &dy_all_dev, &y_all_dev, &dx_all_dev);
}

int stage_run_subschedule(stage_t* st, const stage_subop_t* ops, int n_ops, const void* x_all_dev, const void* dy_all_dev,
                          void* y_all_dev, void* dx_all_dev) {
  if (!st || n_ops < 0 || (n_ops > 0 && !ops)) return STAGE_E_INVAL;
  if (st->sticky) return st->sticky;
  for (int i = 0; i < n_ops; ++i)
    if (ops[i].sub < 0 || ops[i].sub >= st->D.n_sub) return STAGE_E_INVAL;
  return run_list(&st, 1, n_ops, [&](int i, int& c, int& k, int& m, int& s) { c = 0; k = ops[i].kind; m = ops[i].mb; s = ops[i].sub; },
                  &x_all_dev, &dy_all_dev, &y_all_dev, &dx_all_dev);
}

int stage_run_chunk_schedule(stage_t* const* chunks, int n_chunks, const stage_chunkop_t* ops, int n_ops,
                             const void* const* x_all_dev, const void* const* dy_all_dev, void* const* y_all_dev,
                             void* const* dx_all_dev) {
  if (!chunks || n_chunks < 1 || n_chunks > 16 || n_ops < 0 || (n_ops > 0 && !ops) || !x_all_dev || !dy_all_dev || !y_all_dev ||
      !dx_all_dev)
    return STAGE_E_INVAL;
  for (int c = 0; c < n_chunks; ++c) {
    if (!chunks[c] || chunks[c]->pool != chunks[0]->pool) return STAGE_E_INVAL;      // chunks of one stash only
    for (int e = 0; e < c; ++e) if (chunks[e] == chunks[c]) return STAGE_E_INVAL;
    if (chunks[c]->sticky) return chunks[c]->sticky;
  }
  for (int i = 0; i < n_ops; ++i) {
    const int c = ops[i].chunk;
    if (c < 0 || c >= n_chunks || ops[i].sub < -1 || ops[i].sub >= chunks[c]->D.n_sub) return STAGE_E_INVAL;
  }
  return run_list(chunks, n_chunks, n_ops,
                  [&](int i, int& c, int& k, int& m, int& s) { c = ops[i].chunk; k = ops[i].kind; m = ops[i].mb; s = ops[i].sub; },
                  x_all_dev, dy_all_dev, y_all_dev, dx_all_dev);
}

int stage_validate_chunk_schedule(const stage_config_t* cfg, int n_chunks, const stage_chunkop_t* ops, int n_ops,
                                  int* first_bad_index, int* peak_live) {
  Dims D;
  if (first_bad_index) *first_bad_index = -1;
  if (peak_live) *peak_live = 0;
  if (!make_dims(cfg, &D) || n_chunks < 1 || n_chunks > 16 || n_ops < 0 || (n_ops > 0 && !ops)) return STAGE_E_INVAL;
  std::vector<Tracker> t(n_chunks);
  for (auto& x : t) x.init(D, cfg->enforce_mb_order);
  int live = 0, hlive = 0, peak = 0;
  for (int i = 0; i < n_ops; ++i) {
    const int c = ops[i].chunk, sub = ops[i].sub;
    int rc = STAGE_E_INVAL;
    if (c >= 0 && c < n_chunks && sub >= -1 && sub < D.n_sub) {
      t[c].ext_live = live - t[c].live; t[c].ext_hlive = hlive - t[c].hlive;
      rc = sub < 0 ? t[c].step(ops[i].kind, ops[i].mb) : t[c].step_sub(ops[i].kind, ops[i].mb, sub);
    }
    if (rc != STAGE_OK) {
      if (first_bad_index) *first_bad_index = i;
      if (peak_live) *peak_live = peak;
      return rc;
    }
    live = t[c].live + t[c].ext_live; hlive = t[c].hlive + t[c].ext_hlive;
    if (live > peak) peak = live;
  }
  if (peak_live) *peak_live = peak;
  return STAGE_OK;
}

int stage_validate_subschedule(const stage_config_t* cfg, const stage_subop_t* ops, int n_ops, int* first_bad_index,
                               int* peak_live) {
  Dims D;
  if (first_bad_index) *first_bad_index = -1;
  if (peak_live) *peak_live = 0;
  if (!make_dims(cfg, &D) || n_ops < 0 || (n_ops > 0 && !ops)) return STAGE_E_INVAL;
  Tracker t; t.init(D, cfg->enforce_mb_order);
  for (int i = 0; i < n_ops; ++i) {
    const int rc = t.step_sub(ops[i].kind, ops[i].mb, ops[i].sub);
    if (rc != STAGE_OK) {
      if (first_bad_index) *first_bad_index = i;
      if (peak_live) *peak_live = t.peak;
      return rc;
    }
  }
  if (peak_live) *peak_live = t.peak;
  return STAGE_OK;
}

int stage_grads(stage_t* st, float** grads_dev, size_t* n_elems) {
  if (!st || !grads_dev || !n_elems) return STAGE_E_INVAL;
  *grads_dev = st->grads; *n_elems = st->n_param_elems;
  return STAGE_OK;
}

int stage_zero_grads(stage_t* st) {
  if (!st) return STAGE_E_INVAL;
  if (st->sticky) return st->sticky;
  HIPCHK(fill_zero_f32(st->grads, st->n_param_elems, st->stream));
  return STAGE_OK;
}

int stage_stats(stage_t* st, int* live, int* peak_live, size_t* peak_stash_bytes) {
  if (!st) return STAGE_E_INVAL;
  if (live) *live = st->tr.live;
  if (peak_live) *peak_live = st->pool.use_count() > 1 ? st->pool->peak : st->tr.peak;
  if (peak_stash_bytes) *peak_stash_bytes = st->pool->peak_b > st->tr.peak_b ? st->pool->peak_b : st->tr.peak_b;
  return STAGE_OK;
}

int stage_set_kernel_set(stage_t* st, int which) {
  if (!st || (which != 0 && which != 1)) return STAGE_E_INVAL;
  st->kernel_set = which;
  return STAGE_OK;
}

int stage_profile(stage_t* st, int enable) {
  if (!st) return STAGE_E_INVAL;
  for (auto& r : st->prof) { st->event_pool.push_back(r.t0); st->event_pool.push_back(r.t1); }
  st->prof.clear();
  st->profiling = enable != 0;
  return STAGE_OK;
}

int stage_profile_read(stage_t* st, int kernel_class, double* total_ms, int64_t* launches, double* work) {
  if (!st || kernel_class < 0 || kernel_class >= STAGE_K_COUNT || !total_ms || !launches || !work) return STAGE_E_INVAL;
  if (hipStreamSynchronize(st->stream) != hipSuccess) { st->sticky = STAGE_E_HIP; return STAGE_E_HIP; }
  double ms = 0.0, w = 0.0; int64_t n = 0;
  for (auto& r : st->prof) {
    if (r.cls != kernel_class) continue;
    float t = 0.f;
    if (hipEventElapsedTime(&t, r.t0, r.t1) != hipSuccess) return STAGE_E_HIP;
    ms += t; w += r.work; ++n;
  }
  *total_ms = ms; *launches = n; *work = w;
  return STAGE_OK;
}

void stage_destroy(stage_t* st) {
  if (!st) return;
  for (auto& r : st->prof) { (void)hipEventDestroy(r.t0); (void)hipEventDestroy(r.t1); }
  for (auto e : st->event_pool) (void)hipEventDestroy(e);
  delete st;
}

const char* stage_strerror(int code) {
  switch (code) {
    case STAGE_OK: return "ok";
    case STAGE_E_INVAL: return "invalid argument (null pointer, bad shape, unsupported head_dim, or microbatch out of range)";
    case STAGE_E_ORDER: return "op order violates the microbatch state machine EMPTY-F->FWD-B->BWD-W->EMPTY or the microbatch-order rule";
    case STAGE_E_STASH_FULL: return "refused: stash_cap microbatches are already live (F), or recompute_cap hold a rebuilt stash (B)";
    case STAGE_E_HIP: return "a HIP launch or runtime call failed";
    default: return "unknown error code";
  }
}

}  // extern "C"

// ---------------------------------------------------------------------------
// kernel-level entry points (include/stage_kernels.h)
// ---------------------------------------------------------------------------
#include "../../include/stage_kernels.h"

extern "C" {

static int hip_rc(hipError_t e) { return e == hipSuccess ? STAGE_OK : (e == hipErrorInvalidValue ? STAGE_E_INVAL : STAGE_E_HIP); }
static bool dtype_ok(int dt) { return dt == STAGE_DTYPE_FP32 || dt == STAGE_DTYPE_BF16; }

int stage_kernel_gemm(int dtype, int mode, int M, int N, int K, const void* A, int64_t lda, const void* B, int64_t ldb,
                      void* C, int64_t ldc, const void* R, int64_t ldr, int acc_f32, int kernel_set, void* hip_stream) {
  if (!dtype_ok(dtype) || mode < 0 || mode > 2 || M < 0 || N < 0 || K < 0 || !A || !B || !C) return STAGE_E_INVAL;
  if ((mode == GEMM_TN) != (acc_f32 != 0) || (acc_f32 && R)) return STAGE_E_INVAL;
  GemmArgs g{mode, M, N, K, A, lda, B, ldb, C, ldc, R, ldr, acc_f32};
  if (kernel_set != 1 && dtype == STAGE_DTYPE_BF16 && gemm_mfma_supported(g))
    return hip_rc(gemm_mfma(g, (hipStream_t)hip_stream, kernel_set == 2 ? 1 : kernel_set == 3 ? 2 : kernel_set == 4 ? 3 : 0));
  return hip_rc(gemm_ref((DType)dtype, g, (hipStream_t)hip_stream));
}

int stage_kernel_gemm_act(int dtype, int act, int M, int f, int K, const void* A, int64_t lda, const void* B, int64_t ldb,
                          void* Z, int64_t ldz, void* Aout, int64_t lda_out, int kernel_set, void* hip_stream) {
  if (!dtype_ok(dtype) || (act != STAGE_ACT_GELU && act != STAGE_ACT_SWIGLU) || M <= 0 || f <= 0 || K <= 0 || !A || !B || !Z || !Aout)
    return STAGE_E_INVAL;
  const int fin = act == STAGE_ACT_SWIGLU ? 2 * f : f;
  if (lda < K || ldb < fin || ldz < fin || lda_out < f) return STAGE_E_INVAL;
  GemmArgs g{GEMM_NN, M, fin, K, A, lda, B, ldb, Z, ldz, nullptr, 0, 0, 0, 0};
  g.act = act == STAGE_ACT_SWIGLU ? 2 : 1; g.C2 = Aout; g.ldc2 = lda_out;
  if (kernel_set != 1 && dtype == STAGE_DTYPE_BF16 && gemm_mfma_supported(g))
    return hip_rc(gemm_mfma(g, (hipStream_t)hip_stream, kernel_set == 2 ? 1 : kernel_set == 3 ? 2 : 0));
  // plain kernels: the product, then the activation from the stored z (needs dense rows)
  if (ldz != fin || lda_out != f) return STAGE_E_INVAL;
  g.act = 0; g.C2 = nullptr;
  const hipError_t e = gemm_ref((DType)dtype, g, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_rc(e);
  ActArgs ac{}; ac.kind = act; ac.rows = M; ac.f = f; ac.z = Z; ac.a = Aout;
  return hip_rc(act_fwd((DType)dtype, ac, (hipStream_t)hip_stream));
}

int stage_kernel_gemm_act_bwd(int dtype, int act, int M, int f, int K, const void* dY, int64_t ldy, const void* W, int64_t ldw,
                              void* Z, int64_t ldz, void* da_scratch, int kernel_set, void* hip_stream) {
  if (!dtype_ok(dtype) || (act != STAGE_ACT_GELU && act != STAGE_ACT_SWIGLU) || M <= 0 || f <= 0 || K <= 0 || !dY || !W || !Z)
    return STAGE_E_INVAL;
  const int nop = act == STAGE_ACT_SWIGLU ? 2 : 1;
  if (ldy < K || ldw < K || ldz < (int64_t)nop * f) return STAGE_E_INVAL;
  GemmArgs g{GEMM_NT, M, f, K, dY, ldy, W, ldw, nullptr, (int64_t)f, nullptr, 0, 0, 0, 0};
  g.act_bwd = nop; g.Z = Z; g.ldz = ldz;
  if (kernel_set != 1 && dtype == STAGE_DTYPE_BF16 && gemm_mfma_supported(g))
    return hip_rc(gemm_mfma(g, (hipStream_t)hip_stream, kernel_set == 2 ? 1 : kernel_set == 3 ? 2 : 0));
  // plain kernels: the product into the scratch, then the activation backward kernel (dense z rows)
  if (!da_scratch || ldz != (int64_t)nop * f) return STAGE_E_INVAL;
  g.act_bwd = 0; g.Z = nullptr; g.C = da_scratch;
  const hipError_t e = gemm_ref((DType)dtype, g, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_rc(e);
  ActArgs ac{}; ac.kind = act; ac.rows = M; ac.f = f; ac.z = Z; ac.da = da_scratch;
  return hip_rc(act_bwd((DType)dtype, ac, (hipStream_t)hip_stream));
}

int stage_kernel_wgrad_group(int dtype, int n, const int* M, const int* N, const int* K, const void* const* A,
                             const int64_t* lda, const void* const* B, const int64_t* ldb, float* const* C,
                             const int64_t* ldc, int kernel_set, void* hip_stream) {
  if (!dtype_ok(dtype) || n < 0) return STAGE_E_INVAL;
  if (n == 0) return STAGE_OK;
  if (!M || !N || !K || !A || !lda || !B || !ldb || !C || !ldc) return STAGE_E_INVAL;
  std::vector<GemmArgs> list(n);
  for (int i = 0; i < n; ++i) {
    if (M[i] < 0 || N[i] < 0 || K[i] < 0 || !A[i] || !B[i] || !C[i]) return STAGE_E_INVAL;
    list[i] = GemmArgs{GEMM_TN, M[i], N[i], K[i], A[i], lda[i], B[i], ldb[i], C[i], ldc[i], nullptr, 0, 1, 0, 0};
  }
  return hip_rc(wgrad_list((DType)dtype, kernel_set, list.data(), n, 1, nullptr, (hipStream_t)hip_stream));
}

static bool attn_shape(int dtype, int b, int s, int h, int hkv, int hd, int causal) {
  return dtype_ok(dtype) && b > 0 && s > 0 && s <= 65536 && h > 0 && hkv > 0 && h % hkv == 0 && (hd == 64 || hd == 128) &&
         (causal == 0 || causal == 1);
}

int stage_kernel_attention_fwd(int dtype, int b, int s, int h, int hkv, int hd, int causal, const void* qkv, void* o,
                               float* lse, int kernel_set, void* hip_stream) {
  if (!attn_shape(dtype, b, s, h, hkv, hd, causal) || !qkv || !o || !lse) return STAGE_E_INVAL;
  AttnArgs a{}; a.b = b; a.s = s; a.h = h; a.hkv = hkv; a.hd = hd; a.causal = causal;
  a.qkv = qkv; a.ld = (int64_t)(h + 2 * hkv) * hd; a.o = o; a.lse = lse;
  a.width = kernel_set == 2 ? 1 : kernel_set == 3 ? 2 : kernel_set == 4 ? 3 : 0;
  if (kernel_set != 1 && dtype == STAGE_DTYPE_BF16 && attn_mfma_supported(a)) return hip_rc(attn_fwd_mfma(a, (hipStream_t)hip_stream));
  return hip_rc(attn_fwd_ref((DType)dtype, a, (hipStream_t)hip_stream));
}

int stage_kernel_rope_table(int s, int hd, float theta, float* table, void* hip_stream) {
  if (s < 1 || (hd != 64 && hd != 128) || !(theta > 0.f) || !table) return STAGE_E_INVAL;
  return hip_rc(rope_table(table, s, hd, (double)theta, (hipStream_t)hip_stream));
}

int stage_kernel_rope(int dtype, int b, int s, int n_heads, int hd, int inverse, void* x, int64_t ld, const float* table,
                      void* hip_stream) {
  if (!dtype_ok(dtype) || b < 1 || s < 1 || n_heads < 1 || (hd != 64 && hd != 128) || !x || !table || ld < (int64_t)n_heads * hd)
    return STAGE_E_INVAL;
  return hip_rc(rope_apply((DType)dtype, x, ld, (int64_t)b * s, s, n_heads, hd, table, inverse != 0, (hipStream_t)hip_stream));
}

size_t stage_kernel_attention_bwd_scratch_bytes(int b, int s, int h, int hkv, int hd) {
  if (b < 1 || s < 1 || h < 1 || hkv < 1 || h % hkv || (hd != 64 && hd != 128)) return 0;
  return attn_bwd_part_bytes(b, s, h, hkv, hd);
}

int stage_kernel_attention_bwd(int dtype, int b, int s, int h, int hkv, int hd, int causal, const void* qkv,
                               const void* o, const float* lse, const void* dout, void* dqkv, float* delta,
                               int kernel_set, void* hip_stream) {
  return stage_kernel_attention_bwd_ws(dtype, b, s, h, hkv, hd, causal, qkv, o, lse, dout, dqkv, delta, nullptr, 0,
                                       kernel_set, hip_stream);
}

int stage_kernel_attention_bwd_ws(int dtype, int b, int s, int h, int hkv, int hd, int causal, const void* qkv,
                                  const void* o, const float* lse, const void* dout, void* dqkv, float* delta,
                                  void* scratch, size_t scratch_bytes, int kernel_set, void* hip_stream) {
  if (!attn_shape(dtype, b, s, h, hkv, hd, causal) || !qkv || !o || !lse || !dout || !dqkv || !delta) return STAGE_E_INVAL;
  if (scratch && (scratch_bytes < attn_bwd_part_bytes(b, s, h, hkv, hd) || ((uintptr_t)scratch & 15))) return STAGE_E_INVAL;
  AttnArgs a{}; a.b = b; a.s = s; a.h = h; a.hkv = hkv; a.hd = hd; a.causal = causal;
  a.qkv = qkv; a.ld = (int64_t)(h + 2 * hkv) * hd; a.o = (void*)o; a.lse = (float*)lse;
  a.dout = dout; a.dqkv = dqkv; a.delta = delta;
  a.dkv_part = attn_bwd_part_bytes(b, s, h, hkv, hd) ? (float*)scratch : nullptr;
  a.width = kernel_set == 2 ? 1 : kernel_set == 3 ? 2 : kernel_set == 4 ? 3 : 0;
  if (kernel_set != 1 && dtype == STAGE_DTYPE_BF16 && attn_mfma_supported(a)) return hip_rc(attn_bwd_mfma(a, (hipStream_t)hip_stream));
  return hip_rc(attn_bwd_ref((DType)dtype, a, (hipStream_t)hip_stream));
}

int stage_kernel_norm_fwd(int dtype, int norm, int rows, int d, float eps, const void* x, const void* gamma,
                          const void* beta, void* out, float* stats, void* hip_stream) {
  if (!dtype_ok(dtype) || (norm != 0 && norm != 1) || rows <= 0 || d <= 0 || !x || !gamma || (norm == 0 && !beta) || !out || !stats)
    return STAGE_E_INVAL;
  NormArgs n{}; n.kind = norm; n.rows = rows; n.d = d; n.eps = eps; n.x = x; n.gamma = gamma; n.beta = beta; n.out = out; n.stats = stats;
  return hip_rc(norm_fwd((DType)dtype, n, (hipStream_t)hip_stream));
}

int stage_kernel_norm_bwd(int dtype, int norm, int rows, int d, const void* x, const float* stats, const void* gamma,
                          const void* dout, const void* resid, void* dx, float* dgamma, float* dbeta, float* partial,
                          void* hip_stream) {
  if (!dtype_ok(dtype) || (norm != 0 && norm != 1) || rows <= 0 || d <= 0 || !x || !stats || !gamma || !dout || !dx || !dgamma ||
      (norm == 0 && !dbeta) || !partial)
    return STAGE_E_INVAL;
  NormArgs n{}; n.kind = norm; n.rows = rows; n.d = d; n.x = x; n.stats = (float*)stats; n.gamma = gamma; n.dout = dout;
  n.resid = resid; n.out = dx; n.dgamma = dgamma; n.dbeta = dbeta; n.partial = partial;
  return hip_rc(norm_bwd((DType)dtype, n, (hipStream_t)hip_stream));
}

int stage_kernel_norm_bwd_noalloc(int dtype, int norm, int rows, int d, const void* x, const float* stats, const void* gamma,
                                  const void* dout, const void* resid, void* dx, float* dgamma, float* dbeta, void* hip_stream) {
  if (!dtype_ok(dtype) || (norm != 0 && norm != 1) || rows <= 0 || d <= 0 || !x || !stats || !gamma || !dout || !dx || !dgamma ||
      (norm == 0 && !dbeta))
    return STAGE_E_INVAL;
  if (d > norm_bwd_noalloc_max_d()) return STAGE_E_INVAL;      // wider rows than the fixed scratch holds partials for
  NormArgs n{}; n.kind = norm; n.rows = rows; n.d = d; n.x = x; n.stats = (float*)stats; n.gamma = gamma; n.dout = dout;
  n.resid = resid; n.out = dx; n.dgamma = dgamma; n.dbeta = dbeta;
  return hip_rc(norm_bwd_noalloc((DType)dtype, n, (hipStream_t)hip_stream));
}

size_t stage_kernel_bias_grad_scratch_bytes(int n) { return bias_grad_partial_bytes(n); }

int stage_kernel_bias_grad(int dtype, int rows, int n, const void* dz, int64_t ld, float* dbias, float* scratch, void* hip_stream) {
  if (!dtype_ok(dtype) || rows <= 0 || n <= 0 || !dz || ld < n || !dbias || !scratch) return STAGE_E_INVAL;
  return hip_rc(bias_grad((DType)dtype, dz, ld, rows, n, scratch, dbias, (hipStream_t)hip_stream));
}

size_t stage_kernel_norm_partial_bytes(int d) { return d > 0 ? (size_t)norm_partial_rows() * 2 * d * sizeof(float) : 0; }

int stage_kernel_act_fwd(int dtype, int act, int rows, int f, const void* z, void* a, void* hip_stream) {
  if (!dtype_ok(dtype) || (act != 0 && act != 1) || rows <= 0 || f <= 0 || !z || !a) return STAGE_E_INVAL;
  ActArgs ac{}; ac.kind = act; ac.rows = rows; ac.f = f; ac.z = (void*)z; ac.a = a;
  return hip_rc(act_fwd((DType)dtype, ac, (hipStream_t)hip_stream));
}

int stage_kernel_act_bwd(int dtype, int act, int rows, int f, void* z, const void* da, void* hip_stream) {
  if (!dtype_ok(dtype) || (act != 0 && act != 1) || rows <= 0 || f <= 0 || !z || !da) return STAGE_E_INVAL;
  ActArgs ac{}; ac.kind = act; ac.rows = rows; ac.f = f; ac.z = z; ac.da = da;
  return hip_rc(act_bwd((DType)dtype, ac, (hipStream_t)hip_stream));
}

}  // extern "C"
