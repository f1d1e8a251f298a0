// Host-side CrossUDSub greedy schedule generator and pipeline performance model
// (paper Algorithm 1, sections 4.2.2-4.2.3, 2.2 and 3.5).  No GPU code here.
#include "../../include/crosspipe_sched.h"

#include <algorithm>
#include <limits>
#include <map>
#include <utility>
#include <vector>

namespace {

constexpr double INF = std::numeric_limits<double>::infinity();

// occupied transmission windows of one directed link, kept sorted by start time
struct Link {
  std::vector<std::pair<double, double>> busy;
  // earliest window of length t_bw starting at or after t_ready; returns its end
  double reserve(double t_ready, double t_bw) {
    if (t_bw <= 0.0) return t_ready;
    double start = t_ready;
    size_t at = 0;
    for (; at < busy.size(); ++at) {
      if (start + t_bw <= busy[at].first) break;
      if (busy[at].second > start) start = busy[at].second;
    }
    busy.insert(busy.begin() + at, std::make_pair(start, start + t_bw));
    return start + t_bw;
  }
};

struct Model {
  const crosspipe_params_t& p;
  std::vector<Link> links;
  explicit Model(const crosspipe_params_t& pp) : p(pp), links((size_t)pp.n_pp * pp.n_pp) {}
  double dur(int stage, int kind) const {
    const double* t = kind == CROSSPIPE_F ? p.t_f : kind == CROSSPIPE_D ? p.t_d : p.t_w;
    return t[stage] / p.n_sub;
  }
  // arrival time at dst of the message produced at t_ready on src (alpha-beta with queuing on the link)
  double comm(int src, int dst, double t_ready) {
    const size_t ij = (size_t)src * p.n_pp + dst;
    const double a = p.alpha ? p.alpha[ij] : 0.0, b = p.beta ? p.beta[ij] : 0.0;
    return links[ij].reserve(t_ready, b * p.msg_bytes) + a;
  }
  // block that depends on a finished (stage, kind) block; false if none
  bool successor(int stage, int kind, int* ns, int* nk) const {
    if (kind == CROSSPIPE_F) {
      if (stage + 1 < p.n_pp) { *ns = stage + 1; *nk = CROSSPIPE_F; } else { *ns = stage; *nk = CROSSPIPE_D; }
      return true;
    }
    if (kind == CROSSPIPE_D && stage > 0) { *ns = stage - 1; *nk = CROSSPIPE_D; return true; }
    return false;
  }
};

typedef std::pair<int, int> Op;   // (kind, mb)

struct StageState {
  double end = 0.0, mem = 0.0;
  std::map<Op, double> avail;     // schedulable blocks -> T_avail
  std::map<Op, int> done_sub;     // sub-blocks already scheduled
  int n_f_started = 0;
  int last_full = -1;             // kind of the last F or D block started
};

bool params_ok(const crosspipe_params_t* p) {
  return p && p->n_pp > 0 && p->n_mb > 0 && p->n_sub > 0 && p->t_f && p->t_d && p->t_w;
}

}  // namespace

extern "C" {

int crosspipe_greedy(const crosspipe_params_t* pp, crosspipe_slot_t* out, int capacity, int* n_out, double* makespan) {
  if (!params_ok(pp) || !out || !n_out || !makespan) return CROSSPIPE_E_INVAL;
  const crosspipe_params_t& p = *pp;
  const int64_t total = (int64_t)3 * p.n_mb * p.n_sub * p.n_pp;
  if (capacity < total) return CROSSPIPE_E_INVAL;
  Model M(p);
  std::vector<StageState> st(p.n_pp);
  for (int m = 0; m < p.n_mb; ++m) st[0].avail[Op(CROSSPIPE_F, m)] = 0.0;
  int n = 0;
  double mk = 0.0;
  // an F block not yet started is infeasible while it would exceed the memory limit
  auto feasible = [&](const StageState& S, const Op& op) {
    if (op.first != CROSSPIPE_F) return true;
    auto it = S.done_sub.find(op);
    if (it != S.done_sub.end() && it->second > 0) return true;
    return S.mem + p.m_f <= p.m_limit + 1e-12;
  };
  for (;;) {
    // stage selection: earliest schedulable time, ties to the lowest stage
    int cur = -1;
    double t_cur = INF;
    for (int s = 0; s < p.n_pp; ++s) {
      double first = INF;
      for (const auto& kv : st[s].avail)
        if (feasible(st[s], kv.first)) first = std::min(first, kv.second);
      if (first == INF) continue;
      const double t = std::max(st[s].end, first);
      if (t < t_cur) { t_cur = t; cur = s; }
    }
    if (cur < 0) break;
    StageState& S = st[cur];
    // operation selection among feasible blocks available at t_cur
    Op pick(-1, -1);
    for (const auto& kv : S.avail) {            // a started F or D block continues first (map order: F before D, low mb first)
      if (kv.second > t_cur || kv.first.first == CROSSPIPE_W) continue;
      auto it = S.done_sub.find(kv.first);
      if (it != S.done_sub.end() && it->second > 0 && it->second < p.n_sub) { pick = kv.first; break; }
    }
    if (pick.first < 0) {
      int first_of[3] = {-1, -1, -1};           // lowest available microbatch per kind
      for (const auto& kv : S.avail)
        if (kv.second <= t_cur && feasible(S, kv.first) && first_of[kv.first.first] < 0) first_of[kv.first.first] = kv.first.second;
      int order[3], no = 0;
      if (S.n_f_started >= p.n_mb) { order[no++] = CROSSPIPE_D; order[no++] = CROSSPIPE_W; }               // tear-down
      else if (S.last_full == CROSSPIPE_D) { order[no++] = CROSSPIPE_F; order[no++] = CROSSPIPE_D; order[no++] = CROSSPIPE_W; }
      else { order[no++] = CROSSPIPE_D; order[no++] = CROSSPIPE_F; order[no++] = CROSSPIPE_W; }           // warm-up / after an F
      for (int i = 0; i < no && pick.first < 0; ++i)
        if (first_of[order[i]] >= 0) pick = Op(order[i], first_of[order[i]]);
      if (pick.first < 0) pick = Op(CROSSPIPE_W, first_of[CROSSPIPE_W]);
    }
    // operation scheduling: the next sub-block of the picked block
    const int kind = pick.first, mb = pick.second;
    const int sub = S.done_sub[pick];
    if (sub == 0) {
      if (kind == CROSSPIPE_F) { S.mem += p.m_f; ++S.n_f_started; S.last_full = CROSSPIPE_F; }
      else if (kind == CROSSPIPE_D) S.last_full = CROSSPIPE_D;
    }
    const double t_end = t_cur + M.dur(cur, kind);
    out[n++] = crosspipe_slot_t{cur, kind, mb, kind == CROSSPIPE_D ? p.n_sub - 1 - sub : sub, t_cur, t_end};
    S.end = t_end;
    mk = std::max(mk, t_end);
    S.done_sub[pick] = sub + 1;
    if (sub + 1 == p.n_sub) {                   // block complete
      S.avail.erase(pick);
      if (kind == CROSSPIPE_D) { S.mem += p.m_d; S.avail[Op(CROSSPIPE_W, mb)] = t_end; }
      else if (kind == CROSSPIPE_W) S.mem += p.m_w;
      int ns, nk;
      if (M.successor(cur, kind, &ns, &nk)) st[ns].avail[Op(nk, mb)] = ns == cur ? t_end : M.comm(cur, ns, t_end);
    }
  }
  *n_out = n;
  *makespan = mk;
  return n == total ? CROSSPIPE_OK : CROSSPIPE_E_INVAL;
}

int crosspipe_simulate(const crosspipe_params_t* pp, const crosspipe_slot_t* sched, int n, crosspipe_slot_t* out,
                       double* makespan) {
  if (!params_ok(pp) || n < 0 || (n > 0 && (!sched || !out)) || !makespan) return CROSSPIPE_E_INVAL;
  const crosspipe_params_t& p = *pp;
  std::vector<std::vector<const crosspipe_slot_t*>> lists(p.n_pp);
  for (int i = 0; i < n; ++i) {
    const crosspipe_slot_t& x = sched[i];
    if (x.stage < 0 || x.stage >= p.n_pp || x.kind < 0 || x.kind > 2 || x.mb < 0 || x.mb >= p.n_mb || x.sub < 0 || x.sub >= p.n_sub)
      return CROSSPIPE_E_INVAL;
    lists[x.stage].push_back(&x);
  }
  Model M(p);
  std::vector<size_t> pos(p.n_pp, 0);
  std::vector<double> end(p.n_pp, 0.0);
  std::vector<std::map<Op, double>> avail(p.n_pp);
  std::vector<std::map<Op, int>> done(p.n_pp);
  for (int m = 0; m < p.n_mb; ++m) avail[0][Op(CROSSPIPE_F, m)] = 0.0;
  double mk = 0.0;
  for (int k = 0; k < n; ++k) {
    int cur = -1;
    double t_cur = INF;
    for (int s = 0; s < p.n_pp; ++s) {
      if (pos[s] >= lists[s].size()) continue;
      const crosspipe_slot_t& x = *lists[s][pos[s]];
      auto it = avail[s].find(Op(x.kind, x.mb));
      if (it == avail[s].end()) continue;                   // its input has not been produced yet
      const double t = std::max(end[s], it->second);
      if (t < t_cur) { t_cur = t; cur = s; }
    }
    if (cur < 0) return CROSSPIPE_E_DEADLOCK;
    const crosspipe_slot_t& x = *lists[cur][pos[cur]++];
    const double t_end = t_cur + M.dur(cur, x.kind);
    out[k] = crosspipe_slot_t{cur, x.kind, x.mb, x.sub, t_cur, t_end};
    end[cur] = t_end;
    mk = std::max(mk, t_end);
    const Op op(x.kind, x.mb);
    if (++done[cur][op] == p.n_sub) {
      if (x.kind == CROSSPIPE_D) avail[cur][Op(CROSSPIPE_W, x.mb)] = t_end;
      int ns, nk;
      if (M.successor(cur, x.kind, &ns, &nk)) avail[ns][Op(nk, x.mb)] = ns == cur ? t_end : M.comm(cur, ns, t_end);
    }
  }
  *makespan = mk;
  return CROSSPIPE_OK;
}

int crosspipe_stage_ops(const crosspipe_slot_t* sched, int n, int stage, stage_subop_t* out, int capacity, int* n_out) {
  if (n < 0 || (n > 0 && !sched) || !out || !n_out || stage < 0) return CROSSPIPE_E_INVAL;
  int k = 0;
  for (int i = 0; i < n; ++i) {
    if (sched[i].stage != stage) continue;
    if (k >= capacity) return CROSSPIPE_E_INVAL;
    out[k++] = stage_subop_t{sched[i].kind, sched[i].mb, sched[i].sub};
  }
  *n_out = k;
  return CROSSPIPE_OK;
}

}  // extern "C"
