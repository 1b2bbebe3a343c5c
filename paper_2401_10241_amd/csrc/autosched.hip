// Host side of the schedule work: the p-stage timing model behind the bubble rate (Sec. 5.3,
// Appendix G) and the heuristic automatic scheduler (Sec. 3.1).  No device code.
//
// Everything here is plain double arithmetic in a fixed order (no contraction into fused
// multiply-adds), so that a schedule is a pure function of its arguments.
#include <stdint.h>

#include <limits>
#include <vector>

#include "../../include/zb_stage.h"

#pragma clang fp contract(off)

namespace {

constexpr double kInf = std::numeric_limits<double>::infinity();

struct Times {
  double f, b, w, comm;
  double of(int pass) const { return pass == ZB_PASS_F ? f : pass == ZB_PASS_B ? b : w; }
};

bool valid_times(const zb_pass_times* t) {
  return t && t->t_f > 0 && t->t_b > 0 && t->t_w > 0 && t->t_comm >= 0 && t->t_f < kInf && t->t_b < kInf &&
         t->t_w < kInf && t->t_comm < kInf;
}

// Every (pass, microbatch) exactly once per stage, F before B before W of the same microbatch.
bool valid_orders(int p, int m, const zb_op* orders) {
  std::vector<char> seen((size_t)3 * m);
  for (int i = 0; i < p; ++i) {
    std::fill(seen.begin(), seen.end(), 0);
    for (int q = 0; q < 3 * m; ++q) {
      const zb_op& op = orders[(size_t)i * 3 * m + q];
      if (op.pass < 0 || op.pass > 2 || op.mb < 0 || op.mb >= m) return false;
      if (seen[(size_t)op.pass * m + op.mb]) return false;
      if (op.pass > 0 && !seen[(size_t)(op.pass - 1) * m + op.mb]) return false;
      seen[(size_t)op.pass * m + op.mb] = 1;
    }
  }
  return true;
}

// A pass starts when the previous pass of its stage has ended and its input from the neighbouring stage
// has arrived (F from stage i-1, B from stage i+1, each T_comm after the producer ended).  With
// fused_backward the input gradient leaves a stage only after the W of that microbatch (the single
// backward function of 1F1B).  Returns false if the orders deadlock.
bool run_timing(int p, int m, const zb_op* orders, const Times& t, bool fused_backward, std::vector<double>* first,
                std::vector<double>* last, double t_w_next = -1.0) {
  const size_t n = (size_t)3 * m;
  std::vector<double> end((size_t)p * n, -1.0);  // [stage][pass][mb]
  std::vector<int> ptr(p, 0);
  std::vector<double> clock(p, 0.0);
  first->assign(p, 0.0);
  last->assign(p, 0.0);
  size_t remaining = (size_t)p * n;
  while (remaining) {
    bool progressed = false;
    for (int i = 0; i < p; ++i) {
      while (ptr[i] < (int)n) {
        const zb_op& op = orders[(size_t)i * n + ptr[i]];
        double ready = clock[i];
        if (op.pass == ZB_PASS_F && i > 0) {
          const double e = end[(size_t)(i - 1) * n + (size_t)ZB_PASS_F * m + op.mb];
          if (e < 0) break;
          if (e + t.comm > ready) ready = e + t.comm;
        } else if (op.pass == ZB_PASS_B && i < p - 1) {
          const int src = fused_backward ? ZB_PASS_W : ZB_PASS_B;
          const double e = end[(size_t)(i + 1) * n + (size_t)src * m + op.mb];
          if (e < 0) break;
          if (e + t.comm > ready) ready = e + t.comm;
        }
        if (ptr[i] == 0) (*first)[i] = ready;
        // a W right behind another W of the same stage shares that one's gradient traffic (one launch)
        const bool w_run = t_w_next >= 0 && op.pass == ZB_PASS_W && ptr[i] > 0 &&
                           orders[(size_t)i * n + ptr[i] - 1].pass == ZB_PASS_W;
        clock[i] = ready + (w_run ? t_w_next : t.of(op.pass));
        end[(size_t)i * n + (size_t)op.pass * m + op.mb] = clock[i];
        (*last)[i] = clock[i];
        ++ptr[i];
        --remaining;
        progressed = true;
      }
    }
    if (!progressed) return false;
  }
  return true;
}

// The heuristic of Sec. 3.1, its four steps in the order the section gives them.
//   Step 1 (warm-up): stage 0 may hold floor(M_limit / M_B) forwards, every later stage one fewer than the
//   stage before it (step 3's guarantee that stage i stays a forward ahead of stage i+1), never fewer than
//   one.  How many of those a stage takes depends on when its first backward can start, which depends on the
//   stages after it, so the counts are settled from the last stage back to the first; the forwards of a stage
//   run back to back from the moment the first microbatch reaches it.
//   Step 2 (steady state): rounds of one backward per stage (last stage first) and one forward per stage
//   (first stage first).  A pass that cannot start yet leaves a gap; pending W go into it while a whole one
//   fits, and one more when idling instead would raise the largest cumulative bubble of all stages.  W also
//   run to make room for a forward that does not fit under M_limit.
//   Step 3: the forward of a round is left out if it would bring the stage level with its predecessor, or -
//   second option - if the stage leads its successor by more than one and has a W to work on instead; the
//   forward that the next round's backward needs is always taken.
//   Step 4: the W that are left.
struct StageClock {
  double now = 0, mem = 0, bubble = 0;
  int nf = 0, nb = 0, nw = 0, len = 0;
};

class RoundScheduler {
 public:
  RoundScheduler(int p, int m, const Times& t, const zb_memory_model& mm, zb_op* out)
      : p_(p), m_(m), t_(t), mm_(mm), out_(out), st_(p), endf_((size_t)p * m, 0.0), endb_((size_t)p * m, 0.0) {
    eps_ = 1e-9 * (t.f + t.b + t.w);
    cap_ = mm.m_limit * (1 + 1e-12);
  }

  void plan_warmup(bool extra, std::vector<int>* counts) const {
    const double eps = 1e-9 * (t_.f + t_.b);
    std::vector<int> room(p_);
    long long fit = (long long)(cap_ / mm_.m_b);
    if (fit > m_) fit = m_;
    room[0] = fit < 1 ? 1 : (int)fit;
    for (int i = 1; i < p_; ++i) room[i] = room[i - 1] > 2 ? room[i - 1] - 1 : 1;
    counts->assign(p_, 1);
    double b0_done = 0;
    for (int i = p_ - 1; i >= 0; --i) {
      const double lead_in = i * (t_.f + t_.comm);  // the first microbatch reaches the stage
      const double b0_can = i == p_ - 1 ? lead_in + 1 * t_.f : b0_done + t_.comm;
      int n = 1;
      while (n < room[i] && lead_in + (n + 1) * t_.f <= b0_can + eps) ++n;
      if (extra && n < room[i] && lead_in + n * t_.f < b0_can - eps) ++n;
      (*counts)[i] = n;
      const double f_done = lead_in + n * t_.f;
      b0_done = (b0_can > f_done ? b0_can : f_done) + t_.b;
    }
  }

  bool build(bool extra, bool skip) {
    std::vector<int> warm;
    plan_warmup(extra, &warm);
    for (int i = 0; i < p_; ++i)
      for (int q = 0; q < warm[i]; ++q) place(i, ZB_PASS_F);
    for (int round = 0; round < m_; ++round) {
      for (int i = p_ - 1; i >= 0; --i) {
        soak(i, can_start(i, ZB_PASS_B));
        place(i, ZB_PASS_B);
      }
      for (int i = 0; i < p_; ++i) {
        StageClock& s = st_[i];
        if (s.nf == m_) continue;
        const bool owed = s.nf <= round + 1;  // B of the next round reads this forward
        if (!owed) {
          if (i > 0 && st_[i - 1].nf < m_ && s.nf + 1 >= st_[i - 1].nf) continue;
          if (skip && i < p_ - 1 && s.nf - st_[i + 1].nf > 1 && s.nw < s.nb) continue;
        }
        while (!(s.mem + mm_.m_b <= cap_)) {
          if (!(s.nw < s.nb)) return false;
          place(i, ZB_PASS_W);
        }
        soak(i, can_start(i, ZB_PASS_F));
        place(i, ZB_PASS_F);
      }
    }
    for (int i = 0; i < p_; ++i)
      while (st_[i].nw < st_[i].nb) place(i, ZB_PASS_W);
    return true;
  }

 private:
  double can_start(int i, int pass) const {
    const StageClock& s = st_[i];
    double t = s.now;
    if (pass == ZB_PASS_F && i > 0) {
      const double a = endf_[(size_t)(i - 1) * m_ + s.nf] + t_.comm;
      if (a > t) t = a;
    } else if (pass == ZB_PASS_B && i < p_ - 1) {
      const double a = endb_[(size_t)(i + 1) * m_ + s.nb] + t_.comm;
      if (a > t) t = a;
    }
    return t;
  }

  void place(int i, int pass) {
    StageClock& s = st_[i];
    const double at = can_start(i, pass);
    if (s.len > 0) s.bubble += at - s.now;
    s.now = at + t_.of(pass);
    int k;
    if (pass == ZB_PASS_F) { k = s.nf++; endf_[(size_t)i * m_ + k] = s.now; s.mem += mm_.m_b; }
    else if (pass == ZB_PASS_B) { k = s.nb++; endb_[(size_t)i * m_ + k] = s.now; s.mem += mm_.m_w - mm_.m_b; }
    else { k = s.nw++; s.mem += -mm_.m_w; }
    out_[(size_t)i * 3 * m_ + s.len++] = zb_op{pass, k};
  }

  // pending W into the gap before a pass that can start at `until`
  void soak(int i, double until) {
    StageClock& s = st_[i];
    while (s.nw < s.nb && s.now + t_.w <= until + eps_) place(i, ZB_PASS_W);
    const double gap = until - s.now;
    if (s.nw < s.nb && gap > eps_) {
      double worst = st_[0].bubble;
      for (int j = 1; j < p_; ++j)
        if (st_[j].bubble > worst) worst = st_[j].bubble;
      if (s.bubble + gap > worst + eps_) place(i, ZB_PASS_W);
    }
  }

  int p_, m_;
  Times t_;
  zb_memory_model mm_;
  zb_op* out_;
  double eps_, cap_;
  std::vector<StageClock> st_;
  std::vector<double> endf_, endb_;
};

bool valid_memory(const zb_memory_model* mm) {
  return mm && mm->m_b > 0 && mm->m_w >= 0 && mm->m_w <= mm->m_b && mm->m_limit >= mm->m_b && mm->m_limit < kInf;
}

double span_cost(const std::vector<double>& first, const std::vector<double>& last) {
  double c = 0;
  for (size_t i = 0; i < first.size(); ++i)
    if (last[i] - first[i] > c) c = last[i] - first[i];
  return c;
}

}  // namespace

extern "C" {

zb_status zb_simulate_pipeline(int32_t p, int32_t m, const zb_op* orders, const zb_pass_times* times,
                               int32_t fused_backward, double* cost, double* bubble_rate, double* stage_span) {
  if (p < 1 || m < 1 || !orders || !valid_times(times)) return ZB_EINVAL;
  if (!valid_orders(p, m, orders)) return ZB_EORDER;
  const Times t{times->t_f, times->t_b, times->t_w, times->t_comm};
  std::vector<double> first, last;
  if (!run_timing(p, m, orders, t, fused_backward != 0, &first, &last)) return ZB_EORDER;
  const double c = span_cost(first, last);
  if (cost) *cost = c;
  if (bubble_rate) *bubble_rate = (c - m * (t.f + t.b + t.w)) / c;
  if (stage_span)
    for (int i = 0; i < p; ++i) stage_span[i] = last[i] - first[i];
  return ZB_OK;
}

zb_status zb_simulate_pipeline_w_runs(int32_t p, int32_t m, const zb_op* orders, const zb_pass_times* times,
                                      double t_w_next, double* cost, double* stage_span) {
  if (p < 1 || m < 1 || !orders || !valid_times(times) || !(t_w_next >= 0)) return ZB_EINVAL;
  if (!valid_orders(p, m, orders)) return ZB_EORDER;
  const Times t{times->t_f, times->t_b, times->t_w, times->t_comm};
  std::vector<double> first, last;
  if (!run_timing(p, m, orders, t, false, &first, &last, t_w_next)) return ZB_EORDER;
  if (cost) *cost = span_cost(first, last);
  if (stage_span)
    for (int i = 0; i < p; ++i) stage_span[i] = last[i] - first[i];
  return ZB_OK;
}

zb_status zb_auto_schedule(int32_t p, int32_t m, const zb_pass_times* times, const zb_memory_model* mem,
                           int32_t extra_warmup_f, int32_t skip_f, zb_op* orders) {
  if (p < 1 || m < 1 || !orders || !valid_times(times) || !valid_memory(mem)) return ZB_EINVAL;
  const Times t{times->t_f, times->t_b, times->t_w, times->t_comm};
  RoundScheduler h(p, m, t, *mem, orders);
  return h.build(extra_warmup_f != 0, skip_f != 0) ? ZB_OK : ZB_ENOMEM;
}

zb_status zb_auto_schedule_search(int32_t p, int32_t m, const zb_pass_times* times, const zb_memory_model* mem,
                                  zb_op* orders, double* cost, double* bubble_rate, int32_t* extra_warmup_f,
                                  int32_t* skip_f) {
  if (p < 1 || m < 1 || !orders || !valid_times(times) || !valid_memory(mem)) return ZB_EINVAL;
  const Times t{times->t_f, times->t_b, times->t_w, times->t_comm};
  const size_t total = (size_t)p * 3 * m;
  std::vector<zb_op> trial(total);
  bool have = false;
  double best = 0;
  for (int combo = 0; combo < 4; ++combo) {  // (0,0) (0,1) (1,0) (1,1); the first of equal costs wins
    const bool ew = (combo >> 1) != 0, sk = (combo & 1) != 0;
    RoundScheduler h(p, m, t, *mem, trial.data());
    if (!h.build(ew, sk)) continue;
    std::vector<double> first, last;
    if (!run_timing(p, m, trial.data(), t, false, &first, &last)) continue;
    const double c = span_cost(first, last);
    if (!have || c < best) {
      have = true;
      best = c;
      for (size_t q = 0; q < total; ++q) orders[q] = trial[q];
      if (extra_warmup_f) *extra_warmup_f = ew;
      if (skip_f) *skip_f = sk;
    }
  }
  if (!have) return ZB_ENOMEM;
  if (cost) *cost = best;
  if (bubble_rate) *bubble_rate = (best - m * (t.f + t.b + t.w)) / best;
  return ZB_OK;
}

// ---- ZB-V (Sec. 6): two chunks per worker, virtual microbatch v = chunk * m + microbatch ------------

namespace {

struct VDep { int worker, pass, v; bool link, none; };

// whose end worker i (0-based) waits for before (pass, chunk, k); chunk 0 runs worker 0..p-1, chunk 1 back
VDep v_producer(int p, int m, int i, int pass, int ch, int k) {
  if (pass == ZB_PASS_F) {
    if (ch == 0) return i == 0 ? VDep{0, 0, 0, false, true} : VDep{i - 1, ZB_PASS_F, k, true, false};
    return i < p - 1 ? VDep{i + 1, ZB_PASS_F, m + k, true, false} : VDep{i, ZB_PASS_F, k, false, false};
  }
  if (pass == ZB_PASS_B) {
    if (ch == 1) return i > 0 ? VDep{i - 1, ZB_PASS_B, m + k, true, false} : VDep{i, ZB_PASS_F, m + k, false, false};
    return i < p - 1 ? VDep{i + 1, ZB_PASS_B, k, true, false} : VDep{i, ZB_PASS_B, m + k, false, false};
  }
  return VDep{i, ZB_PASS_B, ch * m + k, false, false};
}

// phases 1 and 2 of worker sigma + 1: warm-up forwards, then F-B-W groups of one chunk
void v_static_part(int p, int sigma, int m, std::vector<zb_op>* ops) {
  const int i = sigma + 1;
  int nf[2] = {0, 0}, nb[2] = {0, 0}, nw[2] = {0, 0};
  auto f = [&](int c) { if (nf[c] < m) ops->push_back(zb_op{ZB_PASS_F, c * m + nf[c]++}); };
  auto b = [&](int c) { if (nb[c] < nf[c]) ops->push_back(zb_op{ZB_PASS_B, c * m + nb[c]++}); };
  auto w = [&](int c) { if (nw[c] < nb[c]) ops->push_back(zb_op{ZB_PASS_W, c * m + nw[c]++}); };
  for (int q = 0; q < 2 * (p - i) + 1; ++q) f(0);
  for (int q = 0; q < i - 1; ++q) { f(1); f(0); }
  int lead = p - i;  // groups of chunk 1 before the alternation starts
  int turn = 1;
  while (!(nf[0] == m && nf[1] == m)) {
    int c;
    if (lead > 0) { c = 1; --lead; }
    else { c = turn; turn ^= 1; }
    f(c); b(c); w(c);
  }
}

}  // namespace

zb_status zb_schedule_order_v(int32_t p, int32_t m, zb_op* orders) {
  if (p < 1 || m < 1 || !orders) return ZB_EINVAL;
  const size_t n = (size_t)6 * m;
  std::vector<std::vector<zb_op>> stat(p);
  for (int s = 0; s < p; ++s) v_static_part(p, s, m, &stat[s]);
  // final phase: unit pass times, no communication; a free worker runs a ready B (chunk 0 first), else
  // its oldest pending W (chunk 1 first among equals)
  std::vector<int> end((size_t)p * 3 * 2 * m, -1);  // [worker][pass][v]
  auto at = [&](int i, int pass, int v) -> int& { return end[((size_t)i * 3 + pass) * 2 * m + v]; };
  std::vector<int> len(p, 0), nb((size_t)p * 2, 0), nw((size_t)p * 2, 0);
  size_t done = 0;
  for (int t = 0; done < (size_t)p * n; ++t) {
    if (t > 600 * (m + p)) return ZB_ESTATE;
    std::vector<zb_op> chosen(p, zb_op{-1, -1});
    auto ready = [&](int i, int pass, int ch, int k) {
      const VDep d = v_producer(p, m, i, pass, ch, k);
      if (d.none) return true;
      const int e = at(d.worker, d.pass, d.v);
      return e >= 0 && e <= t;
    };
    for (int i = 0; i < p; ++i) {
      if (len[i] < (int)stat[i].size()) {
        const zb_op& op = stat[i][len[i]];
        if (ready(i, op.pass, op.mb / m, op.mb % m)) chosen[i] = op;
        continue;
      }
      for (int ch = 0; ch < 2 && chosen[i].pass < 0; ++ch) {
        const int k = nb[i * 2 + ch];
        if (k < m && ready(i, ZB_PASS_B, ch, k)) chosen[i] = zb_op{ZB_PASS_B, ch * m + k};
      }
      if (chosen[i].pass < 0) {
        int best_k = -1, best_ch = -1;
        for (int ch = 1; ch >= 0; --ch) {
          const int k = nw[i * 2 + ch];
          if (k < nb[i * 2 + ch] && (best_ch < 0 || k < best_k)) { best_k = k; best_ch = ch; }
        }
        if (best_ch >= 0) chosen[i] = zb_op{ZB_PASS_W, best_ch * m + best_k};
      }
    }
    for (int i = 0; i < p; ++i) {
      const zb_op& op = chosen[i];
      if (op.pass < 0) continue;
      orders[(size_t)i * n + len[i]++] = op;
      at(i, op.pass, op.mb) = t + 1;
      ++done;
      if (op.pass == ZB_PASS_B) nb[i * 2 + op.mb / m] = op.mb % m + 1;
      else if (op.pass == ZB_PASS_W) nw[i * 2 + op.mb / m] = op.mb % m + 1;
    }
  }
  return ZB_OK;
}

zb_status zb_simulate_pipeline_v(int32_t p, int32_t m, const zb_op* orders, const zb_pass_times* times, double* cost,
                                 double* bubble_rate, double* stage_span) {
  if (p < 1 || m < 1 || !orders || !valid_times(times)) return ZB_EINVAL;
  if (!valid_orders(p, 2 * m, orders)) return ZB_EORDER;  // 2m virtual microbatches per worker
  const Times t{times->t_f, times->t_b, times->t_w, times->t_comm};
  const size_t n = (size_t)6 * m;
  std::vector<double> end((size_t)p * n, -1.0), clock(p, 0.0), first(p, 0.0), last(p, 0.0);
  std::vector<int> ptr(p, 0);
  auto at = [&](int i, int pass, int v) -> double& { return end[((size_t)i * 3 + pass) * 2 * m + v]; };
  size_t remaining = (size_t)p * n;
  while (remaining) {
    bool progressed = false;
    for (int i = 0; i < p; ++i) {
      while (ptr[i] < (int)n) {
        const zb_op& op = orders[(size_t)i * n + ptr[i]];
        double ready = clock[i];
        const VDep d = v_producer(p, m, i, op.pass, op.mb / m, op.mb % m);
        if (!d.none) {
          const double e = at(d.worker, d.pass, d.v);
          if (e < 0) break;
          const double a = e + (d.link ? t.comm : 0.0);
          if (a > ready) ready = a;
        }
        if (ptr[i] == 0) first[i] = ready;
        clock[i] = ready + t.of(op.pass);
        at(i, op.pass, op.mb) = clock[i];
        last[i] = clock[i];
        ++ptr[i];
        --remaining;
        progressed = true;
      }
    }
    if (!progressed) return ZB_EORDER;
  }
  const double c = span_cost(first, last);
  if (cost) *cost = c;
  if (bubble_rate) *bubble_rate = (c - 2 * m * (t.f + t.b + t.w)) / c;
  if (stage_span)
    for (int i = 0; i < p; ++i) stage_span[i] = last[i] - first[i];
  return ZB_OK;
}

zb_status zb_order_group_w(const zb_op* ops, int32_t n, int32_t group, zb_op* out) {
  if (!ops || !out || n < 0 || group < 1) return ZB_EINVAL;
  for (int32_t i = 0; i < n; ++i)
    if (ops[i].pass < 0 || ops[i].pass > 2) return ZB_EINVAL;
  // B W F_j B W F ... B W: `group` times B W with a forward between each two, j a multiple of group
  const int64_t span = 3 * (int64_t)group - 1;
  auto group_starts_at = [&](int32_t i) {
    if (group < 2 || i + span > n || ops[i + 2].mb % group != 0) return false;
    for (int64_t d = 0; d < span; ++d) {
      const int want = d % 3 == 0 ? ZB_PASS_B : d % 3 == 1 ? ZB_PASS_W : ZB_PASS_F;
      if (ops[i + d].pass != want) return false;
    }
    return true;
  };
  int32_t q = 0;
  for (int32_t i = 0; i < n;) {
    if (group_starts_at(i)) {  // the forwards and backwards first, then the W side by side
      for (int64_t d = 0; d < span; ++d)
        if (d % 3 != 1) out[q++] = ops[i + d];
      for (int64_t d = 1; d < span; d += 3) out[q++] = ops[i + d];
      i += (int32_t)span;
    } else {
      out[q++] = ops[i++];
    }
  }
  return ZB_OK;
}

zb_status zb_order_memory_peak(const zb_op* ops, int32_t n, double m_b, double m_w, double* peak) {
  if (!ops || n < 0 || !peak) return ZB_EINVAL;
  double cur = 0, top = 0;
  for (int q = 0; q < n; ++q) {
    if (ops[q].pass == ZB_PASS_F) cur += m_b;
    else if (ops[q].pass == ZB_PASS_B) cur += m_w - m_b;
    else if (ops[q].pass == ZB_PASS_W) cur += -m_w;
    else return ZB_EINVAL;
    if (cur > top) top = cur;
  }
  *peak = top;
  return ZB_OK;
}

}  // extern "C"
