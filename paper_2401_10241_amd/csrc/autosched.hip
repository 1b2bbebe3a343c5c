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
                std::vector<double>* last) {
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
        clock[i] = ready + t.of(op.pass);
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

// The heuristic of Sec. 3.1.  All stages share one clock; repeatedly every unfinished stage proposes
// (pass, start time) from what has been decided so far, the proposal that starts first is carried out
// (lowest stage on ties) and all stages propose again.
class Heuristic {
 public:
  Heuristic(int p, int m, const Times& t, const zb_memory_model& mm, bool extra_warmup_f, bool skip_f)
      : p_(p), m_(m), t_(t), mm_(mm), extra_(extra_warmup_f), skip_(skip_f) {
    tol_ = 1e-9 * (t.f + t.b + t.w);
    cap_ = mm.m_limit * (1 + 1e-12);
    clock_.assign(p, 0.0);
    nf_.assign(p, 0);
    nb_.assign(p, 0);
    nw_.assign(p, 0);
    mem_.assign(p, 0.0);
    idle_.assign(p, 0.0);
    started_.assign(p, 0);
    last_fb_.assign(p, ZB_PASS_F);
    end_f_.assign((size_t)p * m, 0.0);
    end_b_.assign((size_t)p * m, 0.0);
  }

  // orders: [p][3m]; false if no stage can run a pass (memory limit too small)
  bool run(zb_op* orders) {
    std::vector<int> len(p_, 0);
    const size_t n = (size_t)3 * m_;
    for (size_t step = 0; step < (size_t)p_ * n; ++step) {
      double max_idle = idle_[0];
      for (int i = 1; i < p_; ++i)
        if (idle_[i] > max_idle) max_idle = idle_[i];
      int bi = -1, bpass = 0;
      double bstart = 0;
      for (int i = 0; i < p_; ++i) {
        if (len[i] == (int)n) continue;
        int pass;
        double start;
        if (!propose(i, max_idle, &pass, &start)) continue;
        if (bi < 0 || start < bstart) { bi = i; bpass = pass; bstart = start; }
      }
      if (bi < 0) return false;
      const int i = bi;
      int k;
      if (started_[i]) idle_[i] += bstart - clock_[i];
      started_[i] = 1;
      const double e = bstart + t_.of(bpass);
      clock_[i] = e;
      if (bpass == ZB_PASS_F) {
        k = nf_[i]++;
        end_f_[(size_t)i * m_ + k] = e;
        last_fb_[i] = ZB_PASS_F;
        mem_[i] += mm_.m_b;
      } else if (bpass == ZB_PASS_B) {
        k = nb_[i]++;
        end_b_[(size_t)i * m_ + k] = e;
        last_fb_[i] = ZB_PASS_B;
        mem_[i] += mm_.m_w - mm_.m_b;
      } else {
        k = nw_[i]++;
        mem_[i] += -mm_.m_w;
      }
      orders[(size_t)i * n + len[i]++] = zb_op{bpass, k};
    }
    return true;
  }

 private:
  // W now, or wait for the earlier of the next backward (s_b, if known) and the allowed forward (s_f)
  bool fill(int i, double c, bool has_w, double max_idle, bool know_b, double s_b, bool allow_f, double s_f,
            int* pass, double* start) const {
    double nxt = know_b ? s_b : kInf;
    const bool take_f = allow_f && s_f < nxt;
    if (take_f) nxt = s_f;
    if (has_w) {
      const double gap = nxt - c;
      if (gap >= t_.w - tol_ || idle_[i] + gap > max_idle + tol_) {
        *pass = ZB_PASS_W;
        *start = c;
        return true;
      }
    }
    if (nxt < kInf) {
      *pass = take_f ? ZB_PASS_F : ZB_PASS_B;
      *start = nxt;
      return true;
    }
    return false;
  }

  bool propose(int i, double max_idle, int* pass, double* start) const {
    const double c = clock_[i];
    bool know_f = false, know_b = false;
    double s_f = 0, s_b = 0;
    if (nf_[i] < m_ && (i == 0 || nf_[i - 1] > nf_[i])) {
      know_f = true;
      s_f = c;
      if (i > 0) {
        const double a = end_f_[(size_t)(i - 1) * m_ + nf_[i]] + t_.comm;
        if (a > s_f) s_f = a;
      }
    }
    if (nb_[i] < nf_[i] && (i == p_ - 1 || nb_[i + 1] > nb_[i])) {
      know_b = true;
      s_b = c;
      if (i < p_ - 1) {
        const double a = end_b_[(size_t)(i + 1) * m_ + nb_[i]] + t_.comm;
        if (a > s_b) s_b = a;
      }
    }
    const bool has_w = nw_[i] < nb_[i];
    const bool mem_ok = mem_[i] + mm_.m_b <= cap_;
    const bool f_arrived = know_f && s_f <= c + tol_;
    const bool b_now = know_b && s_b <= c + tol_;
    const bool fits = know_f && (!know_b || s_f + t_.f <= s_b + tol_);
    auto now = [&](int what) {
      *pass = what;
      *start = c;
      return true;
    };
    if (nb_[i] == 0) {  // warm-up
      if (b_now) return now(ZB_PASS_B);
      const bool ok = know_f && mem_ok && (fits || (extra_ && (!know_b || s_f < s_b - tol_)));
      return fill(i, c, has_w, max_idle, know_b, s_b, ok, s_f, pass, start);
    }
    if (nf_[i] == m_ && nb_[i] == m_) return has_w ? now(ZB_PASS_W) : false;
    if (last_fb_[i] == ZB_PASS_B && nf_[i] < m_) {  // a forward is due
      if (f_arrived) {
        if (mem_ok) return now(ZB_PASS_F);
        if (has_w) return now(ZB_PASS_W);  // release memory for the forward
        if (b_now) return now(ZB_PASS_B);
        return fill(i, c, has_w, max_idle, know_b, s_b, false, 0, pass, start);
      }
      if (b_now) return now(ZB_PASS_B);
      return fill(i, c, has_w, max_idle, know_b, s_b, know_f && mem_ok, s_f, pass, start);
    }
    if (b_now) return now(ZB_PASS_B);  // a backward is due
    const int lead = nf_[i] - (i < p_ - 1 ? nf_[i + 1] : nb_[i]);
    const bool ok = know_f && mem_ok && fits && !(skip_ && lead >= 1);
    return fill(i, c, has_w, max_idle, know_b, s_b, ok, s_f, pass, start);
  }

  int p_, m_;
  Times t_;
  zb_memory_model mm_;
  bool extra_, skip_;
  double tol_, cap_;
  std::vector<double> clock_, mem_, idle_, end_f_, end_b_;
  std::vector<int> nf_, nb_, nw_, last_fb_;
  std::vector<char> started_;
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

zb_status zb_auto_schedule(int32_t p, int32_t m, const zb_pass_times* times, const zb_memory_model* mem,
                           int32_t extra_warmup_f, int32_t skip_f, zb_op* orders) {
  if (p < 1 || m < 1 || !orders || !valid_times(times) || !valid_memory(mem)) return ZB_EINVAL;
  const Times t{times->t_f, times->t_b, times->t_w, times->t_comm};
  Heuristic h(p, m, t, *mem, extra_warmup_f != 0, skip_f != 0);
  return h.run(orders) ? ZB_OK : ZB_ENOMEM;
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
    Heuristic h(p, m, t, *mem, ew, sk);
    if (!h.run(trial.data())) continue;
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
