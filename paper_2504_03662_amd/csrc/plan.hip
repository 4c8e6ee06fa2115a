// Layer-wise strategy plan search (host code only): the discovery-phase search of the strategy
// selector, given a per-layer cost table.  Decision-tree style pruning of the candidates first
// (feasibility, dominance), then an exact dynamic program over layers whose state is the last
// layer's strategy and a Pareto frontier of (memory used, time spent).
#include "../../include/gx.h"

#include <algorithm>
#include <cmath>
#include <new>
#include <limits>
#include <vector>

namespace {

struct Pt {
  double mem, time;
  int prev_s, prev_i;     // strategy of the previous layer and index into its frontier
};

constexpr size_t MAX_POINTS = 1u << 22;     // per (layer, strategy) candidate list; beyond: coarser quantum needed

// Memory after rounding: k * q for the least whole k whose product k * q (in double arithmetic) is
// not below x; a memory that is already such a product is unchanged.  The quotient only seeds the
// search, so its rounding cannot move the result.
double round_up(double x, double q) {
  if (!(q > 0.0)) return x;
  double k = std::floor(x / q);
  while (k * q < x) k += 1.0;
  while (k >= 1.0 && (k - 1.0) * q >= x) k -= 1.0;
  return k * q;
}

}  // namespace

namespace {
gx_status search(const gx_plan_problem* p, int32_t* choice, gx_plan_result* out) {
  if (!p || !choice || !out || !p->time_ms || !p->mem_bytes) return GX_ERR_NULL;
  const int L = p->layers, S = p->strategies;
  if (L <= 0 || S <= 0 || L > 4096 || S > 1024) return GX_ERR_SHAPE;
  if (!(p->mem_budget_bytes >= 0.0) || !(p->mem_quantum_bytes >= 0.0)) return GX_ERR_SHAPE;
  const double B = p->mem_budget_bytes;
  std::vector<double> mem((size_t)L * S);
  for (size_t i = 0; i < mem.size(); i++) {
    if (!(p->time_ms[i] >= 0.0) || !(p->mem_bytes[i] >= 0.0) || !std::isfinite(p->time_ms[i]) ||
        !std::isfinite(p->mem_bytes[i]))
      return GX_ERR_SHAPE;
    mem[i] = round_up(p->mem_bytes[i], p->mem_quantum_bytes);
  }
  auto T = [&](int l, int s) { return p->time_ms[(size_t)l * S + s]; };
  auto M = [&](int l, int s) { return mem[(size_t)l * S + s]; };
  auto SW = [&](int a, int b) { return (p->switch_ms && a != b) ? p->switch_ms[(size_t)a * S + b] : 0.0; };
  if (p->switch_ms)
    for (int a = 0; a < S; a++)
      for (int b = 0; b < S; b++)
        if (a != b && (!(SW(a, b) >= 0.0) || !std::isfinite(SW(a, b)))) return GX_ERR_SHAPE;

  // pruning.  Rule 1 (feasibility): a strategy whose memory, together with the least memory every
  // other layer can have, exceeds the budget is on no feasible plan.  Rule 2 (dominance): a strategy
  // is dropped at a layer when another one there is no slower, no larger and no costlier to switch
  // to or from, with a strict improvement somewhere or a smaller index.
  std::vector<double> least(L);
  double least_total = 0.0;
  for (int l = 0; l < L; l++) {
    least[l] = M(l, 0);
    for (int s = 1; s < S; s++) least[l] = std::min(least[l], M(l, s));
    least_total += least[l];
  }
  std::vector<char> alive((size_t)L * S, 1);
  int64_t pruned = 0;
  for (int l = 0; l < L; l++)
    for (int s = 0; s < S; s++)
      if (least_total - least[l] + M(l, s) > B * (1.0 + 1e-15)) { alive[(size_t)l * S + s] = 0; pruned++; }
  for (int l = 0; l < L; l++)
    for (int s = 0; s < S; s++) {
      if (!alive[(size_t)l * S + s]) continue;
      for (int d = 0; d < S; d++) {
        if (d == s || !alive[(size_t)l * S + d]) continue;
        const bool no_worse = T(l, d) <= T(l, s) && M(l, d) <= M(l, s);
        const bool strict = T(l, d) < T(l, s) || M(l, d) < M(l, s) || d < s;
        // with switching costs a dominated strategy could still pay off by avoiding a switch, so
        // the rule is only applied when there are none
        if (no_worse && strict && !p->switch_ms) {
          alive[(size_t)l * S + s] = 0;
          pruned++;
          break;
        }
      }
    }

  // dynamic program
  std::vector<std::vector<std::vector<Pt>>> fr(L, std::vector<std::vector<Pt>>(S));
  size_t peak = 0;
  for (int s = 0; s < S; s++)
    if (alive[s] && M(0, s) <= B) {
      fr[0][s].push_back(Pt{M(0, s), T(0, s), -1, -1});
      peak = 1;
    }
  std::vector<Pt> cand;
  for (int l = 1; l < L; l++) {
    for (int s2 = 0; s2 < S; s2++) {
      if (!alive[(size_t)l * S + s2]) continue;
      cand.clear();
      const double m2 = M(l, s2), t2 = T(l, s2);
      for (int s1 = 0; s1 < S; s1++) {
        const std::vector<Pt>& f = fr[l - 1][s1];
        const double sw = SW(s1, s2);
        for (int i = 0; i < (int)f.size(); i++) {
          const double m = f[i].mem + m2;
          if (m > B) break;                      // frontiers are sorted by memory
          cand.push_back(Pt{m, f[i].time + t2 + sw, s1, i});
        }
        if (cand.size() > MAX_POINTS) return GX_ERR_SHAPE;
      }
      std::sort(cand.begin(), cand.end(), [](const Pt& a, const Pt& b) {
        if (a.mem != b.mem) return a.mem < b.mem;
        if (a.time != b.time) return a.time < b.time;
        if (a.prev_s != b.prev_s) return a.prev_s < b.prev_s;
        return a.prev_i < b.prev_i;
      });
      std::vector<Pt>& dst = fr[l][s2];
      double best = INFINITY;
      for (const Pt& c : cand)
        if (c.time < best) { dst.push_back(c); best = c.time; }
      peak = std::max(peak, dst.size());
    }
  }
  int bs = -1, bi = -1;
  for (int s = 0; s < S; s++) {
    const std::vector<Pt>& f = fr[L - 1][s];
    for (int i = 0; i < (int)f.size(); i++) {
      if (bs < 0 || f[i].time < fr[L - 1][bs][bi].time ||
          (f[i].time == fr[L - 1][bs][bi].time && f[i].mem < fr[L - 1][bs][bi].mem)) {
        bs = s;
        bi = i;
      }
    }
  }
  out->pruned = pruned;
  out->frontier_peak = (int64_t)peak;
  if (bs < 0) {
    out->total_ms = 0.0;
    out->total_mem_bytes = 0.0;
    return GX_ERR_INFEASIBLE;
  }
  out->total_ms = fr[L - 1][bs][bi].time;
  out->total_mem_bytes = fr[L - 1][bs][bi].mem;
  for (int l = L - 1; l >= 0; l--) {
    choice[l] = bs;
    const Pt& q = fr[l][bs][bi];
    bs = q.prev_s;
    bi = q.prev_i;
  }
  return GX_OK;
}
}  // namespace

// Nothing may be thrown across the C boundary: running out of host memory for the frontiers is
// reported like a frontier beyond the supported size.
extern "C" gx_status gx_plan_search(const gx_plan_problem* p, int32_t* choice, gx_plan_result* out) {
  try {
    return search(p, choice, out);
  } catch (const std::bad_alloc&) {
    return GX_ERR_SHAPE;
  } catch (...) {
    return GX_ERR_SHAPE;
  }
}

// Per-GPU cost model of one layer under one strategy (host code): what the cost table holds beside
// the measured compute times.  Sizes are exact integers; times follow the ring model stated in
// the header.
extern "C" gx_status gx_strategy_cost(const gx_strategy_query* q, gx_strategy_costs* out) {
  if (!q || !out) return GX_ERR_NULL;
  if (q->dtype != GX_F32 && q->dtype != GX_BF16) return GX_ERR_DTYPE;
  if (q->hidden <= 0 || q->heads <= 0 || q->ffn <= 0 || q->seq <= 0 || q->gpus <= 0 || q->global_batch <= 0 ||
      q->tp_attn <= 0 || q->tp_ffn <= 0 || !(q->link_gbps > 0.0) || !std::isfinite(q->link_gbps))
    return GX_ERR_SHAPE;
  if (q->hidden % q->heads || q->heads % q->tp_attn || q->ffn % q->tp_ffn || q->gpus % q->tp_attn ||
      q->gpus % q->tp_ffn)
    return GX_ERR_DIVIS;
  const int64_t H = q->hidden, F = q->ffn, S = q->seq, N = q->gpus, GB = q->global_batch;
  const int64_t a = q->tp_attn, f = q->tp_ffn;
  // a tensor-parallel group of degree d serves GB * d / N samples per step; it must be a whole number
  if ((GB * a) % N || (GB * f) % N) return GX_ERR_DIVIS;
  const int64_t mba = GB * a / N, mbf = GB * f / N;
  const int64_t e = q->dtype == GX_BF16 ? 2 : 4;
  const int64_t Hl = H / a, Fl = F / f, nl = q->heads / a, dh = H / q->heads;
  // one rank's parameters: LayerNorm gain and bias, the column-parallel matrix and bias, the
  // row-parallel matrix, and the row-parallel bias (replicated)
  const int64_t ea = 2 * H + H * 3 * Hl + 3 * Hl + Hl * H + H;
  const int64_t ef = 2 * H + H * Fl + Fl + Fl * H + H;
  out->micro_batch_attn = mba;
  out->micro_batch_ffn = mbf;
  out->attn_elems = ea;
  out->ffn_elems = ef;
  out->state_bytes = (double)(ea + ef) * (double)(e + 16);
  const double bw = q->link_gbps * 1e9;                 // bytes per second per link
  auto ring_ms = [&](double bytes, int64_t p) {         // all-reduce of `bytes` over p ranks
    return p <= 1 ? 0.0 : 2.0 * (double)(p - 1) / (double)p * bytes / bw * 1e3;
  };
  const double act_a = (double)(mba * S * H * e), act_f = (double)(mbf * S * H * e);
  out->tp_comm_ms = 2.0 * ring_ms(act_a, a) + 2.0 * ring_ms(act_f, f);
  out->dp_comm_ms = ring_ms((double)ea * 4.0, N / a) + ring_ms((double)ef * 4.0, N / f);
  out->switch_ms = 2.0 * ((double)(GB * S * H * e) / (double)N) / bw * 1e3;
  const double Ta = (double)(mba * S), Tf = (double)(mbf * S);
  const double fwd_a = 2.0 * Ta * (double)H * 3.0 * (double)Hl + 2.0 * Ta * (double)Hl * (double)H +
                       4.0 * (double)mba * (double)nl * (double)dh * (double)S * (double)(S + 1) / 2.0;
  const double fwd_f = 4.0 * Tf * (double)H * (double)Fl;
  out->flops_attn = 3.0 * fwd_a;
  out->flops_ffn = 3.0 * fwd_f;
  return GX_OK;
}

// Pipeline regrouping (host code): which consecutive layers each stage holds, chosen so that the
// slowest stage is as fast as possible, and what a change from one grouping to another moves.
namespace {
gx_status partition(int32_t L, int32_t P, const double* ms, int32_t* first, double* bottleneck) {
  // prefix[i] = time of layers 0 .. i-1; every group time below is a difference of two entries,
  // so the same group always gets the same floating-point value
  std::vector<double> prefix((size_t)L + 1, 0.0);
  for (int32_t i = 0; i < L; i++) {
    const double t = ms ? ms[i] : 1.0;
    if (!(t > 0.0) || !std::isfinite(t)) return GX_ERR_SHAPE;
    prefix[i + 1] = prefix[i] + t;
  }
  auto span = [&](int32_t a, int32_t b) { return prefix[b] - prefix[a]; };
  // best[s][i]: smallest bottleneck of layers i .. L-1 in s stages (s <= L - i)
  const double INF = std::numeric_limits<double>::infinity();
  std::vector<std::vector<double>> best((size_t)P + 1, std::vector<double>((size_t)L + 1, INF));
  for (int32_t i = 0; i < L; i++) best[1][i] = span(i, L);
  for (int32_t s = 2; s <= P; s++)
    for (int32_t i = 0; i + s <= L; i++) {
      double b = INF;
      for (int32_t e = i + 1; e + (s - 1) <= L; e++) b = std::min(b, std::max(span(i, e), best[s - 1][e]));
      best[s][i] = b;
    }
  const double opt = best[P][0];
  // among the groupings that reach it: every stage, from the first, as short as it can be
  first[0] = 0;
  for (int32_t s = 0; s + 1 < P; s++) {
    const int32_t i = first[s], rest = P - s - 1;
    int32_t e = i + 1;
    while (!(span(i, e) <= opt && best[rest][e] <= opt)) e++;      // ends: the optimum exists
    first[s + 1] = e;
  }
  first[P] = L;
  if (bottleneck) *bottleneck = opt;
  return GX_OK;
}
}  // namespace

extern "C" gx_status gx_stage_partition(int32_t layers, int32_t stages, const double* layer_ms, int32_t* first,
                                        double* bottleneck_ms) {
  if (!first) return GX_ERR_NULL;
  if (layers <= 0 || stages <= 0 || stages > layers || layers > 65536 || stages > 4096) return GX_ERR_SHAPE;
  try {
    return partition(layers, stages, layer_ms, first, bottleneck_ms);
  } catch (...) {
    return GX_ERR_SHAPE;
  }
}

extern "C" gx_status gx_stage_moves(int32_t layers, int32_t old_stages, const int32_t* old_first, int32_t new_stages,
                                    const int32_t* new_first, int32_t* new_stage_of, int32_t* moved) {
  if (!old_first || !new_first || !new_stage_of || !moved) return GX_ERR_NULL;
  if (layers <= 0 || old_stages <= 0 || new_stages <= 0 || old_stages > layers || new_stages > layers)
    return GX_ERR_SHAPE;
  auto valid = [&](const int32_t* f, int32_t n) {
    if (f[0] != 0 || f[n] != layers) return false;
    for (int32_t s = 0; s < n; s++)
      if (f[s + 1] <= f[s]) return false;
    return true;
  };
  if (!valid(old_first, old_stages) || !valid(new_first, new_stages)) return GX_ERR_SHAPE;
  int32_t so = 0, sn = 0, count = 0;
  for (int32_t l = 0; l < layers; l++) {
    while (l >= old_first[so + 1]) so++;
    while (l >= new_first[sn + 1]) sn++;
    new_stage_of[l] = sn;
    if (so != sn) count++;
  }
  *moved = count;
  return GX_OK;
}
