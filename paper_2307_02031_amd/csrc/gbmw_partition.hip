// Algorithm 2's inner loop (bi-objective pipeline-partition search, Section 4.2.2
// and Appendix B) for many (batch size, PP degree) pairs in lockstep.  See
// include/gbmw.h for the contract.
//
// Every (pair, stage) owns a slot: table rows for as many layers as the stage can
// ever hold, a pair of fp32 layer tables, its best row.  The slots live for the
// whole call, so a round only computes what the accepted move invalidated:
//   the stage whose FIRST layer changed          all of its layers again
//   the stage that gained a layer at its END     one more layer step on its kept table
//   the stage that lost its LAST layer           nothing but the final reduce, if the
//                                                table of its new last layer is still there
//   every other stage                            nothing
// Per round the host only decides which slots are touched (it mirrors the
// partitions from the accept flags it reads back); everything that produces a
// value runs in kernels:
//   k_gather        rows of the resident model -> the rows of the touched slots
//   table solve     the layer kernels of gbmw_kernels.hip on the touched slots
//   k_stage_bup / k_stage_check   with O_b / O_ms tables: Appendix A, Algorithm 3's walk over
//                   the forward budgets (the first one whose plan's overall memory exceeds E)
//   k_stage_result  plan at e = E (at the budget that walk chose) of every touched stage
//                   -> strategies, C, Cns, O
//   k_chain_step    Eq. 8, Eq. 6, PP_Partition_Adjust, Validate, trace entry
#include <algorithm>
#include <climits>
#include <cmath>
#include <cstring>
#include <utility>
#include <vector>

#include "gbmw_ctx.h"

namespace gbmw {

struct Search {
  int n_chain, S, E, Pmax, max_iter;
  const int *P, *Lm, *m, *lrow, *prow, *mrow;      // [n_chain]
  const float *c, *cns, *R;                        // resident model (cns may be null)
  const int* M;
  const int *Ob, *Oms;                             // resident, indexed like M; null: plain search
  int *Ob_g, *Oms_g;                               // rows of the slots, like Tables::M
  int *bup, *first_bad;                            // [sumP] per slot: largest O_b of its layers; lowest
                                                   // checked budget whose plan does not fit (INT_MAX: none)
  int* part;                                       // [sumP] partition being searched
  int* Ot;                                         // [n_chain]
  float *stC, *stCns;                              // [sumP] results of the current stages
  int* stO;
  uint8_t* strat;                                  // [sumLm]
  int *n_iter, *live, *moved;                      // [n_chain], [n_chain], [2 n_chain]
  int *tr_p, *tr_O;                                // [n_chain][max_iter][Pmax]
  float *tr_C, *tr_Cns;
  float *tr_cost, *tr_at, *tr_am;                  // [n_chain][max_iter]
};

__global__ void k_fill_u32(uint32_t* p, size_t n, uint32_t v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// One workgroup per row: c and M of a model layer -> a slot row, and the layer's R straight
// into the row's transposed table (Rt[s][s'] = R[s'][s], zero padding, then c(s) and the bits
// of M(s): the layout the layer kernels read), so that only touched rows are prepared.
__global__ __launch_bounds__(256) void k_gather(const float* __restrict__ c,
                                                const int* __restrict__ M,
                                                const float* __restrict__ R,
                                                const int* __restrict__ row_src,
                                                const int* __restrict__ row_msrc,
                                                const int* __restrict__ row_dst, int S, int SP, int RS,
                                                float* __restrict__ c_g, int* __restrict__ M_g,
                                                float* __restrict__ Rt,
                                                const int* __restrict__ Ob, const int* __restrict__ Oms,
                                                int* __restrict__ Ob_g, int* __restrict__ Oms_g) {
  const size_t src = (size_t)row_src[blockIdx.x], msrc = (size_t)row_msrc[blockIdx.x];
  const size_t dst = (size_t)row_dst[blockIdx.x];
  for (int i = threadIdx.x; i < S; i += 256) {
    c_g[dst * S + i] = c[src * S + i];
    M_g[dst * S + i] = M[msrc * S + i];
    if (Ob) {
      Ob_g[dst * S + i] = Ob[msrc * S + i];
      Oms_g[dst * S + i] = Oms[msrc * S + i];
    }
  }
  const float* __restrict__ Rl = R + src * S * S;
  float* __restrict__ out = Rt + dst * S * RS;
  for (int i = threadIdx.x; i < S * RS; i += 256) {
    const int s = i / RS, sp = i % RS;
    float v = 0.0f;
    if (sp < S) v = Rl[(size_t)sp * S + s];
    else if (sp == SP) v = c[src * S + s];
    else if (sp == SP + 1) v = __int_as_float(M[msrc * S + s]);
    out[i] = v;
  }
}

// Overall memory (Eq. 2) of the plan of slot b at forward budget e, one lane on its own.
// Going from the last layer to the first, the forward prefix of layer i is F - suf_i with F
// the sum of all O_f and suf_i the sum over the layers above i, so
//   E_all = F + max_i (O_b(i) - suf_i) + sum O_ms.
__device__ long long plan_e_all(const Tables& t, const Search& s, int b, int e) {
  const int n = t.L[b], row0 = t.off[b], S = t.S;
  int sx = t.best_s[(size_t)b * t.EP + e];
  long long suf = 0, ms = 0, mx = 0;
  for (int l = n - 1; l >= 0; --l) {
    const size_t cell = (size_t)(row0 + l) * S + sx;
    const int m = t.M[cell], oms = s.Oms_g[cell];
    const long long here = (long long)s.Ob_g[cell] - suf;
    mx = (l == n - 1 || here > mx) ? here : mx;
    suf += m - oms;
    ms += oms;
    if (l > 0) {
      e -= m;                                              // budget left for layers < l
      if (m < 0 || e < 0) return -2;                       // only reachable with invalid inputs
      sx = pred_strategy(t, row0 + l, sx, e);
    }
  }
  return suf + mx + ms;
}

// Algorithm 3's walk over the forward budgets, in three launches per round.  Plans up to
// E - b_up (b_up = the stage's largest O_b) fit without a check; above it every budget's plan
// is walked and its overall memory compared with E, and the first one that does not fit ends
// the walk.
// k_stage_bup: one wave per touched stage: b_up, and no failing budget known yet.
__global__ __launch_bounds__(64) void k_stage_bup(Tables t, Search s, const int* __restrict__ touched) {
  const int lane = threadIdx.x;
  const int b = touched[blockIdx.x];
  const int n = t.L[b], S = t.S, row0 = t.off[b];
  int bup = 0;
  for (int i = lane; i < n * S; i += 64) {
    const int v = s.Ob_g[(size_t)row0 * S + i];
    bup = v > bup ? v : bup;
  }
  for (int d = 32; d >= 1; d >>= 1) {
    const int o = __shfl_xor(bup, d, 64);
    bup = o > bup ? o : bup;
  }
  if (lane == 0) {
    s.bup[b] = bup;
    s.first_bad[b] = INT_MAX;
  }
}

// k_stage_check: one wave per (touched stage, 64 budgets of its window), one lane per budget.
// The lowest failing budget of a stage is the minimum over its waves; a wave whose budgets lie
// above a failure already recorded has nothing to add and leaves at once.
__global__ __launch_bounds__(64) void k_stage_check(Tables t, Search s, const int* __restrict__ touched) {
  const int lane = threadIdx.x;
  const int b = touched[blockIdx.y];
  const int bup = s.bup[b];
  const int init = t.E >= bup ? t.E - bup : -1;
  const int base = init + 1 + (int)blockIdx.x * 64;
  if (base > t.E) return;
  if (*(volatile const int*)&s.first_bad[b] < base) return;
  const int e = base + lane;
  bool bad = false;
  if (e <= t.E && t.best[(size_t)b * t.EP + e] != INFINITY) {   // no plan: nothing to check
    const long long ea = plan_e_all(t, s, b, e);
    bad = ea > (long long)t.E || ea < 0;
  }
  const unsigned long long hit = __ballot(bad);
  if (hit && lane == 0) atomicMin(&s.first_bad[b], base + __ffsll((long long)hit) - 1);
}

// One wave per solved stage.  The budget the plan is read at is E, or, with O_b / O_ms
// tables, the last budget below the first failing one that has a plan (E - b_up if there is
// none above it).  The wave walks that plan down the argmin records (every lane the same
// plan; without records the lanes share each step's recomputation) and leaves the strategies
// in the model-wide array, the stage's time, memory and time without gradient
// synchronisation in the pair's stage slots.
__global__ __launch_bounds__(64) void k_stage_result(Tables t, Search s,
                                                     const int* __restrict__ touched, int nt,
                                                     const int* __restrict__ slot_chain,
                                                     const int* __restrict__ slot_first) {
  const int lane = threadIdx.x;
  const int b = touched[blockIdx.x];                       // slot = instance of the table solve
  const int k = slot_chain[b], a = slot_first[b], n = t.L[b], S = t.S;
  const size_t lrow = (size_t)s.lrow[k] + a;
  const int slot = b;
  const int row0 = t.off[b];
  const float* best = t.best + (size_t)b * t.EP;
  uint8_t* st = s.strat + lrow;
  int e_sel = t.E;
  if (s.Ob_g) {
    const int bup = s.bup[b], first_bad = s.first_bad[b];
    const int init = t.E >= bup ? t.E - bup : -1;
    const int last = first_bad == INT_MAX ? t.E : first_bad - 1;
    e_sel = (last > init && best[last] != INFINITY) ? last : init;
  }
  float C = e_sel >= 0 ? best[e_sel] : INFINITY;
  long long mem = 0;
  if (C != INFINITY) {
    int sx = t.best_s[(size_t)b * t.EP + e_sel], e = e_sel;
    long long suf = 0, ms = 0, mx = 0;
    for (int l = n - 1; l >= 0; --l) {
      st[l] = (uint8_t)sx;
      const size_t cell = (size_t)(row0 + l) * S + sx;
      const int m = t.M[cell];
      if (s.Ob_g) {
        const int oms = s.Oms_g[cell];
        const long long here = (long long)s.Ob_g[cell] - suf;
        mx = (l == n - 1 || here > mx) ? here : mx;
        suf += m - oms;
        ms += oms;
      } else {
        suf += m;
      }
      if (l > 0) {
        e -= m;                                            // budget left for layers < l
        if (m < 0 || e < 0) { C = INFINITY; break; }       // only reachable with invalid inputs
        sx = pred_strategy_wave(t, row0 + l, sx, e, lane);
      }
    }
    mem = suf + mx + ms;
  }
  if (C == INFINITY) {
    for (int l = 0; l < n; ++l) st[l] = 0xFF;
    s.stC[slot] = INFINITY;
    s.stCns[slot] = INFINITY;
    s.stO[slot] = -1;
    return;
  }
  float Cns = C;
  if (s.cns) {
    int sp = st[0];
    float v = s.cns[lrow * S + sp];
    for (int l = 1; l < n; ++l) {
      const int sn = st[l];
      const float r = s.R[((lrow + l) * S + sp) * S + sn];
      v = (v + r) + s.cns[(lrow + l) * S + sn];
      sp = sn;
    }
    Cns = v;
  }
  s.stC[slot] = C;
  s.stCns[slot] = Cns;
  s.stO[slot] = (int)mem;
}

// One wave per pair; lane i works on stage i (P <= 64).  phase 0: the searched partition
// was p_t, keep its largest stage memory as limit 3.  phase 1: trace entry for the searched
// partition, then adjust and validate; the accepted partition replaces s.part.
__global__ __launch_bounds__(64) void k_chain_step(Search s, int phase) {
  const int k = blockIdx.x, lane = threadIdx.x;
  if (phase == 1 && !s.live[k]) return;
  const int P = s.P[k], pr = s.prow[k], S = s.S;
  const float* C = s.stC + pr;
  const float* Cns = s.stCns + pr;
  const int* O = s.stO + pr;

  // Eq. 8 and the slowest stage (lowest index among equals): a left fold in stage order,
  // done by every lane alike
  float total = C[0], mx = Cns[0], cmax = C[0];
  int imax = 0, omax = O[0];
  long long osum = O[0];
  for (int i = 1; i < P; ++i) {
    total = total + C[i];
    mx = Cns[i] > mx ? Cns[i] : mx;
    if (C[i] > cmax) { cmax = C[i]; imax = i; }
    omax = O[i] > omax ? O[i] : omax;
    osum += O[i];
  }
  float cost = INFINITY;
  if (total != INFINITY && mx != INFINITY) {
    const float head = (float)(s.m[k] - 1) * mx;
    cost = head + total;
  }
  const bool feasible = cost != INFINITY;
  if (phase == 0) {
    if (lane == 0) s.Ot[k] = feasible ? omax : INT_MAX;
    return;
  }

  int* p = s.part + pr;
  const int it = s.n_iter[k];
  const size_t e1 = (size_t)k * s.max_iter + it, eP = e1 * s.Pmax;
  float a_t = 0.0f, a_m = 0.0f;
  if (feasible) {                                           // Eq. 6
    if (total != 0.0f) a_t = 1.0f - cmax / total;
    if (osum != 0) a_m = (float)(1.0 - (double)omax / (double)osum);
  }
  const bool mine = lane < P;
  const int p_own = mine ? p[lane] : 0;
  if (mine) {
    s.tr_p[eP + lane] = p_own;
    s.tr_C[eP + lane] = C[lane];
    s.tr_Cns[eP + lane] = Cns[lane];
    s.tr_O[eP + lane] = O[lane];
  }
  if (lane == 0) {
    s.tr_cost[e1] = cost;
    s.tr_at[e1] = a_t;
    s.tr_am[e1] = a_m;
    s.n_iter[k] = it + 1;
    s.live[k] = 0;
  }
  if (!feasible || it + 1 >= s.max_iter) return;

  // PP_Partition_Adjust
  if (P < 2 || p[imax] < 2) return;
  int j;
  if (imax == 0) j = 1;
  else if (imax == P - 1) j = P - 2;
  else j = (C[imax + 1] < C[imax - 1]) ? imax + 1 : imax - 1;
  const int q_own = p_own - (lane == imax ? 1 : 0) + (lane == j ? 1 : 0);   // this lane's stage under p'

  // searched before?  (entry `it` is p itself, written above by these same lanes)
  for (int tt = 0; tt < it; ++tt) {
    const int* old = s.tr_p + ((size_t)k * s.max_iter + tt) * s.Pmax;
    const bool differs = mine && old[lane] != q_own;
    if (__ballot(differs) == 0) return;
  }

  // Validate: lane kk evaluates stage kk of the new partition under the strategies just found
  bool ok = true;
  if (mine) {
    int a = 0;                                               // first layer of this lane's stage under p'
    for (int i = 0; i < lane; ++i) a += p[i] - (i == imax ? 1 : 0) + (i == j ? 1 : 0);
    const int Lm = s.Lm[k];
    const size_t lrow = (size_t)s.lrow[k], mr = (size_t)s.mrow[k] + (size_t)lane * Lm;
    const uint8_t* st = s.strat + lrow;
    int sp = st[a];
    float v = s.c[(lrow + a) * S + sp];
    // memory: the sum of M, or with O_b / O_ms tables the overall memory of Eq. 2:
    // max over the layers of (forward activations so far + own backward) + all model states
    long long fwd = 0, ms = 0, peak = 0;
    auto account = [&](int l, int sx) {
      const size_t cell = (mr + l) * S + sx;
      const long long oms = s.Ob ? s.Oms[cell] : 0;
      fwd += s.M[cell] - oms;
      ms += oms;
      const long long here = fwd + (s.Ob ? s.Ob[cell] : 0);
      peak = here > peak ? here : peak;
    };
    account(a, sp);
    for (int l = a + 1; l < a + q_own; ++l) {
      const int sn = st[l];
      const float r = s.R[((lrow + l) * S + sp) * S + sn];
      v = (v + r) + s.c[(lrow + l) * S + sn];
      account(l, sn);
      sp = sn;
    }
    const long long mem = peak + ms;
    ok = v <= cmax && mem <= (long long)s.E && mem <= (long long)s.Ot[k];
  }
  if (__ballot(!ok) != 0) return;
  if (mine) p[lane] = q_own;
  if (lane == 0) {
    s.moved[2 * k] = imax;
    s.moved[2 * k + 1] = j;
    s.live[k] = 1;
  }
}

// Outer loops of Algorithm 1 / 2 on the pairs' final costs (one lane): out[0] = Tpt,
// out[1] = group, out[2] = pair (as int bits).
__global__ void k_throughput(Search s, const float* __restrict__ batch, const int* __restrict__ group,
                             float* __restrict__ out) {
  float tpt = 0.0f;
  int arg_g = -1, arg_k = -1;
  int k = 0;
  while (k < s.n_chain) {
    const int g = group[k];
    float c_opt = INFINITY;
    int k_opt = k;
    const float B = batch[k];
    for (; k < s.n_chain && group[k] == g; ++k) {
      const float cst = s.tr_cost[(size_t)k * s.max_iter + s.n_iter[k] - 1];
      if (cst < c_opt) { c_opt = cst; k_opt = k; }
    }
    if (c_opt == INFINITY) break;                          // out of memory: larger batches are not tried
    const float tp = B / c_opt;
    if (tp > tpt) { tpt = tp; arg_g = g; arg_k = k_opt; }
  }
  out[0] = tpt;
  out[1] = __int_as_float(arg_g);
  out[2] = __int_as_float(arg_k);
}

}  // namespace gbmw

using gbmw_detail::fail;

namespace {

struct Carver {
  char* base;
  size_t used = 0;
  explicit Carver(void* p) : base((char*)p) {}
  template <typename T>
  T* take(size_t n) {
    used = (used + 255) / 256 * 256;
    T* r = base ? (T*)(base + used) : nullptr;
    used += n * sizeof(T);
    return r;
  }
};

struct Dims {
  size_t n, sumP, sumLm, sumPL, S, tr, trP;
};

// The resident copy of the model and of the pairs' descriptions.
struct ModelOnDevice {
  int *P, *Lm, *m, *lrow, *prow, *mrow, *M, *Ob, *Oms;
  float *c, *cns, *R;
  uint32_t* zero_begin;      // the part of the state that starts as zero
  size_t zero_words;
};

// One layout for sizing (base == nullptr) and for carving.
size_t carve_search(Carver& cv, const Dims& d, bool with_cns, bool with_split, gbmw::Search& s,
                    ModelOnDevice& md) {
  md.P = cv.take<int>(d.n); md.Lm = cv.take<int>(d.n); md.m = cv.take<int>(d.n);
  md.lrow = cv.take<int>(d.n); md.prow = cv.take<int>(d.n); md.mrow = cv.take<int>(d.n);
  md.c = cv.take<float>(d.sumLm * d.S);
  md.cns = with_cns ? cv.take<float>(d.sumLm * d.S) : nullptr;
  md.R = cv.take<float>(d.sumLm * d.S * d.S);
  md.M = cv.take<int>(d.sumPL * d.S);
  md.Ob = with_split ? cv.take<int>(d.sumPL * d.S) : nullptr;
  md.Oms = with_split ? cv.take<int>(d.sumPL * d.S) : nullptr;
  s.part = cv.take<int>(d.sumP);
  s.stC = cv.take<float>(d.sumP);
  s.stCns = cv.take<float>(d.sumP);
  s.stO = cv.take<int>(d.sumP);
  s.strat = cv.take<uint8_t>(d.sumLm);
  s.moved = cv.take<int>(2 * d.n);
  s.live = cv.take<int>(d.n);
  s.bup = with_split ? cv.take<int>(d.sumP) : nullptr;
  s.first_bad = with_split ? cv.take<int>(d.sumP) : nullptr;
  // everything from here on starts as zero
  cv.used = (cv.used + 255) / 256 * 256;
  const size_t z0 = cv.used;
  md.zero_begin = cv.base ? (uint32_t*)(cv.base + z0) : nullptr;
  s.n_iter = cv.take<int>(d.n);
  s.Ot = cv.take<int>(d.n);
  s.tr_p = cv.take<int>(d.trP);
  s.tr_O = cv.take<int>(d.trP);
  s.tr_C = cv.take<float>(d.trP);
  s.tr_Cns = cv.take<float>(d.trP);
  s.tr_cost = cv.take<float>(d.tr);
  s.tr_at = cv.take<float>(d.tr);
  s.tr_am = cv.take<float>(d.tr);
  cv.used = (cv.used + 255) / 256 * 256;
  md.zero_words = (cv.used - z0) / 4;
  return cv.used;
}

}  // namespace

extern "C" gbmw_status gbmw_partition_search(const gbmw_partition_problem* q, uint32_t flags,
                                             gbmw_partition_result* out, gbmw_ctx** ctxp) {
  gbmw_detail::clear_error();
  if (!q || !out || !ctxp) return fail(GBMW_ERR_INVALID_ARG, "null problem, result or context pointer");
  if (!q->P || !q->Lm || !q->m || !q->c || !q->R || !q->M || !q->p0)
    return fail(GBMW_ERR_INVALID_ARG, "null P/Lm/m/c/R/M/p0");
  if (!out->n_iter) return fail(GBMW_ERR_INVALID_ARG, "null n_iter output");
  if (q->n_chain < 1 || q->n_chain > 65535) return fail(GBMW_ERR_INVALID_ARG, "n_chain=%d not in 1..65535", q->n_chain);
  if (q->S < 1 || q->S > GBMW_MAX_S) return fail(GBMW_ERR_INVALID_ARG, "S=%d not in 1..256", q->S);
  if (q->E < 0 || q->E > (1 << 28)) return fail(GBMW_ERR_INVALID_ARG, "E=%d out of range", q->E);
  if (q->max_iter < 1 || q->max_iter > 4096) return fail(GBMW_ERR_INVALID_ARG, "max_iter=%d not in 1..4096", q->max_iter);
  if (flags & ~(uint32_t)(GBMW_FLAG_RESOLVE_ALL | GBMW_FLAG_LAZY_ARGMIN | GBMW_FLAG_DENSE_ARITHMETIC))
    return fail(GBMW_ERR_INVALID_ARG, "unknown flag bits 0x%x", flags);

  const int n = q->n_chain, S = q->S, E = q->E;
  std::vector<int> lrow(n), prow(n), mrow(n);
  long long sumLm = 0, sumP = 0, sumPL = 0;
  int Pmax = 0, Lmmax = 0;
  for (int k = 0; k < n; ++k) {
    const int P = q->P[k], Lm = q->Lm[k];
    if (P < 1 || P > 64) return fail(GBMW_ERR_INVALID_ARG, "P[%d]=%d not in 1..64", k, P);
    if (Lm < P) return fail(GBMW_ERR_INVALID_ARG, "Lm[%d]=%d < P=%d", k, Lm, P);
    if (q->m[k] < 1) return fail(GBMW_ERR_INVALID_ARG, "m[%d]=%d < 1", k, q->m[k]);
    lrow[k] = (int)sumLm; prow[k] = (int)sumP; mrow[k] = (int)sumPL;
    sumLm += Lm; sumP += P; sumPL += (long long)P * Lm;
    Pmax = std::max(Pmax, P); Lmmax = std::max(Lmmax, Lm);
    if (sumLm > (1 << 24) || sumPL > (1 << 26)) return fail(GBMW_ERR_INVALID_ARG, "model too large");
    for (const int32_t* part : {q->p0, q->p_t}) {
      if (!part) continue;
      long long sum = 0;
      for (int i = 0; i < P; ++i) {
        if (part[prow[k] + i] < 1)
          return fail(GBMW_ERR_INVALID_ARG, "pair %d: stage %d of %s is empty", k, i, part == q->p0 ? "p0" : "p_t");
        sum += part[prow[k] + i];
      }
      if (sum != Lm)
        return fail(GBMW_ERR_INVALID_ARG, "pair %d: %s sums to %lld, not Lm=%d", k, part == q->p0 ? "p0" : "p_t", sum, Lm);
    }
  }
  if (sumP > 65535) return fail(GBMW_ERR_INVALID_ARG, "more than 65535 stages");
  if ((q->batch_size == nullptr) != (q->batch_group == nullptr))
    return fail(GBMW_ERR_INVALID_ARG, "batch_size and batch_group go together");
  if (q->batch_size)
    for (int k = 0; k < n; ++k) {
      if (!(q->batch_size[k] > 0.0f) || !std::isfinite(q->batch_size[k]))
        return fail(GBMW_ERR_INVALID_ARG, "batch_size[%d] must be positive", k);
      if (k > 0 && q->batch_group[k] < q->batch_group[k - 1])
        return fail(GBMW_ERR_INVALID_ARG, "batch_group must be non-decreasing (pair %d)", k);
      if (k > 0 && q->batch_group[k] == q->batch_group[k - 1] && q->batch_size[k] != q->batch_size[k - 1])
        return fail(GBMW_ERR_INVALID_ARG, "pairs of group %d differ in batch size", q->batch_group[k]);
    }
  const size_t tr = (size_t)n * q->max_iter, trP = tr * Pmax;
  if (trP > ((size_t)1 << 28)) return fail(GBMW_ERR_INVALID_ARG, "trace too large (n_chain * max_iter * Pmax)");
  for (size_t i = 0; i < (size_t)sumLm * S; ++i) {
    if (!(q->c[i] >= 0.0f)) return fail(GBMW_ERR_INVALID_ARG, "c[%zu] is NaN or negative", i);
    if (q->c_nosync && !(q->c_nosync[i] >= 0.0f)) return fail(GBMW_ERR_INVALID_ARG, "c_nosync[%zu] is NaN or negative", i);
  }
  if ((q->O_b == nullptr) != (q->O_ms == nullptr))
    return fail(GBMW_ERR_INVALID_ARG, "O_b and O_ms go together");
  const bool split = q->O_b != nullptr;
  int ob_max = 0;                                    // sizes the range of budgets the final reduce fills
  for (size_t i = 0; i < (size_t)sumPL * S; ++i) {
    if (q->M[i] < 0) return fail(GBMW_ERR_INVALID_ARG, "M[%zu] is negative", i);
    if (split) {
      if (q->O_b[i] < 0) return fail(GBMW_ERR_INVALID_ARG, "O_b[%zu] is negative", i);
      if (q->O_ms[i] < 0 || q->O_ms[i] > q->M[i])
        return fail(GBMW_ERR_INVALID_ARG, "O_ms[%zu] is not in 0..M", i);
      ob_max = std::max(ob_max, q->O_b[i]);
    }
  }
  for (int k = 0; k < n; ++k)          // the slab of the model's first layer is never used
    for (size_t i = ((size_t)lrow[k] + 1) * S * S; i < ((size_t)lrow[k] + q->Lm[k]) * S * S; ++i)
      if (!(q->R[i] >= 0.0f)) return fail(GBMW_ERR_INVALID_ARG, "R[%zu] is NaN or negative", i);

  gbmw_ctx* c = *ctxp;
  const bool fresh = (c == nullptr);
  if (fresh) {
    gbmw_status st = gbmw_detail::new_ctx(&c);
    if (st != GBMW_OK) return st;
  }
  hipEvent_t ev0 = nullptr, ev1 = nullptr;
  auto bail = [&](gbmw_status st) {
    if (ev0) (void)hipEventDestroy(ev0);
    if (ev1) (void)hipEventDestroy(ev1);
    if (fresh) gbmw_destroy(c);
    return st;
  };
#define TRY(expr)                       \
  do {                                  \
    gbmw_status s_ = (expr);            \
    if (s_ != GBMW_OK) return bail(s_); \
  } while (0)
#define HIP_TRY_B(expr)                                                                        \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess) {                                                                    \
      (void)hipGetLastError();                                                                 \
      return bail(fail(e_ == hipErrorOutOfMemory ? GBMW_ERR_OOM : GBMW_ERR_DEVICE, "%s: %s",   \
                       #expr, hipGetErrorString(e_)));                                         \
    }                                                                                          \
  } while (0)

  HIP_TRY_B(hipSetDevice(c->device));
  hipStream_t st = (hipStream_t)q->stream;
  c->solved = false;
  c->index_on_device = false;
  c->stream = st;

  // ---- slots: one per (pair, stage), with room for the longest stage it can become ----
  const int B = (int)sumP;
  std::vector<int> slot_chain(B), slot_stage(B), off(B), cap(B);
  long long rows_total = 0;
  for (int k = 0, b = 0; k < n; ++k)
    for (int i = 0; i < q->P[k]; ++i, ++b) {
      slot_chain[b] = k; slot_stage[b] = i;
      cap[b] = q->Lm[k] - q->P[k] + 1;
      off[b] = (int)rows_total;
      rows_total += cap[b];
    }
  if (rows_total > (1 << 24)) return bail(fail(GBMW_ERR_INVALID_ARG, "too many table rows (%lld)", rows_total));
  const int SP = (S + 3) / 4 * 4, RS = (SP + 2 + 3) / 4 * 4, EP = (E + 1 + 255) / 256 * 256;
  const size_t slab = (size_t)S * EP;

  // ---- device state -------------------------------------------------------
  const Dims d{(size_t)n, (size_t)sumP, (size_t)sumLm, (size_t)sumPL, (size_t)S, tr, trP};
  gbmw::Search s{};
  s.n_chain = n; s.S = S; s.E = E; s.Pmax = Pmax; s.max_iter = q->max_iter;
  ModelOnDevice md{};
  {
    Carver sizing(nullptr);
    TRY(c->d_search.reserve(carve_search(sizing, d, q->c_nosync != nullptr, split, s, md)));
    Carver cv(c->d_search.p);
    carve_search(cv, d, q->c_nosync != nullptr, split, s, md);
  }
  s.P = md.P; s.Lm = md.Lm; s.m = md.m; s.lrow = md.lrow; s.prow = md.prow; s.mrow = md.mrow;
  s.c = md.c; s.cns = md.cns; s.R = md.R; s.M = md.M; s.Ob = md.Ob; s.Oms = md.Oms;
  int *dP = md.P, *dLm = md.Lm, *dm = md.m, *dlrow = md.lrow, *dprow = md.prow, *dmrow = md.mrow, *dM = md.M;
  float *dc = md.c, *dcns = md.cns, *dR = md.R;
  uint32_t* zero_begin = md.zero_begin;
  const size_t zero_words = md.zero_words;

  // rows of the slots (what the layer kernels read) and the per-round index arrays
  const size_t rows = (size_t)rows_total;
  float* gc = nullptr;
  int *gM = nullptr, *g_src = nullptr, *g_msrc = nullptr, *g_dst = nullptr, *g_touched = nullptr,
      *g_chain = nullptr, *g_first = nullptr, *g_group = nullptr;
  float *g_batch = nullptr, *g_tpt = nullptr;
  auto carve_gather = [&](Carver& w) {
    gc = w.take<float>(rows * d.S);
    gM = w.take<int>(rows * d.S);
    s.Ob_g = split ? w.take<int>(rows * d.S) : nullptr;
    s.Oms_g = split ? w.take<int>(rows * d.S) : nullptr;
    g_src = w.take<int>(rows);
    g_msrc = w.take<int>(rows);
    g_dst = w.take<int>(rows);
    g_touched = w.take<int>(d.sumP);
    g_chain = w.take<int>(d.sumP);
    g_first = w.take<int>(d.sumP);
    g_group = w.take<int>(d.n);
    g_batch = w.take<float>(d.n);
    g_tpt = w.take<float>(4);
    return w.used;
  };
  {
    Carver sizing(nullptr);
    TRY(c->d_gather.reserve(carve_gather(sizing)));
    Carver cv(c->d_gather.p);
    carve_gather(cv);
  }
  TRY(c->d_L.reserve(sizeof(int) * B));
  TRY(c->d_off.reserve(sizeof(int) * B));
  TRY(c->d_perm.reserve(sizeof(int) * B));
  TRY(c->d_status.reserve(sizeof(int)));
  TRY(c->d_Rt.reserve(sizeof(float) * rows * S * RS));
  // with argmin records: a rolling pair of fp32 layer tables per slot and one byte per cell of
  // every layer; without: the fp32 tables of all layers
  const bool lazy = (flags & GBMW_FLAG_LAZY_ARGMIN) != 0;
  const bool runs = (flags & GBMW_FLAG_DENSE_ARITHMETIC) == 0 && gbmw::layer0_in_registers(S);
  if (runs) TRY(c->d_sum.reserve(sizeof(float) * ((size_t)S * (EP / 64)) * (lazy ? rows : (size_t)2 * B)));
  if (lazy) {
    TRY(c->d_C.reserve(sizeof(float) * slab * rows));
  } else {
    TRY(c->d_C.reserve(sizeof(float) * slab * 2 * B));
    TRY(c->d_A.reserve(slab * rows));
    if (runs) TRY(c->d_asum.reserve((size_t)S * (EP / 64) * rows));
  }
  TRY(c->d_best.reserve(sizeof(float) * (size_t)B * EP));
  TRY(c->d_best_s.reserve((size_t)B * EP));
  constexpr int kFreshGroups = 2;
  TRY(gbmw_detail::ensure_streams(c, kFreshGroups));

  gbmw::Tables& t = c->t;
  t.B = B; t.S = S; t.SP = SP; t.RS = RS; t.E = E; t.EP = EP; t.keep_all = lazy ? 1 : 0;
  t.runs = runs ? 2 : 0;
  t.Tsum = runs ? (float*)c->d_sum.p : nullptr;
  t.final_from = std::max(0, E - ob_max);              // Algorithm 3 reads best(e) from E - b_up on
  t.L = (const int*)c->d_L.p; t.off = (const int*)c->d_off.p; t.perm = (const int*)c->d_perm.p;
  t.c = gc; t.M = gM; t.Rt = (const float*)c->d_Rt.p;
  t.Cbuf = (float*)c->d_C.p; t.A = lazy ? nullptr : (uint8_t*)c->d_A.p;
  t.Asum = (!lazy && runs) ? (uint8_t*)c->d_asum.p : nullptr;
  t.best = (float*)c->d_best.p; t.best_s = (uint8_t*)c->d_best_s.p;
  t.status = (int*)c->d_status.p;
  t.counts = nullptr;
  t.prev_full = 0;

  HIP_TRY_B(hipEventCreate(&ev0));
  HIP_TRY_B(hipEventCreate(&ev1));
  HIP_TRY_B(hipEventRecord(ev0, st));
  const hipMemcpyKind H2D = hipMemcpyHostToDevice;
  HIP_TRY_B(hipMemcpyAsync(dP, q->P, sizeof(int) * n, H2D, st));
  HIP_TRY_B(hipMemcpyAsync(dLm, q->Lm, sizeof(int) * n, H2D, st));
  HIP_TRY_B(hipMemcpyAsync(dm, q->m, sizeof(int) * n, H2D, st));
  HIP_TRY_B(hipMemcpyAsync(dlrow, lrow.data(), sizeof(int) * n, H2D, st));
  HIP_TRY_B(hipMemcpyAsync(dprow, prow.data(), sizeof(int) * n, H2D, st));
  HIP_TRY_B(hipMemcpyAsync(dmrow, mrow.data(), sizeof(int) * n, H2D, st));
  HIP_TRY_B(hipMemcpyAsync(dc, q->c, sizeof(float) * d.sumLm * S, H2D, st));
  if (dcns) HIP_TRY_B(hipMemcpyAsync(dcns, q->c_nosync, sizeof(float) * d.sumLm * S, H2D, st));
  HIP_TRY_B(hipMemcpyAsync(dR, q->R, sizeof(float) * d.sumLm * S * S, H2D, st));
  HIP_TRY_B(hipMemcpyAsync(dM, q->M, sizeof(int) * d.sumPL * S, H2D, st));
  if (split) {
    HIP_TRY_B(hipMemcpyAsync(md.Ob, q->O_b, sizeof(int) * d.sumPL * S, H2D, st));
    HIP_TRY_B(hipMemcpyAsync(md.Oms, q->O_ms, sizeof(int) * d.sumPL * S, H2D, st));
  }
  HIP_TRY_B(hipMemcpyAsync(s.part, q->p0, sizeof(int) * d.sumP, H2D, st));
  HIP_TRY_B(hipMemcpyAsync(c->d_off.p, off.data(), sizeof(int) * B, H2D, st));
  HIP_TRY_B(hipMemcpyAsync(g_chain, slot_chain.data(), sizeof(int) * B, H2D, st));
  hipLaunchKernelGGL(gbmw::k_fill_u32, dim3((unsigned)((zero_words + 255) / 256)), dim3(256), 0, st,
                     zero_begin, zero_words, 0u);
  hipLaunchKernelGGL(gbmw::k_fill_u32, dim3((unsigned)((d.n + 255) / 256)), dim3(256), 0, st,
                     (uint32_t*)s.live, d.n, 1u);
  hipLaunchKernelGGL(gbmw::k_fill_u32, dim3((unsigned)((d.n + 255) / 256)), dim3(256), 0, st,
                     (uint32_t*)s.Ot, d.n, (uint32_t)INT_MAX);      // no limit 3 until p_t is searched
  hipLaunchKernelGGL(gbmw::k_fill_u32, dim3(1), dim3(256), 0, st, (uint32_t*)c->d_status.p, (size_t)1, 0u);
  // every row of the slots is readable from the start (rows beyond a stage's layers are never used)
  for (auto [ptr, words] : {std::pair<void*, size_t>{gc, rows * d.S}, {gM, rows * d.S},
                            {s.Ob_g, split ? rows * d.S : 0}, {s.Oms_g, split ? rows * d.S : 0},
                            {c->d_Rt.p, rows * d.S * (size_t)RS}})
    if (words) {
      hipLaunchKernelGGL(gbmw::k_fill_u32, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st,
                         (uint32_t*)ptr, words, 0u);
    }
  HIP_TRY_B(hipGetLastError());

  // ---- rounds -------------------------------------------------------------
  enum Mode { kSkip = 0, kFresh = 1, kAppend = 2, kFinalOnly = 3 };
  std::vector<std::vector<int>> part(n);             // host mirror of the partitions
  std::vector<char> live(n, 1);
  // per slot: layers it holds, first model layer, and which of its fp32 layer tables are in
  // memory (the rolling pair keeps the last two computed; hi = -1: none)
  std::vector<int> slotL(B, 0), slot_first(B, 0), c_hi(B, -1), c_lo(B, -1), mode(B, kSkip);
  std::vector<char> last_full(B, 0);                 // the slot's newest table has every cell written
  std::vector<int> h_src, h_msrc, h_dst, h_touched, h_perm, h_flags(3 * (size_t)n);
  int rounds = 0, stage_solves = 0;
  long long cell_updates = 0;
  const bool l0_in_regs = gbmw::layer0_in_registers(S);

  // One round: the slots with mode != kSkip get their new layer count slotL / first layer
  // slot_first, are brought up to date and read back into the pairs' stage results.
  auto run_round = [&](int phase) -> gbmw_status {
    h_src.clear(); h_msrc.clear(); h_dst.clear(); h_touched.clear();
    std::vector<int> fresh, append, final_only;
    for (int b = 0; b < B; ++b) {
      if (mode[b] == kSkip) continue;
      const int k = slot_chain[b], i = slot_stage[b], L = slotL[b];
      h_touched.push_back(b);
      if (mode[b] == kFresh) {
        fresh.push_back(b);
        for (int l = 0; l < L; ++l) {
          h_src.push_back(lrow[k] + slot_first[b] + l);
          h_msrc.push_back(mrow[k] + i * q->Lm[k] + slot_first[b] + l);
          h_dst.push_back(off[b] + l);
        }
        cell_updates += (long long)(L - 1) * (E + 1) * S * S;
        // what a complete solve leaves in the rolling pair: L-1 and L-2, layer 0 only if it
        // was written to memory (stages of one or two layers, or S > 64)
        c_hi[b] = L - 1;
        c_lo[b] = (L >= 2 && (L - 2 >= 1 || L <= 2 || !l0_in_regs)) ? L - 2 : -1;
        if (lazy) c_lo[b] = 0;                       // every layer's table is kept: [c_lo, c_hi]
      } else if (mode[b] == kAppend) {
        append.push_back(b);
        h_src.push_back(lrow[k] + slot_first[b] + L - 1);
        h_msrc.push_back(mrow[k] + i * q->Lm[k] + slot_first[b] + L - 1);
        h_dst.push_back(off[b] + L - 1);
        cell_updates += (long long)(E + 1) * S * S;
        if (!lazy) c_lo[b] = L - 2;
        c_hi[b] = L - 1;
      } else {
        final_only.push_back(b);
        last_full[b] = 0;                            // its newest table is now an older one
      }
    }
    const int nt = (int)h_touched.size();
    if (nt == 0) return GBMW_OK;
    ++rounds;
    stage_solves += nt;
    // launch order: two groups of complete solves (longest first, dealt alternately), the
    // one-step slots ordered by their layer index, the reduce-only slots
    auto longer = [&](int a2, int b2) { return slotL[a2] > slotL[b2]; };
    std::stable_sort(fresh.begin(), fresh.end(), longer);
    std::stable_sort(append.begin(), append.end(), longer);
    const int G = std::max(1, std::min(kFreshGroups, (int)fresh.size()));
    h_perm.clear();
    std::vector<int> gfirst(G + 1, 0);
    for (int g = 0; g < G; ++g) {
      gfirst[g] = (int)h_perm.size();
      for (size_t x = g; x < fresh.size(); x += G) h_perm.push_back(fresh[x]);
    }
    gfirst[G] = (int)h_perm.size();
    const int a_first = (int)h_perm.size();
    h_perm.insert(h_perm.end(), append.begin(), append.end());
    h_perm.insert(h_perm.end(), final_only.begin(), final_only.end());

    const int nrows = (int)h_src.size();
    HIP_TRY(hipMemcpyAsync(c->d_L.p, slotL.data(), sizeof(int) * B, H2D, st));
    HIP_TRY(hipMemcpyAsync(c->d_perm.p, h_perm.data(), sizeof(int) * h_perm.size(), H2D, st));
    HIP_TRY(hipMemcpyAsync(g_first, slot_first.data(), sizeof(int) * B, H2D, st));
    HIP_TRY(hipMemcpyAsync(g_touched, h_touched.data(), sizeof(int) * nt, H2D, st));
    if (nrows) {
      HIP_TRY(hipMemcpyAsync(g_src, h_src.data(), sizeof(int) * nrows, H2D, st));
      HIP_TRY(hipMemcpyAsync(g_msrc, h_msrc.data(), sizeof(int) * nrows, H2D, st));
      HIP_TRY(hipMemcpyAsync(g_dst, h_dst.data(), sizeof(int) * nrows, H2D, st));
      hipLaunchKernelGGL(gbmw::k_gather, dim3(nrows), dim3(256), 0, st, dc, dM, dR, g_src, g_msrc, g_dst, S,
                         SP, RS, gc, gM, (float*)c->d_Rt.p, s.Ob, s.Oms, s.Ob_g, s.Oms_g);
    }
    // layer 0 goes to memory where something reads it from there
    for (int g = 0; g < G; ++g) {
      int n_init = gfirst[g + 1] - gfirst[g];
      if (l0_in_regs && !lazy) {
        n_init = 0;
        for (int x = gfirst[g + 1] - 1; x >= gfirst[g] && slotL[h_perm[x]] <= 2; --x) ++n_init;
      }
      gbmw::launch_init_layer0(t, gfirst[g + 1] - n_init, n_init, st);
    }
    HIP_TRY(hipGetLastError());
    if (G > 1) HIP_TRY(hipEventRecord(c->ev_fork, st));
    for (int g = 0; g < G; ++g) {
      hipStream_t sg = (g == 0) ? st : c->aux[g - 1];
      if (g > 0) HIP_TRY(hipStreamWaitEvent(sg, c->ev_fork, 0));
      if (g == G - 1) {
        // the one-step slots: all slots whose new last layer has the same index share a launch
        for (size_t x = 0; x < append.size();) {
          size_t y = x;
          while (y < append.size() && slotL[append[y]] == slotL[append[x]]) ++y;
          // the kept table that the step extends: every cell written if all of these slots got
          // theirs from a split launch
          bool all_full = true;
          for (size_t z = x; z < y; ++z) all_full = all_full && last_full[append[z]];
          gbmw::launch_minplus(t, slotL[append[x]] - 1, a_first + (int)x, (int)(y - x), sg, all_full ? -1 : 0);
          const bool now_full = gbmw::launch_is_split(t, (int)(y - x));
          for (size_t z = x; z < y; ++z) last_full[append[z]] = now_full;
          x = y;
        }
        gbmw::launch_final(t, a_first, (int)h_perm.size() - a_first, sg);
      }
      const int gn = gfirst[g + 1] - gfirst[g];
      const int Lmax_g = gn ? slotL[h_perm[gfirst[g]]] : 0;
      int n_prev = 0;                                      // a complete solve: layer l - 1 comes from the launch before
      for (int l = 1; l < Lmax_g; ++l) {
        int na = 0;
        while (na < gn && slotL[h_perm[gfirst[g] + na]] > l) ++na;
        gbmw::launch_minplus(t, l, gfirst[g], na, sg, n_prev);
        n_prev = na;
        // the slots whose last layer this launch produced
        for (int x = 0; x < na; ++x)
          if (slotL[h_perm[gfirst[g] + x]] == l + 1) last_full[h_perm[gfirst[g] + x]] = gbmw::launch_is_split(t, na);
      }
      gbmw::launch_final(t, gfirst[g], gn, sg);
      if (g > 0) {
        HIP_TRY(hipEventRecord(c->ev_join[g - 1], sg));
        HIP_TRY(hipStreamWaitEvent(st, c->ev_join[g - 1], 0));
      }
    }
    if (split) {
      const int window = std::min(ob_max, E + 1);      // budgets above E - b_up, at most
      hipLaunchKernelGGL(gbmw::k_stage_bup, dim3(nt), dim3(64), 0, st, t, s, g_touched);
      if (window > 0) {
        hipLaunchKernelGGL(gbmw::k_stage_check, dim3((window + 63) / 64, nt), dim3(64), 0, st, t, s, g_touched);
      }
    }
    hipLaunchKernelGGL(gbmw::k_stage_result, dim3(nt), dim3(64), 0, st, t, s, g_touched, nt,
                       g_chain, g_first);
    hipLaunchKernelGGL(gbmw::k_chain_step, dim3(n), dim3(64), 0, st, s, phase);
    HIP_TRY(hipGetLastError());
    // accept flags: live | moved (two per pair); the wait also ends the round for the host vectors
    HIP_TRY(hipMemcpyAsync(h_flags.data(), s.live, sizeof(int) * n, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(h_flags.data() + n, s.moved, sizeof(int) * 2 * n, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    return GBMW_OK;
  };

  // every stage of every pair from scratch, under the partitions `part`
  auto all_fresh = [&]() {
    for (int k = 0; k < n; ++k) {
      int a = 0;
      for (int i = 0; i < q->P[k]; ++i) {
        const int b = prow[k] + i;
        mode[b] = kFresh; slotL[b] = part[k][i]; slot_first[b] = a;
        a += part[k][i];
      }
    }
  };
  if (q->p_t) {
    for (int k = 0; k < n; ++k) part[k].assign(q->p_t + prow[k], q->p_t + prow[k] + q->P[k]);
    all_fresh();
    TRY(run_round(0));
  }
  for (int k = 0; k < n; ++k) part[k].assign(q->p0 + prow[k], q->p0 + prow[k] + q->P[k]);
  all_fresh();
  const bool resolve_all = (flags & GBMW_FLAG_RESOLVE_ALL) != 0;
  // is the fp32 table of layer `layer` of slot b still in memory?
  auto in_memory = [&](int b, int layer) {
    return lazy ? (c_lo[b] <= layer && layer <= c_hi[b]) : (layer == c_hi[b] || layer == c_lo[b]);
  };
  for (int it = 0; it < q->max_iter; ++it) {
    TRY(run_round(1));
    std::fill(mode.begin(), mode.end(), (int)kSkip);
    bool any = false;
    for (int k = 0; k < n; ++k) {
      if (!live[k]) continue;
      live[k] = (char)(h_flags[k] != 0);
      if (!live[k]) continue;
      const int i = h_flags[n + 2 * k], j = h_flags[n + 2 * k + 1];
      if (i < 0 || i >= q->P[k] || j < 0 || j >= q->P[k] || (j != i - 1 && j != i + 1) || part[k][i] < 2)
        return bail(fail(GBMW_ERR_DEVICE, "pair %d: inconsistent adjustment (%d -> %d)", k, i, j));
      part[k][i] -= 1;
      part[k][j] += 1;
      any = true;
      const int bi = prow[k] + i, bj = prow[k] + j;
      slotL[bi] -= 1;
      slotL[bj] += 1;
      if (resolve_all) {
        for (int x = 0; x < q->P[k]; ++x) mode[prow[k] + x] = kFresh;
      } else if (j == i - 1) {
        // the earlier stage takes the first layer of stage i: one more step at its end
        const int need = slotL[bj] - 2;              // the table the new last layer is computed from
        mode[bj] = in_memory(bj, need) ? kAppend : kFresh;
        mode[bi] = kFresh;
      } else {
        // the later stage takes the last layer of stage i: stage i's table is a prefix of itself
        const int need = slotL[bi] - 1;
        mode[bi] = in_memory(bi, need) ? kFinalOnly : kFresh;
        mode[bj] = kFresh;
      }
      if (j == i - 1) slot_first[bi] += 1; else slot_first[bj] -= 1;
    }
    if (!any) break;
  }
  float h_tpt[3] = {0.0f, 0.0f, 0.0f};
  if (q->batch_size) {
    float* d_batch = g_batch;
    int* d_group = g_group;
    float* d_out = g_tpt;
    HIP_TRY_B(hipMemcpyAsync(d_batch, q->batch_size, sizeof(float) * n, H2D, st));
    HIP_TRY_B(hipMemcpyAsync(d_group, q->batch_group, sizeof(int) * n, H2D, st));
    hipLaunchKernelGGL(gbmw::k_throughput, dim3(1), dim3(1), 0, st, s, d_batch, d_group, d_out);
    HIP_TRY_B(hipGetLastError());
    HIP_TRY_B(hipMemcpyAsync(h_tpt, d_out, sizeof(h_tpt), hipMemcpyDeviceToHost, st));
  }
  HIP_TRY_B(hipEventRecord(ev1, st));

  // ---- results ------------------------------------------------------------
  const hipMemcpyKind D2H = hipMemcpyDeviceToHost;
  HIP_TRY_B(hipMemcpyAsync(out->n_iter, s.n_iter, sizeof(int) * n, D2H, st));
  if (out->O_t) HIP_TRY_B(hipMemcpyAsync(out->O_t, s.Ot, sizeof(int) * n, D2H, st));
  if (out->p) HIP_TRY_B(hipMemcpyAsync(out->p, s.tr_p, sizeof(int) * trP, D2H, st));
  if (out->O) HIP_TRY_B(hipMemcpyAsync(out->O, s.tr_O, sizeof(int) * trP, D2H, st));
  if (out->C) HIP_TRY_B(hipMemcpyAsync(out->C, s.tr_C, sizeof(float) * trP, D2H, st));
  if (out->Cns) HIP_TRY_B(hipMemcpyAsync(out->Cns, s.tr_Cns, sizeof(float) * trP, D2H, st));
  if (out->cost) HIP_TRY_B(hipMemcpyAsync(out->cost, s.tr_cost, sizeof(float) * tr, D2H, st));
  if (out->alpha_t) HIP_TRY_B(hipMemcpyAsync(out->alpha_t, s.tr_at, sizeof(float) * tr, D2H, st));
  if (out->alpha_m) HIP_TRY_B(hipMemcpyAsync(out->alpha_m, s.tr_am, sizeof(float) * tr, D2H, st));
  std::vector<uint8_t> h_strat;
  if (out->strat) {
    h_strat.resize(d.sumLm);
    HIP_TRY_B(hipMemcpyAsync(h_strat.data(), s.strat, d.sumLm, D2H, st));
  }
  HIP_TRY_B(hipStreamSynchronize(st));
  if (out->strat) {
    memset(out->strat, 0xFF, (size_t)n * Lmmax);
    for (int k = 0; k < n; ++k)
      memcpy(out->strat + (size_t)k * Lmmax, h_strat.data() + lrow[k], (size_t)q->Lm[k]);
  }
  float ms = 0.0f;
  HIP_TRY_B(hipEventElapsedTime(&ms, ev0, ev1));
  out->rounds = rounds;
  out->stage_solves = stage_solves;
  out->cell_updates = cell_updates;
  out->device_ms = ms;
  out->tpt = h_tpt[0];
  out->tpt_group = -1;
  out->tpt_pair = -1;
  if (q->batch_size) {
    memcpy(&out->tpt_group, &h_tpt[1], sizeof(int));
    memcpy(&out->tpt_pair, &h_tpt[2], sizeof(int));
  }
  (void)hipEventDestroy(ev0);
  (void)hipEventDestroy(ev1);
#undef TRY
#undef HIP_TRY_B
  // the context's layout now belongs to this search: an ordinary solve re-creates its own
  c->B = 0; c->L.clear(); c->off.clear(); c->perm.clear();
  *ctxp = c;
  return GBMW_OK;
}
