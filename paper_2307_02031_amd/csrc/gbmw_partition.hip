// Algorithm 2's inner loop (bi-objective pipeline-partition search, Section 4.2.2
// and Appendix B) for many (batch size, PP degree) pairs in lockstep.  See
// include/gbmw.h for the contract.
//
// Per round the host only decides WHICH stages are solved (it mirrors the
// partitions from the accept flags it reads back); everything that produces a
// value runs in kernels:
//   k_gather        rows of the resident model -> the batch the table solve reads
//   (table solve)   gbmw_dp_solve_batched on device pointers
//   k_stage_result  plan at e = E of every solved stage -> strategies, C, Cns, O
//   k_chain_step    Eq. 8, Eq. 6, PP_Partition_Adjust, Validate, trace entry
#include <algorithm>
#include <climits>
#include <cmath>
#include <cstring>
#include <vector>

#include "gbmw_ctx.h"

namespace gbmw {

struct Search {
  int n_chain, S, E, Pmax, max_iter;
  const int *P, *Lm, *m, *lrow, *prow, *mrow;      // [n_chain]
  const float *c, *cns, *R;                        // resident model (cns may be null)
  const int* M;
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

// one workgroup per batch row: c, M and the S x S slab of R of its source layer
__global__ __launch_bounds__(256) void k_gather(const float* __restrict__ c,
                                                const int* __restrict__ M,
                                                const float* __restrict__ R,
                                                const int* __restrict__ row_src,
                                                const int* __restrict__ row_msrc, int S,
                                                float* __restrict__ c_g, int* __restrict__ M_g,
                                                float* __restrict__ R_g) {
  const int r = blockIdx.x;
  const size_t src = (size_t)row_src[r], msrc = (size_t)row_msrc[r];
  for (int i = threadIdx.x; i < S; i += 256) {
    c_g[(size_t)r * S + i] = c[src * S + i];
    M_g[(size_t)r * S + i] = M[msrc * S + i];
  }
  const int SS = S * S;
  for (int i = threadIdx.x; i < SS; i += 256) R_g[(size_t)r * SS + i] = R[src * SS + i];
}

// One lane per solved stage: walk its plan at e = E down the argmin records,
// leave the strategies in the model-wide array, the stage's time, memory and
// time without gradient synchronisation in the pair's stage slots.
__global__ __launch_bounds__(64) void k_stage_result(Tables t, Search s,
                                                     const int* __restrict__ inst_chain,
                                                     const int* __restrict__ inst_stage,
                                                     const int* __restrict__ inst_first, int nb) {
  const int b = blockIdx.x * 64 + threadIdx.x;
  if (b >= nb) return;
  const int k = inst_chain[b], i = inst_stage[b], a = inst_first[b], n = t.L[b], S = t.S;
  const size_t lrow = (size_t)s.lrow[k] + a;
  const int slot = s.prow[k] + i;
  uint8_t* st = s.strat + lrow;
  float C = t.best[(size_t)b * t.EP + t.E];
  int mem = 0;
  if (C != INFINITY) {
    int sx = t.best_s[(size_t)b * t.EP + t.E], e = t.E;
    const int row0 = t.off[b];
    for (int l = n - 1; l >= 1; --l) {
      st[l] = (uint8_t)sx;
      const int m = t.M[(size_t)(row0 + l) * S + sx];
      mem += m;
      e -= m;                                            // budget left for layers < l
      if (m < 0 || e < 0) { C = INFINITY; break; }       // only reachable with invalid inputs
      sx = t.A[((size_t)(row0 + l) * S + sx) * t.EP + e];
    }
    if (C != INFINITY) {
      st[0] = (uint8_t)sx;
      mem += t.M[(size_t)row0 * S + sx];
    }
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
  s.stO[slot] = mem;
}

// One lane per pair.  phase 0: the searched partition was p_t, keep its largest
// stage memory as limit 3.  phase 1: trace entry for the searched partition,
// then adjust and validate; the accepted partition replaces s.part.
__global__ __launch_bounds__(64) void k_chain_step(Search s, int phase) {
  const int k = blockIdx.x * 64 + threadIdx.x;
  if (k >= s.n_chain) return;
  if (phase == 1 && !s.live[k]) return;
  const int P = s.P[k], pr = s.prow[k], S = s.S;
  const float* C = s.stC + pr;
  const float* Cns = s.stCns + pr;
  const int* O = s.stO + pr;

  // Eq. 8 and the slowest stage (lowest index among equals)
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
    s.Ot[k] = feasible ? omax : INT_MAX;
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
  for (int i = 0; i < P; ++i) {
    s.tr_p[eP + i] = p[i];
    s.tr_C[eP + i] = C[i];
    s.tr_Cns[eP + i] = Cns[i];
    s.tr_O[eP + i] = O[i];
  }
  s.tr_cost[e1] = cost;
  s.tr_at[e1] = a_t;
  s.tr_am[e1] = a_m;
  s.n_iter[k] = it + 1;
  s.live[k] = 0;
  if (!feasible || it + 1 >= s.max_iter) return;

  // PP_Partition_Adjust
  if (P < 2 || p[imax] < 2) return;
  int j;
  if (imax == 0) j = 1;
  else if (imax == P - 1) j = P - 2;
  else j = (C[imax + 1] < C[imax - 1]) ? imax + 1 : imax - 1;
  auto q = [&](int i) { return p[i] - (i == imax ? 1 : 0) + (i == j ? 1 : 0); };

  // searched before?
  for (int tt = 0; tt <= it; ++tt) {
    const int* old = s.tr_p + ((size_t)k * s.max_iter + tt) * s.Pmax;
    bool same = true;
    for (int i = 0; i < P; ++i) same = same && (old[i] == q(i));
    if (same) return;
  }

  // Validate: every stage of the new partition under the strategies just found
  const int Lm = s.Lm[k];
  const size_t lrow = (size_t)s.lrow[k], mrow = (size_t)s.mrow[k];
  const uint8_t* st = s.strat + lrow;
  const long long Ot = s.Ot[k];
  int a = 0;
  for (int kk = 0; kk < P; ++kk) {
    const int n = q(kk);
    const size_t mr = mrow + (size_t)kk * Lm;
    int sp = st[a];
    float v = s.c[(lrow + a) * S + sp];
    long long mem = s.M[(mr + a) * S + sp];
    for (int l = a + 1; l < a + n; ++l) {
      const int sn = st[l];
      const float r = s.R[((lrow + l) * S + sp) * S + sn];
      v = (v + r) + s.c[(lrow + l) * S + sn];
      mem += s.M[(mr + l) * S + sn];
      sp = sn;
    }
    if (!(v <= cmax && mem <= (long long)s.E && mem <= Ot)) return;
    a += n;
  }
  for (int i = 0; i < P; ++i) {
    const int qi = q(i);
    p[i] = qi;
  }
  s.moved[2 * k] = imax;
  s.moved[2 * k + 1] = j;
  s.live[k] = 1;
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

// One layout for sizing (base == nullptr) and for carving.
size_t carve_search(Carver& cv, const Dims& d, bool with_cns, gbmw::Search& s, int*& dP, int*& dLm,
                    int*& dm, int*& dlrow, int*& dprow, int*& dmrow, float*& dc, float*& dcns,
                    float*& dR, int*& dM, uint32_t*& zero_begin, size_t& zero_words) {
  dP = cv.take<int>(d.n); dLm = cv.take<int>(d.n); dm = cv.take<int>(d.n);
  dlrow = cv.take<int>(d.n); dprow = cv.take<int>(d.n); dmrow = cv.take<int>(d.n);
  dc = cv.take<float>(d.sumLm * d.S);
  dcns = with_cns ? cv.take<float>(d.sumLm * d.S) : nullptr;
  dR = cv.take<float>(d.sumLm * d.S * d.S);
  dM = cv.take<int>(d.sumPL * d.S);
  s.part = cv.take<int>(d.sumP);
  s.stC = cv.take<float>(d.sumP);
  s.stCns = cv.take<float>(d.sumP);
  s.stO = cv.take<int>(d.sumP);
  s.strat = cv.take<uint8_t>(d.sumLm);
  s.moved = cv.take<int>(2 * d.n);
  s.live = cv.take<int>(d.n);
  // everything from here on starts as zero
  cv.used = (cv.used + 255) / 256 * 256;
  const size_t z0 = cv.used;
  zero_begin = cv.base ? (uint32_t*)(cv.base + z0) : nullptr;
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
  zero_words = (cv.used - z0) / 4;
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
  if (flags & ~(uint32_t)GBMW_FLAG_RESOLVE_ALL) return fail(GBMW_ERR_INVALID_ARG, "unknown flag bits 0x%x", flags);

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
  const size_t tr = (size_t)n * q->max_iter, trP = tr * Pmax;
  if (trP > ((size_t)1 << 28)) return fail(GBMW_ERR_INVALID_ARG, "trace too large (n_chain * max_iter * Pmax)");
  for (size_t i = 0; i < (size_t)sumLm * S; ++i) {
    if (!(q->c[i] >= 0.0f)) return fail(GBMW_ERR_INVALID_ARG, "c[%zu] is NaN or negative", i);
    if (q->c_nosync && !(q->c_nosync[i] >= 0.0f)) return fail(GBMW_ERR_INVALID_ARG, "c_nosync[%zu] is NaN or negative", i);
  }
  for (size_t i = 0; i < (size_t)sumPL * S; ++i)
    if (q->M[i] < 0) return fail(GBMW_ERR_INVALID_ARG, "M[%zu] is negative", i);
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

  // ---- device state -------------------------------------------------------
  const Dims d{(size_t)n, (size_t)sumP, (size_t)sumLm, (size_t)sumPL, (size_t)S, tr, trP};
  gbmw::Search s{};
  s.n_chain = n; s.S = S; s.E = E; s.Pmax = Pmax; s.max_iter = q->max_iter;
  int *dP, *dLm, *dm, *dlrow, *dprow, *dmrow, *dM;
  float *dc, *dcns, *dR;
  uint32_t* zero_begin;
  size_t zero_words;
  {
    Carver sizing(nullptr);
    const size_t bytes = carve_search(sizing, d, q->c_nosync != nullptr, s, dP, dLm, dm, dlrow, dprow,
                                      dmrow, dc, dcns, dR, dM, zero_begin, zero_words);
    TRY(c->d_search.reserve(bytes));
    Carver cv(c->d_search.p);
    carve_search(cv, d, q->c_nosync != nullptr, s, dP, dLm, dm, dlrow, dprow, dmrow, dc, dcns, dR, dM,
                 zero_begin, zero_words);
  }
  s.P = dP; s.Lm = dLm; s.m = dm; s.lrow = dlrow; s.prow = dprow; s.mrow = dmrow;
  s.c = dc; s.cns = dcns; s.R = dR; s.M = dM;

  // per-round batch: gathered inputs and the index arrays that describe it
  float *gc = nullptr, *gR = nullptr;
  int *gM = nullptr, *g_src = nullptr, *g_msrc = nullptr, *g_chain = nullptr, *g_stage = nullptr,
      *g_first = nullptr;
  auto carve_gather = [&](Carver& w) {
    gc = w.take<float>(d.sumLm * d.S);
    gM = w.take<int>(d.sumLm * d.S);
    gR = w.take<float>(d.sumLm * d.S * d.S);
    g_src = w.take<int>(d.sumLm);
    g_msrc = w.take<int>(d.sumLm);
    g_chain = w.take<int>(d.sumP);
    g_stage = w.take<int>(d.sumP);
    g_first = w.take<int>(d.sumP);
    return w.used;
  };
  {
    Carver sizing(nullptr);
    TRY(c->d_gather.reserve(carve_gather(sizing)));
    Carver cv(c->d_gather.p);
    carve_gather(cv);
  }

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
  HIP_TRY_B(hipMemcpyAsync(s.part, q->p0, sizeof(int) * d.sumP, H2D, st));
  hipLaunchKernelGGL(gbmw::k_fill_u32, dim3((unsigned)((zero_words + 255) / 256)), dim3(256), 0, st,
                     zero_begin, zero_words, 0u);
  hipLaunchKernelGGL(gbmw::k_fill_u32, dim3((unsigned)((d.n + 255) / 256)), dim3(256), 0, st,
                     (uint32_t*)s.live, d.n, 1u);
  hipLaunchKernelGGL(gbmw::k_fill_u32, dim3((unsigned)((d.n + 255) / 256)), dim3(256), 0, st,
                     (uint32_t*)s.Ot, d.n, (uint32_t)INT_MAX);      // no limit 3 until p_t is searched
  HIP_TRY_B(hipGetLastError());

  // ---- rounds -------------------------------------------------------------
  std::vector<std::vector<int>> part(n);             // host mirror of the partitions
  std::vector<char> live(n, 1);
  std::vector<int> h_L, h_src, h_msrc, h_chain, h_stage, h_first, h_flags(3 * (size_t)n);
  int rounds = 0, stage_solves = 0;
  long long cell_updates = 0;

  // stages[k]: which stages of pair k are solved this round, under partition pp[k]
  auto run_round = [&](const std::vector<std::vector<int>>& pp, const std::vector<std::vector<int>>& stages,
                       int phase) -> gbmw_status {
    h_L.clear(); h_src.clear(); h_msrc.clear(); h_chain.clear(); h_stage.clear(); h_first.clear();
    for (int k = 0; k < n; ++k) {
      if (stages[k].empty()) continue;
      std::vector<int> first(pp[k].size(), 0);
      for (size_t i = 1; i < pp[k].size(); ++i) first[i] = first[i - 1] + pp[k][i - 1];
      for (int i : stages[k]) {
        h_chain.push_back(k); h_stage.push_back(i); h_first.push_back(first[i]); h_L.push_back(pp[k][i]);
        for (int l = first[i]; l < first[i] + pp[k][i]; ++l) {
          h_src.push_back(lrow[k] + l);
          h_msrc.push_back(mrow[k] + i * q->Lm[k] + l);
        }
        cell_updates += (long long)(pp[k][i] - 1) * (E + 1) * S * S;
      }
    }
    const int nb = (int)h_L.size(), rows = (int)h_src.size();
    if (nb == 0) return GBMW_OK;
    ++rounds;
    stage_solves += nb;
    HIP_TRY(hipMemcpyAsync(g_src, h_src.data(), sizeof(int) * rows, H2D, st));
    HIP_TRY(hipMemcpyAsync(g_msrc, h_msrc.data(), sizeof(int) * rows, H2D, st));
    HIP_TRY(hipMemcpyAsync(g_chain, h_chain.data(), sizeof(int) * nb, H2D, st));
    HIP_TRY(hipMemcpyAsync(g_stage, h_stage.data(), sizeof(int) * nb, H2D, st));
    HIP_TRY(hipMemcpyAsync(g_first, h_first.data(), sizeof(int) * nb, H2D, st));
    hipLaunchKernelGGL(gbmw::k_gather, dim3(rows), dim3(256), 0, st, dc, dM, dR, g_src, g_msrc, S, gc, gM, gR);
    HIP_TRY(hipGetLastError());
    gbmw_problem pr{};
    pr.B = nb; pr.S = S; pr.E = E; pr.L = h_L.data();
    pr.c = gc; pr.M = gM; pr.R = gR; pr.ptr_space = GBMW_PTR_DEVICE; pr.stream = st;
    gbmw_ctx* cc = c;
    gbmw_status rs = gbmw_detail::solve_batched(&pr, 0, &cc, E);   // only best(E) is read
    if (rs != GBMW_OK) return rs;
    c->solved = false;                                 // the tables are an intermediate of this call
    hipLaunchKernelGGL(gbmw::k_stage_result, dim3((nb + 63) / 64), dim3(64), 0, st, c->t, s, g_chain,
                       g_stage, g_first, nb);
    hipLaunchKernelGGL(gbmw::k_chain_step, dim3((n + 63) / 64), dim3(64), 0, st, s, phase);
    HIP_TRY(hipGetLastError());
    // accept flags: live | moved (two per pair); also ends the round for the host vectors above
    HIP_TRY(hipMemcpyAsync(h_flags.data(), s.live, sizeof(int) * n, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(h_flags.data() + n, s.moved, sizeof(int) * 2 * n, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    return GBMW_OK;
  };

  std::vector<std::vector<int>> stages(n);
  if (q->p_t) {
    for (int k = 0; k < n; ++k) {
      part[k].assign(q->p_t + prow[k], q->p_t + prow[k] + q->P[k]);
      stages[k].resize(q->P[k]);
      for (int i = 0; i < q->P[k]; ++i) stages[k][i] = i;
    }
    TRY(run_round(part, stages, 0));
  }
  for (int k = 0; k < n; ++k) {
    part[k].assign(q->p0 + prow[k], q->p0 + prow[k] + q->P[k]);
    stages[k].resize(q->P[k]);
    for (int i = 0; i < q->P[k]; ++i) stages[k][i] = i;
  }
  const bool resolve_all = (flags & GBMW_FLAG_RESOLVE_ALL) != 0;
  for (int it = 0; it < q->max_iter; ++it) {
    TRY(run_round(part, stages, 1));
    bool any = false;
    for (int k = 0; k < n; ++k) {
      stages[k].clear();
      if (!live[k]) continue;
      live[k] = (char)(h_flags[k] != 0);
      if (!live[k]) continue;
      const int i = h_flags[n + 2 * k], j = h_flags[n + 2 * k + 1];
      if (i < 0 || i >= q->P[k] || j < 0 || j >= q->P[k] || part[k][i] < 2)
        return bail(fail(GBMW_ERR_DEVICE, "pair %d: inconsistent adjustment (%d -> %d)", k, i, j));
      part[k][i] -= 1;
      part[k][j] += 1;
      if (resolve_all) {
        for (int x = 0; x < q->P[k]; ++x) stages[k].push_back(x);
      } else {
        stages[k].push_back(std::min(i, j));
        stages[k].push_back(std::max(i, j));
      }
      any = true;
    }
    if (!any) break;
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
  {
    int status = 0;
    HIP_TRY_B(hipMemcpy(&status, c->t.status, sizeof(int), hipMemcpyDeviceToHost));
    if (status) return bail(fail(GBMW_ERR_INVALID_ARG, "device-side input check failed (0x%x)", status));
  }
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
  (void)hipEventDestroy(ev0);
  (void)hipEventDestroy(ev1);
#undef TRY
#undef HIP_TRY_B
  *ctxp = c;
  return GBMW_OK;
}
