/*
 * CPU oracle for the layer-wise strategy search -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain reference that the GPU library is checked
 * against.  It is used by tests/, by the smoke check and by the benchmark's
 * CPU-baseline leg; the product path never calls it, and it shares no code
 * with the HIP sources.
 *
 * What it computes (paper: Section 4.1.2, Eq. 3; Appendix A, Algorithm 3):
 * for a pipeline stage of L layers, a strategy set of size S and a forward
 * memory budget of E units, the minimum total execution time when every layer
 * l picks one strategy s_l, subject to sum_l M[l][s_l] <= e, for EVERY budget
 * e = 0..E at once, together with the argmin records needed to read the plan
 * back.  M[l][s] is the paper's O_f(l,s) + O_ms(l,s) (the amount Eq. 3
 * subtracts from E_fwd), c[l][s] is c(l, S_j) and R[l][s'][s] is
 * R(l, S_i, S_j), the layout-transformation cost between layer l-1 under s'
 * and layer l under s.
 *
 * Eq. 3 writes its state as C(L, E_fwd) although R needs the previous layer's
 * strategy; the state used here carries it:  C[l][e][s] = best time of layers
 * 0..l with layer l under s and total forward memory <= e.
 *
 * Arithmetic contract: IEEE binary32, round-to-nearest-even, two separately
 * rounded additions per transition in the order (C_prev + R) + c, no fused
 * multiply-add, no reassociation; every min keeps the LOWEST index on ties
 * (an update happens only on strict "<"); a cell whose forward memory
 * exceeds the budget is infeasible and holds +infinity (Section 4.1.2).
 * Build with -ffp-contract=off and without -ffast-math.
 *
 * Two forms are given, as the method is exact:
 *   - gbmw_oracle_bruteforce: the plain definition, enumerating all S^L plans;
 *   - gbmw_oracle_solve:      the recurrence, step by step, producing tables.
 *
 * Logical table layout everywhere in this file: [l][e][s], s fastest.
 * A[l][e'][s] (l >= 1) is indexed by the budget e' left for layers < l, i.e.
 * BEFORE layer l's own memory is added; the A[0] slab is all zero.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* Plain definition of one plan's cost and memory (Eq. 3 unrolled).    */
/* ------------------------------------------------------------------ */
void gbmw_oracle_plan_cost(int L, int S, const float *c, const int32_t *M,
                           const float *R, const uint8_t *plan,
                           float *cost_out, int64_t *mem_out)
{
    float v = c[0 * S + plan[0]];
    int64_t mem = M[0 * S + plan[0]];
    for (int l = 1; l < L; ++l) {
        int sp = plan[l - 1], s = plan[l];
        float t = v + R[((size_t)l * S + sp) * S + s];
        v = t + c[(size_t)l * S + s];
        mem += M[(size_t)l * S + s];
    }
    *cost_out = v;
    *mem_out = mem;
}

/* ------------------------------------------------------------------ */
/* Brute force: OPT(e) = min{ cost(plan) : mem(plan) <= e }.           */
/* opt[e] (E+1 floats) and nopt[e] = number of plans with mem <= e     */
/* whose cost equals opt[e].  If e_q >= 0, plan_q receives the first    */
/* optimal plan for budget e_q in odometer order (layer 0 slowest),     */
/* or 0xFF bytes when none is feasible.  Returns the number of plans    */
/* enumerated, or -1 if S^L exceeds limit.                              */
/* ------------------------------------------------------------------ */
int64_t gbmw_oracle_bruteforce(int L, int S, int E, const float *c,
                               const int32_t *M, const float *R, float *opt,
                               int64_t *nopt, int e_q, uint8_t *plan_q,
                               int64_t limit)
{
    double total = 1.0;
    for (int l = 0; l < L; ++l) total *= S;
    if (total > (double)limit) return -1;

    /* bucket[m] = cheapest plan using exactly m units (m <= E) */
    float *bucket = (float *)malloc(sizeof(float) * (size_t)(E + 1));
    int64_t *bcount = (int64_t *)calloc((size_t)(E + 1), sizeof(int64_t));
    for (int e = 0; e <= E; ++e) bucket[e] = INFINITY;

    uint8_t *plan = (uint8_t *)calloc((size_t)L, 1);
    int64_t n = 0;
    for (;;) {
        float cost;
        int64_t mem;
        gbmw_oracle_plan_cost(L, S, c, M, R, plan, &cost, &mem);
        ++n;
        if (mem <= E) {
            if (cost < bucket[mem]) { bucket[mem] = cost; bcount[mem] = 1; }
            else if (cost == bucket[mem]) bcount[mem] += 1;
        }
        int l = L - 1;                       /* odometer, last layer fastest */
        while (l >= 0 && ++plan[l] == S) { plan[l] = 0; --l; }
        if (l < 0) break;
    }
    float run = INFINITY;
    int64_t cnt = 0;
    for (int e = 0; e <= E; ++e) {
        if (bucket[e] < run) { run = bucket[e]; cnt = bcount[e]; }
        else if (bucket[e] == run && run != INFINITY) cnt += bcount[e];
        opt[e] = run;
        if (nopt) nopt[e] = (run == INFINITY) ? 0 : cnt;
    }
    if (e_q >= 0 && plan_q) {
        memset(plan_q, 0xFF, (size_t)L);
        if (opt[e_q] != INFINITY) {
            memset(plan, 0, (size_t)L);
            for (;;) {
                float cost;
                int64_t mem;
                gbmw_oracle_plan_cost(L, S, c, M, R, plan, &cost, &mem);
                if (mem <= e_q && cost == opt[e_q]) { memcpy(plan_q, plan, (size_t)L); break; }
                int l = L - 1;
                while (l >= 0 && ++plan[l] == S) { plan[l] = 0; --l; }
                if (l < 0) break;
            }
        }
    }
    free(bucket); free(bcount); free(plan);
    return n;
}

/* ------------------------------------------------------------------ */
/* The recurrence, one layer at a time.                                 */
/*   C  : [L][E+1][S] floats, or NULL (two rolling layers are used)     */
/*   A  : [L][E+1][S] bytes,  or NULL                                   */
/*   T  : [L][E+1][S] floats, or NULL  (the min-plus product before the */
/*        shift; T[0] is left untouched)                                */
/*   best, best_s : [E+1]                                               */
/* nthreads > 1 splits the rows e of one layer over OpenMP threads;     */
/* rows are independent within a layer, so the result is identical.     */
/* Returns 0, or 1 on allocation failure / bad sizes.                   */
/* ------------------------------------------------------------------ */
int gbmw_oracle_solve(int L, int S, int E, const float *c, const int32_t *M,
                      const float *R, float *C, uint8_t *A, float *T_out,
                      float *best, uint8_t *best_s, int nthreads)
{
    if (L < 1 || S < 1 || S > 256 || E < 0) return 1;
    const size_t rows = (size_t)E + 1, slab = rows * (size_t)S;
    float *roll = NULL, *T = NULL;
    if (!C) {
        roll = (float *)malloc(sizeof(float) * slab * 2);
        if (!roll) return 1;
    }
    if (!T_out) {
        T = (float *)malloc(sizeof(float) * slab);
        if (!T) { free(roll); return 1; }
    }
#ifdef _OPENMP
    if (nthreads < 1) nthreads = 1;
#else
    (void)nthreads;
#endif

    /* layer 0: nothing precedes it, so no R term (C(0, .) = 0 in the paper) */
    float *Cl = C ? C : roll;
    for (size_t e = 0; e < rows; ++e)
        for (int s = 0; s < S; ++s)
            Cl[e * S + s] = ((int64_t)e >= (int64_t)M[s]) ? c[s] : INFINITY;
    if (A) memset(A, 0, slab);

    for (int l = 1; l < L; ++l) {
        const float *Cp = C ? C + (size_t)(l - 1) * slab : roll + (size_t)((l - 1) & 1) * slab;
        float *Cn = C ? C + (size_t)l * slab : roll + (size_t)(l & 1) * slab;
        float *Tl = T_out ? T_out + (size_t)l * slab : T;
        uint8_t *Al = A ? A + (size_t)l * slab : NULL;
        const float *Rl = R + (size_t)l * S * S;
        const float *cl = c + (size_t)l * S;
        const int32_t *Ml = M + (size_t)l * S;

        /* min-plus step: T[e'][s] = min_{s'} (C_{l-1}[e'][s'] + R_l[s'][s]) */
#ifdef _OPENMP
#pragma omp parallel for num_threads(nthreads) schedule(static)
#endif
        for (int64_t e = 0; e < (int64_t)rows; ++e) {
            for (int s = 0; s < S; ++s) {
                float t = INFINITY;
                int a = 0;
                for (int sp = 0; sp < S; ++sp) {
                    float x = Cp[(size_t)e * S + sp] + Rl[(size_t)sp * S + s];
                    if (x < t) { t = x; a = sp; }
                }
                Tl[(size_t)e * S + s] = t;
                if (Al) Al[(size_t)e * S + s] = (uint8_t)a;
            }
        }
        /* shift by the layer's own memory and add its own cost */
#ifdef _OPENMP
#pragma omp parallel for num_threads(nthreads) schedule(static)
#endif
        for (int64_t e = 0; e < (int64_t)rows; ++e) {
            for (int s = 0; s < S; ++s) {
                int64_t ep = e - (int64_t)Ml[s];
                Cn[(size_t)e * S + s] =
                    (ep >= 0) ? Tl[(size_t)ep * S + s] + cl[s] : INFINITY;
            }
        }
    }

    const float *Clast = C ? C + (size_t)(L - 1) * slab : roll + (size_t)((L - 1) & 1) * slab;
    for (size_t e = 0; e < rows; ++e) {
        float t = INFINITY;
        int a = 0;
        for (int s = 0; s < S; ++s) {
            float x = Clast[e * S + s];
            if (x < t) { t = x; a = s; }
        }
        best[e] = t;
        best_s[e] = (uint8_t)a;
    }
    free(roll); free(T);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Read the plan for budget e_q back out of the argmin records.         */
/* plan[L] gets the strategies (0xFF everywhere if infeasible);          */
/* cost = best[e_q]; mem = sum of M along the plan (-1 if infeasible).   */
/* ------------------------------------------------------------------ */
void gbmw_oracle_backtrack(int L, int S, int E, const int32_t *M,
                           const uint8_t *A, const float *best,
                           const uint8_t *best_s, int e_q, uint8_t *plan,
                           float *cost_out, int64_t *mem_out)
{
    const size_t slab = ((size_t)E + 1) * (size_t)S;
    *cost_out = best[e_q];
    if (best[e_q] == INFINITY) {
        memset(plan, 0xFF, (size_t)L);
        *mem_out = -1;
        return;
    }
    int s = best_s[e_q];
    int64_t e = e_q, mem = 0;
    for (int l = L - 1; l >= 1; --l) {
        plan[l] = (uint8_t)s;
        mem += M[(size_t)l * S + s];
        e -= M[(size_t)l * S + s];            /* budget left for layers < l */
        s = A[(size_t)l * slab + (size_t)e * S + s];
    }
    plan[0] = (uint8_t)s;
    mem += M[s];
    *mem_out = mem;
}

/* ------------------------------------------------------------------ */
/* Overall memory of a plan (Section 4.1.2, Eq. 2): when layer i runs    */
/* its backward pass, the forward activations of layers 1..i, the         */
/* backward activations of layer i and the model states of ALL layers     */
/* are alive;  E_all is the largest such peak.                            */
/*   E_all = max_i { sum_{k<=i} O_f(k,s_k) + O_b(i,s_i) } + sum_k O_ms(k,s_k) */
/* (the equation prints O_b(i, S_{j_k}); the subscript is read as j_i).   */
/* ------------------------------------------------------------------ */
int64_t gbmw_oracle_e_all(int L, int S, const int32_t *Of, const int32_t *Ob,
                          const int32_t *Oms, const uint8_t *plan)
{
    int64_t fwd = 0, ms = 0, peak = 0;
    for (int i = 0; i < L; ++i) {
        int s = plan[i];
        fwd += Of[(size_t)i * S + s];
        ms += Oms[(size_t)i * S + s];
        int64_t here = fwd + Ob[(size_t)i * S + s];
        if (i == 0 || here > peak) peak = here;
    }
    return peak + ms;
}

/* ------------------------------------------------------------------ */
/* The outer loop of Appendix A, Algorithm 3, on top of a filled table    */
/* (M = O_f + O_ms was the memory the table was filled with, E the total  */
/* device budget).  b_up = max O_b bounds the backward peak, so every     */
/* E_fwd <= E - b_up is valid without a check; the budgets above that are */
/* visited in increasing order, each plan's E_all is checked against E,   */
/* and the walk stops at the first plan that does not fit.                */
/* Readings: E_fwd^opt starts at E - b_up with that budget's plan; if     */
/* E - b_up < 0 nothing is valid a priori (start: none, window from 0);   */
/* a budget with no feasible plan (best = +inf) has nothing to check and  */
/* is passed over.                                                        */
/* Outputs: *e_opt (-1: none), *cost = best[e_opt] (+inf if none or       */
/* infeasible), plan[L] (0xFF if none/infeasible), *e_all (-1 likewise).  */
/* ------------------------------------------------------------------ */
void gbmw_oracle_select_budget(int L, int S, int E, const int32_t *M,
                               const uint8_t *A, const float *best,
                               const uint8_t *best_s, const int32_t *Of,
                               const int32_t *Ob, const int32_t *Oms,
                               int32_t *e_opt, float *cost, uint8_t *plan,
                               int64_t *e_all)
{
    int64_t b_up = 0;
    for (size_t i = 0; i < (size_t)L * S; ++i)
        if (Ob[i] > b_up) b_up = Ob[i];
    int64_t opt = (int64_t)E - b_up;
    if (opt < 0) opt = -1;
    uint8_t *cur = (uint8_t *)malloc((size_t)L);
    for (int64_t e = opt + 1; e <= E; ++e) {
        if (best[e] == INFINITY) continue;
        float c_;
        int64_t m_;
        gbmw_oracle_backtrack(L, S, E, M, A, best, best_s, (int)e, cur, &c_, &m_);
        if (gbmw_oracle_e_all(L, S, Of, Ob, Oms, cur) <= E) opt = e;
        else break;
    }
    free(cur);
    *e_opt = (int32_t)opt;
    *cost = INFINITY;
    *e_all = -1;
    memset(plan, 0xFF, (size_t)L);
    if (opt >= 0 && best[opt] != INFINITY) {
        int64_t m_;
        gbmw_oracle_backtrack(L, S, E, M, A, best, best_s, (int)opt, plan, cost, &m_);
        *e_all = gbmw_oracle_e_all(L, S, Of, Ob, Oms, plan);
    }
}

/* ------------------------------------------------------------------ */
/* Pipeline time of P stages run with m micro-batches (Section 4.2.1,    */
/* Eq. 5; Appendix C, Eq. 8):                                             */
/*   C = (m - 1) * max_i Cns_i + sum_i C_i                                */
/* C_i is a stage's time for the last micro-batch (with gradient          */
/* synchronisation), Cns_i its time without it (Eq. 5 is the case         */
/* Cns = C).  fp32: the sum is a left fold over the stages, the product   */
/* and the final addition are rounded separately.  A stage with no        */
/* feasible plan (+inf) makes the pipeline +inf.                          */
/* ------------------------------------------------------------------ */
float gbmw_oracle_pipeline_cost(int P, int m, const float *C, const float *Cns)
{
    float total = C[0], mx = Cns[0];
    for (int i = 1; i < P; ++i) {
        total = total + C[i];
        if (Cns[i] > mx) mx = Cns[i];
    }
    if (total == INFINITY || mx == INFINITY) return INFINITY;
    float head = (float)(m - 1) * mx;
    return head + total;
}

int gbmw_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
