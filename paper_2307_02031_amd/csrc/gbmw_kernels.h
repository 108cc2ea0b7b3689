// Internal launch interface between the C-ABI layer (gbmw_api.hip) and the
// gfx950 kernels (gbmw_kernels.hip).  Not installed; not part of the ABI.
//
// Device data layout ("SoA by strategy", budget axis contiguous):
//   C table of one (instance, layer):  float  [S][EP]   C[s*EP + e]
//   A table of one (instance, layer):  uint8  [S][EP]   A[s*EP + e']   (with the run shortcut one byte
//       per group of 64 budgets stands for the group's 64 records where they are equal: Tables::Asum)
//   EP = (E + 1) rounded up to a multiple of 256 (row stride in elements)
//   Rt: transposed, padded transformation cost with the layer's own cost and
//       memory riding along:  float [sumL][S][RS],  Rt[row][s][s'] = R[row][s'][s]
//       for s' < S, zero for S <= s' < SP, Rt[row][s][SP] = c[row][s],
//       Rt[row][s][SP+1] = bits of M[row][s]; SP = S rounded up to a multiple of 4,
//       RS = SP + 2 rounded up to a multiple of 4 (rows are whole float4s).
// A wave's 64 lanes hold 64 consecutive budgets e of one strategy, so every
// table access is a coalesced 256-byte segment and every R / c / M operand is
// wave-uniform.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gbmw {

struct Tables {
  int B, S, SP, RS, E, EP;
  int keep_all;        // 1: Call[row][S][EP] for every layer row; 0: rolling pair
  int final_from;      // the final reduce fills best / best_s for e >= final_from only
  int prev_full;       // set per launch: the input tables have every cell written (see runs)
  int runs;            // != 0: a wave whose 64 budgets all have the same input column (the tables are
                       // step functions of the budget) computes that column once, one output
                       // strategy per lane, and leaves its cells of the fp32 table unwritten: the
                       // summaries say what they hold (see Tsum and table_cell); 0: every lane
                       // computes and writes its own cell, and there are no summaries
  const int* L;        // [B]   device
  const int* off;      // [B]   device, first row of each instance
  const int* perm;     // [B]   device, instances ordered by L descending
  const float* c;      // [sumL][S]  owned by the context (a copy of the caller's)
  const int* M;        // [sumL][S]  owned by the context
  const float* Rt;     // [sumL][S][RS]
  float* Cbuf;         // keep_all ? [sumL][S][EP] : [2][B][S][EP]
  uint8_t* A;          // [sumL][S][EP]; null: records are not kept (needs keep_all), the
                       // walkers recompute the one they need from the kept tables
  float* Tsum;         // per table (indexed like Cbuf) [S][EP/64]: for every strategy and every group
                       // of 64 budgets e' of the layer's min-plus product, the value T + c if it is the
                       // same for all 64 (those inside the table), NaN otherwise; written by every
                       // launch when runs != 0; null when runs == 0.  Where the word is a number the
                       // table's cells of that group (at e = e' + M) may be unwritten; where it is
                       // NaN they are written
  uint8_t* Asum;       // [sumL][S][EP/64], beside A when runs != 0, else null: the record of a whole
                       // group of 64 budgets e' where one record holds for all of them (the groups whose
                       // summary word in Tsum is a number: equal input columns give equal minimisers),
                       // kNoGroupRecord where the group's records are in A.  Every launch that writes
                       // records writes this byte for every group it covers, and the 64 bytes of A only
                       // for the groups it marks kNoGroupRecord
  float* best;         // [B][EP]
  uint8_t* best_s;     // [B][EP]
  int* status;         // device word; bit 0: bad c, bit 1: bad M, bit 2: bad R
  unsigned long long* counts;  // null, or four counters of the launch, for measurements: [0] workgroups
                       // whose four waves shared one column (S * S' updates computed per workgroup)
                       // and [3] the waves inside the table that those workgroups covered;
                       // [1] waves recognised as a run from the summaries and [2] from the loaded
                       // table values (S * S' updates per wave).  Every other wave inside the table
                       // computed its 64 * S cells one by one
};

#if defined(__HIPCC__)
constexpr int kNaNBits = 0x7fc00000;
__device__ __forceinline__ bool is_nan_bits(int b) { return (b & 0x7fffffff) > 0x7f800000; }

// C(l, e, s) of the layer whose table starts at Ctab ([S][EP]), whose summaries start at Tsum_tab
// ([S][EP/64], unused when runs == 0) and whose M row is Mrow: +inf below M(l, s) (a negative M, or
// one beyond the budget axis, leaves no feasible budget), else the summary of the group that
// e - M falls in if it is a number, else the table's cell.
__device__ __forceinline__ float table_cell(const Tables& t, const float* __restrict__ Ctab,
                                            const float* __restrict__ Tsum_tab, const int* __restrict__ Mrow,
                                            int s, int e) {
  if (t.runs == 0) return Ctab[(size_t)s * t.EP + e];
  const int m = Mrow[s];
  if (m < 0 || e < m) return INFINITY;
  const float w = Tsum_tab[(size_t)s * (t.EP >> 6) + ((e - m) >> 6)];
  return is_nan_bits(__float_as_int(w)) ? Ctab[(size_t)s * t.EP + e] : w;
}

// Marks a group of 64 budgets whose records are in A (strategy indices with the run shortcut
// stay below 64).
constexpr int kNoGroupRecord = 0xff;

// The argmin record of table row `row`, strategy s, budget e' = e (t.A != null).  Both bytes are
// asked for at once (the one in A may never have been written; it is then not used).
__device__ __forceinline__ int record(const Tables& t, int row, int s, int e) {
  const int own = t.A[((size_t)row * t.S + s) * t.EP + e];
  if (t.Asum == nullptr) return own;
  const int group = t.Asum[((size_t)row * t.S + s) * (t.EP >> 6) + (e >> 6)];
  return group == kNoGroupRecord ? own : group;
}

// Predecessor strategy of table row `row` (layer l >= 1 of some instance) under strategy s
// when e units are left for the layers below: the recorded one, or, where records are not
// kept, recomputed from the kept table of layer l - 1 with the recurrence's own arithmetic
// ((C + R), lowest index among equals, 0 if every candidate is +inf).
__device__ __forceinline__ int pred_strategy(const Tables& t, int row, int s, int e) {
  if (t.A) return record(t, row, s, e);
  const float* __restrict__ Cp = t.Cbuf + (size_t)(row - 1) * t.S * t.EP;
  const float* __restrict__ Tp = t.Tsum ? t.Tsum + (size_t)(row - 1) * t.S * (t.EP >> 6) : nullptr;
  const int* __restrict__ Mp = t.M + (size_t)(row - 1) * t.S;
  const float* __restrict__ Rr = t.Rt + ((size_t)row * t.S + s) * t.RS;
  float best = INFINITY;
  int a = 0;
  for (int sp = 0; sp < t.S; ++sp) {
    const float x = table_cell(t, Cp, Tp, Mp, sp, e) + Rr[sp];
    if (x < best) { best = x; a = sp; }
  }
  return a;
}

// The same for a whole wave walking ONE plan (all 64 lanes hold the same row, s, e and get
// the same answer): without records the lanes take the candidates s' = lane, lane + 64, ...
// and the minimum with its lowest index is found by a butterfly over the wave.
__device__ __forceinline__ int pred_strategy_wave(const Tables& t, int row, int s, int e, int lane) {
  if (t.A) return record(t, row, s, e);
  const float* __restrict__ Cp = t.Cbuf + (size_t)(row - 1) * t.S * t.EP;
  const float* __restrict__ Tp = t.Tsum ? t.Tsum + (size_t)(row - 1) * t.S * (t.EP >> 6) : nullptr;
  const int* __restrict__ Mp = t.M + (size_t)(row - 1) * t.S;
  const float* __restrict__ Rr = t.Rt + ((size_t)row * t.S + s) * t.RS;
  float best = INFINITY;
  int a = 0x7fffffff;
  for (int sp = lane; sp < t.S; sp += 64) {
    const float x = table_cell(t, Cp, Tp, Mp, sp, e) + Rr[sp];
    if (x < best) { best = x; a = sp; }
  }
  for (int d = 32; d >= 1; d >>= 1) {
    const float ob = __shfl_xor(best, d, 64);
    const int oa = __shfl_xor(a, d, 64);
    if (ob < best || (ob == best && oa < a)) { best = ob; a = oa; }
  }
  return best == INFINITY ? 0 : a;
}
#endif

// R -> Rt (transpose + pad), validation of device-resident inputs, and the copy of the
// caller's c / M (src_c, src_M) into the context's own arrays t.c / t.M where they differ.
void launch_prepare(const Tables& t, const float* R, const float* src_c, const int* src_M, int sumL,
                    bool validate, hipStream_t st);
// Zeroes n measurement counters (a fill kernel, not a memset node).
void launch_clear_counts(unsigned long long* counts, int n, hipStream_t st);
// C(0, e, s) written to the table for instances perm[first .. first + count).  Needed
// where something reads layer 0 from memory: instances with L_b <= 2 (final reduce,
// export), every instance when all layers are kept or S > 64.
void launch_init_layer0(const Tables& t, int first, int count, hipStream_t st);
// True when the layer-1 launch builds layer 0 in registers and does not read it.
bool layer0_in_registers(int S);
// One layer l >= 1 for instances perm[first .. first + n_active):
// min-plus product with argmin, fused with the shift by M(l,s), the + c(l,s)
// and the +inf prefix.
// n_prev: instances in the launch that produced this one's input tables (layer l - 1 of the same
// instances and more); 0 if not known (tables kept from other launches); < 0: whatever produced
// them wrote every cell (split launches: launch_is_split).
void launch_minplus(const Tables& t, int l, int first, int n_active, hipStream_t st, int n_prev = 0);
// Does a launch over n_active instances take the split shape (which writes every table cell)?
bool launch_is_split(const Tables& t, int n_active);
// best(e), best_s(e) for e = final_from .. E over the last layer of instances
// perm[first .. first + count).
void launch_final(const Tables& t, int first, int count, hipStream_t st);
// Plans for nq queries (all pointers device).
void launch_backtrack(const Tables& t, int nq, const int* q_inst, const int* q_e, int Lmax,
                      uint8_t* plan, float* cost, int* mem_used, hipStream_t st);
// Algorithm 3's outer loop (all pointers device): Of/Ob/Oms [sumL][S], bup [B]
// (max O_b per instance), first_bad [B] scratch, outputs per instance.
void launch_select(const Tables& t, const int* Of, const int* Ob, const int* Oms, const int* bup,
                   int max_window, int Lmax, int* first_bad, int* e_opt, float* cost,
                   uint8_t* plan, int* e_all, hipStream_t st);
// Pipeline time (all pointers device): per stage C = best and Cns = the plan under
// c_ns (nullptr: C); per pipeline (m - 1) * max Cns + sum C.
void launch_pipeline_cost(const Tables& t, int n_stage, const int* st_inst, const int* st_e,
                          const float* c_ns, uint8_t* plan_scratch, int Lmax, float* st_C,
                          float* st_Cns, int n_pipe, const int* st_begin, const int* mb,
                          float* cost, hipStream_t st);
// [S][EP] -> [E+1][S] for rows [row0, row0+n) of C (fp32; base pointer given) or A (bytes).
// C(l, ., .) of one layer as [E+1][S]; Ctab / Tsum_tab / Mrow as for table_cell.
void launch_export_c(const Tables& t, const float* Ctab, const float* Tsum_tab, const int* Mrow, float* dst,
                     hipStream_t st);
void launch_export_u8(const uint8_t* src, uint8_t* dst, int n, int S, int E, int EP, hipStream_t st);
// The argmin records of one table row, [S][EP] bytes, recomputed from the kept tables.
void launch_argmin_row(const Tables& t, int row, uint8_t* dst, hipStream_t st);

// ---- the single-launch fill of small problems (gbmw_persistent.hip)
// Words of the context's synchronisation block (unsigned long long each).  The header words
// hold the epoch of the solve that set them; then one word per table row (its R tile is
// transposed: holds the epoch), then one per (instance slot, tile): epoch << 20 | layers done.
// Epochs only grow, so a word left by an earlier solve never satisfies a later one.
constexpr int kSyncBadC = 0, kSyncBadM = 1, kSyncBadR = 2, kSyncGaveUp = 3, kSyncLeave = 4, kSyncHeader = 8;
struct PersistArgs {
  unsigned long long* sync;     // device, kSyncHeader + sumL + n_slots * tiles words
  unsigned long long epoch;     // of this solve, >= 1, < 2^43
  const float* src_c;           // the caller's c / M / R on the device (or the context's uploads)
  const int* src_M;
  const float* R;
  long long wait_ticks;         // bound of every wait, in ticks of the constant 100 MHz clock
  int wait_polls;               // and in polls
  int sumL, validate, tiles, n_slots, first;
  int extra_wait;               // testing: every wait asks for a layer that is never published
};
// Workgroups of the single-launch kernel with `waves` (4 or 8) waves per tile that the device
// holds at once (0: no such kernel).
int layers_resident_workgroups(int S, int waves, bool records);
hipError_t launch_layers(const Tables& t, const PersistArgs& a, int waves, bool cooperative, hipStream_t st);

const char* minplus_variant(int S);

}  // namespace gbmw
