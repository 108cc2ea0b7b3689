// gfx950 kernels of the batched layer-wise strategy search (Section 4.1.2,
// Eq. 3; Appendix A, Algorithm 3 of the paper).  See gbmw_kernels.h for the
// device layout.  (min,+) is not a multiply-accumulate, so the matrix cores
// are not used: the work is fp32 VALU adds and mins with wave-uniform R
// operands, streamed along the budget axis.
#include "gbmw_kernels.h"

#include <math.h>

namespace gbmw {

#define GBMW_AS4 __attribute__((address_space(4)))
typedef const GBMW_AS4 float* cf32_t;   // uniform, read-only -> scalar loads
typedef const GBMW_AS4 int* ci32_t;

template <typename T>
__device__ __forceinline__ const GBMW_AS4 T* as_const(const T* p) {
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wold-style-cast"
  return (const GBMW_AS4 T*)(p);
#pragma clang diagnostic pop
}

// Summary of a table, laid out and indexed like the table itself: [S][EP / 64].
__device__ __forceinline__ float* sum_table(const Tables& t, int inst, int row, int l) {
  const size_t slab = (size_t)t.S * (t.EP >> 6);
  return t.keep_all ? t.Tsum + (size_t)row * slab
                    : t.Tsum + ((size_t)(l & 1) * t.B + inst) * slab;
}


// The group records of table row `row`: [S][EP / 64] bytes (null without them).
__device__ __forceinline__ uint8_t* group_records(const Tables& t, int row) {
  return t.Asum ? t.Asum + (size_t)row * t.S * (t.EP >> 6) : nullptr;
}

__device__ __forceinline__ float* c_table(const Tables& t, int inst, int row, int l) {
  const size_t slab = (size_t)t.S * t.EP;
  return t.keep_all ? t.Cbuf + (size_t)row * slab
                    : t.Cbuf + ((size_t)(l & 1) * t.B + inst) * slab;
}

// ---------------------------------------------------------------------------
// prepare: Rt[row][s][0..SP) = R[row][.][s] (zero padding), Rt[row][s][SP] = c,
// Rt[row][s][SP+1] = bits of M; + input validation.  c and M are read from the caller's
// arrays (src_c, src_M) and, where those are not the context's own (device-resident inputs),
// copied into the context's (t.c, t.M), which is what every later kernel and every later call
// reads: the caller's arrays are not touched again once this kernel has run.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_prepare(Tables t, const float* __restrict__ R, int sumL,
                                                 int validate, float* __restrict__ Rt,
                                                 const float* __restrict__ src_c,
                                                 const int* __restrict__ src_M) {
  const int SP = t.SP, S = t.S, RS = t.RS;
  const size_t n = (size_t)sumL * S * RS;
  const bool copy = src_c != t.c;
  int bad = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x) {
    const int sp = (int)(i % RS);
    const int s = (int)((i / RS) % S);
    const size_t row = i / ((size_t)RS * S);
    float v = 0.0f;
    if (sp < S) {
      v = R[(row * S + sp) * S + s];
    } else if (sp == SP) {
      v = src_c[row * S + s];
      if (validate && !(v >= 0.0f)) bad |= 1;
      if (copy) const_cast<float*>(t.c)[row * S + s] = v;
    } else if (sp == SP + 1) {
      const int m = src_M[row * S + s];
      if (validate && m < 0) bad |= 2;
      if (copy) const_cast<int*>(t.M)[row * S + s] = m;
      v = __int_as_float(m);
    }
    Rt[i] = v;
  }
  if (validate && bad) atomicOr(t.status, bad);
}

// R is validated per instance because the l == 0 slab is ignored by contract
// and may hold anything.
__global__ __launch_bounds__(256) void k_validate_R(Tables t, const float* __restrict__ R) {
  const int inst = blockIdx.y;
  const int S = t.S;
  const int Lb = t.L[inst];
  const size_t base = ((size_t)t.off[inst] + 1) * S * S;   // skip layer 0
  const size_t n = (size_t)(Lb - 1) * S * S;
  int bad = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x)
    if (!(R[base + i] >= 0.0f)) bad = 4;
  if (bad) atomicOr(t.status, bad);
}

__global__ void k_clear_status(int* status) { *status = 0; }

__global__ void k_clear_counts(unsigned long long* counts, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) counts[i] = 0;
}

void launch_clear_counts(unsigned long long* counts, int n, hipStream_t st) {
  if (n > 0) hipLaunchKernelGGL(k_clear_counts, dim3((n + 255) / 256), dim3(256), 0, st, counts, n);
}

void launch_prepare(const Tables& t, const float* R, const float* src_c, const int* src_M, int sumL,
                    bool validate, hipStream_t st) {
  // a fill kernel rather than a memset node, so that the sequence can be captured
  hipLaunchKernelGGL(k_clear_status, dim3(1), dim3(1), 0, st, t.status);
  const size_t n = (size_t)sumL * t.S * t.RS;
  int blocks = (int)((n + 255) / 256);
  if (blocks > 65536) blocks = 65536;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(k_prepare, dim3(blocks), dim3(256), 0, st, t, R, sumL, validate ? 1 : 0,
                     const_cast<float*>(t.Rt), src_c, src_M);
  if (validate) hipLaunchKernelGGL(k_validate_R, dim3(64, t.B), dim3(256), 0, st, t, R);
}

// ---------------------------------------------------------------------------
// layer 0:  C(0, e, s) = e >= M(0, s) ? c(0, s) : +inf
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_init_layer0(Tables t, int first) {
  const int inst = t.perm[first + blockIdx.z], s = blockIdx.y;
  const int e = (blockIdx.x * 256 + threadIdx.x) * 4;     // EP is a multiple of 256: whole float4s
  if (e >= t.EP) return;
  const int row = t.off[inst];
  const int m = t.M[(size_t)row * t.S + s];
  const float cs = t.c[(size_t)row * t.S + s];
  float* C0 = c_table(t, inst, row, 0);
  float4 v;                                                // padding rows: +inf
  v.x = (m >= 0 && e >= m && e <= t.E) ? cs : INFINITY;
  v.y = (m >= 0 && e + 1 >= m && e + 1 <= t.E) ? cs : INFINITY;
  v.z = (m >= 0 && e + 2 >= m && e + 2 <= t.E) ? cs : INFINITY;
  v.w = (m >= 0 && e + 3 >= m && e + 3 <= t.E) ? cs : INFINITY;
  *reinterpret_cast<float4*>(C0 + (size_t)s * t.EP + e) = v;
  // T + c of layer 0 is c(0, s) at every budget: one summary word per group of 64
  if (t.runs != 0 && (e & 63) == 0 && e <= t.E) sum_table(t, inst, row, 0)[(size_t)s * (t.EP >> 6) + (e >> 6)] = cs;
}

void launch_init_layer0(const Tables& t, int first, int count, hipStream_t st) {
  if (count <= 0) return;
  hipLaunchKernelGGL(k_init_layer0, dim3((t.EP + 1023) / 1024, t.S, count), dim3(256), 0, st, t, first);
}

// ---------------------------------------------------------------------------
// min-plus + argmin + shift-add, register-blocked.
//   wave: 64*K consecutive budgets e' of one instance; lane owns e' = e0 + 64*j.
//   The SP values C_{l-1}[e'][0..SP) of each owned e' stay in VGPRs for the
//   whole kernel.  The layer's R tile (with c and M riding in each row) is
//   staged once per workgroup in LDS; every output strategy s reads its row
//   with wave-uniform 128-bit LDS reads (broadcast, conflict-free, returned in
//   order so the reads pipeline ahead of the adds).
//
//   Value pass: the SP candidates x = C + R are folded into chunk minima of CH
//   candidates (3-input min), and the chunk minima into a running prefix
//   minimum P[k] = min(P[k-1], chunk 2k-1, chunk 2k); T is the last prefix.
//   One add and half a min per candidate, no compare in the chain.  The R row is
//   consumed quad by quad as it arrives and only the prefix minima stay live.
//   Argmin: P[k] == T is monotone in k, so the lowest-index minimiser lies in
//   the first block k whose prefix equals T.  The block tests are independent
//   compares into wave masks; a block is re-scanned only when some lane of
//   the wave first hits it, which for neighbouring budgets is usually one; the
//   re-scan redoes the block's sums from the LDS row (same operands, same bits,
//   so equality with T is exact).
//   ARG = false leaves the argmin out altogether (values-only fill).
// ---------------------------------------------------------------------------
// Word 3 of a gfx9-family raw buffer descriptor: 32-bit data format, no swizzle.
constexpr int kBufWord3 = 0x00020000;
// Cache policy of a buffer store: non-temporal.  The argmin records of an unsplit launch are
// written once and not read again before the solve ends, and the previous table is read once
// (streaming loads): keeping both out of the way leaves the L2 to the fp32 stores, whose
// shifted rows meet their neighbours' in shared cache lines and are merged there (the same
// hint on those stores costs 20 %: the halves of a line are then written back separately).
constexpr int kStreaming = 2;

__device__ __forceinline__ float fmin3(float a, float b, float c) {
  return __builtin_fminf(__builtin_fminf(a, b), c);
}

// A wave whose 64 budgets all carry the same column C_{l-1}[e'][.] (a run of the step function
// that the table is along the budget axis) has 64 identical cells per output strategy.  It is
// computed once, with the lanes over the output strategies instead (colv: lane s' holds
// column[s'], +inf beyond the last strategy): lane j forms
// min_s' (column[s'] + R[s'][s_begin + j]) with the lowest minimising s' (strict compare in index
// order) and adds c.  Same operands and operations per cell as the dense path, hence the same
// bits.  The value goes into the layer's summary word of that group and strategy and nowhere
// else: the 64 cells of the fp32 table stay unwritten, every reader takes the word where it is
// a number (table_cell).  The argmin record, one for the 64 budgets as well, goes into the
// group's byte of the row's group records (Tables::Asum) and the 64 bytes of A stay unwritten.
template <int SP>
__device__ __forceinline__ void uniform_min(const float colv, const float4* rt_lds, int srow, int& outv,
                                            int& a) {
  constexpr int RS = (SP + 2 + 3) / 4 * 4;
  constexpr int RQ = RS / 4;
  float best = INFINITY, cs = 0.0f;
  a = 0;
  int roff = srow * RQ;
#pragma unroll
  for (int q = 0; q < RQ; ++q) {
    // one quad of the row in flight at a time: the read of quad q waits for the fold of quad
    // q - 1, so that the row never occupies more than four registers (this path is bound by
    // its stores, not by this latency)
    asm volatile("" : "+v"(roff), "+v"(best));
    const float4 v = rt_lds[roff + q];
    const float rq[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const int i = 4 * q + i4;
      if (i < SP) {
        const float f = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(colv), i));
        const float x = f + rq[i4];
        if (x < best) { best = x; a = i; }
      }
    }
    if (4 * q == SP) cs = rq[0];
  }
  outv = __float_as_int(best + cs);
}

template <int SP, bool ARG>
__device__ __forceinline__ void uniform_tile(const float colv, const float4* rt_lds, int s_begin,
                                             int s_end, int lane, int e0, int wbase, float* __restrict__ Cn,
                                             uint8_t* __restrict__ Ag, float* __restrict__ sum_cur, int E,
                                             int EP, unsigned long long* cnt) {
  const int srow = (s_begin + lane < s_end) ? s_begin + lane : s_begin;   // idle lanes redo a valid row
  int outv, a;
  uniform_min<SP>(colv, rt_lds, srow, outv, a);
  // the layer's own summary: every strategy's 64 cells are equal
  if (s_begin + lane < s_end) sum_cur[(size_t)(s_begin + lane) * (EP >> 6) + (wbase >> 6)] = __int_as_float(outv);
  // the summary word stands for the 64 cells, and one byte for their 64 records
  if (ARG && s_begin + lane < s_end) Ag[(size_t)(s_begin + lane) * (EP >> 6) + (wbase >> 6)] = (uint8_t)a;
  if (cnt && lane == 0) atomicAdd(cnt, 1ull);             // measurement only, when nothing else is live
}

// The same for a whole workgroup whose four waves (256 budgets from `base`) all carry that one
// column: lane j writes the four summary words of strategy s_begin + j and, with records, the
// four group records (one dword: EP is a multiple of 256, so a row of group records is whole
// dwords and `base >> 6` a multiple of 4).
template <int SP, bool ARG>
__device__ __forceinline__ void wide_tile(const float colv, const float4* rt_lds, int s_begin, int s_end,
                                          int lane, int base, float* __restrict__ Cn,
                                          uint8_t* __restrict__ Ag, float* __restrict__ sum_cur, int E,
                                          int EP, unsigned long long* cnt, int inside) {
  const int srow = (s_begin + lane < s_end) ? s_begin + lane : s_begin;
  int outv, a;
  uniform_min<SP>(colv, rt_lds, srow, outv, a);
  if (s_begin + lane < s_end) {
    float* sp_ = sum_cur + (size_t)(s_begin + lane) * (EP >> 6) + (base >> 6);
    const int last_group = E >> 6;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if ((base >> 6) + k <= last_group) sp_[k] = __int_as_float(outv);
  }
  if (ARG && s_begin + lane < s_end)
    *reinterpret_cast<uint32_t*>(Ag + (size_t)(s_begin + lane) * (EP >> 6) + (base >> 6)) = (unsigned)a * 0x01010101u;
  if (cnt && threadIdx.x == 0) {                          // measurement only: workgroups, and their waves
    atomicAdd(cnt, 1ull);
    atomicAdd(cnt + 3, (unsigned long long)inside);
  }
}

// How a launch's workgroups map to (instance, tile): the divisors of that mapping come with
// floor(2^32 / d) from the host, so that a workgroup finds its place with a multiply, a
// subtract and one correction per division (the quotient estimate is never more than one
// short) instead of the thirty-instruction sequence of a division by a run-time value: every
// wave pays for them before it can ask for its first byte.
constexpr int kDealChunk = 4;                            // consecutive tiles of one instance per XCD
struct Deal {
  int n;                                                 // instances in the launch
  unsigned inv_tiles, inv_rowlen, inv_cl, inv_n;         // of tiles, n * kDealChunk, tiles % kDealChunk, n
};

__device__ __forceinline__ void divmod(unsigned p, unsigned d, unsigned inv, int& q, int& r) {
  unsigned qq = __umulhi(p, inv), rr = p - qq * d;
  if (rr >= d) { ++qq; rr -= d; }
  q = (int)qq; r = (int)rr;
}

static unsigned inv_of(unsigned d) { return d <= 1 ? 0xffffffffu : (unsigned)((1ull << 32) / d); }

static Deal make_deal(int tiles, int n) {
  Deal d;
  d.n = n;
  d.inv_tiles = inv_of((unsigned)tiles);
  d.inv_rowlen = inv_of((unsigned)(n * kDealChunk));
  d.inv_cl = inv_of((unsigned)(tiles % kDealChunk));
  d.inv_n = inv_of((unsigned)n);
  return d;
}

// RUNS: waves whose budgets share one input column take uniform_tile (never in split mode:
// those launches are bound by a wave's own latency, which the test would lengthen).
// COUNT: the same kernel with one atomic per run-path wave or workgroup into t.counts, for
// measurements.  The paths a wave takes depend on the inputs alone, so the counts of this
// instantiation are those of the plain one, which is the one that is timed (the atomics cost a
// few registers, and with them occupancy at some sizes).
template <int SP, int K, int NW, int CH, int MINW, bool FIRST, bool ARG, bool SPLIT, bool RUNS, bool COUNT = false>
__global__ __launch_bounds__(64 * NW, MINW) void k_minplus(Tables t, int l, int tiles, int first, Deal deal) {
  constexpr bool split = SPLIT;
  static_assert(!(SPLIT && RUNS), "no run shortcut in split mode");
  static_assert(RUNS || !COUNT, "only the run paths are counted");
  unsigned long long* const counts = COUNT ? t.counts : nullptr;
  // With the run shortcut the waves that compute every cell are few and sit among waves that
  // hardly use the VALU: nothing hides the latency of their reads of the R tile, so they keep
  // PD quads of R in flight ahead of the fold, across the end of the row into the next one
  // (a rotating software pipeline: the fold of a quad takes about 30 cycles, an LDS read
  // about 130; the whole next row, tried first, costs 48 registers instead of 16 and with them
  // a wave per SIMD).
  constexpr bool PRE = RUNS && SP <= 56;                 // beyond, the table values leave no room for it
  constexpr int NC = (SP + CH - 1) / CH;                 // chunks (last may be short)
  constexpr int NP = NC / 2 + 1;                         // prefix minima / blocks
  constexpr int RS = (SP + 2 + 3) / 4 * 4;               // row: SP x R, c, M, padding
  constexpr int RQ = RS / 4;
  constexpr int PD = 4;                                  // quads of R in flight ahead of the fold (PRE)
  constexpr int RQP = (RQ + PD - 1) / PD * PD;           // the row's quads, padded to whole rounds of PD
  extern __shared__ float4 rt_lds[];                     // [S][RQ]

  // Workgroups go to the 8 XCDs (each with its own L2) round-robin by their index, and an XCD
  // works through its share in index order.  With the run shortcut the (instance, tile) pairs
  // are dealt out accordingly:
  //  - in chunks of kChunk consecutive tiles of one instance per XCD, so that neighbouring
  //    tiles, whose shifted stores share a cache line at their common border, mostly meet in
  //    one L2;
  //  - chunk row by chunk row across the instances (all chunks 0, then all chunks 1, ...): the
  //    tiles that must be computed cell by cell lie at the low budgets of every instance and
  //    take many times longer than the others, so they have to start early, all of them, and
  //    leave the end of the launch to the quick ones;
  //  - each chunk row starting one instance further on, so that the chunks of an instance go
  //    round the XCDs instead of all landing on one: the instances differ in how many such
  //    tiles they have, and an XCD cannot take work from another.
  // With dense arithmetic every tile costs the same and the plain order is kept.
  int slot, tile;
  if (RUNS) {
    constexpr int kChunk = kDealChunk, kRound = 8 * kChunk;   // one round: a chunk for each XCD
    const int b = blockIdx.x, nb = gridDim.x, n = deal.n;
    int p = b;                                            // place in the dealt order (the ragged end keeps its own)
    if (b < nb / kRound * kRound) {
      const int w = b % kRound;                           // b = 8 * (round * kChunk + r) + xcd
      p = ((b / kRound) * 8 + (w & 7)) * kChunk + (w >> 3);
    }
    const int full = tiles / kChunk, rowlen = n * kChunk;
    int c, k, r;
    if (p < full * rowlen) {
      int rem;
      divmod((unsigned)p, (unsigned)rowlen, deal.inv_rowlen, c, rem);
      k = rem / kChunk; r = rem % kChunk;
    } else {                                              // the short last chunk of every instance
      const int cl = tiles - full * kChunk, pp = p - full * rowlen;
      c = full;
      divmod((unsigned)pp, (unsigned)cl, deal.inv_cl, k, r);
    }
    int turns;
    divmod((unsigned)(k + c), (unsigned)n, deal.inv_n, turns, slot);
    tile = c * kChunk + r;
  } else {
    divmod(blockIdx.x, (unsigned)tiles, deal.inv_tiles, slot, tile);
  }
  const int inst = t.perm[first + slot];
  const int S = t.S, E = t.E, EP = t.EP;
  const int row = t.off[inst] + l;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, scalar
  const int lane = threadIdx.x & 63;
  // Normal mode: the workgroup's waves take consecutive row tiles and every
  // output strategy.  Split mode (small problems, too few workgroups to fill the
  // chip): the waves share one row tile and divide the output strategies, which
  // shortens the serial chain per wave NW-fold at the price of loading the tile
  // NW times (from L2).
  const int wbase = (split ? tile : tile * NW + wave) * (64 * K);
  const bool present = wbase <= E;                       // else: whole wave beyond the table
  const int n_in = (E - wbase + 1 < 64) ? E - wbase + 1 : 64;   // budgets of this wave inside the table

  // The run test's words (the previous layer's M, then two summaries whose place depends on
  // it: two memory round trips in a row) are asked for around the loads that stage the tile
  // of R, so that the three overlap instead of following one another.
  int rt_m = 0, rt_b1 = 0, rt_b2 = 0;
  float rt_c = INFINITY;
  const bool rt_lane = RUNS && present && lane < S;
  if (rt_lane) {
    rt_m = t.M[(size_t)(row - 1) * S + lane];
    if (FIRST) rt_c = t.c[(size_t)(row - 1) * S + lane];
  }
  {
    const float4* __restrict__ src = reinterpret_cast<const float4*>(t.Rt + (size_t)row * S * RS);
    constexpr int NSTG = (SP * RQ + 64 * NW - 1) / (64 * NW);
    float4 stg[NSTG];
#pragma unroll
    for (int k = 0; k < NSTG; ++k) {
      const int i = threadIdx.x + k * 64 * NW;
      stg[k] = (i < S * RQ) ? src[i] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    }
    if (rt_lane && !FIRST) {
      const int m = (rt_m < 0 || rt_m > E + 1) ? E + 1 : rt_m;
      const int e_last = wbase + n_in - 1;
      if (e_last >= m) {                                 // else: +inf throughout
        // the words of the (at most two) groups that this wave's budgets fall in; the run test
        // is decided without them where the column starts inside the wave (wbase < m), but the
        // dense path wants them there too
        const float* __restrict__ sp_ = sum_table(t, inst, row - 1, l - 1) + (size_t)lane * (EP >> 6);
        rt_b1 = __float_as_int(sp_[(wbase > m ? wbase - m : 0) >> 6]);
        rt_b2 = __float_as_int(sp_[(e_last - m) >> 6]);
      }
    }
#pragma unroll
    for (int k = 0; k < NSTG; ++k) {
      const int i = threadIdx.x + k * 64 * NW;
      if (i < S * RQ) rt_lds[i] = stg[k];
    }
  }
  __syncthreads();
  if (!RUNS && !present) return;
  const int s_begin = split ? (wave * S) / NW : 0;
  const int s_end = split ? ((wave + 1) * S) / NW : S;
  const float* __restrict__ Cp = c_table(t, inst, row - 1, l - 1);
  float* __restrict__ Cn = c_table(t, inst, row, l);
  uint8_t* __restrict__ An = ARG ? t.A + (size_t)row * S * EP : nullptr;
  // group records: kept beside A whenever the context uses the run shortcut, by split launches
  // too (the pointer is formed where it is used: it would stay live across the row loop)
  constexpr bool GROUPS = ARG && (RUNS || SPLIT);
  const int e0 = wbase + lane;

  // Summaries: besides its table every layer leaves, per strategy and per group of 64 budgets
  // e' of its min-plus product, the value T + c if all 64 are equal and NaN if not (sum_cur).
  // With the run shortcut the next layer reads those few words first: column s' of its input
  // over the wave's budgets [wbase, e_last] is C_{l-1}[s'][e] = +inf below M(l-1, s') and the
  // previous layer's T + c at e - M above, which spans at most two of its groups; the column
  // is constant if both summaries are the same number.  If every column is, the wave takes
  // uniform_tile and never loads the table; otherwise it loads it and computes every cell.
  // The layer-1 launch tests layer 0's closed form at the two ends (the columns are monotone).
  const bool want_sum = RUNS ? true : (SPLIT ? t.runs != 0 : false);
  // A split launch writes every cell, so NaN in all its words is as good as the true words
  // for every reader; the true ones only help a later unsplit launch to recognise runs, which
  // happens in the partition search (runs == 2) and never inside one solve (launches shrink).
  const bool true_sum = RUNS ? true : (SPLIT ? t.runs == 2 : false);
  float* __restrict__ sum_cur = want_sum ? sum_table(t, inst, row, l) : nullptr;
  if (RUNS) {
    static_assert(!RUNS || (K == 1 && SP <= 64), "one budget per lane, one lane per strategy");
    const int e_last = wbase + n_in - 1;
    bool ok = true;
    float v = INFINITY;
    if (rt_lane) {
      const int m = (rt_m < 0 || rt_m > E + 1) ? E + 1 : rt_m;
      if (FIRST) {
        const float cv = rt_c;
        v = wbase >= m ? cv : INFINITY;
        const float hi = e_last >= m ? cv : INFINITY;
        ok = __float_as_int(v) == __float_as_int(hi);
      } else if (e_last < m) {
        // the whole range lies in the +inf prefix
      } else if (wbase < m) {
        ok = false;
      } else {
        ok = rt_b1 == rt_b2 && !is_nan_bits(rt_b1);
        v = __int_as_float(rt_b1);
      }
    }
    const bool mine = __builtin_amdgcn_ballot_w64(!ok) == 0;
    // Do all waves of the workgroup (those inside the table) carry the same one column?  Each
    // publishes its verdict and its column, and every wave forms the same answer from them.
    static_assert(!RUNS || NW == 4, "four waves share their columns");
    __shared__ float x_col[NW][64];
    __shared__ int x_ok[NW];
    x_col[wave][lane] = v;
    if (lane == 0) x_ok[wave] = present ? (mine ? 1 : 0) : 2;       // 2: not inside the table
    __syncthreads();
    const float v0 = x_col[0][lane];
    bool same = true;
    int inside = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const int st = x_ok[w];
      same = same && (st == 2 || (st == 1 && __float_as_int(x_col[w][lane]) == __float_as_int(v0)));
      inside += (st != 2) ? 1 : 0;
    }
    if (__builtin_amdgcn_ballot_w64(!same) == 0) {
      // one wave does it, a lane per output strategy: the loop over the candidates is as long
      // for eleven lanes as for all of them, and the other three leave their issue slots to
      // the waves that compute cell by cell
      if (wave == 0)
        wide_tile<SP, ARG>(v0, rt_lds, 0, S, lane, tile * NW * 64, Cn,
                           GROUPS ? group_records(t, row) : nullptr, sum_cur, E, EP, counts, inside);
      return;
    }
    if (!present) return;
    if (mine) {
      uniform_tile<SP, ARG>(v, rt_lds, s_begin, s_end, lane, e0, wbase, Cn,
                            GROUPS ? group_records(t, row) : nullptr, sum_cur, E, EP, counts ? counts + 1 : nullptr);
      return;
    }
  }
  int sumv = kNaNBits;                                    // lane j: summary of strategy s_begin + j

  // EP is a multiple of 64*K and wbase <= E < EP, so rows e0 + 64*j < EP are
  // inside the allocation; rows in (E, EP) are padding whose results are
  // never stored into the table proper.
  float cp[K][SP];
  // the table values are formed here, after the run test, not before it (they would stay live
  // across the run paths otherwise)
  int e0d = e0;
  asm volatile("" : "+v"(e0d));
  if (FIRST) {
    // l == 1: layer 0 is a closed form, C(0, e, s') = e >= M(0, s') ? c(0, s') : +inf,
    // built here instead of being written to and read back from HBM.
    cf32_t c0 = as_const(t.c) + (size_t)(row - 1) * S;
    ci32_t m0 = as_const(t.M) + (size_t)(row - 1) * S;
#pragma unroll
    for (int sp = 0; sp < SP; ++sp) {
      const bool col = (sp < SP - 3 || sp < S);
      const float cv = col ? c0[sp] : INFINITY;
      const int mv = col ? m0[sp] : 0;
#pragma unroll
      for (int j = 0; j < K; ++j) {
        const int e = e0d + 64 * j;
        cp[j][sp] = (mv >= 0 && e >= mv && e <= E) ? cv : INFINITY;
      }
    }
  } else if (RUNS) {
    // With summaries the previous layer's cells are written only where their group's word is
    // NaN (see table_cell); below M(l-1, s') the cell is +inf.  The words of this wave's groups
    // are already here, in the lane of their column (the run test asked for them): the cell is
    // loaded whatever it holds, and the word wins where it is a number.
    static_assert(K == 1, "one budget per lane");
#pragma unroll
    for (int sp = 0; sp < SP; ++sp) {
      float c = INFINITY;
      if (sp < SP - 3 || sp < S) c = __builtin_nontemporal_load(&Cp[(size_t)sp * EP + e0d]);
      cp[0][sp] = c;
    }
#pragma unroll
    for (int sp = 0; sp < SP; ++sp) {
      if (sp < SP - 3 || sp < S) {
        const int m_raw = __builtin_amdgcn_readlane(rt_m, sp);
        const int m = (m_raw < 0 || m_raw > E + 1) ? E + 1 : m_raw;
        const int b1 = __builtin_amdgcn_readlane(rt_b1, sp), b2 = __builtin_amdgcn_readlane(rt_b2, sp);
        // the first budget of the second group; which word is a number is known per wave
        const int thr = m + ((((wbase > m ? wbase - m : 0) >> 6) + 1) << 6);
        const float v1 = is_nan_bits(b1) ? cp[0][sp] : __int_as_float(b1);
        const float v2 = is_nan_bits(b2) ? cp[0][sp] : __int_as_float(b2);
        cp[0][sp] = e0d < m ? INFINITY : e0d < thr ? v1 : v2;
      }
    }
  } else if (SPLIT && t.runs != 0 && !t.prev_full) {
    // A split launch whose input came from an unsplit one with the run shortcut, or from an
    // unknown launch (the partition search's kept tables): the same rule, but no words at
    // hand.  (A split launch that follows a split launch finds every cell written and takes
    // the plain loads below.)
    static_assert(K == 1, "one budget per lane");
    const float* __restrict__ Tp = sum_table(t, inst, row - 1, l - 1);
    // lane s' holds M(l-1, s')
    const int mprev = (lane < S) ? t.M[(size_t)(row - 1) * S + lane] : 0;
    // First the summaries of all columns, into the registers of the table values.  Then one
    // more load per column from an address chosen by what came: the cell where the word is
    // NaN, the word once more where it is a number (a cache hit).  No branch, so the loads of
    // the second round go out back to back, and never two values per column in registers
    // (asking for word and cell of every column at once takes 2 SP registers; a branch around
    // each cell's load makes every one of them a round trip of its own).
#pragma unroll
    for (int sp = 0; sp < SP; ++sp) {
      float w = INFINITY;
      if (sp < SP - 3 || sp < S) {
        const int m_raw = __builtin_amdgcn_readlane(mprev, sp);
        const int m = (m_raw < 0 || m_raw > E + 1) ? E + 1 : m_raw;
        const int idx = e0d - m;
        w = Tp[(size_t)sp * (EP >> 6) + ((idx > 0 ? idx : 0) >> 6)];
      }
      cp[0][sp] = w;
    }
#pragma unroll
    for (int sp = 0; sp < SP; ++sp) {
      if (sp < SP - 3 || sp < S) {
        const int m_raw = __builtin_amdgcn_readlane(mprev, sp);
        const int m = (m_raw < 0 || m_raw > E + 1) ? E + 1 : m_raw;
        const int idx = e0d - m;
        const float* again = &Tp[(size_t)sp * (EP >> 6) + ((idx > 0 ? idx : 0) >> 6)];
        const float* cell = &Cp[(size_t)sp * EP + e0d];
        cp[0][sp] = *(is_nan_bits(__float_as_int(cp[0][sp])) ? cell : again);
      }
    }
#pragma unroll
    for (int sp = 0; sp < SP; ++sp) {
      if (sp < SP - 3 || sp < S) {
        const int m_raw = __builtin_amdgcn_readlane(mprev, sp);
        const int m = (m_raw < 0 || m_raw > E + 1) ? E + 1 : m_raw;
        cp[0][sp] = e0d < m ? INFINITY : cp[0][sp];
      }
    }
  } else {
#pragma unroll
    for (int sp = 0; sp < SP; ++sp) {
#pragma unroll
      for (int j = 0; j < K; ++j)
        {
        // a large launch reads every table value exactly once: streaming loads leave the
        // caches to the stores; a split launch is small enough to find its table in cache
        const float* src = &Cp[(size_t)sp * EP + e0d + 64 * j];
        cp[j][sp] = !(sp < SP - 3 || sp < S) ? INFINITY : SPLIT ? *src : __builtin_nontemporal_load(src);
      }
    }
  }

  if (RUNS) {
    // The summaries speak for whole groups of 64 budgets of the previous layer's product, and a
    // column of this wave lies across two of them: about half of the waves that arrive here
    // have 64 equal columns after all, as the loaded values show.  They take the run path too,
    // with the column put together from the first lane's values.
    bool differs = false;
#pragma unroll
    for (int sp = 0; sp < SP; ++sp) {
      const int b = __float_as_int(cp[0][sp]);
      differs = differs || (b != __builtin_amdgcn_readfirstlane(b));
    }
    if (__builtin_amdgcn_ballot_w64(differs && e0 <= E) == 0) {
      float colv = INFINITY;
#pragma unroll
      for (int sp = 0; sp < SP; ++sp) {
        const int f = __builtin_amdgcn_readfirstlane(__float_as_int(cp[0][sp]));
        colv = (lane == sp) ? __int_as_float(f) : colv;
      }
      uniform_tile<SP, ARG>(colv, rt_lds, s_begin, s_end, lane, e0, wbase, Cn,
                            GROUPS ? group_records(t, row) : nullptr, sum_cur, E, EP, counts ? counts + 2 : nullptr);
      return;
    }
  }

  // this wave's records will be in A, whatever its summary words say (said here, before the row
  // loop, where registers are free)
  if (GROUPS) {
    uint8_t* __restrict__ Ag = group_records(t, row);
    if (Ag && s_begin + lane < s_end) Ag[(size_t)(s_begin + lane) * (EP >> 6) + (wbase >> 6)] = (uint8_t)kNoGroupRecord;
  }

  if (!ARG) {
    // Values only: the argmin records are not materialised (the walkers recompute the
    // one record they need per layer from the kept tables).  One add and half a
    // three-input min per candidate; the R row is consumed quad by quad as it arrives.
    static_assert(K == 1 || ARG, "the values-only path handles one budget per lane");
    float4 rowq[PRE ? PD : 1];
    if (PRE) {
#pragma unroll
      for (int q = 0; q < PD; ++q) rowq[q] = rt_lds[s_begin * RQ + (q < RQ ? q : RQ - 1)];
    }
#pragma unroll 1
    for (int s = s_begin; s < s_end; ++s) {
      float acc = INFINITY, cs = 0.0f;
      int m_raw = 0;
      const int s_next = (s + 1 < s_end) ? s + 1 : s;      // the last row is fetched once more, unused
#pragma unroll
      for (int q = 0; q < (PRE ? RQP : RQ); ++q) {
        float4 v;
        if (PRE) {
          const int nq = q + PD, qq = nq < RQP ? nq : nq - RQP;
          v = rowq[q % PD];
          rowq[q % PD] = rt_lds[(nq < RQP ? s : s_next) * RQ + (qq < RQ ? qq : RQ - 1)];
        } else v = rt_lds[s * RQ + q];
        const float rq[4] = {v.x, v.y, v.z, v.w};
        float xq[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) xq[i] = (4 * q + i < SP) ? cp[0][(4 * q + i < SP) ? 4 * q + i : 0] + rq[i] : INFINITY;
        if (4 * q + 3 < SP) {
          acc = fmin3(acc, xq[0], xq[1]);
          acc = fmin3(acc, xq[2], xq[3]);
        }
        // SP is a multiple of 4: c(l,s) and M(l,s) sit in the quad after the last candidates
        if (4 * q == SP) {
          cs = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(rq[0])));
          m_raw = __builtin_amdgcn_readfirstlane(__float_as_int(rq[1]));
        }
      }
      const int m = (m_raw < 0 || m_raw > E + 1) ? E + 1 : m_raw;
      float* Cs = Cn + (size_t)s * EP;
      const __amdgpu_buffer_rsrc_t bc = __builtin_amdgcn_make_buffer_rsrc(Cs, 0, (E + 1) * 4, kBufWord3);
      const __amdgpu_buffer_rsrc_t binf = __builtin_amdgcn_make_buffer_rsrc(Cs, 0, m * 4, kBufWord3);
      const int outb = __float_as_int(acc + cs);
      __builtin_amdgcn_raw_buffer_store_b32((unsigned)outb, bc, (e0 + m) * 4, 0, 0);
      if (!RUNS && wbase < m)                              // wave-uniform: some lane is below M (with
        __builtin_amdgcn_raw_buffer_store_b32(0x7f800000u, binf, e0 * 4, 0, 0);   // the run shortcut the readers know)
      if (true_sum) {
        // T + c is non-increasing along the budgets: all equal exactly when the ends are
        const int first = __builtin_amdgcn_readfirstlane(outb), last = __builtin_amdgcn_readlane(outb, n_in - 1);
        sumv = (lane == s - s_begin) ? (first == last ? first : kNaNBits) : sumv;
      }
    }
    if (want_sum && s_begin + lane < s_end)
      sum_cur[(size_t)(s_begin + lane) * (EP >> 6) + (wbase >> 6)] = __int_as_float(sumv);
    return;
  }

  static_assert(K == 1, "one budget per lane");
  float4 rowq[PRE ? PD : 1];
  if (PRE) {
#pragma unroll
    for (int q = 0; q < PD; ++q) rowq[q] = rt_lds[s_begin * RQ + (q < RQ ? q : RQ - 1)];
  }
#pragma unroll 1
  for (int s = s_begin; s < s_end; ++s) {
    const int s_next = (s + 1 < s_end) ? s + 1 : s;        // the last row is fetched once more, unused
    // ---- value pass, streaming: the R row is consumed quad by quad as it arrives from LDS,
    // candidates fold into chunk minima and those into the prefix minima at once, so that
    // only the prefix minima stay live (the sums are not kept: the rescan redoes the few it
    // needs).  c(l,s) and M(l,s) sit in the quad after the last candidates (SP % 4 == 0).
    float P[NP];
    float xs[CH], cm_odd = INFINITY;
    float cs = 0.0f;
    int m_raw = 0;
#pragma unroll
    for (int q = 0; q < (PRE ? RQP : RQ); ++q) {
      float4 v;
      if (PRE) {
        const int nq = q + PD, qq = nq < RQP ? nq : nq - RQP;
        v = rowq[q % PD];
        rowq[q % PD] = rt_lds[(nq < RQP ? s : s_next) * RQ + (qq < RQ ? qq : RQ - 1)];
      } else v = rt_lds[s * RQ + q];
      const float rq[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int i = 4 * q + i4;
        if (i < SP) {
          const int c = i / CH, pos = i % CH;
          xs[pos] = cp[0][i] + rq[i4];
          const int hi = ((c + 1) * CH < SP) ? (c + 1) * CH : SP;     // end of chunk c
          if (i == hi - 1) {                                          // chunk c complete
            const int len = hi - c * CH;
            const float cmv = len == 3 ? fmin3(xs[0], xs[1], xs[2])
                              : len == 2 ? __builtin_fminf(xs[0], xs[1]) : xs[0];
            if (c == 0) P[0] = cmv;
            else if (c % 2 == 1) {
              cm_odd = cmv;
              if (c == NC - 1) P[(c + 1) / 2] = __builtin_fminf(P[(c - 1) / 2], cm_odd);
            } else {
              P[c / 2] = fmin3(P[c / 2 - 1], cm_odd, cmv);
            }
          }
        }
      }
      if (4 * q == SP) {
        cs = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(rq[0])));
        m_raw = __builtin_amdgcn_readfirstlane(__float_as_int(rq[1]));
      }
    }
    const float T = P[NP - 1];
    // invalid (negative) M: the column is infeasible; beyond E + 1 nothing changes
    const int m = (m_raw < 0 || m_raw > E + 1) ? E + 1 : m_raw;
    // Stores go through buffer descriptors of column s: the address is a scalar base
    // plus the lane's byte offset (no per-lane pointer arithmetic in the loop), and
    // the hardware range check drops what lies outside [0, num_records):
    //   bc:   rows 0..E of column s         -> the shifted store at e' + m is dropped
    //                                          beyond E without a compare
    //   binf: rows 0..m-1 of column s       -> the +inf prefix
    //   ba:   rows 0..EP-1 of column s of A (padding rows are harmless)
    float* Cs = Cn + (size_t)s * EP;
    const __amdgpu_buffer_rsrc_t bc = __builtin_amdgcn_make_buffer_rsrc(Cs, 0, (E + 1) * 4, kBufWord3);
    const __amdgpu_buffer_rsrc_t binf = __builtin_amdgcn_make_buffer_rsrc(Cs, 0, m * 4, kBufWord3);
    const __amdgpu_buffer_rsrc_t ba = __builtin_amdgcn_make_buffer_rsrc(An + (size_t)s * EP, 0, EP, kBufWord3);
    {
      constexpr int j = 0;
      // ---- argmin: first block whose prefix minimum reaches T
      int arg = 0;
      bool prev = false;
      unsigned long long prevm = 0;
#pragma unroll
      for (int k = 0; k < NP; ++k) {
        const bool eq = (k == NP - 1) ? true : (P[k] == T);
        const unsigned long long eqm = (k == NP - 1) ? ~0ull : __builtin_amdgcn_ballot_w64(eq);
        if (__builtin_expect((eqm & ~prevm) != 0, 0)) {  // wave-uniform: a lane first hits block k
          if (eq && !prev) {
            const int clo = (k == 0) ? 0 : 2 * k - 1;    // chunks of block k
            const int chi = (k == 0) ? 1 : ((2 * k + 1 < NC) ? 2 * k + 1 : NC);
            const int lo = clo * CH, hi = (chi * CH < SP) ? chi * CH : SP;
            int a = hi - 1;                              // implied when no earlier one matches
            {
              // The sums are not kept: redo them from the R row (same operands, same
              // bits).  The row offset goes through an opaque register so that these
              // reads are not merged with the value pass's (which would keep the whole
              // row live), yet can be issued together.
              int roff = s * RS;
              asm volatile("" : "+v"(roff));
              const float* rl = reinterpret_cast<const float*>(rt_lds) + roff;
              float rr[2 * CH];
#pragma unroll
              for (int i = lo; i < hi - 1; ++i) rr[i - lo] = rl[i];
#pragma unroll
              for (int i = hi - 2; i >= lo; --i) a = (cp[j][i] + rr[i - lo] == T) ? i : a;
            }
            arg = a;
          }
        }
        prev = eq;
        prevm = eqm;
      }

      const int e = e0 + 64 * j;                         // pre-shift budget e'
      __builtin_amdgcn_raw_buffer_store_b8((unsigned char)arg, ba, e, 0, SPLIT ? 0 : kStreaming);
      const int outb = __float_as_int(T + cs);
      __builtin_amdgcn_raw_buffer_store_b32((unsigned)outb, bc, (e + m) * 4, 0, 0);
      if (!RUNS && wbase + 64 * j < m)                   // wave-uniform: some lane is below M (with
        __builtin_amdgcn_raw_buffer_store_b32(0x7f800000u, binf, e * 4, 0, 0);    // the run shortcut the readers know)
      if (true_sum) {
        const int first = __builtin_amdgcn_readfirstlane(outb), last = __builtin_amdgcn_readlane(outb, n_in - 1);
        sumv = (lane == s - s_begin) ? (first == last ? first : kNaNBits) : sumv;
      }
    }
  }
  if (want_sum && s_begin + lane < s_end)
    sum_cur[(size_t)(s_begin + lane) * (EP >> 6) + (wbase >> 6)] = __int_as_float(sumv);
}

// Any S up to 256 (used above 128): the C_{l-1} tile of 64 budgets is staged in LDS as
// [S][64]; wave w handles output strategies w, w+4, ...
__global__ __launch_bounds__(256) void k_minplus_generic(Tables t, int l, int tiles, int first) {
  extern __shared__ float lds[];
  const int inst = t.perm[first + blockIdx.x / tiles];
  const int tile = blockIdx.x % tiles;
  const int S = t.S, RS = t.RS, E = t.E, EP = t.EP;
  const int row = t.off[inst] + l;
  const float* __restrict__ Cp = c_table(t, inst, row - 1, l - 1);
  float* __restrict__ Cn = c_table(t, inst, row, l);
  uint8_t* __restrict__ An = t.A ? t.A + (size_t)row * S * EP : nullptr;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int e = tile * 64 + lane;

  for (int sp = wave; sp < S; sp += 4)
    lds[sp * 64 + lane] = (e <= E) ? Cp[(size_t)sp * EP + e] : INFINITY;
  __syncthreads();

  cf32_t Rrow = as_const(t.Rt) + (size_t)row * S * RS;
  for (int s = wave; s < S; s += 4) {
    float tmin = INFINITY;
    int arg = 0;
    for (int sp = 0; sp < S; ++sp) {
      const float x = lds[sp * 64 + lane] + Rrow[s * RS + sp];
      if (x < tmin) { tmin = x; arg = sp; }
    }
    const int m = t.M[(size_t)row * S + s];
    const float cs = t.c[(size_t)row * S + s];
    if (e <= E) {
      if (An) An[(size_t)s * EP + e] = (uint8_t)arg;
      if (m >= 0 && m <= E - e) Cn[(size_t)s * EP + e + m] = tmin + cs;
      if (m < 0 || e < m) Cn[(size_t)s * EP + e] = INFINITY;
    }
  }
}

template <int SP>
struct Blocking {                       // budgets per lane for a given strategy count
  static constexpr int K = 1;
  // waves per workgroup.  Beyond 64 strategies the R tile takes 20 to 68 KB of LDS, so that one or
  // two workgroups fit a compute unit: they are made large enough to bring the waves per SIMD
  // that the registers allow (4 up to 96 strategies, 3 up to 128)
  static constexpr int NW = (SP <= 64) ? 4 : (SP <= 96) ? 8 : 12;
  static constexpr int CH = 3;          // candidates per chunk minimum
  // waves per SIMD the register allocation must allow: SP live table values plus about 20
  // working registers out of 512 (the value pass streams the R row and keeps only the
  // prefix minima; the candidate sums are not kept)
  static constexpr int MINW = (SP <= 44) ? 8 : (SP <= 56) ? 6 : (SP <= 64) ? 5 : (SP <= 96) ? 4 : 3;
  static constexpr int MINW_SPLIT = 4;
  // the layer-1 variant builds layer 0 from c and M and needs a few registers more
  static constexpr int MINW_FIRST = (SP > 40 && SP <= 44) ? 7 : MINW;
  // without the argmin pass: the SP table values plus about 16 working registers
  static constexpr int MINW_VALUES = (SP <= 44) ? 8 : (SP <= 52) ? 7 : (SP <= 60) ? 6 : (SP <= 64) ? 5 : (SP <= 96) ? 4 : 3;
  // with the run shortcut compiled in: the summaries, the exchange, the second look at the
  // loaded columns and (up to 56 strategies) four quads of R in flight ahead of the fold (see
  // PRE in the kernel) take a few registers more; targets found by compiling every size.  The
  // values-only kernels would fit one wave more at some sizes; measured, that is no gain
  // (S=44: 7 waves 1.80 ms per solve, 5 or 4 waves 1.76).
  static constexpr int MINW_RUNS = (SP <= 24) ? 8 : (SP == 32) ? 6 : (SP <= 36) ? 7 : (SP <= 40) ? 6 : 5;   // (32: 7 spills four registers)
  static constexpr int MINW_VALUES_RUNS = (SP <= 24) ? 8 : (SP <= 28) ? 7 : (SP <= 32) ? 6 : (SP <= 40) ? 5
                                          : (SP <= 52) ? 4 : (SP <= 56) ? 3 : 5;
};

template <int SP>
static void launch_minplus_sp(const Tables& t_in, int l, int first, int n_active, int n_prev, hipStream_t st) {
  constexpr int K = Blocking<SP>::K, NW = Blocking<SP>::NW, CH = Blocking<SP>::CH,
                MINW = Blocking<SP>::MINW;
  Tables t = t_in;
  int tiles = (t.E + 1 + 64 * K * NW - 1) / (64 * K * NW);
  // fewer than two and a half workgroups per compute unit: split the strategies over the waves
  const int split = ((long long)tiles * n_active < 640) ? 1 : 0;
  // did the launch that produced this one's input split too (and so write every cell)?
  t.prev_full = (n_prev < 0 || (n_prev > 0 && (long long)tiles * n_prev < 640)) ? 1 : 0;
  if (split) tiles = (t.E + 1 + 64 * K - 1) / (64 * K);
  constexpr int RS = (SP + 2 + 3) / 4 * 4;
  const dim3 grid((unsigned)tiles * n_active), block(64 * NW);
  const size_t lds = (size_t)t.S * RS * sizeof(float);
  // Split launches are the small ones, where a wave's own latency counts and registers are
  // plentiful: a low occupancy target lets the compiler keep the whole R row in flight.
  constexpr int MS = Blocking<SP>::MINW_SPLIT;
#define GBMW_LAUNCH(MW, FIRST_, ARG_, SPLIT_, RUNS_)                                                        \
  hipLaunchKernelGGL((k_minplus<SP, K, NW, CH, MW, FIRST_, ARG_, SPLIT_, RUNS_>), grid, block, lds, st, t, l, \
                     tiles, first, make_deal(tiles, n_active))
  const bool runs = t.runs != 0;
  if (runs && !split && t.counts) {                      // the counting twin of the unsplit run-shortcut kernels
#define GBMW_LAUNCH_COUNT(FIRST_, ARG_)                                                                      \
  hipLaunchKernelGGL((k_minplus<SP, K, NW, CH, 2, FIRST_, ARG_, false, true, true>), grid, block, lds, st, t, l, \
                     tiles, first, make_deal(tiles, n_active))
    if (t.A == nullptr) { if (l == 1) GBMW_LAUNCH_COUNT(true, false); else GBMW_LAUNCH_COUNT(false, false); }
    else { if (l == 1) GBMW_LAUNCH_COUNT(true, true); else GBMW_LAUNCH_COUNT(false, true); }
#undef GBMW_LAUNCH_COUNT
    return;
  }
  if (t.A == nullptr) {
    constexpr int MW = Blocking<SP>::MINW_VALUES, MWR = Blocking<SP>::MINW_VALUES_RUNS;
    if (l == 1) {
      if (split) GBMW_LAUNCH(MS, true, false, true, false);
      else if (runs) GBMW_LAUNCH(MWR, true, false, false, true);
      else GBMW_LAUNCH(MW, true, false, false, false);
    } else {
      if (split) GBMW_LAUNCH(MS, false, false, true, false);
      else if (runs) GBMW_LAUNCH(MWR, false, false, false, true);
      else GBMW_LAUNCH(MW, false, false, false, false);
    }
  } else {
    constexpr int M1 = Blocking<SP>::MINW_FIRST, MR = Blocking<SP>::MINW_RUNS;
    if (l == 1) {
      if (split) GBMW_LAUNCH(MS, true, true, true, false);
      else if (runs) GBMW_LAUNCH(MR, true, true, false, true);
      else GBMW_LAUNCH(M1, true, true, false, false);
    } else {
      if (split) GBMW_LAUNCH(MS, false, true, true, false);
      else if (runs) GBMW_LAUNCH(MR, false, true, false, true);
      else GBMW_LAUNCH(MINW, false, true, false, false);
    }
  }
#undef GBMW_LAUNCH
}

// 65 to 128 strategies: the same register-blocked kernel, every lane with its S' table values
// in registers (148 to 168 of them at 128 strategies: three waves per SIMD), in larger workgroups
// (see Blocking::NW).  No run shortcut, no split shape, layer 0 read from memory.
template <int SP>
static void launch_minplus_big(const Tables& t, int l, int first, int n_active, hipStream_t st) {
  constexpr int NW = Blocking<SP>::NW, CH = Blocking<SP>::CH;
  const int tiles = (t.E + 1 + 64 * NW - 1) / (64 * NW);
  constexpr int RS = (SP + 2 + 3) / 4 * 4;
  const dim3 grid((unsigned)tiles * n_active), block(64 * NW);
  const size_t lds = (size_t)t.S * RS * sizeof(float);
  if (t.A == nullptr)
    hipLaunchKernelGGL((k_minplus<SP, 1, NW, CH, Blocking<SP>::MINW_VALUES, false, false, false, false>), grid, block, lds,
                       st, t, l, tiles, first, make_deal(tiles, n_active));
  else
    hipLaunchKernelGGL((k_minplus<SP, 1, NW, CH, Blocking<SP>::MINW, false, true, false, false>), grid, block, lds, st, t,
                       l, tiles, first, make_deal(tiles, n_active));
}

void launch_minplus(const Tables& t, int l, int first, int n_active, hipStream_t st, int n_prev) {
  if (n_active <= 0) return;
  switch (t.SP) {
#define GBMW_CASE(N) case N: launch_minplus_sp<N>(t, l, first, n_active, n_prev, st); return;
    GBMW_CASE(4) GBMW_CASE(8) GBMW_CASE(12) GBMW_CASE(16) GBMW_CASE(20) GBMW_CASE(24)
    GBMW_CASE(28) GBMW_CASE(32) GBMW_CASE(36) GBMW_CASE(40) GBMW_CASE(44) GBMW_CASE(48)
    GBMW_CASE(52) GBMW_CASE(56) GBMW_CASE(60) GBMW_CASE(64)
#undef GBMW_CASE
  // (a launch of fewer waves than the chip has SIMDs is better off with the generic kernel below,
  // whose waves divide the output strategies: four times the waves)
#define GBMW_CASE(N) case N: if ((long long)((t.E + 64) / 64) * n_active < 1024) break; launch_minplus_big<N>(t, l, first, n_active, st); return;
    GBMW_CASE(68) GBMW_CASE(72) GBMW_CASE(76) GBMW_CASE(80) GBMW_CASE(84) GBMW_CASE(88)
    GBMW_CASE(92) GBMW_CASE(96) GBMW_CASE(100) GBMW_CASE(104) GBMW_CASE(108) GBMW_CASE(112)
    GBMW_CASE(116) GBMW_CASE(120) GBMW_CASE(124) GBMW_CASE(128)
#undef GBMW_CASE
    default: break;
  }
  const int tiles = (t.E + 64) / 64;
  hipLaunchKernelGGL(k_minplus_generic, dim3((unsigned)tiles * n_active), dim3(256),
                     (size_t)t.S * 64 * sizeof(float), st, t, l, tiles, first);
}

bool layer0_in_registers(int S) { return S <= 64; }

bool launch_is_split(const Tables& t, int n_active) {
  return t.S <= 64 && (long long)((t.E + 256) / 256) * n_active < 640;
}

const char* minplus_variant(int S) {
  return S <= 128 ? "register-blocked, LDS-staged R tile, prefix-min value pass + on-demand argmin rescan"
                  : "generic LDS-staged (S > 128)";
}

// ---------------------------------------------------------------------------
// final reduce: best(e) = min_s C(L_b - 1, e, s), lowest-index argmin
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_final(Tables t, int first) {
  const int inst = t.perm[first + blockIdx.y];
  const int e = t.final_from + blockIdx.x * 256 + threadIdx.x;
  if (e > t.E) return;
  const int l = t.L[inst] - 1;
  const float* __restrict__ C = c_table(t, inst, t.off[inst] + l, l);
  float b = INFINITY;
  int a = 0;
  if (t.runs != 0) {
    // the summaries stand for the cells of their groups where they are numbers (table_cell)
    const float* __restrict__ Ts = sum_table(t, inst, t.off[inst] + l, l);
    const int* __restrict__ Ml = t.M + (size_t)(t.off[inst] + l) * t.S;
    int s = 0;
    for (; s + 8 <= t.S; s += 8) {
      float x[8], w[8];
      int idx[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int m = Ml[s + i];
        idx[i] = (m < 0) ? -1 : e - m;
        w[i] = Ts[(size_t)(s + i) * (t.EP >> 6) + ((idx[i] > 0 ? idx[i] : 0) >> 6)];
      }
      // the cell is asked for only where its group's word does not stand for it (most groups
      // of a step-function table are runs: their cells were never written and need not be read)
#pragma unroll
      for (int i = 0; i < 8; ++i)
        x[i] = (idx[i] >= 0 && is_nan_bits(__float_as_int(w[i]))) ? C[(size_t)(s + i) * t.EP + e] : w[i];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float v = idx[i] < 0 ? INFINITY : x[i];
        if (v < b) { b = v; a = s + i; }
      }
    }
    for (; s < t.S; ++s) {
      const float v = table_cell(t, C, Ts, Ml, s, e);
      if (v < b) { b = v; a = s; }
    }
    t.best[(size_t)inst * t.EP + e] = b;
    t.best_s[(size_t)inst * t.EP + e] = (uint8_t)a;
    return;
  }
  // eight loads in flight, then the compares in strategy order
  int s = 0;
  for (; s + 8 <= t.S; s += 8) {
    float x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = __builtin_nontemporal_load(&C[(size_t)(s + i) * t.EP + e]);
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (x[i] < b) { b = x[i]; a = s + i; }
  }
  for (; s < t.S; ++s) {
    const float x = C[(size_t)s * t.EP + e];
    if (x < b) { b = x; a = s; }
  }
  t.best[(size_t)inst * t.EP + e] = b;
  t.best_s[(size_t)inst * t.EP + e] = (uint8_t)a;
}

void launch_final(const Tables& t, int first, int count, hipStream_t st) {
  if (count <= 0) return;
  hipLaunchKernelGGL(k_final, dim3((t.E - t.final_from + 256) / 256, count), dim3(256), 0, st, t, first);
}

// ---------------------------------------------------------------------------
// backtrack: one lane per query walks the argmin records from the last layer
// down; each step is one dependent byte gather.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_backtrack(Tables t, int nq, const int* __restrict__ q_inst,
                                                  const int* __restrict__ q_e, int Lmax,
                                                  uint8_t* __restrict__ plan,
                                                  float* __restrict__ cost,
                                                  int* __restrict__ mem_used) {
  const int q = blockIdx.x * 64 + threadIdx.x;
  if (q >= nq) return;
  const int inst = q_inst[q];
  int e = q_e[q];
  uint8_t* p = plan + (size_t)q * Lmax;
  const int Lb = t.L[inst];
  const float b = t.best[(size_t)inst * t.EP + e];
  cost[q] = b;
  if (b == INFINITY) {
    for (int l = 0; l < Lmax; ++l) p[l] = 0xFF;
    mem_used[q] = -1;
    return;
  }
  for (int l = Lb; l < Lmax; ++l) p[l] = 0xFF;
  int s = t.best_s[(size_t)inst * t.EP + e];
  const int row0 = t.off[inst];
  int mem = 0;
  for (int l = Lb - 1; l >= 1; --l) {
    p[l] = (uint8_t)s;
    const int m = t.M[(size_t)(row0 + l) * t.S + s];
    mem += m;
    e -= m;                                            // budget left for layers < l
    if (m < 0 || e < 0) { mem = -2; break; }           // only reachable with invalid inputs
    s = pred_strategy(t, row0 + l, s, e);
  }
  if (mem != -2) {
    p[0] = (uint8_t)s;
    mem += t.M[(size_t)row0 * t.S + s];
  }
  mem_used[q] = mem;
}

// The same walk without argmin records: every step has to redo the minimum over the S
// predecessors from the kept table of the layer below, so a whole wave takes one query, its
// lanes over the predecessors (pred_strategy_wave), and lane 0 writes the plan.
__global__ __launch_bounds__(256) void k_backtrack_wave(Tables t, int nq, const int* __restrict__ q_inst,
                                                        const int* __restrict__ q_e, int Lmax,
                                                        uint8_t* __restrict__ plan, float* __restrict__ cost,
                                                        int* __restrict__ mem_used) {
  const int q = blockIdx.x * 4 + (threadIdx.x >> 6);      // wave-uniform
  const int lane = threadIdx.x & 63;
  if (q >= nq) return;
  const int inst = q_inst[q];
  int e = q_e[q];
  uint8_t* p = plan + (size_t)q * Lmax;
  const int Lb = t.L[inst];
  const float b = t.best[(size_t)inst * t.EP + e];
  if (b == INFINITY) {
    for (int l = lane; l < Lmax; l += 64) p[l] = 0xFF;
    if (lane == 0) { cost[q] = b; mem_used[q] = -1; }
    return;
  }
  for (int l = Lb + lane; l < Lmax; l += 64) p[l] = 0xFF;
  int s = t.best_s[(size_t)inst * t.EP + e];
  const int row0 = t.off[inst];
  int mem = 0;
  for (int l = Lb - 1; l >= 1; --l) {
    if (lane == 0) p[l] = (uint8_t)s;
    const int m = t.M[(size_t)(row0 + l) * t.S + s];
    mem += m;
    e -= m;                                              // budget left for layers < l
    if (m < 0 || e < 0) { mem = -2; break; }             // only reachable with invalid inputs
    s = pred_strategy_wave(t, row0 + l, s, e, lane);
  }
  if (mem != -2) {
    if (lane == 0) p[0] = (uint8_t)s;
    mem += t.M[(size_t)row0 * t.S + s];
  }
  if (lane == 0) { cost[q] = b; mem_used[q] = mem; }
}

void launch_backtrack(const Tables& t, int nq, const int* q_inst, const int* q_e, int Lmax,
                      uint8_t* plan, float* cost, int* mem_used, hipStream_t st) {
  if (nq <= 0) return;
  if (t.A == nullptr) {
    hipLaunchKernelGGL(k_backtrack_wave, dim3((nq + 3) / 4), dim3(256), 0, st, t, nq, q_inst, q_e, Lmax, plan, cost,
                       mem_used);
    return;
  }
  hipLaunchKernelGGL(k_backtrack, dim3((nq + 63) / 64), dim3(64), 0, st, t, nq, q_inst, q_e, Lmax,
                     plan, cost, mem_used);
}

// ---------------------------------------------------------------------------
// Algorithm 3's outer loop.  walk_plan follows the argmin records of instance
// `inst` from budget e down and evaluates Eq. 2 on the way.  Going from the last
// layer to the first, the forward prefix of layer i is F - suf_i with F the sum
// of all O_f and suf_i the sum over the layers above i, so
//   E_all = F + max_i (O_b(i) - suf_i) + sum O_ms.
// ---------------------------------------------------------------------------
__device__ long long walk_plan(const Tables& t, int inst, int e, const int* __restrict__ Of,
                               const int* __restrict__ Ob, const int* __restrict__ Oms,
                               uint8_t* plan) {
  const int Lb = t.L[inst], row0 = t.off[inst], S = t.S;
  int s = t.best_s[(size_t)inst * t.EP + e];
  long long suf = 0, ms = 0, mx = 0;
  for (int l = Lb - 1; l >= 0; --l) {
    const size_t cell = (size_t)(row0 + l) * S + s;
    if (plan) plan[l] = (uint8_t)s;
    const long long here = (long long)Ob[cell] - suf;
    mx = (l == Lb - 1 || here > mx) ? here : mx;
    suf += Of[cell];
    ms += Oms[cell];
    if (l > 0) {
      const int m = t.M[cell];
      e -= m;                                            // budget left for layers < l
      if (m < 0 || e < 0) return -2;                     // only reachable with invalid inputs
      s = pred_strategy(t, row0 + l, s, e);
    }
  }
  return suf + mx + ms;
}

__global__ void k_select_init(int B, int* first_bad) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) first_bad[b] = 0x7fffffff;
}

// one lane per (instance, budget of its window): record the lowest budget
// whose plan does not fit the overall memory
__global__ __launch_bounds__(64) void k_select_check(Tables t, const int* __restrict__ Of,
                                                     const int* __restrict__ Ob,
                                                     const int* __restrict__ Oms,
                                                     const int* __restrict__ bup,
                                                     int* __restrict__ first_bad) {
  const int inst = blockIdx.y;
  const int base = t.E - bup[inst];                      // last budget that needs no check
  const int lo = (base < 0 ? -1 : base) + 1;
  const int e = lo + blockIdx.x * 64 + threadIdx.x;
  if (e > t.E) return;
  if (t.best[(size_t)inst * t.EP + e] == INFINITY) return;   // no plan: nothing to check
  const long long ea = walk_plan(t, inst, e, Of, Ob, Oms, nullptr);
  if (ea > (long long)t.E || ea < 0) atomicMin(&first_bad[inst], e);
}

__global__ __launch_bounds__(64) void k_select_pick(Tables t, const int* __restrict__ Of,
                                                    const int* __restrict__ Ob,
                                                    const int* __restrict__ Oms,
                                                    const int* __restrict__ bup,
                                                    const int* __restrict__ first_bad, int Lmax,
                                                    int* __restrict__ e_opt,
                                                    float* __restrict__ cost,
                                                    uint8_t* __restrict__ plan,
                                                    int* __restrict__ e_all) {
  const int inst = blockIdx.x * 64 + threadIdx.x;
  if (inst >= t.B) return;
  const int base = t.E - bup[inst];
  const int init = base < 0 ? -1 : base;
  const int fb = first_bad[inst];
  const int last = (fb == 0x7fffffff) ? t.E : fb - 1;
  int opt = init;
  if (last > init && t.best[(size_t)inst * t.EP + last] != INFINITY) opt = last;
  uint8_t* p = plan + (size_t)inst * Lmax;
  for (int l = 0; l < Lmax; ++l) p[l] = 0xFF;
  e_opt[inst] = opt;
  float cst = INFINITY;
  long long ea = -1;
  if (opt >= 0) {
    cst = t.best[(size_t)inst * t.EP + opt];
    if (cst != INFINITY) ea = walk_plan(t, inst, opt, Of, Ob, Oms, p);
  }
  cost[inst] = cst;
  e_all[inst] = (int)ea;
}

void launch_select(const Tables& t, const int* Of, const int* Ob, const int* Oms, const int* bup,
                   int max_window, int Lmax, int* first_bad, int* e_opt, float* cost,
                   uint8_t* plan, int* e_all, hipStream_t st) {
  hipLaunchKernelGGL(k_select_init, dim3((t.B + 63) / 64), dim3(64), 0, st, t.B, first_bad);
  if (max_window > 0)
    hipLaunchKernelGGL(k_select_check, dim3((max_window + 63) / 64, t.B), dim3(64), 0, st, t, Of,
                       Ob, Oms, bup, first_bad);
  hipLaunchKernelGGL(k_select_pick, dim3((t.B + 63) / 64), dim3(64), 0, st, t, Of, Ob, Oms, bup,
                     first_bad, Lmax, e_opt, cost, plan, e_all);
}

// ---------------------------------------------------------------------------
// Pipeline time (Eq. 5 / Eq. 8).  One lane per stage walks its plan down the
// argmin records into a scratch row, then re-evaluates it upward with the costs
// without gradient synchronisation; R(l, s', s) is read from the transposed
// table Rt[row][s][s'].
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_stage_cost(Tables t, int n_stage,
                                                   const int* __restrict__ st_inst,
                                                   const int* __restrict__ st_e,
                                                   const float* __restrict__ c_ns,
                                                   uint8_t* __restrict__ plan_scratch, int Lmax,
                                                   float* __restrict__ st_C,
                                                   float* __restrict__ st_Cns) {
  const int q = blockIdx.x * 64 + threadIdx.x;
  if (q >= n_stage) return;
  const int inst = st_inst[q];
  int e = st_e[q];
  float C = INFINITY, Cns = INFINITY;
  if (e >= 0) C = t.best[(size_t)inst * t.EP + e];
  if (C != INFINITY) {
    if (!c_ns) {
      Cns = C;
    } else {
      const int Lb = t.L[inst], row0 = t.off[inst], S = t.S;
      uint8_t* plan = plan_scratch + (size_t)q * Lmax;
      int s = t.best_s[(size_t)inst * t.EP + e];
      bool ok = true;
      for (int l = Lb - 1; l >= 1; --l) {
        plan[l] = (uint8_t)s;
        e -= t.M[(size_t)(row0 + l) * S + s];
        if (e < 0) { ok = false; break; }                // only reachable with invalid inputs
        s = pred_strategy(t, row0 + l, s, e);
      }
      if (ok) {
        plan[0] = (uint8_t)s;
        float v = c_ns[(size_t)row0 * S + s];
        for (int l = 1; l < Lb; ++l) {
          const int sn = plan[l];
          const float r = t.Rt[((size_t)(row0 + l) * S + sn) * t.RS + s];
          v = (v + r) + c_ns[(size_t)(row0 + l) * S + sn];
          s = sn;
        }
        Cns = v;
      }
    }
  }
  st_C[q] = C;
  st_Cns[q] = Cns;
}

__global__ __launch_bounds__(64) void k_pipeline_cost(int n_pipe, const int* __restrict__ st_begin,
                                                      const int* __restrict__ mb,
                                                      const float* __restrict__ st_C,
                                                      const float* __restrict__ st_Cns,
                                                      float* __restrict__ cost) {
  const int p = blockIdx.x * 64 + threadIdx.x;
  if (p >= n_pipe) return;
  const int b = st_begin[p], e = st_begin[p + 1];
  float total = st_C[b], mx = st_Cns[b];
  for (int i = b + 1; i < e; ++i) {
    total = total + st_C[i];
    mx = st_Cns[i] > mx ? st_Cns[i] : mx;
  }
  float out = INFINITY;
  if (total != INFINITY && mx != INFINITY) {
    const float head = (float)(mb[p] - 1) * mx;
    out = head + total;
  }
  cost[p] = out;
}

void launch_pipeline_cost(const Tables& t, int n_stage, const int* st_inst, const int* st_e,
                          const float* c_ns, uint8_t* plan_scratch, int Lmax, float* st_C,
                          float* st_Cns, int n_pipe, const int* st_begin, const int* mb,
                          float* cost, hipStream_t st) {
  hipLaunchKernelGGL(k_stage_cost, dim3((n_stage + 63) / 64), dim3(64), 0, st, t, n_stage, st_inst,
                     st_e, c_ns, plan_scratch, Lmax, st_C, st_Cns);
  hipLaunchKernelGGL(k_pipeline_cost, dim3((n_pipe + 63) / 64), dim3(64), 0, st, n_pipe, st_begin,
                     mb, st_C, st_Cns, cost);
}

// ---------------------------------------------------------------------------
// export: device [n][S][EP] -> logical [n][E+1][S] through a 64x64 LDS tile
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_export(const T* __restrict__ src, T* __restrict__ dst, int S,
                                                int E, int EP) {
  __shared__ T tile[64][65];
  const int n = blockIdx.z;
  const int e0 = blockIdx.x * 64, s0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const T* in = src + (size_t)n * S * EP;
  T* out = dst + (size_t)n * (E + 1) * S;
  for (int i = ty; i < 64; i += 4) {
    const int s = s0 + i, e = e0 + tx;
    if (s < S && e <= E) tile[i][tx] = in[(size_t)s * EP + e];
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int e = e0 + i, s = s0 + tx;
    if (s < S && e <= E) out[(size_t)e * S + s] = tile[tx][i];
  }
}

__global__ __launch_bounds__(256) void k_argmin_row(Tables t, int row, uint8_t* __restrict__ dst) {
  const int e = blockIdx.x * 256 + threadIdx.x, s = blockIdx.y;
  if (e >= t.EP) return;
  dst[(size_t)s * t.EP + e] = (e <= t.E) ? (uint8_t)pred_strategy(t, row, s, e) : 0;
}

void launch_argmin_row(const Tables& t, int row, uint8_t* dst, hipStream_t st) {
  hipLaunchKernelGGL(k_argmin_row, dim3(t.EP / 256, t.S), dim3(256), 0, st, t, row, dst);
}

__global__ __launch_bounds__(256) void k_export_c(Tables t, const float* __restrict__ Ctab,
                                                  const float* __restrict__ Tsum_tab, const int* __restrict__ Mrow,
                                                  float* __restrict__ dst) {
  const int e = blockIdx.x * 256 + threadIdx.x, s = blockIdx.y;
  if (e > t.E) return;
  dst[(size_t)e * t.S + s] = table_cell(t, Ctab, Tsum_tab, Mrow, s, e);
}
void launch_export_c(const Tables& t, const float* Ctab, const float* Tsum_tab, const int* Mrow, float* dst,
                     hipStream_t st) {
  hipLaunchKernelGGL(k_export_c, dim3((t.E + 256) / 256, t.S), dim3(256), 0, st, t, Ctab, Tsum_tab, Mrow, dst);
}
void launch_export_u8(const uint8_t* src, uint8_t* dst, int n, int S, int E, int EP,
                      hipStream_t st) {
  hipLaunchKernelGGL(k_export<uint8_t>, dim3((E + 64) / 64, (S + 63) / 64, n), dim3(256), 0, st,
                     src, dst, S, E, EP);
}

}  // namespace gbmw
