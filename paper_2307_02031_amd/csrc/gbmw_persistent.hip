// The whole table fill of a SMALL problem in one launch (Section 4.1.2, Eq. 3 for every
// layer, then best(e) = min_s C(L-1, e, s)).
//
// A problem whose row tiles all fit on the chip at once is bound by the latency of its
// per-layer launches (a few microseconds of work between launches of 5 to 10 microseconds
// each).  Here one workgroup owns one tile of 64 budgets of one instance for the whole solve
// and walks the layers itself.  What a tile needs from other tiles is local along the budget
// axis: the min-plus product of tile j reads column entries C(l-1, e, .) of its OWN budgets
// only, and those were written, shifted by M(l-1, s), by the tiles at or below j within
// max_s M(l-1, s) budgets.  So there is no grid-wide barrier: every tile publishes the number
// of layers it has finished in a word of its own (one store, single writer, once its table
// stores are acknowledged), and a tile about to start layer l polls the words of the tiles in
// its window until all of them show l - 1:
//   - below:  tiles j - ceil(max_s M(l-1,s) / 64) .. j   (their stores make up my input)
//   - above:  tiles j .. j + (63 + max_s M(l,s)) / 64    (rolling pair of tables only: my
//             stores of layer l overwrite layer l - 2, which those tiles read in step l - 1)
// One wave polls, 64 words per load.  The R tiles are transposed inside the same launch (row
// l of an instance by its tile l mod tiles) and published the same way.  All words carry the
// solve's epoch, which only grows, so nothing has to be cleared between solves.
//
// Visibility without cache flushes: the chip's eight L2 caches are not coherent with each other
// for ordinary accesses, and a device-scope fence pair (write back one L2, invalidate another) per
// tile and layer costs more than the layer.  Instead everything one workgroup writes for another
// (table cells, R tiles, the words) is written and read with device-scope accesses (relaxed
// atomic loads and stores, "sc1": they go to the memory side and do not stop at a stale line of the
// local L2), the writer waits for its stores to be acknowledged before it publishes its word, and
// the reader polls the word before it issues its loads.
//
// Every wait is bounded (clock ticks and polls): a tile that gives up records it, tells all
// others to leave, and the kernel ends normally; the host reports GBMW_ERR_DEVICE.  The host
// takes this path only when the occupancy query says the whole grid is resident at once.
#include "gbmw_kernels.h"

#include <math.h>

namespace gbmw {

namespace {

constexpr int kBufWord3 = 0x00020000;   // raw buffer descriptor word 3: 32-bit data format, no swizzle

__device__ __forceinline__ float fmin3(float a, float b, float c) {
  return __builtin_fminf(__builtin_fminf(a, b), c);
}

__device__ __forceinline__ float* c_table(const Tables& t, int inst, int row, int l) {
  const size_t slab = (size_t)t.S * t.EP;
  return t.keep_all ? t.Cbuf + (size_t)row * slab : t.Cbuf + ((size_t)(l & 1) * t.B + inst) * slab;
}

__device__ __forceinline__ unsigned long long load_word(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// device-scope accesses to data that another workgroup wrote or will read
__device__ __forceinline__ float load_shared(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_shared(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// cache policy of a buffer store: device scope (sc1)
constexpr int kDeviceScope = 16;
// the wave's stores have been acknowledged and later accesses are not moved above this point
__device__ __forceinline__ void stores_done() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup"); }
__device__ __forceinline__ void loads_after() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup"); }

// Largest M(row, s) that leads to a store (0 <= M <= E), over the strategies; 0 if none.
// Every lane of the wave gets the result.
__device__ __forceinline__ int max_shift(const int* __restrict__ Mrow, int S, int E, int lane) {
  int m = 0;
  for (int s = lane; s < S; s += 64) {
    const int v = Mrow[s];
    if (v >= 0 && v <= E && v > m) m = v;
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const int o = __shfl_xor(m, d, 64);
    m = o > m ? o : m;
  }
  return m;
}

// Wave 0 of a workgroup waits until every word prog[lo..hi] has reached `target`.  Returns false
// if it gave up (recorded in the header) or was told to leave.  Bounded by ticks of the constant
// 100 MHz clock and by polls.  (Two samples in flight half a round trip apart, tried, change
// nothing: what a tile waits for is its neighbours' stores on their way through the memory side.)
__device__ bool wait_for(const PersistArgs& a, const unsigned long long* prog, int lo, int hi,
                         unsigned long long target, int lane) {
  const long long t0 = (long long)wall_clock64();
  int polls = 0;
  for (;;) {
    bool ok = true;
    for (int k = lo + lane; k <= hi; k += 64) ok = ok && load_word(prog + k) >= target;
    const bool leave = load_word(a.sync + kSyncLeave) == a.epoch;
    if (__builtin_amdgcn_ballot_w64(!ok) == 0) return true;
    if (__builtin_amdgcn_ballot_w64(leave) != 0) return false;
    ++polls;
    if (polls > a.wait_polls || (long long)wall_clock64() - t0 > a.wait_ticks) {
      if (lane == 0) {
        atomicMax(a.sync + kSyncGaveUp, a.epoch);
        atomicMax(a.sync + kSyncLeave, a.epoch);
      }
      return false;
    }
    __builtin_amdgcn_s_sleep(2);
  }
}

// Rt[row][s][0..SP) = R[row][.][s] (zero padding), Rt[row][s][SP] = c, Rt[row][s][SP+1] = bits of
// M, with validation of device-resident inputs and the context's own copies of c and M: the
// work of the prepare kernel for one table row, by one workgroup.
__device__ void prepare_row(const Tables& t, const PersistArgs& a, int row, bool layer0) {
  const int S = t.S, SP = t.SP, RS = t.RS;
  float* __restrict__ Rt = const_cast<float*>(t.Rt) + (size_t)row * S * RS;
  const float* __restrict__ R = a.R + (size_t)row * S * S;
  const bool copy = a.src_c != t.c;
  int bad = 0;
  for (int i = threadIdx.x; i < S * RS; i += blockDim.x) {
    const int sp = i % RS, s = i / RS;
    float v = 0.0f;
    if (sp < S) {
      v = R[(size_t)sp * S + s];
      if (a.validate && !layer0 && !(v >= 0.0f)) bad |= 4;          // the l == 0 slab may hold anything
    } else if (sp == SP) {
      v = a.src_c[(size_t)row * S + s];
      if (a.validate && !(v >= 0.0f)) bad |= 1;
      if (copy) const_cast<float*>(t.c)[(size_t)row * S + s] = v;
    } else if (sp == SP + 1) {
      const int m = a.src_M[(size_t)row * S + s];
      if (a.validate && m < 0) bad |= 2;
      if (copy) const_cast<int*>(t.M)[(size_t)row * S + s] = m;
      v = __int_as_float(m);
    }
    store_shared(Rt + i, v);
  }
  if (bad & 1) atomicMax(a.sync + kSyncBadC, a.epoch);
  if (bad & 2) atomicMax(a.sync + kSyncBadM, a.epoch);
  if (bad & 4) atomicMax(a.sync + kSyncBadR, a.epoch);
}

}  // namespace

// One workgroup of NW waves per (instance, tile of 64 budgets); the waves share the tile and
// divide the output strategies.  A lane owns one budget e'.
template <int SP, int NW, bool ARG>
__global__ __launch_bounds__(64 * NW, (NW >= 8 && SP <= 44) ? 4 : 2) void k_layers(Tables t, PersistArgs a) {
  constexpr int CH = 3;                                  // candidates per chunk minimum
  constexpr int NC = (SP + CH - 1) / CH;                 // chunks (the last may be short)
  constexpr int RS = (SP + 2 + 3) / 4 * 4;
  constexpr int RQ = RS / 4;
  constexpr int NSTG = (SP * RQ * 2 + 64 * NW - 1) / (64 * NW);   // 8-byte words of the R tile per thread
  constexpr int NCOL = (SP + NW - 1) / NW;               // table columns a wave fetches for the workgroup
  extern __shared__ float4 lds[];
  float4* const rt_lds = lds;                            // [S][RQ]   the layer's R tile
  float* const cp_lds = reinterpret_cast<float*>(lds + SP * RQ);   // [SP][64] the tile's table values
  __shared__ int go;

  const int slot = blockIdx.x / a.tiles, tile = blockIdx.x % a.tiles;
  const int inst = t.perm[a.first + slot];
  const int S = t.S, E = t.E, EP = t.EP;
  const int Lb = t.L[inst], row0 = t.off[inst];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int wbase = tile * 64, e0 = wbase + lane;
  const int s_begin = (wave * S) / NW, s_end = ((wave + 1) * S) / NW;
  const int n_tile = (E - wbase + 1 < 64) ? E - wbase + 1 : 64;   // budgets of the tile inside the table
  const bool thin = n_tile <= 8;
  unsigned long long* const prep = a.sync + kSyncHeader;                     // [sumL]
  unsigned long long* const prog = prep + a.sumL + (size_t)slot * a.tiles;   // [tiles] of this instance
  const unsigned long long base = a.epoch << 20;
  const unsigned long long never = a.extra_wait ? (1ull << 19) : 0ull;       // testing: a layer that never comes

  // ---- the R tiles of this instance: tile k transposes the rows of layers k, k + tiles, ...
  for (int l = tile; l < Lb; l += a.tiles) {
    prepare_row(t, a, row0 + l, l == 0);
    stores_done();
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(prep + row0 + l, a.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // ... and waits until all of them are there (once; the rows are few and done at once)
  if (Lb >= 2) {
    if (wave == 0) {
      const bool ok = wait_for(a, prep + row0, 1, Lb - 1, a.epoch, lane);
      if (lane == 0) go = ok ? 1 : 0;
    }
    __syncthreads();
    if (!go) return;
    loads_after();
  }

  // ---- layer 0 in memory where something reads it from there (every layer kept; one or two layers)
  const float* __restrict__ c0 = a.src_c + (size_t)row0 * S;
  const int* __restrict__ m0 = a.src_M + (size_t)row0 * S;
  if (t.keep_all || Lb <= 2) {
    float* C0 = c_table(t, inst, row0, 0);
    for (int s = s_begin; s < s_end; ++s) {
      const int m = m0[s];
      C0[(size_t)s * EP + e0] = (m >= 0 && e0 >= m && e0 <= E) ? c0[s] : INFINITY;
    }
  }

  int mprev = 0;                                         // max_s M(l-1, s) among the shifts that store
  for (int l = 1; l < Lb; ++l) {
    const int row = row0 + l;
    // ---- ask for the R tile of layer l now; it goes into LDS after the wait
    unsigned long long stg[NSTG];
    {
      const unsigned long long* __restrict__ src =
          reinterpret_cast<const unsigned long long*>(t.Rt + (size_t)row * S * RS);
#pragma unroll
      for (int k = 0; k < NSTG; ++k) {
        const int i = threadIdx.x + k * 64 * NW;
        stg[k] = (i < S * RQ * 2) ? load_word(src + i) : 0ull;
      }
    }
    // ---- wait for the neighbours' layer l - 1
    if (l >= 2) {
      if (wave == 0) {
        const int mcur = max_shift(a.src_M + (size_t)row * S, S, E, lane);
        const int lo = tile - (mprev + 63) / 64;
        const int hi = t.keep_all ? tile : tile + (63 + mcur) / 64;
        const bool ok = wait_for(a, prog, lo < 0 ? 0 : lo, hi > a.tiles - 1 ? a.tiles - 1 : hi,
                                 base + (unsigned)(l - 1) + never, lane);
        mprev = mcur;
        if (lane == 0) go = ok ? 1 : 0;
      }
      __syncthreads();
      if (!go) return;                                   // every wave of the workgroup leaves
      loads_after();
    } else if (wave == 0) {
      mprev = max_shift(a.src_M + (size_t)row * S, S, E, lane);
    }

    // ---- the tile's table values: every wave fetches a share of the columns for all of them
    if (l >= 2 && !thin) {
      const float* __restrict__ Cp = c_table(t, inst, row - 1, l - 1);
      float col[NCOL];
#pragma unroll
      for (int k = 0; k < NCOL; ++k) {
        const int sp = wave + k * NW;
        col[k] = (sp < S) ? load_shared(&Cp[(size_t)sp * EP + e0]) : INFINITY;
      }
#pragma unroll
      for (int k = 0; k < NCOL; ++k) {
        const int sp = wave + k * NW;
        if (sp < SP) cp_lds[sp * 64 + lane] = col[k];
      }
    }
    {
      unsigned long long* dst = reinterpret_cast<unsigned long long*>(rt_lds);
#pragma unroll
      for (int k = 0; k < NSTG; ++k) {
        const int i = threadIdx.x + k * 64 * NW;
        if (i < S * RQ * 2) dst[i] = stg[k];
      }
    }
    __syncthreads();
    float* __restrict__ Cn = c_table(t, inst, row, l);
    uint8_t* __restrict__ An = ARG ? t.A + (size_t)row * S * EP : nullptr;
    if (thin) {
      // A last tile of a few budgets (E + 1 just above a multiple of 64) would cost its compute
      // unit, which it shares with another tile, a whole tile's arithmetic for nearly nothing.
      // Its budgets are computed one by one instead, with the lanes over the OUTPUT strategies:
      // lane s folds min_s' (C_{l-1}[e][s'] + R[s'][s]) in index order with a strict compare (the
      // lowest minimiser, 0 if all are +inf), then adds c(l, s).  Same operands, same bits.
      const float* __restrict__ Cp = c_table(t, inst, row - 1, l - 1);
      const int srow = lane < S ? lane : 0;
      for (int b = wave; b < n_tile; b += NW) {
        const int e = wbase + b;
        float colv = INFINITY;                             // lane s': C_{l-1}[e][s']
        if (lane < S) {
          if (l == 1) { const int mv = m0[lane]; colv = (mv >= 0 && e >= mv) ? c0[lane] : INFINITY; }
          else colv = load_shared(&Cp[(size_t)lane * EP + e]);
        }
        float best = INFINITY;
        int arg = 0;
#pragma unroll
        for (int q = 0; q < SP / 4; ++q) {
          const float4 v = rt_lds[srow * RQ + q];
          const float rq[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            const float f = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(colv), 4 * q + i4));
            const float x = f + rq[i4];
            if (x < best) { best = x; arg = 4 * q + i4; }
          }
        }
        const float4 tl = rt_lds[srow * RQ + SP / 4];      // c(l, s) and the bits of M(l, s), per lane
        if (lane < S) {
          const int m_raw = __float_as_int(tl.y);
          const int m = (m_raw < 0 || m_raw > E + 1) ? E + 1 : m_raw;
          if (ARG) An[(size_t)lane * EP + e] = (uint8_t)arg;
          if (m <= E - e) store_shared(&Cn[(size_t)lane * EP + e + m], best + tl.x);
          if (e < m) store_shared(&Cn[(size_t)lane * EP + e], INFINITY);
        }
      }
    } else {
    float cp[SP];
    if (l == 1) {
#pragma unroll
      for (int sp = 0; sp < SP; ++sp) {
        const bool col = (sp < SP - 3 || sp < S);
        const float cv = col ? c0[sp] : INFINITY;
        const int mv = col ? m0[sp] : 0;
        cp[sp] = (mv >= 0 && e0 >= mv && e0 <= E) ? cv : INFINITY;
      }
    } else {
#pragma unroll
      for (int sp = 0; sp < SP; ++sp) cp[sp] = cp_lds[sp * 64 + lane];
    }

#pragma unroll 1
    for (int s = s_begin; s < s_end; ++s) {
      float x[SP], cm[NC];
#pragma unroll
      for (int q = 0; q < SP / 4; ++q) {
        const float4 v = rt_lds[s * RQ + q];
        x[4 * q] = cp[4 * q] + v.x; x[4 * q + 1] = cp[4 * q + 1] + v.y;
        x[4 * q + 2] = cp[4 * q + 2] + v.z; x[4 * q + 3] = cp[4 * q + 3] + v.w;
      }
      const float4 tail = rt_lds[s * RQ + SP / 4];       // c(l,s), bits of M(l,s)
      // chunk minima of three candidates, then their minimum T: one add and half a min per candidate
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int lo = c * CH, len = ((c + 1) * CH < SP ? (c + 1) * CH : SP) - lo;
        cm[c] = len == 3 ? fmin3(x[lo], x[lo + 1], x[lo + 2]) : len == 2 ? __builtin_fminf(x[lo], x[lo + 1]) : x[lo];
      }
      float T = cm[0];
#pragma unroll
      for (int c = 1; c < NC; c += 2) T = (c + 1 < NC) ? fmin3(T, cm[c], cm[c + 1]) : __builtin_fminf(T, cm[c]);
      const float cs = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(tail.x)));
      const int m_raw = __builtin_amdgcn_readfirstlane(__float_as_int(tail.y));
      const int m = (m_raw < 0 || m_raw > E + 1) ? E + 1 : m_raw;
      float* Cs = Cn + (size_t)s * EP;
      const __amdgpu_buffer_rsrc_t bc = __builtin_amdgcn_make_buffer_rsrc(Cs, 0, (E + 1) * 4, kBufWord3);
      const __amdgpu_buffer_rsrc_t binf = __builtin_amdgcn_make_buffer_rsrc(Cs, 0, m * 4, kBufWord3);
      if (ARG) {
        // Lowest-index minimiser without a branch (a wave is nearly alone on its SIMD here, and a
        // taken branch costs it more than the selects): going down the chunks, the lowest chunk whose
        // minimum equals T leaves its index and its first two sums behind; the minimiser is the
        // first of the chunk's (at most three) sums that equals T.  Same sums, same bits.
        int cidx = NC - 1;
        float a0 = x[(NC - 1) * CH], a1 = ((NC - 1) * CH + 1 < SP) ? x[(NC - 1) * CH + 1] : INFINITY;
#pragma unroll
        for (int c = NC - 2; c >= 0; --c) {
          const bool eq = cm[c] == T;
          cidx = eq ? c : cidx;
          a0 = eq ? x[c * CH] : a0;
          a1 = eq ? x[c * CH + 1] : a1;
        }
        const int arg = cidx * CH + (a0 == T ? 0 : a1 == T ? 1 : 2);
        const __amdgpu_buffer_rsrc_t ba = __builtin_amdgcn_make_buffer_rsrc(An + (size_t)s * EP, 0, EP, kBufWord3);
        __builtin_amdgcn_raw_buffer_store_b8((unsigned char)arg, ba, e0, 0, 0);
      }
      __builtin_amdgcn_raw_buffer_store_b32((unsigned)__float_as_int(T + cs), bc, (e0 + m) * 4, 0, kDeviceScope);
      if (wbase < m) __builtin_amdgcn_raw_buffer_store_b32(0x7f800000u, binf, e0 * 4, 0, kDeviceScope);
    }

    }

    // ---- publish: this tile has finished layer l
    stores_done();
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(prog + tile, base + (unsigned)l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  // ---- best(e) = min_s C(L-1, e, s) for the tile's budgets, lowest index among equals
  if (Lb >= 2) {
    if (wave == 0) {
      const int lo = tile - (mprev + 63) / 64;
      const bool ok = wait_for(a, prog, lo < 0 ? 0 : lo, tile, base + (unsigned)(Lb - 1) + never, lane);
      if (lane == 0) go = ok ? 1 : 0;
    }
    __syncthreads();
    if (!go) return;
    loads_after();
  } else {
    __syncthreads();                                     // layer 0 was written by this workgroup
  }
  if (wave == 0 && e0 >= t.final_from && e0 <= E) {
    const float* __restrict__ C = c_table(t, inst, row0 + Lb - 1, Lb - 1);
    float b = INFINITY;
    int arg = 0;
    int s = 0;
    for (; s + 8 <= S; s += 8) {
      float v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = load_shared(&C[(size_t)(s + i) * EP + e0]);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (v[i] < b) { b = v[i]; arg = s + i; }
    }
    for (; s < S; ++s) {
      const float v = load_shared(&C[(size_t)s * EP + e0]);
      if (v < b) { b = v; arg = s; }
    }
    t.best[(size_t)inst * EP + e0] = b;
    t.best_s[(size_t)inst * EP + e0] = (uint8_t)arg;
  }
}

namespace {

template <int SP>
struct LayersKernel {
  static const void* get(int nw, bool arg) {
    if (nw == 8)
      return arg ? reinterpret_cast<const void*>(&k_layers<SP, 8, true>)
                 : reinterpret_cast<const void*>(&k_layers<SP, 8, false>);
    return arg ? reinterpret_cast<const void*>(&k_layers<SP, 4, true>)
               : reinterpret_cast<const void*>(&k_layers<SP, 4, false>);
  }
};

const void* layers_kernel(int SP, int nw, bool arg) {
  switch (SP) {
#define GBMW_CASE(N) case N: return LayersKernel<N>::get(nw, arg);
    GBMW_CASE(4) GBMW_CASE(8) GBMW_CASE(12) GBMW_CASE(16) GBMW_CASE(20) GBMW_CASE(24)
    GBMW_CASE(28) GBMW_CASE(32) GBMW_CASE(36) GBMW_CASE(40) GBMW_CASE(44) GBMW_CASE(48)
    GBMW_CASE(52) GBMW_CASE(56) GBMW_CASE(60) GBMW_CASE(64)
#undef GBMW_CASE
    default: return nullptr;
  }
}

size_t layers_lds_bytes(int S) {
  const int SP = (S + 3) / 4 * 4, RS = (SP + 2 + 3) / 4 * 4;
  return (size_t)SP * RS * sizeof(float) + (size_t)SP * 64 * sizeof(float);
}

}  // namespace

int layers_resident_workgroups(int S, int waves, bool records) {
  const int SP = (S + 3) / 4 * 4;
  const void* k = layers_kernel(SP, waves, records);
  if (!k || (waves != 4 && waves != 8)) return 0;
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k, 64 * waves, layers_lds_bytes(S)) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  return cus * per_cu;
}

hipError_t launch_layers(const Tables& t, const PersistArgs& a, int waves, bool cooperative, hipStream_t st) {
  const void* k = layers_kernel(t.SP, waves, t.A != nullptr);
  if (!k || (waves != 4 && waves != 8)) return hipErrorInvalidValue;
  Tables tt = t;
  PersistArgs aa = a;
  void* args[] = {&tt, &aa};
  // the cooperative launch API starts the kernel only when all its workgroups fit at once
  if (cooperative)
    return hipLaunchCooperativeKernel(k, dim3((unsigned)a.tiles * a.n_slots), dim3(64 * waves), args,
                                      (unsigned)layers_lds_bytes(t.S), st);
  return hipLaunchKernel(k, dim3((unsigned)a.tiles * a.n_slots), dim3(64 * waves), args, layers_lds_bytes(t.S), st);
}

}  // namespace gbmw
