// C-ABI layer of the batched layer-wise strategy search: argument checking,
// device buffers, the per-layer launch sequence, result read-back.  See
// include/gbmw.h for the contract of every entry point.
#include "../../include/gbmw.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <numeric>
#include <vector>

#include "gbmw_ctx.h"
#include "gbmw_kernels.h"

// Staging block of gbmw_backtrack_static: queries in, plans out.  One copy per GPU, held
// until the process ends.  Host code never uses the array's name as an address: the device
// address is looked up once per device (static_scratch) and that pointer is what copies and
// kernels get.
static constexpr size_t kStaticScratchBytes = (size_t)GBMW_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

// Device address of `scratch` on device `dev`, which must be the current device.
static gbmw_status static_scratch(int dev, void** out) {
  if (dev < 0 || dev >= kMaxDevices)
    return gbmw_detail::fail(GBMW_ERR_UNSUPPORTED, "device %d: only devices 0..%d are supported", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return gbmw_detail::fail(GBMW_ERR_DEVICE, "hipGetSymbolAddress(scratch) on device %d: %s", dev,
                               hipGetErrorString(e));
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return GBMW_OK;
}

namespace {

thread_local char g_err[512] = "";

// Workgroups of the single-launch kernel that the current device holds at once, per (S, waves
// per tile, records): asked once per process and variant (one device type per process is assumed).
int resident_workgroups(int S, int waves, bool records) {
  static std::mutex mu;
  static int cache[GBMW_MAX_S + 1][2][2];
  static bool known[GBMW_MAX_S + 1][2][2];
  std::lock_guard<std::mutex> lock(mu);
  const int w = waves == 8 ? 1 : 0, r = records ? 1 : 0;
  if (!known[S][w][r]) {
    cache[S][w][r] = gbmw::layers_resident_workgroups(S, waves, records);
    known[S][w][r] = true;
  }
  return cache[S][w][r];
}

// Instance groups per solve (each on its own stream).  Two is where the gain
// from overlapping one group's ramp-down with the other's launch saturates.
constexpr int kGroups = 2;

}  // namespace

namespace gbmw_detail {

gbmw_status fail(gbmw_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

void clear_error() { g_err[0] = 0; }

}  // namespace gbmw_detail

using gbmw_detail::DevBuf;
using gbmw_detail::fail;
using gbmw_detail::wait_and_check;

namespace {

void free_ctx(gbmw_ctx* c) {
  if (!c) return;
  (void)hipSetDevice(c->device);
  (void)hipStreamSynchronize(c->stream);
  for (DevBuf* b : {&c->d_L, &c->d_off, &c->d_perm, &c->d_c, &c->d_M, &c->d_R, &c->d_Rt, &c->d_C, &c->d_sum,
                    &c->d_A, &c->d_best, &c->d_best_s, &c->d_status, &c->d_q, &c->d_stage,
                    &c->d_search, &c->d_gather, &c->d_counts, &c->d_sync, &c->d_asum})
    b->release();
  if (c->ev0) (void)hipEventDestroy(c->ev0);
  if (c->ev1) (void)hipEventDestroy(c->ev1);
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  for (hipEvent_t e : c->ev_join) (void)hipEventDestroy(e);
  for (hipStream_t a : c->aux) { (void)hipStreamSynchronize(a); (void)hipStreamDestroy(a); }
  for (hipEvent_t e : c->ev_layer) (void)hipEventDestroy(e);
  delete c;
}

gbmw_status check_host_values(const gbmw_problem* p, const std::vector<int>& L,
                              const std::vector<int>& off) {
  const int S = p->S;
  const size_t sumL = (size_t)off.back() + L.back();
  for (size_t i = 0; i < sumL * S; ++i) {
    if (!(p->c[i] >= 0.0f)) return fail(GBMW_ERR_INVALID_ARG, "c[%zu] is NaN or negative", i);
    if (p->M[i] < 0) return fail(GBMW_ERR_INVALID_ARG, "M[%zu] is negative", i);
  }
  for (int b = 0; b < p->B; ++b)
    for (size_t i = ((size_t)off[b] + 1) * S * S; i < ((size_t)off[b] + L[b]) * S * S; ++i)
      if (!(p->R[i] >= 0.0f)) return fail(GBMW_ERR_INVALID_ARG, "R[%zu] is NaN or negative", i);
  return GBMW_OK;
}

}  // namespace

namespace gbmw_detail {

gbmw_status ensure_streams(gbmw_ctx* c, int G) {
  while ((int)c->aux.size() < G - 1) {
    hipStream_t a;
    HIP_TRY(hipStreamCreateWithFlags(&a, hipStreamNonBlocking));   // default priority
    c->aux.push_back(a);
    hipEvent_t e;
    HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    c->ev_join.push_back(e);
  }
  if (G > 1 && !c->ev_fork) HIP_TRY(hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming));
  return GBMW_OK;
}

gbmw_status new_ctx(gbmw_ctx** out) {
  gbmw_ctx* c = new (std::nothrow) gbmw_ctx();
  if (!c) return fail(GBMW_ERR_OOM, "host allocation failed");
  if (hipGetDevice(&c->device) != hipSuccess) {
    delete c;
    return fail(GBMW_ERR_DEVICE, "no HIP device available");
  }
  *out = c;
  return GBMW_OK;
}

gbmw_status wait_and_check(gbmw_ctx* c) {
  if (!c) return fail(GBMW_ERR_INVALID_ARG, "null context");
  if (!c->solved) return fail(GBMW_ERR_INVALID_ARG, "context holds no solution");
  HIP_TRY(hipSetDevice(c->device));
  HIP_TRY(hipStreamSynchronize(c->stream));
  int status = 0;
  if (c->single_epoch != 0) {                              // the single-launch fill keeps epochs, not bits
    unsigned long long w[5];
    HIP_TRY(hipMemcpy(w, c->d_sync.p, sizeof(w), hipMemcpyDeviceToHost));
    if (w[gbmw::kSyncGaveUp] == c->single_epoch)
      return fail(GBMW_ERR_DEVICE, "the single-launch fill gave up waiting for a neighbouring tile (its workgroups "
                                   "were not all running at once, or the device was held by other work for seconds); "
                                   "the context holds no solution, solve again (GBMW_FLAG_LAYER_LAUNCHES avoids this path)");
    status = (w[gbmw::kSyncBadC] == c->single_epoch ? 1 : 0) | (w[gbmw::kSyncBadM] == c->single_epoch ? 2 : 0) |
             (w[gbmw::kSyncBadR] == c->single_epoch ? 4 : 0);
  } else {
    HIP_TRY(hipMemcpy(&status, c->d_status.p, sizeof(int), hipMemcpyDeviceToHost));
  }
  if (status)
    return fail(GBMW_ERR_INVALID_ARG, "device inputs rejected:%s%s%s",
                (status & 1) ? " c has NaN/negative values;" : "",
                (status & 2) ? " M has negative values;" : "",
                (status & 4) ? " R has NaN/negative values;" : "");
  return GBMW_OK;
}

}  // namespace gbmw_detail

extern "C" {

const char* gbmw_last_error(void) { return g_err; }

const char* gbmw_version(void) {
  return "gbmw 0.1 (gfx950; fused min-plus/argmin/shift-add; [s][e] tables)";
}

gbmw_status gbmw_dp_solve_batched(const gbmw_problem* p, uint32_t flags, gbmw_ctx** out) {
  g_err[0] = 0;
  return gbmw_detail::solve_batched(p, flags, out, 0);
}

}  // extern "C"

gbmw_status gbmw_detail::solve_batched(const gbmw_problem* p, uint32_t flags, gbmw_ctx** out,
                                       int final_from) {
  if (!p || !out) return fail(GBMW_ERR_INVALID_ARG, "null problem or context pointer");
  if (!p->L || !p->c || !p->M || !p->R) return fail(GBMW_ERR_INVALID_ARG, "null L/c/M/R");
  if (p->B < 1 || p->B > 65535) return fail(GBMW_ERR_INVALID_ARG, "B=%d not in 1..65535", p->B);
  if (p->S < 1 || p->S > GBMW_MAX_S) return fail(GBMW_ERR_INVALID_ARG, "S=%d not in 1..256", p->S);
  if (p->E < 0 || p->E > (1 << 28)) return fail(GBMW_ERR_INVALID_ARG, "E=%d out of range", p->E);
  if (p->ptr_space != GBMW_PTR_HOST && p->ptr_space != GBMW_PTR_DEVICE)
    return fail(GBMW_ERR_INVALID_ARG, "ptr_space=%d", p->ptr_space);
  if (flags & ~(uint32_t)(GBMW_FLAG_KEEP_ALL_C | GBMW_FLAG_TIME_KERNELS | GBMW_FLAG_ONE_STREAM |
                          GBMW_FLAG_LAZY_ARGMIN | GBMW_FLAG_DENSE_ARITHMETIC | GBMW_FLAG_COUNT_WORK |
                          GBMW_FLAG_LAYER_LAUNCHES | GBMW_FLAG_TEST_WAIT_GIVES_UP | GBMW_FLAG_COOPERATIVE_LAUNCH))
    return fail(GBMW_ERR_INVALID_ARG, "unknown flag bits 0x%x", flags);

  const int B = p->B, S = p->S, E = p->E;
  std::vector<int> L(p->L, p->L + B), off(B), perm(B);
  long long sum = 0;
  int Lmax = 0;
  for (int b = 0; b < B; ++b) {
    if (L[b] < 1) return fail(GBMW_ERR_INVALID_ARG, "L[%d]=%d < 1", b, L[b]);
    off[b] = (int)sum;
    sum += L[b];
    Lmax = std::max(Lmax, L[b]);
    if (sum > (1 << 24)) return fail(GBMW_ERR_INVALID_ARG, "sum of L too large");
  }
  const int sumL = (int)sum;
  if (p->ptr_space == GBMW_PTR_HOST) {
    gbmw_status st = check_host_values(p, L, off);
    if (st != GBMW_OK) return st;
  }
  std::iota(perm.begin(), perm.end(), 0);
  std::stable_sort(perm.begin(), perm.end(), [&](int a, int b) { return L[a] > L[b]; });
  // Instance groups: group g takes every G-th instance of the L-sorted order, so
  // groups are balanced and, inside a group, the instances still active at
  // layer l are a prefix.  Groups run on separate streams: layers of different
  // instances are independent, so one group's launch fills the ramp-down of
  // another's.
  const bool timed = (flags & GBMW_FLAG_TIME_KERNELS) != 0;
  const bool counting = (flags & GBMW_FLAG_COUNT_WORK) != 0;
  // A problem whose tiles of 64 budgets are all resident at once is filled by ONE launch in
  // which every tile walks the layers itself (gbmw_persistent.hip) instead of one launch per
  // layer: those launches would be bound by their own latency.
  const int tiles64 = (E + 64) / 64;
  int single_waves = 0;                                  // waves per tile of the single launch; 0: layer launches
  if (S <= 64 && Lmax < (1 << 19) && !timed && !counting && (flags & GBMW_FLAG_LAYER_LAUNCHES) == 0) {
    const bool records = (flags & GBMW_FLAG_LAZY_ARGMIN) == 0;
    // eight waves per tile where that fits (a wave then has an eighth of the strategies to itself)
    // (up to 44 strategies: beyond, a wave's registers do not allow two workgroups per compute unit)
    if (S >= 16 && S <= 44 && (long long)tiles64 * B <= (long long)resident_workgroups(S, 8, records)) single_waves = 8;
    else if ((long long)tiles64 * B <= (long long)resident_workgroups(S, 4, records)) single_waves = 4;
  }
  const bool single = single_waves != 0;
  if ((flags & GBMW_FLAG_TEST_WAIT_GIVES_UP) && !single)
    return fail(GBMW_ERR_INVALID_ARG, "GBMW_FLAG_TEST_WAIT_GIVES_UP needs a problem that takes the single-launch path");
  int G = (timed || counting || single || (flags & GBMW_FLAG_ONE_STREAM)) ? 1 : kGroups;
  if (G > B) G = B;
  std::vector<int> grouped, gfirst(G + 1, 0);
  for (int g = 0; g < G; ++g) {
    gfirst[g] = (int)grouped.size();
    for (int i = g; i < B; i += G) grouped.push_back(perm[i]);
  }
  gfirst[G] = B;
  perm = grouped;
  auto active_in_group = [&](int g, int l) {
    int n = 0;
    for (int i = gfirst[g]; i < gfirst[g + 1]; ++i) n += (L[perm[i]] > l) ? 1 : 0;
    return n;
  };

  gbmw_ctx* c = *out;
  const bool fresh = (c == nullptr);
  if (fresh) {
    gbmw_status st_new = gbmw_detail::new_ctx(&c);
    if (st_new != GBMW_OK) return st_new;
  }
  c->solved = false;

  auto bail = [&](gbmw_status st) {
    if (fresh) free_ctx(c);
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
  hipStream_t st = (hipStream_t)p->stream;
  c->stream = st;
  c->flags = flags;
  c->B = B; c->S = S; c->E = E; c->sumL = sumL; c->Lmax = Lmax;
  c->SP = (S + 3) / 4 * 4;
  c->EP = (E + 1 + 255) / 256 * 256;
  // a repeated solve of the same batch layout keeps the index arrays already on the device
  const bool same_layout = !fresh && c->index_on_device && c->L == L && c->off == off && c->perm == perm;
  c->L = L; c->off = off; c->perm = perm;
  const int SP = c->SP, EP = c->EP;
  const bool lazy = (flags & GBMW_FLAG_LAZY_ARGMIN) != 0;
  // The single launch keeps every layer's table where that is cheap (a small problem by
  // definition): with a rolling pair a tile also has to wait for the readers of the table it
  // overwrites, which ties the tiles to the slowest one.  What gbmw_export_tables hands out
  // still follows the flags.
  const bool keep = lazy || (flags & GBMW_FLAG_KEEP_ALL_C) != 0 ||
                    (single && sizeof(float) * (size_t)S * ((E + 1 + 255) / 256 * 256) * (size_t)sumL <= ((size_t)1 << 30));
  const size_t slab = (size_t)S * EP;

  TRY(c->d_L.reserve(sizeof(int) * B));
  TRY(c->d_off.reserve(sizeof(int) * B));
  TRY(c->d_perm.reserve(sizeof(int) * B));
  TRY(c->d_status.reserve(sizeof(int)));
  const int RS = (SP + 2 + 3) / 4 * 4;
  TRY(c->d_Rt.reserve(sizeof(float) * (size_t)sumL * S * RS));
  TRY(c->d_C.reserve(sizeof(float) * slab * (keep ? (size_t)sumL : (size_t)2 * B)));
  // the run shortcut and its summaries exist for the register-blocked kernels (S <= 64)
  const bool runs = (flags & GBMW_FLAG_DENSE_ARITHMETIC) == 0 && gbmw::layer0_in_registers(S) && !single;
  if (runs) TRY(c->d_sum.reserve(sizeof(float) * ((size_t)S * (EP / 64)) * (keep ? (size_t)sumL : (size_t)2 * B)));
  if (!lazy) TRY(c->d_A.reserve(slab * (size_t)sumL));
  // with both, one record per group of 64 budgets where the group's 64 are equal (Tables::Asum)
  if (!lazy && runs) TRY(c->d_asum.reserve((size_t)S * (EP / 64) * (size_t)sumL));
  TRY(c->d_best.reserve(sizeof(float) * (size_t)B * EP));
  TRY(c->d_best_s.reserve((size_t)B * EP));
  if (single) {
    // the synchronisation words of the single launch; new memory starts at zero, and since epochs
    // only grow nothing is ever cleared again
    const size_t words = (size_t)gbmw::kSyncHeader + (size_t)sumL + (size_t)B * tiles64;
    const size_t before = c->d_sync.cap;
    TRY(c->d_sync.reserve(words * sizeof(unsigned long long)));
    if (c->d_sync.cap != before) HIP_TRY_B(hipMemsetAsync(c->d_sync.p, 0, c->d_sync.cap, (hipStream_t)p->stream));
  }
  if (!c->ev0) {
    HIP_TRY_B(hipEventCreate(&c->ev0));
    HIP_TRY_B(hipEventCreate(&c->ev1));
  }

  // c and M always end up in arrays the context owns (the walkers, the export and the later
  // entry points read them long after this call): uploaded here for host inputs, copied by the
  // prepare kernel for device inputs.  R is only read by the prepare kernel.
  TRY(c->d_c.reserve(sizeof(float) * (size_t)sumL * S));
  TRY(c->d_M.reserve(sizeof(int) * (size_t)sumL * S));
  const float *src_c, *dR;
  const int* src_M;
  if (p->ptr_space == GBMW_PTR_HOST) {
    TRY(c->d_R.reserve(sizeof(float) * (size_t)sumL * S * S));
    HIP_TRY_B(hipMemcpyAsync(c->d_c.p, p->c, sizeof(float) * (size_t)sumL * S, hipMemcpyHostToDevice, st));
    HIP_TRY_B(hipMemcpyAsync(c->d_M.p, p->M, sizeof(int) * (size_t)sumL * S, hipMemcpyHostToDevice, st));
    HIP_TRY_B(hipMemcpyAsync(c->d_R.p, p->R, sizeof(float) * (size_t)sumL * S * S, hipMemcpyHostToDevice, st));
    src_c = (const float*)c->d_c.p; src_M = (const int*)c->d_M.p; dR = (const float*)c->d_R.p;
    c->h_M.assign(p->M, p->M + (size_t)sumL * S);
    c->h_M_valid = true;
  } else {
    src_c = p->c; src_M = p->M; dR = p->R;
    c->h_M_valid = false;
  }
  const float* dc = (const float*)c->d_c.p;
  const int* dM = (const int*)c->d_M.p;
  // The small index arrays come from host vectors owned by the context, which
  // outlive the copies.
  if (!same_layout) {
    c->index_on_device = false;
    HIP_TRY_B(hipMemcpyAsync(c->d_L.p, c->L.data(), sizeof(int) * B, hipMemcpyHostToDevice, st));
    HIP_TRY_B(hipMemcpyAsync(c->d_off.p, c->off.data(), sizeof(int) * B, hipMemcpyHostToDevice, st));
    HIP_TRY_B(hipMemcpyAsync(c->d_perm.p, c->perm.data(), sizeof(int) * B, hipMemcpyHostToDevice, st));
    c->index_on_device = true;
  }

  gbmw::Tables& t = c->t;
  t.B = B; t.S = S; t.SP = SP; t.RS = RS; t.E = E; t.EP = EP; t.keep_all = keep ? 1 : 0;
  t.final_from = std::min(std::max(final_from, 0), E);
  t.runs = runs ? 1 : 0;
  t.Tsum = runs ? (float*)c->d_sum.p : nullptr;
  t.L = (const int*)c->d_L.p; t.off = (const int*)c->d_off.p; t.perm = (const int*)c->d_perm.p;
  t.c = dc; t.M = dM; t.Rt = (const float*)c->d_Rt.p;
  t.Cbuf = (float*)c->d_C.p; t.A = lazy ? nullptr : (uint8_t*)c->d_A.p;
  t.Asum = (!lazy && runs) ? (uint8_t*)c->d_asum.p : nullptr;
  t.best = (float*)c->d_best.p; t.best_s = (uint8_t*)c->d_best_s.p;
  t.status = (int*)c->d_status.p;
  t.prev_full = 0;

  c->timed_launches = 0;
  c->counted_launches = 0;
  c->counted_waves.clear();
  t.counts = nullptr;
  if (counting) TRY(c->d_counts.reserve(sizeof(unsigned long long) * 4 * (size_t)Lmax));
  if (timed) {
    while ((int)c->ev_layer.size() < 2 * Lmax) {
      hipEvent_t e;
      HIP_TRY_B(hipEventCreate(&e));
      c->ev_layer.push_back(e);
    }
  }

  TRY(gbmw_detail::ensure_streams(c, G));

  if (counting) gbmw::launch_clear_counts((unsigned long long*)c->d_counts.p, 4 * Lmax, st);
  c->single_epoch = 0;
  if (single) {
    gbmw::PersistArgs a{};
    a.sync = (unsigned long long*)c->d_sync.p;
    a.epoch = ++c->epoch;
    a.src_c = src_c; a.src_M = src_M; a.R = dR;
    const bool give_up = (flags & GBMW_FLAG_TEST_WAIT_GIVES_UP) != 0;
    a.wait_ticks = give_up ? 100000 : 200000000;         // 1 ms : 2 s at 100 MHz
    a.wait_polls = give_up ? 2000 : 4000000;
    a.sumL = sumL; a.validate = p->ptr_space == GBMW_PTR_DEVICE ? 1 : 0;
    a.tiles = tiles64; a.n_slots = B; a.first = 0;
    a.extra_wait = give_up ? 1 : 0;
    HIP_TRY_B(hipEventRecord(c->ev0, st));
    HIP_TRY_B(gbmw::launch_layers(t, a, single_waves, (flags & GBMW_FLAG_COOPERATIVE_LAUNCH) != 0, st));
    HIP_TRY_B(hipEventRecord(c->ev1, st));
    HIP_TRY_B(hipGetLastError());
    c->single_epoch = a.epoch;
    c->solved = true;
    *out = c;
    return GBMW_OK;
  }
  HIP_TRY_B(hipEventRecord(c->ev0, st));
  gbmw::launch_prepare(t, dR, src_c, src_M, sumL, p->ptr_space == GBMW_PTR_DEVICE, st);
  {
    // Layer 0 goes to memory only where something reads it from there.  Inside a
    // group the instances are ordered by L descending, so the short ones are a suffix.
    const bool all = keep || !gbmw::layer0_in_registers(S);
    if (all) {
      gbmw::launch_init_layer0(t, 0, B, st);
    } else {
      for (int g = 0; g < G; ++g) {
        int n_short = 0;
        for (int i = gfirst[g + 1] - 1; i >= gfirst[g] && L[perm[i]] <= 2; --i) ++n_short;
        gbmw::launch_init_layer0(t, gfirst[g + 1] - n_short, n_short, st);
      }
    }
  }
  if (G > 1) HIP_TRY_B(hipEventRecord(c->ev_fork, st));
  for (int g = 0; g < G; ++g) {
    hipStream_t sg = (g == 0) ? st : c->aux[g - 1];
    if (g > 0) HIP_TRY_B(hipStreamWaitEvent(sg, c->ev_fork, 0));
    for (int l = 1; l < Lmax; ++l) {
      const int na = active_in_group(g, l);
      if (na == 0) break;
      if (timed) HIP_TRY_B(hipEventRecord(c->ev_layer[2 * c->timed_launches], sg));
      if (counting) {
        t.counts = (unsigned long long*)c->d_counts.p + 4 * (size_t)c->counted_launches++;
        c->counted_waves.push_back((unsigned long long)na * (unsigned long long)((E + 64) / 64));
      }
      gbmw::launch_minplus(t, l, gfirst[g], na, sg, l > 1 ? active_in_group(g, l - 1) : 0);
      if (timed) {
        HIP_TRY_B(hipEventRecord(c->ev_layer[2 * c->timed_launches + 1], sg));
        ++c->timed_launches;
      }
    }
    gbmw::launch_final(t, gfirst[g], gfirst[g + 1] - gfirst[g], sg);
    if (g > 0) {
      HIP_TRY_B(hipEventRecord(c->ev_join[g - 1], sg));
      HIP_TRY_B(hipStreamWaitEvent(st, c->ev_join[g - 1], 0));
    }
  }
  t.counts = nullptr;
  HIP_TRY_B(hipEventRecord(c->ev1, st));
  HIP_TRY_B(hipGetLastError());
#undef TRY
#undef HIP_TRY_B
  c->solved = true;
  *out = c;
  return GBMW_OK;
}

extern "C" {

gbmw_status gbmw_synchronize(gbmw_ctx* ctx) {
  g_err[0] = 0;
  return wait_and_check(ctx);
}

int32_t gbmw_max_layers(const gbmw_ctx* ctx) { return (ctx && ctx->solved) ? ctx->Lmax : 0; }

gbmw_status gbmw_get_best(gbmw_ctx* c, float* best, uint8_t* best_s) {
  g_err[0] = 0;
  gbmw_status st = wait_and_check(c);
  if (st != GBMW_OK) return st;
  const size_t w = (size_t)c->E + 1;
  if (best)
    HIP_TRY(hipMemcpy2D(best, w * sizeof(float), c->d_best.p, (size_t)c->EP * sizeof(float),
                        w * sizeof(float), c->B, hipMemcpyDeviceToHost));
  if (best_s)
    HIP_TRY(hipMemcpy2D(best_s, w, c->d_best_s.p, (size_t)c->EP, w, c->B, hipMemcpyDeviceToHost));
  return GBMW_OK;
}

}  // extern "C"

namespace {

// Shared by gbmw_backtrack and gbmw_backtrack_static: `block` is device memory of at least
// backtrack_block_bytes(nq, Lmax) bytes, laid out q_inst | q_e | cost | mem | plan.
size_t backtrack_block_bytes(size_t nq, size_t Lmax) { return nq * (4 * sizeof(int)) + nq * Lmax; }

gbmw_status check_queries(const gbmw_ctx* c, int32_t nq, const int32_t* q_instance, const int32_t* q_e,
                          const uint8_t* plan, const float* cost, const int32_t* mem_used) {
  if (!q_instance || !q_e || !plan || !cost || !mem_used)
    return fail(GBMW_ERR_INVALID_ARG, "null query or output pointer");
  for (int i = 0; i < nq; ++i) {
    if (q_instance[i] < 0 || q_instance[i] >= c->B)
      return fail(GBMW_ERR_INVALID_ARG, "q_instance[%d]=%d not in 0..%d", i, q_instance[i], c->B - 1);
    if (q_e[i] < 0 || q_e[i] > c->E)
      return fail(GBMW_ERR_INVALID_ARG, "q_e[%d]=%d not in 0..%d", i, q_e[i], c->E);
  }
  return GBMW_OK;
}

gbmw_status backtrack_in_block(gbmw_ctx* c, void* block, int32_t nq, const int32_t* q_instance,
                               const int32_t* q_e, uint8_t* plan, float* cost, int32_t* mem_used) {
  const size_t n = (size_t)nq, Lm = (size_t)c->Lmax;
  int* d_qi = (int*)block;
  int* d_qe = d_qi + n;
  float* d_cost = (float*)(d_qe + n);
  int* d_mem = (int*)(d_cost + n);
  uint8_t* d_plan = (uint8_t*)(d_mem + n);
  HIP_TRY(hipMemcpyAsync(d_qi, q_instance, n * sizeof(int), hipMemcpyHostToDevice, c->stream));
  HIP_TRY(hipMemcpyAsync(d_qe, q_e, n * sizeof(int), hipMemcpyHostToDevice, c->stream));
  gbmw::launch_backtrack(c->t, nq, d_qi, d_qe, c->Lmax, d_plan, d_cost, d_mem, c->stream);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipMemcpyAsync(cost, d_cost, n * sizeof(float), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipMemcpyAsync(mem_used, d_mem, n * sizeof(int), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipMemcpyAsync(plan, d_plan, n * Lm, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));
  return GBMW_OK;
}

}  // namespace

extern "C" {

gbmw_status gbmw_backtrack(gbmw_ctx* c, int32_t nq, const int32_t* q_instance, const int32_t* q_e,
                           uint8_t* plan, float* cost, int32_t* mem_used) {
  g_err[0] = 0;
  gbmw_status st = wait_and_check(c);
  if (st != GBMW_OK) return st;
  if (nq < 0) return fail(GBMW_ERR_INVALID_ARG, "nq=%d", nq);
  if (nq == 0) return GBMW_OK;
  st = check_queries(c, nq, q_instance, q_e, plan, cost, mem_used);
  if (st != GBMW_OK) return st;
  st = c->d_q.reserve(backtrack_block_bytes((size_t)nq, (size_t)c->Lmax));
  if (st != GBMW_OK) return st;
  return backtrack_in_block(c, c->d_q.p, nq, q_instance, q_e, plan, cost, mem_used);
}

gbmw_status gbmw_backtrack_static(gbmw_ctx* c, int32_t nq, const int32_t* q_instance, const int32_t* q_e,
                                  uint8_t* plan, float* cost, int32_t* mem_used) {
  g_err[0] = 0;
  gbmw_status st = wait_and_check(c);                    // makes the context's device current
  if (st != GBMW_OK) return st;
  if (nq < 0) return fail(GBMW_ERR_INVALID_ARG, "nq=%d", nq);
  if (nq == 0) return GBMW_OK;
  st = check_queries(c, nq, q_instance, q_e, plan, cost, mem_used);
  if (st != GBMW_OK) return st;
  const size_t need = backtrack_block_bytes((size_t)nq, (size_t)c->Lmax);
  if (need > kStaticScratchBytes)
    return fail(GBMW_ERR_UNSUPPORTED,
                "gbmw_backtrack_static: %d queries of %d layers need %zu bytes of staging, the static block "
                "holds %zu (at most %zu queries at this depth)",
                nq, c->Lmax, need, kStaticScratchBytes, kStaticScratchBytes / (16 + (size_t)c->Lmax));
  void* block = nullptr;
  st = static_scratch(c->device, &block);
  if (st != GBMW_OK) return st;
  return backtrack_in_block(c, block, nq, q_instance, q_e, plan, cost, mem_used);
}

gbmw_status gbmw_select_forward_budget(gbmw_ctx* c, const int32_t* O_f, const int32_t* O_b,
                                       const int32_t* O_ms, int32_t* e_opt, float* cost,
                                       uint8_t* plan, int32_t* e_all) {
  g_err[0] = 0;
  gbmw_status st = wait_and_check(c);
  if (st != GBMW_OK) return st;
  if (!O_f || !O_b || !O_ms) return fail(GBMW_ERR_INVALID_ARG, "null O_f/O_b/O_ms");
  const size_t n = (size_t)c->sumL * c->S, B = (size_t)c->B, Lm = (size_t)c->Lmax;
  // O_f + O_ms must be the M the tables were filled with
  if (!c->h_M_valid) {                    // device-resident inputs: fetched once per solve
    c->h_M.resize(n);
    HIP_TRY(hipMemcpy(c->h_M.data(), c->t.M, n * sizeof(int), hipMemcpyDeviceToHost));
    c->h_M_valid = true;
  }
  const std::vector<int>& M = c->h_M;
  for (size_t i = 0; i < n; ++i) {
    if (O_f[i] < 0 || O_b[i] < 0 || O_ms[i] < 0)
      return fail(GBMW_ERR_INVALID_ARG, "negative O_f/O_b/O_ms at %zu", i);
    if ((long long)O_f[i] + O_ms[i] != M[i])
      return fail(GBMW_ERR_INVALID_ARG, "O_f + O_ms differs from the solve's M at %zu", i);
  }
  std::vector<int> bup(B, 0);
  int max_window = 0;
  for (size_t b = 0; b < B; ++b) {
    const size_t lo = (size_t)c->off[b] * c->S, hi = lo + (size_t)c->L[b] * c->S;
    for (size_t i = lo; i < hi; ++i) bup[b] = std::max(bup[b], O_b[i]);
    max_window = std::max(max_window, std::min(bup[b], c->E + 1));
  }
  // one device block: Of | Ob | Oms | bup | first_bad | e_opt | e_all | cost | plan
  const size_t bytes = (3 * n + 4 * B) * sizeof(int) + B * sizeof(float) + B * Lm;
  st = c->d_q.reserve(bytes);
  if (st != GBMW_OK) return st;
  int* d_of = (int*)c->d_q.p;
  int* d_ob = d_of + n;
  int* d_oms = d_ob + n;
  int* d_bup = d_oms + n;
  int* d_fb = d_bup + B;
  int* d_eopt = d_fb + B;
  int* d_eall = d_eopt + B;
  float* d_cost = (float*)(d_eall + B);
  uint8_t* d_plan = (uint8_t*)(d_cost + B);
  hipStream_t s = c->stream;
  HIP_TRY(hipMemcpyAsync(d_of, O_f, n * sizeof(int), hipMemcpyHostToDevice, s));
  HIP_TRY(hipMemcpyAsync(d_ob, O_b, n * sizeof(int), hipMemcpyHostToDevice, s));
  HIP_TRY(hipMemcpyAsync(d_oms, O_ms, n * sizeof(int), hipMemcpyHostToDevice, s));
  HIP_TRY(hipMemcpyAsync(d_bup, bup.data(), B * sizeof(int), hipMemcpyHostToDevice, s));
  gbmw::launch_select(c->t, d_of, d_ob, d_oms, d_bup, max_window, c->Lmax, d_fb, d_eopt, d_cost,
                      d_plan, d_eall, s);
  HIP_TRY(hipGetLastError());
  if (e_opt) HIP_TRY(hipMemcpyAsync(e_opt, d_eopt, B * sizeof(int), hipMemcpyDeviceToHost, s));
  if (e_all) HIP_TRY(hipMemcpyAsync(e_all, d_eall, B * sizeof(int), hipMemcpyDeviceToHost, s));
  if (cost) HIP_TRY(hipMemcpyAsync(cost, d_cost, B * sizeof(float), hipMemcpyDeviceToHost, s));
  if (plan) HIP_TRY(hipMemcpyAsync(plan, d_plan, B * Lm, hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));     // also keeps the host vector bup alive long enough
  return GBMW_OK;
}

gbmw_status gbmw_pipeline_cost(gbmw_ctx* c, int32_t n_pipe, const int32_t* stage_begin,
                               const int32_t* stage_instance, const int32_t* stage_e,
                               const int32_t* microbatches, const float* c_nosync, float* cost,
                               float* stage_cost, float* stage_cost_nosync) {
  g_err[0] = 0;
  gbmw_status st = wait_and_check(c);
  if (st != GBMW_OK) return st;
  if (n_pipe < 0) return fail(GBMW_ERR_INVALID_ARG, "n_pipe=%d", n_pipe);
  if (n_pipe == 0) return GBMW_OK;
  if (!stage_begin || !stage_instance || !stage_e || !microbatches || !cost)
    return fail(GBMW_ERR_INVALID_ARG, "null argument");
  if (stage_begin[0] != 0) return fail(GBMW_ERR_INVALID_ARG, "stage_begin[0] must be 0");
  for (int p = 0; p < n_pipe; ++p) {
    if (stage_begin[p + 1] <= stage_begin[p])
      return fail(GBMW_ERR_INVALID_ARG, "pipeline %d has no stage", p);
    if (microbatches[p] < 1) return fail(GBMW_ERR_INVALID_ARG, "microbatches[%d]=%d", p, microbatches[p]);
  }
  const size_t ns = (size_t)stage_begin[n_pipe], np_ = (size_t)n_pipe, Lm = (size_t)c->Lmax;
  for (size_t i = 0; i < ns; ++i) {
    if (stage_instance[i] < 0 || stage_instance[i] >= c->B)
      return fail(GBMW_ERR_INVALID_ARG, "stage_instance[%zu]=%d", i, stage_instance[i]);
    if (stage_e[i] < -1 || stage_e[i] > c->E)
      return fail(GBMW_ERR_INVALID_ARG, "stage_e[%zu]=%d not in -1..%d", i, stage_e[i], c->E);
  }
  const size_t ncs = c_nosync ? (size_t)c->sumL * c->S : 0;
  for (size_t i = 0; i < ncs; ++i)
    if (!(c_nosync[i] >= 0.0f)) return fail(GBMW_ERR_INVALID_ARG, "c_nosync[%zu] is NaN or negative", i);
  // one device block: begin | mb | inst | e | C | Cns | cost | c_nosync | plan scratch
  const size_t bytes = (np_ + 1 + np_ + 2 * ns) * sizeof(int) + (2 * ns + np_ + ncs) * sizeof(float) + ns * Lm;
  st = c->d_q.reserve(bytes);
  if (st != GBMW_OK) return st;
  int* d_begin = (int*)c->d_q.p;
  int* d_mb = d_begin + np_ + 1;
  int* d_inst = d_mb + np_;
  int* d_e = d_inst + ns;
  float* d_C = (float*)(d_e + ns);
  float* d_Cns = d_C + ns;
  float* d_cost = d_Cns + ns;
  float* d_cns = d_cost + np_;
  uint8_t* d_plan = (uint8_t*)(d_cns + ncs);
  hipStream_t s = c->stream;
  HIP_TRY(hipMemcpyAsync(d_begin, stage_begin, (np_ + 1) * sizeof(int), hipMemcpyHostToDevice, s));
  HIP_TRY(hipMemcpyAsync(d_mb, microbatches, np_ * sizeof(int), hipMemcpyHostToDevice, s));
  HIP_TRY(hipMemcpyAsync(d_inst, stage_instance, ns * sizeof(int), hipMemcpyHostToDevice, s));
  HIP_TRY(hipMemcpyAsync(d_e, stage_e, ns * sizeof(int), hipMemcpyHostToDevice, s));
  if (ncs) HIP_TRY(hipMemcpyAsync(d_cns, c_nosync, ncs * sizeof(float), hipMemcpyHostToDevice, s));
  gbmw::launch_pipeline_cost(c->t, (int)ns, d_inst, d_e, ncs ? d_cns : nullptr, d_plan, c->Lmax, d_C,
                             d_Cns, n_pipe, d_begin, d_mb, d_cost, s);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipMemcpyAsync(cost, d_cost, np_ * sizeof(float), hipMemcpyDeviceToHost, s));
  if (stage_cost) HIP_TRY(hipMemcpyAsync(stage_cost, d_C, ns * sizeof(float), hipMemcpyDeviceToHost, s));
  if (stage_cost_nosync)
    HIP_TRY(hipMemcpyAsync(stage_cost_nosync, d_Cns, ns * sizeof(float), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  return GBMW_OK;
}

gbmw_status gbmw_export_tables(gbmw_ctx* c, int32_t inst, int32_t l0, int32_t l1, float* C,
                               uint8_t* A) {
  g_err[0] = 0;
  gbmw_status st = wait_and_check(c);
  if (st != GBMW_OK) return st;
  if (inst < 0 || inst >= c->B) return fail(GBMW_ERR_INVALID_ARG, "instance=%d", inst);
  const int Lb = c->L[inst];
  if (l0 < 0 || l1 > Lb || l0 > l1) return fail(GBMW_ERR_INVALID_ARG, "layers [%d,%d) of %d", l0, l1, Lb);
  if (l0 == l1) return GBMW_OK;
  const bool lazy = (c->flags & GBMW_FLAG_LAZY_ARGMIN) != 0;
  const bool keep = lazy || (c->flags & GBMW_FLAG_KEEP_ALL_C) != 0;
  if (C && !keep && l0 < Lb - 2)
    return fail(GBMW_ERR_UNSUPPORTED, "only the last two layers of C were kept (asked for layer %d of %d)", l0, Lb);
  const size_t rows = (size_t)c->E + 1, S = (size_t)c->S, slab = S * c->EP;
  const int row0 = c->off[inst];
  // one layer at a time through a staging buffer of [E+1][S] floats
  st = c->d_stage.reserve(rows * S * sizeof(float));
  if (st != GBMW_OK) return st;
  for (int l = l0; l < l1; ++l) {
    if (C) {
      const size_t tab = c->t.keep_all ? (size_t)(row0 + l) : (size_t)(l & 1) * c->B + inst;   // as c_table / sum_table
      const float* src = (const float*)c->d_C.p + tab * slab;
      const float* sum = c->t.Tsum ? c->t.Tsum + tab * (S * (c->EP >> 6)) : nullptr;
      gbmw::launch_export_c(c->t, src, sum, c->t.M + (size_t)(row0 + l) * S, (float*)c->d_stage.p, c->stream);
      HIP_TRY(hipGetLastError());
      HIP_TRY(hipMemcpyAsync(C + (size_t)(l - l0) * rows * S, c->d_stage.p, rows * S * sizeof(float),
                             hipMemcpyDeviceToHost, c->stream));
      HIP_TRY(hipStreamSynchronize(c->stream));
    }
    if (A) {
      uint8_t* dst = A + (size_t)(l - l0) * rows * S;
      if (l == 0) {
        memset(dst, 0, rows * S);
      } else {
        const uint8_t* src = (const uint8_t*)c->d_A.p + (size_t)(row0 + l) * slab;
        if (lazy || c->t.Asum) {                         // the records of this row, recomputed or put together
          st = c->d_q.reserve(slab);
          if (st != GBMW_OK) return st;
          gbmw::launch_argmin_row(c->t, row0 + l, (uint8_t*)c->d_q.p, c->stream);
          src = (const uint8_t*)c->d_q.p;
        }
        gbmw::launch_export_u8(src, (uint8_t*)c->d_stage.p, 1, c->S, c->E, c->EP, c->stream);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipMemcpyAsync(dst, c->d_stage.p, rows * S, hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(hipStreamSynchronize(c->stream));
      }
    }
  }
  return GBMW_OK;
}

gbmw_status gbmw_last_solve_ms(gbmw_ctx* c, float* total_ms, float* minplus_ms,
                               int32_t* minplus_launches) {
  g_err[0] = 0;
  gbmw_status st = wait_and_check(c);
  if (st != GBMW_OK) return st;
  if (total_ms) HIP_TRY(hipEventElapsedTime(total_ms, c->ev0, c->ev1));
  float sum = 0.0f;
  for (int i = 0; i < c->timed_launches; ++i) {
    float ms = 0.0f;
    HIP_TRY(hipEventElapsedTime(&ms, c->ev_layer[2 * i], c->ev_layer[2 * i + 1]));
    sum += ms;
  }
  if (minplus_ms) *minplus_ms = sum;
  if (minplus_launches) *minplus_launches = c->timed_launches;
  return GBMW_OK;
}

gbmw_status gbmw_last_solve_work(gbmw_ctx* c, int32_t launch, uint64_t work[4]) {
  g_err[0] = 0;
  gbmw_status st = wait_and_check(c);
  if (st != GBMW_OK) return st;
  if (!work) return fail(GBMW_ERR_INVALID_ARG, "null output pointer");
  work[0] = work[1] = work[2] = work[3] = 0;
  if (c->counted_launches == 0) return GBMW_OK;
  if (launch < -1 || launch >= c->counted_launches)
    return fail(GBMW_ERR_INVALID_ARG, "launch=%d not in -1..%d", launch, c->counted_launches - 1);
  std::vector<unsigned long long> h(4 * (size_t)c->counted_launches);
  HIP_TRY(hipMemcpy(h.data(), c->d_counts.p, h.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
  unsigned long long waves = 0, covered = 0;
  for (int i = 0; i < c->counted_launches; ++i) {
    if (launch >= 0 && i != launch) continue;
    work[0] += h[4 * i]; work[1] += h[4 * i + 1]; work[2] += h[4 * i + 2];
    covered += h[4 * i + 1] + h[4 * i + 2] + h[4 * i + 3];
    waves += c->counted_waves[i];
  }
  work[3] = (waves - covered) * (uint64_t)c->S;
  return GBMW_OK;
}

void gbmw_destroy(gbmw_ctx* ctx) { free_ctx(ctx); }

}  // extern "C"
