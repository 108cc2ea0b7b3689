// Internal: the solver context and the small helpers shared by the C-ABI source
// files.  Not installed; not part of the ABI.
#pragma once
#include <hip/hip_runtime.h>

#include <vector>

#include "../../include/gbmw.h"
#include "gbmw_kernels.h"

namespace gbmw_detail {

// Records the message returned by gbmw_last_error() and hands back `st`.
gbmw_status fail(gbmw_status st, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

#define HIP_TRY(expr)                                                                        \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess) {                                                                  \
      (void)hipGetLastError();                                                               \
      return gbmw_detail::fail(e_ == hipErrorOutOfMemory ? GBMW_ERR_OOM : GBMW_ERR_DEVICE,   \
                               "%s: %s", #expr, hipGetErrorString(e_));                      \
    }                                                                                        \
  } while (0)

struct DevBuf {
  void* p = nullptr;
  size_t cap = 0;
  gbmw_status reserve(size_t bytes) {
    if (bytes <= cap) return GBMW_OK;
    if (p) { (void)hipFree(p); p = nullptr; cap = 0; }
    if (bytes == 0) return GBMW_OK;
    HIP_TRY(hipMalloc(&p, bytes));
    cap = bytes;
    return GBMW_OK;
  }
  void release() {
    if (p) (void)hipFree(p);
    p = nullptr;
    cap = 0;
  }
};

// gbmw_dp_solve_batched with one more knob: best / best_s are produced for budgets
// e >= final_from only (0: all of them; E: just the full budget).
gbmw_status solve_batched(const gbmw_problem* p, uint32_t flags, gbmw_ctx** ctx, int final_from);

// Helper streams (default priority) and fork / join events for G instance groups.
gbmw_status ensure_streams(gbmw_ctx* c, int G);

// A new, empty context on the current device.
gbmw_status new_ctx(gbmw_ctx** out);

// Waits for the context's stream and turns the device-side input checks into a status.
gbmw_status wait_and_check(gbmw_ctx* c);

}  // namespace gbmw_detail

struct gbmw_ctx {
  int device = 0;
  hipStream_t stream = nullptr;
  bool solved = false;
  bool index_on_device = false;   // d_L / d_off / d_perm hold this->L / off / perm
  uint32_t flags = 0;
  int B = 0, S = 0, SP = 0, E = 0, EP = 0, sumL = 0, Lmax = 0;
  std::vector<int> L, off, perm;
  std::vector<int> h_M;                      // host mirror of the solve's M (see h_M_valid)
  bool h_M_valid = false;                    // filled at the solve for host inputs, on first use else
  gbmw::Tables t{};
  gbmw_detail::DevBuf d_L, d_off, d_perm, d_c, d_M, d_R, d_Rt, d_C, d_sum, d_A, d_best, d_best_s, d_status,
      d_q, d_stage, d_search, d_gather, d_counts, d_sync, d_asum;
  hipEvent_t ev0 = nullptr, ev1 = nullptr, ev_fork = nullptr;
  std::vector<hipStream_t> aux;              // extra streams for instance groups
  std::vector<hipEvent_t> ev_join;
  std::vector<hipEvent_t> ev_layer;          // pairs around min-plus launches
  unsigned long long epoch = 0;              // of the last single-launch fill on this context
  unsigned long long single_epoch = 0;       // != 0: the solution came from a single-launch fill of that epoch
  int timed_launches = 0;
  int counted_launches = 0;
  std::vector<unsigned long long> counted_waves; // per counted launch: waves (64 budgets) inside the tables
};
