// Candidate strategies of one layer (Section 3.2: decision-tree rules, Takeaway #3)
// and the analytic cost model that turns layer shapes into the search's inputs
// (Section 5 for what the paper fixes).  See include/gbmw.h for the contract and for
// the model's formulas; the kernels below evaluate them in fp64 in exactly the
// order written there.
#include <algorithm>
#include <climits>
#include <cmath>
#include <vector>

#include "gbmw_ctx.h"

using gbmw_detail::fail;

namespace {

// ordered tuples of factors from {2, 4, 8, ...} with product g
void factorisations(int g, std::vector<int>& cur, std::vector<std::vector<int>>& out) {
  if (g == 1) {
    out.push_back(cur);
    return;
  }
  for (long long d = 2; d <= g; d *= 2) {
    if (g % d) continue;
    cur.push_back((int)d);
    factorisations(g / (int)d, cur, out);
    cur.pop_back();
  }
}

struct Derived {
  int dp = 1, sdp = 1, tp = 1, span_dp = 1, span_sdp = 1, span_tp = 1;
  int nkey = 0;
  int key[3] = {0, 0, 0};       // per level: degree, negated for TP levels
};

__host__ __device__ inline Derived derive(const gbmw_strategy& s) {
  Derived d;
  int inner = 1;
  for (int i = s.n_levels - 1; i >= 0; --i) {
    const int k = s.kind[i], g = s.degree[i];
    if (k == GBMW_DP) { d.dp = g; d.span_dp = g * inner; }
    else if (k == GBMW_SDP) { d.sdp = g; d.span_sdp = g * inner; }
    else { d.tp = g; d.span_tp = g * inner; }
    inner *= g;
  }
  d.nkey = s.n_levels;
  for (int i = 0; i < s.n_levels; ++i) d.key[i] = (s.kind[i] == GBMW_TP) ? -s.degree[i] : s.degree[i];
  return d;
}

__device__ inline double ov(double a, double b, double slow) {
  const double lo = a <= b ? a : b, hi = a <= b ? b : a;
  return slow * lo + (hi - lo);
}

__device__ inline int to_units(double x, double unit, int* status) {
  const double u = ceil(x / unit);
  if (!(u <= 2147483647.0)) {
    atomicOr(status, 1);
    return INT_MAX;
  }
  return (int)u;
}

// one lane per (layer, strategy)
__global__ __launch_bounds__(256) void k_cost_layers(const gbmw_layer_shape* __restrict__ layers, int L,
                                                     const gbmw_strategy* __restrict__ strat, int S,
                                                     gbmw_hardware hw, double Bm, int P,
                                                     float* __restrict__ c, float* __restrict__ c_ns,
                                                     int* __restrict__ Of, int* __restrict__ Ob,
                                                     int* __restrict__ Oms, int* __restrict__ M,
                                                     int* __restrict__ status) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= L * S) return;
  const int l = idx / S, s = idx % S;
  const gbmw_layer_shape ly = layers[l];
  const gbmw_strategy st = strat[s];
  const Derived d = derive(st);
  const double bw_tp = d.span_tp <= hw.island ? hw.bw_in : hw.bw_out;
  const double bw_sdp = d.span_sdp <= hw.island ? hw.bw_in : hw.bw_out;
  const double bw_dp = d.span_dp <= hw.island ? hw.bw_in : hw.bw_out;
  const double lb = Bm / (double)(d.dp * d.sdp);
  const double t_f = lb * ly.flops / (double)d.tp / hw.rate;
  const double t_b = 2.0 * t_f;
  const double tp_ar = d.tp > 1 ? 2.0 * (double)(d.tp - 1) / (double)d.tp * (lb * ly.bnd) / bw_tp : 0.0;
  const double pbytes = ly.params * hw.param_bytes / (double)d.tp;
  const double sdp_ag = d.sdp > 1 ? (double)(d.sdp - 1) / (double)d.sdp * pbytes / bw_sdp : 0.0;
  const double dp_ar = d.dp > 1 ? 2.0 * (double)(d.dp - 1) / (double)d.dp * pbytes / bw_dp : 0.0;
  const double fwd = t_f + tp_ar + sdp_ag;
  double bwd = t_b + tp_ar;
  if (st.ckpt) bwd = bwd + (t_f + tp_ar);
  const double sync = dp_ar + sdp_ag;
  const double cv = fwd + ov(bwd, sdp_ag + sync, hw.slow);
  const double cn = fwd + ov(bwd, sdp_ag, hw.slow);
  const double ms = ly.params * hw.state_bytes / (double)(d.tp * d.sdp);
  double act_f, act_b;
  if (st.ckpt) {
    act_f = lb * ly.bnd;
    act_b = lb * (ly.intm / (double)d.tp);
  } else {
    act_f = lb * (ly.bnd + ly.intm / (double)d.tp);
    act_b = 0.0;
  }
  const int of = to_units(act_f, hw.unit_bytes, status);
  const int ob = to_units(act_b, hw.unit_bytes, status);
  const int oms = to_units(ms, hw.unit_bytes, status);
  if (c) c[idx] = (float)cv;
  if (c_ns) c_ns[idx] = (float)cn;
  if (Of) Of[idx] = of;
  if (Ob) Ob[idx] = ob;
  if (Oms) Oms[idx] = oms;
  if (M) {
    for (int i = 0; i < P; ++i) {
      const long long m = (long long)oms + (long long)(P - i) * of;
      if (m > INT_MAX) atomicOr(status, 1);
      M[(size_t)i * L * S + idx] = m > INT_MAX ? INT_MAX : (int)m;
    }
  }
}

// one lane per (layer, previous strategy, strategy)
__global__ __launch_bounds__(256) void k_cost_transform(const gbmw_layer_shape* __restrict__ layers, int L,
                                                        const gbmw_strategy* __restrict__ strat, int S,
                                                        gbmw_hardware hw, double Bm, float* __restrict__ R) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t SS = (size_t)S * S;
  if (idx >= (size_t)L * SS) return;
  const int l = (int)(idx / SS), sp = (int)((idx % SS) / S), s = (int)(idx % S);
  float out = 0.0f;
  if (l > 0) {
    const Derived a = derive(strat[sp]), b = derive(strat[s]);
    bool same = a.nkey == b.nkey;
    for (int i = 0; i < 3; ++i) same = same && (a.key[i] == b.key[i]);
    if (!same) {
      const int b0 = a.dp * a.sdp, b1 = b.dp * b.sdp;
      const double share = b0 != b1 ? fabs(1.0 / (double)b1 - 1.0 / (double)b0) : 1.0 / (double)b1;
      out = (float)(Bm * layers[l - 1].bnd * share / hw.bw_out);
    }
  }
  R[idx] = out;
}

}  // namespace

extern "C" int32_t gbmw_enumerate_strategies(int32_t group_size, int32_t with_ckpt, int32_t takeaway3,
                                             gbmw_strategy* out, int32_t cap) {
  gbmw_detail::clear_error();
  if (group_size < 1 || group_size > (1 << 20) || (group_size & (group_size - 1))) {
    fail(GBMW_ERR_INVALID_ARG, "group_size=%d is not a power of two in 1..2^20", group_size);
    return -1;
  }
  std::vector<std::vector<int>> facts;
  std::vector<int> cur;
  factorisations(group_size, cur, facts);
  std::sort(facts.begin(), facts.end(), [](const std::vector<int>& a, const std::vector<int>& b) {
    return a.size() != b.size() ? a.size() < b.size() : a < b;
  });
  std::vector<gbmw_strategy> trees;
  for (const auto& degs : facts) {
    const int n = (int)degs.size();
    if (n > 3) continue;                                     // three paradigms: at most three levels
    int kinds[3] = {GBMW_DP, GBMW_SDP, GBMW_TP};
    // n-permutations of (DP, SDP, TP) in lexicographic order
    for (int a = 0; a < 3; ++a)
      for (int b = 0; b < 3; ++b)
        for (int c3 = 0; c3 < 3; ++c3) {
          if (n < 3 && c3 > 0) continue;
          if (n < 2 && b > 0) continue;
          if (n < 1 && a > 0) continue;
          if (n >= 2 && b == a) continue;
          if (n >= 3 && (c3 == a || c3 == b)) continue;
          const int pick[3] = {a, b, c3};
          bool has_dp = false, has_sdp = false;
          gbmw_strategy t{};
          t.n_levels = n;
          for (int i = 0; i < n; ++i) {
            t.kind[i] = kinds[pick[i]];
            t.degree[i] = degs[i];
            has_dp = has_dp || t.kind[i] == GBMW_DP;
            has_sdp = has_sdp || t.kind[i] == GBMW_SDP;
          }
          if (takeaway3 && has_dp && has_sdp) continue;
          trees.push_back(t);
        }
  }
  const size_t total = trees.size() * (with_ckpt ? 2 : 1);
  if (total > (size_t)INT_MAX) return -1;
  if (out) {
    size_t k = 0;
    for (int ck = 0; ck < (with_ckpt ? 2 : 1); ++ck)
      for (const gbmw_strategy& t : trees) {
        if (k >= (size_t)std::max(cap, 0)) break;
        out[k] = t;
        out[k].ckpt = ck;
        ++k;
      }
  }
  return (int32_t)total;
}

extern "C" gbmw_status gbmw_cost_model(const gbmw_layer_shape* layers, int32_t L,
                                       const gbmw_strategy* strategies, int32_t S,
                                       const gbmw_hardware* hw, double Bm, int32_t P, int32_t out_space,
                                       float* c, float* c_nosync, int32_t* O_f, int32_t* O_b,
                                       int32_t* O_ms, int32_t* M, float* R, void* stream) {
  gbmw_detail::clear_error();
  if (!layers || !strategies || !hw) return fail(GBMW_ERR_INVALID_ARG, "null layers / strategies / hw");
  if (L < 1 || L > (1 << 24)) return fail(GBMW_ERR_INVALID_ARG, "L=%d out of range", L);
  if (S < 1 || S > GBMW_MAX_S) return fail(GBMW_ERR_INVALID_ARG, "S=%d not in 1..256", S);
  if (P < 1 || P > 64) return fail(GBMW_ERR_INVALID_ARG, "P=%d not in 1..64", P);
  if (out_space != GBMW_PTR_HOST && out_space != GBMW_PTR_DEVICE)
    return fail(GBMW_ERR_INVALID_ARG, "out_space=%d", out_space);
  if (!(Bm > 0.0) || !std::isfinite(Bm)) return fail(GBMW_ERR_INVALID_ARG, "Bm must be positive");
  if (!(hw->rate > 0.0) || !(hw->bw_in > 0.0) || !(hw->bw_out > 0.0) || !(hw->unit_bytes > 0.0) ||
      !(hw->param_bytes >= 0.0) || !(hw->state_bytes >= 0.0) || !(hw->slow >= 1.0) || hw->island < 1)
    return fail(GBMW_ERR_INVALID_ARG, "hardware description out of range");
  for (int l = 0; l < L; ++l)
    if (!(layers[l].params >= 0.0) || !(layers[l].flops >= 0.0) || !(layers[l].bnd >= 0.0) ||
        !(layers[l].intm >= 0.0) || !std::isfinite(layers[l].params + layers[l].flops + layers[l].bnd + layers[l].intm))
      return fail(GBMW_ERR_INVALID_ARG, "layer %d has a negative or non-finite shape", l);
  for (int s = 0; s < S; ++s) {
    const gbmw_strategy& t = strategies[s];
    if (t.n_levels < 0 || t.n_levels > 3) return fail(GBMW_ERR_INVALID_ARG, "strategy %d: n_levels=%d", s, t.n_levels);
    long long prod = 1;
    for (int i = 0; i < t.n_levels; ++i) {
      if (t.kind[i] < GBMW_DP || t.kind[i] > GBMW_TP) return fail(GBMW_ERR_INVALID_ARG, "strategy %d: kind", s);
      if (t.degree[i] < 2 || (t.degree[i] & (t.degree[i] - 1))) return fail(GBMW_ERR_INVALID_ARG, "strategy %d: degree", s);
      for (int j = 0; j < i; ++j)
        if (t.kind[j] == t.kind[i]) return fail(GBMW_ERR_INVALID_ARG, "strategy %d repeats a paradigm", s);
      prod *= t.degree[i];
      if (prod > (1 << 20)) return fail(GBMW_ERR_INVALID_ARG, "strategy %d: group too large", s);
    }
  }

  hipStream_t st = (hipStream_t)stream;
  const bool host_out = out_space == GBMW_PTR_HOST;
  const size_t LS = (size_t)L * S, LSS = LS * S;
  // device block: layers | strategies | status | (host outputs only) c | c_ns | Of | Ob | Oms | M | R
  gbmw_detail::DevBuf buf;
  size_t bytes = sizeof(gbmw_layer_shape) * L + sizeof(gbmw_strategy) * S + 256;
  if (host_out) bytes += 4 * (5 * LS + (size_t)P * LS + LSS) + 256;
  gbmw_status rs = buf.reserve(bytes);
  if (rs != GBMW_OK) return rs;
  char* base = (char*)buf.p;
  gbmw_layer_shape* d_layers = (gbmw_layer_shape*)base;
  gbmw_strategy* d_strat = (gbmw_strategy*)(d_layers + L);
  int* d_status = (int*)(((uintptr_t)(d_strat + S) + 255) / 256 * 256);
  float* dc = c; float* dcn = c_nosync; int* dOf = O_f; int* dOb = O_b; int* dOms = O_ms; int* dM = M; float* dR = R;
  if (host_out) {
    float* w = (float*)(d_status + 64);
    dc = c ? w : nullptr; w += LS;
    dcn = c_nosync ? w : nullptr; w += LS;
    dOf = O_f ? (int*)w : nullptr; w += LS;
    dOb = O_b ? (int*)w : nullptr; w += LS;
    dOms = O_ms ? (int*)w : nullptr; w += LS;
    dM = M ? (int*)w : nullptr; w += (size_t)P * LS;
    dR = R ? w : nullptr;
  }
  auto done = [&](gbmw_status s2) {
    (void)hipStreamSynchronize(st);
    buf.release();
    return s2;
  };
#define HIP_TRY_D(expr)                                                                     \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) {                                                                 \
      (void)hipGetLastError();                                                              \
      return done(fail(GBMW_ERR_DEVICE, "%s: %s", #expr, hipGetErrorString(e_)));           \
    }                                                                                       \
  } while (0)
  const int zero = 0;
  HIP_TRY_D(hipMemcpyAsync(d_layers, layers, sizeof(gbmw_layer_shape) * L, hipMemcpyHostToDevice, st));
  HIP_TRY_D(hipMemcpyAsync(d_strat, strategies, sizeof(gbmw_strategy) * S, hipMemcpyHostToDevice, st));
  HIP_TRY_D(hipMemcpyAsync(d_status, &zero, sizeof(int), hipMemcpyHostToDevice, st));
  hipLaunchKernelGGL(k_cost_layers, dim3((unsigned)((LS + 255) / 256)), dim3(256), 0, st, d_layers, L, d_strat,
                     S, *hw, Bm, P, dc, dcn, dOf, dOb, dOms, dM, d_status);
  if (dR)
    hipLaunchKernelGGL(k_cost_transform, dim3((unsigned)((LSS + 255) / 256)), dim3(256), 0, st, d_layers, L,
                       d_strat, S, *hw, Bm, dR);
  HIP_TRY_D(hipGetLastError());
  int status = 0;
  HIP_TRY_D(hipMemcpyAsync(&status, d_status, sizeof(int), hipMemcpyDeviceToHost, st));
  if (host_out) {
    const hipMemcpyKind D2H = hipMemcpyDeviceToHost;
    if (c) HIP_TRY_D(hipMemcpyAsync(c, dc, 4 * LS, D2H, st));
    if (c_nosync) HIP_TRY_D(hipMemcpyAsync(c_nosync, dcn, 4 * LS, D2H, st));
    if (O_f) HIP_TRY_D(hipMemcpyAsync(O_f, dOf, 4 * LS, D2H, st));
    if (O_b) HIP_TRY_D(hipMemcpyAsync(O_b, dOb, 4 * LS, D2H, st));
    if (O_ms) HIP_TRY_D(hipMemcpyAsync(O_ms, dOms, 4 * LS, D2H, st));
    if (M) HIP_TRY_D(hipMemcpyAsync(M, dM, 4 * (size_t)P * LS, D2H, st));
    if (R) HIP_TRY_D(hipMemcpyAsync(R, dR, 4 * LSS, D2H, st));
  }
  HIP_TRY_D(hipStreamSynchronize(st));
#undef HIP_TRY_D
  buf.release();
  if (status) return fail(GBMW_ERR_INVALID_ARG, "a memory amount does not fit 32-bit units (unit_bytes too small)");
  return GBMW_OK;
}
