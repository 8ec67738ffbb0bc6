// Layer budgets B_l = e_l / sum(e) * total (Alg. 2, inner loop) as integers.
//
// The paper gives the real-valued rule only; the integer rule implemented here is: floor the
// quotas, hand the leftover units to the largest fractional parts (lower layer first on ties),
// pin layers that violate a bound and split the rest again.  The host path (on_device == 0) runs
// the sequential routine; the device runs the same arithmetic spread over one wavefront per
// sequence, so both paths return identical integers.
#include <math.h>

#include <vector>

#include "budget_wave.h"
#include "common.h"

namespace lava {

// One sequence.  Returns 0, or 1 when the bounds are infeasible.
// Scratch arrays (length n each): quota, base, freelist, frac.
__host__ __device__ inline int allocate_budgets(int n, const float* e, long long total,
                                                const long long* lo, const long long* hi,
                                                long long* out, double* quota, long long* base,
                                                int* freel, double* frac) {
#pragma clang fp contract(off)  // host and device must round every quota identically
  long long slo = 0, shi = 0;
  for (int i = 0; i < n; ++i) {
    if (lo[i] > hi[i] || lo[i] < 0) return 1;
    slo += lo[i];
    shi += hi[i];
  }
  if (slo > total || shi < total) return 1;
  int nf = n;
  for (int i = 0; i < n; ++i) freel[i] = i;
  long long remaining = total;
  while (nf > 0) {
    // proportional split of `remaining` over the free layers, largest remainder
    double wsum = 0.0;
    for (int j = 0; j < nf; ++j) wsum += (double)e[freel[j]];
    const bool uniform = !(wsum > 0.0);
    if (uniform) wsum = (double)nf;
    long long given = 0;
    for (int j = 0; j < nf; ++j) {
      const double wj = uniform ? 1.0 : (double)e[freel[j]];
      quota[j] = (wj / wsum) * (double)remaining;
      base[j] = (long long)floor(quota[j]);
      frac[j] = quota[j] - (double)base[j];
      given += base[j];
    }
    long long left = remaining - given;
    if (left > 0) {
      // position j receives ceil-share of the units: one per full cycle plus one more if its
      // rank (by descending fraction, ties to the lower position) is below the remainder
      const long long cycles = left / nf, rem = left % nf;
      for (int j = 0; j < nf; ++j) {
        int rank = 0;
        for (int t = 0; t < nf; ++t) rank += (frac[t] > frac[j]) || (frac[t] == frac[j] && t < j);
        base[j] += cycles + (rank < rem ? 1 : 0);
      }
    } else if (left < 0) {
      // only reachable through floating-point rounding of the quotas: take units back from the
      // smallest fractions (largest rank first), skipping layers already at zero
      int guard = 0;
      while (left < 0 && guard < 4 * nf) {
        const int want = nf - 1 - (guard % nf);
        for (int j = 0; j < nf; ++j) {
          int rank = 0;
          for (int t = 0; t < nf; ++t) rank += (frac[t] > frac[j]) || (frac[t] == frac[j] && t < j);
          if (rank == want && base[j] > 0 && left < 0) {
            base[j] -= 1;
            left += 1;
          }
        }
        ++guard;
      }
    }
    // bound violations
    long long excess = 0, deficit = 0;
    int n_over = 0, n_under = 0;
    for (int j = 0; j < nf; ++j) {
      const int i = freel[j];
      if (base[j] > hi[i]) { excess += base[j] - hi[i]; ++n_over; }
      if (base[j] < lo[i]) { deficit += lo[i] - base[j]; ++n_under; }
    }
    if (n_over == 0 && n_under == 0) {
      for (int j = 0; j < nf; ++j) out[freel[j]] = base[j];
      break;
    }
    const bool pin_over = n_over > 0 && excess >= deficit;
    int keep = 0;
    for (int j = 0; j < nf; ++j) {
      const int i = freel[j];
      const bool pin = pin_over ? (base[j] > hi[i]) : (base[j] < lo[i]);
      if (pin) {
        out[i] = pin_over ? hi[i] : lo[i];
        remaining -= out[i];
      } else {
        freel[keep++] = i;
      }
    }
    nf = keep;
  }
  return 0;
}

int32_t budgets_host(int32_t batch, int32_t n_layers, const float* e, const int64_t* total,
                     const int64_t* lo, const int64_t* hi, int64_t* out) {
  std::vector<double> quota(n_layers), frac(n_layers);
  std::vector<long long> base(n_layers), lo_(n_layers), hi_(n_layers), out_(n_layers);
  std::vector<int> freel(n_layers);
  // validate every sequence before writing anything
  for (int pass = 0; pass < 2; ++pass) {
    for (int b = 0; b < batch; ++b) {
      for (int i = 0; i < n_layers; ++i) {
        lo_[i] = lo[(size_t)b * n_layers + i];
        hi_[i] = hi[(size_t)b * n_layers + i];
      }
      const int bad = allocate_budgets(n_layers, e + (size_t)b * n_layers, total[b], lo_.data(),
                                       hi_.data(), out_.data(), quota.data(), base.data(),
                                       freel.data(), frac.data());
      if (bad) return LAVA_ERR_BUDGET;
      if (pass == 1)
        for (int i = 0; i < n_layers; ++i) out[(size_t)b * n_layers + i] = out_[i];
    }
  }
  return LAVA_OK;
}

__global__ void __launch_bounds__(64) budgets_kernel(int n_layers, const float* __restrict__ e,
                                                     const int64_t* __restrict__ total,
                                                     const int64_t* __restrict__ lo,
                                                     const int64_t* __restrict__ hi,
                                                     int64_t* __restrict__ out) {
  __shared__ BudgetScratch sc;
  const size_t b = blockIdx.x;
  for (int i = threadIdx.x; i < n_layers; i += 64) {
    sc.ed[i] = (double)e[b * n_layers + i];
    sc.lo[i] = (long long)lo[b * n_layers + i];
    sc.hi[i] = (long long)hi[b * n_layers + i];
  }
  __syncthreads();
  long long* out_b = reinterpret_cast<long long*>(out) + b * n_layers;
  const int bad = allocate_budgets_wave<BlockSync>((int)threadIdx.x, n_layers, sc.ed, (long long)total[b], sc.lo, sc.hi, out_b, sc.quota,
                                        sc.base, sc.freel, sc.frac, sc.state);
  if (bad)
    for (int i = threadIdx.x; i < n_layers; i += 64) out_b[i] = -1;
}

// A step of the cascade: budgets of the layers seen so far (same bounds for every layer), then the
// rows each layer will keep = its budget, but no more than it holds (for the newest layer: its
// dense size `hi`), and from those the first row of every layer in the pool the step writes.
__global__ void __launch_bounds__(64) cascade_plan_kernel(int n_layers, int n_heads, const float* __restrict__ e,
                                                          long long total, long long lo, long long hi,
                                                          long long bound,
                                                          const int64_t* __restrict__ head_offsets_cur,
                                                          int64_t* __restrict__ out,
                                                          int64_t* __restrict__ layer_start,
                                                          unsigned int* __restrict__ gather_sync,
                                                          const SelectRegions regions) {
  // workgroups 1 .. n_layers: each clears the workspace region and the survivor counts of one of the
  // step's selections, which then need no clearing launch of their own; workgroup 0: the plan
  if (blockIdx.x > 0) {
    const int t = (int)blockIdx.x - 1;
    char* region = regions.ws + (size_t)t * regions.stride;
    unsigned int* hist = reinterpret_cast<unsigned int*>(region + regions.off_hist);
    unsigned int* state = reinterpret_cast<unsigned int*>(region + regions.off_state);
    for (int i = threadIdx.x; i < 3 * kSelBins; i += 64) hist[i] = 0u;
    if (threadIdx.x < kSelStateWords) state[threadIdx.x] = 0u;
    for (int i = threadIdx.x; i < n_heads; i += 64) regions.head_counts[(size_t)t * n_heads + i] = 0;
    return;
  }
  __shared__ BudgetScratch sc;
  // the in-place gather later in the same step meets at a grid-wide barrier: its counter starts at zero
  if (gather_sync != nullptr) {
    gather_sync[threadIdx.x] = 0u;
    gather_sync[64 + threadIdx.x] = 0u;
  }
  for (int i = threadIdx.x; i < n_layers; i += 64) {
    sc.ed[i] = (double)e[i];
    sc.lo[i] = lo;
    sc.hi[i] = hi;
  }
  __syncthreads();
  long long* out_b = reinterpret_cast<long long*>(out);
  const int bad = allocate_budgets_wave<BlockSync>((int)threadIdx.x, n_layers, sc.ed, total, sc.lo, sc.hi, out_b, sc.quota, sc.base, sc.freel,
                                        sc.frac, sc.state);
  if (bad)
    for (int i = threadIdx.x; i < n_layers; i += 64) out_b[i] = -1;
  __syncthreads();
  for (int t = threadIdx.x; t < n_layers; t += 64) {
    long long held = hi;
    if (t + 1 < n_layers) {
      held = (long long)head_offsets_cur[(long long)t * (n_heads + 1) + n_heads];
      held = held < 0 ? 0 : held;
    }
    const long long cap = held < bound ? held : bound;
    long long kept = out_b[t];
    kept = kept < 0 ? 0 : (kept < cap ? kept : cap);
    sc.base[t] = kept;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    long long start = 0;
    for (int t = 0; t < n_layers; ++t) {
      layer_start[t] = start;
      start += sc.base[t];
    }
    layer_start[n_layers] = start;
  }
}

int32_t launch_cascade_plan(int32_t n_layers, int32_t n_heads, const float* e, int64_t total, int64_t lo, int64_t hi,
                            int64_t bound, const int64_t* head_offsets_cur, int64_t* budgets, int64_t* layer_start,
                            unsigned int* gather_sync, const SelectRegions& regions, hipStream_t s) {
  if (n_layers > kMaxLayers) return LAVA_ERR_SHAPE;
  ProfScope ps(KID_BUDGETS, s);
  hipLaunchKernelGGL(cascade_plan_kernel, dim3(1 + (regions.ws != nullptr ? n_layers : 0)), dim3(64), 0, s, n_layers,
                     n_heads, e, (long long)total, (long long)lo, (long long)hi, (long long)bound, head_offsets_cur,
                     budgets, layer_start, gather_sync, regions);
  return launch_status();
}

int32_t launch_budgets(int32_t batch, int32_t n_layers, const float* e, const int64_t* total,
                       const int64_t* lo, const int64_t* hi, int64_t* out, hipStream_t s) {
  if (n_layers > kMaxLayers) return LAVA_ERR_SHAPE;
  ProfScope ps(KID_BUDGETS, s);
  hipLaunchKernelGGL(budgets_kernel, dim3(batch), dim3(64), 0, s, n_layers, e, total, lo, hi, out);
  return launch_status();
}

}  // namespace lava
