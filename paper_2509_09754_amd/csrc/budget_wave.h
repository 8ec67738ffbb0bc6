// Layer budgets on the device: the integer rule of the host routine (floor the quotas, leftover units to the
// largest fractional parts, pin layers that violate a bound and split the rest again; Alg. 2, inner loop)
// spread over the 64 lanes of ONE wavefront.  Shared by the budgets kernels and by the score kernels, whose
// last workgroup can run it right after it has formed the layer statistic.
#pragma once

#include <hip/hip_runtime.h>
#include <math.h>

namespace lava {

constexpr int kMaxLayers = 1024;        // budgets kernels
constexpr int kMaxPlannedLayers = 128;  // budgets formed at the end of a scores launch (LAVA_PLAN_MAX_LAYERS): the scratch
                                        // has to fit what is left of one wavefront's tile ring

// How the lanes of the wavefront wait for each other's LDS writes: a workgroup barrier where the
// wavefront is the whole workgroup, otherwise (one wavefront of a larger workgroup; LDS operations of
// one wavefront complete in order) only a point the compiler moves no LDS access across.
struct BlockSync {
  __device__ static __forceinline__ void sync() { __syncthreads(); }
};
struct WaveSync {
  __device__ static __forceinline__ void sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
};

__device__ __forceinline__ long long wave_sum(long long x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
  return x;
}

// The same routine run by the 64 lanes of one wavefront (the workgroup): every per-layer quantity
// is computed by one lane with the arithmetic of allocate_budgets, integer sums are reduced
// across lanes (exact in any order), the fp64 weight sum is taken in layer order by every lane, and
// the rare and order-dependent parts (units taken back after a rounding overshoot, the free list)
// stay with lane 0.  Results are identical to the sequential routine.  All control flow is uniform.
// Scratch in LDS (length n each): ed, quota, frac, base, freel; state: two words.
template <typename Sync>
__device__ inline int allocate_budgets_wave(int lane, int n, const double* ed, long long total, const long long* lo,
                                            const long long* hi, long long* out, double* quota,
                                            long long* base, int* freel, double* frac, long long* state) {
#pragma clang fp contract(off)
  long long slo = 0, shi = 0, bad = 0;
  for (int i = lane; i < n; i += 64) {
    if (lo[i] > hi[i] || lo[i] < 0) bad = 1;
    slo += lo[i];
    shi += hi[i];
    freel[i] = i;
  }
  bad = wave_sum(bad);
  slo = wave_sum(slo);
  shi = wave_sum(shi);
  if (bad != 0 || slo > total || shi < total) return 1;
  Sync::sync();
  int nf = n;
  long long remaining = total;
  while (nf > 0) {
    double wsum = 0.0;
    for (int j = 0; j < nf; ++j) wsum += ed[freel[j]];
    const bool uniform = !(wsum > 0.0);
    if (uniform) wsum = (double)nf;
    long long given = 0;
    for (int j = lane; j < nf; j += 64) {
      const double wj = uniform ? 1.0 : ed[freel[j]];
      quota[j] = (wj / wsum) * (double)remaining;
      base[j] = (long long)floor(quota[j]);
      frac[j] = quota[j] - (double)base[j];
      given += base[j];
    }
    given = wave_sum(given);
    Sync::sync();
    const long long left = remaining - given;
    if (left > 0) {
      const long long cycles = left / nf, rem = left % nf;
      for (int j = lane; j < nf; j += 64) {
        const double fj = frac[j];
        int rank = 0;
        for (int t = 0; t < nf; ++t) {
          const double ft = frac[t];
          rank += (ft > fj) || (ft == fj && t < j);
        }
        base[j] += cycles + (rank < rem ? 1 : 0);
      }
    } else if (left < 0) {
      if (lane == 0) {
        long long l = left;
        int guard = 0;
        while (l < 0 && guard < 4 * nf) {
          const int want = nf - 1 - (guard % nf);
          for (int j = 0; j < nf; ++j) {
            int rank = 0;
            for (int t = 0; t < nf; ++t) rank += (frac[t] > frac[j]) || (frac[t] == frac[j] && t < j);
            if (rank == want && base[j] > 0 && l < 0) {
              base[j] -= 1;
              l += 1;
            }
          }
          ++guard;
        }
      }
    }
    Sync::sync();
    long long excess = 0, deficit = 0, n_over = 0, n_under = 0;
    for (int j = lane; j < nf; j += 64) {
      const int i = freel[j];
      if (base[j] > hi[i]) { excess += base[j] - hi[i]; ++n_over; }
      if (base[j] < lo[i]) { deficit += lo[i] - base[j]; ++n_under; }
    }
    excess = wave_sum(excess);
    deficit = wave_sum(deficit);
    n_over = wave_sum(n_over);
    n_under = wave_sum(n_under);
    if (n_over == 0 && n_under == 0) {
      for (int j = lane; j < nf; j += 64) out[freel[j]] = base[j];
      break;
    }
    const bool pin_over = n_over > 0 && excess >= deficit;
    if (lane == 0) {
      int keep = 0;
      long long rest = remaining;
      for (int j = 0; j < nf; ++j) {
        const int i = freel[j];
        const bool pin = pin_over ? (base[j] > hi[i]) : (base[j] < lo[i]);
        if (pin) {
          out[i] = pin_over ? hi[i] : lo[i];
          rest -= out[i];
        } else {
          freel[keep++] = i;
        }
      }
      state[0] = rest;
      state[1] = keep;
    }
    Sync::sync();
    remaining = state[0];
    nf = (int)state[1];
    Sync::sync();
  }
  return 0;
}

template <int N>
struct BudgetScratchT {
  double ed[N], quota[N], frac[N];
  long long base[N], lo[N], hi[N];
  int freel[N];
  long long state[2];
};
using BudgetScratch = BudgetScratchT<kMaxLayers>;

}  // namespace lava
