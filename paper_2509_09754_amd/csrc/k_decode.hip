// Decode-step attention over the compressed layer cache (Sec. 2 decoding step under the mask of
// Sec. 3): one query token per sequence, the G query heads of a KV group share the group's
// retained rows, which sit packed and variable-length per head as the selection wrote them.
//
//   decode_kernel   one workgroup per "unit" = up to C consecutive rows of one head (packed rows
//                   first, then the rows appended since the eviction).  Each wavefront streams
//                   32-row tiles: K through its private LDS ring (two tiles ahead), V straight
//                   into registers (one tile ahead; a lane owns the same columns of every row, so
//                   a row is one coalesced load and needs no LDS).  The step is latency-bound
//                   unless enough bytes are in flight per compute unit, and registers are the
//                   larger buffer:
//                     logits   K_tile x Q^T on the matrix cores (the G heads are G columns of the
//                              32-wide operand; the product is exact, accumulation fp32)
//                     softmax  online, in the exp2 domain, per head, kept in the column's lanes
//                     output   acc[head][dims of this lane] += p[key][head] * V[key][dims]: the
//                              probabilities go through LDS as fp32 and are broadcast per key;
//                              V is never rounded or transposed
//                   then the wavefronts' partial (max, sum, acc) are merged and written out.
//   decode_merge    one workgroup per (sequence, KV head): merges the units of the head in unit
//                   order (deterministic) and normalises.
//
// The step is bound by HBM: 2 * d_h * elem bytes per retained row against 4 * G * d_h flop.
#include <math.h>

#include "common.h"
#include "tile_ring.h"

namespace lava {

namespace {

constexpr int kDecWaves = 4;
constexpr int kDecThreads = kDecWaves * 64;

// Two ring stages per wavefront (the K and the V tile of the moment): a workgroup then takes
// well under half of a compute unit's LDS, so two workgroups share a unit and the set-up of one
// overlaps the streaming of the other.
template <int DT, int D>
struct DecShape {
  using T = Tile<DT, D>;
  static constexpr int kStages = 2;
  static constexpr int kBpl = T::kRowBytes / 64;              // bytes of a row one lane owns
  static constexpr int kDpl = kBpl / Elem<DT>::kBytes;        // elements of a row one lane owns
  static_assert(kDpl == 1 || kDpl == 2, "one or two output columns per lane");
  static_assert(kDecWaves * kStages * T::kTileBytes >= kDecWaves * 8 * D * 4, "the ring doubles as the merge buffer");
};

template <int BYTES> struct RawBits;
template <> struct RawBits<2> { using type = unsigned short; };
template <> struct RawBits<4> { using type = unsigned int; };
template <> struct RawBits<8> { using type = uint2; };

// The kDpl elements of a row this lane owns, from their raw bits to floats.
template <int DT, int D>
__device__ __forceinline__ void unpack_v(const typename RawBits<DecShape<DT, D>::kBpl>::type& raw,
                                         float (&x)[DecShape<DT, D>::kDpl]) {
  using S = DecShape<DT, D>;
  if constexpr (DT == LAVA_BF16 && S::kDpl == 1) {
    x[0] = __uint_as_float((unsigned int)raw << 16);
  } else if constexpr (DT == LAVA_BF16) {
    x[0] = __uint_as_float(raw << 16);
    x[1] = __uint_as_float(raw & 0xffff0000u);
  } else if constexpr (S::kDpl == 1) {
    x[0] = __uint_as_float(raw);
  } else {
    x[0] = __uint_as_float(raw.x);
    x[1] = __uint_as_float(raw.y);
  }
}

struct DecodeArgs {
  const u32x4* q;
  const char* k_hat;
  const char* v_hat;
  const long long* head_offsets;   // [batch][H_kv + 1]
  const long long* seq_base;       // [batch] or null
  long long rows_capacity;
  const char* k_tail;
  const char* v_tail;
  long long tail_len, tail_capacity;
  int H, H_kv, G;
  int rows_per_unit;               // C, a multiple of 32 * kDecWaves
  int units_bound;                 // grid.x: units a sequence can have at most
  float c2;                        // softmax scale * log2 e
  float2* part_ml;                 // [batch][units_bound][GP]  (max in log2 units, sum)
  float* part_acc;                 // [batch][units_bound][GP][D]
};

__device__ __forceinline__ long long ceil_div(long long a, long long b) { return (a + b - 1) / b; }

__device__ __forceinline__ long long uniform64(long long x) {
  const unsigned int lo = __builtin_amdgcn_readfirstlane((unsigned int)((unsigned long long)x & 0xffffffffull));
  const unsigned int hi = __builtin_amdgcn_readfirstlane((unsigned int)((unsigned long long)x >> 32));
  return (long long)(((unsigned long long)hi << 32) | lo);
}

// The units of one sequence, found by every wavefront on its own with one coalesced load of the
// head offsets: lane g holds head g.  Units are numbered head by head, each head's packed chunks
// first, then its tail chunks.  Offsets a kernel may follow start at >= 0, never decrease and end
// within the stated capacity; anything else makes `usable` false and nothing is read.
struct UnitMap {
  bool usable;
  unsigned int total;        // units of the sequence
  unsigned int incl;         // lane g: units of heads 0..g
  unsigned int cnt;          // lane g: units of head g
  unsigned int packed;       // lane g: packed units of head g
  long long off, len;        // lane g: first packed row and number of packed rows of head g
};

__device__ __forceinline__ UnitMap map_units(const long long* __restrict__ offs, int n_heads, long long capacity,
                                             int rows_per_unit, long long tail_len, int lane) {
  UnitMap m;
  // lane g holds offs[g]; the end of the last head comes from a load of its own, because with 64
  // heads no lane is left to hold offs[64]
  const bool head = lane < n_heads;
  const long long o = head ? offs[lane] : 0;
  const long long o_end = offs[n_heads];
  const long long o_down = __shfl_down(o, 1);
  const long long o_next = lane == n_heads - 1 ? o_end : o_down;
  const bool bad = (head && o_next < o) || (lane == 0 && o < 0) || o_end > capacity;
  m.usable = __ballot(bad) == 0ull;
  m.off = o;
  m.len = head && m.usable ? o_next - o : 0;
  const unsigned int tail_units = tail_len > 0 ? (unsigned int)ceil_div(tail_len, rows_per_unit) : 0u;
  m.packed = (unsigned int)ceil_div(m.len, rows_per_unit);
  m.cnt = head && m.usable ? m.packed + tail_units : 0u;
  unsigned int incl = m.cnt;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const unsigned int up = __shfl_up(incl, d);
    if (lane >= d) incl += up;
  }
  m.incl = incl;
  m.total = __shfl(incl, 63);
  return m;
}

template <int DT, int D, int GP>
__global__ void __launch_bounds__(kDecThreads) decode_kernel(DecodeArgs a) {
  using S = DecShape<DT, D>;
  using T = Tile<DT, D>;
  constexpr int kStages = S::kStages;
  constexpr int kDpl = S::kDpl;
  __shared__ u32x4 s_tile[kDecWaves][kStages][T::kTileChunks];   // after the sweep: float [kDecWaves][GP][D]
  constexpr int kPs = GP < 4 ? 4 : GP;                      // floats per key in s_p (one or two 128-bit reads)
  __shared__ __attribute__((aligned(16))) float s_p[kDecWaves][kTileKeys + 1][kPs];   // probabilities; row 32: rescale factors
  __shared__ float s_m[kDecWaves][GP], s_l[kDecWaves][GP];

  const int lane = threadIdx.x & 63, wave = wave_index();
  const int b = blockIdx.y;
  const UnitMap um = map_units(a.head_offsets + (long long)b * (a.H_kv + 1), a.H_kv, a.rows_capacity,
                               a.rows_per_unit, a.tail_len, lane);
  if (!um.usable || blockIdx.x >= um.total) return;         // bad offsets (the merge reports them) or no such unit
  const int g = __builtin_ctzll(__ballot(um.incl > blockIdx.x));
  const long long u = (long long)blockIdx.x - (__builtin_amdgcn_readfirstlane(__shfl(um.incl, g)) -
                                                __builtin_amdgcn_readfirstlane(__shfl(um.cnt, g)));
  const long long packed_units = __builtin_amdgcn_readfirstlane(__shfl(um.packed, g));
  const long long off_g = uniform64(__shfl(um.off, g)), len_g = uniform64(__shfl(um.len, g));

  const char* kb;
  const char* vb;
  long long n_rows;
  if (u < packed_units) {
    const long long base = (a.seq_base ? a.seq_base[b] : (long long)b * a.rows_capacity) + off_g +
                           u * a.rows_per_unit;
    n_rows = len_g - u * a.rows_per_unit;
    kb = a.k_hat + base * T::kRowBytes;
    vb = a.v_hat + base * T::kRowBytes;
  } else {
    const long long c = u - packed_units;
    const long long base = ((long long)b * a.H_kv + g) * a.tail_capacity + c * a.rows_per_unit;
    n_rows = a.tail_len - c * a.rows_per_unit;
    kb = a.k_tail + base * T::kRowBytes;
    vb = a.v_tail + base * T::kRowBytes;
  }
  if (n_rows > a.rows_per_unit) n_rows = a.rows_per_unit;

  // This wavefront's tiles: wave, wave + kDecWaves, ...  Vector-memory operations complete in issue
  // order and the K ring is awaited by count, so the order below is part of the protocol:
  //   K_0, K_1 | query rows, V_0 | then per tile i:  K_{i+2} ... V_{i+1}
  using VRaw = typename RawBits<S::kBpl>::type;
  TileDma<DT, D> dma;
  dma.init(lane);
  const long long n_tiles = ceil_div(n_rows, kTileKeys);
  const int cnt = wave < n_tiles ? (int)((n_tiles - wave + kDecWaves - 1) / kDecWaves) : 0;
  u32x4* ring = s_tile[wave][0];
  FragReader<DT, D> frags;
  frags.init_at(lane, lds_addr(ring));
  const unsigned int p_addr = lds_addr(&s_p[wave][0][0]);
  auto issue_k = [&](int i) {
    dma.issue(kb, wave + (long long)i * kDecWaves, n_rows, lane, ring + (i % kStages) * T::kTileChunks);
  };
  const unsigned int v_lane = (unsigned int)lane * S::kBpl;   // a row is a uniform address plus this
  auto load_v = [&](VRaw (&dst)[kTileKeys], int i) {
    const long long row0 = (wave + (long long)i * kDecWaves) * kTileKeys;
    const char* p = vb + row0 * T::kRowBytes;
    if (row0 + kTileKeys <= n_rows) {
#pragma unroll
      for (int kk = 0; kk < kTileKeys; ++kk) dst[kk] = *reinterpret_cast<const VRaw*>(p + kk * T::kRowBytes + v_lane);
    } else {                                                // rows beyond the unit repeat its last row
      const int last = (int)(n_rows - 1 - row0);            // 0 .. 30, uniform
#pragma unroll
      for (int kk = 0; kk < kTileKeys; ++kk)
        dst[kk] = *reinterpret_cast<const VRaw*>(p + (kk < last ? kk : last) * T::kRowBytes + v_lane);
    }
  };
  if (cnt > 0) issue_k(0);
  if (cnt > 1) issue_k(1);
  asm volatile("" ::: "memory");

  // the group's query rows as the 32-column operand: column t < G is head g*G + t
  const int col = lane & 31, half = lane >> 5;
  u32x4 qf[T::kSteps];
#pragma unroll
  for (int j = 0; j < T::kSteps; ++j) {
    u32x4 x = u32x4{0u, 0u, 0u, 0u};
    if (col < a.G) x = a.q[((long long)b * a.H + (long long)g * a.G + col) * T::kCpr + 2 * j + half];
    qf[j] = x;
  }
  const unsigned int p_col = p_addr + (unsigned int)(col * 4);                  // row 0 of s_p, this head's column
  const unsigned int p_mine = p_col + (unsigned int)(4 * half * kPs * 4);       // first key this lane's results cover
  VRaw v0[kTileKeys], v1[kTileKeys];
  if (cnt > 0) load_v(v0, 0);

  float m_run = -INFINITY, l_run = 0.0f;                    // of head `col` (lanes col < G)
  float acc[GP][kDpl];
#pragma unroll
  for (int t = 0; t < GP; ++t)
#pragma unroll
    for (int e = 0; e < kDpl; ++e) acc[t][e] = 0.0f;

  // PAR = it % 2 is the ring stage of K_it
  auto step = [&](auto par, int it, VRaw (&v_cur)[kTileKeys], VRaw (&v_next)[kTileKeys]) {
    constexpr int PAR = decltype(par)::value;
    const long long tile = wave + (long long)it * kDecWaves;
    // ---------------- K tile: logits, online softmax, probabilities to LDS
    {
      // everything older than V_it (32 loads) and, if it was requested, K_{it+1} has landed
      if (it + 1 < cnt) wait_vmcnt<T::kLoads + kTileKeys>(); else wait_vmcnt<kTileKeys>();
      u32x4 kf[T::kSteps];
      frags.template read_at<PAR * T::kTileBytes>(kf);      // in registers on return: the stage is free
      if (it + 2 < cnt) issue_k(it + 2);
      asm volatile("" ::: "memory");
      // two independent accumulation chains halve the latency of the dependent MFMAs
      f32x16 x = {0}, x2 = {0};
#pragma unroll
      for (int j = 0; j < T::kSteps; j += 2) {
        x = mfma_chunk<DT>(kf[j], qf[j], x);
        x2 = mfma_chunk<DT>(kf[j + 1], qf[j + 1], x2);
      }
      x += x2;                                              // x[v]: key 8*(v/4) + 4*half + v%4, head col
      const long long left = n_rows - tile * kTileKeys;     // rows of the unit from this tile on (uniform)
      float mt = -INFINITY;
      if (left >= kTileKeys) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          x[v] *= a.c2;
          mt = fmaxf(mt, x[v]);
        }
      } else {                                              // the unit's last, partial tile
        int h4 = 4 * half;
        asm volatile("" : "+v"(h4));                        // keeps this path's temporaries out of the hot loop
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float s = (h4 + 8 * (v / 4) + (v % 4) < (int)left) ? x[v] * a.c2 : -INFINITY;
          x[v] = s;
          mt = fmaxf(mt, s);
        }
      }
      mt = fmaxf(mt, __shfl_xor(mt, 32));
      const float m_new = fmaxf(m_run, mt);                 // finite: a tile holds at least one row
      const float alpha = fast_exp2(m_run - m_new);
      float ls = 0.0f;
      if (col < GP) {
        static_for<16>([&](auto vc) {
          constexpr int v = decltype(vc)::value;
          const float p = fast_exp2(x[v] - m_new);
          ls += p;
          lds_write32_at<(8 * (v / 4) + (v % 4)) * kPs * 4>(p_mine, p);
        });
        if (half == 0) lds_write32_at<kTileKeys * kPs * 4>(p_col, alpha);
      }
      l_run = l_run * alpha + ls;
      m_run = m_new;
    }
    lds_reads_done();                                       // LDS operations of a wavefront execute in order
    // ---------------- V tile (already requested): request the next one, rescale, accumulate
    {
      if (it + 1 < cnt) load_v(v_next, it + 1);
      asm volatile("" ::: "memory");
      u32x4 al[kPs / 4];
      static_for<kPs / 4>([&](auto cc) {
        constexpr int c = decltype(cc)::value;
        lds_read128_at<(kTileKeys * kPs + 4 * c) * 4>(p_addr, al[c]);
      });
#pragma unroll
      for (int t = 0; t < GP; ++t)
#pragma unroll
        for (int e = 0; e < kDpl; ++e) acc[t][e] *= __uint_as_float(al[t / 4][t % 4]);
      // probabilities of four keys per read batch
      static_for<kTileKeys / 4>([&](auto kc) {
        constexpr int k4 = 4 * decltype(kc)::value;
        u32x4 pr[kPs / 4][4];
        static_for<kPs / 4>([&](auto cc) {
          constexpr int c = decltype(cc)::value;
          lds_read128x4_strided<kPs * 4, (k4 * kPs + 4 * c) * 4>(p_addr, pr[c][0], pr[c][1], pr[c][2], pr[c][3]);
        });
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          float vx[kDpl];
          unpack_v<DT, D>(v_cur[k4 + kk], vx);
#pragma unroll
          for (int t = 0; t < GP; ++t) {
            const float p = __uint_as_float(pr[t / 4][kk][t % 4]);
#pragma unroll
            for (int e = 0; e < kDpl; ++e) acc[t][e] = fmaf(p, vx[e], acc[t][e]);
          }
        }
        // pin the accumulators here: otherwise the multiply-adds of all batches sink below the reads
        // of all batches, which then have to stay in registers together
#pragma unroll
        for (int t = 0; t < GP; ++t)
#pragma unroll
          for (int e = 0; e < kDpl; ++e) asm volatile("" : "+v"(acc[t][e]));
      });
    }
  };
  int it = 0;
  for (; it + 1 < cnt; it += 2) {
    step(std::integral_constant<int, 0>{}, it, v0, v1);
    step(std::integral_constant<int, 1>{}, it + 1, v1, v0);
  }
  if (it < cnt) step(std::integral_constant<int, 0>{}, it, v0, v1);
  wait_vmcnt<0>();

  // ---------------- merge the wavefronts of the unit
  l_run += __shfl_xor(l_run, 32);
  if (lane < GP) {
    s_m[wave][lane] = m_run;
    s_l[wave][lane] = l_run;
  }
  __syncthreads();                                          // every wavefront is done with its ring
  float (*s_acc)[GP][D] = reinterpret_cast<float (*)[GP][D]>(&s_tile[0][0][0]);
#pragma unroll
  for (int t = 0; t < GP; ++t)
#pragma unroll
    for (int e = 0; e < kDpl; ++e) s_acc[wave][t][lane * kDpl + e] = acc[t][e];
  __syncthreads();
  const long long slot = (long long)b * a.units_bound + blockIdx.x;
  for (int idx = threadIdx.x; idx < GP * D; idx += kDecThreads) {
    const int t = idx / D, e = idx % D;
    float M = s_m[0][t];
#pragma unroll
    for (int w2 = 1; w2 < kDecWaves; ++w2) M = fmaxf(M, s_m[w2][t]);
    float sum = 0.0f;
#pragma unroll
    for (int w2 = 0; w2 < kDecWaves; ++w2) sum += fast_exp2(s_m[w2][t] - M) * s_acc[w2][t][e];
    a.part_acc[(slot * GP + t) * D + e] = sum;
    if (e == 0) {
      float L = 0.0f;
#pragma unroll
      for (int w2 = 0; w2 < kDecWaves; ++w2) L += fast_exp2(s_m[w2][t] - M) * s_l[w2][t];
      a.part_ml[slot * GP + t] = make_float2(M, L);
    }
  }
}

// One workgroup per (KV head, sequence): merge the head's units in unit order (deterministic).
// Units are taken kMergeChunk at a time: their (max, sum) pairs go through LDS, every thread then
// knows the chunk's maximum per head without a second trip to memory, and the loads of the partial
// outputs of a whole chunk are independent of each other, so the kernel's time does not grow with the
// number of units the way a loop of dependent round trips does.  Across chunks the running result is
// rescaled as in the online softmax.
constexpr int kMergeChunk = 32;
template <int D, int GP>
__global__ void __launch_bounds__(256) decode_merge_kernel(DecodeArgs a, float* __restrict__ out,
                                                           float* __restrict__ lse) {
  const int b = blockIdx.y, g = blockIdx.x;
  const UnitMap um = map_units(a.head_offsets + (long long)b * (a.H_kv + 1), a.H_kv, a.rows_capacity,
                               a.rows_per_unit, a.tail_len, (int)(threadIdx.x & 63));
  const int mine = (int)__builtin_amdgcn_readfirstlane(__shfl(um.cnt, g));
  const long long first = (long long)__builtin_amdgcn_readfirstlane(__shfl(um.incl, g)) - mine;
  const bool overflow = !um.usable || um.total > (unsigned int)a.units_bound;
  const float2* ml = a.part_ml + ((long long)b * a.units_bound + first) * GP;
  const float* pa = a.part_acc + ((long long)b * a.units_bound + first) * GP * D;
  __shared__ float2 s_ml[kMergeChunk][GP];
  constexpr int kOut = (GP * D + 255) / 256;                // outputs per thread: (t, e) = (idx / D, idx % D), idx = tid + 256 j
  float M[kOut], L[kOut], sum[kOut];
#pragma unroll
  for (int j = 0; j < kOut; ++j) { M[j] = -INFINITY; L[j] = 0.0f; sum[j] = 0.0f; }
  for (int c0 = 0; c0 < (overflow ? 0 : mine); c0 += kMergeChunk) {
    const int nu = mine - c0 < kMergeChunk ? mine - c0 : kMergeChunk;
    for (int i = threadIdx.x; i < nu * GP; i += 256) s_ml[i / GP][i % GP] = ml[(long long)c0 * GP + i];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kOut; ++j) {
      const int idx = (int)threadIdx.x + 256 * j;
      if (idx >= a.G * D) continue;
      const int t = idx / D, e = idx % D;
      float mc = s_ml[0][t].x;
      for (int u = 1; u < nu; ++u) mc = fmaxf(mc, s_ml[u][t].x);
      const float m_new = fmaxf(M[j], mc);                   // finite: a unit holds at least one row
      const float keep = fast_exp2(M[j] - m_new);            // exp2(-inf) = 0 for the first chunk
      float l_new = L[j] * keep, s_new = sum[j] * keep;
      const float* col = pa + ((long long)c0 * GP + t) * D + e;
      for (int u0 = 0; u0 < nu; u0 += 16) {                  // sixteen independent loads per round trip
        float pv[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) pv[u] = u0 + u < nu ? col[(long long)(u0 + u) * GP * D] : 0.0f;
#pragma unroll
        for (int u = 0; u < 16; ++u) {                       // unit order: the result does not depend on timing
          if (u0 + u < nu) {
            const float2 st = s_ml[u0 + u][t];
            const float wgt = fast_exp2(st.x - m_new);
            l_new += wgt * st.y;
            s_new += wgt * pv[u];
          }
        }
      }
      M[j] = m_new;
      L[j] = l_new;
      sum[j] = s_new;
    }
    __syncthreads();                                         // the next chunk overwrites s_ml
  }
#pragma unroll
  for (int j = 0; j < kOut; ++j) {
    const int idx = (int)threadIdx.x + 256 * j;
    if (idx >= a.G * D) continue;
    const int t = idx / D, e = idx % D;
    float result = 0.0f, lse_v = -INFINITY;
    if (overflow) {
      result = lse_v = NAN;
    } else if (mine > 0) {
      result = sum[j] / L[j];
      lse_v = (M[j] + log2f(L[j])) * 0.6931471805599453f;
    }
    out[((long long)b * a.H + (long long)g * a.G + t) * D + e] = result;
    if (lse != nullptr && e == 0) lse[(long long)b * a.H + (long long)g * a.G + t] = lse_v;
  }
}

template <int DT, int D, int GP>
int32_t launch_one(const DecodeArgs& a, int batch, float* out, float* lse, hipStream_t s) {
  {
    ProfScope ps(KID_DECODE, s);
    hipLaunchKernelGGL((decode_kernel<DT, D, GP>), dim3(a.units_bound, batch), dim3(kDecThreads), 0, s, a);
  }
  int32_t st = launch_status();
  if (st != LAVA_OK) return st;
  {
    ProfScope ps(KID_DECODE_MERGE, s);
    hipLaunchKernelGGL((decode_merge_kernel<D, GP>), dim3(a.H_kv, batch), dim3(256), 0, s, a, out, lse);
  }
  return launch_status();
}

int padded_group(int G) { return G <= 1 ? 1 : G <= 2 ? 2 : G <= 4 ? 4 : 8; }

int device_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      return 256;
  }
  return cus;
}

}  // namespace

DecodePlan make_decode_plan(const lava_layer_desc& d, int32_t batch, int64_t rows_capacity, int64_t tail_len) {
  DecodePlan p;
  const int64_t step = kTileKeys * kDecWaves;
  const int64_t total = (int64_t)batch * (rows_capacity + (int64_t)d.n_kv_heads * tail_len);
  // Rows per unit: the device holds two workgroups per compute unit at a time; the units should fill
  // a whole number of such rounds, at least two (units differ in length, heads end in partial units,
  // and only a second round lets the dispatcher even that out), with as few units as that allows
  // (every unit pays its set-up and leaves a partial result to merge).  A head is expected to waste
  // half a unit.  Measured on 64 x 8192 rows: 768 rows (two rounds) 60.7 us, 512 rows (two and a
  // half) 62.7 us.
  const int64_t resident = 2 * (int64_t)device_cus();
  const int64_t heads = (int64_t)batch * d.n_kv_heads;
  int64_t c = 16 * step;
  for (int64_t rounds = 2; rounds <= 64; ++rounds) {
    const int64_t room = rounds * resident - heads / 2;
    if (room <= 0) continue;
    c = ((total + room - 1) / room + step - 1) / step * step;
    if (c <= 16 * step) break;
  }
  if (c < step) c = step;
  if (c > 16 * step) c = 16 * step;
  if (tuning().decode_rows_per_unit >= step) c = tuning().decode_rows_per_unit / step * step;   // caller's tuning
  p.rows_per_unit = (int)c;
  p.group_pad = padded_group(d.n_q_heads / d.n_kv_heads);
  const int64_t tail_units = tail_len > 0 ? (tail_len + c - 1) / c : 0;
  p.units_bound = (rows_capacity + c - 1) / c + d.n_kv_heads + d.n_kv_heads * tail_units;
  if (p.units_bound < 1) p.units_bound = 1;
  const size_t slots = (size_t)batch * (size_t)p.units_bound * p.group_pad;
  p.off_ml = 0;
  p.off_acc = align_up(slots * sizeof(float2));
  p.bytes = p.off_acc + align_up(slots * d.head_dim * sizeof(float));
  return p;
}

int32_t launch_decode(const lava_layer_desc& d, int32_t batch, const void* q, const void* k_hat,
                      const void* v_hat, const int64_t* head_offsets, const int64_t* seq_base,
                      int64_t rows_capacity, const void* k_tail, const void* v_tail, int64_t tail_len,
                      int64_t tail_capacity, float* out, float* lse, void* ws, const DecodePlan& p,
                      hipStream_t s) {
  DecodeArgs a;
  a.q = static_cast<const u32x4*>(q);
  a.k_hat = static_cast<const char*>(k_hat);
  a.v_hat = static_cast<const char*>(v_hat);
  a.head_offsets = reinterpret_cast<const long long*>(head_offsets);
  a.seq_base = reinterpret_cast<const long long*>(seq_base);
  a.rows_capacity = rows_capacity;
  a.k_tail = static_cast<const char*>(k_tail);
  a.v_tail = static_cast<const char*>(v_tail);
  a.tail_len = tail_len;
  a.tail_capacity = tail_capacity;
  a.H = d.n_q_heads;
  a.H_kv = d.n_kv_heads;
  a.G = d.n_q_heads / d.n_kv_heads;
  a.rows_per_unit = p.rows_per_unit;
  a.units_bound = (int)p.units_bound;
  const float scale = d.softmax_scale > 0.0f ? d.softmax_scale : 1.0f / sqrtf((float)d.head_dim);
  a.c2 = scale * kLog2e;
  a.part_ml = reinterpret_cast<float2*>(static_cast<char*>(ws) + p.off_ml);
  a.part_acc = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_acc);

#define LAVA_DECODE_CASE(DT, D, GP) \
  if (d.dtype == DT && d.head_dim == D && p.group_pad == GP) return launch_one<DT, D, GP>(a, batch, out, lse, s);
#define LAVA_DECODE_GROUPS(DT, D) \
  LAVA_DECODE_CASE(DT, D, 1) LAVA_DECODE_CASE(DT, D, 2) LAVA_DECODE_CASE(DT, D, 4) LAVA_DECODE_CASE(DT, D, 8)
  LAVA_DECODE_GROUPS(LAVA_BF16, 128)
  LAVA_DECODE_GROUPS(LAVA_BF16, 64)
  LAVA_DECODE_GROUPS(LAVA_F32, 128)
  LAVA_DECODE_GROUPS(LAVA_F32, 64)
#undef LAVA_DECODE_GROUPS
#undef LAVA_DECODE_CASE
  return LAVA_ERR_SHAPE;
}

}  // namespace lava
