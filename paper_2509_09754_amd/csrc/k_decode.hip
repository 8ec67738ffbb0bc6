// Decode-step attention over the compressed layer cache (Sec. 2 decoding step under the mask of
// Sec. 3): one query token per sequence, the G query heads of a KV group share the group's
// retained rows, which sit packed and variable-length per head as the selection wrote them.
//
//   decode_kernel   one workgroup per "unit" = up to C consecutive rows of one head (packed rows
//                   first, then the rows appended since the eviction).  Each wavefront streams
//                   32-row K and V tiles alternately through its private tile ring:
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

template <int DT, int D>
struct DecShape {
  using T = Tile<DT, D>;
  static constexpr int kStagesRaw = (128 * 1024) / (kDecWaves * T::kTileBytes);
  static constexpr int kStages = kStagesRaw > kMaxRingStages ? kMaxRingStages : kStagesRaw;
  static_assert(kStages >= 2, "ring needs a K and a V stage");
  static constexpr int kBpl = T::kRowBytes / 64;              // bytes of a row one lane owns
  static constexpr int kDpl = kBpl / Elem<DT>::kBytes;        // elements of a row one lane owns
  static_assert(kDpl == 1 || kDpl == 2, "one or two output columns per lane");
};

__device__ __forceinline__ void wait_lds() { __builtin_amdgcn_s_waitcnt(0xc07f); }   // lgkmcnt(0)

// What the lanes of one wavefront wrote to LDS is visible to its other lanes after this.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The kDpl elements of row `row` this lane owns, as floats.  voff[j] is the lane's byte offset
// inside a row whose (row & 7) == j (the tile is XOR-swizzled in 16-byte chunks).
template <int DT, int D>
__device__ __forceinline__ void read_v(const char* __restrict__ stage, int row, const unsigned int (&voff)[8],
                                       float (&x)[DecShape<DT, D>::kDpl]) {
  using S = DecShape<DT, D>;
  const char* p = stage + row * S::T::kRowBytes + voff[row & 7];
  if constexpr (DT == LAVA_BF16 && S::kDpl == 1) {
    x[0] = __uint_as_float((unsigned int)(*reinterpret_cast<const unsigned short*>(p)) << 16);
  } else if constexpr (DT == LAVA_BF16) {
    const unsigned int b = *reinterpret_cast<const unsigned int*>(p);
    x[0] = __uint_as_float(b << 16);
    x[1] = __uint_as_float(b & 0xffff0000u);
  } else if constexpr (S::kDpl == 1) {
    x[0] = *reinterpret_cast<const float*>(p);
  } else {
    const float2 f = *reinterpret_cast<const float2*>(p);
    x[0] = f.x;
    x[1] = f.y;
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

// Units of head g: packed chunks, then tail chunks.
__device__ __forceinline__ long long head_len(const long long* __restrict__ off, int g) {
  const long long len = off[g + 1] - off[g];
  return len > 0 ? len : 0;
}

// Offsets a kernel may follow: start at >= 0, never decrease, end within the stated capacity.
__device__ __forceinline__ bool offsets_usable(const long long* __restrict__ off, int n_heads, long long capacity) {
  bool ok = off[0] >= 0 && off[n_heads] <= capacity;
  for (int g = 0; g < n_heads; ++g) ok = ok && off[g + 1] >= off[g];
  return ok;
}

template <int DT, int D, int GP>
__global__ void __launch_bounds__(kDecThreads) decode_kernel(DecodeArgs a) {
  using S = DecShape<DT, D>;
  using T = Tile<DT, D>;
  constexpr int kStages = S::kStages;
  constexpr int kDpl = S::kDpl;
  __shared__ u32x4 s_tile[kDecWaves][kStages][T::kTileChunks];
  __shared__ float s_p[kDecWaves][kTileKeys + 1][GP];      // probabilities of the tile; row 32: rescale factors
  __shared__ float s_acc[kDecWaves][GP][D];
  __shared__ float s_m[kDecWaves][GP], s_l[kDecWaves][GP];

  const int lane = threadIdx.x & 63, wave = wave_index();
  const int b = blockIdx.y;
  const long long* off = a.head_offsets + (long long)b * (a.H_kv + 1);
  const long long tail_units = a.tail_len > 0 ? ceil_div(a.tail_len, a.rows_per_unit) : 0;
  if (!offsets_usable(off, a.H_kv, a.rows_capacity)) return;   // the merge reports it

  // which head and chunk this unit is (wave-uniform scalar loop over at most 64 heads)
  long long u = blockIdx.x;
  int g = 0;
  long long packed_units = 0;
  for (; g < a.H_kv; ++g) {
    packed_units = ceil_div(head_len(off, g), a.rows_per_unit);
    if (u < packed_units + tail_units) break;
    u -= packed_units + tail_units;
  }
  if (g >= a.H_kv) return;                                  // beyond the sequence's last unit

  const char* kb;
  const char* vb;
  long long n_rows;
  if (u < packed_units) {
    const long long base = (a.seq_base ? a.seq_base[b] : (long long)b * a.rows_capacity) + off[g] +
                           u * a.rows_per_unit;
    n_rows = head_len(off, g) - u * a.rows_per_unit;
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

  // the group's query rows as the 32-column operand: column t < G is head g*G + t
  const int col = lane & 31, half = lane >> 5;
  u32x4 qf[T::kSteps];
#pragma unroll
  for (int j = 0; j < T::kSteps; ++j) {
    u32x4 x = u32x4{0u, 0u, 0u, 0u};
    if (col < a.G) x = a.q[((long long)b * a.H + (long long)g * a.G + col) * T::kCpr + 2 * j + half];
    qf[j] = x;
  }
  TileDma<DT, D> dma;
  dma.init(lane);
  unsigned int voff[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const unsigned int byte = (unsigned int)lane * S::kBpl;
    voff[j] = (((byte >> 4) ^ (unsigned int)j) << 4) | (byte & 15u);
  }
  wait_vmcnt<0>();                                          // the ring counts its own loads only

  float m_run = -INFINITY, l_run = 0.0f;                    // of head `col` (lanes col < G)
  float acc[GP][kDpl];
#pragma unroll
  for (int t = 0; t < GP; ++t)
#pragma unroll
    for (int e = 0; e < kDpl; ++e) acc[t][e] = 0.0f;

  // ring items of this wavefront: K tile j0, V tile j0, K tile j0 + kDecWaves, ...
  const long long n_tiles = ceil_div(n_rows, kTileKeys);
  const int cnt = wave < n_tiles ? (int)((n_tiles - wave + kDecWaves - 1) / kDecWaves) : 0;
  const int n_items = 2 * cnt;
  u32x4* ring = s_tile[wave][0];
  auto issue_item = [&](int item) {
    const long long tile = wave + (long long)(item >> 1) * kDecWaves;
    dma.issue((item & 1) ? vb : kb, tile, n_rows, lane, ring + (item % kStages) * T::kTileChunks);
  };
#pragma unroll
  for (int p = 0; p < kStages - 1; ++p)
    if (p < n_items) issue_item(p);

  for (int it = 0; it < cnt; ++it) {
    const long long tile = wave + (long long)it * kDecWaves;
    // ---------------- K tile: logits, online softmax, probabilities to LDS
    {
      const int item = 2 * it;
      wait_lds();                                           // reads of the stage about to be refilled are done
      if (item + kStages - 1 < n_items) issue_item(item + kStages - 1);
      const int younger = n_items - 1 - item < kStages - 1 ? n_items - 1 - item : kStages - 1;
      wait_tile<DT, D>(younger);
      u32x4 kf[T::kSteps];
      lds_to_frag<DT, D>(ring + (item % kStages) * T::kTileChunks, lane, kf);
      asm volatile("" ::: "memory");
      f32x16 x = dot_tile<DT, D, true>(kf, qf);             // x[v]: key 8*(v/4) + 4*half + v%4, head col
      const long long key0 = tile * kTileKeys;
      const bool ragged = key0 + kTileKeys > n_rows;
      float mt = -INFINITY;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float s = x[v] * a.c2;
        if (ragged && key0 + 8 * (v / 4) + 4 * half + (v % 4) >= n_rows) s = -INFINITY;
        x[v] = s;
        mt = fmaxf(mt, s);
      }
      mt = fmaxf(mt, __shfl_xor(mt, 32));
      const float m_new = fmaxf(m_run, mt);                 // finite: a tile holds at least one row
      const float alpha = fast_exp2(m_run - m_new);
      float ls = 0.0f;
      if (col < GP) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = fast_exp2(x[v] - m_new);
          ls += p;
          s_p[wave][8 * (v / 4) + 4 * half + (v % 4)][col] = p;
        }
        if (half == 0) s_p[wave][kTileKeys][col] = alpha;
      }
      l_run = l_run * alpha + ls;
      m_run = m_new;
    }
    wave_lds_sync();
    // ---------------- V tile: rescale, accumulate
    {
      const int item = 2 * it + 1;
      wait_lds();
      if (item + kStages - 1 < n_items) issue_item(item + kStages - 1);
      const int younger = n_items - 1 - item < kStages - 1 ? n_items - 1 - item : kStages - 1;
      wait_tile<DT, D>(younger);
      const char* stage = reinterpret_cast<const char*>(ring + (item % kStages) * T::kTileChunks);
#pragma unroll
      for (int t = 0; t < GP; ++t) {
        const float al = s_p[wave][kTileKeys][t];
#pragma unroll
        for (int e = 0; e < kDpl; ++e) acc[t][e] *= al;
      }
#pragma unroll
      for (int kk = 0; kk < kTileKeys; ++kk) {
        float vx[kDpl];
        read_v<DT, D>(stage, kk, voff, vx);
#pragma unroll
        for (int t = 0; t < GP; ++t) {
          const float p = s_p[wave][kk][t];
#pragma unroll
          for (int e = 0; e < kDpl; ++e) acc[t][e] = fmaf(p, vx[e], acc[t][e]);
        }
      }
      asm volatile("" ::: "memory");
    }
    wave_lds_sync();                                        // next tile's probabilities overwrite s_p
  }

  // ---------------- merge the wavefronts of the unit
  l_run += __shfl_xor(l_run, 32);
  if (lane < GP) {
    s_m[wave][lane] = m_run;
    s_l[wave][lane] = l_run;
  }
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

// One workgroup per (KV head, sequence): merge the head's units in unit order.
template <int D, int GP>
__global__ void __launch_bounds__(256) decode_merge_kernel(DecodeArgs a, float* __restrict__ out,
                                                           float* __restrict__ lse) {
  const int b = blockIdx.y, g = blockIdx.x;
  const long long* off = a.head_offsets + (long long)b * (a.H_kv + 1);
  const long long tail_units = a.tail_len > 0 ? ceil_div(a.tail_len, a.rows_per_unit) : 0;
  long long first = 0, total = 0, mine = 0;
  for (int gg = 0; gg < a.H_kv; ++gg) {
    const long long c = ceil_div(head_len(off, gg), a.rows_per_unit) + tail_units;
    if (gg < g) first += c;
    if (gg == g) mine = c;
    total += c;
  }
  const bool overflow = total > a.units_bound || !offsets_usable(off, a.H_kv, a.rows_capacity);
  const float2* ml = a.part_ml + ((long long)b * a.units_bound + first) * GP;
  const float* pa = a.part_acc + ((long long)b * a.units_bound + first) * GP * D;
  for (int idx = threadIdx.x; idx < a.G * D; idx += 256) {
    const int t = idx / D, e = idx % D;
    float result = 0.0f, lse_v = -INFINITY;
    if (overflow) {
      result = lse_v = NAN;
    } else if (mine > 0) {
      float M = -INFINITY;
      for (long long i = 0; i < mine; ++i) M = fmaxf(M, ml[i * GP + t].x);
      float L = 0.0f, sum = 0.0f;
      for (long long i = 0; i < mine; ++i) {
        const float2 s = ml[i * GP + t];
        const float wgt = fast_exp2(s.x - M);
        L += wgt * s.y;
        sum += wgt * pa[(i * GP + t) * D + e];
      }
      result = sum / L;
      lse_v = (M + log2f(L)) * 0.6931471805599453f;
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
  int64_t c = (total / (4 * (int64_t)device_cus()) + step - 1) / step * step;
  if (c < step) c = step;
  if (c > 8 * step) c = 8 * step;
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
