// Wavefront-private tile ring shared by the kernels that stream a cache through the matrix cores.
//
// A 32-row tile of one head is a contiguous span of HBM.  It travels HBM -> LDS with coalesced
// 128-bit direct-to-LDS loads (no staging registers) into a ring of XOR-swizzled buffers owned by
// one wavefront, several tiles ahead of the one being consumed; arrival of a tile is a vmcnt wait
// that leaves the younger tiles in flight, so a sweep needs no workgroup barrier.  The tile is
// then read in MFMA operand layout.
//
// MFMA 32x32 layouts (wave64): operand lane l supplies row/column l%32 and k-slice l/32; result
// register v of lane l is element (8*(v/4) + 4*(l/32) + v%4, l%32).
#pragma once

#include <hip/hip_runtime.h>

#include <utility>

#include "common.h"

namespace lava {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes held in registers

constexpr float kLog2e = 1.4426950408889634f;

template <int DT> struct Elem;
template <> struct Elem<LAVA_BF16> { static constexpr int kBytes = 2; };
template <> struct Elem<LAVA_F32> { static constexpr int kBytes = 4; };

// acc += A(16 bytes of k) x B(16 bytes of k).  Both operands use the same lane -> k mapping, so
// any fixed assignment of a row's elements to (step, lane half) gives the full dot product.
template <int DT>
__device__ __forceinline__ f32x16 mfma_chunk(const u32x4& a, const u32x4& b, f32x16 acc) {
  if constexpr (DT == LAVA_BF16) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
  } else {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
    return acc;
  }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

#define LAVA_GLOBAL_AS __attribute__((address_space(1)))
#define LAVA_LDS_AS __attribute__((address_space(3)))

// Wait until at most N vector-memory operations of this wavefront are still outstanding.  Loads
// complete in issue order, so this guarantees every load older than the N youngest has landed.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
  asm volatile("" ::: "memory");
}

// (m1, z1) (+) (m2, z2) for sums of exp2((x - m) * c2); empty sets are (-inf, 0).
__device__ __forceinline__ void merge_stat(float& m, float& z, float m2, float z2, float c2) {
  const float mn = fmaxf(m, m2);
  const float f1 = (m == mn) ? 1.0f : fast_exp2((m - mn) * c2);
  const float f2 = (m2 == mn) ? 1.0f : fast_exp2((m2 - mn) * c2);
  z = z * f1 + z2 * f2;
  m = mn;
}

template <int DT, int D>
struct Tile {
  static constexpr int kRowBytes = D * Elem<DT>::kBytes;
  static constexpr int kCpr = kRowBytes / 16;          // 16-byte chunks per row
  static constexpr int kSteps = kCpr / 2;              // chunk steps (two lane halves per step)
  static constexpr int kLoads = kTileKeys * kCpr / 64; // 128-bit loads per lane per tile
  static constexpr int kTileChunks = kTileKeys * kCpr;
  static constexpr int kTileBytes = kTileKeys * kRowBytes;
};

// Direct-to-LDS reads of 32-key tiles into a ring stage.  Instruction i moves 1 KiB: lane l lands
// at chunk slot i*64 + l of the stage, i.e. row (i*64+l)/kCpr, slot s = (i*64+l)%kCpr, and fetches
// the row's chunk s ^ (row & 7): the swizzle is applied on the global side because the LDS side
// of such a load is linear.  The per-lane byte offsets inside a tile are computed once; a full tile
// is then (wave-uniform tile address) + (per-lane offset), which needs no vector arithmetic.
template <int DT, int D>
struct TileDma {
  using T = Tile<DT, D>;
  static constexpr int kRowsPerLoad = 64 / T::kCpr;                                // rows one instruction covers
  static constexpr int kVariants = kRowsPerLoad >= 8 ? 1 : 8 / kRowsPerLoad;        // distinct (row & 7) patterns
  unsigned int loff[kVariants];   // per-lane byte offset inside the 1 KiB slice of load i, variant i % kVariants

  __device__ __forceinline__ void init(int lane) {
#pragma unroll
    for (int i = 0; i < kVariants; ++i) {
      const int q = i * 64 + lane;
      const int row = q / T::kCpr, slot = q % T::kCpr;
      loff[i] = (unsigned int)((row - i * kRowsPerLoad) * T::kRowBytes + ((slot ^ (row & 7)) << 4));
    }
  }

  // Every row of the tile exists.  Load i covers bytes [i KiB, (i+1) KiB) of the tile on both sides;
  // the common part of the offset is an instruction immediate (< 4 KiB) applied to the global and
  // the LDS address alike, plus a scalar 4 KiB step, so a load costs no vector arithmetic.
  __device__ __forceinline__ void issue_full(const char* __restrict__ tile_base, u32x4* stage) const {
#pragma unroll
    for (int i = 0; i < T::kLoads; ++i) {
      const char* src = tile_base + (i / 4) * 4096 + loff[i % kVariants];
      u32x4* dst = stage + (i / 4) * 256;
      switch (i % 4) {
        case 0: __builtin_amdgcn_global_load_lds((const LAVA_GLOBAL_AS void*)src, (LAVA_LDS_AS void*)dst, 16, 0, 0); break;
        case 1: __builtin_amdgcn_global_load_lds((const LAVA_GLOBAL_AS void*)src, (LAVA_LDS_AS void*)dst, 16, 1024, 0); break;
        case 2: __builtin_amdgcn_global_load_lds((const LAVA_GLOBAL_AS void*)src, (LAVA_LDS_AS void*)dst, 16, 2048, 0); break;
        default: __builtin_amdgcn_global_load_lds((const LAVA_GLOBAL_AS void*)src, (LAVA_LDS_AS void*)dst, 16, 3072, 0); break;
      }
    }
  }

  // rows at or beyond n are read from row n - 1 (callers mask or drop them)
  __device__ __forceinline__ void issue_clamped(const char* __restrict__ head_base, long long tile,
                                                long long n, int lane, u32x4* stage) const {
    // This path runs once per sweep.  The lane index goes through an opaque move so that nothing
    // derived from it is computed ahead of the hot loop and kept in registers across it.
    asm volatile("" : "+v"(lane));
    const char* tile_base = head_base + tile * T::kTileBytes;
    const int last = (int)(n - 1 - tile * kTileKeys);      // last existing row of the tile, 0 .. 30
#pragma unroll
    for (int i = 0; i < T::kLoads; ++i) {
      const int q = i * 64 + lane;
      const int row = q / T::kCpr, slot = q % T::kCpr;
      const int src_row = row < last ? row : last;
      const char* src = tile_base + (unsigned int)(src_row * T::kRowBytes + ((slot ^ (row & 7)) << 4));
      __builtin_amdgcn_global_load_lds((const LAVA_GLOBAL_AS void*)src, (LAVA_LDS_AS void*)(stage + i * 64), 16,
                                       0, 0);
    }
  }

  __device__ __forceinline__ void issue(const char* __restrict__ head_base, long long tile, long long n,
                                        int lane, u32x4* stage) const {
    if ((tile + 1) * kTileKeys <= n) {
      issue_full(head_base + tile * T::kTileBytes, stage);
    } else {
      issue_clamped(head_base, tile, n, lane, stage);
    }
  }
};

// Wait for the oldest tile of a ring while `younger` (0 .. kMaxRingStages-1) tiles stay in flight.
constexpr int kMaxRingStages = 4;
template <int DT, int D>
__device__ __forceinline__ void wait_tile(int younger) {
  using T = Tile<DT, D>;
  switch (younger) {
    case 0: wait_vmcnt<0>(); break;
    case 1: wait_vmcnt<T::kLoads>(); break;
    case 2: wait_vmcnt<2 * T::kLoads>(); break;
    default: wait_vmcnt<3 * T::kLoads>(); break;
  }
}

// ------------------------------------------------------------------------------------------
// LDS accesses written as instructions.
//
// While direct-to-LDS loads are in flight the compiler cannot tell which LDS bytes they will
// write, so before EVERY ordinary LDS access it waits for all of them (vmcnt(0)), which turns the
// ring into one tile in flight per wavefront.  The ring protocol already guarantees that a stage
// is only read after its own loads have landed (wait_tile) and only refilled after its reads have
// returned (lds_reads_done), so the LDS accesses inside a sweep are issued as instructions the
// compiler does not reason about.  Each read helper ends with its own wait: its results are valid
// on return.  Addresses are LDS byte offsets (lds_addr).
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned int lds_addr(const void* p) {
  return (unsigned int)(unsigned long long)(LAVA_LDS_AS const char*)p;
}

// every LDS operation this wavefront has issued is complete
__device__ __forceinline__ void lds_reads_done() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

__device__ __forceinline__ void lds_read128x4(unsigned int a0, unsigned int a1, unsigned int a2, unsigned int a3,
                                              u32x4& o0, u32x4& o1, u32x4& o2, u32x4& o3) {
  asm volatile(
      "ds_read_b128 %0, %4\n\t"
      "ds_read_b128 %1, %5\n\t"
      "ds_read_b128 %2, %6\n\t"
      "ds_read_b128 %3, %7\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3)
      : "v"(a0), "v"(a1), "v"(a2), "v"(a3)
      : "memory");
}

// Offsets known at compile time travel in the instruction (16-bit field), so that one address
// register serves every access of a loop instead of one hoisted register per access.
// four reads at byte offsets OFF, OFF + STRIDE, OFF + 2*STRIDE, OFF + 3*STRIDE from one address
template <int STRIDE, int OFF = 0>
__device__ __forceinline__ void lds_read128x4_strided(unsigned int a, u32x4& o0, u32x4& o1, u32x4& o2, u32x4& o3) {
  static_assert(OFF >= 0 && OFF + 3 * STRIDE < 65536, "LDS instruction offset field");
  asm volatile(
      "ds_read_b128 %0, %4 offset:%5\n\t"
      "ds_read_b128 %1, %4 offset:%6\n\t"
      "ds_read_b128 %2, %4 offset:%7\n\t"
      "ds_read_b128 %3, %4 offset:%8\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3)
      : "v"(a), "n"(OFF), "n"(OFF + STRIDE), "n"(OFF + 2 * STRIDE), "n"(OFF + 3 * STRIDE)
      : "memory");
}

// four reads at one compile-time offset from four addresses
template <int OFF>
__device__ __forceinline__ void lds_read128x4_at(unsigned int a0, unsigned int a1, unsigned int a2, unsigned int a3,
                                                 u32x4& o0, u32x4& o1, u32x4& o2, u32x4& o3) {
  static_assert(OFF >= 0 && OFF < 65536, "LDS instruction offset field");
  asm volatile(
      "ds_read_b128 %0, %4 offset:%8\n\t"
      "ds_read_b128 %1, %5 offset:%8\n\t"
      "ds_read_b128 %2, %6 offset:%8\n\t"
      "ds_read_b128 %3, %7 offset:%8\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3)
      : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "n"(OFF)
      : "memory");
}

template <int OFF>
__device__ __forceinline__ void lds_read128_at(unsigned int a, u32x4& o) {
  static_assert(OFF >= 0 && OFF < 65536, "LDS instruction offset field");
  asm volatile("ds_read_b128 %0, %1 offset:%2\n\ts_waitcnt lgkmcnt(0)" : "=&v"(o) : "v"(a), "n"(OFF) : "memory");
}

template <int OFF>
__device__ __forceinline__ void lds_write32_at(unsigned int a, float x) {
  static_assert(OFF >= 0 && OFF < 65536, "LDS instruction offset field");
  asm volatile("ds_write_b32 %0, %1 offset:%2" : : "v"(a), "v"(x), "n"(OFF) : "memory");
}

// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}): a loop whose
// index is a constant expression inside the body
template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

__device__ __forceinline__ void lds_read128(unsigned int a, u32x4& o) {
  asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(o) : "v"(a) : "memory");
}

// *a += 1 in LDS, returns the value before.  Call from ONE lane.
__device__ __forceinline__ unsigned int lds_fetch_inc(unsigned int a) {
  unsigned int v;
  const unsigned int one = 1u;
  asm volatile("ds_add_rtn_u32 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(a), "v"(one) : "memory");
  return v;
}

__device__ __forceinline__ void lds_write32(unsigned int a, float x) {
  asm volatile("ds_write_b32 %0, %1" : : "v"(a), "v"(x) : "memory");
}

// Per-lane addresses of a tile's MFMA operand fragments: lane l holds row l % 32 and, at step j,
// the row's 16-byte chunk 2j + l/32 (stored at slot chunk ^ (row & 7)).
template <int DT, int D>
struct FragReader {
  using T = Tile<DT, D>;
  unsigned int foff[T::kSteps];

  __device__ __forceinline__ void init(int lane) {
    const int row = lane & 31, half = lane >> 5;
#pragma unroll
    for (int j = 0; j < T::kSteps; ++j) foff[j] = (unsigned int)((row * T::kCpr + ((2 * j + half) ^ (row & 7))) << 4);
  }

  // Variant for a ring whose stage is known at compile time: init_at folds the ring's address into
  // the per-lane offsets once, read_at<OFF> then needs no address arithmetic at all.
  __device__ __forceinline__ void init_at(int lane, unsigned int ring) {
    init(lane);
#pragma unroll
    for (int j = 0; j < T::kSteps; ++j) foff[j] += ring;
  }
  template <int OFF>
  __device__ __forceinline__ void read_at(u32x4 (&frag)[T::kSteps]) const {
#pragma unroll
    for (int j = 0; j < T::kSteps; j += 4)
      lds_read128x4_at<OFF>(foff[j], foff[j + 1], foff[j + 2], foff[j + 3], frag[j], frag[j + 1], frag[j + 2],
                            frag[j + 3]);
  }

  // `stage`: LDS byte address of the ring stage.  The fragments are in registers on return.
  __device__ __forceinline__ void read(unsigned int stage, u32x4 (&frag)[T::kSteps]) const {
    static_assert(T::kSteps % 4 == 0, "fragments are read four at a time");
#pragma unroll
    for (int j = 0; j < T::kSteps; j += 4)
      lds_read128x4(stage + foff[j], stage + foff[j + 1], stage + foff[j + 2], stage + foff[j + 3], frag[j],
                    frag[j + 1], frag[j + 2], frag[j + 3]);
  }
};

// The matrix cores take 32 query rows at a time, so a head whose window has more than 32 rows is
// handled as `bph` (1 or 2) row blocks of 32: block index hb = head * bph + block, rows block * 32 ..
// Everything up to the point where a head's window rows are summed treats a row block as a head.
//
// Query fragments of the chunk's row blocks hb0 .. hb0 + nh - 1, one copy per wavefront straight from
// global memory: row r = lane % 32 of the block (zero beyond the window or the chunk).
template <int DT, int D, int GT>
__device__ __forceinline__ void load_q(const u32x4* __restrict__ qg, int hb0, int nh, int w, int bph, int lane,
                                       u32x4 (&qf)[GT][Tile<DT, D>::kSteps]) {
  using T = Tile<DT, D>;
  const int r = lane & 31, half = lane >> 5;
#pragma unroll
  for (int t = 0; t < GT; ++t) {
    const int head = (hb0 + t) / bph, row = ((hb0 + t) % bph) * 32 + r;
#pragma unroll
    for (int j = 0; j < T::kSteps; ++j) {
      u32x4 x = u32x4{0u, 0u, 0u, 0u};
      if (t < nh && row < w) x = qg[((long long)head * w + row) * T::kCpr + 2 * j + half];
      qf[t][j] = x;
    }
  }
}

// Query rows of the chunk's row blocks, copied once per workgroup into tile-shaped LDS buffers (one per
// block: row r of block t at row r, 16-byte chunks swizzled like a key tile, zero beyond the window
// or the chunk), from where every wavefront reads them as fragments with FragReader.  Letting each
// wavefront fetch its own copy from global memory costs kWaves times the traffic on a handful of
// cache lines that every workgroup of the grid wants at the same moment.
// bufs(t) returns the buffer of head t.  The caller synchronises the workgroup afterwards.
template <int DT, int D, int GT, int THREADS, class BUFS>
__device__ __forceinline__ void stage_q(const u32x4* __restrict__ qg, int hb0, int nh, int w, int bph, BUFS&& bufs) {
  using T = Tile<DT, D>;
  constexpr int kPerHead = kTileKeys * T::kCpr;
  constexpr int kTotal = GT * kPerHead;
#pragma unroll
  for (int i = 0; i < (kTotal + THREADS - 1) / THREADS; ++i) {
    const int c = i * THREADS + (int)threadIdx.x;
    if (kTotal % THREADS != 0 && c >= kTotal) break;
    const int t = c / kPerHead, rr = (c / T::kCpr) % kTileKeys, ch = c % T::kCpr;
    u32x4 x = u32x4{0u, 0u, 0u, 0u};
    const int head = (hb0 + t) / bph, row = ((hb0 + t) % bph) * 32 + rr;
    if (t < nh && row < w) x = qg[((long long)head * w + row) * T::kCpr + ch];
    bufs(t)[rr * T::kCpr + (ch ^ (rr & 7))] = x;
  }
}

// One head's 32 x 32 block of raw dot products: keys x rows (KEYS_AS_ROWS) or rows x keys.
template <int DT, int D, bool KEYS_AS_ROWS>
__device__ __forceinline__ f32x16 dot_tile(const u32x4 (&kf)[Tile<DT, D>::kSteps],
                                           const u32x4 (&qh)[Tile<DT, D>::kSteps]) {
  f32x16 acc = {0};
#pragma unroll
  for (int j = 0; j < Tile<DT, D>::kSteps; ++j)
    acc = KEYS_AS_ROWS ? mfma_chunk<DT>(kf[j], qh[j], acc) : mfma_chunk<DT>(qh[j], kf[j], acc);
  return acc;
}

// Index of the wavefront inside its workgroup as a scalar, so that everything derived from it
// (tile numbers, ring stages, loop bounds) stays in scalar registers and scalar branches.
__device__ __forceinline__ int wave_index() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

}  // namespace lava
