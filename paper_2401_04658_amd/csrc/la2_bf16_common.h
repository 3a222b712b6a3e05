// Shared pieces of the 16-bit (bf16 / fp16) MFMA kernels (gfx950): vector types, MFMA and LDS helpers, the swizzled tile
// layout, direct HBM -> LDS tile loads, the state <-> accumulator mapping and the update weights.
//
// The scan kernels: one workgroup (4 waves) walks the blocks (B = 64 positions) of one sequence chunk of one
// (batch, head) chain.  The X, Y, Z tiles of the NEXT block stream from HBM straight into LDS
// (global_load_lds, no registers), two blocks ahead of the block being computed (three tile buffers).
//
// Work split: wave w owns the 32 value features dv = 32 (w % NT) .. +31 (NT = D / 32) of the output
// and of the running state, for all key features.  Its slice S[:, dv] of the fp32 state never
// leaves its MFMA accumulator registers: the inter-block product reads it as an MFMA operand
// straight from those registers, so the state needs no LDS copy and no extra workgroup barrier.
// For d = 128 a wave covers both 32-row tiles of the block; for d = 64 two waves share a value tile,
// one row tile each (and keep identical copies of the state slice).  Every wave computes the masked
// score tiles it needs itself, so the scores never leave registers either.  One barrier per block.
//
// MFMA 32x32x16 (v_mfma_f32_32x32x16_bf16) lane layouts (wave64, lane l, l32 = l % 32, hh = l / 32):
//   A[m][k]: m = l32, k = 8 hh + j (j = 0..7)     B[k][n]: n = l32, k = 8 hh + j
//   C[m][n]: n = l32, m = 8 (v / 4) + 4 hh + v % 4 (v = 0..15)
// An accumulator tile C[m][n] is reused as an operand with n as the lane index and m as the
// contraction index: elements v = 8 q + j (j = 0..7) of a lane are the contraction indices
//   perm(q, hh, j) = 16 q + 8 (j / 4) + 4 hh + j % 4
// of one 16-wide k-step.  The other operand of such a product is read in the same order
// ("permuted k-order"); because both operands agree the result is unaffected.
// Outputs are accumulated TRANSPOSED (C rows = value feature, C columns = position) so that each
// lane ends up with 4 consecutive features of one position, which packs into 8-byte LDS writes.
//
// Tile layout in LDS: row-major, UNPADDED (the direct loads write 1 KiB contiguous per wave
// instruction), with the 16-byte chunk index of every row XOR-swizzled by swz(row) so that both the
// 16-byte row reads (lanes = rows) and the transposing reads (4 rows x 64 bytes per 32 lanes) are
// bank-conflict free.
#ifndef LA2_BF16_COMMON_H_
#define LA2_BF16_COMMON_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "la2_internal.h"

namespace la2 {
namespace bf16k {


// 16-bit element types: __bf16 (LA2_BF16) and _Float16 (LA2_F16).  Every kernel is a template over the
// element type E; only the conversions to and from fp32 and the MFMA instruction depend on it.
template <typename E> using ex8 = E __attribute__((ext_vector_type(8)));
template <typename E> using ex4 = E __attribute__((ext_vector_type(4)));
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int kB = 64;        // block size (positions per block)
constexpr int kThreads = 256; // 4 waves

template <int D, int B = kB>
struct Cfg {
  static constexpr int KS = D / 16;            // MFMA k-steps along a feature dimension
  static constexpr int NT = D / 32;            // 32-wide tiles along a feature dimension
  static constexpr int WPD = NT >= 4 ? 1 : 4 / NT;   // waves sharing one value-feature tile (1 or 2)
  static constexpr int RT = 2 / WPD;           // 32-row tiles of the block per wave (2 or 1)
  static constexpr int CPR = D / 8;            // 16-byte chunks per tile row
  static constexpr int TILE = B * D;           // elements per tile
  static constexpr int DMA_PER_TILE = TILE / 512;   // wave instructions (1 KiB each) per tile
  static constexpr int DMA_PER_WAVE = DMA_PER_TILE / 4;
  static constexpr int LW = 32;                // staging row: 32 features = 64 bytes, unpadded, 16-byte chunks
                                               // XOR-swizzled by (row / 4) % 4 (LDS is full: no room for padding)
};

__device__ __forceinline__ f32x16 mfma(ex8<__bf16> a, ex8<__bf16> b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma(ex8<_Float16> a, ex8<_Float16> b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// MFMA 16x16x32: A 16 x 32 (lane l: row l % 16, k = 8 (l / 16) .. + 7), B 32 x 16 (column l % 16, same k),
// D 16 x 16 (column l % 16, rows 4 (l / 16) .. + 3).
__device__ __forceinline__ f32x4 mfma16(ex8<__bf16> a, ex8<__bf16> b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma16(ex8<_Float16> a, ex8<_Float16> b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// 2^x for x <= 0 with the bare hardware instruction (no denormal-range fix-up: results below
// 2^-126 flush to 0, which is where these decay weights are negligible anyway).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int v = 0; v < 16; v++) z[v] = 0.f;
  return z;
}

// Raw buffer descriptor over one chain's rows: stores beyond `bytes` are dropped, which is how the
// rows of a ragged last block are masked on output without branches.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00027000);
}

// Transposing LDS read.  Within each group of 16 lanes, lane s passes the address of 4 consecutive
// elements of row (s / 4), columns 4 (s % 4) .. +3 of a 4 x 16 sub-matrix; lane s receives the 4
// rows of column s.
__device__ __forceinline__ s16x4 lds_read_tr(const void* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
}

// Physical 16-byte chunk of logical chunk c in tile row `row`: c ^ swz<D>(row).
template <int D>
__device__ __forceinline__ int swz(int row) {
  // m = index of the 256-byte LDS line the row starts in (d=128: one row per line, d=64: two).
  // d=128: ((m & 3) << 2) | ((m >> 2) & 3);  d=64: ((m & 1) << 2) | ((m >> 1) & 3).
  // - 16 consecutive rows reading the same logical chunk (16-byte row reads, 16 lanes per cycle)
  //   land in 16 different 16-byte bank groups;
  // - 4 consecutive rows x 4 consecutive chunks (transposing reads, 32 lanes per cycle) likewise.
  // Depends on row % 16 only.
  // d=256 (two lines per row): as d=128.  d=96 (12 chunks per row, rows 192 bytes apart): (row >> 2) & 3, which
  // keeps a chunk inside its aligned group of four and still spreads 16 consecutive rows over the 16 groups.
  if (D == 128 || D == 256) return ((row & 3) << 2) | ((row >> 2) & 3);
  if (D == 96) return (row >> 2) & 3;
  const int m = row >> 1;
  return ((m & 1) << 2) | ((m >> 1) & 3);
}

// Workgroup barrier that orders LDS traffic only: waits for this wave's outstanding LDS operations
// and then joins the barrier, WITHOUT waiting for vector-memory operations.  __syncthreads() would
// also drain vmcnt, i.e. stall on the direct loads of the next block that are meant to stay in
// flight.  The "memory" clobber keeps the compiler from moving LDS accesses across it.  Waves that
// need their own direct loads visible wait for vmcnt(0) before calling this.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Direct global -> LDS copy, 16 bytes per lane: lane i reads base + voff (its own byte offset) and
// writes LDS byte address lds_base + 16 i (lds_base is wave-uniform and travels in M0).  The tiles are
// read exactly once, so the load carries the non-temporal hint (measured 5-10 % faster).
// Written as inline assembly on purpose: the compiler then keeps no record of an asynchronous LDS
// write and inserts no vmcnt(0) wait in front of later LDS reads (it cannot always prove that they
// touch a different tile buffer).  Completion is tracked by hand: see the s_waitcnt at the end of
// each block, followed by the workgroup barrier.
__device__ __forceinline__ void dma16(const void* base, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
               :
               : "v"(voff), "s"(base), "s"(lds_base)
               : "m0", "memory");
}

__device__ __forceinline__ uint32_t lds_offset(const void* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// Exchange between lanes l and l + 32 that turns a row fragment in natural k-order (this lane holds
// features 8 hh .. 8 hh + 7 of a 16-wide k-step) into permuted k-order (features 4 hh .. 4 hh + 3 and
// 8 + 4 hh .. 8 + 4 hh + 3).  v_permlane32_swap(a, b): lanes >= 32 of a <-> lanes < 32 of b.
template <typename V>
__device__ __forceinline__ V to_perm_order(V f) {
  static_assert(sizeof(V) == 16, "eight 16-bit elements");
  union { V v; u32x4 u; } x;
  x.v = f;
  const u32x2 s0 = __builtin_amdgcn_permlane32_swap(x.u[0], x.u[2], false, false);
  const u32x2 s1 = __builtin_amdgcn_permlane32_swap(x.u[1], x.u[3], false, false);
  x.u[0] = s0[0]; x.u[1] = s1[0]; x.u[2] = s0[1]; x.u[3] = s1[1];
  return x.v;
}

// Pins a value to this point of the program: an empty volatile asm that "rewrites" the register.
// Arithmetic and MFMA intrinsics have no side effects, so instruction selection may place them
// anywhere between their operands and their first use, across scheduling barriers.  Volatile asm
// statements keep their order, so a value pinned at the end of a slot is computed inside that slot,
// and everything computed from the pinned value comes later.
template <typename T>
__device__ __forceinline__ void pin(T& x) {
  asm volatile("" : "+v"(x));
}

// The same for a value that is only ever an MFMA operand, placed right before its use: it has to be
// in an accumulation register there.  LDS reads can target those directly, which keeps such operands
// out of the (scarcer) registers that the vector ALU can address.
template <typename T>
__device__ __forceinline__ void pin_acc(T& x) {
  asm volatile("" : "+a"(x));
}

// Per-lane addressing of the swizzled tiles.
template <int D>
struct LaneAddr {
  int rowk;         // 16-byte row reads: logical chunk 2 ks + hh of row 32 t + l32 sits at element
                    // 32 t D + (rowk ^ 16 ks)                    [swz(32 t + l32) == swz(l32)]
  int tr0, tr1;     // transposing reads in permuted k-order: rows c0 + 4 hh + s / 4 (+8), c0 % 16 == 0
  __device__ __forceinline__ LaneAddr(int l) {
    const int l32 = l & 31, hh = l >> 5, s16 = l & 15, g2 = (l >> 4) & 1;
    rowk = l32 * D + 8 * (hh ^ swz<D>(l32));
    // lane s = l % 16 addresses row c + s / 4, logical columns 32 t + 16 g2 + 4 (s % 4), i.e. chunk
    // 4 t + trc, half trh; the tile index t is applied later as an XOR with 32 t elements
    const int trc = 2 * g2 + ((s16 & 3) >> 1);
    const int trh = 4 * (s16 & 1);
    const int r0 = 4 * hh + (s16 >> 2), r1 = r0 + 8;
    tr0 = r0 * D + 8 * (trc ^ swz<D>(r0)) + trh;
    tr1 = r1 * D + 8 * (trc ^ swz<D>(r1)) + trh;
  }
  // Fragment for a contraction over the 16 tile rows c0 .. c0 + 15 (c0 % 16 == 0) in permuted
  // k-order, for column 32 t + l32: element j of lane (l32, hh) is row c0 + perm(0, hh, j).
  template <typename E>
  __device__ __forceinline__ ex8<E> read_cols(const E* tile, int c0, int t) const {
    union { struct { s16x4 lo, hi; } s; ex8<E> v; } u;
    u.s.lo = lds_read_tr(tile + c0 * D + (tr0 ^ (32 * t)));
    u.s.hi = lds_read_tr(tile + c0 * D + (tr1 ^ (32 * t)));
    return u.v;
  }
  // Row fragment in natural k-order: features 16 ks + 8 hh .. + 7 of row 32 t + l32.
  template <typename E>
  __device__ __forceinline__ ex8<E> read_row(const E* tile, int t, int ks) const {
    return *reinterpret_cast<const ex8<E>*>(tile + 32 * t * D + (rowk ^ (16 * ks)));
  }
};

// Direct HBM -> LDS loads of one tile set.  This wave issues instructions j = DMA_PER_WAVE w + i of
// every tile; lane l of instruction j fills LDS chunk q = 64 j + l, i.e. row q / CPR, physical chunk
// q % CPR, which holds logical chunk (q % CPR) ^ swz(row).
template <int D, int NTILES, int B = kB, int NW = 4>
struct TileLoader {
  using C = Cfg<D, B>;
  static constexpr int DMA_PER_WAVE = C::DMA_PER_TILE / NW;   // NW waves share the work
  int row[DMA_PER_WAVE], col[DMA_PER_WAVE];
  int w, l, n;
  uint32_t stride_n;
  uint32_t wave_lds;   // byte offset of this wave's part of a tile (wave-uniform, scalar register)
  const char* g[NTILES];
  __device__ __forceinline__ TileLoader(int w_, int l_, int n_, uint32_t stride_n_)
      : w(w_), l(l_), n(n_), stride_n(stride_n_) {
    wave_lds = (uint32_t)__builtin_amdgcn_readfirstlane(1024 * DMA_PER_WAVE * w_);
#pragma unroll
    for (int i = 0; i < DMA_PER_WAVE; i++) {
      const int q = 64 * (DMA_PER_WAVE * w + i) + l;
      row[i] = q / C::CPR;
      col[i] = 8 * ((q % C::CPR) ^ swz<D>(q / C::CPR));
    }
  }
  template <typename E>
  __device__ __forceinline__ void issue(E (*sT)[C::TILE], int blk) const {
#pragma unroll
    for (int i = 0; i < DMA_PER_WAVE; i++) {
      const int pos = min(blk * B + row[i], n - 1);   // rows past the end are re-zeroed by zero_tail
      // 32-bit byte offset from the (wave-uniform) chain base; the host checked that a chain spans < 4 GiB
      const uint32_t off = ((uint32_t)pos * stride_n + (uint32_t)col[i]) * 2u;
#pragma unroll
      for (int t = 0; t < NTILES; t++) dma16(g[t], off, lds_offset(&sT[t][0]) + wave_lds + 1024u * i);
    }
  }
  // The same loads one at a time (j = 0 .. NTILES DMA_PER_WAVE - 1), so that they can be spread over
  // the block's compute slots: offsets() once per block, then issue_one(j).
  // `valid` false (no such block): every lane reads the chain's first 16 bytes instead, a single
  // cache line per instruction, so that the loads can be issued unconditionally (no branches inside the
  // hand-scheduled block body, same count of outstanding operations for every block).
  __device__ __forceinline__ void offsets(int blk, bool valid, uint32_t (&off)[DMA_PER_WAVE]) const {
#pragma unroll
    for (int i = 0; i < DMA_PER_WAVE; i++) {
      const int pos = min(blk * B + row[i], n - 1);
      off[i] = valid ? ((uint32_t)pos * stride_n + (uint32_t)col[i]) * 2u : 0u;
    }
  }
  template <typename E>
  __device__ __forceinline__ void issue_one(E (*sT)[C::TILE], const uint32_t (&off)[DMA_PER_WAVE], int j) const {
    const int i = j / NTILES, t = j % NTILES;
    // LDS address = tile base (a constant once the buffer index is one) + scalar wave offset
    dma16(g[t], off[i], lds_offset(&sT[t][0]) + wave_lds + 1024u * i);
  }
  // after this wave's loads have landed: zero the rows of a ragged last block
  template <typename E>
  __device__ __forceinline__ void zero_tail(E (*sT)[C::TILE], int blk) const {
    if ((blk + 1) * B > n) {
#pragma unroll
      for (int i = 0; i < DMA_PER_WAVE; i++) {
        if (blk * B + row[i] >= n) {
          const i32x4 z = {0, 0, 0, 0};
#pragma unroll
          for (int t = 0; t < NTILES; t++)
            *reinterpret_cast<i32x4*>(reinterpret_cast<char*>(&sT[t][0]) + (wave_lds + 1024u * i + 16u * l)) = z;
        }
      }
    }
  }
};

// state slice element (t, v) of a lane <-> key feature dk, value feature dv of the d x d state
template <int D>
__device__ __forceinline__ int state_index(int dvt, int l32, int hh, int t, int v, bool transposed) {
  const int dk = 32 * t + 8 * (v >> 2) + 4 * hh + (v & 3);
  const int dv = 32 * dvt + l32;
  return transposed ? dv * D + dk : dk * D + dv;
}

// A wave-uniform value moved to a scalar register for good: the compiler folds the builtin below away when it can
// prove the value uniform, and then keeps a loop invariant like that in a vector register (or spills it).
// The compiler does not look into an asm statement for the wait states that gfx950 wants between a vector
// instruction that writes a register and a lane read of it, and between a vector instruction that writes a scalar
// register and one that reads it: the statement brings its own.
__device__ __forceinline__ float scalar_reg(float x) {
  uint32_t r;
  asm("s_nop 1\n\tv_readfirstlane_b32 %0, %1\n\ts_nop 1" : "=s"(r) : "v"(__float_as_uint(x)));
  return __uint_as_float(r);
}

// A wave-uniform value, told to the compiler (lands in a scalar register instead of a vector one).
__device__ __forceinline__ float uniform(float x) {
  return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x)));
}

// Row weights of the state update, S <- lambda^B S + Y^T decay(Z) with row c weighted lambda^(B-1-c)
// (forward) or lambda^(c+1) (reverse), applied to the Z fragments (permuted k-order, 16 rows from c0).
// Element j of lane half hh is row c0 + 4 hh + nj, nj = 8 (j / 4) + j % 4.  The weight is split into
// a per-lane factor (one exp2 per fragment) and a wave-uniform factor per element:
//   forward  lambda^(B-16-c0 + 4 (1-hh)) * lambda^(11-nj)      reverse  lambda^(c0 + 4 hh + 1) * lambda^nj
// All exponents are non-negative.
template <bool REV, int B = kB>
struct UpdateDecay {
  float gj[8];   // wave-uniform
  float l2;
  int hh;
  __device__ __forceinline__ UpdateDecay(float l2_, int hh_) : l2(l2_), hh(hh_) {
#pragma unroll
    for (int j = 0; j < 8; j++) {
      const int nj = 8 * (j >> 2) + (j & 3);
      gj[j] = uniform(exp2f(l2 * (float)(REV ? nj : 11 - nj)));
    }
  }
  // `scale`: one more factor on every weight (the chunk-state pre-pass folds a block's whole-block decay in)
  template <typename E>
  __device__ __forceinline__ ex8<E> apply(ex8<E> z, int c0, float scale = 1.f) const {
    const float step = scale * fast_exp2(l2 * (float)(REV ? c0 + 4 * hh + 1 : B - 16 - c0 + 4 * (1 - hh)));
    ex8<E> r;
#pragma unroll
    for (int j = 0; j < 8; j++) r[j] = (E)((float)z[j] * (step * gj[j]));
    return r;
  }
};

}  // namespace bf16k

// per-kernel launchers (one translation unit each); launch_scan_bf16 picks among the first two
hipError_t launch_scan_bf16_full(int dtype, int head_dim, bool reverse, const ScanParams& p, hipStream_t s);
hipError_t launch_scan_bf16_half(int dtype, int head_dim, bool reverse, bool twin, const ScanParams& p, hipStream_t s);

}  // namespace la2
#endif
