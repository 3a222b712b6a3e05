// bf16 MFMA kernels for the decayed causal scan (Algorithm 1; both loops of Algorithm 2), gfx950.
//
// One workgroup (4 waves) walks the blocks (B = 64 positions) of one sequence chunk of one
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
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "la2_internal.h"

namespace la2 {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
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
  static constexpr int WPD = 4 / NT;           // waves sharing one value-feature tile (1 or 2)
  static constexpr int RT = 2 / WPD;           // 32-row tiles of the block per wave (2 or 1)
  static constexpr int CPR = D / 8;            // 16-byte chunks per tile row
  static constexpr int TILE = B * D;           // elements per tile
  static constexpr int DMA_PER_TILE = TILE / 512;   // wave instructions (1 KiB each) per tile
  static constexpr int DMA_PER_WAVE = DMA_PER_TILE / 4;
  static constexpr int LW = 32;                // staging row: 32 features = 64 bytes, unpadded, 16-byte chunks
                                               // XOR-swizzled by (row / 4) % 4 (LDS is full: no room for padding)
};

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
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
__device__ __forceinline__ s16x4 lds_read_tr(const __bf16* p) {
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
  if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
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
__device__ __forceinline__ bf16x8 to_perm_order(bf16x8 f) {
  union { bf16x8 v; u32x4 u; } x;
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
  __device__ __forceinline__ bf16x8 read_cols(const __bf16* tile, int c0, int t) const {
    union { struct { s16x4 lo, hi; } s; bf16x8 v; } u;
    u.s.lo = lds_read_tr(tile + c0 * D + (tr0 ^ (32 * t)));
    u.s.hi = lds_read_tr(tile + c0 * D + (tr1 ^ (32 * t)));
    return u.v;
  }
  // Row fragment in natural k-order: features 16 ks + 8 hh .. + 7 of row 32 t + l32.
  __device__ __forceinline__ bf16x8 read_row(const __bf16* tile, int t, int ks) const {
    return *reinterpret_cast<const bf16x8*>(tile + 32 * t * D + (rowk ^ (16 * ks)));
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
  __device__ __forceinline__ void issue(__bf16 (*sT)[C::TILE], int blk) const {
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
  __device__ __forceinline__ void issue_one(__bf16 (*sT)[C::TILE], const uint32_t (&off)[DMA_PER_WAVE],
                                            int j) const {
    const int i = j / NTILES, t = j % NTILES;
    // LDS address = tile base (a constant once the buffer index is one) + scalar wave offset
    dma16(g[t], off[i], lds_offset(&sT[t][0]) + wave_lds + 1024u * i);
  }
  // after this wave's loads have landed: zero the rows of a ragged last block
  __device__ __forceinline__ void zero_tail(__bf16 (*sT)[C::TILE], int blk) const {
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
  __device__ __forceinline__ bf16x8 apply(bf16x8 z, int c0) const {
    const float step = fast_exp2(l2 * (float)(REV ? c0 + 4 * hh + 1 : B - 16 - c0 + 4 * (1 - hh)));
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; j++) r[j] = (__bf16)((float)z[j] * (step * gj[j]));
    return r;
  }
};

template <int D, bool REV>
__global__ __launch_bounds__(kThreads, 1) void scan_bf16_kernel(ScanParams p) {
  using C = Cfg<D>;
  constexpr int KS = C::KS, NT = C::NT, RT = C::RT, TILE = C::TILE, LW = C::LW;
  // two tile buffers as two distinct LDS objects ([X, Y, Z] each) so that reads of one buffer are
  // provably independent of the direct loads in flight into the other
  __shared__ __attribute__((aligned(1024))) __bf16 sT0[3][TILE];
  __shared__ __attribute__((aligned(1024))) __bf16 sT1[3][TILE];
  __shared__ __attribute__((aligned(1024))) __bf16 sT2[3][TILE];
  __shared__ __attribute__((aligned(16))) __bf16 sW[4][32 * RT * LW];
  // vector-memory operations a wave issues per block: direct loads (3 tiles) and output stores
  constexpr int LOADS_PER_BLOCK = 3 * C::DMA_PER_WAVE, STORES_PER_BLOCK = 32 * RT * 4 / 64;
  // s_waitcnt immediate for "at most N vector-memory operations outstanding" (gfx9 encoding)
  constexpr int VM_YOUNGER = STORES_PER_BLOCK + LOADS_PER_BLOCK;
  constexpr int WAIT_NEXT_TILES = (VM_YOUNGER & 15) | ((VM_YOUNGER >> 4) << 14) | 0x0F70;

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int dvt = w % NT;                                  // this wave's value-feature tile
  const int rt0 = (C::WPD == 1) ? 0 : (w / NT) * RT;       // its first row tile
  // Dual launch: two workgroups run scan 0 and scan 1 of the same (chain, chunk).  Workgroups are
  // dealt to the 8 XCDs round-robin by index and every XCD has its own L2, so the two partners are
  // the workgroups i and i + 8 of a group of 16: same XCD, dispatched together, and the tiles both
  // read are in that XCD's L2 for whichever comes second.  (A launch whose pair count is not a
  // multiple of 8 pairs neighbours instead; that is correct, only the tile sharing is weaker.)
  int which = 0, wg = (int)blockIdx.x;
  if (p.nscan == 2) {
    if (((gridDim.x >> 1) & 7) == 0) {
      which = (int)(blockIdx.x >> 3) & 1;
      wg = (int)((blockIdx.x >> 4) << 3) | (int)(blockIdx.x & 7);
    } else {
      which = (int)(blockIdx.x & 1);
      wg = (int)(blockIdx.x >> 1);
    }
  }
  const int chain = wg / p.nchunks, chunk = wg % p.nchunks;
  const int bi = chain / p.heads, hi = chain % p.heads;
  const int64_t base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h;
  const int n = p.n;
  const uint32_t stride_n = (uint32_t)p.stride_n;
  const uint32_t chain_bytes = ((uint32_t)(n - 1) * stride_n + D) * 2u;
  const __amdgpu_buffer_rsrc_t bw =
      make_rsrc(reinterpret_cast<__bf16*>(which ? p.w[1] : p.w[0]) + base, chain_bytes);
  const float l2 = log2f(p.lambda[hi]);

  const int nblocks = (n + kB - 1) / kB;
  const int cb = p.chunk_tokens / kB;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);
  if (blk_lo >= blk_hi) return;
  const int nblk = blk_hi - blk_lo;

  TileLoader<D, 3> loader(w, l, n, stride_n);
  loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(which ? p.x[1] : p.x[0]) + base);
  loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(which ? p.y[1] : p.y[0]) + base);
  loader.g[2] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(which ? p.z[1] : p.z[0]) + base);
  const LaneAddr<D> la(l);

  // ---- running state slice S[:, dv tile]: NT accumulator tiles (key-feature tiles), fp32
  f32x16 kv[NT];
  const float* gs = nullptr;   // start state: chunk start state, the caller's start state, or zero
  bool tr = false;
  if (p.states != nullptr) {
    gs = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
    tr = (p.state_transposed >> which) & 1;
  } else if (D == 64 && (which ? p.init[1] : p.init[0]) != nullptr) {   // d = 128 with states: half-block kernel
    gs = (which ? p.init[1] : p.init[0]) + (int64_t)chain * (D * D);
    tr = (p.init_transposed >> which) & 1;
  }
  if (gs != nullptr) {
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) kv[t][v] = gs[state_index<D>(dvt, l32, hh, t, v, tr)];
  } else {
#pragma unroll
    for (int t = 0; t < NT; t++) kv[t] = zero16();
  }

  // The two key tiles of the block as seen from this wave: slot 0 / slot 1.  d = 128: key tiles 0, 1.
  // d = 64: slot 0 is the wave's own (diagonal) key tile, slot 1 the other one.
  const int ct0 = (RT == 2) ? 0 : rt0, ct1 = 1 - ct0;
  // Besides the diagonal pairs one (row tile, key tile) pair exists per block: forward the later row
  // tile sees the earlier key tile, reverse the earlier row tile sees the later key tile.
  constexpr int OFF_RT = REV ? 0 : 1;                          // row tile of that pair
  const bool has_off = (RT == 2) || (rt0 == OFF_RT);           // wave-uniform: this wave owns that row tile
  constexpr int OFF_ACC = (RT == 2) ? OFF_RT : 0;              // its index among the wave's row tiles
  constexpr int OFF_SLOT = (RT == 2) ? 1 - OFF_RT : 1;         // slot of that pair's key tile

  // ---- per-lane constants.  Score tile S^T[c][r]: this lane's position is column l32, accumulator
  // element v is key row cc[v] = 8 (v / 4) + 4 hh + v % 4 of the key tile.  Decay mask lambda^|r-c|
  // with non-negative exponents only (lambda^r * lambda^-c would overflow):
  //   diagonal tile (key tile == row tile): lambda^(l32 - cc[v]) on the causal side, else 0
  //   the other tile (32 rows away):        lambda^(l32 + 32 - cc[v])      (reverse: l32, cc swapped)
  // A wave that does not own the off-diagonal pair (d = 64) computes it all the same, branch-free,
  // with an all-zero mask.
  // The off-diagonal mask is split into a per-lane factor and a wave-uniform factor per element
  // (cc[v] = mv + 4 hh, mv = 8 (v / 4) + v % 4):
  //   forward  lambda^(l32 + 5 - 4 hh) * lambda^(27 - mv)       reverse  lambda^(32 - l32 + 4 hh) * lambda^mv
  float dg[16], ou[16];
#pragma unroll
  for (int v = 0; v < 16; v++) {
    const int mv = 8 * (v >> 2) + (v & 3);
    const int e = REV ? mv + 4 * hh - l32 : l32 - mv - 4 * hh;
    dg[v] = (e >= 0) ? exp2f(l2 * (float)e) : 0.f;
    ou[v] = uniform(exp2f(l2 * (float)(REV ? mv : 27 - mv)));
  }
  const float oa = has_off ? exp2f(l2 * (float)(REV ? 32 - l32 + 4 * hh : l32 + 5 - 4 * hh)) : 0.f;
  // weight of the carried state at this lane's position r = 32 rt + l32: forward lambda^(r+1),
  // reverse lambda^(B-1-r)
  float inter_scale[RT];
#pragma unroll
  for (int i = 0; i < RT; i++) {
    const int r = 32 * (rt0 + i) + l32;
    inter_scale[i] = exp2f(l2 * (float)(REV ? kB - 1 - r : r + 1));
  }
  const UpdateDecay<REV> decay(l2, hh);
  const float lamB = exp2f(l2 * (float)kB);

  // ---- prologue: first block's tiles
  {
    const int b0 = REV ? blk_hi - 1 : blk_lo, b1 = REV ? b0 - 1 : b0 + 1;
    loader.issue(sT0, b0);
    if (nblk > 1) loader.issue(sT1, b1);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    loader.zero_tail(sT0, b0);
    if (nblk > 1) loader.zero_tail(sT1, b1);
  }
  __syncthreads();

  // Row fragments (natural k-order, only ever MFMA operands) are read from LDS two slots ahead of
  // the MFMAs that consume them: the X rows of this wave's row tiles for phase 1, and again together
  // with the Y rows of the same (diagonal) key tiles and of the off-diagonal pair's key tile for
  // phase 2.  (Reading X twice costs LDS bandwidth that is there; holding a block's fragments for two
  // phases costs registers that are not.)  The first two k-steps of phase 1 are read across the
  // barrier, underneath the last MFMAs of the previous block.
  constexpr int AHEAD = 2;
  bf16x8 xa[RT][KS];
  auto read_xa = [&](const __bf16 (*sB)[TILE], int ks) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < RT; i++) xa[i][ks] = la.read_row(sB[0], rt0 + i, ks);
  };
#pragma unroll
  for (int ks = 0; ks < AHEAD; ks++) read_xa(sT0, ks);

  // State tile ks / 2, k-step ks % 2 as a bf16 MFMA operand in NATURAL k-order: the accumulator
  // layout gives permuted order, the exchange between the wave's halves undoes it, so that the X
  // fragments serve the score product and the inter-block product unchanged.
  auto state_operand = [&](int ks) __attribute__((always_inline)) {
    bf16x8 f;
#pragma unroll
    for (int j = 0; j < 8; j++) f[j] = (__bf16)kv[ks >> 1][8 * (ks & 1) + j];
    return to_perm_order(f);   // the exchange is its own inverse
  };

  // Finished output of the previous block (transposed: value feature x position), stored while the
  // next block computes; and the first state operand of the block about to be computed.
  f32x16 outp[RT];
#pragma unroll
  for (int i = 0; i < RT; i++) outp[i] = zero16();
  bf16x8 sa_first = state_operand(0);
  __bf16* const stage = sW[w];
  constexpr int NST = 32 * RT * 4 / 64;   // 16-byte stores per lane and block
  // Output of block `oblk` in three steps: pack to bf16 and stage through LDS (so that the stores are
  // 16 bytes per lane, 64 contiguous bytes per row); read back; store.  `valid` false (no previous
  // block): the offset is pushed out of the buffer's range and the stores are dropped.
  auto out_pack = [&](int i) __attribute__((always_inline)) {
#pragma unroll
    for (int g = 0; g < 4; g++) {
      bf16x4 pk;
#pragma unroll
      for (int e = 0; e < 4; e++) pk[e] = (__bf16)outp[i][4 * g + e];
      const int row = 32 * i + l32;
      *reinterpret_cast<bf16x4*>(stage + row * LW + 8 * (g ^ ((row >> 2) & 3)) + 4 * hh) = pk;
    }
  };
  auto out_read = [&](i32x4 (&ov)[NST]) __attribute__((always_inline)) {
    // same-wave LDS write -> read: ordered by the LDS queue, no workgroup barrier needed
#pragma unroll
    for (int i = 0; i < NST; i++) {
      const int id = l + 64 * i;
      const int row = id >> 2, cc = id & 3;
      ov[i] = *reinterpret_cast<const i32x4*>(stage + row * LW + 8 * (cc ^ ((row >> 2) & 3)));
    }
  };
  auto out_store = [&](const i32x4 (&ov)[NST], int oblk, bool valid) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NST; i++) {
      const int id = l + 64 * i;
      const int row = id >> 2, cc = id & 3;
      const uint32_t off = ((uint32_t)(oblk * kB + 32 * rt0 + row) * stride_n + (uint32_t)(32 * dvt + cc * 8)) * 2u;
      __builtin_amdgcn_raw_buffer_store_b128(ov[i], bw, valid ? off : 0xFFFFFFF0u, 0, 0);
    }
  };

  // One block of the loop.  Block `it` lives in tile buffer it % 3, which is a compile-time constant
  // (the loop below is unrolled by three).
  //
  // A workgroup is one wave per SIMD, so nothing but this wave's own instruction order overlaps the
  // matrix pipe with LDS reads, conversions, masks and the issue of loads and stores.  The body is
  // therefore branch-free and written as a sequence of SLOTS: a slot holds a few MFMAs plus the side
  // work that should run in their shadow; values produced in a slot are pinned at its end and a
  // scheduling barrier closes it, so that the compiler keeps the slots apart and in order (inside
  // a slot it interleaves freely).  The phases of block it:
  //   1  inter-block  W^T = State^T X^T       (KS slots)  + output of block it-1: pack, stage, store;
  //                                                         direct loads of block it+2; next state
  //                                                         operand; Z reads
  //   2  score chains S^T = Y X^T             (KS slots)  + rest of the direct loads; lambda^B on the
  //                                                         state; position decay on W^T; update
  //                                                         weights on Z
  //   3  state update State += Y^T decay(Z)   (4 slots)   + decay masks of the scores
  //      then the barrier and the first row fragments of block it+1
  //   4  intra-block  W^T += Z^T P^T          (one slot)  + first state operand of block it+1
  // Returns false after the last block.
#define LA2_SLOT_END()                 \
  do {                                 \
    asm volatile("" ::: "memory");     \
    __builtin_amdgcn_sched_barrier(0); \
  } while (0)
  constexpr int NDMA = 3 * C::DMA_PER_WAVE;   // direct loads per wave and block, one per slot of 1, 2
  static_assert(NDMA <= 2 * KS, "one direct load per slot");
  auto block_step = [&](auto cur_tag, int it) __attribute__((always_inline)) -> bool {
    constexpr int cur = decltype(cur_tag)::value;
    __bf16 (*const sCur)[TILE] = cur == 0 ? sT0 : (cur == 1 ? sT1 : sT2);     // block it
    __bf16 (*const sNext)[TILE] = cur == 0 ? sT1 : (cur == 1 ? sT2 : sT0);    // block it + 1 (in flight or landed)
    __bf16 (*const sAhead)[TILE] = cur == 0 ? sT2 : (cur == 1 ? sT0 : sT1);   // block it + 2 (free since block it - 1)
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    const bool has_next = it + 1 < nblk, has_ahead = it + 2 < nblk;
    const int nb = REV ? blk - 1 : blk + 1, pb = REV ? blk + 1 : blk - 1;
    const __bf16* tY = sCur[1];
    const __bf16* tZ = sCur[2];
    uint32_t doff[C::DMA_PER_WAVE];
    loader.offsets(REV ? blk - 2 : blk + 2, has_ahead, doff);

    bf16x8 zf[2][2];     // Z columns of this wave's value tile: [key-tile slot][k-step], permuted k-order
    bf16x8 zd[2][2];     // the same, weighted for the state update
    bf16x8 yt[NT][2][2]; // Y columns (key features): [key-feature tile][slot][k-step], permuted k-order
    bf16x8 xb[RT][KS], yb[RT][KS], yo[KS];   // phase 2 operands
    auto read_xy = [&](int ks) __attribute__((always_inline)) {
#pragma unroll
      for (int i = 0; i < RT; i++) xb[i][ks] = la.read_row(sCur[0], rt0 + i, ks);
#pragma unroll
      for (int i = 0; i < RT; i++) yb[i][ks] = la.read_row(sCur[1], rt0 + i, ks);
      if (RT == 1) yo[ks] = la.read_row(sCur[1], ct1, ks);
    };
    auto read_yt = [&](int sq) __attribute__((always_inline)) {   // operands of update k-step sq
      const int s = sq >> 1, q = sq & 1;
#pragma unroll
      for (int t = 0; t < NT; t++) yt[t][s][q] = la.read_cols(tY, 32 * (s ? ct1 : ct0) + 16 * q, t);
    };

    // ---- phase 1: W^T[dv][r] = sum_dk State[dk][dv] X[r][dk] from the state in registers
    f32x16 inter[RT];
#pragma unroll
    for (int i = 0; i < RT; i++) inter[i] = zero16();
    i32x4 ov[NST];
    bf16x8 sa = sa_first;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
#pragma unroll
      for (int i = 0; i < RT; i++) pin_acc(xa[i][ks]);
#pragma unroll
      for (int i = 0; i < RT; i++) inter[i] = mfma(sa, xa[i][ks], inter[i]);
      if (ks + AHEAD < KS) read_xa(sCur, ks + AHEAD);
      else read_xy(ks + AHEAD - KS);
      if (ks + 1 < KS) { sa = state_operand(ks + 1); pin(sa); }
      if (ks < NDMA) loader.issue_one(sAhead, doff, ks);
      if (ks < 4) {
        const int s = ks >> 1, q = ks & 1;
        zf[s][q] = la.read_cols(tZ, 32 * (s ? ct1 : ct0) + 16 * q, dvt);
      }
      if (ks < RT) out_pack(ks);
      if (ks == RT) out_read(ov);
      if (ks == RT + 1) out_store(ov, pb, it > 0);
#pragma unroll
      for (int i = 0; i < RT; i++) pin(inter[i]);
      LA2_SLOT_END();
    }

    // ---- phase 2: score tiles S^T[c][r] = sum_k Y[c][k] X[r][k]
    f32x16 sd[RT], so = zero16();
#pragma unroll
    for (int i = 0; i < RT; i++) sd[i] = zero16();
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
#pragma unroll
      for (int i = 0; i < RT; i++) { pin_acc(xb[i][ks]); pin_acc(yb[i][ks]); }
      if (RT == 1) pin_acc(yo[ks]);
#pragma unroll
      for (int i = 0; i < RT; i++) sd[i] = mfma(yb[i][ks], xb[i][ks], sd[i]);
      if (RT == 2) so = mfma(yb[(RT == 2) ? OFF_SLOT : 0][ks], xb[OFF_ACC][ks], so);
      else so = mfma(yo[ks], xb[0][ks], so);
      if (ks + AHEAD < KS) read_xy(ks + AHEAD);
      if (ks == KS - 1) read_yt(0);
      if (KS + ks < NDMA) loader.issue_one(sAhead, doff, KS + ks);
      // the fp32 state takes its lambda^B for the update (all its bf16 operands have been made)
      if (ks % (KS / NT) == 0) {
        const int t = ks / (KS / NT);
#pragma unroll
        for (int v = 0; v < 16; v++) kv[t][v] *= lamB;
        pin(kv[t]);
      }
      // the carried part takes the decay at this lane's position
      if ((ks & 1) && (ks >> 1) < RT) {
        const int i = ks >> 1;
#pragma unroll
        for (int v = 0; v < 16; v++) inter[i][v] *= inter_scale[i];
        pin(inter[i]);
      }
      if (ks >= KS - 4) {
        const int f = ks - (KS - 4), s = f >> 1, q = f & 1;
        zd[s][q] = decay.apply(zf[s][q], 32 * (s ? ct1 : ct0) + 16 * q);
        pin(zd[s][q]);
      }
#pragma unroll
      for (int i = 0; i < RT; i++) pin(sd[i]);
      pin(so);
      LA2_SLOT_END();
    }

    // ---- phase 3: state slice <- lambda^B state + Y^T decay(Z), contraction over this block's rows in
    // 4 k-steps; meanwhile the decay masks turn the finished score tiles into bf16 operands.
    // (After the last block the state is not needed; the update runs anyway, branch-free.)
    bf16x8 pd[RT][2], po[2];
#pragma unroll
    for (int sq = 0; sq < 4; sq++) {
#pragma unroll
      for (int t = 0; t < NT; t++) pin_acc(yt[t][sq >> 1][sq & 1]);
#pragma unroll
      for (int t = 0; t < NT; t++) kv[t] = mfma(yt[t][sq >> 1][sq & 1], zd[sq >> 1][sq & 1], kv[t]);
      if (sq + 1 < 4) read_yt(sq + 1);
#pragma unroll
      for (int e = 0; e < 4; e++) {
        const int v = 4 * sq + e;
#pragma unroll
        for (int i = 0; i < RT; i++) pd[i][v >> 3][v & 7] = (__bf16)(sd[i][v] * dg[v]);
        po[v >> 3][v & 7] = (__bf16)((so[v] * oa) * ou[v]);
      }
#pragma unroll
      for (int i = 0; i < RT; i++) pin(pd[i][sq >> 1]);
      pin(po[sq >> 1]);
#pragma unroll
      for (int t = 0; t < NT; t++) pin(kv[t]);
      LA2_SLOT_END();
    }

    if (has_next) {
      // This wave's direct loads of block it + 1 must have landed.  Vector-memory operations complete
      // in issue order; younger than those loads are the stores of block it - 1 and the loads (real
      // or dummy) of block it + 2.
      __builtin_amdgcn_s_waitcnt(WAIT_NEXT_TILES);
      loader.zero_tail(sNext, nb);
      lds_barrier();                       // next tiles visible to all waves; current tiles free
#pragma unroll
      for (int ks = 0; ks < AHEAD; ks++) read_xa(sNext, ks);
    }
    LA2_SLOT_END();

    // ---- phase 4: intra-block part Z^T P^T on top of the decayed carried part
#pragma unroll
    for (int i = 0; i < RT; i++) {
#pragma unroll
      for (int q = 0; q < 2; q++) inter[i] = mfma(zf[(RT == 2) ? i : 0][q], pd[i][q], inter[i]);
    }
#pragma unroll
    for (int q = 0; q < 2; q++) inter[OFF_ACC] = mfma(zf[OFF_SLOT][q], po[q], inter[OFF_ACC]);
    sa_first = state_operand(0);
    pin(sa_first);
#pragma unroll
    for (int i = 0; i < RT; i++) {
      outp[i] = inter[i];
      pin(outp[i]);
    }
    LA2_SLOT_END();
    return has_next;
  };
  int it = 0;
  for (;; it += 3) {
    if (!block_step(std::integral_constant<int, 0>{}, it)) break;
    if (!block_step(std::integral_constant<int, 1>{}, it + 1)) { it += 1; break; }
    if (!block_step(std::integral_constant<int, 2>{}, it + 2)) { it += 2; break; }
  }
  // output of the last block
  {
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    i32x4 ov[NST];
#pragma unroll
    for (int i = 0; i < RT; i++) out_pack(i);
    out_read(ov);
    out_store(ov, blk, true);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the dummy direct loads before the LDS is given up
  }
  // state after the chain's last block, if the caller wants it (the update ran on every block)
  float* gf = which ? p.fin[1] : p.fin[0];
  if (D == 64 && gf != nullptr && (REV ? chunk == 0 : chunk == p.nchunks - 1) && rt0 == 0) {
    gf += (int64_t)chain * (D * D);
    const bool trf = (p.fin_transposed >> which) & 1;
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) gf[state_index<D>(dvt, l32, hh, t, v, trf)] = kv[t][v];
  }
#undef LA2_SLOT_END
}

// Half-block variant for d = 128: blocks of 32 positions, 80 KiB of LDS and at most 256 registers, so
// that TWO workgroups share a compute unit (two waves per SIMD).  One wave alone issues its
// instructions one after the other (an MFMA holds the issue port for about half its run time, a
// 16-byte-per-lane memory instruction for about 60 cycles), so a single wave per SIMD leaves the
// matrix pipe idle most of the time; a second, independent wave fills those gaps.  Used when a launch
// has enough workgroups to put two on every compute unit.  Same math as scan_bf16_kernel with a
// single (diagonal) 32 x 32 score tile per block; wave w owns value features 32 w .. 32 w + 31.
constexpr int kBH = 32;
//
// TWIN: both scans of a dual launch in ONE workgroup of 8 waves (waves 0-3 scan 0, waves 4-7 scan 1;
// again two waves per SIMD).  The dual launch is Algorithm 2's second loop, whose two scans read the
// same two tensors with the roles of Y and Z exchanged (dV: y = Q, z = dO; dK: y = dO, z = Q), so the
// workgroup streams FOUR tiles per block (x of scan 0, x of scan 1, Q, dO) instead of six and every
// tile is fetched exactly once.  Requires y[1] == z[0] and z[1] == y[0].
//
// NBUF tile buffers: block it + NBUF - 1 streams in while block it is computed.  With 3 buffers two
// (plain) workgroups fit on a compute unit.
template <bool REV, bool TWIN, int NBUF>
__global__ __launch_bounds__(TWIN ? 512 : 256, TWIN ? 1 : 2) void scan_bf16_half_kernel(ScanParams p) {
  constexpr int D = 128, B = kBH;
  using C = Cfg<D, B>;
  constexpr int KS = C::KS, NT = C::NT, TILE = C::TILE, LW = C::LW;
  constexpr int NW = TWIN ? 8 : 4;             // waves
  constexpr int NTL = TWIN ? 4 : 3;            // tiles per block
  using Loader = TileLoader<D, NTL, B, NW>;
  __shared__ __attribute__((aligned(1024))) __bf16 sT[NBUF][NTL][TILE];
  __shared__ __attribute__((aligned(16))) __bf16 sW[NW][32 * LW];
  constexpr int NDMA = NTL * Loader::DMA_PER_WAVE;   // direct loads per wave and block
  constexpr int NST = 32 * 4 / 64;             // 16-byte stores per lane and block
  static_assert(NDMA <= KS, "one direct load per slot of phase 1");
  // vector-memory operations of this wave that are younger than the direct loads of block it + 1 when block
  // it waits for them: the loads of blocks it + 2 .. it + NBUF - 1 and as many blocks' stores
  constexpr int VM_YOUNGER = (NBUF - 2) * (NST + NDMA);
  static_assert(VM_YOUNGER < 64, "vmcnt is a 6-bit counter");
  constexpr int WAIT_NEXT_TILES = (VM_YOUNGER & 15) | ((VM_YOUNGER >> 4) << 14) | 0x0F70;

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int dvt = w & 3;
  int which = 0, wg = (int)blockIdx.x;
  if (TWIN) {
    which = __builtin_amdgcn_readfirstlane(w >> 2);
  } else if (p.nscan == 2) {   // same pairing as scan_bf16_kernel
    if (((gridDim.x >> 1) & 7) == 0) {
      which = (int)(blockIdx.x >> 3) & 1;
      wg = (int)((blockIdx.x >> 4) << 3) | (int)(blockIdx.x & 7);
    } else {
      which = (int)(blockIdx.x & 1);
      wg = (int)(blockIdx.x >> 1);
    }
  }
  // In a twin workgroup the two wave groups run two instantiations of the body, so that each sees
  // its tiles at compile-time LDS offsets.
  auto run = [&](auto wh_tag) __attribute__((always_inline)) {
  constexpr int WH = decltype(wh_tag)::value;
  const int chain = wg / p.nchunks, chunk = wg % p.nchunks;
  const int bi = chain / p.heads, hi = chain % p.heads;
  const int64_t base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h;
  const int n = p.n;
  const uint32_t stride_n = (uint32_t)p.stride_n;
  const uint32_t chain_bytes = ((uint32_t)(n - 1) * stride_n + D) * 2u;
  const __amdgpu_buffer_rsrc_t bw =
      make_rsrc(reinterpret_cast<__bf16*>(which ? p.w[1] : p.w[0]) + base, chain_bytes);
  const float l2 = log2f(p.lambda[hi]);

  const int nblocks = (n + B - 1) / B;
  const int cb = p.chunk_tokens / B;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);
  if (blk_lo >= blk_hi) return;
  const int nblk = blk_hi - blk_lo;

  Loader loader(w, l, n, stride_n);
  if (TWIN) {
    loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(p.x[0]) + base);
    loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(p.x[1]) + base);
    loader.g[2] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(p.y[0]) + base);
    loader.g[NTL - 1] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(p.z[0]) + base);
  } else {
    loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(which ? p.x[1] : p.x[0]) + base);
    loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(which ? p.y[1] : p.y[0]) + base);
    loader.g[2] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(which ? p.z[1] : p.z[0]) + base);
  }
  // this wave's X, Y, Z among the tiles of a block
  constexpr int xi = TWIN ? WH : 0, yi = TWIN ? 2 + WH : 1, zi = TWIN ? 3 - WH : 2;
  const LaneAddr<D> la(l);

  f32x16 kv[NT];
  const float* gs = nullptr;   // start state: chunk start state, the caller's start state, or zero
  bool tr = false;
  if (p.states != nullptr) {
    gs = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
    tr = (p.state_transposed >> which) & 1;
  } else if ((which ? p.init[1] : p.init[0]) != nullptr) {
    gs = (which ? p.init[1] : p.init[0]) + (int64_t)chain * (D * D);
    tr = (p.init_transposed >> which) & 1;
  }
  if (gs != nullptr) {
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) kv[t][v] = gs[state_index<D>(dvt, l32, hh, t, v, tr)];
  } else {
#pragma unroll
    for (int t = 0; t < NT; t++) kv[t] = zero16();
  }

  // decay mask of the score tile S^T[c][r] (lane: r = l32; element v: c = 8 (v / 4) + 4 hh + v % 4)
  float dg[16];
#pragma unroll
  for (int v = 0; v < 16; v++) {
    const int cc = 8 * (v >> 2) + 4 * hh + (v & 3);
    const int e = REV ? cc - l32 : l32 - cc;
    dg[v] = (e >= 0) ? exp2f(l2 * (float)e) : 0.f;
  }
  const float inter_scale = exp2f(l2 * (float)(REV ? B - 1 - l32 : l32 + 1));
  const UpdateDecay<REV, B> decay(l2, hh);
  const float lamB = uniform(exp2f(l2 * (float)B));

  // prologue: the first NBUF - 1 blocks' tiles
#pragma unroll
  for (int j = 0; j < NBUF - 1; j++)
    if (j < nblk) loader.issue(sT[j], REV ? blk_hi - 1 - j : blk_lo + j);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
#pragma unroll
  for (int j = 0; j < NBUF - 1; j++)
    if (j < nblk) loader.zero_tail(sT[j], REV ? blk_hi - 1 - j : blk_lo + j);
  __syncthreads();

  constexpr int AHEAD = 1;   // LDS operands are read one slot ahead (the other wave on the SIMD covers the rest)
  bf16x8 xa[KS], ya[KS];     // X and Y row fragments (natural k-order) of the block being computed
#pragma unroll
  for (int ks = 0; ks < AHEAD; ks++) {
    xa[ks] = la.read_row(sT[0][xi], 0, ks);
    ya[ks] = la.read_row(sT[0][yi], 0, ks);
  }
  auto state_operand = [&](int ks) __attribute__((always_inline)) {
    bf16x8 f;
#pragma unroll
    for (int j = 0; j < 8; j++) f[j] = (__bf16)kv[ks >> 1][8 * (ks & 1) + j];
    return to_perm_order(f);
  };
  bf16x8 sa_first = state_operand(0);
  __bf16* const stage = sW[w];

#define LA2_SLOT_END()                 \
  do {                                 \
    asm volatile("" ::: "memory");     \
    __builtin_amdgcn_sched_barrier(0); \
  } while (0)
  // Phases as in scan_bf16_kernel (1 inter-block product and 2 scores, here interleaved; 3 state update;
  // barrier; 4 intra-block product), then the block's output.
  auto block_step = [&](auto cur_tag, int it) __attribute__((always_inline)) -> bool {
    constexpr int cur = decltype(cur_tag)::value;
    __bf16 (*const sCur)[TILE] = sT[cur];                          // block it
    __bf16 (*const sNext)[TILE] = sT[(cur + 1) % NBUF];            // block it + 1 (in flight or landed)
    __bf16 (*const sAhead)[TILE] = sT[(cur + NBUF - 1) % NBUF];    // block it + NBUF - 1 (free since block it - 1)
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    const bool has_next = it + 1 < nblk, has_ahead = it + NBUF - 1 < nblk;
    const int nb = REV ? blk - 1 : blk + 1;
    const __bf16* tX = sCur[xi];
    const __bf16* tY = sCur[yi];
    const __bf16* tZ = sCur[zi];
    uint32_t doff[Loader::DMA_PER_WAVE];
    loader.offsets(REV ? blk - (NBUF - 1) : blk + (NBUF - 1), has_ahead, doff);

    bf16x8 zf[2], zd[2], yt[2][NT];
    auto read_xy = [&](int ks) __attribute__((always_inline)) {
      xa[ks] = la.read_row(tX, 0, ks);
      ya[ks] = la.read_row(tY, 0, ks);
    };
    // Y^T fragments of update k-step q for the key-feature tiles 2 h, 2 h + 1
    auto read_yt = [&](int q, int h) __attribute__((always_inline)) {
#pragma unroll
      for (int t = 2 * h; t < 2 * h + 2; t++) yt[q][t] = la.read_cols(tY, 16 * q, t);
    };

    // ---- phases 1 and 2, one k-step of each per slot so that an X fragment is read from LDS once:
    //   1  W^T[dv][r] = sum_dk State[dk][dv] X[r][dk] from the state in registers
    //   2  S^T[c][r]  = sum_k Y[c][k] X[r][k]
    // Side work: the next state operand; lambda^B on a state tile once both its operands are made; the
    // update weights on Z; the direct loads of block it + NBUF - 1.
    f32x16 inter = zero16(), sd = zero16();
    bf16x8 sa = sa_first;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      inter = mfma(sa, xa[ks], inter);
      sd = mfma(ya[ks], xa[ks], sd);
      if (ks + AHEAD < KS) read_xy(ks + AHEAD);
      if (ks + 1 < KS) { sa = state_operand(ks + 1); pin(sa); }
      if (ks < NDMA) loader.issue_one(sAhead, doff, ks);
      if (ks < 2) zf[ks] = la.read_cols(tZ, 16 * ks, dvt);
      if (ks >= 2 && (ks & 1) == 0) {   // state tile ks / 2 - 1: both operands made in slots <= ks - 1
        const int t = (ks >> 1) - 1;
#pragma unroll
        for (int v = 0; v < 16; v++) kv[t][v] *= lamB;
        pin(kv[t]);
      }
      if (ks == 3 || ks == 5) {
        const int q = (ks - 3) >> 1;
        zd[q] = decay.apply(zf[q], 16 * q);
        pin(zd[q]);
      }
      if (ks == KS - 1) read_yt(0, 0);
      pin(inter);
      pin(sd);
      LA2_SLOT_END();
    }
    {
#pragma unroll
      for (int v = 0; v < 16; v++) kv[NT - 1][v] *= lamB;
      pin(kv[NT - 1]);
      // the carried part takes the decay at this lane's position
#pragma unroll
      for (int v = 0; v < 16; v++) inter[v] *= inter_scale;
      pin(inter);
    }
    // ---- phase 3
    bf16x8 pd[2];
#pragma unroll
    for (int s4 = 0; s4 < 4; s4++) {   // slot s4: k-step q = s4 / 2, key-feature tiles 2 h, 2 h + 1, h = s4 % 2
      const int q = s4 >> 1, h = s4 & 1;
#pragma unroll
      for (int t = 2 * h; t < 2 * h + 2; t++) kv[t] = mfma(yt[q][t], zd[q], kv[t]);
      if (s4 + 1 < 4) read_yt((s4 + 1) >> 1, (s4 + 1) & 1);
#pragma unroll
      for (int e = 0; e < 4; e++) pd[q][4 * h + e] = (__bf16)(sd[8 * q + 4 * h + e] * dg[8 * q + 4 * h + e]);
      pin(pd[q]);
#pragma unroll
      for (int t = 2 * h; t < 2 * h + 2; t++) pin(kv[t]);
      LA2_SLOT_END();
    }
    if (has_next) {
      __builtin_amdgcn_s_waitcnt(WAIT_NEXT_TILES);
      loader.zero_tail(sNext, nb);
      lds_barrier();
#pragma unroll
      for (int ks = 0; ks < AHEAD; ks++) {
        xa[ks] = la.read_row(sNext[xi], 0, ks);
        ya[ks] = la.read_row(sNext[yi], 0, ks);
      }
    }
    LA2_SLOT_END();
    // ---- phase 4 and the block's output
#pragma unroll
    for (int q = 0; q < 2; q++) inter = mfma(zf[q], pd[q], inter);
    sa_first = state_operand(0);
    pin(sa_first);
    pin(inter);
    LA2_SLOT_END();
#pragma unroll
    for (int g = 0; g < 4; g++) {
      bf16x4 pk;
#pragma unroll
      for (int e = 0; e < 4; e++) pk[e] = (__bf16)inter[4 * g + e];
      *reinterpret_cast<bf16x4*>(stage + l32 * LW + 8 * (g ^ ((l32 >> 2) & 3)) + 4 * hh) = pk;
    }
#pragma unroll
    for (int i = 0; i < NST; i++) {
      const int id = l + 64 * i;
      const int row = id >> 2, cc = id & 3;
      const i32x4 v = *reinterpret_cast<const i32x4*>(stage + row * LW + 8 * (cc ^ ((row >> 2) & 3)));
      const uint32_t off = ((uint32_t)(blk * B + row) * stride_n + (uint32_t)(32 * dvt + cc * 8)) * 2u;
      __builtin_amdgcn_raw_buffer_store_b128(v, bw, off, 0, 0);
    }
    LA2_SLOT_END();
    return has_next;
  };
  for (int it = 0;; it += NBUF) {   // unrolled by the number of buffers: compile-time buffer index
    if (!block_step(std::integral_constant<int, 0>{}, it)) break;
    if (!block_step(std::integral_constant<int, 1>{}, it + 1)) break;
    if (!block_step(std::integral_constant<int, 2>{}, it + 2)) break;
    if (NBUF > 3 && !block_step(std::integral_constant<int, (NBUF > 3 ? 3 : 0)>{}, it + 3)) break;
    if (NBUF > 4 && !block_step(std::integral_constant<int, (NBUF > 4 ? 4 : 0)>{}, it + 4)) break;
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the dummy direct loads before the LDS is given up
  // state after the chain's last block, if the caller wants it (the update ran on every block)
  float* gf = which ? p.fin[1] : p.fin[0];
  if (gf != nullptr && (REV ? chunk == 0 : chunk == p.nchunks - 1)) {
    gf += (int64_t)chain * (D * D);
    const bool trf = (p.fin_transposed >> which) & 1;
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) gf[state_index<D>(dvt, l32, hh, t, v, trf)] = kv[t][v];
  }
#undef LA2_SLOT_END
  };
  if (TWIN && which == 1) run(std::integral_constant<int, 1>{});
  else run(std::integral_constant<int, 0>{});
}

// Local state of every chunk that has a successor: forward sum_c lambda^(C-1-c) y_c^T z_c over the
// chunk's positions c, reverse sum_c lambda^c y_c^T z_c.  Written fp32 row-major [dk][dv].  Same
// streaming and the same state-update step as the scan kernel, without X, scores or outputs.
template <int D, bool REV>
__global__ __launch_bounds__(kThreads, 2) void chunk_state_bf16_kernel(ScanParams p) {
  using C = Cfg<D>;
  constexpr int NT = C::NT, TILE = C::TILE;
  __shared__ __attribute__((aligned(1024))) __bf16 sT0[2][TILE];   // [Y, Z]
  __shared__ __attribute__((aligned(1024))) __bf16 sT1[2][TILE];

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int dvt = w % NT;
  const int chain = blockIdx.x / p.nchunks, chunk = blockIdx.x % p.nchunks;
  if (REV ? (chunk == 0) : (chunk == p.nchunks - 1)) return;  // no successor needs it
  const int bi = chain / p.heads, hi = chain % p.heads;
  const int64_t base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h;
  const int n = p.n;
  const float l2 = log2f(p.lambda[hi]);
  const int nblocks = (n + kB - 1) / kB;
  const int cb = p.chunk_tokens / kB;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);
  const int nblk = blk_hi - blk_lo;

  TileLoader<D, 2> loader(w, l, n, (uint32_t)p.stride_n);
  loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(p.y[0]) + base);
  loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(p.z[0]) + base);
  const LaneAddr<D> la(l);
  const UpdateDecay<REV> decay(l2, hh);
  const float lamB = exp2f(l2 * (float)kB);

  f32x16 kv[NT];
#pragma unroll
  for (int t = 0; t < NT; t++) kv[t] = zero16();

  if (nblk > 0) {
    const int b0 = REV ? blk_hi - 1 : blk_lo;
    loader.issue(sT0, b0);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    loader.zero_tail(sT0, b0);
  }
  __syncthreads();

  auto block_step = [&](auto cur_tag, int it) {
    constexpr int cur = decltype(cur_tag)::value;
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    const bool has_next = it + 1 < nblk;
    const int nb = REV ? blk - 1 : blk + 1;
    if (has_next) loader.issue(cur ? sT0 : sT1, nb);
    const __bf16* tY = cur ? sT1[0] : sT0[0];
    const __bf16* tZ = cur ? sT1[1] : sT0[1];
    bf16x8 zf[4], yt[NT][4];   // [16-row k-step of the block]
#pragma unroll
    for (int k = 0; k < 4; k++) {
      zf[k] = la.read_cols(tZ, 16 * k, dvt);
#pragma unroll
      for (int t = 0; t < NT; t++) yt[t][k] = la.read_cols(tY, 16 * k, t);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) kv[t][v] *= lamB;
#pragma unroll
    for (int k = 0; k < 4; k++) {
      const bf16x8 zd = decay.apply(zf[k], 16 * k);
#pragma unroll
      for (int t = 0; t < NT; t++) kv[t] = mfma(yt[t][k], zd, kv[t]);
    }
    if (has_next) {
      __builtin_amdgcn_s_waitcnt(0x0F70);
      loader.zero_tail(cur ? sT0 : sT1, nb);
      lds_barrier();
    }
  };
  for (int it = 0; it < nblk; it += 2) {
    block_step(std::integral_constant<int, 0>{}, it);
    if (it + 1 < nblk) block_step(std::integral_constant<int, 1>{}, it + 1);
  }

  if (w < NT) {   // for d = 64 waves w and w + 2 hold the same slice
    float* gs = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) gs[state_index<D>(dvt, l32, hh, t, v, false)] = kv[t][v];
  }
}

// In place: states[chain][j] (local state of chunk j) -> start state of chunk j.
//   forward: G_0 = 0, G_{j+1} = lambda^C G_j + L_j        reverse: G_last = 0, G_{j-1} = lambda^C G_j + L_j
// The chunk processed first starts from init (element e read at its transposed place if init_tr) or 0.
// The carried state decays by lambda^(chunk length): all chunks are chunk_tokens long except the last
// one of the sequence, which a reverse scan passes first.
__global__ void state_scan_kernel(float* states, const float* lambda, int heads, int nchunks, int chunk_tokens,
                                  int dd, int reverse, const float* init, int init_tr, int d, int n) {
  const int chain = blockIdx.y;
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= dd) return;
  const float l2 = log2f(lambda[chain % heads]);
  const float lamFull = exp2f(l2 * (float)chunk_tokens);
  const float lamLast = exp2f(l2 * (float)(n - (nchunks - 1) * chunk_tokens));
  float* s = states + (int64_t)chain * nchunks * dd + e;
  float g = 0.f;
  if (init != nullptr) g = init[(int64_t)chain * dd + (init_tr ? (e % d) * d + e / d : e)];
  for (int i = 0; i < nchunks; i++) {
    const int j = reverse ? nchunks - 1 - i : i;
    const bool last = (i == nchunks - 1);
    const float loc = last ? 0.f : s[(int64_t)j * dd];
    s[(int64_t)j * dd] = g;
    g = (j == nchunks - 1 ? lamLast : lamFull) * g + loc;
  }
}


// ------------------------------------------------------------------------------------------------------
// Left-product form for comparison: O = [(Q K^T) * M] V computed tile by tile over ALL earlier key blocks
// (the O(n^2 d) evaluation that the block recurrence replaces; Sec. 3.1 eq. (1) with the decay mask of
// Sec. 3.2).  Forward only, bf16.  One workgroup per (chain, 128 query rows); wave w owns query rows
// 32 w .. 32 w + 31 and all value features; the key and value blocks (64 positions) stream through LDS,
// double buffered.  Same MFMA operand layouts, LDS tile layout and mask tables as the scan kernels.
template <int D>
__global__ __launch_bounds__(kThreads, 1) void left_product_bf16_kernel(ScanParams p) {
  using C = Cfg<D>;
  constexpr int KS = C::KS, NT = C::NT, TILE = C::TILE, LW = C::LW;
  constexpr int QB = 128;   // query rows per workgroup
  __shared__ __attribute__((aligned(1024))) __bf16 sT[2][2][TILE];   // [buffer][K, V]
  __shared__ __attribute__((aligned(16))) __bf16 sW[4][32 * LW];

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int nqb = (p.n + QB - 1) / QB;
  const int chain = blockIdx.x / nqb;
  const int qb = nqb - 1 - (int)(blockIdx.x % nqb);   // long rows of the triangle first
  const int bi = chain / p.heads, hi = chain % p.heads;
  const int64_t base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h;
  const int n = p.n;
  const uint32_t stride_n = (uint32_t)p.stride_n;
  const uint32_t chain_bytes = ((uint32_t)(n - 1) * stride_n + D) * 2u;
  const __amdgpu_buffer_rsrc_t bw = make_rsrc(reinterpret_cast<__bf16*>(p.w[0]) + base, chain_bytes);
  const float l2 = log2f(p.lambda[hi]);

  // this lane's query row as B-operand fragments (natural k-order), straight from global memory
  const int qrow = qb * QB + 32 * w + l32;
  bf16x8 xf[KS];
  {
    const __bf16* gq = reinterpret_cast<const __bf16*>(p.x[0]) + base + (int64_t)min(qrow, n - 1) * stride_n + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      xf[ks] = *reinterpret_cast<const bf16x8*>(gq + 16 * ks);
      if (qrow >= n) {
#pragma unroll
        for (int j = 0; j < 8; j++) xf[ks][j] = (__bf16)0.f;
      }
    }
  }
  // decay mask tables (score tile S^T[c][r]: lane = query row r = l32, element v = key row cc[v])
  float dg[16], od[16];
#pragma unroll
  for (int v = 0; v < 16; v++) {
    const int cc = 8 * (v >> 2) + 4 * hh + (v & 3);
    const int e = l32 - cc;
    dg[v] = (e >= 0) ? exp2f(l2 * (float)e) : 0.f;
    od[v] = exp2f(l2 * (float)(e + 32));
  }

  TileLoader<D, 2> loader(w, l, n, stride_n);
  loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(p.y[0]) + base);
  loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const __bf16*>(p.z[0]) + base);
  const LaneAddr<D> la(l);

  f32x16 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; t++) acc[t] = zero16();

  // key blocks 0 .. jmax reach this query block
  const int nkb = (n + kB - 1) / kB;
  const int jmax = min((qb * QB + QB - 1) / kB, nkb - 1);
  loader.issue(sT[0], 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  loader.zero_tail(sT[0], 0);
  __syncthreads();
  for (int j = 0; j <= jmax; j++) {
    const int cur = j & 1;
    if (j < jmax) loader.issue(sT[cur ^ 1], j + 1);
    const __bf16* tK = sT[cur][0];
    const __bf16* tV = sT[cur][1];
#pragma unroll
    for (int kt = 0; kt < 2; kt++) {
      // distance between this wave's first query row and the key tile's first row: a multiple of 32
      const int dist = qb * QB + 32 * w - (j * kB + 32 * kt);
      if (dist < 0) continue;   // wave-uniform: the whole tile is above the diagonal
      f32x16 st = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ks++) st = mfma(la.read_row(tK, kt, ks), xf[ks], st);
      bf16x8 pf[2];
      if (dist == 0) {
#pragma unroll
        for (int v = 0; v < 16; v++) pf[v >> 3][v & 7] = (__bf16)(st[v] * dg[v]);
      } else {
        const float far = fast_exp2(l2 * (float)(dist - 32));
#pragma unroll
        for (int v = 0; v < 16; v++) pf[v >> 3][v & 7] = (__bf16)(st[v] * (far * od[v]));
      }
#pragma unroll
      for (int t = 0; t < NT; t++)
#pragma unroll
        for (int q = 0; q < 2; q++) acc[t] = mfma(la.read_cols(tV, 32 * kt + 16 * q, t), pf[q], acc[t]);
    }
    if (j < jmax) {
      __builtin_amdgcn_s_waitcnt(0x0F70);   // this wave's part of the next blocks has landed
      loader.zero_tail(sT[cur ^ 1], j + 1);
    }
    __syncthreads();
  }

  // output: value-feature tile by tile through this wave's staging area, 16-byte stores
  __bf16* stage = sW[w];
#pragma unroll
  for (int t = 0; t < NT; t++) {
#pragma unroll
    for (int g = 0; g < 4; g++) {
      bf16x4 pk;
#pragma unroll
      for (int e = 0; e < 4; e++) pk[e] = (__bf16)acc[t][4 * g + e];
      *reinterpret_cast<bf16x4*>(stage + l32 * LW + 8 * (g ^ ((l32 >> 2) & 3)) + 4 * hh) = pk;
    }
#pragma unroll
    for (int i = 0; i < 2; i++) {
      const int id = l + 64 * i;
      const int row = id >> 2, cc = id & 3;
      const i32x4 v = *reinterpret_cast<const i32x4*>(stage + row * LW + 8 * (cc ^ ((row >> 2) & 3)));
      const uint32_t off = ((uint32_t)(qb * QB + 32 * w + row) * stride_n + (uint32_t)(32 * t + cc * 8)) * 2u;
      __builtin_amdgcn_raw_buffer_store_b128(v, bw, off, 0, 0);
    }
  }
}

}  // namespace

int block_size_bf16(int) { return kB; }




hipError_t launch_scan_bf16(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (int64_t)p.batch * p.heads * p.nchunks * p.nscan;
  if (grid == 0 || p.n == 0) return hipSuccess;
  dim3 g((unsigned)grid), b(kThreads);
  // the half-block kernel measured faster at every launch size, also at one workgroup per compute unit;
  // it is also the only d = 128 kernel that takes start states and hands out final states
  const bool with_state = p.init[0] || p.init[1] || p.fin[0] || p.fin[1];
  const bool half = p.variant != 1 || with_state;
  if (head_dim == 128 && half && p.chunk_tokens % kBH == 0) {
    const bool twin = p.nscan == 2 && p.y[1] == p.z[0] && p.z[1] == p.y[0];
    // Three tile buffers in every case.  More buffers (5 for a plain, 4 for a twin workgroup that has the
    // compute unit to itself) measured no faster: such launches are bound by the workgroup's own
    // instruction stream, not by the bytes in flight.
    if (twin) {
      dim3 gt((unsigned)(grid / 2)), bt(512);
      if (reverse) hipLaunchKernelGGL((scan_bf16_half_kernel<true, true, 3>), gt, bt, 0, s, p);
      else         hipLaunchKernelGGL((scan_bf16_half_kernel<false, true, 3>), gt, bt, 0, s, p);
    } else {
      if (reverse) hipLaunchKernelGGL((scan_bf16_half_kernel<true, false, 3>), g, b, 0, s, p);
      else         hipLaunchKernelGGL((scan_bf16_half_kernel<false, false, 3>), g, b, 0, s, p);
    }
  } else if (head_dim == 128) {
    if (reverse) hipLaunchKernelGGL((scan_bf16_kernel<128, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((scan_bf16_kernel<128, false>), g, b, 0, s, p);
  } else {
    if (reverse) hipLaunchKernelGGL((scan_bf16_kernel<64, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((scan_bf16_kernel<64, false>), g, b, 0, s, p);
  }
  return hipGetLastError();
}

hipError_t launch_chunk_states_bf16(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (int64_t)p.batch * p.heads * p.nchunks;
  if (grid == 0 || p.n == 0) return hipSuccess;
  dim3 g((unsigned)grid), b(kThreads);
  if (head_dim == 128) {
    if (reverse) hipLaunchKernelGGL((chunk_state_bf16_kernel<128, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((chunk_state_bf16_kernel<128, false>), g, b, 0, s, p);
  } else {
    if (reverse) hipLaunchKernelGGL((chunk_state_bf16_kernel<64, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((chunk_state_bf16_kernel<64, false>), g, b, 0, s, p);
  }
  return hipGetLastError();
}

hipError_t launch_state_scan(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int chains = p.batch * p.heads;
  if (chains == 0 || p.n == 0) return hipSuccess;
  const int dd = head_dim * head_dim;
  dim3 g((dd + 255) / 256, chains), b(256);
  hipLaunchKernelGGL(state_scan_kernel, g, b, 0, s, p.states, p.lambda, p.heads, p.nchunks, p.chunk_tokens, dd,
                     reverse ? 1 : 0, p.init[0], p.init_transposed & 1, head_dim, p.n);
  return hipGetLastError();
}

hipError_t launch_left_product_bf16(int head_dim, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (int64_t)p.batch * p.heads * ((p.n + 127) / 128);
  if (grid == 0 || p.n == 0) return hipSuccess;
  dim3 g((unsigned)grid), b(kThreads);
  if (head_dim == 128) hipLaunchKernelGGL((left_product_bf16_kernel<128>), g, b, 0, s, p);
  else                 hipLaunchKernelGGL((left_product_bf16_kernel<64>), g, b, 0, s, p);
  return hipGetLastError();
}

}  // namespace la2
