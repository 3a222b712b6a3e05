// bf16 MFMA kernels for the decayed causal scan (Algorithm 1; both loops of Algorithm 2), gfx950.
//
// One workgroup (4 waves) walks the blocks (B = 64 positions) of one sequence chunk of one
// (batch, head) chain.  The X, Y, Z tiles of the NEXT block stream from HBM straight into LDS
// (global_load_lds, no registers) while the current block is computed; the fp32 running state
// (D x D) lives in MFMA accumulator registers split over the four waves, with a bf16 copy
// (transposed) in LDS as the operand of the inter-block product.  Wave w owns block rows
// 32 (w / 2) .. +31 and one half of the value features from the score tile to the output, so the
// masked scores never leave registers.  All products use v_mfma_f32_32x32x16_bf16, fp32 accumulate.
//
// MFMA 32x32x16 lane layouts (wave64, lane l, l32 = l % 32, hh = l / 32):
//   A[m][k]: m = l32, k = 8 hh + j (j = 0..7)     B[k][n]: n = l32, k = 8 hh + j
//   C[m][n]: n = l32, m = 8 (v / 4) + 4 hh + v % 4 (v = 0..15)
// Outputs are accumulated TRANSPOSED (C rows = value feature, C columns = position) so that each
// lane ends up with 4 consecutive features of one position, which packs into 8-byte LDS writes.
//
// Tile layout in LDS: row-major, UNPADDED (the direct loads write 1 KiB contiguous per wave
// instruction), with the 16-byte chunk index of every row XOR-swizzled by swz(row) so that both the
// 16-byte row reads (lanes = rows) and the transposing reads (4 rows x 32 bytes per 16 lanes) are
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

constexpr int kB = 64;        // block size (positions per block)
constexpr int kThreads = 256; // 4 waves

template <int D>
struct Tile {
  static constexpr int LD = D + 8;       // padded LDS row stride (elements): 16 consecutive rows cover all 64 banks
  static constexpr int NT = D / 32;      // 32-wide tiles along a feature dimension
  static constexpr int KS = D / 16;      // MFMA k-steps along a feature dimension
  static constexpr int CPR = D / 8;      // 16-byte chunks per row
  static constexpr int LOADS = kB * CPR / kThreads;  // 16-byte chunks per thread per tile
  // fp32 state ownership: the NT x NT grid of 32 x 32 state tiles is split over the 4 waves; a wave
  // holds SC value-feature tiles of ONE key-feature tile, so it decays one Y fragment per k-step.
  static constexpr int SC = NT * NT / 4;  // state tiles per wave (d=128: 4, d=64: 1)
  static constexpr int WPT = NT / SC;     // waves sharing one key-feature tile (d=128: 1, d=64: 2)
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

// Raw buffer descriptor over one chain's rows: loads beyond `bytes` return 0 and stores beyond it
// are dropped, which is how ragged last blocks are masked without branches.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00027000);
}

// Transposing LDS read.  Within each group of 16 lanes, lane s passes the address of 4 consecutive
// elements of row (s / 4), columns 4 (s % 4) .. +3 of a 4 x 16 sub-matrix; lane s receives the 4
// rows of column s.
__device__ __forceinline__ s16x4 lds_read_tr(const __bf16* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
}

// Operand fragment for a contraction over tile ROWS: lane (l32, hh) receives, for column
// col0 + l32 of the row-major LDS tile, the rows row_lo + 0..3 (elements 0..3) and row_hi + 0..3
// (elements 4..7).  `lane_off` = (l % 16 / 4) * LD + 16 * (l / 16 % 2) + 4 * (l % 4).
template <int LD>
__device__ __forceinline__ bf16x8 read_cols(const __bf16* tile, int row_lo, int row_hi, int col0, int lane_off) {
  union { struct { s16x4 lo, hi; } s; bf16x8 v; } u;
  u.s.lo = lds_read_tr(tile + row_lo * LD + col0 + lane_off);
  u.s.hi = lds_read_tr(tile + row_hi * LD + col0 + lane_off);
  return u.v;
}

template <int D>
__device__ __forceinline__ void load_tile_regs(i32x4 (&r)[Tile<D>::LOADS], __amdgpu_buffer_rsrc_t rs,
                                               uint32_t stride_n, int row0, int tid) {
  constexpr int CPR = Tile<D>::CPR;
#pragma unroll
  for (int i = 0; i < Tile<D>::LOADS; i++) {
    const int id = tid + kThreads * i;
    const uint32_t off = ((uint32_t)(row0 + id / CPR) * stride_n + (uint32_t)(id % CPR) * 8u) * 2u;
    r[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
  }
}

template <int D>
__device__ __forceinline__ void store_tile_lds(__bf16* s, const i32x4 (&r)[Tile<D>::LOADS], int tid) {
  constexpr int CPR = Tile<D>::CPR;
#pragma unroll
  for (int i = 0; i < Tile<D>::LOADS; i++) {
    const int id = tid + kThreads * i;
    *reinterpret_cast<i32x4*>(s + (id / CPR) * Tile<D>::LD + (id % CPR) * 8) = r[i];
  }
}

// state <- lambda^B state + (decay(Y))^T Z over one block held in LDS (contraction over the block's
// rows).  Forward: row c is weighted lambda^(B-1-c); reverse: lambda^c.  The operand fragments of
// k-step ks+1 are requested from LDS before the MFMAs of k-step ks are issued.
template <int D, bool REV>
__device__ __forceinline__ void state_update(f32x16 (&kv)[Tile<D>::SC], const __bf16* sY, const __bf16* sZ,
                                             float l2, int w, int hh, int lane_off) {
  using T = Tile<D>;
  constexpr int LD = T::LD, SC = T::SC;
  const int ycol = 32 * (w / T::WPT), zcol = 32 * ((w % T::WPT) * SC);
  const float lamB = exp2f(l2 * (float)kB);
#pragma unroll
  for (int b = 0; b < SC; b++)
#pragma unroll
    for (int v = 0; v < 16; v++) kv[b][v] *= lamB;
  float fj[8];
#pragma unroll
  for (int j = 0; j < 8; j++) fj[j] = exp2f(l2 * (float)(REV ? j : 7 - j));
  bf16x8 yr[2], zf[2][SC];
  {
    const int c0 = 8 * hh;
    yr[0] = read_cols<LD>(sY, c0, c0 + 4, ycol, lane_off);
#pragma unroll
    for (int b = 0; b < SC; b++) zf[0][b] = read_cols<LD>(sZ, c0, c0 + 4, zcol + 32 * b, lane_off);
  }
#pragma unroll
  for (int ks = 0; ks < kB / 16; ks++) {
    const int cur = ks & 1, nxt = cur ^ 1;
    if (ks + 1 < kB / 16) {
      const int c1 = 16 * (ks + 1) + 8 * hh;
      yr[nxt] = read_cols<LD>(sY, c1, c1 + 4, ycol, lane_off);
#pragma unroll
      for (int b = 0; b < SC; b++) zf[nxt][b] = read_cols<LD>(sZ, c1, c1 + 4, zcol + 32 * b, lane_off);
    }
    const int c0 = 16 * ks + 8 * hh;  // this lane's 8 rows: c0 .. c0+7
    const float fb = fast_exp2(l2 * (float)(REV ? c0 : kB - 8 - c0));
    bf16x8 af;
#pragma unroll
    for (int j = 0; j < 8; j++) af[j] = (__bf16)((float)yr[cur][j] * (fb * fj[j]));
#pragma unroll
    for (int b = 0; b < SC; b++) kv[b] = mfma(af, zf[cur][b], kv[b]);
  }
}

// fp32 state element (b, v) of wave w sits at key feature dk, value feature dv:
//   dk = 32 (w / WPT) + 8 (v / 4) + 4 hh + v % 4,   dv = 32 ((w % WPT) SC + b) + l32
// The transposed bf16 copy sS[dv][dk] is written 16 bytes at a time: lanes l and l + 32 (same dv)
// first exchange halves (v_permlane32_swap) so that lane hh = 0 holds key features 0..15 and lane
// hh = 1 holds 16..31 of the wave's 32-row key tile.
template <int D>
__device__ __forceinline__ void state_to_lds(__bf16* sS, const f32x16 (&kv)[Tile<D>::SC], int w, int l32, int hh) {
  using T = Tile<D>;
  constexpr int LD = T::LD, SC = T::SC;
  typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
  typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
#pragma unroll
  for (int b = 0; b < SC; b++) {
    unsigned pk[4][2];   // pk[g][i]: bf16 pair (4 g' + 2 i, +1) of key features 8 g + 4 hh + ...
#pragma unroll
    for (int g = 0; g < 4; g++)
#pragma unroll
      for (int i = 0; i < 2; i++) {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
        union { bf16x2 h; unsigned u; } cv;
        cv.h[0] = (__bf16)kv[b][4 * g + 2 * i];
        cv.h[1] = (__bf16)kv[b][4 * g + 2 * i + 1];
        pk[g][i] = cv.u;
      }
    __bf16* row = sS + (32 * ((w % T::WPT) * SC + b) + l32) * LD + 32 * (w / T::WPT) + 16 * hh;
#pragma unroll
    for (int g = 0; g < 2; g++) {
      // swap(g, g + 2): lane hh = 0 ends with features 8 g .. 8 g + 7, lane hh = 1 with 16 + 8 g .. + 7
      const u32x2 s0 = __builtin_amdgcn_permlane32_swap(pk[g][0], pk[g + 2][0], false, false);
      const u32x2 s1 = __builtin_amdgcn_permlane32_swap(pk[g][1], pk[g + 2][1], false, false);
      const u32x4 chunk = {s0[0], s1[0], s0[1], s1[1]};
      *reinterpret_cast<u32x4*>(row + 8 * g) = chunk;
    }
  }
}

template <int D>
__device__ __forceinline__ int state_index(int w, int l32, int hh, int b, int v) {
  using T = Tile<D>;
  const int dk = 32 * (w / T::WPT) + 8 * (v >> 2) + 4 * hh + (v & 3);
  const int dv = 32 * ((w % T::WPT) * T::SC + b) + l32;
  return dk * D + dv;
}

// ---- swizzled, unpadded tiles (filled by direct global->LDS loads) -------------------------------------
// Physical 16-byte chunk of logical chunk c in row `row`: c ^ swz<D>(row).
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
// flight across the barrier.  The "memory" clobber keeps the compiler from moving LDS accesses
// across it.  Waves that need their own direct loads visible wait for vmcnt(0) before calling this.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ void dma16(const __bf16* g, __bf16* lds_wave_base) {
  // each lane copies 16 bytes from its own global address to lds_wave_base + 16 * lane
  __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)g,
                                   (void __attribute__((address_space(3)))*)lds_wave_base, 16, 0, 0);
}

template <int D, bool REV>
__global__ __launch_bounds__(kThreads, 1) void scan_bf16_kernel(ScanParams p) {
  using T = Tile<D>;
  constexpr int LD = T::LD, KS = T::KS, SC = T::SC, CPR = T::CPR;
  constexpr int NH = D / 64;                 // output tiles (32 value features each) per wave
  constexpr int TILE = kB * D;               // elements per tile
  constexpr int DMA_PER_TILE = TILE / 512;   // wave instructions (1 KiB each) per tile
  constexpr int DMA_PER_WAVE = DMA_PER_TILE / 4;
  constexpr int LW = D / 2 + 8;              // staging row stride (elements)
  // two tile buffers as two distinct LDS objects: [X, Y, Z] each
  __shared__ __attribute__((aligned(1024))) __bf16 sT0[3][TILE];
  __shared__ __attribute__((aligned(1024))) __bf16 sT1[3][TILE];
  __shared__ __attribute__((aligned(16))) __bf16 sS[D * LD];
  __shared__ __attribute__((aligned(16))) __bf16 sW[4][32 * LW];

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int rg = w >> 1, ch = w & 1;         // row group (32 rows) and value-feature half of this wave
  // dual launch: even workgroups run scan 0, odd workgroups scan 1 of the same (chain, chunk)
  const int which = (p.nscan == 2) ? (int)(blockIdx.x & 1) : 0;
  const int wg = (p.nscan == 2) ? (int)(blockIdx.x >> 1) : (int)blockIdx.x;
  const int chain = wg / p.nchunks, chunk = wg % p.nchunks;
  const int bi = chain / p.heads, hi = chain % p.heads;
  const int64_t base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h;
  const __bf16* gx = reinterpret_cast<const __bf16*>(which ? p.x[1] : p.x[0]) + base;
  const __bf16* gy = reinterpret_cast<const __bf16*>(which ? p.y[1] : p.y[0]) + base;
  const __bf16* gz = reinterpret_cast<const __bf16*>(which ? p.z[1] : p.z[0]) + base;
  const int n = p.n;
  const int64_t stride_n = p.stride_n;
  const uint32_t chain_bytes = ((uint32_t)(n - 1) * (uint32_t)stride_n + D) * 2u;
  const __amdgpu_buffer_rsrc_t bw =
      make_rsrc(reinterpret_cast<__bf16*>(which ? p.w[1] : p.w[0]) + base, chain_bytes);
  const float l2 = log2f(p.lambda[hi]);

  const int nblocks = (n + kB - 1) / kB;
  const int cb = p.chunk_tokens / kB;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);
  if (blk_lo >= blk_hi) return;

  // ---- direct-load plan: this wave issues instructions j = DMA_PER_WAVE w + i of every tile; lane l
  // of instruction j fills LDS chunk q = 64 j + l, i.e. row q / CPR, physical chunk q % CPR.
  int dma_row[DMA_PER_WAVE], dma_col[DMA_PER_WAVE];
#pragma unroll
  for (int i = 0; i < DMA_PER_WAVE; i++) {
    const int q = 64 * (DMA_PER_WAVE * w + i) + l;
    dma_row[i] = q / CPR;
    dma_col[i] = 8 * ((q % CPR) ^ swz<D>(q / CPR));   // logical column held by that physical chunk
  }
  auto issue_tile_loads = [&](auto buf_tag, int blk) {
    __bf16 (*sT)[TILE] = decltype(buf_tag)::value ? sT1 : sT0;
#pragma unroll
    for (int i = 0; i < DMA_PER_WAVE; i++) {
      const int pos = min(blk * kB + dma_row[i], n - 1);   // rows past the end are re-zeroed below
      // 32-bit byte offset from the (wave-uniform) chain base; the host checked that a chain spans < 4 GiB
      const uint32_t off = ((uint32_t)pos * (uint32_t)stride_n + (uint32_t)dma_col[i]) * 2u;
      const int dst = 512 * (DMA_PER_WAVE * w + i);
      dma16(reinterpret_cast<const __bf16*>(reinterpret_cast<const char*>(gx) + off), &sT[0][dst]);
      dma16(reinterpret_cast<const __bf16*>(reinterpret_cast<const char*>(gy) + off), &sT[1][dst]);
      dma16(reinterpret_cast<const __bf16*>(reinterpret_cast<const char*>(gz) + off), &sT[2][dst]);
    }
  };
  // after this wave's loads have landed: zero the rows of a ragged last block
  auto zero_tail_rows = [&](auto buf_tag, int blk) {
    __bf16 (*sT)[TILE] = decltype(buf_tag)::value ? sT1 : sT0;
    if ((blk + 1) * kB > n) {
#pragma unroll
      for (int i = 0; i < DMA_PER_WAVE; i++) {
        if (blk * kB + dma_row[i] >= n) {
          const int dst = 512 * (DMA_PER_WAVE * w + i) + 8 * l;
          const i32x4 z = {0, 0, 0, 0};
          *reinterpret_cast<i32x4*>(&sT[0][dst]) = z;
          *reinterpret_cast<i32x4*>(&sT[1][dst]) = z;
          *reinterpret_cast<i32x4*>(&sT[2][dst]) = z;
        }
      }
    }
  };

  // ---- running state: registers (fp32) + LDS copy (bf16, transposed)
  f32x16 kv[SC];
  if (p.states != nullptr) {
    const float* gs = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
    const bool tr = (p.state_transposed >> which) & 1;
#pragma unroll
    for (int b = 0; b < SC; b++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int idx = state_index<D>(w, l32, hh, b, v);          // dk * D + dv
        kv[b][v] = gs[tr ? (idx % D) * D + idx / D : idx];
      }
  } else {
#pragma unroll
    for (int b = 0; b < SC; b++) kv[b] = zero16();
  }
  state_to_lds<D>(sS, kv, w, l32, hh);

  // ---- per-lane constants.  This lane's position is row r = 32 rg + l32 of the block; accumulator
  // element v of a score tile belongs to key row 32 ct + cc[v], cc[v] = 8 (v / 4) + 4 hh + v % 4.
  const int r = 32 * rg + l32;
  // weight of the carried state: forward lambda^(r+1), reverse lambda^(B-r)
  const float inter_scale = exp2f(l2 * (float)(REV ? kB - r : r + 1));
  // Key tiles (32 rows) this wave's rows can see: tile A always, tile B for the later row group.
  //   forward: rg 0 -> A = tile 0 (diagonal);  rg 1 -> A = tile 0 (earlier), B = tile 1 (diagonal)
  //   reverse: rg 0 -> A = tile 0 (diagonal), B = tile 1 (later);  rg 1 -> A = tile 1 (diagonal)
  const bool two_tiles = REV ? (rg == 0) : (rg == 1);   // wave-uniform
  const int ctA = REV ? rg : 0, ctB = 1;
  // decay mask lambda^|r-c| with non-negative exponents only (lambda^r * lambda^-c would overflow):
  //   diagonal tile:  lambda^(l32 - cc[v]) on the causal side, else 0   (reverse: l32 and cc[v] swapped)
  //   other tile:     lambda^(l32 + 32 - cc[v])
  float mA[16], mB[16];
#pragma unroll
  for (int v = 0; v < 16; v++) {
    const int cc = 8 * (v >> 2) + 4 * hh + (v & 3);
    const int e = REV ? cc - l32 : l32 - cc;
    const float dg = (e >= 0) ? exp2f(l2 * (float)e) : 0.f;
    const float od = exp2f(l2 * (float)(e + 32));
    mA[v] = (ctA == rg) ? dg : od;
    mB[v] = (ctB == rg) ? dg : od;
  }
  // state-update row weights: this lane's rows of k-step ks are c = 16 ks + 8 hh + j; forward
  // lambda^(B-1-c), reverse lambda^c, split as fks(ks) * fj[j] with both exponents non-negative
  float fj[8];
#pragma unroll
  for (int j = 0; j < 8; j++) fj[j] = exp2f(l2 * (float)(REV ? j + 8 * hh : 7 - j + 8 * (1 - hh)));
  const float lamB = exp2f(l2 * (float)kB);
  // row reads of X / Y (16 bytes = logical chunk 2 ks + hh of row 32 t + l32): element offset
  // 32 t D + (rowk ^ 16 ks), rowk = l32 D + 8 (hh ^ swz(l32))   [swz(32 t + l32) == swz(l32)]
  const int rowk = l32 * D + 8 * (hh ^ swz<D>(l32));
  // transposing reads (4 rows x 16 columns per 16 lanes): lane s = l % 16 addresses row c0 + s / 4,
  // logical columns 32 t + 16 (l / 16 % 2) + 4 (s % 4), i.e. chunk 4 t + trc, half trh.  c0 is a
  // multiple of 4 with c0 % 16 = 4 hh (+ 8 for the second read) for the P Z operands and
  // 8 hh (+ 4 for the second read) for the state-update operands.
  const int s16 = l & 15, g2 = (l >> 4) & 1;
  const int trc = 2 * g2 + ((s16 & 3) >> 1);                       // chunk within the 32-column tile
  const int trh = 4 * (s16 & 1);                                   // half of the chunk
  auto tr_lane = [&](int c0_mod16) {
    return (s16 >> 2) * D + 8 * (trc ^ swz<D>(c0_mod16 + (s16 >> 2))) + trh;
  };
  const int tr_pv0 = tr_lane(4 * hh), tr_pv1 = tr_lane(4 * hh + 8);
  const int tr_up0 = tr_lane(8 * hh), tr_up1 = tr_lane(8 * hh + 4);
  auto read_tr2 = [&](const __bf16* tile, int row_lo, int row_hi, int t, int lane_lo, int lane_hi) {
    union { struct { s16x4 lo, hi; } s; bf16x8 v; } u;
    u.s.lo = lds_read_tr(tile + row_lo * D + (lane_lo ^ (32 * t)));
    u.s.hi = lds_read_tr(tile + row_hi * D + (lane_hi ^ (32 * t)));
    return u.v;
  };

  // ---- prologue: first block's tiles
  {
    const int b0 = REV ? blk_hi - 1 : blk_lo;
    issue_tile_loads(std::integral_constant<int, 0>{}, b0);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    zero_tail_rows(std::integral_constant<int, 0>{}, b0);
  }
  __syncthreads();

  const int nblk = blk_hi - blk_lo;
  // One block of the loop.  The tile buffer index is a compile-time constant (the loop below is
  // unrolled by two) so that the LDS reads of buffer `cur` are provably independent of the direct
  // loads in flight into buffer `cur ^ 1` and need not wait for them.  Returns false after the last block.
  auto block_step = [&](auto cur_tag, int it) -> bool {
    constexpr int cur = decltype(cur_tag)::value;
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    const bool has_next = it + 1 < nblk;
    const int nb = REV ? blk - 1 : blk + 1;
    if (has_next) issue_tile_loads(std::integral_constant<int, cur ^ 1>{}, nb);
    const __bf16* tX = cur ? sT1[0] : sT0[0];
    const __bf16* tY = cur ? sT1[1] : sT0[1];
    const __bf16* tZ = cur ? sT1[2] : sT0[2];

    // The loop body is software-pipelined by hand: the LDS reads of a stage are issued one stage
    // ahead of the MFMAs that consume them, and sched_barrier keeps the compiler from sinking them
    // back next to their uses (which would expose the LDS latency before every MFMA).
#define LA2_STAGE() __builtin_amdgcn_sched_barrier(0)
    auto ld_rows = [&](bf16x8 (&f)[KS], const __bf16* tile_rows) {   // 16-byte row reads, lanes = rows
#pragma unroll
      for (int ks = 0; ks < KS; ks++) f[ks] = *reinterpret_cast<const bf16x8*>(tile_rows + (rowk ^ (16 * ks)));
    };
    auto ld_state = [&](bf16x8 (&f)[KS], int t) {                    // rows of the transposed state copy
#pragma unroll
      for (int ks = 0; ks < KS; ks++)
        f[ks] = *reinterpret_cast<const bf16x8*>(sS + (32 * t + l32) * LD + 16 * ks + 8 * hh);
    };
    auto chain = [&](const bf16x8 (&a)[KS], const bf16x8 (&b)[KS]) {
      f32x16 c = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ks++) c = mfma(a[ks], b[ks], c);
      return c;
    };
    // P Z operands of key tile ct: the 16 block rows of k-step q are c = 32 ct + 16 q + {8 (j / 4) + 4 hh + j % 4}
    auto ld_pz = [&](bf16x8 (&z)[2][NH], int ct) {
#pragma unroll
      for (int q = 0; q < 2; q++)
#pragma unroll
        for (int j = 0; j < NH; j++) {
          const int c0 = 32 * ct + 16 * q + 4 * hh;
          z[q][j] = read_tr2(tZ, c0, c0 + 8, NH * ch + j, tr_pv0, tr_pv1);
        }
    };
    auto mask_pack = [&](bf16x8 (&pf)[2], const f32x16& st, const float (&m)[16]) {
#pragma unroll
      for (int v = 0; v < 16; v++) pf[v >> 3][v & 7] = (__bf16)(st[v] * m[v]);
    };

    // ---- stage 0: this wave's X rows and the first state fragments
    bf16x8 xf[KS], fa[KS], fb[KS];
    ld_rows(xf, tX + 32 * rg * D);
    ld_state(fa, NH * ch);
    LA2_STAGE();
    // ---- inter-block part: W^T[dv][r] = sum_dk S^T[dv][dk] X^T[dk][r]; then the score tiles S^T[c][r]
    f32x16 acc[NH], stA, stB;
    bf16x8 zA[2][NH], zB[2][NH];
    if (NH == 2) {
      ld_state(fb, NH * ch + 1);
      LA2_STAGE();
      acc[0] = chain(fa, xf);
      ld_rows(fa, tY + 32 * ctA * D);
      LA2_STAGE();
      acc[NH - 1] = chain(fb, xf);
      if (two_tiles) ld_rows(fb, tY + 32 * ctB * D);
      ld_pz(zA, ctA);
      LA2_STAGE();
      stA = chain(fa, xf);
    } else {
      ld_rows(fb, tY + 32 * ctA * D);
      ld_pz(zA, ctA);
      LA2_STAGE();
      acc[0] = chain(fa, xf);
      if (two_tiles) ld_rows(fa, tY + 32 * ctB * D);
      LA2_STAGE();
      stA = chain(fb, xf);
    }
    if (two_tiles) ld_pz(zB, ctB);
    LA2_STAGE();
    if (two_tiles) stB = chain(NH == 2 ? fb : fa, xf);
    // the carried state's decay at this lane's position, then the masked scores times Z
#pragma unroll
    for (int j = 0; j < NH; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[j][v] *= inter_scale;
    {
      bf16x8 pf[2];
      mask_pack(pf, stA, mA);
#pragma unroll
      for (int q = 0; q < 2; q++)
#pragma unroll
        for (int j = 0; j < NH; j++) acc[j] = mfma(zA[q][j], pf[q], acc[j]);
    }
    if (two_tiles) {
      bf16x8 pf[2];
      mask_pack(pf, stB, mB);
#pragma unroll
      for (int q = 0; q < 2; q++)
#pragma unroll
        for (int j = 0; j < NH; j++) acc[j] = mfma(zB[q][j], pf[q], acc[j]);
    }
    LA2_STAGE();

    // ---- operands of the state update (they come from the tiles, not from sS, so they may be
    // requested before the barrier): Y rows as key features, Z rows as value features
    constexpr int UK = kB / 16;
    bf16x8 uy[UK], uz[UK][SC];
    if (has_next) {
      const int ycol = w / T::WPT, zt0 = (w % T::WPT) * SC;   // key-feature tile, first value-feature tile
#pragma unroll
      for (int ks = 0; ks < UK; ks++) {
        const int c0 = 16 * ks + 8 * hh;  // this lane's 8 rows: c0 .. c0+7
        uy[ks] = read_tr2(tY, c0, c0 + 4, ycol, tr_up0, tr_up1);
#pragma unroll
        for (int b = 0; b < SC; b++) uz[ks][b] = read_tr2(tZ, c0, c0 + 4, zt0 + b, tr_up0, tr_up1);
      }
    }
    LA2_STAGE();

    // ---- output: stage this wave's 32 rows x D/2 features, then coalesced 16-byte stores
    __bf16* stage = sW[w];
#pragma unroll
    for (int j = 0; j < NH; j++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        bf16x4 pk;
#pragma unroll
        for (int e = 0; e < 4; e++) pk[e] = (__bf16)acc[j][4 * g + e];
        *reinterpret_cast<bf16x4*>(stage + l32 * LW + 32 * j + 8 * g + 4 * hh) = pk;
      }
    // same-wave LDS write -> read: ordered by the LDS queue, no workgroup barrier needed
    constexpr int CW = D / 16;   // 16-byte chunks per staged row
#pragma unroll
    for (int i = 0; i < 32 * CW / 64; i++) {
      const int id = l + 64 * i;
      const int row = id / CW, cc = id % CW;
      const i32x4 v = *reinterpret_cast<const i32x4*>(stage + row * LW + cc * 8);
      const uint32_t off =
          ((uint32_t)(blk * kB + 32 * rg + row) * (uint32_t)stride_n + (uint32_t)(D / 2 * ch + cc * 8)) * 2u;
      __builtin_amdgcn_raw_buffer_store_b128(v, bw, off, 0, 0);
    }

    if (!has_next) return false;         // the state after a chunk's last block is never used
    lds_barrier();                       // every wave is done reading sS

    // ---- state <- lambda^B state + (decay(Y))^T Z, contraction over this block's rows
#pragma unroll
    for (int b = 0; b < SC; b++)
#pragma unroll
      for (int v = 0; v < 16; v++) kv[b][v] *= lamB;
#pragma unroll
    for (int ks = 0; ks < UK; ks++) {
      // weight of rows 16 ks + 8 hh + j: fks * fj[j]
      const float fks = fast_exp2(l2 * (float)(REV ? 16 * ks : kB - 16 - 16 * ks));
      bf16x8 af;
#pragma unroll
      for (int j = 0; j < 8; j++) af[j] = (__bf16)((float)uy[ks][j] * (fks * fj[j]));
#pragma unroll
      for (int b = 0; b < SC; b++) kv[b] = mfma(af, uz[ks][b], kv[b]);
    }
#undef LA2_STAGE
    state_to_lds<D>(sS, kv, w, l32, hh);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // this wave's direct loads of the next block have landed
    zero_tail_rows(std::integral_constant<int, cur ^ 1>{}, nb);
    lds_barrier();                       // next tiles + new state copy visible; current tiles free
    return true;
  };
  for (int it = 0; it < nblk; it += 2) {
    if (!block_step(std::integral_constant<int, 0>{}, it)) break;
    if (!block_step(std::integral_constant<int, 1>{}, it + 1)) break;
  }
}

// Local state of every chunk that has a successor: forward sum_c lambda^(C-1-c) y_c^T z_c over the
// chunk's positions c, reverse sum_c lambda^c y_c^T z_c.  Written fp32 row-major [dk][dv].
template <int D, bool REV>
__global__ __launch_bounds__(kThreads, 1) void chunk_state_bf16_kernel(ScanParams p) {
  using T = Tile<D>;
  constexpr int LD = T::LD, SC = T::SC;
  __shared__ __attribute__((aligned(16))) __bf16 sY[kB * LD];
  __shared__ __attribute__((aligned(16))) __bf16 sZ[kB * LD];

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int lane_off = ((l & 15) >> 2) * LD + 16 * ((l >> 4) & 1) + 4 * (l & 3);
  const int chain = blockIdx.x / p.nchunks, chunk = blockIdx.x % p.nchunks;
  if (REV ? (chunk == 0) : (chunk == p.nchunks - 1)) return;  // no successor needs it
  const int bi = chain / p.heads, hi = chain % p.heads;
  const int64_t base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h;
  const int n = p.n;
  const uint32_t stride_n = (uint32_t)p.stride_n;
  const uint32_t chain_bytes = ((uint32_t)(n - 1) * stride_n + D) * 2u;
  const __amdgpu_buffer_rsrc_t by = make_rsrc(reinterpret_cast<const __bf16*>(p.y[0]) + base, chain_bytes);
  const __amdgpu_buffer_rsrc_t bz = make_rsrc(reinterpret_cast<const __bf16*>(p.z[0]) + base, chain_bytes);
  const float l2 = log2f(p.lambda[hi]);
  const int nblocks = (n + kB - 1) / kB;
  const int cb = p.chunk_tokens / kB;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);

  f32x16 kv[SC];
#pragma unroll
  for (int b = 0; b < SC; b++) kv[b] = zero16();

  i32x4 ry[T::LOADS], rz[T::LOADS];
  const int nblk = blk_hi - blk_lo;
  if (nblk > 0) {
    const int b0 = REV ? blk_hi - 1 : blk_lo;
    load_tile_regs<D>(ry, by, stride_n, b0 * kB, tid);
    load_tile_regs<D>(rz, bz, stride_n, b0 * kB, tid);
  }
  for (int it = 0; it < nblk; it++) {
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    __syncthreads();  // previous block's tiles are no longer read
    store_tile_lds<D>(sY, ry, tid);
    store_tile_lds<D>(sZ, rz, tid);
    __syncthreads();
    if (it + 1 < nblk) {
      const int nb = REV ? blk - 1 : blk + 1;
      load_tile_regs<D>(ry, by, stride_n, nb * kB, tid);
      load_tile_regs<D>(rz, bz, stride_n, nb * kB, tid);
    }
    state_update<D, REV>(kv, sY, sZ, l2, w, hh, lane_off);
  }
  float* gs = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
#pragma unroll
  for (int b = 0; b < SC; b++)
#pragma unroll
    for (int v = 0; v < 16; v++) gs[state_index<D>(w, l32, hh, b, v)] = kv[b][v];
}

// In place: states[chain][j] (local state of chunk j) -> start state of chunk j.
//   forward: G_0 = 0, G_{j+1} = lambda^C G_j + L_j        reverse: G_last = 0, G_{j-1} = lambda^C G_j + L_j
__global__ void state_scan_kernel(float* states, const float* lambda, int heads, int nchunks, int chunk_tokens,
                                  int dd, int reverse) {
  const int chain = blockIdx.y;
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= dd) return;
  const float lamC = exp2f(log2f(lambda[chain % heads]) * (float)chunk_tokens);
  float* s = states + (int64_t)chain * nchunks * dd + e;
  float g = 0.f;
  for (int i = 0; i < nchunks; i++) {
    const int j = reverse ? nchunks - 1 - i : i;
    const bool last = (i == nchunks - 1);
    const float loc = last ? 0.f : s[(int64_t)j * dd];
    s[(int64_t)j * dd] = g;
    g = lamC * g + loc;
  }
}

}  // namespace

int block_size_bf16(int) { return kB; }

hipError_t launch_scan_bf16(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (int64_t)p.batch * p.heads * p.nchunks * p.nscan;
  if (grid == 0 || p.n == 0) return hipSuccess;
  dim3 g((unsigned)grid), b(kThreads);
  if (head_dim == 128) {
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
                     reverse ? 1 : 0);
  return hipGetLastError();
}

}  // namespace la2
