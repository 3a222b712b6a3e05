// fp32 kernels for the decayed causal scan (Algorithm 1; both loops of Algorithm 2), gfx950.
//
// fp32 storage, fp32 products and fp32 accumulation throughout (v_mfma_f32_32x32x2_f32: no reduced
// precision anywhere), for callers that need the 1e-5 accuracy class.  Same organisation as the bf16
// kernels: one workgroup walks the blocks (B = 32 positions) of one sequence chunk of one (batch, head)
// chain; wave w owns value features 32 w .. 32 w + 31 of the output and of the running state, whose
// slice stays in MFMA accumulator registers and is used as an MFMA operand straight from there; the X,
// Y, Z tiles of the next block stream from HBM into LDS (global_load_lds) while the current block is
// computed.
//
// MFMA 32x32x2 fp32 lane layouts (wave64, lane l, l32 = l % 32, hh = l / 32), one float per operand:
//   A[m][k]: m = l32, k = hh       B[k][n]: n = l32, k = hh
//   C[m][n]: n = l32, m = 8 (v / 4) + 4 hh + v % 4 (v = 0..15)
// so one instruction contracts TWO indices, one supplied by each half of the wave.  An accumulator
// register v is therefore directly an operand whose two contraction indices are m(v, 0) and m(v, 1) =
// m(v, 0) + 4; the other operand of such a product is fetched with the same pairing.
//
// Tile layout in LDS: row-major fp32, unpadded, the 16-byte chunk index of a row XOR-ed with row % 16:
// the 16-byte row reads (lanes = rows) are then bank-conflict free, the 4-byte column reads
// (lanes = consecutive features of one row per wave half) stay contiguous per row.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "la2_internal.h"

namespace la2 {
namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int kB = 32;   // block size (positions per block)

__device__ __forceinline__ f32x16 mfma(float a, float b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int v = 0; v < 16; v++) z[v] = 0.f;
  return z;
}

// Direct global -> LDS copy, 16 bytes per lane (as in the bf16 kernels: issued from inline assembly,
// completion tracked by hand with s_waitcnt vmcnt).
__device__ __forceinline__ void dma16(const void* base, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
               :
               : "v"(voff), "s"(base), "s"(lds_base)
               : "m0", "memory");
}

__device__ __forceinline__ uint32_t lds_offset(const void* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// element offset of feature f of tile row `row` (D floats per row, 16-byte chunks swizzled by row % 16)
template <int D>
__device__ __forceinline__ int tile_off(int row, int f) {
  return row * D + ((((f >> 2) ^ (row & 15)) << 2) | (f & 3));
}

// key feature dk, value feature dv of state-slice element (t, v) of a lane <-> index into a d x d state
template <int D>
__device__ __forceinline__ int state_index(int dvt, int l32, int hh, int t, int v, bool transposed) {
  const int dk = 32 * t + 8 * (v >> 2) + 4 * hh + (v & 3);
  const int dv = 32 * dvt + l32;
  return transposed ? dv * D + dk : dk * D + dv;
}

// Scan kernel (STATE_ONLY = false) and chunk-state pre-pass (STATE_ONLY = true: only Y, Z and the state
// update; the local state of the chunk is written to p.states).  D / 32 waves.
template <int D, bool REV, bool STATE_ONLY>
__global__ __launch_bounds__(2 * D, 1) void scan_f32_kernel(ScanParams p) {
  constexpr int NT = D / 32;          // waves; 32-wide feature tiles
  constexpr int NJ = D / 8;           // pairs of 16-byte chunks per row (one pair per 8 features)
  constexpr int TILE = kB * D;        // floats per tile
  constexpr int NTL = STATE_ONLY ? 2 : 3;
  constexpr int DMA_PER_WAVE = (TILE * 4 / 1024) / NT;   // 1 KiB instructions per tile and wave (= 4)
  __shared__ __attribute__((aligned(1024))) float sT[2][NTL][TILE];
  __shared__ float sRed[STATE_ONLY ? 1 : kB * NT];   // Norm epilogue: partial sums of squares, [row][wave]

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int dvt = w;
  const int chain = blockIdx.x / p.nchunks, chunk = blockIdx.x % p.nchunks;
  const int bi = chain / p.heads, hi = chain % p.heads;
  int64_t base;
  int n;
  chain_extent(p, bi, hi, base, n);
  const uint32_t stride_n = (uint32_t)p.stride_n;
  const float l2 = log2f(p.lambda[hi]);
  const float lamB = exp2f(l2 * (float)kB);

  const int nblocks = (n + kB - 1) / kB;
  const int cb = p.chunk_tokens / kB;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);
  if (!STATE_ONLY && blk_lo >= blk_hi) return;
  // pre-pass: the chunk a scan of THIS chain passes last has no successor (packed batch: chains of different lengths)
  if (STATE_ONLY && (REV ? (chunk == 0) : (blk_hi >= nblocks))) return;
  const int nblk = max(blk_hi - blk_lo, 0);

  const char* g[3];
  if (STATE_ONLY) {
    g[0] = reinterpret_cast<const char*>(reinterpret_cast<const float*>(p.y[0]) + base);
    g[1] = reinterpret_cast<const char*>(reinterpret_cast<const float*>(p.z[0]) + base);
    g[2] = nullptr;
  } else {
    g[0] = reinterpret_cast<const char*>(reinterpret_cast<const float*>(p.x[0]) + base);
    g[1] = reinterpret_cast<const char*>(reinterpret_cast<const float*>(p.y[0]) + base);
    g[2] = reinterpret_cast<const char*>(reinterpret_cast<const float*>(p.z[0]) + base);
  }
  constexpr int TX = 0, TY = STATE_ONLY ? 0 : 1, TZ = STATE_ONLY ? 1 : 2;

  // direct loads: instruction i of this wave fills LDS chunks q = 64 (DMA_PER_WAVE w + i) + l of a tile,
  // i.e. row q / (D / 4), physical chunk q % (D / 4), which holds logical chunk (q % (D / 4)) ^ (row % 16)
  int drow[DMA_PER_WAVE], dcol[DMA_PER_WAVE];
#pragma unroll
  for (int i = 0; i < DMA_PER_WAVE; i++) {
    const int q = 64 * (DMA_PER_WAVE * w + i) + l;
    drow[i] = q / (D / 4);
    dcol[i] = 4 * ((q % (D / 4)) ^ (drow[i] & 15));
  }
  const uint32_t wave_lds = (uint32_t)__builtin_amdgcn_readfirstlane(1024 * DMA_PER_WAVE * w);
  auto issue = [&](int buf, int blk) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < DMA_PER_WAVE; i++) {
      const int pos = min(blk * kB + drow[i], n - 1);   // rows past the end are zeroed after landing
      const uint32_t off = ((uint32_t)pos * stride_n + (uint32_t)dcol[i]) * 4u;
#pragma unroll
      for (int t = 0; t < NTL; t++) dma16(g[t], off, lds_offset(&sT[buf][t][0]) + wave_lds + 1024u * i);
    }
  };
  auto zero_tail = [&](int buf, int blk) __attribute__((always_inline)) {
    if ((blk + 1) * kB > n) {
#pragma unroll
      for (int i = 0; i < DMA_PER_WAVE; i++)
        if (blk * kB + drow[i] >= n) {
          const i32x4 z = {0, 0, 0, 0};
#pragma unroll
          for (int t = 0; t < NTL; t++)
            *reinterpret_cast<i32x4*>(reinterpret_cast<char*>(&sT[buf][t][0]) + (wave_lds + 1024u * i + 16u * l)) = z;
        }
    }
  };

  // ---- running state slice S[:, dv tile]: NT accumulator tiles (key-feature tiles), fp32
  f32x16 kv[NT];
  {
    const float* gs = nullptr;
    bool tr = false;
    if (!STATE_ONLY && p.states != nullptr) {
      gs = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
      tr = p.state_transposed & 1;
    } else if (!STATE_ONLY && p.init[0] != nullptr) {
      gs = p.init[0] + (int64_t)chain * (D * D);
      tr = p.init_transposed & 1;
    }
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) kv[t][v] = gs ? gs[state_index<D>(dvt, l32, hh, t, v, tr)] : 0.f;
  }

  // ---- per-lane constants (accumulator element v <-> tile row cc[v] = 8 (v / 4) + 4 hh + v % 4):
  // decay mask of the score tile S^T[c][r] (lane: r = l32), update weight of row c, carried-state weight
  float dg[16], wz[16];
#pragma unroll
  for (int v = 0; v < 16; v++) {
    const int cc = 8 * (v >> 2) + 4 * hh + (v & 3);
    const int e = REV ? cc - l32 : l32 - cc;
    dg[v] = (e >= 0) ? exp2f(l2 * (float)e) : 0.f;
    wz[v] = exp2f(l2 * (float)(REV ? cc + 1 : kB - 1 - cc));
  }
  const float inter_scale = exp2f(l2 * (float)(REV ? kB - 1 - l32 : l32 + 1));
  float* gw = STATE_ONLY ? nullptr : reinterpret_cast<float*>(p.w[0]) + base;

  if (nblk > 0) {
    const int b0 = REV ? blk_hi - 1 : blk_lo;
    issue(0, b0);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    zero_tail(0, b0);
  }
  __syncthreads();

  for (int it = 0; it < nblk; it++) {
    const int cur = it & 1;
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    const bool has_next = it + 1 < nblk;
    const int nb = REV ? blk - 1 : blk + 1;
    if (has_next) issue(cur ^ 1, nb);
    const float* tX = sT[cur][TX];
    const float* tY = sT[cur][TY];
    const float* tZ = sT[cur][TZ];

    // Z column fragments: row cc[v] of the block, this wave's value feature l32 (used by the intra-block
    // product and, weighted, by the state update)
    float zc[16];
#pragma unroll
    for (int v = 0; v < 16; v++) zc[v] = tZ[tile_off<D>(8 * (v >> 2) + 4 * hh + (v & 3), 32 * dvt + l32)];

    if (!STATE_ONLY) {
      // X row fragments: row l32, features 8 j + 4 hh .. + 3 (j = 0 .. NJ - 1): one 16-byte read each.  They
      // serve the score product (paired with the same features of Y) and the inter-block product (state
      // register v of tile t pairs features 32 t + 8 (v / 4) + v % 4 and + 4, i.e. j = 4 t + v / 4).
      f32x4 xr[NJ];
#pragma unroll
      for (int j = 0; j < NJ; j++) xr[j] = *reinterpret_cast<const f32x4*>(&tX[tile_off<D>(l32, 8 * j + 4 * hh)]);
      // inter-block part W^T[dv][r] = sum_dk State[dk][dv] X[r][dk], state straight from its registers
      f32x16 acc = zero16();
#pragma unroll
      for (int t = 0; t < NT; t++)
#pragma unroll
        for (int v = 0; v < 16; v++) acc = mfma(kv[t][v], xr[4 * t + (v >> 2)][v & 3], acc);
      // score tile S^T[c][r] = sum_k Y[c][k] X[r][k]
      f32x16 st = zero16();
#pragma unroll
      for (int j = 0; j < NJ; j++) {
        const f32x4 yr = *reinterpret_cast<const f32x4*>(&tY[tile_off<D>(l32, 8 * j + 4 * hh)]);
#pragma unroll
        for (int i = 0; i < 4; i++) st = mfma(yr[i], xr[j][i], st);
      }
      // carried part takes its decay, scores take the mask, then the intra-block part Z^T P^T
#pragma unroll
      for (int v = 0; v < 16; v++) acc[v] *= inter_scale;
#pragma unroll
      for (int v = 0; v < 16; v++) acc = mfma(zc[v], st[v] * dg[v], acc);
      const int pos = blk * kB + l32;
      if (p.rstd != nullptr) {   // Norm epilogue (eq. (2)); the previous block's reads ended before its last barrier
        norm_publish<NT>(acc, sRed, l32, hh, dvt);
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // LDS only: the next tiles stay in flight
        const float r = norm_collect<NT>(sRed, l32, 1.f / (float)D, p.eps);
#pragma unroll
        for (int v = 0; v < 16; v++) acc[v] *= r;
        if (dvt == 0 && hh == 0 && pos < n) p.rstd[rstd_chain_offset(p, bi, hi) + pos] = r;
      }
      // output: lane = position l32, elements v = 4 g .. 4 g + 3 are value features 32 dvt + 8 g + 4 hh .. + 3
      if (pos < n) {
        float* orow = gw + (int64_t)pos * stride_n + 32 * dvt + 4 * hh;
#pragma unroll
        for (int gq = 0; gq < 4; gq++) {
          f32x4 o4 = {acc[4 * gq], acc[4 * gq + 1], acc[4 * gq + 2], acc[4 * gq + 3]};
          *reinterpret_cast<f32x4*>(orow + 8 * gq) = o4;
        }
      }
    }

    // state slice <- lambda^B state + Y^T decay(Z), contraction over this block's rows, paired as the
    // Z fragments are: lanes of half hh supply row cc[v]
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) kv[t][v] *= lamB;
#pragma unroll
    for (int v = 0; v < 16; v++) {
      const float zw = zc[v] * wz[v];
      const int row = 8 * (v >> 2) + 4 * hh + (v & 3);
#pragma unroll
      for (int t = 0; t < NT; t++) kv[t] = mfma(tY[tile_off<D>(row, 32 * t + l32)], zw, kv[t]);
    }

    if (has_next) {
      __builtin_amdgcn_s_waitcnt(0x0F70);   // this wave's part of the next tiles has landed (and its stores)
      zero_tail(cur ^ 1, nb);
    }
    __syncthreads();
  }

  // the chunk's local state (pre-pass) or the state after the chain's last block (on request)
  float* gf = nullptr;
  bool trf = false;
  if (STATE_ONLY) {
    gf = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
  } else if (p.fin[0] != nullptr && (REV ? chunk == 0 : chunk == p.nchunks - 1)) {
    gf = p.fin[0] + (int64_t)chain * (D * D);
    trf = p.fin_transposed & 1;
  }
  if (gf != nullptr) {
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) gf[state_index<D>(dvt, l32, hh, t, v, trf)] = kv[t][v];
  }
}

template <bool STATE_ONLY>
hipError_t launch(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (int64_t)p.batch * p.heads * p.nchunks;
  if (grid == 0 || p.n == 0) return hipSuccess;
  dim3 g((unsigned)grid);
  if (head_dim == 128) {
    if (reverse) hipLaunchKernelGGL((scan_f32_kernel<128, true, STATE_ONLY>), g, dim3(256), 0, s, p);
    else         hipLaunchKernelGGL((scan_f32_kernel<128, false, STATE_ONLY>), g, dim3(256), 0, s, p);
  } else {
    if (reverse) hipLaunchKernelGGL((scan_f32_kernel<64, true, STATE_ONLY>), g, dim3(128), 0, s, p);
    else         hipLaunchKernelGGL((scan_f32_kernel<64, false, STATE_ONLY>), g, dim3(128), 0, s, p);
  }
  return hipGetLastError();
}

}  // namespace

int block_size_f32(int) { return kB; }

hipError_t launch_scan_f32(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  return launch<false>(head_dim, reverse, p, s);
}

hipError_t launch_chunk_states_f32(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  return launch<true>(head_dim, reverse, p, s);
}

}  // namespace la2
