// bf16 MFMA kernels for the decayed causal scan (Algorithm 1; both loops of Algorithm 2), gfx950.
//
// One workgroup (4 waves) walks the blocks of one sequence chunk of one (batch, head) chain.  Per
// block of B = 128 positions it holds the X, Y, Z tiles (B x D bf16) in LDS, the fp32 running
// state (D x D) in MFMA accumulator registers split over the four waves, and a bf16 copy of the
// state (transposed) in LDS as the operand of the inter-block product.  Wave w owns rows
// 32w .. 32w+31 of the block from the score tile to the output, so the masked scores never leave
// registers.  All products use v_mfma_f32_32x32x16_bf16 with fp32 accumulation.
//
// MFMA 32x32x16 lane layouts (wave64, lane l, l32 = l % 32, hh = l / 32):
//   A[m][k]: m = l32, k = 8 hh + j (j = 0..7)     B[k][n]: n = l32, k = 8 hh + j
//   C[m][n]: n = l32, m = 8 (v / 4) + 4 hh + v % 4 (v = 0..15)
// Outputs are accumulated TRANSPOSED (C rows = value feature, C columns = position) so that each
// lane ends up with 4 consecutive features of one position, which packs into 8-byte LDS writes.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "la2_internal.h"

namespace la2 {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int kB = 128;       // block size (positions per block)
constexpr int kThreads = 256; // 4 waves

template <int D>
struct Tile {
  static constexpr int LD = D + 16;      // padded LDS row stride (elements): 8-bank shift per row
  static constexpr int NT = D / 32;      // 32-wide tiles along a feature dimension
  static constexpr int KS = D / 16;      // MFMA k-steps along a feature dimension
  static constexpr int ST = D / 64;      // state tiles per wave along each state dimension
  static constexpr int CPR = D / 8;      // 16-byte chunks per row
  static constexpr int LOADS = kB * CPR / kThreads;  // 16-byte chunks per thread per tile
};

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
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
__device__ __forceinline__ void load_tile_regs(i32x4 (&r)[Tile<D>::LOADS], const __bf16* g, int64_t stride_n,
                                               int row0, int n, int tid) {
  constexpr int CPR = Tile<D>::CPR;
#pragma unroll
  for (int i = 0; i < Tile<D>::LOADS; i++) {
    int id = tid + kThreads * i;
    int row = id / CPR, cc = id % CPR;
    int pos = row0 + row;
    i32x4 v = {0, 0, 0, 0};
    if (pos < n) v = *reinterpret_cast<const i32x4*>(g + (int64_t)pos * stride_n + cc * 8);
    r[i] = v;
  }
}

template <int D>
__device__ __forceinline__ void store_tile_lds(__bf16* s, const i32x4 (&r)[Tile<D>::LOADS], int tid) {
  constexpr int CPR = Tile<D>::CPR;
#pragma unroll
  for (int i = 0; i < Tile<D>::LOADS; i++) {
    int id = tid + kThreads * i;
    int row = id / CPR, cc = id % CPR;
    *reinterpret_cast<i32x4*>(s + row * Tile<D>::LD + cc * 8) = r[i];
  }
}

// state <- lambda^B state + (decay(Y))^T Z over one block held in LDS (contraction over the block's
// rows).  Forward: row c is weighted lambda^(B-1-c); reverse: lambda^c.
template <int D, bool REV>
__device__ __forceinline__ void state_update(f32x16 (&kv)[Tile<D>::ST][Tile<D>::ST], const __bf16* sY,
                                             const __bf16* sZ, float l2, int w, int hh, int lane_off) {
  constexpr int LD = Tile<D>::LD, ST = Tile<D>::ST;
  const float lamB = exp2f(l2 * (float)kB);
#pragma unroll
  for (int a = 0; a < ST; a++)
#pragma unroll
    for (int b = 0; b < ST; b++)
#pragma unroll
      for (int v = 0; v < 16; v++) kv[a][b][v] *= lamB;
  float fj[8];
#pragma unroll
  for (int j = 0; j < 8; j++) fj[j] = exp2f(l2 * (float)(REV ? j : 7 - j));
#pragma unroll 2
  for (int ks = 0; ks < kB / 16; ks++) {
    const int c0 = 16 * ks + 8 * hh;  // this lane's 8 rows: c0 .. c0+7
    const float fb = exp2f(l2 * (float)(REV ? c0 : kB - 8 - c0));
    bf16x8 af[ST], zf[ST];
#pragma unroll
    for (int a = 0; a < ST; a++) {
      bf16x8 y = read_cols<LD>(sY, c0, c0 + 4, 32 * (ST * (w >> 1) + a), lane_off);
#pragma unroll
      for (int j = 0; j < 8; j++) af[a][j] = (__bf16)((float)y[j] * (fb * fj[j]));
    }
#pragma unroll
    for (int b = 0; b < ST; b++) zf[b] = read_cols<LD>(sZ, c0, c0 + 4, 32 * (ST * (w & 1) + b), lane_off);
#pragma unroll
    for (int a = 0; a < ST; a++)
#pragma unroll
      for (int b = 0; b < ST; b++) kv[a][b] = mfma(af[a], zf[b], kv[a][b]);
  }
}

// fp32 state tile element (a, b, v) of wave w sits at key feature dk, value feature dv:
//   dk = 32 (ST (w / 2) + a) + 8 (v / 4) + 4 hh + v % 4,   dv = 32 (ST (w % 2) + b) + l32
template <int D>
__device__ __forceinline__ void state_to_lds(__bf16* sS, const f32x16 (&kv)[Tile<D>::ST][Tile<D>::ST], int w,
                                             int l32, int hh) {
  constexpr int LD = Tile<D>::LD, ST = Tile<D>::ST;
#pragma unroll
  for (int a = 0; a < ST; a++)
#pragma unroll
    for (int b = 0; b < ST; b++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        int dk = 32 * (ST * (w >> 1) + a) + 8 * g + 4 * hh;
        int dv = 32 * (ST * (w & 1) + b) + l32;
        bf16x4 pk;
#pragma unroll
        for (int j = 0; j < 4; j++) pk[j] = (__bf16)kv[a][b][4 * g + j];
        *reinterpret_cast<bf16x4*>(sS + dv * LD + dk) = pk;  // transposed copy: sS[dv][dk]
      }
}

template <int D, bool REV>
__global__ __launch_bounds__(kThreads, 1) void scan_bf16_kernel(ScanParams p) {
  using T = Tile<D>;
  constexpr int LD = T::LD, NT = T::NT, KS = T::KS, ST = T::ST;
  __shared__ __attribute__((aligned(16))) __bf16 sX[kB * LD];
  __shared__ __attribute__((aligned(16))) __bf16 sY[kB * LD];
  __shared__ __attribute__((aligned(16))) __bf16 sZ[kB * LD];
  __shared__ __attribute__((aligned(16))) __bf16 sS[D * LD];

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int lane_off = ((l & 15) >> 2) * LD + 16 * ((l >> 4) & 1) + 4 * (l & 3);
  const int chain = blockIdx.x / p.nchunks, chunk = blockIdx.x % p.nchunks;
  const int bi = chain / p.heads, hi = chain % p.heads;
  const int64_t base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h;
  const __bf16* gx = reinterpret_cast<const __bf16*>(p.x) + base;
  const __bf16* gy = reinterpret_cast<const __bf16*>(p.y) + base;
  const __bf16* gz = reinterpret_cast<const __bf16*>(p.z) + base;
  __bf16* gw = reinterpret_cast<__bf16*>(p.w) + base;
  const int n = p.n;
  const float l2 = log2f(p.lambda[hi]);

  const int nblocks = (n + kB - 1) / kB;
  const int cb = p.chunk_tokens / kB;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);
  if (blk_lo >= blk_hi) return;

  // ---- running state: registers (fp32) + LDS copy (bf16, transposed)
  f32x16 kv[ST][ST];
  if (p.states != nullptr) {
    const float* gs = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
#pragma unroll
    for (int a = 0; a < ST; a++)
#pragma unroll
      for (int b = 0; b < ST; b++)
#pragma unroll
        for (int v = 0; v < 16; v++) {
          int dk = 32 * (ST * (w >> 1) + a) + 8 * (v >> 2) + 4 * hh + (v & 3);
          int dv = 32 * (ST * (w & 1) + b) + l32;
          kv[a][b][v] = gs[dk * D + dv];
        }
  } else {
#pragma unroll
    for (int a = 0; a < ST; a++)
#pragma unroll
      for (int b = 0; b < ST; b++)
#pragma unroll
        for (int v = 0; v < 16; v++) kv[a][b][v] = 0.f;
  }
  state_to_lds<D>(sS, kv, w, l32, hh);

  // weight of the carried state for this lane's position (row r = 32 w + l32 of the block):
  // forward lambda^(r+1), reverse lambda^(B-r)
  const int r = 32 * w + l32;
  const float inter_scale = exp2f(l2 * (float)(REV ? kB - r : r + 1));

  i32x4 rx[T::LOADS], ry[T::LOADS], rz[T::LOADS];
  {
    const int b0 = REV ? blk_hi - 1 : blk_lo;
    load_tile_regs<D>(rx, gx, p.stride_n, b0 * kB, n, tid);
    load_tile_regs<D>(ry, gy, p.stride_n, b0 * kB, n, tid);
    load_tile_regs<D>(rz, gz, p.stride_n, b0 * kB, n, tid);
    store_tile_lds<D>(sX, rx, tid);
    store_tile_lds<D>(sY, ry, tid);
    store_tile_lds<D>(sZ, rz, tid);
  }
  __syncthreads();

  const int nblk = blk_hi - blk_lo;
  for (int it = 0; it < nblk; it++) {
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    const bool has_next = it + 1 < nblk;
    if (has_next) {
      const int nb = REV ? blk - 1 : blk + 1;
      load_tile_regs<D>(rx, gx, p.stride_n, nb * kB, n, tid);
      load_tile_regs<D>(ry, gy, p.stride_n, nb * kB, n, tid);
      load_tile_regs<D>(rz, gz, p.stride_n, nb * kB, n, tid);
    }

    // ---- this wave's X rows as MFMA operand fragments
    bf16x8 xf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) xf[ks] = *reinterpret_cast<const bf16x8*>(sX + r * LD + 16 * ks + 8 * hh);

    // ---- inter-block part: W^T[dv][r] = sum_dk S^T[dv][dk] X^T[dk][r], then the position's decay
    f32x16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
#pragma unroll
      for (int v = 0; v < 16; v++) acc[nt][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        bf16x8 sf = *reinterpret_cast<const bf16x8*>(sS + (32 * nt + l32) * LD + 16 * ks + 8 * hh);
        acc[nt] = mfma(sf, xf[ks], acc[nt]);
      }
#pragma unroll
      for (int v = 0; v < 16; v++) acc[nt][v] *= inter_scale;
    }

    // ---- intra-block part: masked scores S^T[c][r] for the key tiles this wave's rows can see
#pragma unroll
    for (int ct = 0; ct < kB / 32; ct++) {
      const bool needed = REV ? (ct >= w) : (ct <= w);   // wave-uniform
      if (needed) {
        f32x16 st;
#pragma unroll
        for (int v = 0; v < 16; v++) st[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
          bf16x8 yf = *reinterpret_cast<const bf16x8*>(sY + (32 * ct + l32) * LD + 16 * ks + 8 * hh);
          st = mfma(yf, xf[ks], st);
        }
        // decay mask: forward lambda^(r-c) for r >= c, reverse lambda^(c-r) for c >= r, else 0
        bf16x8 pf[2];
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const int c = 32 * ct + 8 * (v >> 2) + 4 * hh + (v & 3);
          const int e = REV ? c - r : r - c;
          const float m = (e >= 0) ? exp2f(l2 * (float)e) : 0.f;
          pf[v >> 3][v & 7] = (__bf16)(st[v] * m);
        }
        // P V: the 16 block rows of k-step q are c = 32 ct + 16 q + {8 (j / 4) + 4 hh + j % 4}
#pragma unroll
        for (int q = 0; q < 2; q++) {
          const int c0 = 32 * ct + 16 * q + 4 * hh;
#pragma unroll
          for (int nt = 0; nt < NT; nt++) {
            bf16x8 zf = read_cols<LD>(sZ, c0, c0 + 8, 32 * nt, lane_off);
            acc[nt] = mfma(zf, pf[q], acc[nt]);
          }
        }
      }
    }

    // ---- output: stage this wave's 32 rows in its own (now free) rows of sX, then coalesced stores
#pragma unroll
    for (int nt = 0; nt < NT; nt++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        bf16x4 pk;
#pragma unroll
        for (int j = 0; j < 4; j++) pk[j] = (__bf16)acc[nt][4 * g + j];
        *reinterpret_cast<bf16x4*>(sX + r * LD + 32 * nt + 8 * g + 4 * hh) = pk;
      }
    // same-wave LDS write -> read: ordered by the LDS queue, no workgroup barrier needed
#pragma unroll
    for (int i = 0; i < 32 * T::CPR / 64; i++) {
      const int id = l + 64 * i;
      const int row = id / T::CPR, cc = id % T::CPR;
      const int pos = blk * kB + 32 * w + row;
      i32x4 v = *reinterpret_cast<const i32x4*>(sX + (32 * w + row) * LD + cc * 8);
      if (pos < n) *reinterpret_cast<i32x4*>(gw + (int64_t)pos * p.stride_n + cc * 8) = v;
    }

    if (!has_next) break;                // the state after a chunk's last block is never used
    __syncthreads();                     // every wave is done with sS (and sX)

    state_update<D, REV>(kv, sY, sZ, l2, w, hh, lane_off);
    state_to_lds<D>(sS, kv, w, l32, hh);
    __syncthreads();                     // every wave is done with sY, sZ
    store_tile_lds<D>(sX, rx, tid);
    store_tile_lds<D>(sY, ry, tid);
    store_tile_lds<D>(sZ, rz, tid);
    __syncthreads();
  }
}

// Local state of every chunk that has a successor: forward sum_c lambda^(C-1-c) y_c^T z_c over the
// chunk's positions c, reverse sum_c lambda^c y_c^T z_c.  Written fp32 row-major [dk][dv].
template <int D, bool REV>
__global__ __launch_bounds__(kThreads, 1) void chunk_state_bf16_kernel(ScanParams p) {
  using T = Tile<D>;
  constexpr int LD = T::LD, ST = T::ST;
  __shared__ __attribute__((aligned(16))) __bf16 sY[kB * LD];
  __shared__ __attribute__((aligned(16))) __bf16 sZ[kB * LD];

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int lane_off = ((l & 15) >> 2) * LD + 16 * ((l >> 4) & 1) + 4 * (l & 3);
  const int chain = blockIdx.x / p.nchunks, chunk = blockIdx.x % p.nchunks;
  if (REV ? (chunk == 0) : (chunk == p.nchunks - 1)) return;  // no successor needs it
  const int bi = chain / p.heads, hi = chain % p.heads;
  const int64_t base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h;
  const __bf16* gy = reinterpret_cast<const __bf16*>(p.y) + base;
  const __bf16* gz = reinterpret_cast<const __bf16*>(p.z) + base;
  const int n = p.n;
  const float l2 = log2f(p.lambda[hi]);
  const int nblocks = (n + kB - 1) / kB;
  const int cb = p.chunk_tokens / kB;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);

  f32x16 kv[ST][ST];
#pragma unroll
  for (int a = 0; a < ST; a++)
#pragma unroll
    for (int b = 0; b < ST; b++)
#pragma unroll
      for (int v = 0; v < 16; v++) kv[a][b][v] = 0.f;

  i32x4 ry[T::LOADS], rz[T::LOADS];
  const int nblk = blk_hi - blk_lo;
  if (nblk > 0) {
    const int b0 = REV ? blk_hi - 1 : blk_lo;
    load_tile_regs<D>(ry, gy, p.stride_n, b0 * kB, n, tid);
    load_tile_regs<D>(rz, gz, p.stride_n, b0 * kB, n, tid);
  }
  for (int it = 0; it < nblk; it++) {
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    __syncthreads();  // previous block's tiles are no longer read
    store_tile_lds<D>(sY, ry, tid);
    store_tile_lds<D>(sZ, rz, tid);
    __syncthreads();
    if (it + 1 < nblk) {
      const int nb = REV ? blk - 1 : blk + 1;
      load_tile_regs<D>(ry, gy, p.stride_n, nb * kB, n, tid);
      load_tile_regs<D>(rz, gz, p.stride_n, nb * kB, n, tid);
    }
    state_update<D, REV>(kv, sY, sZ, l2, w, hh, lane_off);
  }
  float* gs = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
#pragma unroll
  for (int a = 0; a < ST; a++)
#pragma unroll
    for (int b = 0; b < ST; b++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        int dk = 32 * (ST * (w >> 1) + a) + 8 * (v >> 2) + 4 * hh + (v & 3);
        int dv = 32 * (ST * (w & 1) + b) + l32;
        gs[dk * D + dv] = kv[a][b][v];
      }
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
  const int64_t grid = (int64_t)p.batch * p.heads * p.nchunks;
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
