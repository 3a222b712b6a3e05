// Left-product form of the forward and backward pass, for comparison (bf16 MFMA, gfx950).
#include "la2_bf16_common.h"

namespace la2 {
namespace {
using namespace bf16k;
using bf16x8 = ex8<__bf16>;   // this comparison kernel takes bf16 only
using bf16x4 = ex4<__bf16>;

// Left-product form for comparison: O = [(Q K^T) * M] V computed tile by tile over ALL earlier key blocks
// (the O(n^2 d) evaluation that the block recurrence replaces; Sec. 3.1 eq. (1) with the decay mask of
// Sec. 3.2).  bf16.  One workgroup per (chain, 128 query rows); wave w owns query rows
// 32 w .. 32 w + 31 and all value features; the key and value blocks (64 positions) stream through LDS,
// double buffered.  Same MFMA operand layouts, LDS tile layout and mask tables as the scan kernels.
// As with the scan kernels this is one generic operation on (x, y, z): forward W = [(X Y^T) * M] Z (O from
// (Q, K, V); dQ from (dO, V, K)), and with REV the transposed mask, W = [(X Y^T) * M^T] Z over all LATER
// blocks of y and z (dV from (K, Q, dO), dK from (V, dO, Q): the gradients of Sec. 3.2.2 as plain masked
// products).
template <int D, bool REV>
__global__ __launch_bounds__(kThreads, 1) void left_product_bf16_kernel(ScanParams p) {
  using C = Cfg<D>;
  constexpr int KS = C::KS, NT = C::NT, TILE = C::TILE, LW = C::LW;
  constexpr int QB = 128;   // query rows per workgroup
  __shared__ __attribute__((aligned(1024))) __bf16 sT[2][2][TILE];   // [buffer][K, V]
  __shared__ __attribute__((aligned(16))) __bf16 sW[4][32 * LW];

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int nqb = (p.n + QB - 1) / QB;
  const int chain = blockIdx.x / nqb;
  // long rows of the triangle first: the last query block looks back furthest, with REV the first looks ahead furthest
  const int qb = REV ? (int)(blockIdx.x % nqb) : nqb - 1 - (int)(blockIdx.x % nqb);
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
    const int e = REV ? cc - l32 : l32 - cc;
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

  // key blocks jmin .. jmax reach this query block: all earlier ones and its own, or (REV) its own and all later
  const int nkb = (n + kB - 1) / kB;
  const int jmin = REV ? (qb * QB) / kB : 0;
  const int jmax = REV ? nkb - 1 : min((qb * QB + QB - 1) / kB, nkb - 1);
  loader.issue(sT[0], jmin);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  loader.zero_tail(sT[0], jmin);
  __syncthreads();
  for (int j = jmin; j <= jmax; j++) {
    const int cur = (j - jmin) & 1;
    if (j < jmax) loader.issue(sT[cur ^ 1], j + 1);
    const __bf16* tK = sT[cur][0];
    const __bf16* tV = sT[cur][1];
#pragma unroll
    for (int kt = 0; kt < 2; kt++) {
      // distance between this wave's first query row and the key tile's first row: a multiple of 32
      const int ahead = qb * QB + 32 * w - (j * kB + 32 * kt);
      const int dist = REV ? -ahead : ahead;
      if (dist < 0) continue;   // wave-uniform: the whole tile is on the masked side of the diagonal
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

hipError_t launch_left_product_bf16(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (int64_t)p.batch * p.heads * ((p.n + 127) / 128);
  if (grid == 0 || p.n == 0) return hipSuccess;
  dim3 g((unsigned)grid), b(kThreads);
  if (head_dim == 128) {
    if (reverse) hipLaunchKernelGGL((left_product_bf16_kernel<128, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((left_product_bf16_kernel<128, false>), g, b, 0, s, p);
  } else {
    if (reverse) hipLaunchKernelGGL((left_product_bf16_kernel<64, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((left_product_bf16_kernel<64, false>), g, b, 0, s, p);
  }
  return hipGetLastError();
}

}  // namespace la2
