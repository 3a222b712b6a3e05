// Short runs of positions in bf16 (the tail of a segment whose final state is wanted, a multi-token decode),
// gfx950: Algorithm 1 over positions [t0, t1) of every chain from a given start state, in blocks of 32, with
// the state after the LAST position handed out exactly even when that position is not the end of a block.
//
// The scan kernels form the state after whole blocks only: their update weights lambda^(B-1-c) and the decay
// lambda^B of the carried state assume B valid rows.  Here a block with nv <= 32 valid rows uses
//     S <- lambda^nv S + sum_{c < nv} lambda^(nv-1-c) y_c^T z_c
// (rows c >= nv are zero; their weight is clamped to lambda^0 so that it stays finite for any lambda).
// Same MFMA layouts, LDS tile layout and direct loads as the scan kernels (la2_bf16_common.h), one tile
// buffer and no instruction scheduling: a launch is a few blocks per chain and is bound by reading and
// writing the d x d fp32 state once.  D / 32 waves; wave w owns value features 32 w .. 32 w + 31.
#include "la2_bf16_common.h"

namespace la2 {
namespace {
using namespace bf16k;

// Three waves per SIMD at head_dim 128 (168 registers, no spills; the allocator takes 222 and two waves when left
// alone): a workgroup loads its state slice, computes and stores one after the other, and a third resident workgroup
// per compute unit keeps more of the state in flight (8 tokens x 4096 chains: 0.0907 against 0.0942 ms; four waves
// spill and take 0.148 ms).
// NORM: the Norm epilogue of eq. (2) (the waves exchange the sums of squares of their 32 features of every row
// through LDS, one more barrier per block; wave 0 stores r).
template <typename E, int D, bool NORM = false>
__global__ __launch_bounds__(2 * D) __attribute__((amdgpu_waves_per_eu(D == 128 ? 3 : 1))) void tail_bf16_kernel(RecurParams p) {
  constexpr int B = 32;
  using C = Cfg<D, B>;
  constexpr int KS = C::KS, NT = C::NT, TILE = C::TILE;
  using Loader = TileLoader<D, 3, B, NT>;
  __shared__ __attribute__((aligned(1024))) E sT[3][TILE];   // X, Y, Z
  float* const sRed = NormExchange<NORM ? B * NT : 0>::get();   // [position][wave]

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int dvt = w;
  const int64_t chain = blockIdx.x;
  const int bi = (int)(chain / p.heads), hi = (int)(chain % p.heads);
  const int64_t base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h + (int64_t)p.t0 * p.stride_n;
  const int n = p.t1 - p.t0;                  // positions of this run, counted from t0
  const uint32_t stride_n = (uint32_t)p.stride_n;
  const float l2 = log2f(p.lambda[hi]);

  Loader loader(w, l, n, stride_n);
  loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.x[0]) + base);
  loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.y[0]) + base);
  loader.g[2] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.z[0]) + base);
  E* const gw = reinterpret_cast<E*>(p.w[0]) + base;
  const LaneAddr<D> la(l);

  // state slice S[:, dv tile] in accumulator layout
  f32x16 kv[NT];
  {
    const float* gs = p.init[0] ? p.init[0] + chain * (int64_t)(D * D) : nullptr;
    const bool tr = p.init_transposed & 1;
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) kv[t][v] = gs ? gs[state_index<D>(dvt, l32, hh, t, v, tr)] : 0.f;
  }
  // decay mask of the score tile S^T[c][r] (lane: r = l32; element v: c = 8 (v / 4) + 4 hh + v % 4) and the
  // weight lambda^(r+1) of the carried state at this lane's position
  float dg[16];
#pragma unroll
  for (int v = 0; v < 16; v++) {
    const int e = l32 - (8 * (v >> 2) + 4 * hh + (v & 3));
    dg[v] = (e >= 0) ? exp2f(l2 * (float)e) : 0.f;
  }
  const float inter_scale = exp2f(l2 * (float)(l32 + 1));

  const int nblk = (n + B - 1) / B;
  for (int blk = 0; blk < nblk; blk++) {
    loader.issue(sT, blk);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    loader.zero_tail(sT, blk);
    __syncthreads();
    const int nv = min(B, n - blk * B);    // valid rows of this block

    // inter-block part W^T[dv][r] = sum_dk State[dk][dv] X[r][dk] and scores S^T[c][r] = sum_k Y[c][k] X[r][k]
    f32x16 acc = zero16(), sd = zero16();
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      const ex8<E> xa = la.read_row(sT[0], 0, ks), ya = la.read_row(sT[1], 0, ks);
      ex8<E> f;
#pragma unroll
      for (int j = 0; j < 8; j++) f[j] = (E)kv[ks >> 1][8 * (ks & 1) + j];
      acc = mfma(to_perm_order(f), xa, acc);
      sd = mfma(ya, xa, sd);
    }
#pragma unroll
    for (int v = 0; v < 16; v++) acc[v] *= inter_scale;
    // intra-block part Z^T P^T; the same Z fragments, weighted, update the state
    ex8<E> zf[2];
#pragma unroll
    for (int q = 0; q < 2; q++) {
      zf[q] = la.read_cols(sT[2], 16 * q, dvt);
      ex8<E> pd;
#pragma unroll
      for (int j = 0; j < 8; j++) pd[j] = (E)(sd[8 * q + j] * dg[8 * q + j]);
      acc = mfma(zf[q], pd, acc);
    }
    // output: lane = position l32, elements 4 g .. 4 g + 3 are value features 32 dvt + 8 g + 4 hh .. + 3
    const int pos = blk * B + l32;
    if constexpr (NORM) {
      // the next publish comes after the two barriers that end this block: one exchange buffer is enough
      norm_publish<NT>(acc, sRed, l32, hh, dvt);
      __syncthreads();
      const float r = norm_collect<NT>(sRed, l32, 1.f / (float)D, p.eps);
#pragma unroll
      for (int v = 0; v < 16; v++) acc[v] *= r;
      if (dvt == 0 && hh == 0 && pos < n) p.rstd[chain * p.rstd_stride + p.t0 + pos] = r;
    }
    if (pos < n) {
      E* orow = gw + (int64_t)pos * stride_n + 32 * dvt + 4 * hh;
#pragma unroll
      for (int g = 0; g < 4; g++) {
        ex4<E> pk;
#pragma unroll
        for (int e = 0; e < 4; e++) pk[e] = (E)acc[4 * g + e];
        *reinterpret_cast<ex4<E>*>(orow + 8 * g) = pk;
      }
    }
    // state slice <- lambda^nv state + Y^T decay(Z): element j of a Z fragment is row 16 q + 8 (j / 4) + 4 hh + j % 4
    const float lam_nv = exp2f(l2 * (float)nv);
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) kv[t][v] *= lam_nv;
#pragma unroll
    for (int q = 0; q < 2; q++) {
      ex8<E> zd;
#pragma unroll
      for (int j = 0; j < 8; j++) {
        const int c = 16 * q + 8 * (j >> 2) + 4 * hh + (j & 3);
        zd[j] = (E)((float)zf[q][j] * exp2f(l2 * (float)max(nv - 1 - c, 0)));
      }
#pragma unroll
      for (int t = 0; t < NT; t++) kv[t] = mfma(la.read_cols(sT[1], 16 * q, t), zd, kv[t]);
    }
    __syncthreads();   // the tiles are free for the next block's loads
  }

  if (p.fin[0] != nullptr) {
    float* gf = p.fin[0] + chain * (int64_t)(D * D);
    const bool trf = p.fin_transposed & 1;
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) gf[state_index<D>(dvt, l32, hh, t, v, trf)] = kv[t][v];
  }
}

}  // namespace

hipError_t launch_tail_bf16(int dtype, int head_dim, int batch, const RecurParams& p, hipStream_t s) {
  const int64_t chains = (int64_t)batch * p.heads;
  if (chains == 0 || p.t1 <= p.t0) return hipSuccess;
  dim3 g((unsigned)chains);
#define LA2_LAUNCH_TAIL(E, D)                                                                        \
  do {                                                                                               \
    if (p.rstd != nullptr) hipLaunchKernelGGL((tail_bf16_kernel<E, D, true>), g, dim3(2 * D), 0, s, p); \
    else                   hipLaunchKernelGGL((tail_bf16_kernel<E, D, false>), g, dim3(2 * D), 0, s, p); \
  } while (0)
  if (dtype == kF16) {
    if (head_dim == 128) LA2_LAUNCH_TAIL(_Float16, 128);
    else                 LA2_LAUNCH_TAIL(_Float16, 64);
  } else {
    if (head_dim == 128) LA2_LAUNCH_TAIL(__bf16, 128);
    else                 LA2_LAUNCH_TAIL(__bf16, 64);
  }
#undef LA2_LAUNCH_TAIL
  return hipGetLastError();
}

}  // namespace la2
