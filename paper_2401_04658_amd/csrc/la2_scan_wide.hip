// Scan kernel for the other head dimensions (96 and 256), 16-bit data, gfx950: the decayed causal scan
// (Algorithm 1; both loops of Algorithm 2) and, as a template flag, the chunk-state pre-pass for them.
//
// Same arithmetic, MFMA layouts and direct HBM -> LDS tile loads as the kernels for head_dim 64 / 128
// (la2_bf16_common.h), in the plainest arrangement: blocks of 32 positions, D / 32 waves (wave w owns value
// features 32 w .. 32 w + 31 and that slice of the fp32 state in accumulators), two tile buffers (the next
// block's tiles stream in while this block is computed), one barrier per block, no hand scheduling.
// Head_dim 256 makes a workgroup of 8 waves with 128 state registers per lane; head_dim 96 one of 3 waves.
//
// A ragged last block (nv < 32 valid rows) is handled exactly in both directions, so the state entry points
// need no token-by-token tail for these head dimensions:
//     forward  S <- lambda^nv S + sum_{c < nv} lambda^(nv-1-c) y_c^T z_c,   carried part of row r: lambda^(r+1)
//     reverse  S <- lambda^nv S + sum_{c < nv} lambda^(c+1)    y_c^T z_c,   carried part of row r: lambda^(nv-1-r)
// (rows c >= nv are zero; exponents are clamped at 0 so that every weight stays finite for any lambda).
#include "la2_bf16_common.h"

namespace la2 {
namespace {
using namespace bf16k;

// Per-lane addressing of the swizzled tiles without the power-of-two shortcuts of LaneAddr (head_dim 96).
template <int D>
struct PlainAddr {
  int l32, hh, r0, trc, trh;
  __device__ __forceinline__ PlainAddr(int l) {
    const int s16 = l & 15, g2 = (l >> 4) & 1;
    l32 = l & 31;
    hh = l >> 5;
    r0 = 4 * hh + (s16 >> 2);
    trc = 2 * g2 + ((s16 & 3) >> 1);
    trh = 4 * (s16 & 1);
  }
  // Row fragment in natural k-order: features 16 ks + 8 hh .. + 7 of row l32.
  template <typename E>
  __device__ __forceinline__ ex8<E> read_row(const E* tile, int ks) const {
    return *reinterpret_cast<const ex8<E>*>(tile + l32 * D + 8 * ((2 * ks + hh) ^ swz<D>(l32)));
  }
  // Fragment for a contraction over the 16 tile rows c0 .. c0 + 15 (c0 % 16 == 0) in permuted k-order, for
  // column 32 t + l32 (see LaneAddr::read_cols).
  template <typename E>
  __device__ __forceinline__ ex8<E> read_cols(const E* tile, int c0, int t) const {
    union { struct { s16x4 lo, hi; } s; ex8<E> v; } u;
    u.s.lo = lds_read_tr(tile + (c0 + r0) * D + 8 * ((4 * t + trc) ^ swz<D>(r0)) + trh);
    u.s.hi = lds_read_tr(tile + (c0 + r0 + 8) * D + 8 * ((4 * t + trc) ^ swz<D>(r0 + 8)) + trh);
    return u.v;
  }
};

// NORM: the Norm epilogue of eq. (2) on a forward scan (the waves exchange the sums of squares of their
// 32 features of every row through LDS, one more barrier per block; wave 0 stores r).
// TWIN (head_dim 96, reverse): both scans of Algorithm 2's second loop in one workgroup of two wave groups, as
// in the kernels for head_dim 64 / 128: the two scans read the same two tensors with the roles of Y and Z
// exchanged (requires y[1] == z[0] and z[1] == y[0]), so the workgroup streams four tiles per block (x of scan
// 0, x of scan 1, Q, dO) and fetches each exactly once.  (Head_dim 256: sixteen waves of 128 state registers do
// not fit a compute unit.)
template <typename E, int D, bool REV, bool STATE_ONLY, bool NORM = false, bool TWIN = false>
__global__ __launch_bounds__((TWIN ? 4 : 2) * D, TWIN ? 2 : (D == 96 ? 3 : 2)) void scan_wide_kernel(ScanParams p) {
  static_assert(!NORM || (!REV && !STATE_ONLY), "the Norm epilogue belongs to the forward scan");
  static_assert(!TWIN || (REV && !STATE_ONLY && !NORM), "the twin workgroup is the backward pass's reverse launch");
  constexpr int B = 32;
  using C = Cfg<D, B>;
  constexpr int KS = C::KS, NT = C::NT, TILE = C::TILE;
  constexpr int NTL = TWIN ? 4 : STATE_ONLY ? 2 : 3;   // tiles of a block: [X,] Y, Z; twin: X0, X1, Y0 = Z1, Z0 = Y1
  using Loader = TileLoader<D, NTL, B, (TWIN ? 2 : 1) * NT>;
  __shared__ __attribute__((aligned(1024))) E sT[2][NTL][TILE];
  float* const sRed = NormExchange<NORM ? B * (D / 32) : 0>::get();   // [position][wave]

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int dvt = w % NT;
  const int group = TWIN ? __builtin_amdgcn_readfirstlane(w / NT) : 0;   // twin: which scan this wave belongs to
  // this wave's X, Y, Z among the tiles of a block
  const int xi = TWIN ? group : 0, yi = TWIN ? 2 + group : NTL - 2, zi = TWIN ? 3 - group : NTL - 1;
  // A dual launch (the dK and the dV scan of Algorithm 2, which both read Q and dO) has two workgroups per (chain,
  // chunk), one per scan.  They sit eight workgroup numbers apart, i.e. on the same XCD and started at about the same
  // time, so that the second read of a shared tile can hit that XCD's L2 (workgroup numbers go round the eight XCDs);
  // when the count of pairs is no multiple of eight they are neighbours instead.
  int which = group, wg = (int)blockIdx.x;
  if (!TWIN && !STATE_ONLY && p.nscan == 2) {
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
  int64_t base;
  int n;
  chain_extent(p, bi, hi, base, n);
  const int nblocks = (n + B - 1) / B;
  const int cb = p.chunk_tokens / B;
  const int nch = (nblocks + cb - 1) / cb;   // chunks this chain really has (<= p.nchunks)
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);
  if (blk_lo >= blk_hi) return;
  // pre-pass: the local state of the chunk a scan passes last is read by nobody
  if (STATE_ONLY && (REV ? chunk == 0 : chunk == nch - 1)) return;
  const int nblk = blk_hi - blk_lo;
  const uint32_t stride_n = (uint32_t)p.stride_n;
  const float l2 = log2f(p.lambda[hi]);

  Loader loader(w, l, n, stride_n);
  if (TWIN) {
    loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.x[0]) + base);
    loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.x[1]) + base);
    loader.g[2] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.y[0]) + base);
    loader.g[NTL - 1] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.z[0]) + base);
  } else {
    if (!STATE_ONLY)
      loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(which ? p.x[1] : p.x[0]) + base);
    loader.g[NTL - 2] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(which ? p.y[1] : p.y[0]) + base);
    loader.g[NTL - 1] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(which ? p.z[1] : p.z[0]) + base);
  }
  E* const gw = STATE_ONLY ? nullptr : reinterpret_cast<E*>(which ? p.w[1] : p.w[0]) + base;
  // head_dim 256: LaneAddr's precomputed offsets (one XOR per read); its read_row takes a row tile, always 0 here
  struct Pow2Addr : LaneAddr<D> {
    __device__ __forceinline__ Pow2Addr(int l_) : LaneAddr<D>(l_) {}
    __device__ __forceinline__ ex8<E> read_row(const E* tile, int ks) const { return LaneAddr<D>::read_row(tile, 0, ks); }
  };
  const std::conditional_t<(D & (D - 1)) == 0, Pow2Addr, PlainAddr<D>> la(l);

  // state slice S[:, dv tile] in accumulator layout: chunk start state, the caller's start state, or zero
  // (the pre-pass forms LOCAL states, from zero)
  f32x16 kv[NT];
  {
    const float* gs = nullptr;
    bool tr = false;
    if (!STATE_ONLY) {
      if (p.states != nullptr) {
        gs = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
        tr = (p.state_transposed >> which) & 1;
      } else if ((which ? p.init[1] : p.init[0]) != nullptr) {
        gs = (which ? p.init[1] : p.init[0]) + (int64_t)chain * (D * D);
        tr = (p.init_transposed >> which) & 1;
      }
    }
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) kv[t][v] = gs ? gs[state_index<D>(dvt, l32, hh, t, v, tr)] : 0.f;
  }
  // decay mask of the score tile S^T[c][r] (lane: r = l32; element v: c = 8 (v / 4) + 4 hh + v % 4)
  float dg[16];
#pragma unroll
  for (int v = 0; v < 16; v++) {
    const int cc = 8 * (v >> 2) + 4 * hh + (v & 3);
    const int e = REV ? cc - l32 : l32 - cc;
    dg[v] = (e >= 0) ? exp2f(l2 * (float)e) : 0.f;
  }

  // The decay of the carried state is applied lazily: the registers hold S_st with S = 2^pend S_st (pend <= 0, the
  // same for the whole wave), the carried part of a row and the update weights take the factor instead, and S_st is
  // rescaled only when 2^-pend would grow past 2^40 (for a decay near 1 once in dozens of blocks; for a strong
  // decay every block, which is the plain scheme).  At head_dim 256 the launch is bound by its vector instructions,
  // and the 128 multiplies per lane and block were a fifth of them.  bf16 only: S_st and the scaled update rows
  // are MFMA operands, and fp16's five exponent bits have no room for a factor like that (limit 0: the registers
  // are brought up to date after every block).
  constexpr float kPendLimit = std::is_same<E, __bf16>::value ? -40.f : 0.f;
  float pend = 0.f;
  auto block_at = [&](int it) { return REV ? blk_hi - 1 - it : blk_lo + it; };
  loader.issue(sT[0], block_at(0));
  for (int it = 0; it < nblk; it++) {
    const int blk = block_at(it);
    E (*const cur)[TILE] = sT[it & 1];
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's part of the block's tiles has landed
    loader.zero_tail(cur, blk);
    __syncthreads();                      // ... and everybody's; the other buffer is free (block it - 1 is done)
    if (it + 1 < nblk) loader.issue(sT[(it + 1) & 1], block_at(it + 1));
    const int nv = min(B, n - blk * B);   // valid rows of this block

    ex8<E> zf[2];
#pragma unroll
    for (int q = 0; q < 2; q++) zf[q] = la.read_cols(cur[zi], 16 * q, dvt);

    if (!STATE_ONLY) {
      // inter-block part W^T[dv][r] = sum_dk State[dk][dv] X[r][dk] and scores S^T[c][r] = sum_k Y[c][k] X[r][k]
      f32x16 acc = zero16(), sd = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        const ex8<E> xa = la.read_row(cur[xi], ks), ya = la.read_row(cur[yi], ks);
        ex8<E> f;
#pragma unroll
        for (int j = 0; j < 8; j++) f[j] = (E)kv[ks >> 1][8 * (ks & 1) + j];
        acc = mfma(to_perm_order(f), xa, acc);
        sd = mfma(ya, xa, sd);
      }
      const float carried = fast_exp2(l2 * (float)(REV ? max(nv - 1 - l32, 0) : l32 + 1) + pend);
#pragma unroll
      for (int v = 0; v < 16; v++) acc[v] *= carried;
      // intra-block part Z^T P^T
#pragma unroll
      for (int q = 0; q < 2; q++) {
        ex8<E> pd;
#pragma unroll
        for (int j = 0; j < 8; j++) pd[j] = (E)(sd[8 * q + j] * dg[8 * q + j]);
        acc = mfma(zf[q], pd, acc);
      }
      // output: lane = position l32, elements 4 g .. 4 g + 3 are value features 32 dvt + 8 g + 4 hh .. + 3
      const int pos = blk * B + l32;
      if constexpr (NORM) {
        // The next publish comes after the barrier at the top of the next block, which no wave passes before
        // every wave has collected: one exchange buffer is enough.
        norm_publish<NT>(acc, sRed, l32, hh, dvt);
        __syncthreads();
        const float r = norm_collect<NT>(sRed, l32, 1.f / (float)D, p.eps);
#pragma unroll
        for (int v = 0; v < 16; v++) acc[v] *= r;
        if (dvt == 0 && hh == 0 && pos < n) p.rstd[rstd_chain_offset(p, bi, hi) + pos] = r;
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
    }
    // state slice <- lambda^nv state + Y^T decay(Z): element j of a Z fragment is row 16 q + 8 (j / 4) + 4 hh + j % 4
    pend = uniform(pend + l2 * (float)nv);
    if (pend < kPendLimit) {   // (wave-uniform) bring the registers up to date
      const float scale = uniform(fast_exp2(pend));
#pragma unroll
      for (int t = 0; t < NT; t++)
#pragma unroll
        for (int v = 0; v < 16; v++) kv[t][v] *= scale;
      pend = 0.f;
    }
#pragma unroll
    for (int q = 0; q < 2; q++) {
      ex8<E> zd;
#pragma unroll
      for (int j = 0; j < 8; j++) {
        const int c = 16 * q + 8 * (j >> 2) + 4 * hh + (j & 3);
        zd[j] = (E)((float)zf[q][j] * fast_exp2(l2 * (float)(REV ? c + 1 : max(nv - 1 - c, 0)) - pend));
      }
#pragma unroll
      for (int t = 0; t < NT; t++) kv[t] = mfma(la.read_cols(cur[yi], 16 * q, t), zd, kv[t]);
    }
  }

  // the state after the chunk: the pre-pass keeps every chunk's, a scan hands out the one after its last block
  float* gf = nullptr;
  bool trf = false;
  if (STATE_ONLY) {
    gf = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
  } else if ((which ? p.fin[1] : p.fin[0]) != nullptr && (REV ? chunk == 0 : chunk == nch - 1)) {
    gf = (which ? p.fin[1] : p.fin[0]) + (int64_t)chain * (D * D);
    trf = (p.fin_transposed >> which) & 1;
  }
  if (gf != nullptr) {
    const float scale = fast_exp2(pend);   // the pending decay
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) gf[state_index<D>(dvt, l32, hh, t, v, trf)] = kv[t][v] * scale;
  }
}

template <typename E, int D>
hipError_t launch_wide(bool reverse, bool state_only, const ScanParams& p, hipStream_t s) {
  const dim3 g((unsigned)((int64_t)p.batch * p.heads * p.nchunks * (state_only ? 1 : p.nscan))), b(2 * D);
  if constexpr (D == 96) {
    if (!state_only && reverse && p.nscan == 2 && p.y[1] == p.z[0] && p.z[1] == p.y[0]) {
      hipLaunchKernelGGL((scan_wide_kernel<E, D, true, false, false, true>),
                         dim3((unsigned)((int64_t)p.batch * p.heads * p.nchunks)), dim3(4 * D), 0, s, p);
      return hipGetLastError();
    }
  }
  if (!state_only && !reverse && p.rstd != nullptr) {
    hipLaunchKernelGGL((scan_wide_kernel<E, D, false, false, true>), g, b, 0, s, p);
  } else if (state_only) {
    if (reverse) hipLaunchKernelGGL((scan_wide_kernel<E, D, true, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((scan_wide_kernel<E, D, false, true>), g, b, 0, s, p);
  } else {
    if (reverse) hipLaunchKernelGGL((scan_wide_kernel<E, D, true, false>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((scan_wide_kernel<E, D, false, false>), g, b, 0, s, p);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_scan_wide(int dtype, int head_dim, bool reverse, bool state_only, const ScanParams& p,
                            hipStream_t s) {
  if ((int64_t)p.batch * p.heads * p.nchunks == 0 || p.n == 0) return hipSuccess;
  if (head_dim == 256)
    return dtype == kF16 ? launch_wide<_Float16, 256>(reverse, state_only, p, s)
                         : launch_wide<__bf16, 256>(reverse, state_only, p, s);
  return dtype == kF16 ? launch_wide<_Float16, 96>(reverse, state_only, p, s)
                       : launch_wide<__bf16, 96>(reverse, state_only, p, s);
}

}  // namespace la2
