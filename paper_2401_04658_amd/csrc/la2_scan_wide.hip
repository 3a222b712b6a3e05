// Scan kernel for the other head dimensions (96 and 256), 16-bit data, gfx950: the decayed causal scan
// (Algorithm 1; both loops of Algorithm 2) and, as a template flag, the chunk-state pre-pass for them.
//
// Same arithmetic, MFMA layouts and direct HBM -> LDS tile loads as the kernels for head_dim 64 / 128
// (la2_bf16_common.h): blocks of 32 positions, D / 32 waves (wave w owns value features 32 w .. 32 w + 31 and that
// slice of the fp32 state in accumulators), two tile buffers (the next block's tiles stream in while this block
// is computed), one barrier per block (two with the Norm epilogue, three at head_dim 256).  Head_dim 256 makes a
// workgroup of 8 waves with 128 state registers per lane, which leaves no register to spare; head_dim 96 one of
// 3 waves (6 in the twin form).  What differs from those kernels:
//   - the block body is a sequence of slots closed by scheduling barriers (LDS reads issued ahead of their MFMAs);
//   - transposing reads take their columns in a permuted order (read_cols_pi), so that the state operand needs no
//     lane shuffle and a lane stores 16 bytes at a time;
//   - lane-dependent loop invariants live in LDS or scalar registers, not in vector registers;
//   - head_dim 256: one masked score tile per workgroup instead of one per wave (waves 0 .. 3 compute a quarter
//     each while waves 4 .. 7 issue the tile loads), and a block's last two steps run behind the next block's barrier.
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
    // lane s of a group of sixteen takes the 8-byte piece with the two bits of its index s % 4 exchanged (read_cols_pi)
    trc = 2 * g2 + (s16 & 1);
    trh = 4 * ((s16 & 3) >> 1);
  }
  // Row fragment in natural k-order: features 16 ks + 8 hh .. + 7 of row l32.
  template <typename E>
  __device__ __forceinline__ ex8<E> read_row(const E* tile, int ks) const {
    return *reinterpret_cast<const ex8<E>*>(tile + l32 * D + 8 * ((2 * ks + hh) ^ swz<D>(l32)));
  }
  // Fragment for a contraction over the 16 tile rows c0 .. c0 + 15 (c0 % 16 == 0) in permuted k-order (see
  // LaneAddr::read_cols), for column 32 t + pi(l32), pi = bits 2 and 3 of the index exchanged.
  template <typename E>
  __device__ __forceinline__ ex8<E> read_cols_pi(const E* tile, int c0, int t) const {
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
  constexpr bool SHP = D == 256 && !STATE_ONLY;   // shared score tile (see sP below)
  // The tile loads of a block: every wave its share.  With the shared score tile, waves 4 .. 7 load (one
  // instruction per slot of the inter-block product, so that eight waves do not queue 48 of them at the tile
  // addresser right after the barrier) while waves 0 .. 3 compute the score tile.
  constexpr int NLW = SHP ? 4 : (TWIN ? 2 : 1) * NT;
  using Loader = TileLoader<D, NTL, B, NLW>;
  constexpr int NDMA = NTL * Loader::DMA_PER_WAVE;
  __shared__ __attribute__((aligned(1024))) E sT[2][NTL][TILE];
  float* const sRed = NormExchange<NORM ? B * (D / 32) : 0>::get();   // [position][wave]
  // Head_dim 256: the masked, decayed score tile of a block is the same for the eight waves.  Waves 0 .. 3 compute a
  // 16 x 16 quarter each (16x16x32 MFMAs) and leave it in LDS in 16 bits, in the order in which a lane takes it as
  // the intra-block product's operand: row r (80 bytes apart: sixteen rows fall into sixteen different 16-byte bank
  // groups) holds, for k-step q and lane half hh, the eight columns c = 16 q + 8 (j / 4) + 4 hh + j % 4.  Per wave and
  // block that is 16 MFMAs, 16 LDS reads and the 16 accumulators of a score tile less, for one more barrier.
  constexpr int PROW = 40;
  // Without the Norm epilogue the block's last two steps (intra-block product, output store) wait until the next
  // block's first barrier has been passed, which orders them after the score tile's writes as well: one barrier
  // per block again, two score-tile buffers by block parity, and the output stores of a block overlap the next
  // block's first LDS reads.
  constexpr bool DEFER = SHP && !NORM;
  __shared__ __attribute__((aligned(16))) E sP[DEFER ? 2 : 1][SHP ? 32 * PROW : 8];
  __shared__ f32x4 sDg[(STATE_ONLY || SHP) ? 1 : 4][64];               // decay mask, [element group][lane]

  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63, l32 = l & 31, hh = l >> 5;
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

  const bool loads = !SHP || w >= 4;
  Loader loader(SHP ? (w & 3) : w, l, n, stride_n);
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
    int tp0, tp1;   // as LaneAddr's tr0, tr1 with the bits of the piece index exchanged (read_cols_pi)
    __device__ __forceinline__ Pow2Addr(int l_) : LaneAddr<D>(l_) {
      const int h = l_ >> 5, s16 = l_ & 15, g2 = (l_ >> 4) & 1;
      const int trcp = 2 * g2 + (s16 & 1), trhp = 4 * ((s16 & 3) >> 1);
      const int r0 = 4 * h + (s16 >> 2), r1 = r0 + 8;
      tp0 = r0 * D + 8 * (trcp ^ swz<D>(r0)) + trhp;
      tp1 = r1 * D + 8 * (trcp ^ swz<D>(r1)) + trhp;
    }
    __device__ __forceinline__ ex8<E> read_cols_pi(const E* tile, int c0, int t) const {
      union { struct { s16x4 lo, hi; } s; ex8<E> v; } u;
      u.s.lo = lds_read_tr(tile + c0 * D + (tp0 ^ (32 * t)));
      u.s.hi = lds_read_tr(tile + c0 * D + (tp1 ^ (32 * t)));
      return u.v;
    }
    __device__ __forceinline__ ex8<E> read_row(const E* tile, int ks) const { return LaneAddr<D>::read_row(tile, 0, ks); }
  };
  const std::conditional_t<(D & (D - 1)) == 0, Pow2Addr, PlainAddr<D>> la(l);

  // Every transposing read takes the columns of its tile in the order pi (read_cols_pi: bits 2 and 3 of the index
  // exchanged).  Element v of state tile t in a lane is therefore value feature dv = 32 dvt + pi(l32) and key feature
  // dk = 32 t + pi(m), m = 8 (v / 4) + 4 hh + v % 4 the accumulator row: the eight elements a lane converts for a
  // k-step are key features 16 ks + 8 hh .. + 7, the order of a row fragment of X, so the state operand needs no
  // lane shuffle; and a lane's sixteen outputs are value features 32 dvt + 16 (v / 8) + 8 hh + v % 8: two 16-byte stores.
  auto state_index_pi = [&](int t, int v, bool transposed) {
    const int dk = 32 * t + 16 * (v >> 3) + 8 * hh + 4 * ((v >> 2) & 1) + (v & 3);
    const int dv = 32 * dvt + ((l32 & 19) | ((l32 & 4) << 1) | ((l32 & 8) >> 1));
    return transposed ? dv * D + dk : dk * D + dv;
  };
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
      for (int v = 0; v < 16; v++) kv[t][v] = gs ? gs[state_index_pi(t, v, tr)] : 0.f;
  }
  // decay mask of the score tile S^T[c][r] (lane: r = l32; element v: c = 8 (v / 4) + 4 hh + v % 4): the same for
  // every wave and every block.  It lives in LDS, four elements per lane and read, not in sixteen registers: the
  // state slice leaves none to spare, and a register spilled inside the block loop is reloaded through the vector
  // memory counter, behind the tile loads in flight.
  if (!STATE_ONLY && !SHP && w == 0) {
#pragma unroll
    for (int g = 0; g < 4; g++) {
      f32x4 m;
#pragma unroll
      for (int e4 = 0; e4 < 4; e4++) {
        const int cc = 8 * g + 4 * hh + e4;
        const int e = REV ? cc - l32 : l32 - cc;
        m[e4] = (e >= 0) ? exp2f(l2 * (float)e) : 0.f;
      }
      sDg[g][l] = m;
    }
  }   // (the first block's barrier comes before the first read)

  // The decay of the carried state is applied lazily: the registers hold S_st with S = 2^pend S_st (pend <= 0, the
  // same for the whole wave), the carried part of a row and the update weights take the factor instead, and S_st is
  // rescaled only when 2^-pend would grow past 2^40 (for a decay near 1 once in dozens of blocks; for a strong
  // decay every block, which is the plain scheme).  At head_dim 256 the launch is bound by its vector instructions,
  // and the 128 multiplies per lane and block were a fifth of them.  bf16 only: S_st and the scaled update rows
  // are MFMA operands, and fp16's five exponent bits have no room for a factor like that (limit 0: the registers
  // are brought up to date after every block).
  constexpr float kPendLimit = std::is_same<E, __bf16>::value ? -40.f : 0.f;
  float pend = 0.f;

  // The block body is laid out in slots, each closed by a scheduling barrier: a slot issues its MFMAs first, then the
  // LDS reads and the conversions that the NEXT slot's MFMAs take, and pins the results at its end (see pin()).  Left
  // to itself the compiler reads every operand right before the MFMA that takes it, and the wave then sits out an LDS
  // round trip per k-step with one other wave on its SIMD to cover it.
#define LA2_SLOT_END()                 \
  do {                                 \
    asm volatile("" ::: "memory");     \
    __builtin_amdgcn_sched_barrier(0); \
  } while (0)
  constexpr int AH1 = SHP ? 3 : 1;   // slots by which the LDS reads run ahead of their MFMAs: inter-block product,
  constexpr int AH3 = D == 256 ? 2 : 1;   // state update (a slot of one MFMA is shorter than an LDS round trip)
  constexpr int NU = 2 * NT;                           // MFMAs of a block's state update: (k-step q, key tile t), q-major
  constexpr int NS3 = (NU + 1) / 2;                    // ... in slots of two
  constexpr int PPS = NS3 >= 8 ? 2 : NS3 >= 4 ? 4 : 8; // elements of the masked score tile converted per update slot
  auto state_operand = [&](int ks) __attribute__((always_inline)) {
    ex8<E> f;
#pragma unroll
    for (int j = 0; j < 8; j++) f[j] = (E)kv[ks >> 1][8 * (ks & 1) + j];
    return f;
  };
  // Update weights of a full block: lambda^(31 - c) forward, lambda^(c + 1) reverse, for row c = cu + 4 hh with
  // cu = 16 q + 8 (j / 4) + j % 4, as a wave-uniform factor (sixteen scalar registers) times a lane factor, both <= 1
  // for any decay; the block loop then spends two multiplies per element on them instead of an exponential.
  float wu[16];
#pragma unroll
  for (int i = 0; i < 16; i++) {
    const int cu = 16 * (i >> 3) + 8 * ((i >> 2) & 1) + (i & 3);
    wu[i] = scalar_reg(exp2f(l2 * (float)(REV ? cu : 27 - cu)));
  }
  const float wl = exp2f(l2 * (float)(REV ? 4 * hh + 1 : 4 - 4 * hh));
  ex8<E> sa_first = {};
  if (!STATE_ONLY) sa_first = state_operand(0);

  // output: lane = position l32, elements 8 g .. 8 g + 7 are value features 32 dvt + 16 g + 8 hh .. + 7
  // (lr, lh: the lane's position and half; the deferred tail makes them from the lane number inside the loop, so that
  // no lane-dependent address waits in a register, or in scratch, over the block loop)
  auto store_block = [&](const f32x16& a, int blkv, int lr, int lh) __attribute__((always_inline)) {
    const int pos = blkv * B + lr;
    if (pos < n) {
      // wave-uniform base + 32-bit byte offset (a chain spans < 4 GiB, checked on the host)
      char* const orow = reinterpret_cast<char*>(gw) + ((uint32_t)pos * stride_n + (uint32_t)(32 * dvt + 8 * lh)) * 2u;
#pragma unroll
      for (int g = 0; g < 2; g++) {
        ex8<E> pk;
#pragma unroll
        for (int e = 0; e < 8; e++) pk[e] = (E)a[8 * g + e];
        *reinterpret_cast<ex8<E>*>(orow + 32 * g) = pk;
      }
    }
  };
  // deferred tail of a block: intra-block part Z^T P^T from the shared score tile, then the output
  f32x16 acc_prev = zero16();
  ex8<E> zf_prev[2] = {};
  int blk_prev = 0;
  auto finish_block = [&](f32x16 a, const ex8<E> (&zfv)[2], int blkv, const E* tile) __attribute__((always_inline)) {
    int lo = l;
    asm volatile("" : "+v"(lo));
    const int lr = lo & 31, lh = lo >> 5;
    ex8<E> pv[2];
#pragma unroll
    for (int q = 0; q < 2; q++) pv[q] = *reinterpret_cast<const ex8<E>*>(tile + lr * PROW + 16 * q + 8 * lh);
#pragma unroll
    for (int q = 0; q < 2; q++) a = mfma(zfv[q], pv[q], a);
    store_block(a, blkv, lr, lh);
  };
  auto block_at = [&](int it) { return REV ? blk_hi - 1 - it : blk_lo + it; };
  if (loads) loader.issue(sT[0], block_at(0));
  for (int it = 0; it < nblk; it++) {
    const int blk = block_at(it);
    E (*const cur)[TILE] = sT[it & 1];
    // This wave's part of the block's tiles has landed.  Vector memory operations complete in the order of their
    // issue, and the only ones younger than those loads are the two output stores per lane of the block before
    // (always issued: every block has a valid first row; a Norm scan's r store comes before them): they may stay in
    // flight, a store's acknowledgement takes as long as a load.
    // (With the deferred tail the stores are issued before the block's loads and have had a block's time.)
    if (STATE_ONLY || DEFER || it == 0) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    else __builtin_amdgcn_s_waitcnt(0x0F72);                                  // vmcnt(2)
    if (loads) loader.zero_tail(cur, blk);
    __syncthreads();                      // ... and everybody's; the other buffer is free (block it - 1 is done)
    if constexpr (DEFER) {
      if (it > 0) finish_block(acc_prev, zf_prev, blk_prev, sP[(it - 1) & 1]);
    }
    const bool load_next = loads && it + 1 < nblk;
    uint32_t doff[Loader::DMA_PER_WAVE];
    if constexpr (SHP) {
      loader.offsets(block_at(it + 1), load_next, doff);
    } else {
      if (load_next) loader.issue(sT[(it + 1) & 1], block_at(it + 1));
    }
    const int nv = min(B, n - blk * B);   // valid rows of this block
    if constexpr (SHP) {
      if (w < 4) {
        // quarter (a, b) of S^T[c][r] = sum_k Y[c][k] X[r][k]: c = 16 a + 4 (lane / 16) + v, r = 16 b + lane % 16.
        // Every address and mask value is made here from the lane number, not kept in registers over the loop.
        int lo = l;
        asm volatile("" : "+v"(lo));
        const int qa = w >> 1, qb = w & 1, l16 = lo & 15, pg = lo >> 4;
        const int ra = 16 * qa + l16, rb = 16 * qb + l16;
        const E* const pa = cur[yi] + ra * D + 8 * (pg ^ (swz<D>(ra) & 3));
        const E* const pb = cur[xi] + rb * D + 8 * (pg ^ (swz<D>(rb) & 3));
        const int sa4 = 32 * (swz<D>(ra) >> 2), sb4 = 32 * (swz<D>(rb) >> 2);   // chunk bits 2, 3 (elements)
        f32x4 s4 = {0.f, 0.f, 0.f, 0.f};
        if (REV ? w != 1 : w != 2) {   // (the quarter with every c > r, or every c < r in a reverse scan, is all zero)
          ex8<E> fa[D / 32], fb[D / 32];   // all sixteen reads in flight at once (the registers are free here)
#pragma unroll
          for (int kk = 0; kk < D / 32; kk++) {
            fa[kk] = *reinterpret_cast<const ex8<E>*>(pa + ((32 * kk) ^ sa4));
            fb[kk] = *reinterpret_cast<const ex8<E>*>(pb + ((32 * kk) ^ sb4));
          }
#pragma unroll
          for (int kk = 0; kk < D / 32; kk++) {
            pin(fa[kk]);
            pin(fb[kk]);
          }
#pragma unroll
          for (int kk = 0; kk < D / 32; kk++) s4 = mfma16(fa[kk], fb[kk], s4);
        }
        ex4<E> pk;
#pragma unroll
        for (int v = 0; v < 4; v++) {
          const int e = REV ? (16 * qa + 4 * pg + v) - rb : rb - (16 * qa + 4 * pg + v);
          pk[v] = (E)(e >= 0 ? s4[v] * fast_exp2(l2 * (float)e) : 0.f);
        }
        *reinterpret_cast<ex4<E>*>(sP[DEFER ? it & 1 : 0] + rb * PROW + 16 * qa + 8 * (pg & 1) + 4 * (pg >> 1)) = pk;
      }
    }
    const E* const tX = cur[xi];
    const E* const tY = cur[yi];
    const E* const tZ = cur[zi];

    // (wave-uniform) the decay this block adds to the pending one, and whether the registers are brought up to date
    const float pend_new = uniform(pend + l2 * (float)nv);
    const bool rescale = pend_new < kPendLimit;
    const float pend_upd = rescale ? 0.f : pend_new;   // the registers' exponent once this block's update is in

    ex8<E> zf[2], zd[2], yt[NU];
    auto read_yt = [&](int idx) __attribute__((always_inline)) {
      if (idx < NU) yt[idx] = la.read_cols_pi(tY, 16 * (idx / NT), idx % NT);
    };
    // update weights on the Z fragments (element j of fragment q is row c = 16 q + 8 (j / 4) + 4 hh + j % 4)
    auto weigh_z = [&]() __attribute__((always_inline)) {
      if (REV || nv == B) {
        const float ls = wl * fast_exp2(-pend_upd);
#pragma unroll
        for (int q = 0; q < 2; q++)
#pragma unroll
          for (int j = 0; j < 8; j++) zd[q][j] = (E)(((float)zf[q][j] * ls) * wu[8 * q + j]);
      } else {   // ragged last block of a forward scan: lambda^(nv - 1 - c), clamped for the rows past the end
#pragma unroll
        for (int q = 0; q < 2; q++)
#pragma unroll
          for (int j = 0; j < 8; j++) {
            const int c = 16 * q + 8 * (j >> 2) + 4 * hh + (j & 3);
            zd[q][j] = (E)((float)zf[q][j] * fast_exp2(l2 * (float)max(nv - 1 - c, 0) - pend_upd));
          }
      }
      pin(zd[0]);
      pin(zd[1]);
    };
    f32x16 acc = zero16(), sd = zero16();
    if constexpr (!STATE_ONLY) {
      // inter-block part W^T[dv][r] = sum_dk State[dk][dv] X[r][dk] and scores S^T[c][r] = sum_k Y[c][k] X[r][k],
      // one k-step of each per slot
      ex8<E> xa[KS], ya[KS];
#pragma unroll
      for (int a = 0; a < AH1; a++) {
        xa[a] = la.read_row(tX, a);
        if constexpr (!SHP) ya[a] = la.read_row(tY, a);
      }
      ex8<E> sa = sa_first;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        if (ks + AH1 < KS) {
          xa[ks + AH1] = la.read_row(tX, ks + AH1);
          if constexpr (!SHP) ya[ks + AH1] = la.read_row(tY, ks + AH1);
        }
        if (ks == KS - 3 || ks == KS - 2) zf[ks - (KS - 3)] = la.read_cols_pi(tZ, 16 * (ks - (KS - 3)), dvt);
        if (ks == KS - 1) {
#pragma unroll
          for (int i = 0; i < 2 * AH3; i++) read_yt(i);
        }
        __builtin_amdgcn_sched_barrier(0);   // the reads above are issued before the MFMAs below
        acc = mfma(sa, xa[ks], acc);
        if constexpr (!SHP) sd = mfma(ya[ks], xa[ks], sd);
        if (ks + 1 < KS) {
          sa = state_operand(ks + 1);
          pin(sa);
          pin(xa[ks + 1]);
          if constexpr (!SHP) pin(ya[ks + 1]);
        }
        if constexpr (SHP) {
          if (ks < NDMA && load_next) loader.issue_one(sT[(it + 1) & 1], doff, ks);
        }
        pin(acc);
        if constexpr (!SHP) pin(sd);
        LA2_SLOT_END();
      }
      // the carried part takes the decay at this lane's position (and the pending decay of the registers)
      const float carried = fast_exp2(l2 * (float)(REV ? max(nv - 1 - l32, 0) : l32 + 1) + pend);
#pragma unroll
      for (int v = 0; v < 16; v++) acc[v] *= carried;
      pin(acc);
    } else {
#pragma unroll
      for (int q = 0; q < 2; q++) zf[q] = la.read_cols_pi(tZ, 16 * q, dvt);
#pragma unroll
      for (int i = 0; i < 2 * AH3; i++) read_yt(i);
    }
    weigh_z();
    if (rescale) {
      const float scale = uniform(fast_exp2(pend_new));
#pragma unroll
      for (int t = 0; t < NT; t++)
#pragma unroll
        for (int v = 0; v < 16; v++) kv[t][v] *= scale;
    }
    pend = pend_upd;
    LA2_SLOT_END();

    // state slice <- (decayed) state + Y^T weighted(Z); side work: the masked, decayed score tile in 16 bits
    ex8<E> pd[2];
    f32x4 dgv[(PPS + 3) / 4];
#pragma unroll
    for (int s3 = 0; s3 < NS3; s3++) {
      read_yt(2 * (s3 + AH3));
      read_yt(2 * (s3 + AH3) + 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < 2; u++) {
        const int idx = 2 * s3 + u;
        if (idx < NU) kv[idx % NT] = mfma(yt[idx], zd[idx / NT], kv[idx % NT]);
      }
      if constexpr (!STATE_ONLY && !SHP) {
        if (PPS * s3 < 16) {
          if ((PPS * s3) % 4 == 0) {
#pragma unroll
            for (int g = 0; g < (PPS + 3) / 4; g++) dgv[g] = sDg[(PPS * s3) / 4 + g][l];
          }
#pragma unroll
          for (int e = 0; e < PPS; e++) {
            const int v = PPS * s3 + e;
            pd[v >> 3][v & 7] = (E)(sd[v] * dgv[PPS >= 4 ? e >> 2 : 0][v & 3]);
          }
          pin(pd[(PPS * s3) >> 3]);
        }
      }
#pragma unroll
      for (int u = 0; u < 2; u++) {
        if (2 * s3 + u < NU) pin(kv[(2 * s3 + u) % NT]);
        if (2 * s3 + 2 + u < NU) pin(yt[2 * s3 + 2 + u]);
      }
      LA2_SLOT_END();
    }

    if constexpr (DEFER) {
      sa_first = state_operand(0);   // the first state operand of the next block
      pin(sa_first);
      acc_prev = acc;
      zf_prev[0] = zf[0];
      zf_prev[1] = zf[1];
      blk_prev = blk;
    } else if constexpr (!STATE_ONLY) {
      // intra-block part Z^T P^T, and the first state operand of the next block
      if constexpr (SHP) {
        // The quarters were written at the top of the block; the next block's are written after its first barrier,
        // which no wave passes before every wave has read these.
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 2; q++) pd[q] = *reinterpret_cast<const ex8<E>*>(sP[0] + l32 * PROW + 16 * q + 8 * hh);
      }
#pragma unroll
      for (int q = 0; q < 2; q++) acc = mfma(zf[q], pd[q], acc);
      sa_first = state_operand(0);
      pin(sa_first);
      pin(acc);
      LA2_SLOT_END();
      // output: lane = position l32, elements 8 g .. 8 g + 7 are value features 32 dvt + 16 g + 8 hh .. + 7
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
      store_block(acc, blk, l32, hh);
    }
  }
  if constexpr (DEFER) {
    __syncthreads();
    finish_block(acc_prev, zf_prev, blk_prev, sP[(nblk - 1) & 1]);
  }
#undef LA2_SLOT_END

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
      for (int v = 0; v < 16; v++) gf[state_index_pi(t, v, trf)] = kv[t][v] * scale;
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
