// Full-block bf16 scan kernel (B = 64 positions, one workgroup per compute unit) for the decayed causal scan
// (Algorithm 1; both loops of Algorithm 2), gfx950; and the choice between it and the half-block kernel.
// Layout notes: la2_bf16_common.h.
#include "la2_bf16_common.h"

namespace la2 {
namespace {
using namespace bf16k;

// NORM: the Norm epilogue of eq. (2) on a forward scan: the waves that hold the feature tiles of a row
// exchange their sums of squares through LDS (one more workgroup barrier per block), scale the finished
// tile and store r.
template <typename E, int D, bool REV, bool NORM = false>
__global__ __launch_bounds__(kThreads, 1) void scan_bf16_kernel(ScanParams p) {
  static_assert(!NORM || !REV, "the Norm epilogue belongs to the forward pass");
  using C = Cfg<D>;
  constexpr int KS = C::KS, NT = C::NT, RT = C::RT, TILE = C::TILE, LW = C::LW;
  // two tile buffers as two distinct LDS objects ([X, Y, Z] each) so that reads of one buffer are
  // provably independent of the direct loads in flight into the other
  __shared__ __attribute__((aligned(1024))) E sT0[3][TILE];
  __shared__ __attribute__((aligned(1024))) E sT1[3][TILE];
  __shared__ __attribute__((aligned(1024))) E sT2[3][TILE];
  __shared__ __attribute__((aligned(16))) E sW[4][32 * RT * LW];
  float* const sRed = NormExchange<NORM ? 2 * kB * NT : 0>::get();   // [block parity][position][feature tile]
  // vector-memory operations a wave issues per block: direct loads (3 tiles), output stores and r
  constexpr int LOADS_PER_BLOCK = 3 * C::DMA_PER_WAVE, STORES_PER_BLOCK = 32 * RT * 4 / 64 + (NORM ? RT : 0);
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
  int64_t base;
  int n;
  chain_extent(p, bi, hi, base, n);
  const uint32_t stride_n = (uint32_t)p.stride_n;
  const uint32_t chain_bytes = ((uint32_t)(n - 1) * stride_n + D) * 2u;
  const __amdgpu_buffer_rsrc_t bw =
      make_rsrc(reinterpret_cast<E*>(which ? p.w[1] : p.w[0]) + base, chain_bytes);
  const float l2 = log2f(p.lambda[hi]);
  // Norm epilogue: r of this chain's positions; stores past position n - 1 are dropped
  const __amdgpu_buffer_rsrc_t brs =
      make_rsrc(NORM ? p.rstd + rstd_chain_offset(p, bi, hi) : nullptr, NORM ? (uint32_t)n * 4u : 0u);

  const int nblocks = (n + kB - 1) / kB;
  const int cb = p.chunk_tokens / kB;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);
  if (blk_lo >= blk_hi) return;
  const int nblk = blk_hi - blk_lo;

  TileLoader<D, 3> loader(w, l, n, stride_n);
  loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(which ? p.x[1] : p.x[0]) + base);
  loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(which ? p.y[1] : p.y[0]) + base);
  loader.g[2] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(which ? p.z[1] : p.z[0]) + base);
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
  ex8<E> xa[RT][KS];
  auto read_xa = [&](const E (*sB)[TILE], int ks) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < RT; i++) xa[i][ks] = la.read_row(sB[0], rt0 + i, ks);
  };
#pragma unroll
  for (int ks = 0; ks < AHEAD; ks++) read_xa(sT0, ks);

  // State tile ks / 2, k-step ks % 2 as a bf16 MFMA operand in NATURAL k-order: the accumulator
  // layout gives permuted order, the exchange between the wave's halves undoes it, so that the X
  // fragments serve the score product and the inter-block product unchanged.
  auto state_operand = [&](int ks) __attribute__((always_inline)) {
    ex8<E> f;
#pragma unroll
    for (int j = 0; j < 8; j++) f[j] = (E)kv[ks >> 1][8 * (ks & 1) + j];
    return to_perm_order(f);   // the exchange is its own inverse
  };

  // Finished output of the previous block (transposed: value feature x position), stored while the
  // next block computes; and the first state operand of the block about to be computed.
  f32x16 outp[RT];
#pragma unroll
  for (int i = 0; i < RT; i++) outp[i] = zero16();
  ex8<E> sa_first = state_operand(0);
  E* const stage = sW[w];
  constexpr int NST = 32 * RT * 4 / 64;   // 16-byte stores per lane and block
  // Output of block `oblk` in three steps: pack to bf16 and stage through LDS (so that the stores are
  // 16 bytes per lane, 64 contiguous bytes per row); read back; store.  `valid` false (no previous
  // block): the offset is pushed out of the buffer's range and the stores are dropped.
  auto out_pack = [&](int i) __attribute__((always_inline)) {
#pragma unroll
    for (int g = 0; g < 4; g++) {
      ex4<E> pk;
#pragma unroll
      for (int e = 0; e < 4; e++) pk[e] = (E)outp[i][4 * g + e];
      const int row = 32 * i + l32;
      *reinterpret_cast<ex4<E>*>(stage + row * LW + 8 * (g ^ ((row >> 2) & 3)) + 4 * hh) = pk;
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
      // reverse scans run as the dual launch of the backward pass, a third of whose traffic is stores: the
      // streaming write-through policy (nt + sc1) measured 1-3 % faster there; forward keeps the default
      __builtin_amdgcn_raw_buffer_store_b128(ov[i], bw, valid ? off : 0xFFFFFFF0u, 0, REV ? 18 : 0);
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
    E (*const sCur)[TILE] = cur == 0 ? sT0 : (cur == 1 ? sT1 : sT2);     // block it
    E (*const sNext)[TILE] = cur == 0 ? sT1 : (cur == 1 ? sT2 : sT0);    // block it + 1 (in flight or landed)
    E (*const sAhead)[TILE] = cur == 0 ? sT2 : (cur == 1 ? sT0 : sT1);   // block it + 2 (free since block it - 1)
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    const bool has_next = it + 1 < nblk, has_ahead = it + 2 < nblk;
    const int nb = REV ? blk - 1 : blk + 1, pb = REV ? blk + 1 : blk - 1;
    const E* tY = sCur[1];
    const E* tZ = sCur[2];
    uint32_t doff[C::DMA_PER_WAVE];
    loader.offsets(REV ? blk - 2 : blk + 2, has_ahead, doff);

    ex8<E> zf[2][2];     // Z columns of this wave's value tile: [key-tile slot][k-step], permuted k-order
    ex8<E> zd[2][2];     // the same, weighted for the state update
    ex8<E> yt[NT][2][2]; // Y columns (key features): [key-feature tile][slot][k-step], permuted k-order
    ex8<E> xb[RT][KS], yb[RT][KS], yo[KS];   // phase 2 operands
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
    ex8<E> sa = sa_first;
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
    ex8<E> pd[RT][2], po[2];
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
        for (int i = 0; i < RT; i++) pd[i][v >> 3][v & 7] = (E)(sd[i][v] * dg[v]);
        po[v >> 3][v & 7] = (E)((so[v] * oa) * ou[v]);
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
    if constexpr (NORM) {
      // Two exchange buffers, by block parity: a wave that runs ahead into the next block (whose last
      // block has no tile barrier) must not overwrite sums that a slower wave has yet to read.
      float* const red = sRed + (it & 1) * (kB * NT);
#pragma unroll
      for (int i = 0; i < RT; i++) norm_publish<NT>(outp[i], red + 32 * (rt0 + i) * NT, l32, hh, dvt);
      lds_barrier();
#pragma unroll
      for (int i = 0; i < RT; i++) {
        const float r = norm_collect<NT>(red + 32 * (rt0 + i) * NT, l32, 1.f / (float)D, p.eps);
#pragma unroll
        for (int v = 0; v < 16; v++) outp[i][v] *= r;
        pin(outp[i]);
        // the lanes that hold r of a position store it; every other lane's store is dropped
        const uint32_t roff =
            (dvt == 0 && hh == 0) ? (uint32_t)(blk * kB + 32 * (rt0 + i) + l32) * 4u : 0xFFFFFFF0u;
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(r), brs, roff, 0, 0);
      }
      LA2_SLOT_END();
    }
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

}  // namespace

int block_size_bf16(int) { return bf16k::kB; }

namespace {
template <typename E>
hipError_t launch_full(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (int64_t)p.batch * p.heads * p.nchunks * p.nscan;
  dim3 g((unsigned)grid), b(kThreads);
  if (head_dim == 128) {
    if (reverse) hipLaunchKernelGGL((scan_bf16_kernel<E, 128, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((scan_bf16_kernel<E, 128, false>), g, b, 0, s, p);
  } else {
    if (reverse) hipLaunchKernelGGL((scan_bf16_kernel<E, 64, true>), g, b, 0, s, p);
    else if (p.rstd != nullptr) hipLaunchKernelGGL((scan_bf16_kernel<E, 64, false, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((scan_bf16_kernel<E, 64, false>), g, b, 0, s, p);
  }
  return hipGetLastError();
}
}  // namespace

hipError_t launch_scan_bf16_full(int dtype, int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  return dtype == kF16 ? launch_full<_Float16>(head_dim, reverse, p, s) : launch_full<__bf16>(head_dim, reverse, p, s);
}

// Which scan kernel a launch gets.
hipError_t launch_scan_bf16(int dtype, int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (int64_t)p.batch * p.heads * p.nchunks * p.nscan;
  if (grid == 0 || p.n == 0) return hipSuccess;
  // the half-block kernel measured faster at every launch size, also at one workgroup per compute unit; it is
  // also the only one that takes start states, hands out final states, has the Norm epilogue at both head
  // dimensions and can form the reverse chunk states on the side
  const bool with_state = p.init[0] || p.init[1] || p.fin[0] || p.fin[1];
  const bool half = p.variant != 1 || with_state || p.rstd != nullptr || p.acc_states != nullptr;
  if (half && p.chunk_tokens % 32 == 0) {
    const bool twin = p.nscan == 2 && p.y[1] == p.z[0] && p.z[1] == p.y[0];
    return launch_scan_bf16_half(dtype, head_dim, reverse, twin, p, s);
  }
  return launch_scan_bf16_full(dtype, head_dim, reverse, p, s);
}

}  // namespace la2
