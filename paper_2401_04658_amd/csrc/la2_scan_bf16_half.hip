// Half-block 16-bit scan kernel for head_dim 128 and 64 (B = 32 positions, two waves per SIMD) and its twin
// form (both reverse scans of the backward pass in one workgroup), gfx950.  Layout notes: la2_bf16_common.h.
#include "la2_bf16_common.h"

namespace la2 {
namespace {
using namespace bf16k;

// Blocks of 32 positions, one wave per 32 value features (D / 32 waves per scan: 4 for d = 128, 2 for d = 64),
// at most 256 registers and 80 KiB (d = 128) or 38 KiB (d = 64) of LDS, so that TWO (d = 128) or FOUR (d = 64)
// workgroups share a compute unit: two waves per SIMD.  One wave alone issues its
// instructions one after the other (an MFMA holds the issue port for about half its run time, a
// 16-byte-per-lane memory instruction for about 60 cycles), so a single wave per SIMD leaves the
// matrix pipe idle most of the time; a second, independent wave fills those gaps.  Used when a launch
// has enough workgroups to put two on every compute unit.  Same math as scan_bf16_kernel with a
// single (diagonal) 32 x 32 score tile per block; wave w owns value features 32 w .. 32 w + 31.
constexpr int kBH = 32;
//
// TWIN: both scans of a dual launch in ONE workgroup of two wave groups (d = 128: waves 0-3 scan 0, waves 4-7
// scan 1; d = 64: waves 0-1 and 2-3; again two waves per SIMD).  The dual launch is Algorithm 2's second loop, whose two scans read the
// same two tensors with the roles of Y and Z exchanged (dV: y = Q, z = dO; dK: y = dO, z = Q), so the
// workgroup streams FOUR tiles per block (x of scan 0, x of scan 1, Q, dO) instead of six and every
// tile is fetched exactly once.  Requires y[1] == z[0] and z[1] == y[0].
//
// NBUF tile buffers: block it + NBUF - 1 streams in while block it is computed.  With 3 buffers two
// (plain) workgroups fit on a compute unit.
//
// NORM: the Norm epilogue of eq. (2) on a forward scan: the four waves exchange the sums of squares of
// their quarter rows through LDS (under the block's one barrier, which moves behind the intra-block
// product for this), scale the finished tile and wave 0 stores r.  The LDS is full, so this variant has no
// staging buffer of its own: it stages each wave's output in the block's X tile, which is dead by then.
//
// ACC: a forward scan whose workgroup has a second group of waves (as many again; FOUR tiles per block: X, Y,
// Z and p.acc_y).  The first group runs the scan as usual; the second accumulates
// the reverse local state of the chunk for ANOTHER pair of scans, sum_c lambda^(c+1) acc_y_c^T x_c (c counted
// from the chunk's first position), and leave it in p.acc_states.  Algorithm 2: the dQ scan (x = dO) with
// acc_y = Q leaves the local dKV states of the sequence chunks, so the dK / dV scan needs no pass of its own
// over Q and dO to form them.
//
// RS: states at sequence ends that are not block boundaries (ScanParams::ragged_state; segments of a ragged length
// and packed batches with state hand-over, where every sequence has a length of its own).  Forward: when the chain's last block has rem < B
// rows and the final state is wanted, that block's update weighs row c by lambda^(rem-1-c) and the carried state
// by lambda^rem, which gives the state right after the last position.  Reverse: a start state that enters behind
// such a block reaches row r with lambda^(rem-1-r) and is carried on with lambda^rem.  A chain without positions
// hands its start state (or zero) to fin.  All of it is off the per-block path of a chain's other blocks.
template <typename E, int D, bool REV, bool TWIN, int NBUF, bool NORM = false, bool ACC = false, bool RS = false>
__global__ __launch_bounds__(((TWIN || ACC) ? 4 : 2) * D, ((TWIN || ACC) ? 1 : 2) * (128 / D))
void scan_bf16_half_kernel(ScanParams p) {
  static_assert(D == 128 || D == 64, "head_dim");
  static_assert(!NORM || (!REV && !TWIN), "the Norm epilogue belongs to the forward pass");
  static_assert(!ACC || (!REV && !TWIN && !NORM), "the accumulating wave group rides on a plain forward scan");
  static_assert(!RS || !ACC, "ragged-end states: forward scans (with or without the Norm epilogue) and reverse scans");
  constexpr int B = kBH;
  using C = Cfg<D, B>;
  constexpr int KS = C::KS, NT = C::NT, TILE = C::TILE, LW = C::LW;
  constexpr int SW = NT;                              // waves of one scan: one per tile of 32 value features
  constexpr int NW = (TWIN || ACC) ? 2 * SW : SW;     // waves
  constexpr int NTL = (TWIN || ACC) ? 4 : 3;          // tiles per block
  using Loader = TileLoader<D, NTL, B, NW>;
  __shared__ __attribute__((aligned(1024))) E sT[NBUF][NTL][TILE];
  // Output staging, 32 positions x 32 features per wave.  The NORM variant has no LDS left for it beside its
  // exchange buffer (two workgroups of 80 KiB per compute unit) and stages in the block's own X tile instead,
  // which is dead by then: see the epilogue.
  __shared__ __attribute__((aligned(16))) E sW[ACC ? SW : NW][NORM ? LW : 32 * LW];
  float* const sRed = NormExchange<NORM ? 2 * 32 * SW : 0>::get();   // [block parity][position][wave]
  // Cache policy of the output stores (buffer instruction bits: 2 = nt, 16 = sc1).  Measured: the twin
  // workgroup, a third of whose traffic is stores, runs 9-13 % faster with streaming write-through stores;
  // the plain kernel is 8 % slower with any non-temporal store policy and keeps the default.
  constexpr int kStorePolicy = TWIN ? 18 : 0;
  constexpr int NDMA = NTL * Loader::DMA_PER_WAVE;   // direct loads per wave and block
  constexpr int NST = 32 * 4 / 64 + (NORM ? 1 : 0);   // stores per lane and block: 16-byte output stores, r
  constexpr int DMA_PER_SLOT = (NDMA + KS - 1) / KS;   // direct loads issued in each slot of phase 1
  // vector-memory operations of this wave that are younger than the direct loads of block it + 1 when block
  // it waits for them: the loads of blocks it + 2 .. it + NBUF - 1 and as many blocks' stores
  constexpr int VM_YOUNGER = (NBUF - 2) * (NST + NDMA);
  static_assert(VM_YOUNGER < 64, "vmcnt is a 6-bit counter");
  constexpr int WAIT_NEXT_TILES = (VM_YOUNGER & 15) | ((VM_YOUNGER >> 4) << 14) | 0x0F70;

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int dvt = w % SW;
  int which = 0, wg = (int)blockIdx.x;
  const int group = __builtin_amdgcn_readfirstlane(w / SW);   // TWIN: which scan; ACC: scan waves or accumulating waves
  if (TWIN) {
    which = group;
  } else if (ACC) {
    // one scan only
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
  int bi, hi, chunk, slot_stride;
  int64_t slot;
  if (!place_workgroup(p, wg, bi, hi, chunk, slot, slot_stride)) return;
  const int chain = bi * p.heads + hi;
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

  const int nblocks = (n + B - 1) / B;
  const int cb = p.chunk_tokens / B;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);
  if (RS && n == 0 && chunk == 0) {   // no positions: the state passes through
    float* gf0 = which ? p.fin[1] : p.fin[0];
    if (gf0 != nullptr) {
      const float* gi0 = which ? p.init[1] : p.init[0];
      const bool tri = (p.init_transposed >> which) & 1, trf = (p.fin_transposed >> which) & 1;
      gf0 += (int64_t)chain * (D * D);
      if (gi0 != nullptr) gi0 += (int64_t)chain * (D * D);
#pragma unroll
      for (int t = 0; t < NT; t++)
#pragma unroll
        for (int v = 0; v < 16; v++)
          gf0[state_index<D>(dvt, l32, hh, t, v, trf)] = gi0 != nullptr ? gi0[state_index<D>(dvt, l32, hh, t, v, tri)] : 0.f;
    }
  }
  if (blk_lo >= blk_hi) return;
  const int nblk = blk_hi - blk_lo;

  // Start state: the chunk's start state or the caller's, or zero; with self_prefix (ScanParams) it is formed here.
  // Terms in scan order: the caller's start state, then the local states of the chunks passed before this one.
  // A term stored transposed goes through LDS with workgroup barriers, so the count is the same for every wave.
  const int nch = (nblocks + cb - 1) / cb;   // chunks this chain really has
  const bool any_tr = (p.state_transposed | p.init_transposed) != 0;
  const bool init_any = p.init[0] != nullptr || p.init[1] != nullptr;
  const bool sp = p.self_prefix != 0 && p.states != nullptr && slot >= 0;
  const int nterms = sp ? (init_any ? 1 : 0) + (REV ? nch - 1 - chunk : chunk) : 1;

  Loader loader(w, l, n, stride_n);
  if (ACC) {
    loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.x[0]) + base);
    loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.y[0]) + base);
    loader.g[2] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.z[0]) + base);
    loader.g[NTL - 1] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.acc_y) + base);
  } else if (TWIN) {
    loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.x[0]) + base);
    loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.x[1]) + base);
    loader.g[2] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.y[0]) + base);
    loader.g[NTL - 1] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.z[0]) + base);
  } else {
    loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(which ? p.x[1] : p.x[0]) + base);
    loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(which ? p.y[1] : p.y[0]) + base);
    loader.g[2] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(which ? p.z[1] : p.z[0]) + base);
  }
  // this wave's X, Y, Z among the tiles of a block
  constexpr int xi = TWIN ? WH : 0, yi = TWIN ? 2 + WH : 1, zi = TWIN ? 3 - WH : 2;
  const LaneAddr<D> la(l);

  if constexpr (ACC) {
    if (group == 1) {
      // ---- the accumulating waves: same loads, same barriers as the scan waves; per block only the state
      // update step, on (acc_y, X) with reverse weights.  The block processed it-th lies it blocks above the
      // chunk's first position: its contribution carries lambda^(B it) up front, the sum needs no running decay.
      constexpr int ACC_YOUNGER = (NBUF - 2) * NDMA;   // no stores in this wave group
      constexpr int ACC_WAIT = (ACC_YOUNGER & 15) | ((ACC_YOUNGER >> 4) << 14) | 0x0F70;
      // the scan waves may first stage transposed start states in the tile buffers (below): join their barriers
      // before the first tile load
      if (any_tr) {
#pragma unroll 1
        for (int k = 0; k < nterms * (NW / SW); k++) __syncthreads();
      }
      const UpdateDecay<true, B> adecay(l2, hh);
      f32x16 acc[NT];
#pragma unroll
      for (int t = 0; t < NT; t++) acc[t] = zero16();
#pragma unroll
      for (int j = 0; j < NBUF - 1; j++)
        if (j < nblk) loader.issue(sT[j], blk_lo + j);
      __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
#pragma unroll
      for (int j = 0; j < NBUF - 1; j++)
        if (j < nblk) loader.zero_tail(sT[j], blk_lo + j);
      __syncthreads();
      auto acc_step = [&](auto cur_tag, int it) __attribute__((always_inline)) -> bool {
        constexpr int cur = decltype(cur_tag)::value;
        const bool has_next = it + 1 < nblk, has_ahead = it + NBUF - 1 < nblk;
        uint32_t doff[Loader::DMA_PER_WAVE];
        loader.offsets(blk_lo + it + (NBUF - 1), has_ahead, doff);
#pragma unroll
        for (int j = 0; j < NDMA; j++) loader.issue_one(sT[(cur + NBUF - 1) % NBUF], doff, j);
        const E* tY = sT[cur][NTL - 1];
        const E* tZ = sT[cur][0];
        ex8<E> zf[2], yt[2][NT];
#pragma unroll
        for (int q = 0; q < 2; q++) {
          zf[q] = la.read_cols(tZ, 16 * q, dvt);
#pragma unroll
          for (int t = 0; t < NT; t++) yt[q][t] = la.read_cols(tY, 16 * q, t);
        }
        const float blk_decay = uniform(exp2f(l2 * (float)(B * it)));
#pragma unroll
        for (int q = 0; q < 2; q++) {
          const ex8<E> zd = adecay.apply(zf[q], 16 * q, blk_decay);
#pragma unroll
          for (int t = 0; t < NT; t++) acc[t] = mfma(yt[q][t], zd, acc[t]);
        }
        if (has_next) {
          __builtin_amdgcn_s_waitcnt(ACC_WAIT);
          loader.zero_tail(sT[(cur + 1) % NBUF], blk_lo + it + 1);
          lds_barrier();
        }
        return has_next;
      };
      for (int it = 0;; it += NBUF) {
        if (!acc_step(std::integral_constant<int, 0>{}, it)) break;
        if (!acc_step(std::integral_constant<int, 1>{}, it + 1)) break;
        if (!acc_step(std::integral_constant<int, 2 % NBUF>{}, it + 2)) break;
        if (NBUF > 3 && !acc_step(std::integral_constant<int, 3 % NBUF>{}, it + 3)) break;
        if (NBUF > 4 && !acc_step(std::integral_constant<int, 4 % NBUF>{}, it + 4)) break;
      }
      __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the dummy direct loads before the LDS is given up
      if (chunk != 0) {   // chunk 0 is the last one a reverse scan reaches: nobody starts from its local state
        float* gs = p.acc_states + slot * (D * D);   // a chain with a chunk 1 has state slots
#pragma unroll
        for (int t = 0; t < NT; t++)
#pragma unroll
          for (int v = 0; v < 16; v++) gs[state_index<D>(dvt, l32, hh, t, v, false)] = acc[t][v];
      }
      return;
    }
  }

  f32x16 kv[NT];
  bool have = false;   // a term is in (the next one is added to the decayed sum)
  {
    const float lam_full = exp2f(l2 * (float)p.chunk_tokens);
    const float lam_last = exp2f(l2 * (float)(n - (nch - 1) * p.chunk_tokens));
    float* const lds = reinterpret_cast<float*>(&sT[0][0][0]) + dvt * (32 * (D + 1));
    static_assert(sizeof(sT) >= (size_t)SW * 32 * (D + 1) * sizeof(float), "room for one wave group's slices");
    // Term k: where it lives, whether it is stored transposed, the decay the sum so far takes before it is added.
    auto term = [&](int k, const float*& gs, bool& tr, float& decay) __attribute__((always_inline)) {
      gs = nullptr;
      tr = false;
      decay = 0.f;
      if (!sp) {
        if (p.states != nullptr && slot >= 0) {
          gs = p.states + slot * (D * D);
          tr = (p.state_transposed >> which) & 1;
        } else if ((which ? p.init[1] : p.init[0]) != nullptr) {
          gs = (which ? p.init[1] : p.init[0]) + (int64_t)chain * (D * D);
          tr = (p.init_transposed >> which) & 1;
        }
      } else if (init_any && k == 0) {
        if ((which ? p.init[1] : p.init[0]) != nullptr) {
          gs = (which ? p.init[1] : p.init[0]) + (int64_t)chain * (D * D);
          tr = (p.init_transposed >> which) & 1;
        }
      } else {
        const int i = k - (init_any ? 1 : 0);
        const int j = REV ? nch - 1 - i : i;   // the chunk whose local state is added
        gs = p.states + (slot + (int64_t)(j - chunk) * slot_stride) * (D * D);
        tr = (p.state_transposed >> which) & 1;
        decay = j == nch - 1 ? lam_last : lam_full;
      }
    };
    // The global loads of the next terms are issued before term k is consumed (a term's loads take about a microsecond
    // and the launches that form their start states here are a few microseconds long).  A wave's slice of a term is
    // NT * 16 floats either way: its elements one by one, or (stored transposed) its 32 rows in 16-byte pieces.
    constexpr int NX = NT * 16;
    static_assert(32 * D / 256 * 4 == NX, "a wave's rows in 16-byte pieces per lane");
    constexpr int FA = D == 64 ? kMaxPrefixTerms - 1 : 1;   // terms fetched ahead (head_dim 128: 64 registers a term)
    float xb[FA + 1][NX];
    auto fetch = [&](int k, float (&x)[NX]) __attribute__((always_inline)) {
      const float* gs;
      bool tr;
      float decay;
      term(k, gs, tr, decay);
      if (gs == nullptr) return;
      if (!tr) {
#pragma unroll
        for (int t = 0; t < NT; t++)
#pragma unroll
          for (int v = 0; v < 16; v++) x[16 * t + v] = gs[state_index<D>(dvt, l32, hh, t, v, false)];
      } else {
        const float* rows = gs + (int64_t)(32 * dvt) * D;
#pragma unroll
        for (int i = 0; i < 32 * D / 256; i++) {
          const f32x4 r = *reinterpret_cast<const f32x4*>(rows + 4 * (64 * i + l));
          x[4 * i] = r[0]; x[4 * i + 1] = r[1]; x[4 * i + 2] = r[2]; x[4 * i + 3] = r[3];
        }
      }
    };
#pragma unroll
    for (int a = 0; a < FA; a++)
      if (a < nterms) fetch(a, xb[a]);
#pragma unroll
    for (int k = 0; k < kMaxPrefixTerms; k++) {
      if (k < nterms) {   // (the same for every wave of the workgroup)
        if (k + FA < nterms) fetch(k + FA, xb[(k + FA) % (FA + 1)]);
        const float(&x)[NX] = xb[k % (FA + 1)];
        const float* gs;
        bool tr;
        float decay;
        term(k, gs, tr, decay);
        if (gs != nullptr && !tr) {
#pragma unroll
          for (int t = 0; t < NT; t++)
#pragma unroll
            for (int v = 0; v < 16; v++) kv[t][v] = have ? fmaf(decay, kv[t][v], x[16 * t + v]) : x[16 * t + v];
        }
        // A state stored transposed: this wave's slice is then the 32 ROWS 32 dvt .. + 31 of the stored matrix, 32 D
        // consecutive floats.  Read element by element each lane would touch a cache line of its own (measured
        // +20 us per launch at 256 workgroups); instead the wave copies its rows with 16-byte loads through the tile
        // buffers, which nothing has used yet, and each lane picks its elements out of LDS (row stride D + 1 floats:
        // no bank conflicts).  One wave group at a time, a workgroup barrier after each: the first tile loads, from
        // any wave, overwrite that LDS.  Whether the launch has transposed states at all is uniform over the grid.
        if (any_tr) {
#pragma unroll 1
          for (int gsel = 0; gsel < NW / SW; gsel++) {
            if (gs != nullptr && tr && group == gsel) {
#pragma unroll
              for (int i = 0; i < 32 * D / 256; i++) {
                const int at = 4 * (64 * i + l);
                float* dst = lds + (at / D) * (D + 1) + at % D;
                dst[0] = x[4 * i]; dst[1] = x[4 * i + 1]; dst[2] = x[4 * i + 2]; dst[3] = x[4 * i + 3];
              }
              asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's own writes, before its own reads
#pragma unroll
              for (int t = 0; t < NT; t++)
#pragma unroll
                for (int v = 0; v < 16; v++) {
                  const float y = lds[l32 * (D + 1) + 32 * t + 8 * (v >> 2) + 4 * hh + (v & 3)];
                  kv[t][v] = have ? fmaf(decay, kv[t][v], y) : y;
                }
            }
            __syncthreads();
          }
        }
        if (gs != nullptr) have = true;
      }
    }
    if (!have) {
#pragma unroll
      for (int t = 0; t < NT; t++) kv[t] = zero16();
    }
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
  // RS: rows of the chain's ragged last block when this chunk holds it and its end state matters (forward: the
  // final state is wanted; reverse: a start state comes in behind it), else 0
  int rag_rem = 0;
  if (RS && blk_hi >= nblocks && n % B != 0) {
    if (REV ? have : (which ? p.fin[1] : p.fin[0]) != nullptr) rag_rem = n % B;
  }
  rag_rem = __builtin_amdgcn_readfirstlane(rag_rem);
  // The per-block code has no branch for that block.  The factors that differ there are variables which change
  // between two blocks: the carried state's decay, the weight of the carried part of a row (reverse) and the update
  // weights of the Z fragments (forward: kept in registers in this instantiation, element j of fragment q is row
  // c = 16 q + 4 hh + 8 (j / 4) + j % 4), switched at the top of the block step, outside its scheduled slots.
  float lam_var = lamB, isc_var = inter_scale;
  float wz[2][8];
  auto set_update_weights = [&](int rows) __attribute__((always_inline)) {   // rows valid in the block (B: a full one)
#pragma unroll
    for (int q = 0; q < 2; q++)
#pragma unroll
      for (int j = 0; j < 8; j++) {
        const int c = 16 * q + 4 * hh + 8 * (j >> 2) + (j & 3);
        wz[q][j] = c < rows ? fast_exp2(l2 * (float)(rows - 1 - c)) : 0.f;
      }
  };
  if constexpr (RS && !REV) set_update_weights(B);
  if constexpr (RS && REV) {
    if (rag_rem != 0) {   // the first block this scan meets: the start state sits right behind row rag_rem - 1
      lam_var = uniform(exp2f(l2 * (float)rag_rem));
      isc_var = l32 < rag_rem ? exp2f(l2 * (float)(rag_rem - 1 - l32)) : 0.f;
    }
  }

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
  ex8<E> xa[KS], ya[KS];     // X and Y row fragments (natural k-order) of the block being computed
#pragma unroll
  for (int ks = 0; ks < AHEAD; ks++) {
    xa[ks] = la.read_row(sT[0][xi], 0, ks);
    ya[ks] = la.read_row(sT[0][yi], 0, ks);
  }
  auto state_operand = [&](int ks) __attribute__((always_inline)) {
    ex8<E> f;
#pragma unroll
    for (int j = 0; j < 8; j++) f[j] = (E)kv[ks >> 1][8 * (ks & 1) + j];
    return to_perm_order(f);
  };
  ex8<E> sa_first = state_operand(0);
  E* const stage = sW[w];

#define LA2_SLOT_END()                 \
  do {                                 \
    asm volatile("" ::: "memory");     \
    __builtin_amdgcn_sched_barrier(0); \
  } while (0)
  // Phases as in scan_bf16_kernel (1 inter-block product and 2 scores, here interleaved; 3 state update;
  // barrier; 4 intra-block product), then the block's output.
  auto block_step = [&](auto cur_tag, int it) __attribute__((always_inline)) -> bool {
    constexpr int cur = decltype(cur_tag)::value;
    E (*const sCur)[TILE] = sT[cur];                          // block it
    E (*const sNext)[TILE] = sT[(cur + 1) % NBUF];            // block it + 1 (in flight or landed)
    E (*const sAhead)[TILE] = sT[(cur + NBUF - 1) % NBUF];    // block it + NBUF - 1 (free since block it - 1)
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    const bool has_next = it + 1 < nblk, has_ahead = it + NBUF - 1 < nblk;
    const int nb = REV ? blk - 1 : blk + 1;
    if constexpr (RS && !REV) {   // the ragged block is the last one a forward scan meets
      if (rag_rem != 0 && !has_next) {
        set_update_weights(rag_rem);
        lam_var = uniform(exp2f(l2 * (float)rag_rem));
      }
    }
    if constexpr (RS && REV) {    // ... and the first one of a reverse scan: back to a full block's factors
      if (rag_rem != 0 && it == 1) {
        lam_var = lamB;
        isc_var = inter_scale;
      }
    }
    const float lam_blk = RS ? lam_var : lamB;
    const E* tX = sCur[xi];
    const E* tY = sCur[yi];
    const E* tZ = sCur[zi];
    uint32_t doff[Loader::DMA_PER_WAVE];
    loader.offsets(REV ? blk - (NBUF - 1) : blk + (NBUF - 1), has_ahead, doff);

    ex8<E> zf[2], zd[2], yt[2][NT];
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
    ex8<E> sa = sa_first;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      inter = mfma(sa, xa[ks], inter);
      sd = mfma(ya[ks], xa[ks], sd);
      if (ks + AHEAD < KS) read_xy(ks + AHEAD);
      if (ks + 1 < KS) { sa = state_operand(ks + 1); pin(sa); }
#pragma unroll
      for (int u = 0; u < DMA_PER_SLOT; u++)
        if (ks * DMA_PER_SLOT + u < NDMA) loader.issue_one(sAhead, doff, ks * DMA_PER_SLOT + u);
      if (ks < 2) zf[ks] = la.read_cols(tZ, 16 * ks, dvt);
      if (ks >= 2 && (ks & 1) == 0) {   // state tile ks / 2 - 1: both operands made in slots <= ks - 1
        const int t = (ks >> 1) - 1;
#pragma unroll
        for (int v = 0; v < 16; v++) kv[t][v] *= lam_blk;
        pin(kv[t]);
      }
      // the update weights on the Z fragments, two slots after their LDS reads (d = 64: in the last two slots)
      if ((KS == 8 && (ks == 3 || ks == 5)) || (KS == 4 && (ks == 2 || ks == 3))) {
        const int q = KS == 8 ? (ks - 3) >> 1 : ks - 2;
        if constexpr (RS && !REV) {
#pragma unroll
          for (int j = 0; j < 8; j++) zd[q][j] = (E)((float)zf[q][j] * wz[q][j]);
        } else {
          zd[q] = decay.apply(zf[q], 16 * q);
        }
        pin(zd[q]);
      }
      if (ks == KS - 1) read_yt(0, 0);
      pin(inter);
      pin(sd);
      LA2_SLOT_END();
    }
    {
#pragma unroll
      for (int v = 0; v < 16; v++) kv[NT - 1][v] *= lam_blk;
      pin(kv[NT - 1]);
      // the carried part takes the decay at this lane's position
      const float isc = (RS && REV) ? isc_var : inter_scale;
#pragma unroll
      for (int v = 0; v < 16; v++) inter[v] *= isc;
      pin(inter);
    }
    // ---- phase 3
    ex8<E> pd[2];
    constexpr int NH = NT / 2;          // pairs of key-feature tiles
    constexpr int NS3 = 2 * NH;         // slots of this phase
    constexpr int PPS = 16 / NS3;       // elements of the masked score tile converted per slot
#pragma unroll
    for (int s4 = 0; s4 < NS3; s4++) {   // slot s4: k-step q = s4 / NH, key-feature tiles 2 h, 2 h + 1, h = s4 % NH
      const int q = s4 / NH, h = s4 % NH;
#pragma unroll
      for (int t = 2 * h; t < 2 * h + 2; t++) kv[t] = mfma(yt[q][t], zd[q], kv[t]);
      if (s4 + 1 < NS3) read_yt((s4 + 1) / NH, (s4 + 1) % NH);
#pragma unroll
      for (int e = 0; e < PPS; e++) {
        const int v = PPS * s4 + e;     // element v of the score tile belongs to the P fragment of k-step v / 8
        pd[v >> 3][v & 7] = (E)(sd[v] * dg[v]);
      }
      pin(pd[q]);
#pragma unroll
      for (int t = 2 * h; t < 2 * h + 2; t++) pin(kv[t]);
      LA2_SLOT_END();
    }
    // NORM: the block's one barrier comes after phase 4 instead, where it also publishes the rows' sums of squares
    if (has_next) {
      __builtin_amdgcn_s_waitcnt(WAIT_NEXT_TILES);
      loader.zero_tail(sNext, nb);
      if (!NORM) {
        lds_barrier();
#pragma unroll
        for (int ks = 0; ks < AHEAD; ks++) {
          xa[ks] = la.read_row(sNext[xi], 0, ks);
          ya[ks] = la.read_row(sNext[yi], 0, ks);
        }
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
    if constexpr (NORM) {
      // Two exchange buffers, by block parity: a wave that runs ahead into the next block must not
      // overwrite sums that a slower wave has yet to read.  The barrier is the block's only one: it also
      // makes the next block's tiles visible and frees this block's.
      float* const red = sRed + (it & 1) * (32 * SW);
      norm_publish<SW>(inter, red, l32, hh, dvt);
      lds_barrier();
      if (has_next) {
#pragma unroll
        for (int ks = 0; ks < AHEAD; ks++) {
          xa[ks] = la.read_row(sNext[xi], 0, ks);
          ya[ks] = la.read_row(sNext[yi], 0, ks);
        }
      }
      const float r = norm_collect<SW>(red, l32, 1.f / (float)D, p.eps);
#pragma unroll
      for (int v = 0; v < 16; v++) inter[v] *= r;
      pin(inter);
      // r of this block's positions: the lanes of wave 0 that hold them; every other lane's store is dropped
      const uint32_t roff = (dvt == 0 && hh == 0) ? (uint32_t)(blk * B + l32) * 4u : 0xFFFFFFF0u;
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(r), brs, roff, 0, 0);
    }
    // Staging area of this wave.  NORM: the quarter of this block's X tile that this wave's own direct loads
    // fill.  Every wave is past the block's last tile read (the barrier above), and the next writer of that
    // quarter is this wave's own direct load two blocks on, issued after the reads below have returned.
    E* const st = NORM ? const_cast<E*>(tX) + w * (TILE / SW) : stage;
#pragma unroll
    for (int g = 0; g < 4; g++) {
      ex4<E> pk;
#pragma unroll
      for (int e = 0; e < 4; e++) pk[e] = (E)inter[4 * g + e];
      *reinterpret_cast<ex4<E>*>(st + l32 * LW + 8 * (g ^ ((l32 >> 2) & 3)) + 4 * hh) = pk;
    }
#pragma unroll
    for (int i = 0; i < 32 * 4 / 64; i++) {
      const int id = l + 64 * i;
      const int row = id >> 2, cc = id & 3;
      const i32x4 v = *reinterpret_cast<const i32x4*>(st + row * LW + 8 * (cc ^ ((row >> 2) & 3)));
      const uint32_t off = ((uint32_t)(blk * B + row) * stride_n + (uint32_t)(32 * dvt + cc * 8)) * 2u;
      __builtin_amdgcn_raw_buffer_store_b128(v, bw, off, 0, kStorePolicy);
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
  if (gf != nullptr && (REV ? chunk == 0 : blk_hi >= nblocks)) {   // the chunk this chain's scan passes last
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

}  // namespace

namespace {
template <typename E, int D>
hipError_t launch_half(bool reverse, bool twin, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (p.wg_map != nullptr ? (int64_t)p.wg_pairs * p.heads : (int64_t)p.batch * p.heads * p.nchunks) * p.nscan;
  // Three tile buffers in every case.  More buffers (5 for a plain, 4 for a twin workgroup that has the
  // compute unit to itself) measured no faster: such launches are bound by the memory system, not by the
  // bytes a workgroup keeps in flight.
  constexpr int kPlain = 2 * D, kDouble = 4 * D;   // threads: one wave per 32 value features, or two such groups
  if (p.ragged_state != 0) {   // the host pairs this only with a reverse twin launch or a forward scan without ACC
    if (twin && reverse)
      hipLaunchKernelGGL((scan_bf16_half_kernel<E, D, true, true, 3, false, false, true>), dim3((unsigned)(grid / 2)),
                         dim3(kDouble), 0, s, p);
    else if (!twin && !reverse && p.acc_states == nullptr && p.rstd == nullptr)
      hipLaunchKernelGGL((scan_bf16_half_kernel<E, D, false, false, 3, false, false, true>), dim3((unsigned)grid),
                         dim3(kPlain), 0, s, p);
    else if (!twin && !reverse && p.acc_states == nullptr)
      hipLaunchKernelGGL((scan_bf16_half_kernel<E, D, false, false, 3, true, false, true>), dim3((unsigned)grid),
                         dim3(kPlain), 0, s, p);
    else
      return hipErrorInvalidValue;
  } else if (twin) {
    dim3 gt((unsigned)(grid / 2)), bt(kDouble);
    if (reverse) hipLaunchKernelGGL((scan_bf16_half_kernel<E, D, true, true, 3>), gt, bt, 0, s, p);
    else         hipLaunchKernelGGL((scan_bf16_half_kernel<E, D, false, true, 3>), gt, bt, 0, s, p);
  } else {
    dim3 g((unsigned)grid), b(kPlain);
    if (reverse) hipLaunchKernelGGL((scan_bf16_half_kernel<E, D, true, false, 3>), g, b, 0, s, p);
    else if (p.acc_states != nullptr)
      hipLaunchKernelGGL((scan_bf16_half_kernel<E, D, false, false, 3, false, true>), g, dim3(kDouble), 0, s, p);
    else if (p.rstd != nullptr) hipLaunchKernelGGL((scan_bf16_half_kernel<E, D, false, false, 3, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((scan_bf16_half_kernel<E, D, false, false, 3>), g, b, 0, s, p);
  }
  return hipGetLastError();
}
}  // namespace

hipError_t launch_scan_bf16_half(int dtype, int head_dim, bool reverse, bool twin, const ScanParams& p, hipStream_t s) {
  if (head_dim == 64)
    return dtype == kF16 ? launch_half<_Float16, 64>(reverse, twin, p, s) : launch_half<__bf16, 64>(reverse, twin, p, s);
  return dtype == kF16 ? launch_half<_Float16, 128>(reverse, twin, p, s) : launch_half<__bf16, 128>(reverse, twin, p, s);
}

}  // namespace la2
