// Chunk-state pre-pass of the sequence-chunked launches, gfx950: local state of every chunk (bf16 MFMA, same
// streaming as the scan kernels) and the scan that turns local states into chunk start states (fp32).
#include <algorithm>

#include "la2_bf16_common.h"

namespace la2 {
namespace {
using namespace bf16k;

// Local state of every chunk that has a successor: forward sum_c lambda^(C-1-c) y_c^T z_c over the
// chunk's positions c, reverse sum_c lambda^c y_c^T z_c.  Written fp32 row-major [dk][dv].  Same
// streaming and the same state-update step as the scan kernel, without X, scores or outputs.
//
// A launch has about one workgroup per compute unit (it exists because the chains alone cannot fill the
// device) and hardly any arithmetic, so its speed is the bytes a workgroup keeps in flight: NBUF tile
// buffers, the tiles of block it + NBUF - 1 stream in while block it is used.  Every block's loads are
// issued unconditionally (past the chunk's end as dummy loads of one cache line), so the count of
// outstanding loads is the same in every iteration and one s_waitcnt immediate serves.
// Two waves per SIMD: 2 NT waves (8 at d = 128, 4 at d = 64); wave w owns value features 32 (w % NT) .. + 31 and
// the key-feature tiles of half w / NT of the state slice, so that one wave's LDS and MFMA latencies hide behind
// the other's instructions (a wave issues one instruction at a time).
template <typename E, int D, bool REV, int NBUF>
__global__ __launch_bounds__(128 * (D / 32), 1) void chunk_state_bf16_kernel(ScanParams p) {
  static_assert(NBUF >= 3 && NBUF <= 5, "the block loop below is unrolled for 3 to 5 buffers");
  using C = Cfg<D>;
  constexpr int NT = C::NT, TILE = C::TILE;
  constexpr int KT = NT / 2;   // key-feature tiles per wave
  using Loader = TileLoader<D, 2, kB, 2 * NT>;
  __shared__ __attribute__((aligned(1024))) E sT[NBUF][2][TILE];   // [Y, Z]
  constexpr int NDMA = 2 * Loader::DMA_PER_WAVE;   // direct loads per wave and block
  constexpr int VM_YOUNGER = (NBUF - 2) * NDMA;    // loads younger than those of block it + 1 when it waits for them
  static_assert(VM_YOUNGER < 64, "vmcnt is a 6-bit counter");
  constexpr int WAIT_NEXT_TILES = (VM_YOUNGER & 15) | ((VM_YOUNGER >> 4) << 14) | 0x0F70;

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int dvt = w % NT, kt0 = (w / NT) * KT;
  int bi, hi, chunk, slot_stride;
  int64_t slot;
  if (!place_workgroup(p, (int)blockIdx.x, bi, hi, chunk, slot, slot_stride)) return;
  int64_t base;
  int n;
  chain_extent(p, bi, hi, base, n);
  const float l2 = log2f(p.lambda[hi]);
  const int nblocks = (n + kB - 1) / kB;
  const int cb = p.chunk_tokens / kB;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);
  const int nblk = blk_hi - blk_lo;
  // the chunk a scan of THIS chain passes last has no successor (a packed batch: chains of different lengths)
  if (REV ? (chunk == 0) : (blk_hi >= nblocks)) return;

  Loader loader(w, l, n, (uint32_t)p.stride_n);
  loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.y[0]) + base);
  loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.z[0]) + base);
  const LaneAddr<D> la(l);
  const UpdateDecay<REV> decay(l2, hh);
  f32x16 kv[KT];
#pragma unroll
  for (int t = 0; t < KT; t++) kv[t] = zero16();

  // loads of the chunk's block number `it` (real, or dummy when the chunk has no such block) into `buf`
  auto issue_block = [&](E (*buf)[TILE], int it) __attribute__((always_inline)) {
    uint32_t doff[Loader::DMA_PER_WAVE];
    loader.offsets(REV ? blk_hi - 1 - it : blk_lo + it, it < nblk, doff);
#pragma unroll
    for (int j = 0; j < NDMA; j++) loader.issue_one(buf, doff, j);
  };
  if (nblk <= 0) return;
#pragma unroll
  for (int j = 0; j < NBUF - 1; j++) issue_block(sT[j], j);
  __builtin_amdgcn_s_waitcnt(WAIT_NEXT_TILES);   // the first block's tiles
  loader.zero_tail(sT[0], REV ? blk_hi - 1 : blk_lo);
  lds_barrier();

  auto block_step = [&](auto cur_tag, int it) __attribute__((always_inline)) -> bool {
    constexpr int cur = decltype(cur_tag)::value;
    const bool has_next = it + 1 < nblk;
    const int nb = REV ? blk_hi - 2 - it : blk_lo + it + 1;
    issue_block(sT[(cur + NBUF - 1) % NBUF], it + NBUF - 1);   // that buffer was block it - 1's
    const E* tY = sT[cur][0];
    const E* tZ = sT[cur][1];
    ex8<E> zf[4], yt[KT][4];   // [16-row k-step of the block]
#pragma unroll
    for (int k = 0; k < 4; k++) {
      zf[k] = la.read_cols(tZ, 16 * k, dvt);
#pragma unroll
      for (int t = 0; t < KT; t++) yt[t][k] = la.read_cols(tY, 16 * k, kt0 + t);
    }
    __builtin_amdgcn_sched_barrier(0);
    // Only the state after the chunk's last block is wanted, so instead of decaying the running sum by
    // lambda^B per block, each block's contribution carries its whole decay up front: the block processed
    // `it`-th has nblk - 1 - it blocks after it (forward: later positions; reverse: earlier ones), which
    // saves a quarter of the loop's vector instructions.  Exponents are non-negative: no overflow, and what
    // underflows is what the running decay would have wiped out as well.
    const float blk_decay = uniform(exp2f(l2 * (float)(kB * (nblk - 1 - it))));
#pragma unroll
    for (int k = 0; k < 4; k++) {
      const ex8<E> zd = decay.apply(zf[k], 16 * k, blk_decay);
#pragma unroll
      for (int t = 0; t < KT; t++) kv[t] = mfma(yt[t][k], zd, kv[t]);
    }
    if (has_next) {
      __builtin_amdgcn_s_waitcnt(WAIT_NEXT_TILES);
      loader.zero_tail(sT[(cur + 1) % NBUF], nb);
      lds_barrier();   // next tiles visible to all waves; this block's buffer free
    }
    return has_next;
  };
  for (int it = 0;; it += NBUF) {   // unrolled by the number of buffers: compile-time buffer index
    if (!block_step(std::integral_constant<int, 0>{}, it)) break;
    if (!block_step(std::integral_constant<int, 1>{}, it + 1)) break;
    if (!block_step(std::integral_constant<int, 2 % NBUF>{}, it + 2)) break;
    if (NBUF > 3 && !block_step(std::integral_constant<int, 3 % NBUF>{}, it + 3)) break;
    if (NBUF > 4 && !block_step(std::integral_constant<int, 4 % NBUF>{}, it + 4)) break;
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the dummy loads before the LDS is given up

  float* gs = p.states + slot * (D * D);   // a chunk with a successor: its chain has state slots
#pragma unroll
  for (int t = 0; t < KT; t++)
#pragma unroll
    for (int v = 0; v < 16; v++) gs[state_index<D>(dvt, l32, hh, kt0 + t, v, false)] = kv[t][v];
}

// In place: states[chain][j] (local state of chunk j) -> start state of chunk j.
//   forward: G_0 = 0, G_{j+1} = lambda^C G_j + L_j        reverse: G_last = 0, G_{j-1} = lambda^C G_j + L_j
// The chunk processed first starts from init (element e read at its transposed place if init_tr) or 0.
// The carried state decays by lambda^(chunk length): all chunks are chunk_tokens long except the last
// one of the sequence, which a reverse scan passes first.
// A thread owns four consecutive elements of the d x d state.  With up to MAXC chunks it fetches all local
// states first (independent loads, all in flight together) and then runs the recurrence on registers; the
// launch sits between two kernels that wait for it, so its latency is what counts, not its bytes.
constexpr int kScanMaxChunks = 32;
// wg_map != nullptr (packed batch with a compact grid, see ScanParams): a "unit" is a sequence of long_list and a
// head; the chain's states are `heads` slots apart.
__global__ void state_scan_kernel(float* states, const float* lambda, int heads, int nchunks, int chunk_tokens,
                                  int dd, int reverse, const float* init, int init_tr, int d, int n,
                                  const int32_t* cu_seqlens, const int4* wg_map, const int32_t* long_list) {
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  const int dd4 = dd >> 2;
  const int per_chain = (dd4 + (int)blockDim.x - 1) / (int)blockDim.x;   // workgroups per chain
  const int unit = (int)(blockIdx.x / per_chain);
  const int e4 = (int)(blockIdx.x % per_chain) * (int)blockDim.x + (int)threadIdx.x;
  if (e4 >= dd4) return;
  int bi, hi;
  int64_t first_slot, stride;   // the chain's chunk-0 state slot, slots between its consecutive chunks
  if (wg_map != nullptr) {
    const int pair = long_list[unit / heads];
    if (pair < 0) return;
    const int4 m = wg_map[pair];
    bi = m.x;
    hi = unit % heads;
    first_slot = (int64_t)m.z * heads + hi;
    stride = heads;
  } else {
    bi = unit / heads;
    hi = unit % heads;
    first_slot = (int64_t)unit * nchunks;
    stride = 1;
  }
  const int chain = bi * heads + hi;
  if (cu_seqlens != nullptr) n = cu_seqlens[bi + 1] - cu_seqlens[bi];   // this sequence's length
  int nch = (n + chunk_tokens - 1) / chunk_tokens;   // chunks this chain really has (<= nchunks)
  // (a packed sequence longer than the launch was planned for is the caller's error; it must not reach past the
  // chain's slots.  With a pair map the sequence's slots were counted from this same length.)
  if (wg_map == nullptr) nch = min(nch, nchunks);
  const float l2 = log2f(lambda[hi]);
  const float lamFull = exp2f(l2 * (float)chunk_tokens);
  const float lamLast = exp2f(l2 * (float)(n - (nch - 1) * chunk_tokens));
  f32x4* s = reinterpret_cast<f32x4*>(states + first_slot * dd) + e4;
  const int64_t step = stride * dd4;   // f32x4 elements between consecutive chunks' states
  f32x4 g = {0.f, 0.f, 0.f, 0.f};
  if (init != nullptr) {
    const float* gi = init + (int64_t)chain * dd;
    const int e = 4 * e4;   // d is a multiple of 4: the four elements share a row
    if (init_tr) {
#pragma unroll
      for (int i = 0; i < 4; i++) g[i] = gi[((e + i) % d) * d + e / d];
    } else {
      g = *reinterpret_cast<const f32x4*>(gi + e);
    }
  }
  if (nch <= kScanMaxChunks) {
    f32x4 loc[kScanMaxChunks];
#pragma unroll
    for (int i = 0; i < kScanMaxChunks; i++) {
      const int j = reverse ? nch - 1 - i : i;
      if (i < nch - 1) loc[i] = s[(int64_t)j * step];   // the chunk processed last has no successor: not read
    }
#pragma unroll
    for (int i = 0; i < kScanMaxChunks; i++) {
      if (i < nch) {
        const int j = reverse ? nch - 1 - i : i;
        s[(int64_t)j * step] = g;
        const float decay = (j == nch - 1) ? lamLast : lamFull;
        if (i < nch - 1) g = decay * g + loc[i];
      }
    }
    return;
  }
  for (int i = 0; i < nch; i++) {
    const int j = reverse ? nch - 1 - i : i;
    const bool last = (i == nch - 1);
    f32x4 loc = {0.f, 0.f, 0.f, 0.f};
    if (!last) loc = s[(int64_t)j * step];
    s[(int64_t)j * step] = g;
    g = (j == nch - 1 ? lamLast : lamFull) * g + loc;
  }
}

// Packed batch in sequence chunks: the (sequence, chunk) pairs in order, for the compact launch grid.  One
// workgroup walks the sequences 256 at a time with a running count of pairs and of state slots.
//   map[pair] = {sequence, chunk, first state slot of the sequence (-1: single chunk, no slots), its chunk count}
// Entries past the last pair, up to npairs, get sequence -1.  A batch whose lengths sum to more than the host was
// told would need more entries than the map has, or more state slots than the workspace (nslots per head): such
// pairs are dropped (nothing is written past the end of either; their sequences are not computed).
// long_list[i] = pair of chunk 0 of the i-th sequence with state slots (i < nlong), -1 past the last.
__global__ __launch_bounds__(256) void varlen_map_kernel(const int32_t* cu_seqlens, int batch, int chunk_tokens, int npairs,
                                                         int4* map, int nlong, int32_t* long_list, int nslots) {
  __shared__ int s_pairs[256], s_slots[256], s_long[256];
  __shared__ int base_pairs, base_slots, base_long;
  const int t = (int)threadIdx.x;
  if (t == 0) { base_pairs = 0; base_slots = 0; base_long = 0; }
  __syncthreads();
  for (int b0 = 0; b0 < batch; b0 += 256) {
    const int b = b0 + t;
    int nch = 0;
    // (a sequence without positions keeps one pair: its workgroups pass a start state on where one is handed over)
    if (b < batch) nch = max(1, (cu_seqlens[b + 1] - cu_seqlens[b] + chunk_tokens - 1) / chunk_tokens);
    const int slots = nch > 1 ? nch : 0;
    s_pairs[t] = nch;
    s_slots[t] = slots;
    s_long[t] = slots ? 1 : 0;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {   // inclusive scan of the three counts
      const int ap = t >= off ? s_pairs[t - off] : 0, as = t >= off ? s_slots[t - off] : 0,
                al = t >= off ? s_long[t - off] : 0;
      __syncthreads();
      s_pairs[t] += ap;
      s_slots[t] += as;
      s_long[t] += al;
      __syncthreads();
    }
    const int first_pair = base_pairs + s_pairs[t] - nch;
    const int first_slot = base_slots + s_slots[t] - slots;
    const bool fits = first_pair + nch <= npairs && (!slots || first_slot + slots <= nslots);
    for (int j = 0; j < nch; j++)
      if (first_pair + j < npairs) map[first_pair + j] = make_int4(fits ? b : -1, j, slots ? first_slot : -1, nch);
    if (slots && base_long + s_long[t] - 1 < nlong) long_list[base_long + s_long[t] - 1] = fits ? first_pair : -1;
    __syncthreads();
    if (t == 255) { base_pairs += s_pairs[255]; base_slots += s_slots[255]; base_long += s_long[255]; }
    __syncthreads();
  }
  for (int i = base_pairs + t; i < npairs; i += 256) map[i] = make_int4(-1, 0, -1, 0);
  for (int i = base_long + t; i < nlong; i += 256) long_list[i] = -1;
}

}  // namespace

namespace {
template <typename E>
hipError_t launch_chunk_states(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t grid = p.wg_map != nullptr ? (int64_t)p.wg_pairs * p.heads : (int64_t)p.batch * p.heads * p.nchunks;
  dim3 g((unsigned)grid);
  if (head_dim == 128) {
    if (reverse) hipLaunchKernelGGL((chunk_state_bf16_kernel<E, 128, true, 4>), g, dim3(512), 0, s, p);
    else         hipLaunchKernelGGL((chunk_state_bf16_kernel<E, 128, false, 4>), g, dim3(512), 0, s, p);
  } else {
    if (reverse) hipLaunchKernelGGL((chunk_state_bf16_kernel<E, 64, true, 4>), g, dim3(256), 0, s, p);
    else         hipLaunchKernelGGL((chunk_state_bf16_kernel<E, 64, false, 4>), g, dim3(256), 0, s, p);
  }
  return hipGetLastError();
}
}  // namespace

hipError_t launch_chunk_states_bf16(int dtype, int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (int64_t)p.batch * p.heads * p.nchunks;
  if (grid == 0 || p.n == 0) return hipSuccess;
  return dtype == kF16 ? launch_chunk_states<_Float16>(head_dim, reverse, p, s)
                       : launch_chunk_states<__bf16>(head_dim, reverse, p, s);
}

hipError_t launch_state_scan(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t units = p.wg_map != nullptr ? (int64_t)p.nlong * p.heads : (int64_t)p.batch * p.heads;
  if (units == 0 || p.n == 0) return hipSuccess;
  const int dd = head_dim * head_dim;
  dim3 g((unsigned)(units * ((dd / 4 + 255) / 256))), b(256);   // the host checked that this fits a grid
  hipLaunchKernelGGL(state_scan_kernel, g, b, 0, s, p.states, p.lambda, p.heads, p.nchunks, p.chunk_tokens, dd,
                     reverse ? 1 : 0, p.init[0], p.init_transposed & 1, head_dim, p.n, p.cu_seqlens, p.wg_map, p.long_list);
  return hipGetLastError();
}

hipError_t launch_varlen_map(const ScanParams& p, int4* map, int32_t* long_list, int64_t nslots, hipStream_t s) {
  if (p.wg_pairs <= 0) return hipSuccess;
  hipLaunchKernelGGL(varlen_map_kernel, dim3(1), dim3(256), 0, s, p.cu_seqlens, p.batch, p.chunk_tokens, p.wg_pairs, map,
                     p.nlong, long_list, (int)std::min<int64_t>(nslots, 0x7FFFFFFF));
  return hipGetLastError();
}

}  // namespace la2
