// Chunk-state pre-pass of the sequence-chunked launches, gfx950: local state of every chunk (bf16 MFMA, same
// streaming as the scan kernels) and the scan that turns local states into chunk start states (fp32).
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
template <typename E, int D, bool REV, int NBUF>
__global__ __launch_bounds__(kThreads, 1) void chunk_state_bf16_kernel(ScanParams p) {
  static_assert(NBUF >= 3 && NBUF <= 5, "the block loop below is unrolled for 3 to 5 buffers");
  using C = Cfg<D>;
  constexpr int NT = C::NT, TILE = C::TILE;
  using Loader = TileLoader<D, 2>;
  __shared__ __attribute__((aligned(1024))) E sT[NBUF][2][TILE];   // [Y, Z]
  constexpr int NDMA = 2 * Loader::DMA_PER_WAVE;   // direct loads per wave and block
  constexpr int VM_YOUNGER = (NBUF - 2) * NDMA;    // loads younger than those of block it + 1 when it waits for them
  static_assert(VM_YOUNGER < 64, "vmcnt is a 6-bit counter");
  constexpr int WAIT_NEXT_TILES = (VM_YOUNGER & 15) | ((VM_YOUNGER >> 4) << 14) | 0x0F70;

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
  const int dvt = w % NT;
  const int chain = blockIdx.x / p.nchunks, chunk = blockIdx.x % p.nchunks;
  if (REV ? (chunk == 0) : (chunk == p.nchunks - 1)) return;  // no successor needs it
  const int bi = chain / p.heads, hi = chain % p.heads;
  int64_t base;
  int n;
  chain_extent(p, bi, hi, base, n);
  const float l2 = log2f(p.lambda[hi]);
  const int nblocks = (n + kB - 1) / kB;
  const int cb = p.chunk_tokens / kB;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);
  const int nblk = blk_hi - blk_lo;

  Loader loader(w, l, n, (uint32_t)p.stride_n);
  loader.g[0] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.y[0]) + base);
  loader.g[1] = reinterpret_cast<const char*>(reinterpret_cast<const E*>(p.z[0]) + base);
  const LaneAddr<D> la(l);
  const UpdateDecay<REV> decay(l2, hh);
  f32x16 kv[NT];
#pragma unroll
  for (int t = 0; t < NT; t++) kv[t] = zero16();

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
    ex8<E> zf[4], yt[NT][4];   // [16-row k-step of the block]
#pragma unroll
    for (int k = 0; k < 4; k++) {
      zf[k] = la.read_cols(tZ, 16 * k, dvt);
#pragma unroll
      for (int t = 0; t < NT; t++) yt[t][k] = la.read_cols(tY, 16 * k, t);
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
      for (int t = 0; t < NT; t++) kv[t] = mfma(yt[t][k], zd, kv[t]);
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

  if (w < NT) {   // for d = 64 waves w and w + 2 hold the same slice
    float* gs = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) gs[state_index<D>(dvt, l32, hh, t, v, false)] = kv[t][v];
  }
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
__global__ void state_scan_kernel(float* states, const float* lambda, int heads, int nchunks, int chunk_tokens,
                                  int dd, int reverse, const float* init, int init_tr, int d, int n,
                                  const int32_t* cu_seqlens) {
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  const int dd4 = dd >> 2;
  const int per_chain = (dd4 + (int)blockDim.x - 1) / (int)blockDim.x;   // workgroups per chain
  const int chain = (int)(blockIdx.x / per_chain);
  const int e4 = (int)(blockIdx.x % per_chain) * (int)blockDim.x + (int)threadIdx.x;
  if (e4 >= dd4) return;
  if (cu_seqlens != nullptr) n = cu_seqlens[chain / heads + 1] - cu_seqlens[chain / heads];   // this sequence's length
  const int nch = (n + chunk_tokens - 1) / chunk_tokens;   // chunks this chain really has (<= nchunks)
  const float l2 = log2f(lambda[chain % heads]);
  const float lamFull = exp2f(l2 * (float)chunk_tokens);
  const float lamLast = exp2f(l2 * (float)(n - (nch - 1) * chunk_tokens));
  f32x4* s = reinterpret_cast<f32x4*>(states + (int64_t)chain * nchunks * dd) + e4;
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
      if (i < nch - 1) loc[i] = s[(int64_t)j * dd4];   // the chunk processed last has no successor: not read
    }
#pragma unroll
    for (int i = 0; i < kScanMaxChunks; i++) {
      if (i < nch) {
        const int j = reverse ? nch - 1 - i : i;
        s[(int64_t)j * dd4] = g;
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
    if (!last) loc = s[(int64_t)j * dd4];
    s[(int64_t)j * dd4] = g;
    g = (j == nch - 1 ? lamLast : lamFull) * g + loc;
  }
}

}  // namespace

namespace {
template <typename E>
hipError_t launch_chunk_states(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (int64_t)p.batch * p.heads * p.nchunks;
  dim3 g((unsigned)grid), b(kThreads);
  if (head_dim == 128) {
    if (reverse) hipLaunchKernelGGL((chunk_state_bf16_kernel<E, 128, true, 4>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((chunk_state_bf16_kernel<E, 128, false, 4>), g, b, 0, s, p);
  } else {
    if (reverse) hipLaunchKernelGGL((chunk_state_bf16_kernel<E, 64, true, 4>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((chunk_state_bf16_kernel<E, 64, false, 4>), g, b, 0, s, p);
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
  const int chains = p.batch * p.heads;
  if (chains == 0 || p.n == 0) return hipSuccess;
  const int dd = head_dim * head_dim;
  dim3 g((unsigned)((int64_t)chains * ((dd / 4 + 255) / 256))), b(256);   // the host checked that this fits a grid
  hipLaunchKernelGGL(state_scan_kernel, g, b, 0, s, p.states, p.lambda, p.heads, p.nchunks, p.chunk_tokens, dd,
                     reverse ? 1 : 0, p.init[0], p.init_transposed & 1, head_dim, p.n, p.cu_seqlens);
  return hipGetLastError();
}

}  // namespace la2
