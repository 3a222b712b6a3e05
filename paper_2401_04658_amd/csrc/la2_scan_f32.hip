// fp32 kernels for the decayed causal scan (Algorithm 1; both loops of Algorithm 2), gfx950.
//
// fp32 storage and fp32 FMA arithmetic throughout (no matrix cores, no reduced precision), for
// callers that need the 1e-5 accuracy class.  One workgroup walks the blocks of one sequence chunk
// of one (batch, head) chain with the X, Y, Z tiles, the masked score tile P and the running d x d
// state all in LDS.  Per block: P = (X Y^T) * M, W = P Z + diag(decay) X S, S <- lambda^B S +
// (decay(Y))^T Z -- the three steps of Algorithm 1 in order.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "la2_internal.h"

namespace la2 {
namespace {

constexpr int kThreads = 256;

template <int D>
struct F32Cfg {
  static constexpr int B = (D == 64) ? 64 : 32;  // block size: everything must fit 160 KiB of LDS
  static constexpr int LD = D + 1;               // odd row stride: conflict-free column walks
  static constexpr int LP = B + 1;
};

template <int D>
__device__ __forceinline__ void load_tile(float* s, const float* g, int64_t stride_n, int row0, int n, int tid) {
  constexpr int B = F32Cfg<D>::B, LD = F32Cfg<D>::LD;
  for (int idx = tid; idx < B * D; idx += kThreads) {
    const int row = idx / D, col = idx % D;
    const int pos = row0 + row;
    s[row * LD + col] = (pos < n) ? g[(int64_t)pos * stride_n + col] : 0.f;
  }
}

// S[k][j] <- lambda^B S[k][j] + sum_c decay_c Y[c][k] Z[c][j]; forward decay_c = lambda^(B-1-c),
// reverse lambda^(c+1).  sDec holds decay_c.
template <int D>
__device__ __forceinline__ void state_update(float* sS, const float* sY, const float* sZ, const float* sDec,
                                             float lamB, int tid) {
  constexpr int B = F32Cfg<D>::B, LD = F32Cfg<D>::LD;
  for (int idx = tid; idx < D * D; idx += kThreads) {
    const int k = idx / D, j = idx % D;
    float acc = lamB * sS[k * LD + j];
    for (int c = 0; c < B; c++) acc = fmaf(sDec[c] * sY[c * LD + k], sZ[c * LD + j], acc);
    sS[k * LD + j] = acc;
  }
}

template <int D, bool REV>
__global__ __launch_bounds__(kThreads) void scan_f32_kernel(ScanParams p) {
  using C = F32Cfg<D>;
  constexpr int B = C::B, LD = C::LD, LP = C::LP;
  __shared__ float sX[B * LD], sY[B * LD], sZ[B * LD], sP[B * LP], sS[D * LD], sDec[B], sInter[B];

  const int tid = threadIdx.x;
  const int chain = blockIdx.x / p.nchunks, chunk = blockIdx.x % p.nchunks;
  const int bi = chain / p.heads, hi = chain % p.heads;
  const int64_t base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h;
  const float* gx = reinterpret_cast<const float*>(p.x[0]) + base;
  const float* gy = reinterpret_cast<const float*>(p.y[0]) + base;
  const float* gz = reinterpret_cast<const float*>(p.z[0]) + base;
  float* gw = reinterpret_cast<float*>(p.w[0]) + base;
  const int n = p.n;
  const float l2 = log2f(p.lambda[hi]);
  const float lamB = exp2f(l2 * (float)B);

  const int nblocks = (n + B - 1) / B;
  const int cb = p.chunk_tokens / B;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);
  if (blk_lo >= blk_hi) return;

  // start state: chunk start state, the caller's start state (possibly stored transposed), or zero
  const float* gs = p.states ? p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D) : nullptr;
  bool tr = p.states != nullptr && (p.state_transposed & 1);
  if (gs == nullptr && p.init[0] != nullptr) {
    gs = p.init[0] + (int64_t)chain * (D * D);
    tr = p.init_transposed & 1;
  }
  for (int idx = tid; idx < D * D; idx += kThreads)
    sS[(idx / D) * LD + idx % D] = gs ? gs[tr ? (idx % D) * D + idx / D : idx] : 0.f;
  if (tid < B) {
    sDec[tid] = exp2f(l2 * (float)(REV ? tid + 1 : B - 1 - tid));      // weight of row c in the state update
    sInter[tid] = exp2f(l2 * (float)(REV ? B - 1 - tid : tid + 1));    // weight of the carried state for row r
  }
  float* gf = (p.fin[0] != nullptr && (REV ? chunk == 0 : chunk == p.nchunks - 1)) ? p.fin[0] + (int64_t)chain * (D * D)
                                                                                   : nullptr;

  const int nblk = blk_hi - blk_lo;
  for (int it = 0; it < nblk; it++) {
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    __syncthreads();
    load_tile<D>(sX, gx, p.stride_n, blk * B, n, tid);
    load_tile<D>(sY, gy, p.stride_n, blk * B, n, tid);
    load_tile<D>(sZ, gz, p.stride_n, blk * B, n, tid);
    __syncthreads();
    // masked scores: forward lambda^(r-c) for r >= c, reverse lambda^(c-r) for c >= r
    for (int idx = tid; idx < B * B; idx += kThreads) {
      const int r = idx / B, c = idx % B;
      const int e = REV ? c - r : r - c;
      float s = 0.f;
      if (e >= 0) {
        for (int k = 0; k < D; k++) s = fmaf(sX[r * LD + k], sY[c * LD + k], s);
        s *= exp2f(l2 * (float)e);
      }
      sP[r * LP + c] = s;
    }
    __syncthreads();
    for (int idx = tid; idx < B * D; idx += kThreads) {
      const int r = idx / D, j = idx % D;
      float inter = 0.f;
      for (int k = 0; k < D; k++) inter = fmaf(sX[r * LD + k], sS[k * LD + j], inter);
      float intra = 0.f;
      for (int c = 0; c < B; c++) intra = fmaf(sP[r * LP + c], sZ[c * LD + j], intra);
      const int pos = blk * B + r;
      if (pos < n) gw[(int64_t)pos * p.stride_n + j] = intra + sInter[r] * inter;
    }
    if (it + 1 == nblk && gf == nullptr) break;  // the state after the last block is only needed on request
    __syncthreads();
    state_update<D>(sS, sY, sZ, sDec, lamB, tid);
  }
  if (gf != nullptr) {
    __syncthreads();
    const bool trf = p.fin_transposed & 1;
    for (int idx = tid; idx < D * D; idx += kThreads) gf[trf ? (idx % D) * D + idx / D : idx] = sS[(idx / D) * LD + idx % D];
  }
}

template <int D, bool REV>
__global__ __launch_bounds__(kThreads) void chunk_state_f32_kernel(ScanParams p) {
  using C = F32Cfg<D>;
  constexpr int B = C::B, LD = C::LD;
  __shared__ float sY[B * LD], sZ[B * LD], sS[D * LD], sDec[B];

  const int tid = threadIdx.x;
  const int chain = blockIdx.x / p.nchunks, chunk = blockIdx.x % p.nchunks;
  if (REV ? (chunk == 0) : (chunk == p.nchunks - 1)) return;
  const int bi = chain / p.heads, hi = chain % p.heads;
  const int64_t base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h;
  const float* gy = reinterpret_cast<const float*>(p.y[0]) + base;
  const float* gz = reinterpret_cast<const float*>(p.z[0]) + base;
  const int n = p.n;
  const float l2 = log2f(p.lambda[hi]);
  const float lamB = exp2f(l2 * (float)B);
  const int nblocks = (n + B - 1) / B;
  const int cb = p.chunk_tokens / B;
  const int blk_lo = chunk * cb;
  const int blk_hi = min(blk_lo + cb, nblocks);

  for (int idx = tid; idx < D * D; idx += kThreads) sS[(idx / D) * LD + idx % D] = 0.f;
  if (tid < B) sDec[tid] = exp2f(l2 * (float)(REV ? tid + 1 : B - 1 - tid));
  const int nblk = blk_hi - blk_lo;
  for (int it = 0; it < nblk; it++) {
    const int blk = REV ? blk_hi - 1 - it : blk_lo + it;
    __syncthreads();
    load_tile<D>(sY, gy, p.stride_n, blk * B, n, tid);
    load_tile<D>(sZ, gz, p.stride_n, blk * B, n, tid);
    __syncthreads();
    state_update<D>(sS, sY, sZ, sDec, lamB, tid);
  }
  __syncthreads();
  float* gs = p.states + ((int64_t)chain * p.nchunks + chunk) * (D * D);
  for (int idx = tid; idx < D * D; idx += kThreads) gs[idx] = sS[(idx / D) * LD + idx % D];
}

}  // namespace

int block_size_f32(int head_dim) { return head_dim == 64 ? F32Cfg<64>::B : F32Cfg<128>::B; }

hipError_t launch_scan_f32(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (int64_t)p.batch * p.heads * p.nchunks;
  if (grid == 0 || p.n == 0) return hipSuccess;
  dim3 g((unsigned)grid), b(kThreads);
  if (head_dim == 128) {
    if (reverse) hipLaunchKernelGGL((scan_f32_kernel<128, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((scan_f32_kernel<128, false>), g, b, 0, s, p);
  } else {
    if (reverse) hipLaunchKernelGGL((scan_f32_kernel<64, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((scan_f32_kernel<64, false>), g, b, 0, s, p);
  }
  return hipGetLastError();
}

hipError_t launch_chunk_states_f32(int head_dim, bool reverse, const ScanParams& p, hipStream_t s) {
  const int64_t grid = (int64_t)p.batch * p.heads * p.nchunks;
  if (grid == 0 || p.n == 0) return hipSuccess;
  dim3 g((unsigned)grid), b(kThreads);
  if (head_dim == 128) {
    if (reverse) hipLaunchKernelGGL((chunk_state_f32_kernel<128, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((chunk_state_f32_kernel<128, false>), g, b, 0, s, p);
  } else {
    if (reverse) hipLaunchKernelGGL((chunk_state_f32_kernel<64, true>), g, b, 0, s, p);
    else         hipLaunchKernelGGL((chunk_state_f32_kernel<64, false>), g, b, 0, s, p);
  }
  return hipGetLastError();
}

}  // namespace la2
