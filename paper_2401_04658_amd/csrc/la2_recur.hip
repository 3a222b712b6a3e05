// Token-by-token recurrence over a short run of positions (Sec. 3.2.1, recursive form, and the reverse
// recursion of Sec. 3.2.2), gfx950:  kv_t = lambda kv_{t-1} + k_t^T v_t,  o_t = q_t kv_t  with the fp32
// d x d state of a (batch, head) chain held in registers for the whole run.
//
// Used for (a) multi-token decode (the state is read and written once per launch instead of once per
// token) and (b) the last seqlen % 64 positions of a segment whose final state is wanted (the block
// kernels form states after whole blocks only).  Plain fp32 FMA arithmetic; one workgroup per chain and
// instance; each thread owns float4 pieces of state rows, partial q.kv sums are reduced through LDS.
//
// One launch runs up to two instances (blockIdx.y) over the same positions: the backward tail needs
// dv_t = k_t G_t (state G = sum q^T do) and dk_t = v_t G_t^T, the second being the same recurrence on
// the transposed state with the roles of the operands exchanged.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "la2_internal.h"

namespace la2 {
namespace {

// threads of a workgroup: a multiple of the D / 4 threads that share a state row, 16 or 12 float4 pieces
// of state rows per thread
constexpr int threads_for(int d) { return d == 256 ? 1024 : d == 96 ? 192 : 256; }

// element i of a tensor of type DT (kF32, kBF16 or kF16) as fp32, and the store that goes with it
template <int DT>
__device__ __forceinline__ float load_elem(const void* p, int64_t i) {
  if (DT == kBF16) return (float)reinterpret_cast<const __bf16*>(p)[i];
  if (DT == kF16) return (float)reinterpret_cast<const _Float16*>(p)[i];
  return reinterpret_cast<const float*>(p)[i];
}
template <int DT>
__device__ __forceinline__ void store_elem(void* p, int64_t i, float x) {
  if (DT == kBF16) reinterpret_cast<__bf16*>(p)[i] = (__bf16)x;
  else if (DT == kF16) reinterpret_cast<_Float16*>(p)[i] = (_Float16)x;
  else reinterpret_cast<float*>(p)[i] = x;
}

template <int D, int DT>
__global__ __launch_bounds__(threads_for(D)) void recur_kernel(RecurParams p) {
  constexpr int kThreads = threads_for(D);
  constexpr int TPR = D / 4;            // threads per state row (float4 each)
  constexpr int RG = kThreads / TPR;    // rows in flight per sweep
  constexpr int ITER = D / RG;
  __shared__ float sx[D], sy[D], sz[D];
  __shared__ float4 sacc[RG][TPR];

  const int tid = threadIdx.x;
  const int inst = blockIdx.y;
  const int64_t chain = blockIdx.x;
  const int bi = (int)(chain / p.heads), hi = (int)(chain % p.heads);
  const int64_t base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h;
  const float lam = p.lambda[hi];
  const void* gx = inst ? p.x[1] : p.x[0];
  const void* gy = inst ? p.y[1] : p.y[0];
  const void* gz = inst ? p.z[1] : p.z[0];
  void* gw = inst ? p.w[1] : p.w[0];
  const float* ginit = inst ? p.init[1] : p.init[0];
  float* gfin = inst ? p.fin[1] : p.fin[0];
  const bool init_tr = (p.init_transposed >> inst) & 1, fin_tr = (p.fin_transposed >> inst) & 1;

  const int cg = tid % TPR, rg = tid / TPR;
  float4 s[ITER];
#pragma unroll
  for (int it = 0; it < ITER; it++) {
    const int i = rg + RG * it;   // state row (y feature); columns 4 cg .. 4 cg + 3 (z features)
    if (ginit == nullptr) {
      s[it] = float4{0.f, 0.f, 0.f, 0.f};
    } else if (!init_tr) {
      s[it] = *reinterpret_cast<const float4*>(ginit + chain * (int64_t)(D * D) + (int64_t)i * D + 4 * cg);
    } else {
      const float* g = ginit + chain * (int64_t)(D * D) + i;
      s[it] = float4{g[(4 * cg + 0) * D], g[(4 * cg + 1) * D], g[(4 * cg + 2) * D], g[(4 * cg + 3) * D]};
    }
  }

  const int nt = p.t1 - p.t0;
  for (int step = 0; step < nt; step++) {
    const int t = p.reverse ? p.t1 - 1 - step : p.t0 + step;
    const int64_t row = base + (int64_t)t * p.stride_n;
    if (tid < D) {
      sx[tid] = load_elem<DT>(gx, row + tid);
      sy[tid] = load_elem<DT>(gy, row + tid);
      sz[tid] = load_elem<DT>(gz, row + tid);
    }
    __syncthreads();
    const float4 z4 = *reinterpret_cast<const float4*>(&sz[4 * cg]);
    // forward: the carried state decays before the new term is added (kv_t = lambda kv_{t-1} + k^T v);
    // reverse: after the output (g_t = carried + q^T do, carried to t - 1 as lambda g_t)
    const float pre = p.reverse ? 1.f : lam, post = p.reverse ? lam : 1.f;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int it = 0; it < ITER; it++) {
      const int i = rg + RG * it;
      const float yi = sy[i], xi = sx[i];
      float4 u;
      u.x = fmaf(pre, s[it].x, yi * z4.x);
      u.y = fmaf(pre, s[it].y, yi * z4.y);
      u.z = fmaf(pre, s[it].z, yi * z4.z);
      u.w = fmaf(pre, s[it].w, yi * z4.w);
      acc.x = fmaf(xi, u.x, acc.x);
      acc.y = fmaf(xi, u.y, acc.y);
      acc.z = fmaf(xi, u.z, acc.z);
      acc.w = fmaf(xi, u.w, acc.w);
      s[it] = float4{post * u.x, post * u.y, post * u.z, post * u.w};
    }
    sacc[rg][cg] = acc;
    __syncthreads();
    if (tid < D) {
      const float* flat = reinterpret_cast<const float*>(sacc);
      float sum = 0.f;
#pragma unroll
      for (int g = 0; g < RG; g++) sum += flat[g * D + tid];
      store_elem<DT>(gw, row + tid, sum);
    }
    // the next step's loads into sx, sy, sz come after this step's second barrier; its first barrier
    // orders them against the reads of sacc above
  }

  if (gfin != nullptr) {
#pragma unroll
    for (int it = 0; it < ITER; it++) {
      const int i = rg + RG * it;
      if (!fin_tr) {
        *reinterpret_cast<float4*>(gfin + chain * (int64_t)(D * D) + (int64_t)i * D + 4 * cg) = s[it];
      } else {
        float* g = gfin + chain * (int64_t)(D * D) + i;
        g[(4 * cg + 0) * D] = s[it].x;
        g[(4 * cg + 1) * D] = s[it].y;
        g[(4 * cg + 2) * D] = s[it].z;
        g[(4 * cg + 3) * D] = s[it].w;
      }
    }
  }
}

}  // namespace

hipError_t launch_recur(int head_dim, int dtype, int batch, int ninst, const RecurParams& p, hipStream_t s) {
  const int64_t chains = (int64_t)batch * p.heads;
  if (chains == 0 || ninst == 0) return hipSuccess;
  dim3 g((unsigned)chains, (unsigned)ninst);
#define LA2_LAUNCH_RECUR(D, DT) hipLaunchKernelGGL((recur_kernel<D, DT>), g, dim3(threads_for(D)), 0, s, p)
#define LA2_LAUNCH_RECUR_D(D)                         \
  do {                                                \
    if (dtype == kBF16) LA2_LAUNCH_RECUR(D, kBF16);   \
    else if (dtype == kF16) LA2_LAUNCH_RECUR(D, kF16); \
    else LA2_LAUNCH_RECUR(D, kF32);                   \
  } while (0)
  if (head_dim == 256) LA2_LAUNCH_RECUR_D(256);
  else if (head_dim == 128) LA2_LAUNCH_RECUR_D(128);
  else if (head_dim == 96) LA2_LAUNCH_RECUR_D(96);
  else LA2_LAUNCH_RECUR_D(64);
#undef LA2_LAUNCH_RECUR_D
#undef LA2_LAUNCH_RECUR
  return hipGetLastError();
}

}  // namespace la2
