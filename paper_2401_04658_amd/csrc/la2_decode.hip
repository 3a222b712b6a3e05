// Recurrent decode step (Sec. 3.2.1, recursive form): kv <- lambda kv + k^T v, o = q kv, gfx950.
//
// Memory bound: the fp32 state (d x d per (batch, head)) is read and written once; everything
// else is negligible.  One workgroup per (batch, head); each thread streams float4 pieces of the
// state rows with all of its loads issued up front, then the partial q.kv sums of the row groups
// are reduced through LDS.
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

// NORM: the output row is normalised (eq. (2) read as root-mean-square normalisation over the head's features:
// o <- o / sqrt(mean_j o_j^2 + eps)) before it is stored.
template <int D, int DT, bool NORM = false>
__global__ __launch_bounds__(threads_for(D)) void decode_kernel(const void* q, const void* k, const void* v,
                                                          const float* lambda, float* kv, void* o, int heads,
                                                          float eps) {
  constexpr int kThreads = threads_for(D);
  constexpr int TPR = D / 4;            // threads per state row (float4 each)
  constexpr int RG = kThreads / TPR;    // rows in flight per sweep
  constexpr int ITER = D / RG;
  __shared__ float sq[D], sk[D], sv[D];
  __shared__ float4 sacc[RG][TPR];

  const int tid = threadIdx.x;
  const int64_t chain = blockIdx.x;
  const float lam = lambda[chain % heads];
  if (tid < D) {
    sq[tid] = load_elem<DT>(q, chain * D + tid);
    sk[tid] = load_elem<DT>(k, chain * D + tid);
    sv[tid] = load_elem<DT>(v, chain * D + tid);
  }
  const int cg = tid % TPR, rg = tid / TPR;
  float4* state = reinterpret_cast<float4*>(kv + chain * (int64_t)(D * D));
  float4 s[ITER];
#pragma unroll
  for (int it = 0; it < ITER; it++) s[it] = state[(int64_t)(rg + RG * it) * TPR + cg];
  __syncthreads();
  const float4 v4 = *reinterpret_cast<const float4*>(&sv[4 * cg]);
  float4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int it = 0; it < ITER; it++) {
    const int i = rg + RG * it;
    const float ki = sk[i], qi = sq[i];
    float4 t;
    t.x = fmaf(lam, s[it].x, ki * v4.x);
    t.y = fmaf(lam, s[it].y, ki * v4.y);
    t.z = fmaf(lam, s[it].z, ki * v4.z);
    t.w = fmaf(lam, s[it].w, ki * v4.w);
    {  // streaming (non-temporal) store of the new state row piece: measured 4-7 % faster than the default policy
      typedef __attribute__((ext_vector_type(4))) float f32x4;
      const f32x4 tv = {t.x, t.y, t.z, t.w};
      __builtin_nontemporal_store(tv, reinterpret_cast<f32x4*>(&state[(int64_t)i * TPR + cg]));
    }
    acc.x = fmaf(qi, t.x, acc.x);
    acc.y = fmaf(qi, t.y, acc.y);
    acc.z = fmaf(qi, t.z, acc.z);
    acc.w = fmaf(qi, t.w, acc.w);
  }
  sacc[rg][cg] = acc;
  __syncthreads();
  float sum = 0.f;
  if (tid < D) {
    const float* flat = reinterpret_cast<const float*>(sacc);
#pragma unroll
    for (int g = 0; g < RG; g++) sum += flat[g * D + tid];
  }
  if (NORM) {   // sum of squares over the row: inside each wave by lane exchanges, across the waves through LDS
    constexpr int NWAVE = (D + 63) / 64;   // waves that hold row elements
    __shared__ float ssq[NWAVE];
    float s2 = sum * sum;                  // 0 for tid >= D
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) s2 += __shfl_xor(s2, m);
    if (tid < D && (tid & 63) == 0) ssq[tid >> 6] = s2;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < NWAVE; i++) tot += ssq[i];
    sum *= 1.f / sqrtf(tot * (1.f / (float)D) + eps);
  }
  if (tid < D) store_elem<DT>(o, chain * D + tid, sum);
}

__global__ void state_copy_kernel(float* dst, const float* src, int64_t count) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) dst[i] = src ? src[i] : 0.f;
}

}  // namespace

hipError_t launch_state_copy(float* dst, const float* src, int64_t count, hipStream_t s) {
  if (count <= 0) return hipSuccess;
  hipLaunchKernelGGL(state_copy_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, dst, src, count);
  return hipGetLastError();
}

hipError_t launch_decode(int batch, int heads, int head_dim, int dtype, const void* q, const void* k,
                         const void* v, const float* lambda, float* kv, void* o, bool norm, float eps,
                         hipStream_t s) {
  const int64_t chains = (int64_t)batch * heads;
  if (chains == 0) return hipSuccess;
  dim3 g((unsigned)chains);
#define LA2_LAUNCH_DECODE(D, DT)                                                                                    \
  do {                                                                                                              \
    if (norm) hipLaunchKernelGGL((decode_kernel<D, DT, true>), g, dim3(threads_for(D)), 0, s, q, k, v, lambda, kv, \
                                 o, heads, eps);                                                                    \
    else      hipLaunchKernelGGL((decode_kernel<D, DT, false>), g, dim3(threads_for(D)), 0, s, q, k, v, lambda, kv, \
                                 o, heads, eps);                                                                    \
  } while (0)
#define LA2_LAUNCH_DECODE_D(D)                         \
  do {                                                 \
    if (dtype == kBF16) LA2_LAUNCH_DECODE(D, kBF16);   \
    else if (dtype == kF16) LA2_LAUNCH_DECODE(D, kF16); \
    else LA2_LAUNCH_DECODE(D, kF32);                   \
  } while (0)
  if (head_dim == 256) LA2_LAUNCH_DECODE_D(256);
  else if (head_dim == 128) LA2_LAUNCH_DECODE_D(128);
  else if (head_dim == 96) LA2_LAUNCH_DECODE_D(96);
  else LA2_LAUNCH_DECODE_D(64);
#undef LA2_LAUNCH_DECODE_D
#undef LA2_LAUNCH_DECODE
  return hipGetLastError();
}

}  // namespace la2
