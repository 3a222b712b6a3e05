// Backward of the Norm epilogue (eq. (2) with Norm read as root-mean-square normalisation of every output
// row): one pass over the rows that turns the gradient g of the normalised output o into the gradient of
// the un-normalised output,
//     du_t = r_t (g_t - o_t mean_j(g_tj o_tj)),        r_t = 1 / sqrt(mean_j u_tj^2 + eps)  (kept by the forward)
// which Algorithm 2 then takes as its dO.  Memory-bound: 16 bytes per lane, a row per group of
// D * sizeof(T) / 16 lanes, the row mean by lane exchanges inside the group; streaming (non-temporal)
// loads and stores, measured 9 % faster than the default cache policy.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "la2_internal.h"

namespace la2 {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kThreads = 256;

template <typename T> struct Row16;            // the 16-byte piece of a row that one lane handles
template <> struct Row16<float> {
  static constexpr int N = 4;
  f32x4 v;
  __device__ float get(int i) const { return v[i]; }
  __device__ void set(int i, float x) { v[i] = x; }
};
template <> struct Row16<__bf16> {
  static constexpr int N = 8;
  bf16x8 v;
  __device__ float get(int i) const { return (float)v[i]; }
  __device__ void set(int i, float x) { v[i] = (__bf16)x; }
};
template <> struct Row16<_Float16> {
  static constexpr int N = 8;
  f16x8 v;
  __device__ float get(int i) const { return (float)v[i]; }
  __device__ void set(int i, float x) { v[i] = (_Float16)x; }
};

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void norm_bwd_rows_kernel(NormBwdParams p) {
  constexpr int N = Row16<T>::N;
  constexpr int LPR = D / N;                    // lanes per row (8 .. 32, a power of two)
  constexpr int ROWS = kThreads / LPR;          // rows per workgroup
  const int64_t rows = (int64_t)p.batch * p.heads * p.n;
  const int64_t row = (int64_t)blockIdx.x * ROWS + threadIdx.x / LPR;
  const int piece = threadIdx.x % LPR;
  const bool live = row < rows;                 // whole row groups are live or not: the exchanges stay inside a group
  const int64_t rr = live ? row : 0;
  const int64_t chain = rr / p.n, pos = rr % p.n;
  const int64_t off = (chain / p.heads) * p.stride_b + (chain % p.heads) * p.stride_h + pos * p.stride_n + piece * N;
  Row16<T> o, g, du;
  o.v = __builtin_nontemporal_load(reinterpret_cast<const decltype(o.v)*>(reinterpret_cast<const T*>(p.o) + off));
  g.v = __builtin_nontemporal_load(reinterpret_cast<const decltype(g.v)*>(reinterpret_cast<const T*>(p.g) + off));
  float c = 0.f;
#pragma unroll
  for (int i = 0; i < N; i++) c = fmaf(g.get(i), o.get(i), c);
#pragma unroll
  for (int m = 1; m < LPR; m <<= 1) c += __shfl_xor(c, m);
  c *= 1.f / (float)D;
  const float r = p.rstd[rr];
#pragma unroll
  for (int i = 0; i < N; i++) du.set(i, r * (g.get(i) - o.get(i) * c));
  if (live) __builtin_nontemporal_store(du.v, reinterpret_cast<decltype(du.v)*>(reinterpret_cast<T*>(p.du) + off));
}

template <typename T, int D>
hipError_t launch(const NormBwdParams& p, hipStream_t s) {
  constexpr int ROWS = kThreads / (D / Row16<T>::N);
  const int64_t rows = (int64_t)p.batch * p.heads * p.n;
  const int64_t grid = (rows + ROWS - 1) / ROWS;
  if (grid == 0) return hipSuccess;
  if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL((norm_bwd_rows_kernel<T, D>), dim3((unsigned)grid), dim3(kThreads), 0, s, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_norm_bwd_rows(int head_dim, int dtype, const NormBwdParams& p, hipStream_t s) {
  if (dtype == kBF16) return head_dim == 128 ? launch<__bf16, 128>(p, s) : launch<__bf16, 64>(p, s);
  if (dtype == kF16) return head_dim == 128 ? launch<_Float16, 128>(p, s) : launch<_Float16, 64>(p, s);
  return head_dim == 128 ? launch<float, 128>(p, s) : launch<float, 64>(p, s);
}

}  // namespace la2
