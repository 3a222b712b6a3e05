// Backward of the Norm epilogue (eq. (2) with Norm read as root-mean-square normalisation of every output
// row): one pass over the rows that turns the gradient g of the normalised output o into the gradient of
// the un-normalised output,
//     du_t = r_t (g_t - o_t mean_j(g_tj o_tj)),        r_t = 1 / sqrt(mean_j u_tj^2 + eps)  (kept by the forward)
// which Algorithm 2 then takes as its dO.  Memory-bound: 16-byte pieces, a row per group of a power-of-two
// number of lanes (one piece per lane; three at head_dim 96), the row mean by lane exchanges inside the
// group; streaming (non-temporal) loads and stores, measured 9 % faster than the default cache policy.
//
// Also here: the forward normalisation as a pass of its own, in place, for the paths whose kernels have no
// epilogue (the short-run kernels behind the last whole block of a segment; fp32 data at head_dim 96 / 256,
// which runs the token recurrence).
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

// How the lanes share a row: PPL pieces per lane, LPR lanes per row (a power of two, 4 .. 64); lane `piece`
// of a row handles pieces piece, piece + LPR, ...
template <typename T, int D>
struct RowSplit {
  static constexpr int N = Row16<T>::N;
  static constexpr int PPL = D == 96 ? 3 : 1;
  static constexpr int LPR = D / N / PPL;
  static constexpr int ROWS = kThreads / LPR;   // rows per workgroup
  static_assert((LPR & (LPR - 1)) == 0 && LPR >= 1 && LPR <= 64, "lane exchanges stay inside a wave");
};

// FWD false: du = rstd (g - o mean(g o)).  FWD true: o <- o r in place with r = 1 / sqrt(mean(o^2) + eps), r -> rstd
// (p.g unused, p.du == p.o).
template <typename T, int D, bool FWD>
__global__ __launch_bounds__(kThreads) void norm_rows_kernel(NormBwdParams p, float eps) {
  using S = RowSplit<T, D>;
  constexpr int N = S::N, PPL = S::PPL, LPR = S::LPR, ROWS = S::ROWS;
  const int64_t rows = (int64_t)p.batch * p.heads * p.n;
  const int64_t row = (int64_t)blockIdx.x * ROWS + threadIdx.x / LPR;
  const int piece = threadIdx.x % LPR;
  bool live = row < rows;                       // whole row groups are live or not: the exchanges stay inside a group
  int64_t rr = live ? row : 0;
  if (p.bounds != nullptr) {                    // packed batch: rows in front of the first and behind the last sequence
    const int64_t t = rr % p.n;
    live = live && t >= p.bounds[0] && t < p.bounds[p.nbounds];
    if (!live) rr = (rr / p.n) * p.n + min((int64_t)p.bounds[0], (int64_t)p.n - 1);
  }
  const int64_t chain = rr / p.n, pos = p.t0 + rr % p.n;
  const int64_t ri = chain * p.rstd_stride + pos;   // this row's r
  const int64_t off = (chain / p.heads) * p.stride_b + (chain % p.heads) * p.stride_h + pos * p.stride_n + piece * N;
  Row16<T> o[PPL], g[PPL];
  float c = 0.f;
#pragma unroll
  for (int j = 0; j < PPL; j++) {
    const int64_t at = off + j * LPR * N;
    o[j].v = __builtin_nontemporal_load(reinterpret_cast<const decltype(o[j].v)*>(reinterpret_cast<const T*>(p.o) + at));
    if (!FWD)
      g[j].v = __builtin_nontemporal_load(reinterpret_cast<const decltype(g[j].v)*>(reinterpret_cast<const T*>(p.g) + at));
#pragma unroll
    for (int i = 0; i < N; i++) c = fmaf(FWD ? o[j].get(i) : g[j].get(i), o[j].get(i), c);
  }
#pragma unroll
  for (int m = 1; m < LPR; m <<= 1) c += __shfl_xor(c, m);
  c *= 1.f / (float)D;
  const float r = FWD ? 1.f / sqrtf(c + eps) : p.rstd[ri];
#pragma unroll
  for (int j = 0; j < PPL; j++) {
    Row16<T> out;
#pragma unroll
    for (int i = 0; i < N; i++) out.set(i, FWD ? o[j].get(i) * r : r * (g[j].get(i) - o[j].get(i) * c));
    if (live)
      __builtin_nontemporal_store(out.v, reinterpret_cast<decltype(out.v)*>(reinterpret_cast<T*>(p.du) + off + j * LPR * N));
  }
  if (FWD && live && piece == 0) const_cast<float*>(p.rstd)[ri] = r;
}

template <typename T, int D, bool FWD>
hipError_t launch(const NormBwdParams& p, float eps, hipStream_t s) {
  constexpr int ROWS = RowSplit<T, D>::ROWS;
  const int64_t rows = (int64_t)p.batch * p.heads * p.n;
  const int64_t grid = (rows + ROWS - 1) / ROWS;
  if (grid == 0) return hipSuccess;
  if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL((norm_rows_kernel<T, D, FWD>), dim3((unsigned)grid), dim3(kThreads), 0, s, p, eps);
  return hipGetLastError();
}

template <typename T, bool FWD>
hipError_t launch_d(int head_dim, const NormBwdParams& p, float eps, hipStream_t s) {
  if (head_dim == 256) return launch<T, 256, FWD>(p, eps, s);
  if (head_dim == 128) return launch<T, 128, FWD>(p, eps, s);
  if (head_dim == 96) return launch<T, 96, FWD>(p, eps, s);
  return launch<T, 64, FWD>(p, eps, s);
}

}  // namespace

hipError_t launch_norm_bwd_rows(int head_dim, int dtype, const NormBwdParams& p, hipStream_t s) {
  if (dtype == kBF16) return launch_d<__bf16, false>(head_dim, p, 0.f, s);
  if (dtype == kF16) return launch_d<_Float16, false>(head_dim, p, 0.f, s);
  return launch_d<float, false>(head_dim, p, 0.f, s);
}

hipError_t launch_norm_fwd_rows(int head_dim, int dtype, const NormBwdParams& p, float eps, hipStream_t s) {
  if (dtype == kBF16) return launch_d<__bf16, true>(head_dim, p, eps, s);
  if (dtype == kF16) return launch_d<_Float16, true>(head_dim, p, eps, s);
  return launch_d<float, true>(head_dim, p, eps, s);
}

}  // namespace la2
