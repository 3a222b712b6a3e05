// Measurement helpers of the benchmark, built into a library of their own (libla2_bench.so): nothing here is
// part of the method or of the C ABI in include/la2.h.
//
// 1. A kernel that does nothing but stream, `reads` input streams in
// and `writes` output streams out, 16 bytes per lane and stream, non-temporal loads (as the scan kernels' tile
// loads), stores with the default or the non-temporal policy.  The benchmark times it beside the scan kernels
// on the same number of bytes and the same read : write mix: what the memory system gives a kernel with no
// arithmetic, no LDS and no dependences is the bound the scan kernels are measured against.
// 2. A register-only loop of v_mfma_f32_32x32x16_bf16 (no memory traffic, no LDS): what the matrix pipes of
// this machine deliver at the clock they sustain, the figure the benchmark quotes beside the 2.5 PFLOP/s of
// the data sheet.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

enum { kOk = 0, kErrNull = 1, kErrShape = 2, kErrAlign = 4, kErrLaunch = 6 };   // la2_status values

typedef __attribute__((ext_vector_type(4))) float f32x4;

template <int R, int W, bool NTS>
__global__ __launch_bounds__(256) void stream_probe_kernel(const f32x4* __restrict__ in, f32x4* __restrict__ out,
                                                            size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    f32x4 acc = {1.f, 2.f, 3.f, 4.f};
#pragma unroll
    for (int r = 0; r < R; r++) acc += __builtin_nontemporal_load(in + (size_t)r * n + i);
#pragma unroll
    for (int w = 0; w < W; w++) {
      const f32x4 v = acc * (float)(w + 1);
      if (NTS) __builtin_nontemporal_store(v, out + (size_t)w * n + i);
      else out[(size_t)w * n + i] = v;
    }
    // a read-only probe keeps its loads alive through a store that never happens
    if (W == 0 && acc[0] == 123.456f) out[0] = acc;
  }
}

template <int R, int W>
void launch(bool nts, const void* in, void* out, size_t n, hipStream_t s) {
  const dim3 g(8192), b(256);
  const f32x4* i4 = static_cast<const f32x4*>(in);
  f32x4* o4 = static_cast<f32x4*>(out);
  if (nts) hipLaunchKernelGGL((stream_probe_kernel<R, W, true>), g, b, 0, s, i4, o4, n);
  else     hipLaunchKernelGGL((stream_probe_kernel<R, W, false>), g, b, 0, s, i4, o4, n);
}


// 16 MFMAs per iteration on four independent accumulators (an MFMA's result is ready after its own 16 passes;
// four chains keep the pipe full), operands that never change.  The sink store never happens (the
// accumulators of a bf16 product of small integers cannot hit the sentinel) but keeps the loop alive.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__global__ __launch_bounds__(256) void mfma_peak_kernel(int iters, float* sink) {
  bf16x8 a, b;
#pragma unroll
  for (int j = 0; j < 8; j++) {
    a[j] = (__bf16)(float)((threadIdx.x + j) & 3);
    b[j] = (__bf16)(float)((threadIdx.x * 3 + j) & 1);
  }
  f32x16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
  for (int i = 0; i < iters; i++) {
#pragma unroll
    for (int u = 0; u < 4; u++) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
  }
  const f32x16 c = c0 + c1 + c2 + c3;
  float t = 0.f;
#pragma unroll
  for (int v = 0; v < 16; v++) t += c[v];
  if (t == -1.2345f) sink[0] = t;
}

}  // namespace

// One launch of `workgroups` x 4 waves x iters x 16 MFMAs; flops per launch = workgroups * 4 * iters * 16 * 32768.
extern "C" int la2_bench_mfma_peak(int32_t workgroups, int32_t iters, float* sink, void* hip_stream) {
  if (workgroups <= 0 || iters <= 0) return kErrShape;
  if (sink == nullptr) return kErrNull;
  hipLaunchKernelGGL(mfma_peak_kernel, dim3((unsigned)workgroups), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(hip_stream), iters, sink);
  return hipGetLastError() == hipSuccess ? kOk : kErrLaunch;
}

// One launch of the streaming kernel: reads `reads` (0..4) consecutive streams of bytes_per_stream bytes from
// `in` and writes `writes` (0..2) consecutive streams of the same size to `out` (values are arbitrary), 16 bytes
// per lane, non-temporal loads, stores with the non-temporal policy if nt_stores != 0.  `out` takes at least 16
// bytes also when writes == 0 (never written then).  Device pointers, 16-byte aligned; returns 0 or a code above.
extern "C" int la2_bench_stream_probe(int32_t reads, int32_t writes, int32_t nt_stores, const void* in, void* out,
                                       size_t bytes_per_stream, void* hip_stream) {
  if (reads < 0 || reads > 4 || writes < 0 || writes > 2 || reads + writes == 0) return kErrShape;
  if (bytes_per_stream % 16 != 0) return kErrAlign;
  if (bytes_per_stream == 0) return kOk;
  if (out == nullptr || (reads > 0 && in == nullptr)) return kErrNull;   // a read-only probe still takes 16 bytes of out
  if ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15) return kErrAlign;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  const size_t n = bytes_per_stream / 16;
  const bool nts = nt_stores != 0;
  switch (reads * 3 + writes) {
    case 0 * 3 + 1: launch<0, 1>(nts, in, out, n, s); break;
    case 0 * 3 + 2: launch<0, 2>(nts, in, out, n, s); break;
    case 1 * 3 + 0: launch<1, 0>(nts, in, out, n, s); break;
    case 1 * 3 + 1: launch<1, 1>(nts, in, out, n, s); break;
    case 1 * 3 + 2: launch<1, 2>(nts, in, out, n, s); break;
    case 2 * 3 + 0: launch<2, 0>(nts, in, out, n, s); break;
    case 2 * 3 + 1: launch<2, 1>(nts, in, out, n, s); break;
    case 2 * 3 + 2: launch<2, 2>(nts, in, out, n, s); break;
    case 3 * 3 + 0: launch<3, 0>(nts, in, out, n, s); break;
    case 3 * 3 + 1: launch<3, 1>(nts, in, out, n, s); break;
    case 3 * 3 + 2: launch<3, 2>(nts, in, out, n, s); break;
    case 4 * 3 + 0: launch<4, 0>(nts, in, out, n, s); break;
    case 4 * 3 + 1: launch<4, 1>(nts, in, out, n, s); break;
    default:        launch<4, 2>(nts, in, out, n, s); break;
  }
  return hipGetLastError() == hipSuccess ? kOk : kErrLaunch;
}
