// Measurement helper, not part of the method: a kernel that does nothing but stream, `reads` input streams in
// and `writes` output streams out, 16 bytes per lane and stream, non-temporal loads (as the scan kernels' tile
// loads), stores with the default or the non-temporal policy.  The benchmark times it beside the scan kernels
// on the same number of bytes and the same read : write mix: what the memory system gives a kernel with no
// arithmetic, no LDS and no dependences is the bound the scan kernels are measured against.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/la2.h"

namespace {

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

}  // namespace

extern "C" la2_status la2_stream_probe(int32_t reads, int32_t writes, int32_t nt_stores, const void* in, void* out,
                                       size_t bytes_per_stream, void* hip_stream) {
  if (reads < 0 || reads > 4 || writes < 0 || writes > 2 || reads + writes == 0) return LA2_ERR_SHAPE;
  if (bytes_per_stream % 16 != 0) return LA2_ERR_STRIDE_ALIGN;
  if (bytes_per_stream == 0) return LA2_OK;
  if (out == nullptr || (reads > 0 && in == nullptr)) return LA2_ERR_NULL;   // a read-only probe still takes 16 bytes of out
  if ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15) return LA2_ERR_STRIDE_ALIGN;
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
  return hipGetLastError() == hipSuccess ? LA2_OK : LA2_ERR_LAUNCH;
}
