// Internal declarations shared by the library's translation units (not part of the C ABI).
#ifndef LA2_INTERNAL_H_
#define LA2_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace la2 {

// element types of the sequence tensors (the values of la2_dtype)
enum { kF32 = 0, kBF16 = 1, kF16 = 2 };

// One "decayed causal scan": for every (batch, head) chain
//     forward : w_t = sum_{s<=t} lambda^(t-s) (x_t . y_s) z_s
//     reverse : w_t = sum_{s>=t} lambda^(s-t) (x_t . y_s) z_s
// Algorithm 1 is the forward scan of (q, k, v).  Algorithm 2's first loop is the forward scan of
// (dO, V, K) and its second loop is the reverse scan of (V, dO, Q) for dK and of (K, Q, dO) for dV.
struct ScanParams {
  // Up to two scans of the same shape, direction and decay can share one launch ("dual" launch):
  // workgroup 2 i runs scan 0 and workgroup 2 i + 1 runs scan 1 of the same (chain, chunk), so tiles
  // that both scans read (Algorithm 2's second loop reads Q and dO for dK and for dV) are fetched
  // from HBM once and served from cache the second time.
  const void* x[2];
  const void* y[2];
  const void* z[2];
  void* w[2];
  int32_t nscan;             // 1 or 2
  int32_t state_transposed;  // bit s set: scan s starts from the TRANSPOSE of the stored chunk state
  const float* lambda;       // [heads], device
  float* states;             // [chains][nchunks][D][D] fp32 chunk start states, or nullptr (nchunks == 1)
  int64_t stride_b, stride_h, stride_n;  // elements
  int32_t batch, heads, n;
  int32_t nchunks;       // sequence chunks processed by different workgroups
  int32_t chunk_tokens;  // tokens per chunk (multiple of the block size); last chunk may be short
  int32_t variant;       // bf16 d = 128 scan kernel: 0 automatic, 1 full-block, 2 half-block
  // Optional start state of each scan's chains and destination of the state after each chain's last
  // block: fp32 [chains][D][D], row = y feature, column = z feature (bit s of the *_transposed masks:
  // scan s sees it transposed).  nullptr: zero start / not wanted.  State convention: entering a block
  // that starts at position p the forward state is sum_{s<p} lambda^(p-1-s) y_s^T z_s (+ lambda^p init),
  // entering a block that ends at position p (exclusive) the reverse state is
  // sum_{s>=p} lambda^(s-p+1) y_s^T z_s (+ lambda^(n-p) init), so that both ends of a sequence need no
  // division by lambda.  The final state is only meaningful when n is a multiple of the block size
  // (forward) or when the reverse scan started from zero or n is such a multiple (reverse).
  const float* init[2];
  float* fin[2];
  int32_t init_transposed;
  int32_t fin_transposed;
  // Norm epilogue of a forward scan (eq. (2); scan 0 only, the fp32 kernels and the forward bf16 kernels):
  // when rstd is not nullptr every output row is multiplied by r = 1 / sqrt(mean_j w_j^2 + eps) before it is
  // stored, and r goes to rstd[chain * rstd_stride + position] (fp32; rstd_stride >= n: a launch over the whole
  // blocks of a longer segment writes into the segment's array).
  float* rstd;
  float eps;
  int32_t rstd_stride;
  // Packed sequences of different lengths (nullptr: a dense batch).  Device array of batch + 1 position
  // offsets: sequence b is positions cu_seqlens[b] .. cu_seqlens[b + 1] - 1 of a [total, heads, d] tensor
  // (stride_b unused); n is then the longest sequence's length, what the launch is planned for.
  const int32_t* cu_seqlens;
  // Forward 16-bit scan of head_dim 128 only: a second group of waves in every workgroup accumulates, from the
  // scan's own X tiles (as value-like operand) and the tiles of acc_y (as key-like operand), the REVERSE local
  // state of the workgroup's chunk, sum_c lambda^(c+1) acc_y_c^T x_c over the chunk's positions c (counted from
  // the chunk's first), into acc_states [chains][nchunks][D][D] (chunk 0 of a chain is not written: no chunk
  // follows it in a reverse scan).  Algorithm 2: the dQ scan streams dO anyway; with Q beside it, it leaves
  // the local dKV states that the dK / dV scan's chunks start from.  nullptr: off.
  const void* acc_y;
  float* acc_states;
  // Packed batch cut into sequence chunks (16-bit half-block path only; nullptr otherwise): a compact launch
  // grid.  Instead of batch * heads * nchunks workgroups, most of them for chunks that short sequences do not
  // have, the launch has wg_pairs * heads workgroups and workgroup i serves head i % heads of the (sequence,
  // chunk) pair wg_map[i / heads] = {sequence, chunk, state slot or -1, chunks of the sequence}; entries past
  // the last pair carry sequence -1.  Only sequences of more than one chunk have state slots: chunk j of
  // such a sequence keeps its state at states[(slot + j') * heads + head], consecutive chunks heads states apart.
  // The map is written by varlen_map_kernel from cu_seqlens (launch_varlen_map).
  const int4* wg_map;
  int32_t wg_pairs;
  // ... and the pairs of chunk 0 of the sequences that have state slots, in order (entries past the last: -1):
  // the units of the state scan's launch, which would otherwise be mostly workgroups with nothing to do
  const int32_t* long_list;
  int32_t nlong;
  // 16-bit half-block kernels only: states at sequence ends that are no block boundaries.  Non-zero: a forward
  // scan hands out in fin the state right after a chain's last position even if that position is not a block's
  // last (the update of a ragged last block then weights row c by lambda^(rem-1-c) and the carried state by
  // lambda^rem, rem = rows of that block), a reverse scan's start state enters right behind the chain's last
  // position likewise, and a chain of no positions passes its start state (or zero) on to fin.
  int32_t ragged_state;
  // 16-bit half-block kernels only: non-zero = `states` holds the chunks' LOCAL states (no scan over
  // them has run) and every workgroup forms its own start state from the local states of the chunks its scan
  // passes before: G <- init (or 0); for those chunks j in scan order: G <- lambda^(length of chunk j) G + L_j.
  // For a few chunks on a small problem that is cheaper than one more dependent launch between two short kernels.
  int32_t self_prefix;
};
// self_prefix: most terms a start state is formed from (the caller's start state and the local states of three chunks)
constexpr int kMaxPrefixTerms = 4;

// Which (batch row or sequence, head, chunk) a workgroup of a scan-type launch serves, and where that chunk's
// state lives ([D][D] floats at states + slot * D * D; slot < 0: the chain has a single chunk and no state slot).
// slot_stride: slots between consecutive chunks of the chain.  false: no work for this workgroup.
__device__ __forceinline__ bool place_workgroup(const ScanParams& p, int wg, int& bi, int& hi, int& chunk,
                                                int64_t& slot, int& slot_stride) {
  if (p.wg_map == nullptr) {
    const int chain = wg / p.nchunks;
    chunk = wg % p.nchunks;
    bi = chain / p.heads;
    hi = chain % p.heads;
    slot = (int64_t)chain * p.nchunks + chunk;
    slot_stride = 1;
    return true;
  }
  const int4 m = p.wg_map[wg / p.heads];
  // the same for every lane: say so (the chain's base address has to sit in scalar registers)
  const int seq = __builtin_amdgcn_readfirstlane(m.x), first_slot = __builtin_amdgcn_readfirstlane(m.z);
  hi = wg % p.heads;
  bi = seq;
  chunk = __builtin_amdgcn_readfirstlane(m.y);
  slot = first_slot < 0 ? -1 : ((int64_t)first_slot + chunk) * p.heads + hi;
  slot_stride = p.heads;
  return seq >= 0;
}

// Element offset of chain (bi, hi)'s first position and the chain's length.
__device__ __forceinline__ void chain_extent(const ScanParams& p, int bi, int hi, int64_t& base, int& n) {
  if (p.cu_seqlens != nullptr) {
    const int first = p.cu_seqlens[bi];
    n = p.cu_seqlens[bi + 1] - first;
    base = (int64_t)first * p.stride_n + (int64_t)hi * p.stride_h;
  } else {
    n = p.n;
    base = (int64_t)bi * p.stride_b + (int64_t)hi * p.stride_h;
  }
  // Both are the same for every lane of the workgroup; told to the compiler, so that the chain's base address
  // lives in scalar registers whatever path the indices took (the direct loads take it as a scalar operand).
  n = __builtin_amdgcn_readfirstlane(n);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)base);
  const uint32_t hi32 = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)base >> 32));
  base = (int64_t)(((uint64_t)hi32 << 32) | lo);
}

// Where a chain's r values start in p.rstd: dense batches [batch * heads][rstd_stride positions]; packed batches
// [heads][rstd_stride = total positions], a sequence's values at its packed positions.
__device__ __forceinline__ int64_t rstd_chain_offset(const ScanParams& p, int bi, int hi) {
  if (p.cu_seqlens != nullptr) return (int64_t)hi * p.rstd_stride + p.cu_seqlens[bi];
  return ((int64_t)bi * p.heads + hi) * p.rstd_stride;
}

// Norm epilogue, shared by the scan kernels.  A 32 x 32 output tile sits in MFMA accumulators transposed
// (lane = position l32, 16 features per lane, the other 16 in lane l32 + 32); the NP waves that hold the
// feature tiles of one row exchange their partial sums of squares through `red` ([32 rows][NP] floats per
// row tile).  Between publish and collect the caller places a workgroup barrier.
// The exchange buffer: N floats of LDS in the kernels that ask for them, nothing otherwise.
template <int N>
struct NormExchange {
  static __device__ __forceinline__ float* get() {
    __shared__ float red[N];
    return red;
  }
};
template <>
struct NormExchange<0> {
  static __device__ __forceinline__ float* get() { return nullptr; }
};
template <int NP, typename Acc>
__device__ __forceinline__ void norm_publish(const Acc& sq, float* red, int l32, int hh, int slot) {
  float s = 0.f;
#pragma unroll
  for (int v = 0; v < 16; v++) s = fmaf(sq[v], sq[v], s);
  s += __shfl_xor(s, 32);
  if (hh == 0) red[l32 * NP + slot] = s;
}
template <int NP>
__device__ __forceinline__ float norm_collect(const float* red, int l32, float inv_d, float eps) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NP; i++) s += red[l32 * NP + i];
  return __builtin_amdgcn_rsqf(fmaf(s, inv_d, eps));
}

// Block size (rows of the intra-block tile) per data type / head dim.
int block_size_bf16(int head_dim);
int block_size_f32(int head_dim);

// 16-bit MFMA path (dtype kBF16 or kF16; head_dim 64 or 128)
hipError_t launch_scan_bf16(int dtype, int head_dim, bool reverse, const ScanParams& p, hipStream_t s);
hipError_t launch_chunk_states_bf16(int dtype, int head_dim, bool reverse, const ScanParams& p, hipStream_t s);
// 16-bit path of head_dim 96 and 256: the scan (one or two per launch, as above), or (state_only) the local
// chunk states of its pre-pass; ragged ends are exact, so final states are meaningful for any n
hipError_t launch_scan_wide(int dtype, int head_dim, bool reverse, bool state_only, const ScanParams& p, hipStream_t s);
// O(n^2 d) left-product evaluation of one scan, for comparison (bf16; uses x, y, z, w of scan 0):
// w = [(x y^T) * M] z over all earlier blocks, or with `reverse` the transposed mask over all later blocks
hipError_t launch_left_product_bf16(int head_dim, bool reverse, const ScanParams& p, hipStream_t s);
// fp32 path
hipError_t launch_scan_f32(int head_dim, bool reverse, const ScanParams& p, hipStream_t s);
hipError_t launch_chunk_states_f32(int head_dim, bool reverse, const ScanParams& p, hipStream_t s);
// packed batch in chunks: fills map[0 .. p.wg_pairs) and long_list[0 .. p.nlong) from p.cu_seqlens (one small workgroup)
hipError_t launch_varlen_map(const ScanParams& p, int4* map, int32_t* long_list, int64_t nslots, hipStream_t s);
// turns the per-chunk local states in p.states into chunk start states (any dtype: states are fp32);
// the first chunk starts from p.init[0] (seen through bit 0 of p.init_transposed) or zero
hipError_t launch_state_scan(int head_dim, bool reverse, const ScanParams& p, hipStream_t s);

// Token-by-token recurrence over positions [t0, t1) of every chain, up to two instances per launch:
//   forward (reverse == 0), ascending:   S <- lambda S + y_t^T z_t,  w_t = x_t S
//   reverse (reverse == 1), descending:  S <- S + y_t^T z_t,  w_t = x_t S,  then S <- lambda S
// S starts from init[i] (fp32 [chains][D][D], row = y feature; nullptr = 0; bit i of init_transposed:
// stored transposed) and is written to fin[i] afterwards (may alias init[i]; nullptr = not wanted).
// With these conventions the states are the ones ScanParams describes.
struct RecurParams {
  const void* x[2];
  const void* y[2];
  const void* z[2];
  void* w[2];
  const float* init[2];
  float* fin[2];
  int32_t init_transposed, fin_transposed;
  const float* lambda;   // [heads], device
  int32_t heads;
  int32_t t0, t1;
  int32_t reverse;
  int64_t stride_b, stride_h, stride_n;  // elements, all of x, y, z, w
  // Norm epilogue (launch_tail_bf16 only): as ScanParams; r of position t goes to rstd[chain * rstd_stride + t]
  float* rstd;
  float eps;
  int32_t rstd_stride;
};
hipError_t launch_recur(int head_dim, int dtype, int batch, int ninst, const RecurParams& p, hipStream_t s);
// The forward case of the same for 16-bit data (instance 0 only, reverse == 0) as a block kernel: MFMA in
// blocks of 32 positions, the state after position t1 - 1 exact for any t1 - t0.  Needs t0 < t1.
hipError_t launch_tail_bf16(int dtype, int head_dim, int batch, const RecurParams& p, hipStream_t s);

// Backward of the Norm epilogue, row by row: du = rstd * (g - o * mean_j(g_j o_j)) with o the normalised
// output and g its gradient; o, g, du share the layout given by the strides (elements), rstd is
// [batch * heads][n] fp32.
// The rows are positions t0 .. t0 + n - 1 of every chain; r of position t is rstd[chain * rstd_stride + t].
struct NormBwdParams {
  const void* o;
  const void* g;
  const float* rstd;
  void* du;
  int64_t stride_b, stride_h, stride_n;
  int32_t batch, heads, n;
  int32_t t0, rstd_stride;
  // packed batch (rows = all packed positions, batch = 1): only positions row_lo <= t < row_hi belong to a
  // sequence, with row_lo = bounds[0], row_hi = bounds[nbounds] read on the device (cu_seqlens); nullptr: all rows
  const int32_t* bounds;
  int32_t nbounds;
};
hipError_t launch_norm_bwd_rows(int head_dim, int dtype, const NormBwdParams& p, hipStream_t s);
// The forward normalisation as a pass of its own, in place, over the same rows: o <- o r with
// r = 1 / sqrt(mean_j o_j^2 + eps) written to rstd (p.g unused, p.du == p.o).  For the paths whose kernels have
// no epilogue: the short-run kernels behind a segment's last block, and fp32 data at head_dim 96 / 256.
hipError_t launch_norm_fwd_rows(int head_dim, int dtype, const NormBwdParams& p, float eps, hipStream_t s);

// dst[i] = src ? src[i] : 0 for count floats (a state that passes through an empty sequence)
hipError_t launch_state_copy(float* dst, const float* src, int64_t count, hipStream_t s);

// norm: the output row is divided by sqrt(mean of its squares + eps) before it is stored
hipError_t launch_decode(int batch, int heads, int head_dim, int dtype, const void* q, const void* k,
                         const void* v, const float* lambda, float* kv, void* o, bool norm, float eps,
                         hipStream_t s);

}  // namespace la2
#endif
