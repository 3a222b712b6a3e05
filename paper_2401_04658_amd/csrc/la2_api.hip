// Host side of the C ABI: argument validation, chunk planning and kernel dispatch.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <atomic>

#include "../../include/la2.h"
#include "la2_internal.h"

// Chunk start states of la2_fwd_noalloc: device memory that belongs to the library's code object, so that the
// entry point needs no workspace argument and never allocates.  Every GPU the library runs on holds its own
// copy at its own address; in host code this name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[LA2_NOALLOC_SCRATCH_BYTES];

namespace {

// The two test / tuning knobs are the library's only mutable state besides the per-device scratch address:
// plain atomics, read once per call.
std::atomic<int> g_chunk_tokens_override{0};  // la2_set_chunk_tokens()
std::atomic<int> g_scan_variant{0};           // la2_set_scan_variant()
bool is16(int dtype) { return dtype == LA2_BF16 || dtype == LA2_F16; }
// Head dimensions 96 and 256 have kernels of their own: one 16-bit block kernel that is exact at a ragged end
// (no granule), and the token recurrence for fp32.
bool wide(int head_dim) { return head_dim == 96 || head_dim == 256; }
bool supported_head_dim(int head_dim) { return head_dim == 64 || head_dim == 128 || wide(head_dim); }
// The fp32 block kernels (head_dim 64 and 128) form states after whole blocks of 32 positions only; the 16-bit
// kernels form the state at a ragged end inside their block loop (no granule).
int state_granule(const la2_desc* d) {
  return (wide(d->head_dim) || is16(d->dtype)) ? 1 : 32;
}
// 16-bit half-block kernels (head_dim 64 / 128): a state wanted behind, or coming in behind, a last block that is
// not full needs their ragged-end instantiation (ScanParams::ragged_state)
bool ragged_end(const la2_desc* d) {
  return is16(d->dtype) && !wide(d->head_dim) && d->seqlen % 32 != 0;
}

int device_cu_count() {
  static int cached = 0;
  if (cached > 0) return cached;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0) {
    cached = cus;
    return cus;
  }
  (void)hipGetLastError();
  return 256;  // MI355X; used when no device is visible (host-only callers sizing a workspace)
}

int elem_size(int dtype) { return dtype == LA2_F32 ? 4 : 2; }

// Device address of `scratch` on the current device, looked up once per device (the first call on a device
// may load the code object there; later calls only read the cached pointer).
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

la2_status scratch_on_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return LA2_ERR_LAUNCH;
  }
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr == nullptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
      (void)hipGetLastError();
      return LA2_ERR_LAUNCH;
    }
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // two threads racing here store the same address
  }
  *out = ptr;
  return LA2_OK;
}

la2_status check_desc_fields(const la2_desc* d) {
  if (d == nullptr) return LA2_ERR_NULL;
  if (d->dtype != LA2_F32 && !is16(d->dtype)) return LA2_ERR_DTYPE;
  if (d->batch < 0 || d->heads < 0 || d->seqlen < 0 || d->reserved != 0) return LA2_ERR_SHAPE;
  if (!supported_head_dim(d->head_dim)) return LA2_ERR_SHAPE;
  if ((int64_t)d->batch * d->heads > (int64_t)1 << 24) return LA2_ERR_SHAPE;
  // rows of one tensor: keeps the grids of the row passes (4 rows per workgroup at least) and of the left-product
  // comparison (128 rows per workgroup) below 2^31; more rows than this fit no device's memory anyway
  if ((int64_t)d->batch * d->heads * d->seqlen > (int64_t)1 << 32) return LA2_ERR_SHAPE;
  const int64_t per16 = 16 / elem_size(d->dtype);
  if (d->stride_b < 0 || d->stride_h < 0 || d->stride_n < d->head_dim) return LA2_ERR_STRIDE_ALIGN;
  if (d->stride_b % per16 || d->stride_h % per16 || d->stride_n % per16) return LA2_ERR_STRIDE_ALIGN;
  // The kernels address one chain with 32-bit byte offsets.  The rows of a ragged last block (up to 127
  // positions past the end in the widest kernel) are computed and then dropped by the store's range check,
  // so their offsets must not wrap around either.
  if (((int64_t)d->seqlen + 128) * d->stride_n * elem_size(d->dtype) > ((int64_t)1 << 32)) return LA2_ERR_SHAPE;
  return LA2_OK;
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Granularity of the sequence chunks (the block size of the chunk-state pre-pass; a multiple of every
// scan kernel's block size).
int block_size(const la2_desc* d) {
  return is16(d->dtype) ? la2::block_size_bf16(d->head_dim) : la2::block_size_f32(d->head_dim);
}

struct Plan {
  int nchunks;
  int chunk_tokens;
  size_t workspace;     // bytes of chunk states (one set)
  // packed batch with a compact launch grid (make_plan_varlen): (sequence, chunk) pairs the grid has room for and
  // bytes of the pair map that sits in front of the states; 0 otherwise
  int wg_pairs = 0;
  int nlong = 0;        // sequences of more than one chunk the plan has room for (the state scan's units)
  int64_t wg_slots = 0; // state slots (per head) the workspace has room for
  size_t map_bytes = 0;
};

bool self_prefix(const la2_desc* d, const Plan& pl, const int32_t* cu);
bool fuses_reverse_states(const la2_desc* d);

// Sequence chunks: the block loop of one chain is sequential, so when batch*heads cannot fill the
// compute units the sequence is cut into chunks that run in parallel from pre-computed start states.
Plan make_plan(const la2_desc* d) {
  const int B = block_size(d);
  const int64_t chains = (int64_t)d->batch * d->heads;
  const int nblocks = (d->seqlen + B - 1) / B;
  Plan pl{1, nblocks > 0 ? nblocks * B : B, 0};
  if (chains == 0 || nblocks <= 1) return pl;
  if (wide(d->head_dim) && !is16(d->dtype)) return pl;   // token recurrence: one workgroup walks the chain
  int cb;  // blocks per chunk
  const int chunk_override = g_chunk_tokens_override.load(std::memory_order_relaxed);
  if (chunk_override > 0) {
    cb = (chunk_override + B - 1) / B;
  } else {
    const int cus = device_cu_count();
    if (chains >= cus) return pl;
    // More chains than half the compute units: two chunks would make between one and two workgroups per unit, the
    // launch would move 1.4 times the bytes and most of the bandwidth is already in use (192 chains of 4096
    // positions, forward + backward: 0.58 ms uncut against 0.76 ms in two chunks at head_dim 128, 0.31 / 0.36 at 64,
    // 0.47 / 0.66 at 96).  Head_dim 96, whose kernel runs four workgroups a unit, also at exactly half (0.42 / 0.46).
    if (is16(d->dtype) && (chains * 2 > cus || (d->head_dim == 96 && chains * 2 == cus))) return pl;
    // workgroups to aim for: one per compute unit; two at head_dim 96 (64 chains of 8192 positions: 0.43 ms in eight
    // chunks against 0.47 ms in four)
    // ... and never more than that: the workgroups past one per unit double up on some units while others have one,
    // and the launch takes as long as the doubled ones (48 chains of 4096 positions at head_dim 128, forward +
    // backward: 0.22 ms in four or five chunks, 0.31 ms in six; the same cliff at head_dim 64 and 256).
    int want = (int)(cus / chains);
    if (d->head_dim == 96) {   // ... two per unit while the chunks stay 640 positions or longer (8 chains of 32768
      const int want2 = (int)(2 * (int64_t)cus / chains);   // positions: 0.25 ms in 32 chunks, 0.27 ms in 64)
      if (d->seqlen / want2 >= 640) want = want2;
    }
    // fp32 data at head_dim 64: that kernel is bound by its arithmetic and three of its workgroups share a unit
    // (192 chains of 4096 positions, forward + backward: 2.2 ms uncut, 1.38 ms in four chunks; 64 chains: 0.79 ms in
    // four chunks, 0.57 ms in eleven)
    if (!is16(d->dtype) && d->head_dim == 64) want = (int)(3 * (int64_t)cus / chains);
    if (want < 2) return pl;
    cb = (nblocks + want - 1) / want;
    if (cb < 4) cb = 4;  // keep the state pre-pass a small fraction of the work
    if (cb >= nblocks) return pl;
    // Chunking shortens the scan's sequential loop from nblocks to cb blocks but adds the pre-pass (about a
    // third of a scan block per block) and two more launches (about 15 us): not worth it for short sequences.
    // Measured times of one block of the sequential loop, in microseconds.
    const float t_blk = is16(d->dtype) ? (d->head_dim == 256 ? 3.3f : d->head_dim == 96 ? 3.f : d->head_dim == 64 ? 1.15f : 2.1f)
                                       : (d->head_dim == 128 ? 10.f : 3.f);
    if (is16(d->dtype) && d->head_dim == 256) {
      // One workgroup of this kernel fills a compute unit, and a block takes it 3.3 us with every unit busy but
      // 2.3 us with half of them idle; the pre-pass costs 0.6 of a scan block per block.  Measured at 128 chains of
      // 4096 positions: 0.29 + 0.68 ms uncut (half the units idle) against 0.35 + 0.92 ms in two chunks.
      const int nch = (nblocks + cb - 1) / cb;
      const float rounds = (float)((chains * nch + cus - 1) / cus), pre_rounds = (float)((chains * (nch - 1) + cus - 1) / cus);
      const float t_uncut = (float)nblocks * (chains * 2 <= cus ? 2.3f : 3.3f);
      const float t_cut = (rounds + 0.6f * pre_rounds) * (float)cb * 3.3f + 15.f;
      if (t_cut >= t_uncut) return pl;
    } else {
      // the extra launches: the pre-pass and the scan over the chunk states, which plans of a few chunks do without
      Plan cut{(nblocks + cb - 1) / cb, cb * B, 0};
      const float launches = self_prefix(d, cut, nullptr) ? 8.f : 15.f;
      if ((float)(nblocks - cb) * t_blk - 0.35f * (float)cb * t_blk - launches <= 0.f) return pl;
    }
  }
  if (cb >= nblocks) return pl;
  pl.nchunks = (nblocks + cb - 1) / cb;
  pl.chunk_tokens = cb * B;
  pl.workspace = (size_t)chains * pl.nchunks * d->head_dim * d->head_dim * sizeof(float);
  return pl;
}

// Packed batch of sequences of different lengths (batch chains per head, the longest of seqlen positions,
// total_positions in all; 0 = not known).  With few chains the dense rule above already cuts the sequences.
// With many chains it does not, and then a batch of very unequal lengths runs as long as its longest sequence's
// sequential block loop: when that loop is estimated to outlast the whole batch's memory traffic, the sequences
// are cut into chunks of a quarter of the longest one (at least four blocks).  Shorter sequences then have one
// chunk and no pre-pass work; only the long ones pay the second read of their key-like and value-like rows.
// The launch grid of such a plan is compact: one workgroup per (sequence, chunk) pair that exists and head (a
// grid of batch x heads x nchunks workgroups, most of them for chunks the short sequences do not have, costs
// about 10 ns per empty workgroup and launch: measured 1.16 ms against 0.34 ms uncut for 191 sequences x 16
// heads x 8 chunks).  A sequence of len positions has at most len / C + 1 pairs, and only sequences longer than
// C need state slots, at most 2 len / C each.  16-bit data at head_dim 64 / 128 (the half-block kernels) only.
constexpr int kPackedCut = 4;   // pieces the longest sequence of such a batch is cut into
Plan make_plan_varlen(const la2_desc* d, int64_t total_positions) {
  Plan pl = make_plan(d);
  if (total_positions <= 0 || d->batch <= 0) return pl;
  if (!is16(d->dtype) || wide(d->head_dim) || g_scan_variant.load(std::memory_order_relaxed) == 1) return pl;
  const int B = block_size(d);
  const int nblocks = (d->seqlen + B - 1) / B;
  auto compact = [&](Plan c) {   // the compact grid and its map for a plan that has chunks
    const int64_t all = (int64_t)d->batch * c.nchunks;
    const int64_t pairs = std::min<int64_t>(all, total_positions / c.chunk_tokens + d->batch);
    const int64_t slots = std::min<int64_t>(all, 2 * total_positions / c.chunk_tokens);
    const int64_t nlong = std::min<int64_t>(d->batch, total_positions / c.chunk_tokens);
    if (pairs > ((int64_t)1 << 30)) return c;
    c.wg_pairs = (int)pairs;
    c.nlong = (int)nlong;
    c.wg_slots = slots;
    c.map_bytes = ((size_t)pairs * sizeof(int4) + (size_t)nlong * sizeof(int32_t) + 255) & ~(size_t)255;
    c.workspace = (size_t)slots * d->heads * d->head_dim * d->head_dim * sizeof(float);
    return c;
  };
  // the dense rule (few chains) or the test knob already cut the sequences: same chunks, compact grid
  if (pl.nchunks > 1) return compact(pl);
  if (g_chunk_tokens_override.load(std::memory_order_relaxed) > 0) return pl;
  if (nblocks < 8) return pl;
  if ((int64_t)d->seqlen * d->batch <= 2 * total_positions) return pl;   // lengths about equal
  // microseconds: the longest chain's loop (measured times per block, as in make_plan) against the batch's forward
  // traffic at 5.5 TB/s
  const float t_blk = is16(d->dtype) ? (d->head_dim == 256 ? 3.3f : d->head_dim == 96 ? 3.f : d->head_dim == 64 ? 1.15f : 2.1f)
                                     : (d->head_dim == 128 ? 10.f : 3.f);
  const float t_longest = (float)nblocks * t_blk;
  const float t_traffic = (float)total_positions * d->heads * d->head_dim * 4.f * elem_size(d->dtype) / 5.5e6f;
  if (t_longest <= 1.25f * t_traffic) return pl;
  int cb = (nblocks + kPackedCut - 1) / kPackedCut;
  if (cb < 4) cb = 4;
  if (cb >= nblocks) return pl;
  pl.nchunks = (nblocks + cb - 1) / cb;
  pl.chunk_tokens = cb * B;
  pl.workspace = (size_t)d->batch * d->heads * pl.nchunks * d->head_dim * d->head_dim * sizeof(float);
  const Plan c = compact(pl);
  return c.wg_pairs > 0 ? c : make_plan(d);
}

// Grid sizes of every launch a plan leads to, checked on the host before the first one: the scan kernels take
// chains * nchunks workgroups per scan (two scans in a dual launch), the state scan chains * d * d / 256.
bool plan_fits_a_grid(const la2_desc* d, const Plan& pl) {
  const int64_t chains = (int64_t)d->batch * d->heads;
  const int64_t limit = ((int64_t)1 << 31) - 1;
  if (pl.wg_pairs > 0)   // compact grid: pairs x heads workgroups, and as many units in the state scan
    return (int64_t)pl.wg_pairs * d->heads * ((d->head_dim * d->head_dim + 255) / 256) <= limit;
  if (chains * pl.nchunks * 2 > limit) return false;
  if (pl.nchunks > 1 && chains * ((d->head_dim * d->head_dim + 255) / 256) > limit) return false;
  return true;
}

la2_desc whole_blocks(const la2_desc* d);

// Everything that can be rejected from the descriptor alone, the launch grids included.
la2_status check_desc(const la2_desc* d) {
  const la2_status st = check_desc_fields(d);
  if (st != LA2_OK) return st;
  const la2_desc wb = whole_blocks(d);   // the state entry points may run the block kernels on the whole blocks only
  if (!plan_fits_a_grid(d, make_plan(d)) || !plan_fits_a_grid(&wb, make_plan(&wb))) return LA2_ERR_SHAPE;
  return LA2_OK;
}

// A dense batch with a few more chains than a whole number of chains per compute unit: the units that get one
// workgroup more set the launch's time (n 4096, head_dim 128, bf16, forward + backward: 256 chains 0.67 ms, 320
// chains 1.14 ms; fp32: 9.5 ms for anything from 272 to 480 chains).  The dense entry points run such a batch as two
// calls: the first rows, a whole number of chains per unit (up to four), whole; the rest by the plan for that many chains, i.e. in
// chunks (320 chains: 0.67 + 0.27 ms).  Returns the rows of the first call, 0 for one call.
// Measured, two calls against one, forward + backward, n 2048 / 4096 / 8192 (256 units):
//   chains           272          288          320          352          384
//   bf16 d 64, 128   0.81-0.92    0.80-0.93    0.85-0.95    0.94-1.05    -         (n 1024: 0.95-1.12)
//   bf16 d 96        0.76-0.88    0.82-0.91    0.91-0.98    0.98-1.11    1.04-1.07
//   bf16 d 256       0.82-0.86    0.87-0.96    0.96-1.05    1.01-1.03    1.01
//   fp32 d 128       0.53-0.59    0.57-0.64    0.66-0.71    0.82-0.86    0.84-0.87 (n 1024: 0.64, -, 0.74, -, 0.90)
//   fp32 d 64        0.64-0.67    0.66-0.72    0.72-0.77    0.78-0.81    0.84-0.87 (n 1024: 0.75, -, 0.85, -, 0.94)
//   chains           544          576          640
//   bf16 d 64, 128   0.86-0.98    0.90-0.99    0.98-1.05    (n 4096 and 8192: 0.86-0.90, 0.90-0.94)
//   bf16 d 96        0.87-0.93    0.92-0.98    1.03
//   bf16 d 256       0.96         1.01         1.01
//   fp32 d 128       0.73         0.79         0.91         (n 4096)
//   fp32 d 64        1.06         1.11         1.23         (two workgroups per unit: no step at 512)
//   chains           800          832          864          1056         1088
//   bf16 d 64, 128   0.90-0.93    0.93-0.95    0.97-0.99    0.94         0.96         (n 4096 and 8192)
// The rule below takes the cells at 0.95 or under.
int rows_of_first_call(const la2_desc* d) {
  if (g_chunk_tokens_override.load(std::memory_order_relaxed) > 0) return 0;   // the caller plans
  const int cus = device_cu_count();
  const int n = d->seqlen, hd = d->head_dim;
  const int64_t chains = (int64_t)d->batch * d->heads;
  const int64_t k = chains / cus;   // whole rounds of one chain per unit
  if (k < 1 || k > 4 || d->heads > cus) return 0;
  // the largest partial round, in eighths of the unit count, that is worth a call of its own
  int eighths = 0;
  if (d->dtype == LA2_F32) {
    if (wide(hd)) return 0;
    if (k == 1) eighths = n >= 1024 ? 4 : 0;
    else eighths = k == 2 && hd == 128 && n >= 2048 ? 2 : 0;
  } else if (hd == 256) {
    eighths = k == 1 && n >= 2048 ? 1 : 0;
  } else if (hd == 96) {
    eighths = k == 1 ? (n >= 4096 ? 2 : n >= 2048 ? 1 : 0) : (k == 2 && n >= 4096 ? 1 : 0);
  } else if (k == 1) {
    eighths = n >= 4096 ? 3 : n >= 2048 ? 2 : 0;
  } else {
    eighths = n >= 4096 ? (k <= 3 ? 2 : 1) : 0;
  }
  const int64_t rows = k * cus / d->heads;
  const int64_t rest_chains = chains - rows * d->heads;
  if (rows < 1 || rest_chains <= 0 || rest_chains * 8 > (int64_t)cus * eighths) return 0;
  la2_desc rest = *d;
  rest.batch = d->batch - (int)rows;
  if (make_plan(&rest).nchunks <= 1) return 0;   // sequences too short to cut: the rest would run whole as well
  return (int)rows;
}

// The two parts of such a batch: the first `rows` batch rows and the others.  Byte offsets of the second part in
// the [batch, heads, seqlen, head_dim] tensors, element offsets in the fp32 states and in rstd.
struct RowParts {
  la2_desc first, rest;
  int64_t bytes, state, rstd;
};

RowParts row_parts(const la2_desc* d, int rows) {
  RowParts p{*d, *d, 0, 0, 0};
  p.first.batch = rows;
  p.rest.batch = d->batch - rows;
  p.bytes = (int64_t)rows * d->stride_b * elem_size(d->dtype);   // stride_b is a multiple of 16 bytes
  p.state = (int64_t)rows * d->heads * d->head_dim * d->head_dim;
  p.rstd = (int64_t)rows * d->heads * d->seqlen;
  return p;
}

template <typename T>
T* shifted(T* p, int64_t elements) { return p == nullptr ? nullptr : p + elements; }
const void* shifted_bytes(const void* p, int64_t bytes) {
  return p == nullptr ? nullptr : static_cast<const char*>(p) + bytes;
}
void* shifted_bytes(void* p, int64_t bytes) { return p == nullptr ? nullptr : static_cast<char*>(p) + bytes; }

// A workspace size that holds for the call as it runs: the larger of the two parts' (they run one after the other on
// one stream and share the workspace), or the whole batch's when it runs as one call.
template <typename F>
size_t over_parts(const la2_desc* d, F bytes_of) {
  const int rows = rows_of_first_call(d);
  if (rows == 0) return bytes_of(d);
  const RowParts p = row_parts(d, rows);
  const size_t a = bytes_of(&p.first), b = bytes_of(&p.rest);
  return a > b ? a : b;
}

struct ScanArgs {
  const void* x;
  const void* y;
  const void* z;
  void* w;
  const float* init = nullptr;   // start state [chains][d][d] (row = y feature) or nullptr
  bool init_tr = false;          // ... stored transposed
  float* fin = nullptr;          // state after the last block, or nullptr
  // chunk start states that an earlier call left in ITS workspace for the same (y, z) (or, if saved_tr, for
  // (z, y): the transposed states): the pre-pass is skipped.  Ignored when the plan has one chunk.
  const float* saved_states = nullptr;
  bool saved_tr = false;
  // Norm epilogue (forward scans): r of every position goes here, the output rows are scaled by it
  float* rstd = nullptr;
  float eps = 0.f;
  int rstd_stride = 0;   // positions per chain in rstd
  // packed sequences of different lengths: device array of batch + 1 position offsets, or nullptr
  const int32_t* cu = nullptr;
  // forward 16-bit scan of head_dim 128 in chunks: also accumulate the reverse local chunk states of the
  // (acc_y, x) pair into acc_states (ScanParams::acc_y)
  const void* acc_y = nullptr;
  float* acc_states = nullptr;
  // compact launch grid of a packed batch in chunks: the pair map (device), built by launch_varlen_map
  const int4* map = nullptr;
  // states at sequence ends that are not block boundaries (ScanParams::ragged_state; 16-bit half-block kernels)
  bool ragged_state = false;
};

// A problem cut into a few chunks (16-bit half-block kernels; dense or packed batch): no launch for the scan over the chunks'
// local states; every scan workgroup forms its own start state from them (ScanParams::self_prefix).  At that size
// the launches are a few microseconds each and run one after the other, so a dependent launch less is worth more
// than the few extra state reads (batch 4, H 16, n 2048, d 64, four chunks: each fold takes a 4.3 us launch away and
// adds 1-2 us to the prologue of the scan that follows; forward + backward 0.0871 -> 0.081-0.084 ms; the packed
// benchmark batch, whose longest sequences are cut in four: 69 -> 72 M tokens/s).
constexpr int kSelfPrefixMaxChunks = la2::kMaxPrefixTerms;   // a start state and the local states of chunks - 1 chunks
bool self_prefix(const la2_desc* d, const Plan& pl, const int32_t* cu) {
  (void)cu;   // packed batches too: every sequence's chunks have their own slots, a sequence of one chunk has none
  return pl.nchunks > 1 && pl.nchunks <= kSelfPrefixMaxChunks && is16(d->dtype) &&
         !wide(d->head_dim) && pl.chunk_tokens % 32 == 0 && g_scan_variant.load(std::memory_order_relaxed) != 1;
}

la2::ScanParams base_params(const la2_desc* d, const Plan& pl, const float* lambda, void* workspace,
                            const int32_t* cu = nullptr) {
  la2::ScanParams p{};
  p.cu_seqlens = cu;
  p.nscan = 1;
  p.state_transposed = 0;
  p.lambda = lambda;
  p.states = pl.nchunks > 1 ? reinterpret_cast<float*>(workspace) : nullptr;
  p.stride_b = d->stride_b; p.stride_h = d->stride_h; p.stride_n = d->stride_n;
  p.batch = d->batch; p.heads = d->heads; p.n = d->seqlen;
  p.nchunks = pl.nchunks;
  p.chunk_tokens = pl.chunk_tokens;
  p.variant = g_scan_variant.load(std::memory_order_relaxed);
  p.self_prefix = self_prefix(d, pl, cu) ? 1 : 0;
  return p;
}

// chunk start states of the scan with key-like operand y and value-like operand z -> workspace
// (local_ready: an earlier launch already left the chunks' local states there; only the scan over them runs)
la2_status run_prepass(const la2_desc* d, const Plan& pl, bool reverse, const void* y, const void* z,
                       const float* init, bool init_tr, const float* lambda, void* workspace, hipStream_t s,
                       const int32_t* cu = nullptr, bool local_ready = false, const int4* map = nullptr) {
  if (pl.nchunks <= 1) return LA2_OK;
  la2::ScanParams p = base_params(d, pl, lambda, workspace, cu);
  p.wg_map = map;
  p.wg_pairs = pl.wg_pairs;
  p.long_list = map != nullptr ? reinterpret_cast<const int32_t*>(map + pl.wg_pairs) : nullptr;
  p.nlong = pl.nlong;
  p.y[0] = y; p.z[0] = z;
  p.init[0] = init; p.init_transposed = init_tr ? 1 : 0;
  hipError_t e = local_ready          ? hipSuccess
                : wide(d->head_dim) ? la2::launch_scan_wide(d->dtype, d->head_dim, reverse, true, p, s)
                : is16(d->dtype)   ? la2::launch_chunk_states_bf16(d->dtype, d->head_dim, reverse, p, s)
                                   : la2::launch_chunk_states_f32(d->head_dim, reverse, p, s);
  if (e != hipSuccess) return LA2_ERR_LAUNCH;
  if (p.self_prefix) return LA2_OK;   // the scan's workgroups combine the local states themselves
  e = la2::launch_state_scan(d->head_dim, reverse, p, s);
  return e == hipSuccess ? LA2_OK : LA2_ERR_LAUNCH;
}

la2_status run_scan(const la2_desc* d, const Plan& pl, bool reverse, const ScanArgs& a, const float* lambda,
                    void* workspace, hipStream_t s) {
  const bool saved = a.saved_states != nullptr && pl.nchunks > 1;
  if (!saved) {
    la2_status st = run_prepass(d, pl, reverse, a.y, a.z, a.init, a.init_tr, lambda, workspace, s, a.cu, false, a.map);
    if (st != LA2_OK) return st;
  }
  la2::ScanParams p = base_params(d, pl, lambda, workspace, a.cu);
  p.wg_map = a.map;
  p.wg_pairs = pl.wg_pairs;
  if (saved) {
    p.states = const_cast<float*>(a.saved_states);   // read only
    p.state_transposed = a.saved_tr ? 1 : 0;
  }
  p.x[0] = a.x; p.y[0] = a.y; p.z[0] = a.z; p.w[0] = a.w;
  p.init[0] = a.init; p.init_transposed = a.init_tr ? 1 : 0;
  p.fin[0] = a.fin;
  p.rstd = a.rstd;
  p.eps = a.eps;
  p.rstd_stride = a.rstd_stride;
  p.acc_y = a.acc_y;
  p.acc_states = a.acc_states;
  p.ragged_state = a.ragged_state ? 1 : 0;
  hipError_t e = wide(d->head_dim) ? la2::launch_scan_wide(d->dtype, d->head_dim, reverse, false, p, s)
                : is16(d->dtype)   ? la2::launch_scan_bf16(d->dtype, d->head_dim, reverse, p, s)
                                   : la2::launch_scan_f32(d->head_dim, reverse, p, s);
  return e == hipSuccess ? LA2_OK : LA2_ERR_LAUNCH;
}

// Two reverse scans whose states are transposes of each other (scan 1's y, z are scan 0's z, y): one
// state pre-pass, one launch (16-bit path).
// (local_ready: the workspace already holds the chunks' local states, left there by the dQ scan's launch)
la2_status run_dual_reverse_scan(const la2_desc* d, const Plan& pl, const ScanArgs& a0, const ScanArgs& a1,
                                 const float* lambda, void* workspace, hipStream_t s, bool local_ready = false) {
  la2_status st = run_prepass(d, pl, true, a0.y, a0.z, a0.init, a0.init_tr, lambda, workspace, s, a0.cu, local_ready, a0.map);
  if (st != LA2_OK) return st;
  la2::ScanParams p = base_params(d, pl, lambda, workspace, a0.cu);
  p.wg_map = a0.map;
  p.wg_pairs = pl.wg_pairs;
  p.nscan = 2;
  p.state_transposed = 2;   // scan 1 starts from the transposed state
  p.init[0] = a0.init; p.init[1] = a1.init;
  p.init_transposed = (a0.init_tr ? 1 : 0) | (a1.init_tr ? 2 : 0);
  p.fin[0] = a0.fin; p.fin[1] = a1.fin;
  p.ragged_state = a0.ragged_state ? 1 : 0;
  p.x[0] = a0.x; p.y[0] = a0.y; p.z[0] = a0.z; p.w[0] = a0.w;
  p.x[1] = a1.x; p.y[1] = a1.y; p.z[1] = a1.z; p.w[1] = a1.w;
  const hipError_t e = wide(d->head_dim) ? la2::launch_scan_wide(d->dtype, d->head_dim, true, false, p, s)
                                         : la2::launch_scan_bf16(d->dtype, d->head_dim, true, p, s);
  return e == hipSuccess ? LA2_OK : LA2_ERR_LAUNCH;
}

// The state entry points split a sequence whose length is not a multiple of state_granule() into whole
// blocks (block kernels) and a tail (token recurrence) when the state beyond the tail is asked for.
// Their workspace: chunk states of whichever of the two plans needs more, then (backward only) one
// d x d fp32 state per chain that carries dKV from the tail to the block kernels.
struct StateWorkspace {
  size_t chunk_states;   // bytes, 256-byte multiple
  size_t total;
};

la2_desc whole_blocks(const la2_desc* d) {
  la2_desc w = *d;
  w.seqlen = d->seqlen - d->seqlen % state_granule(d);
  return w;
}

// Algorithm 2 on a sequence-chunked problem, 16-bit data, head_dim 64 / 128: the dQ scan's launch also forms the
// local dKV states of the chunks (its second wave group), so the backward pass keeps two sets of chunk states.
bool fuses_reverse_states(const la2_desc* d) {
  return is16(d->dtype) && !wide(d->head_dim) && g_scan_variant.load(std::memory_order_relaxed) != 1;
}

StateWorkspace state_workspace(const la2_desc* d, bool backward) {
  StateWorkspace w{make_plan(d).workspace * ((backward && fuses_reverse_states(d)) ? 2 : 1), 0};
  if (d->seqlen % state_granule(d) != 0) {
    const la2_desc wb = whole_blocks(d);
    const size_t other = make_plan(&wb).workspace;
    if (other > w.chunk_states) w.chunk_states = other;
  }
  w.chunk_states = (w.chunk_states + 255) & ~(size_t)255;
  w.total = w.chunk_states;
  if (backward && d->seqlen % state_granule(d) != 0)
    w.total += (size_t)d->batch * d->heads * d->head_dim * d->head_dim * sizeof(float);
  return w;
}

// Workspace bytes the backward of a segment needs: the hand-over state only when a gradient comes in at a
// ragged end.
size_t bwd_workspace_need(const la2_desc* d, bool has_d_kv_final) {
  const bool split = has_d_kv_final && d->seqlen % state_granule(d) != 0;
  return split ? state_workspace(d, true).total : make_plan(d).workspace * (fuses_reverse_states(d) ? 2 : 1);
}

la2::RecurParams recur_params(const la2_desc* d, const float* lambda, int t0, int t1, bool reverse) {
  la2::RecurParams p{};
  p.lambda = lambda;
  p.heads = d->heads;
  p.t0 = t0; p.t1 = t1;
  p.reverse = reverse ? 1 : 0;
  p.stride_b = d->stride_b; p.stride_h = d->stride_h; p.stride_n = d->stride_n;
  return p;
}

}  // namespace

extern "C" {

void la2_desc_dense(la2_desc* desc, int32_t batch, int32_t heads, int32_t seqlen, int32_t head_dim,
                    la2_dtype dtype) {
  if (desc == nullptr) return;
  desc->batch = batch;
  desc->heads = heads;
  desc->seqlen = seqlen;
  desc->head_dim = head_dim;
  desc->dtype = (int32_t)dtype;
  desc->reserved = 0;
  desc->stride_n = head_dim;
  desc->stride_h = (int64_t)seqlen * head_dim;
  desc->stride_b = (int64_t)heads * seqlen * head_dim;
}

size_t la2_workspace_bytes(const la2_desc* desc, int32_t op) {
  if (check_desc(desc) != LA2_OK) return 0;
  if (op == LA2_OP_FWD) return over_parts(desc, [](const la2_desc* d) { return make_plan(d).workspace; });
  if (op == LA2_OP_BWD)   // the chunk states of the dQ scan and (when its launch forms them) those of the dK / dV scan
    return over_parts(desc, [](const la2_desc* d) { return make_plan(d).workspace * (fuses_reverse_states(d) ? 2 : 1); });
  if (op == LA2_OP_FWD_STATE) return over_parts(desc, [](const la2_desc* d) { return state_workspace(d, false).total; });
  if (op == LA2_OP_BWD_STATE) return over_parts(desc, [](const la2_desc* d) { return state_workspace(d, true).total; });
  return 0;
}

la2_status la2_chunk_plan(const la2_desc* desc, int32_t* nchunks, int32_t* chunk_tokens) {
  const la2_status st = check_desc(desc);
  if (st != LA2_OK) return st;
  if (nchunks == nullptr || chunk_tokens == nullptr) return LA2_ERR_NULL;
  const Plan pl = make_plan(desc);
  *nchunks = pl.nchunks;
  *chunk_tokens = pl.chunk_tokens;
  return LA2_OK;
}

size_t la2_varlen_workspace_bytes(const la2_desc* desc, int64_t total_positions, int32_t op) {
  if (check_desc(desc) != LA2_OK || total_positions < 0) return 0;
  const Plan pl = make_plan_varlen(desc, total_positions);
  if (!plan_fits_a_grid(desc, pl)) return 0;
  if (op == LA2_OP_FWD) return pl.map_bytes + pl.workspace;
  if (op == LA2_OP_BWD) return pl.map_bytes + pl.workspace * (fuses_reverse_states(desc) ? 2 : 1);
  return 0;
}

int32_t la2_block_size(const la2_desc* desc) {
  if (check_desc(desc) != LA2_OK) return 0;
  // 16-bit, head_dim 64 / 128: the half-block scan kernel unless the full-block one is forced
  if (is16(desc->dtype) && !wide(desc->head_dim) && g_scan_variant.load(std::memory_order_relaxed) != 1) return 32;
  if (wide(desc->head_dim)) return is16(desc->dtype) ? 32 : 1;
  return block_size(desc);
}

void la2_set_chunk_tokens(int32_t tokens) { g_chunk_tokens_override.store(tokens > 0 ? tokens : 0); }

void la2_set_scan_variant(int32_t variant) { g_scan_variant.store((variant == 1 || variant == 2) ? variant : 0); }

}  // extern "C"

namespace {

// la2_fwd_state, and with rstd != nullptr the same with the Norm epilogue (eps validated by the caller)
// check_only: return after everything that can be refused has been checked, before the first launch.
la2_status fwd_state_one_call(const la2_desc* desc, const void* q, const void* k, const void* v, const float* lambda,
                              const float* kv_init, void* o, float* kv_final, float* rstd, float eps, void* workspace,
                              size_t workspace_bytes, void* hip_stream, bool check_only) {
  la2_status st = check_desc(desc);
  if (st != LA2_OK) return st;
  const int64_t chains = (int64_t)desc->batch * desc->heads;
  if (chains == 0) return LA2_OK;  // nothing to do
  if (!aligned(kv_init, 16) || !aligned(kv_final, 16)) return LA2_ERR_STRIDE_ALIGN;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  if (desc->seqlen == 0) {  // the state passes through
    if (kv_final == nullptr || check_only) return LA2_OK;
    return la2::launch_state_copy(kv_final, kv_init, chains * desc->head_dim * desc->head_dim, s) == hipSuccess
               ? LA2_OK : LA2_ERR_LAUNCH;
  }
  if (!q || !k || !v || !o || !lambda) return LA2_ERR_NULL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(lambda, 4) ||
      !aligned(rstd, 4))
    return LA2_ERR_STRIDE_ALIGN;
  // the Norm epilogue as a row pass of its own, in place, over positions [t0, t1): for fp32 rows that the token
  // recurrence wrote (fp32 storage: nothing is lost between the two passes)
  auto normalise_rows = [&](int t0, int t1) {
    const la2::NormBwdParams np{o, nullptr, rstd, o, desc->stride_b, desc->stride_h, desc->stride_n,
                                desc->batch, desc->heads, t1 - t0, t0, desc->seqlen};
    return la2::launch_norm_fwd_rows(desc->head_dim, desc->dtype, np, eps, s) == hipSuccess ? LA2_OK : LA2_ERR_LAUNCH;
  };
  if (wide(desc->head_dim) && !is16(desc->dtype)) {   // fp32 at head_dim 96 / 256: token by token
    if (check_only) return LA2_OK;
    la2::RecurParams r = recur_params(desc, lambda, 0, desc->seqlen, false);
    r.x[0] = q; r.y[0] = k; r.z[0] = v; r.w[0] = o;
    r.init[0] = kv_init;
    r.fin[0] = kv_final;
    if (la2::launch_recur(desc->head_dim, desc->dtype, desc->batch, 1, r, s) != hipSuccess) return LA2_ERR_LAUNCH;
    return rstd != nullptr ? normalise_rows(0, desc->seqlen) : LA2_OK;
  }
  const bool split = kv_final != nullptr && desc->seqlen % state_granule(desc) != 0;
  const la2_desc blocks = split ? whole_blocks(desc) : *desc;   // what the block kernels process
  const Plan pl = make_plan(&blocks);
  if (pl.workspace > 0 && (workspace == nullptr || workspace_bytes < pl.workspace)) return LA2_ERR_WORKSPACE;
  if (pl.workspace > 0 && !aligned(workspace, 256)) return LA2_ERR_WORKSPACE;
  if (check_only) return LA2_OK;
  if (blocks.seqlen > 0) {
    ScanArgs a{q, k, v, o};
    a.init = kv_init;
    a.fin = kv_final;
    a.ragged_state = kv_final != nullptr && ragged_end(desc);
    a.rstd = rstd;
    a.eps = eps;
    a.rstd_stride = desc->seqlen;
    st = run_scan(&blocks, pl, false, a, lambda, workspace, s);
    if (st != LA2_OK || !split) return st;
  }
  // fp32 data: the positions after the last whole block, token by token, from the state the blocks left
  la2::RecurParams r = recur_params(desc, lambda, blocks.seqlen, desc->seqlen, false);
  r.x[0] = q; r.y[0] = k; r.z[0] = v; r.w[0] = o;
  r.init[0] = blocks.seqlen > 0 ? kv_final : kv_init;
  r.fin[0] = kv_final;
  if (la2::launch_recur(desc->head_dim, desc->dtype, desc->batch, 1, r, s) != hipSuccess) return LA2_ERR_LAUNCH;
  return rstd != nullptr ? normalise_rows(blocks.seqlen, desc->seqlen) : LA2_OK;
}

// All dense forward entry points: one call, or two for a batch a little above a whole number of chains per compute
// unit (rows_of_first_call).  Everything either part would refuse is refused before the first launch.
la2_status fwd_state_impl(const la2_desc* desc, const void* q, const void* k, const void* v, const float* lambda,
                          const float* kv_init, void* o, float* kv_final, float* rstd, float eps, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  const int rows = check_desc(desc) == LA2_OK ? rows_of_first_call(desc) : 0;
  if (rows == 0)
    return fwd_state_one_call(desc, q, k, v, lambda, kv_init, o, kv_final, rstd, eps, workspace, workspace_bytes,
                              hip_stream, false);
  const RowParts p = row_parts(desc, rows);
  for (int pass = 0; pass < 2; ++pass) {   // 0: check both parts, 1: run them
    la2_status st = fwd_state_one_call(&p.first, q, k, v, lambda, kv_init, o, kv_final, rstd, eps, workspace,
                                       workspace_bytes, hip_stream, pass == 0);
    if (st != LA2_OK) return st;
    st = fwd_state_one_call(&p.rest, shifted_bytes(q, p.bytes), shifted_bytes(k, p.bytes), shifted_bytes(v, p.bytes),
                            lambda, shifted(kv_init, p.state), shifted_bytes(o, p.bytes), shifted(kv_final, p.state),
                            shifted(rstd, p.rstd), eps, workspace, workspace_bytes, hip_stream, pass == 0);
    if (st != LA2_OK) return st;
  }
  return LA2_OK;
}

}  // namespace

extern "C" {

la2_status la2_fwd_state(const la2_desc* desc, const void* q, const void* k, const void* v, const float* lambda,
                         const float* kv_init, void* o, float* kv_final, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  return fwd_state_impl(desc, q, k, v, lambda, kv_init, o, kv_final, nullptr, 0.f, workspace, workspace_bytes,
                        hip_stream);
}

la2_status la2_fwd(const la2_desc* desc, const void* q, const void* k, const void* v, const float* lambda,
                   void* o, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return la2_fwd_state(desc, q, k, v, lambda, nullptr, o, nullptr, workspace, workspace_bytes, hip_stream);
}

la2_status la2_fwd_noalloc(const la2_desc* desc, const void* q, const void* k, const void* v, const float* lambda,
                           void* o, void* hip_stream) {
  la2_status st = check_desc(desc);
  if (st != LA2_OK) return st;
  if ((int64_t)desc->batch * desc->heads * desc->seqlen == 0) return LA2_OK;  // nothing to do
  if (!q || !k || !v || !o || !lambda) return LA2_ERR_NULL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(lambda, 4))
    return LA2_ERR_STRIDE_ALIGN;
  size_t need = over_parts(desc, [](const la2_desc* d) { return make_plan(d).workspace; });
  bool one_call = false;
  if (need > (size_t)LA2_NOALLOC_SCRATCH_BYTES) {
    // chunk states beyond the built-in scratch.  A batch that would run as two calls (rows_of_first_call) and whose
    // second part asks for that much still runs as one call, which needs none.
    one_call = rows_of_first_call(desc) > 0;
    need = make_plan(desc).workspace;
    if (!one_call || need > (size_t)LA2_NOALLOC_SCRATCH_BYTES) return LA2_ERR_WORKSPACE;
  }
  void* ws = nullptr;
  if (need > 0) {
    st = scratch_on_current_device(&ws);
    if (st != LA2_OK) return st;
  }
  // Nothing in the scratch has to start at zero: the pre-pass writes the local state of every chunk that has a
  // successor and the state scan overwrites all of them, before the scan kernel reads any.
  if (one_call)
    return fwd_state_one_call(desc, q, k, v, lambda, nullptr, o, nullptr, nullptr, 0.f, ws, need, hip_stream, false);
  return fwd_state_impl(desc, q, k, v, lambda, nullptr, o, nullptr, nullptr, 0.f, ws, need, hip_stream);
}

}  // extern "C"

namespace {

// check_only: return after everything that can be refused has been checked, before the first launch.
la2_status bwd_saved_one_call(const la2_desc* desc, const void* q, const void* k, const void* v, const void* d_o,
                              const float* lambda, const float* kv_init, const float* d_kv_final, void* dq, void* dk,
                              void* dv, float* d_kv_init, const void* fwd_workspace, size_t fwd_workspace_bytes,
                              int32_t fwd_wrote_kv_final, void* workspace, size_t workspace_bytes, void* hip_stream,
                              bool check_only) {
  la2_status st = check_desc(desc);
  if (st == LA2_OK && !aligned(fwd_workspace, 256)) return LA2_ERR_WORKSPACE;
  if (st != LA2_OK) return st;
  const int64_t chains = (int64_t)desc->batch * desc->heads;
  if (chains == 0) return LA2_OK;  // nothing to do
  if (!aligned(kv_init, 16) || !aligned(d_kv_final, 16) || !aligned(d_kv_init, 16)) return LA2_ERR_STRIDE_ALIGN;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  if (desc->seqlen == 0) {  // the gradient of the state passes through
    if (d_kv_init == nullptr || check_only) return LA2_OK;
    return la2::launch_state_copy(d_kv_init, d_kv_final, chains * desc->head_dim * desc->head_dim, s) == hipSuccess
               ? LA2_OK : LA2_ERR_LAUNCH;
  }
  if (!q || !k || !v || !d_o || !dq || !dk || !dv || !lambda) return LA2_ERR_NULL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(d_o, 16) || !aligned(dq, 16) ||
      !aligned(dk, 16) || !aligned(dv, 16) || !aligned(lambda, 4))
    return LA2_ERR_STRIDE_ALIGN;
  if (wide(desc->head_dim) && !is16(desc->dtype)) {   // fp32 at head_dim 96 / 256: token by token
    if (check_only) return LA2_OK;
    la2::RecurParams f = recur_params(desc, lambda, 0, desc->seqlen, false);
    f.x[0] = d_o; f.y[0] = v; f.z[0] = k; f.w[0] = dq;      // dq_t = do_t KV_t^T: the (V, K) state is KV^T
    f.init[0] = kv_init;
    f.init_transposed = 1;
    if (la2::launch_recur(desc->head_dim, desc->dtype, desc->batch, 1, f, s) != hipSuccess) return LA2_ERR_LAUNCH;
    la2::RecurParams r = recur_params(desc, lambda, 0, desc->seqlen, true);
    r.x[0] = k; r.y[0] = q; r.z[0] = d_o; r.w[0] = dv;     // dv_t = k_t G_t, G = sum q^T do
    r.x[1] = v; r.y[1] = d_o; r.z[1] = q; r.w[1] = dk;     // dk_t = v_t G_t^T
    r.init[0] = d_kv_final; r.init[1] = d_kv_final;
    r.init_transposed = 2;
    r.fin[0] = d_kv_init;
    return la2::launch_recur(desc->head_dim, desc->dtype, desc->batch, 2, r, s) == hipSuccess ? LA2_OK
                                                                                               : LA2_ERR_LAUNCH;
  }
  // With a gradient coming in at the end of a sequence that does not end on a block boundary, the reverse
  // pass runs the tail token by token first and hands dKV to the block kernels through the workspace.
  const bool split = d_kv_final != nullptr && desc->seqlen % state_granule(desc) != 0;
  const la2_desc blocks = split ? whole_blocks(desc) : *desc;   // what the reverse block kernels process
  const Plan pl = make_plan(desc), pl_rev = make_plan(&blocks);
  // Algorithm 2, first loop (ascending, running KV):  dQ = [(dO V^T) * M] K + Lambda dO KV^T
  // (forward scan of (dO, V, K); its state is KV^T, so a start state KV is read transposed)
  ScanArgs for_dq{d_o, v, k, dq};
  for_dq.init = kv_init;
  for_dq.init_tr = true;
  // The forward pass's chunk start states are those of the (K, V) scan: this scan's, transposed.  Only when
  // that call cut the sequence into the same chunks as this one does (a forward call that handed out kv_final
  // for a ragged length planned its chunks for the whole blocks only); otherwise they are recomputed.
  if (fwd_workspace != nullptr && pl.nchunks > 1) {
    const bool fwd_split = fwd_wrote_kv_final != 0 && desc->seqlen % state_granule(desc) != 0;
    const la2_desc fwd_blocks = fwd_split ? whole_blocks(desc) : *desc;
    const Plan pl_fwd = make_plan(&fwd_blocks);
    if (pl_fwd.nchunks == pl.nchunks && pl_fwd.chunk_tokens == pl.chunk_tokens) {
      if (fwd_workspace_bytes < pl_fwd.workspace) return LA2_ERR_WORKSPACE;   // not the buffer of that call
      for_dq.saved_states = reinterpret_cast<const float*>(fwd_workspace);
      for_dq.saved_tr = true;
    }
  }
  // Sequence chunks, 16-bit data, head_dim 64 / 128: the dQ scan's launch also forms the local dKV states of the
  // chunks (from dO, which it streams anyway, and Q), so the second loop needs no pass of its own over Q and dO
  // before it can start its chunks.  Those states live behind the dQ scan's own chunk states in the workspace
  // (or at its start when the dQ scan reads the forward call's).  Not when the reverse scans run on the whole
  // blocks only (their chunks may then differ from the dQ scan's).
  const bool fuse = !split && pl.nchunks > 1 && fuses_reverse_states(desc);
  const StateWorkspace sw = state_workspace(desc, true);
  const size_t need = split ? sw.total : fuse ? pl.workspace * (for_dq.saved_states != nullptr ? 1 : 2) : pl.workspace;
  if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return LA2_ERR_WORKSPACE;
  if (need > 0 && !aligned(workspace, 256)) return LA2_ERR_WORKSPACE;
  if (check_only) return LA2_OK;
  float* handoff = split ? reinterpret_cast<float*>(static_cast<char*>(workspace) + sw.chunk_states) : nullptr;
  void* rev_workspace = workspace;
  if (fuse) {
    if (for_dq.saved_states == nullptr) rev_workspace = static_cast<char*>(workspace) + pl.workspace;
    for_dq.acc_y = q;
    for_dq.acc_states = reinterpret_cast<float*>(rev_workspace);
  }
  st = run_scan(desc, pl, false, for_dq, lambda, workspace, s);
  if (st != LA2_OK) return st;
  // Algorithm 2, second loop (descending, running dKV):
  //   dV = [(Q K^T) * M]^T dO + decay(K) dKV        reverse scan of (K, Q, dO), state dKV = Q^T dO
  //   dK = [(dO V^T) * M]^T Q + decay(V) dKV^T      reverse scan of (V, dO, Q), state dKV^T
  // dKV starts from the gradient of the final state and ends as the gradient of the start state.
  const float* rev_init = d_kv_final;
  if (split) {
    la2::RecurParams r = recur_params(desc, lambda, blocks.seqlen, desc->seqlen, true);
    r.x[0] = k; r.y[0] = q; r.z[0] = d_o; r.w[0] = dv;     // dv_t = k_t G_t, G = sum q^T do
    r.x[1] = v; r.y[1] = d_o; r.z[1] = q; r.w[1] = dk;     // dk_t = v_t G_t^T
    r.init[0] = d_kv_final; r.init[1] = d_kv_final;
    r.init_transposed = 2;
    r.fin[0] = blocks.seqlen > 0 ? handoff : d_kv_init;
    if (la2::launch_recur(desc->head_dim, desc->dtype, desc->batch, 2, r, s) != hipSuccess)
      return LA2_ERR_LAUNCH;
    if (blocks.seqlen == 0) return LA2_OK;
    rev_init = handoff;
  }
  ScanArgs for_dv{k, q, d_o, dv}, for_dk{v, d_o, q, dk};
  for_dv.init = rev_init;
  for_dv.fin = d_kv_init;
  for_dk.init = rev_init;
  for_dk.init_tr = true;
  for_dv.ragged_state = for_dk.ragged_state = d_kv_final != nullptr && ragged_end(desc);
  if (is16(desc->dtype))
    return run_dual_reverse_scan(&blocks, pl_rev, for_dv, for_dk, lambda, rev_workspace, s, /*local_ready=*/fuse);
  st = run_scan(&blocks, pl_rev, true, for_dv, lambda, workspace, s);
  if (st != LA2_OK) return st;
  return run_scan(&blocks, pl_rev, true, for_dk, lambda, workspace, s);
}

}  // namespace

extern "C" {

// One call, or two for a batch a little above a whole number of chains per compute unit (rows_of_first_call), each
// part with its own states; the forward call's workspace holds the chunk states of its second part, which is the
// part whose backward reads them.
la2_status la2_bwd_saved(const la2_desc* desc, const void* q, const void* k, const void* v, const void* d_o,
                         const float* lambda, const float* kv_init, const float* d_kv_final, void* dq, void* dk,
                         void* dv, float* d_kv_init, const void* fwd_workspace, size_t fwd_workspace_bytes,
                         int32_t fwd_wrote_kv_final, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (check_desc(desc) == LA2_OK && !aligned(fwd_workspace, 256)) return LA2_ERR_WORKSPACE;
  const int rows = check_desc(desc) == LA2_OK ? rows_of_first_call(desc) : 0;
  if (rows == 0)
    return bwd_saved_one_call(desc, q, k, v, d_o, lambda, kv_init, d_kv_final, dq, dk, dv, d_kv_init, fwd_workspace,
                              fwd_workspace_bytes, fwd_wrote_kv_final, workspace, workspace_bytes, hip_stream, false);
  const RowParts p = row_parts(desc, rows);
  for (int pass = 0; pass < 2; ++pass) {   // 0: check both parts, 1: run them
    // the first part never reads the forward call's workspace: should its plan cut (fewer chains than units when the
    // heads do not divide them), its chunk states were overwritten there by the second part's
    la2_status st = bwd_saved_one_call(&p.first, q, k, v, d_o, lambda, kv_init, d_kv_final, dq, dk, dv, d_kv_init,
                                       nullptr, 0, 0, workspace, workspace_bytes, hip_stream, pass == 0);
    if (st != LA2_OK) return st;
    st = bwd_saved_one_call(&p.rest, shifted_bytes(q, p.bytes), shifted_bytes(k, p.bytes), shifted_bytes(v, p.bytes),
                            shifted_bytes(d_o, p.bytes), lambda, shifted(kv_init, p.state), shifted(d_kv_final, p.state),
                            shifted_bytes(dq, p.bytes), shifted_bytes(dk, p.bytes), shifted_bytes(dv, p.bytes),
                            shifted(d_kv_init, p.state), fwd_workspace, fwd_workspace_bytes, fwd_wrote_kv_final,
                            workspace, workspace_bytes, hip_stream, pass == 0);
    if (st != LA2_OK) return st;
  }
  return LA2_OK;
}

la2_status la2_bwd_state(const la2_desc* desc, const void* q, const void* k, const void* v, const void* d_o,
                         const float* lambda, const float* kv_init, const float* d_kv_final, void* dq, void* dk,
                         void* dv, float* d_kv_init, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return la2_bwd_saved(desc, q, k, v, d_o, lambda, kv_init, d_kv_final, dq, dk, dv, d_kv_init, nullptr, 0, 0,
                       workspace, workspace_bytes, hip_stream);
}

la2_status la2_bwd(const la2_desc* desc, const void* q, const void* k, const void* v, const void* d_o,
                   const float* lambda, void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                   void* hip_stream) {
  return la2_bwd_saved(desc, q, k, v, d_o, lambda, nullptr, nullptr, dq, dk, dv, nullptr, nullptr, 0, 0, workspace,
                       workspace_bytes, hip_stream);
}

la2_status la2_fwd_state_norm(const la2_desc* desc, const void* q, const void* k, const void* v,
                              const float* lambda, const float* kv_init, float eps, void* o, float* rstd,
                              float* kv_final, void* workspace, size_t workspace_bytes, void* hip_stream) {
  la2_status st = check_desc(desc);
  if (st != LA2_OK) return st;
  if (!(eps >= 0.f) || eps > 3.0e38f) return LA2_ERR_VALUE;
  if ((int64_t)desc->batch * desc->heads * desc->seqlen != 0 && rstd == nullptr) return LA2_ERR_NULL;
  return fwd_state_impl(desc, q, k, v, lambda, kv_init, o, kv_final, rstd, eps, workspace, workspace_bytes,
                        hip_stream);
}

la2_status la2_fwd_norm(const la2_desc* desc, const void* q, const void* k, const void* v, const float* lambda,
                        float eps, void* o, float* rstd, void* workspace, size_t workspace_bytes,
                        void* hip_stream) {
  return la2_fwd_state_norm(desc, q, k, v, lambda, nullptr, eps, o, rstd, nullptr, workspace, workspace_bytes,
                            hip_stream);
}

la2_status la2_bwd_state_norm(const la2_desc* desc, const void* q, const void* k, const void* v, const void* o,
                              const float* rstd, const void* d_o, const float* lambda, const float* kv_init,
                              const float* d_kv_final, void* d_u, void* dq, void* dk, void* dv, float* d_kv_init,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  la2_status st = check_desc(desc);
  if (st != LA2_OK) return st;
  if ((int64_t)desc->batch * desc->heads * desc->seqlen == 0)   // no rows: only the state's gradient passes through
    return la2_bwd_state(desc, q, k, v, d_o, lambda, kv_init, d_kv_final, dq, dk, dv, d_kv_init, workspace,
                         workspace_bytes, hip_stream);
  if (!q || !k || !v || !o || !rstd || !d_o || !d_u || !dq || !dk || !dv || !lambda) return LA2_ERR_NULL;
  if (!aligned(o, 16) || !aligned(d_o, 16) || !aligned(d_u, 16) || !aligned(rstd, 4)) return LA2_ERR_STRIDE_ALIGN;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(dq, 16) || !aligned(dk, 16) ||
      !aligned(dv, 16) || !aligned(lambda, 4) || !aligned(kv_init, 16) || !aligned(d_kv_final, 16) ||
      !aligned(d_kv_init, 16))
    return LA2_ERR_STRIDE_ALIGN;
  const bool has_final = d_kv_final != nullptr;
  const size_t need = over_parts(desc, [has_final](const la2_desc* d) { return bwd_workspace_need(d, has_final); });
  if (need > 0 && (workspace == nullptr || workspace_bytes < need || !aligned(workspace, 256)))
    return LA2_ERR_WORKSPACE;
  const la2::NormBwdParams np{o, d_o, rstd, d_u, desc->stride_b, desc->stride_h, desc->stride_n,
                              desc->batch, desc->heads, desc->seqlen, 0, desc->seqlen};
  if (la2::launch_norm_bwd_rows(desc->head_dim, desc->dtype, np,
                                reinterpret_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return LA2_ERR_LAUNCH;
  return la2_bwd_state(desc, q, k, v, d_u, lambda, kv_init, d_kv_final, dq, dk, dv, d_kv_init, workspace,
                       workspace_bytes, hip_stream);
}

la2_status la2_bwd_norm(const la2_desc* desc, const void* q, const void* k, const void* v, const void* o,
                        const float* rstd, const void* d_o, const float* lambda, void* d_u, void* dq, void* dk,
                        void* dv, void* workspace, size_t workspace_bytes, void* hip_stream) {
  la2_status st = check_desc(desc);
  if (st != LA2_OK) return st;
  if ((int64_t)desc->batch * desc->heads * desc->seqlen == 0) return LA2_OK;  // nothing to do
  return la2_bwd_state_norm(desc, q, k, v, o, rstd, d_o, lambda, nullptr, nullptr, d_u, dq, dk, dv, nullptr,
                            workspace, workspace_bytes, hip_stream);
}

}  // extern "C"

namespace {
// Packed batches with state hand-over run on the 16-bit half-block kernels (head_dim 64 / 128) only: they are the
// ones that form a state at a sequence end that is no block boundary.
la2_status packed_state_supported(const la2_desc* d) {
  if (!is16(d->dtype)) return LA2_ERR_DTYPE;
  if (wide(d->head_dim)) return LA2_ERR_SHAPE;
  return LA2_OK;
}

// la2_fwd_varlen and la2_fwd_varlen_state, and with rstd != nullptr la2_fwd_varlen_norm (eps validated by the caller)
la2_status fwd_varlen_impl(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions, const void* q,
                           const void* k, const void* v, const float* lambda, const float* kv_init, void* o,
                           float* kv_final, float* rstd, float eps, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
  la2_status st = check_desc(desc);
  if (st != LA2_OK) return st;
  if (total_positions < 0) return LA2_ERR_SHAPE;
  if (wide(desc->head_dim) && !is16(desc->dtype)) return LA2_ERR_DTYPE;   // packed batches at 96 / 256: 16-bit only
  const bool with_state = kv_init != nullptr || kv_final != nullptr;
  if (with_state) {   // the half-block kernels' ragged-end states
    st = packed_state_supported(desc);
    if (st != LA2_OK) return st;
    if (!aligned(kv_init, 16) || !aligned(kv_final, 16)) return LA2_ERR_STRIDE_ALIGN;
  }
  if ((int64_t)desc->batch * desc->heads * desc->seqlen == 0) {
    if (kv_final == nullptr || (int64_t)desc->batch * desc->heads == 0) return LA2_OK;  // nothing to do
    // sequences without positions: the states pass through
    return la2::launch_state_copy(kv_final, kv_init, (int64_t)desc->batch * desc->heads * desc->head_dim * desc->head_dim,
                                  reinterpret_cast<hipStream_t>(hip_stream)) == hipSuccess ? LA2_OK : LA2_ERR_LAUNCH;
  }
  if (!cu_seqlens || !q || !k || !v || !o || !lambda) return LA2_ERR_NULL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(lambda, 4) ||
      !aligned(cu_seqlens, 4))
    return LA2_ERR_STRIDE_ALIGN;
  const Plan pl = make_plan_varlen(desc, total_positions);
  if (!plan_fits_a_grid(desc, pl)) return LA2_ERR_SHAPE;
  const size_t need = pl.map_bytes + pl.workspace;
  if (need > 0 && (workspace == nullptr || workspace_bytes < need || !aligned(workspace, 256)))
    return LA2_ERR_WORKSPACE;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  ScanArgs a{q, k, v, o};
  a.cu = cu_seqlens;
  a.rstd = rstd;   // packed layout [heads][total_positions]
  a.eps = eps;
  a.rstd_stride = (int)total_positions;
  a.init = kv_init;
  a.fin = kv_final;
  a.ragged_state = with_state;
  if (pl.wg_pairs > 0) {   // the pair map of the compact grid, in front of the states
    la2::ScanParams mp = base_params(desc, pl, lambda, nullptr, cu_seqlens);
    mp.wg_pairs = pl.wg_pairs;
    mp.nlong = pl.nlong;
    int4* map = reinterpret_cast<int4*>(workspace);
    if (la2::launch_varlen_map(mp, map, reinterpret_cast<int32_t*>(map + pl.wg_pairs), pl.wg_slots, s) != hipSuccess)
      return LA2_ERR_LAUNCH;
    a.map = map;
  }
  return run_scan(desc, pl, false, a, lambda, static_cast<char*>(workspace) + pl.map_bytes, s);
}

// la2_bwd_varlen and la2_bwd_varlen_state
la2_status bwd_varlen_impl(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions, const void* q,
                           const void* k, const void* v, const void* d_o, const float* lambda, const float* kv_init,
                           const float* d_kv_final, void* dq, void* dk, void* dv, float* d_kv_init, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
  la2_status st = check_desc(desc);
  if (st != LA2_OK) return st;
  if (total_positions < 0) return LA2_ERR_SHAPE;
  if (wide(desc->head_dim) && !is16(desc->dtype)) return LA2_ERR_DTYPE;   // as la2_fwd_varlen
  const bool with_state = kv_init != nullptr || d_kv_final != nullptr || d_kv_init != nullptr;
  if (with_state) {
    st = packed_state_supported(desc);
    if (st != LA2_OK) return st;
    if (!aligned(kv_init, 16) || !aligned(d_kv_final, 16) || !aligned(d_kv_init, 16)) return LA2_ERR_STRIDE_ALIGN;
  }
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  if ((int64_t)desc->batch * desc->heads * desc->seqlen == 0) {
    if (d_kv_init == nullptr || (int64_t)desc->batch * desc->heads == 0) return LA2_OK;  // nothing to do
    // sequences without positions: the gradient of the state passes through
    return la2::launch_state_copy(d_kv_init, d_kv_final, (int64_t)desc->batch * desc->heads * desc->head_dim * desc->head_dim,
                                  s) == hipSuccess ? LA2_OK : LA2_ERR_LAUNCH;
  }
  if (!cu_seqlens || !q || !k || !v || !d_o || !dq || !dk || !dv || !lambda) return LA2_ERR_NULL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(d_o, 16) || !aligned(dq, 16) ||
      !aligned(dk, 16) || !aligned(dv, 16) || !aligned(lambda, 4) || !aligned(cu_seqlens, 4))
    return LA2_ERR_STRIDE_ALIGN;
  const Plan pl = make_plan_varlen(desc, total_positions);
  if (!plan_fits_a_grid(desc, pl)) return LA2_ERR_SHAPE;
  // as la2_bwd: with sequence chunks the dQ scan's launch forms the local dKV states behind its own chunk states
  const bool fuse = pl.nchunks > 1 && fuses_reverse_states(desc);
  const size_t need = pl.map_bytes + pl.workspace * (fuse ? 2 : 1);
  if (need > 0 && (workspace == nullptr || workspace_bytes < need || !aligned(workspace, 256)))
    return LA2_ERR_WORKSPACE;
  // the three scans of la2_bwd, each chain a sequence of its own length; states as in la2_bwd_state
  ScanArgs for_dq{d_o, v, k, dq}, for_dv{k, q, d_o, dv}, for_dk{v, d_o, q, dk};
  for_dq.cu = for_dv.cu = for_dk.cu = cu_seqlens;
  for_dq.init = kv_init;
  for_dq.init_tr = true;
  for_dv.init = d_kv_final;
  for_dv.fin = d_kv_init;
  for_dk.init = d_kv_final;
  for_dk.init_tr = true;
  for_dv.ragged_state = for_dk.ragged_state = with_state;   // the forward dQ scan hands out no state
  if (pl.wg_pairs > 0) {   // the pair map of the compact grid, in front of the states
    la2::ScanParams mp = base_params(desc, pl, lambda, nullptr, cu_seqlens);
    mp.wg_pairs = pl.wg_pairs;
    mp.nlong = pl.nlong;
    int4* map = reinterpret_cast<int4*>(workspace);
    if (la2::launch_varlen_map(mp, map, reinterpret_cast<int32_t*>(map + pl.wg_pairs), pl.wg_slots, s) != hipSuccess)
      return LA2_ERR_LAUNCH;
    for_dq.map = for_dv.map = for_dk.map = map;
  }
  workspace = static_cast<char*>(workspace) + pl.map_bytes;   // the states
  void* rev_workspace = fuse ? static_cast<char*>(workspace) + pl.workspace : workspace;
  if (fuse) {
    for_dq.acc_y = q;
    for_dq.acc_states = reinterpret_cast<float*>(rev_workspace);
  }
  st = run_scan(desc, pl, false, for_dq, lambda, workspace, s);
  if (st != LA2_OK) return st;
  if (is16(desc->dtype)) return run_dual_reverse_scan(desc, pl, for_dv, for_dk, lambda, rev_workspace, s, fuse);
  st = run_scan(desc, pl, true, for_dv, lambda, workspace, s);
  if (st != LA2_OK) return st;
  return run_scan(desc, pl, true, for_dk, lambda, workspace, s);
}
}  // namespace

extern "C" {

la2_status la2_fwd_varlen(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions, const void* q,
                          const void* k, const void* v, const float* lambda, void* o, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  return fwd_varlen_impl(desc, cu_seqlens, total_positions, q, k, v, lambda, nullptr, o, nullptr, nullptr, 0.f,
                         workspace, workspace_bytes, hip_stream);
}

la2_status la2_fwd_varlen_state(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions,
                                const void* q, const void* k, const void* v, const float* lambda,
                                const float* kv_init, void* o, float* kv_final, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
  return fwd_varlen_impl(desc, cu_seqlens, total_positions, q, k, v, lambda, kv_init, o, kv_final, nullptr, 0.f,
                         workspace, workspace_bytes, hip_stream);
}

la2_status la2_bwd_varlen_state(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions,
                                const void* q, const void* k, const void* v, const void* d_o, const float* lambda,
                                const float* kv_init, const float* d_kv_final, void* dq, void* dk, void* dv,
                                float* d_kv_init, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return bwd_varlen_impl(desc, cu_seqlens, total_positions, q, k, v, d_o, lambda, kv_init, d_kv_final, dq, dk, dv,
                         d_kv_init, workspace, workspace_bytes, hip_stream);
}

la2_status la2_fwd_varlen_norm(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions,
                               const void* q, const void* k, const void* v, const float* lambda, float eps, void* o,
                               float* rstd, void* workspace, size_t workspace_bytes, void* hip_stream) {
  la2_status st = check_desc(desc);
  if (st != LA2_OK) return st;
  if (!(eps >= 0.f) || eps > 3.0e38f) return LA2_ERR_VALUE;
  if ((int64_t)desc->batch * desc->heads * desc->seqlen == 0) return LA2_OK;  // nothing to do
  // r is laid out [heads][total_positions]: the total has to be the packed tensors' real extent here
  if (total_positions <= 0 || total_positions > 0x7FFFFFFF) return LA2_ERR_SHAPE;
  if (rstd == nullptr) return LA2_ERR_NULL;
  if (!aligned(rstd, 4)) return LA2_ERR_STRIDE_ALIGN;
  return fwd_varlen_impl(desc, cu_seqlens, total_positions, q, k, v, lambda, nullptr, o, nullptr, rstd, eps, workspace,
                         workspace_bytes, hip_stream);
}

la2_status la2_bwd_varlen_norm(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions,
                               const void* q, const void* k, const void* v, const void* o, const float* rstd,
                               const void* d_o, const float* lambda, void* d_u, void* dq, void* dk, void* dv,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
  la2_status st = check_desc(desc);
  if (st != LA2_OK) return st;
  if (wide(desc->head_dim) && !is16(desc->dtype)) return LA2_ERR_DTYPE;   // as la2_fwd_varlen
  if ((int64_t)desc->batch * desc->heads * desc->seqlen == 0) return LA2_OK;  // nothing to do
  if (total_positions <= 0 || total_positions > 0x7FFFFFFF) return LA2_ERR_SHAPE;
  if (!cu_seqlens || !q || !k || !v || !o || !rstd || !d_o || !d_u || !dq || !dk || !dv || !lambda) return LA2_ERR_NULL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(d_o, 16) ||
      !aligned(d_u, 16) || !aligned(dq, 16) || !aligned(dk, 16) || !aligned(dv, 16) || !aligned(lambda, 4) ||
      !aligned(rstd, 4) || !aligned(cu_seqlens, 4))
    return LA2_ERR_STRIDE_ALIGN;
  const size_t need = la2_varlen_workspace_bytes(desc, total_positions, LA2_OP_BWD);
  if (need > 0 && (workspace == nullptr || workspace_bytes < need || !aligned(workspace, 256)))
    return LA2_ERR_WORKSPACE;
  // the row pass over all packed positions that belong to a sequence (one "chain" per head), then Algorithm 2 on d_u
  la2::NormBwdParams np{o, d_o, rstd, d_u, 0, desc->stride_h, desc->stride_n, 1, desc->heads, (int32_t)total_positions,
                        0, (int32_t)total_positions};
  np.bounds = cu_seqlens;
  np.nbounds = desc->batch;
  if (la2::launch_norm_bwd_rows(desc->head_dim, desc->dtype, np, reinterpret_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return LA2_ERR_LAUNCH;
  return la2_bwd_varlen(desc, cu_seqlens, total_positions, q, k, v, d_u, lambda, dq, dk, dv, workspace, workspace_bytes,
                        hip_stream);
}

la2_status la2_bwd_varlen(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions, const void* q,
                          const void* k, const void* v, const void* d_o, const float* lambda, void* dq, void* dk,
                          void* dv, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return bwd_varlen_impl(desc, cu_seqlens, total_positions, q, k, v, d_o, lambda, nullptr, nullptr, dq, dk, dv,
                         nullptr, workspace, workspace_bytes, hip_stream);
}

la2_status la2_left_product_fwd(const la2_desc* desc, const void* q, const void* k, const void* v,
                                const float* lambda, void* o, void* hip_stream) {
  la2_status st = check_desc(desc);
  if (st != LA2_OK) return st;
  if (desc->dtype != LA2_BF16) return LA2_ERR_DTYPE;
  if (wide(desc->head_dim)) return LA2_ERR_SHAPE;   // comparison kernel: head_dim 64 and 128
  if ((int64_t)desc->batch * desc->heads * desc->seqlen == 0) return LA2_OK;  // nothing to do
  if (!q || !k || !v || !o || !lambda) return LA2_ERR_NULL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(lambda, 4))
    return LA2_ERR_STRIDE_ALIGN;
  Plan one{1, desc->seqlen, 0};
  la2::ScanParams p = base_params(desc, one, lambda, nullptr);
  p.x[0] = q; p.y[0] = k; p.z[0] = v; p.w[0] = o;
  return la2::launch_left_product_bf16(desc->head_dim, false, p, reinterpret_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? LA2_OK : LA2_ERR_LAUNCH;
}

la2_status la2_left_product_bwd(const la2_desc* desc, const void* q, const void* k, const void* v, const void* d_o,
                                const float* lambda, void* dq, void* dk, void* dv, void* hip_stream) {
  la2_status st = check_desc(desc);
  if (st != LA2_OK) return st;
  if (desc->dtype != LA2_BF16) return LA2_ERR_DTYPE;
  if (wide(desc->head_dim)) return LA2_ERR_SHAPE;   // comparison kernel: head_dim 64 and 128
  if ((int64_t)desc->batch * desc->heads * desc->seqlen == 0) return LA2_OK;  // nothing to do
  if (!q || !k || !v || !d_o || !dq || !dk || !dv || !lambda) return LA2_ERR_NULL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(d_o, 16) || !aligned(dq, 16) ||
      !aligned(dk, 16) || !aligned(dv, 16) || !aligned(lambda, 4))
    return LA2_ERR_STRIDE_ALIGN;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  Plan one{1, desc->seqlen, 0};
  la2::ScanParams p = base_params(desc, one, lambda, nullptr);
  // the three gradients of Sec. 3.2.2 as masked products over all earlier (dQ) or all later (dK, dV) positions
  p.x[0] = d_o; p.y[0] = v; p.z[0] = k; p.w[0] = dq;       // dQ = [(dO V^T) * M] K
  if (la2::launch_left_product_bf16(desc->head_dim, false, p, s) != hipSuccess) return LA2_ERR_LAUNCH;
  p.x[0] = k; p.y[0] = q; p.z[0] = d_o; p.w[0] = dv;       // dV = [(Q K^T) * M]^T dO = [(K Q^T) * M^T] dO
  if (la2::launch_left_product_bf16(desc->head_dim, true, p, s) != hipSuccess) return LA2_ERR_LAUNCH;
  p.x[0] = v; p.y[0] = d_o; p.z[0] = q; p.w[0] = dk;       // dK = [(dO V^T) * M]^T Q = [(V dO^T) * M^T] Q
  return la2::launch_left_product_bf16(desc->head_dim, true, p, s) == hipSuccess ? LA2_OK : LA2_ERR_LAUNCH;
}

}  // extern "C"

namespace {
la2_status decode_step_impl(int32_t batch, int32_t heads, int32_t head_dim, int32_t qkv_dtype, const void* q,
                            const void* k, const void* v, const float* lambda, float* kv_state, void* o, bool norm,
                            float eps, void* hip_stream) {
  if (qkv_dtype != LA2_F32 && !is16(qkv_dtype)) return LA2_ERR_DTYPE;
  if (batch < 0 || heads < 0 || !supported_head_dim(head_dim)) return LA2_ERR_SHAPE;
  if ((int64_t)batch * heads > (int64_t)1 << 24) return LA2_ERR_SHAPE;
  if (norm && (!(eps >= 0.f) || eps > 3.0e38f)) return LA2_ERR_VALUE;
  if ((int64_t)batch * heads == 0) return LA2_OK;  // nothing to do
  if (!q || !k || !v || !lambda || !kv_state || !o) return LA2_ERR_NULL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(kv_state, 16) ||
      !aligned(lambda, 4))
    return LA2_ERR_STRIDE_ALIGN;
  hipError_t e = la2::launch_decode(batch, heads, head_dim, qkv_dtype, q, k, v, lambda, kv_state, o, norm, eps,
                                    reinterpret_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? LA2_OK : LA2_ERR_LAUNCH;
}
}  // namespace

extern "C" {

la2_status la2_decode_step(int32_t batch, int32_t heads, int32_t head_dim, int32_t qkv_dtype, const void* q,
                           const void* k, const void* v, const float* lambda, float* kv_state, void* o,
                           void* hip_stream) {
  return decode_step_impl(batch, heads, head_dim, qkv_dtype, q, k, v, lambda, kv_state, o, false, 0.f, hip_stream);
}

la2_status la2_decode_step_norm(int32_t batch, int32_t heads, int32_t head_dim, int32_t qkv_dtype, const void* q,
                                const void* k, const void* v, const float* lambda, float* kv_state, float eps,
                                void* o, void* hip_stream) {
  return decode_step_impl(batch, heads, head_dim, qkv_dtype, q, k, v, lambda, kv_state, o, true, eps, hip_stream);
}

}  // extern "C"

namespace {
// la2_decode_multi, and with rstd != nullptr the same with the Norm epilogue on every output row
la2_status decode_multi_impl(int32_t batch, int32_t heads, int32_t head_dim, int32_t ntokens, int32_t qkv_dtype,
                             const void* q, const void* k, const void* v, const float* lambda, float* kv_state,
                             float* rstd, float eps, void* o, void* hip_stream) {
  if (qkv_dtype != LA2_F32 && !is16(qkv_dtype)) return LA2_ERR_DTYPE;
  if (batch < 0 || heads < 0 || ntokens < 0 || !supported_head_dim(head_dim)) return LA2_ERR_SHAPE;
  if ((int64_t)batch * heads > (int64_t)1 << 24 || ntokens > 65536) return LA2_ERR_SHAPE;
  if ((int64_t)batch * heads * ntokens == 0) return LA2_OK;  // nothing to do
  if (!q || !k || !v || !lambda || !kv_state || !o) return LA2_ERR_NULL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(kv_state, 16) ||
      !aligned(lambda, 4) || !aligned(rstd, 4))
    return LA2_ERR_STRIDE_ALIGN;
  la2_desc d;
  la2_desc_dense(&d, batch, heads, ntokens, head_dim, (la2_dtype)qkv_dtype);
  // A run of at least one whole block goes through the scan kernels (the state in place: a workgroup reads its
  // chain's start state before it writes the final one; fp32 data: only the rest token by token).  Not when that
  // launch would be sequence-chunked: there is no workspace here.  Shorter 16-bit runs take the single-buffered
  // block kernel below, which measured 2-5 us faster on 2 to 8 positions.
  const la2_desc wb = whole_blocks(&d);   // what the scan kernels would process (fp32: the whole blocks only)
  if (ntokens >= 32 && make_plan(&wb).workspace == 0)
    return fwd_state_impl(&d, q, k, v, lambda, kv_state, o, kv_state, rstd, eps, nullptr, 0, hip_stream);
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  if (wide(head_dim) && is16(qkv_dtype)) {   // the block kernel of these head dimensions, in one chunk
    const Plan one{1, ((ntokens + 63) / 64) * 64, 0};
    ScanArgs a{q, k, v, o};
    a.init = kv_state;
    a.fin = kv_state;
    a.rstd = rstd;
    a.eps = eps;
    a.rstd_stride = ntokens;
    return run_scan(&d, one, false, a, lambda, nullptr, s);
  }
  la2::RecurParams r = recur_params(&d, lambda, 0, ntokens, false);
  r.x[0] = q; r.y[0] = k; r.z[0] = v; r.w[0] = o;
  r.init[0] = kv_state;
  r.fin[0] = kv_state;
  if (is16(qkv_dtype)) {   // 16-bit data: one block kernel launch (MFMA), with the epilogue
    r.rstd = rstd;
    r.eps = eps;
    r.rstd_stride = ntokens;
    return la2::launch_tail_bf16(qkv_dtype, head_dim, batch, r, s) == hipSuccess ? LA2_OK : LA2_ERR_LAUNCH;
  }
  // fp32: token by token in fp32, then (Norm) a row pass in place over the rows just written
  if (la2::launch_recur(head_dim, qkv_dtype, batch, 1, r, s) != hipSuccess) return LA2_ERR_LAUNCH;
  if (rstd == nullptr) return LA2_OK;
  const la2::NormBwdParams np{o, nullptr, rstd, o, d.stride_b, d.stride_h, d.stride_n, batch, heads, ntokens, 0, ntokens};
  return la2::launch_norm_fwd_rows(head_dim, qkv_dtype, np, eps, s) == hipSuccess ? LA2_OK : LA2_ERR_LAUNCH;
}
}  // namespace

extern "C" {

la2_status la2_decode_multi(int32_t batch, int32_t heads, int32_t head_dim, int32_t ntokens, int32_t qkv_dtype,
                            const void* q, const void* k, const void* v, const float* lambda, float* kv_state,
                            void* o, void* hip_stream) {
  return decode_multi_impl(batch, heads, head_dim, ntokens, qkv_dtype, q, k, v, lambda, kv_state, nullptr, 0.f, o,
                           hip_stream);
}

la2_status la2_decode_multi_norm(int32_t batch, int32_t heads, int32_t head_dim, int32_t ntokens, int32_t qkv_dtype,
                                 const void* q, const void* k, const void* v, const float* lambda, float* kv_state,
                                 float eps, void* o, float* rstd, void* hip_stream) {
  if (!(eps >= 0.f) || eps > 3.0e38f) return LA2_ERR_VALUE;
  if (batch > 0 && heads > 0 && ntokens > 0 && rstd == nullptr) return LA2_ERR_NULL;
  return decode_multi_impl(batch, heads, head_dim, ntokens, qkv_dtype, q, k, v, lambda, kv_state, rstd, eps, o,
                           hip_stream);
}

const char* la2_status_string(la2_status status) {
  switch (status) {
    case LA2_OK: return "ok";
    case LA2_ERR_NULL: return "a required pointer is NULL";
    case LA2_ERR_SHAPE: return "invalid shape (negative size, unsupported head_dim or too many chains)";
    case LA2_ERR_DTYPE: return "unsupported dtype";
    case LA2_ERR_STRIDE_ALIGN: return "pointer or stride violates the 16-byte alignment / layout rules";
    case LA2_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case LA2_ERR_LAUNCH: return "HIP kernel launch failed";
    case LA2_ERR_VALUE: return "a scalar argument is out of range";
  }
  return "unknown status";
}

}  // extern "C"
