/*
 * la2.h -- C ABI of the MI355X (gfx950) Lightning Attention-2 library.
 *
 * Causal linear attention with a per-head exponential decay lambda_h, per (batch, head):
 *
 *     o_t  = sum_{s<=t} lambda^(t-s) (q_t . k_s) v_s                  (Sec. 3.2.1, first equation)
 *     dq_t = sum_{s<=t} lambda^(t-s) (do_t . v_s) k_s
 *     dk_s = sum_{t>=s} lambda^(t-s) (do_t . v_s) q_t                 (Sec. 3.2.2, first equation,
 *     dv_s = sum_{t>=s} lambda^(t-s) (q_t . k_s) do_t                  with kv_t, dkv_t written out)
 *
 * evaluated block by block as in Algorithm 1 (forward) and Algorithm 2 (backward): an
 * intra-block masked product plus an inter-block product with a running d x d state.
 * No 1/sqrt(d) scaling and no softmax are applied; the output normalisation of eq. (2) only by
 * la2_fwd_norm / la2_bwd_norm.
 *
 * Conventions common to every entry point
 *   - All data pointers are DEVICE pointers on the current HIP device.  The caller owns every
 *     buffer, including the workspace; the library allocates nothing and never synchronises.  Its only
 *     state between calls are the two tuning knobs at the end of this header and, per device, the address of
 *     la2_fwd_noalloc's built-in scratch.
 *     Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default stream).
 *   - Descriptors (`la2_desc`) are HOST structs.
 *   - Sequence tensors (q, k, v, o, d_o, dq, dk, dv) share one shape [batch, heads, seqlen, head_dim]
 *     and one set of element strides (stride_b, stride_h, stride_n; the feature stride is 1).
 *     Base pointers must be 16-byte aligned and every stride a multiple of 16 bytes.
 *   - lambda is a device array of `heads` fp32 values with 0 < lambda <= 1 (a precondition; it is
 *     not read on the host and therefore not validated).
 *   - Outputs are fully overwritten.  Outputs must not alias inputs or each other.
 *   - An empty problem (batch, heads or seqlen equal to 0) returns LA2_OK without touching any
 *     pointer; pointers may then be NULL.
 *   - dtype LA2_BF16 / LA2_F16: bf16 / fp16 storage and MFMA operands, fp32 accumulation and fp32 running
 *     state (fp16: the masked scores and the state, as matrix operands, must stay within the fp16 range).
 *     dtype LA2_F32: fp32 storage and fp32 arithmetic throughout.
 *   - seqlen may be any value >= 0 (a ragged last block is masked) as long as one (batch, head) chain stays
 *     addressable with 32-bit byte offsets: (seqlen + 128) * stride_n * sizeof(element) <= 2^32, else
 *     LA2_ERR_SHAPE (dense bf16, head_dim 128: up to 16,777,088 positions).
 *   - head_dim is 64, 96, 128 or 256.  64 and 128 are the tuned paths and have every entry point.  96 and 256
 *     have every entry point but the left-product comparison (LA2_ERR_SHAPE): for the 16-bit types one MFMA
 *     block kernel, for fp32 the token-by-token recurrence (slow: meant for checking, not for training; no
 *     packed variant: LA2_ERR_DTYPE).
 *   - Argument errors are detected on the host BEFORE anything is launched and are reported through
 *     the return code; nothing aborts.  A failed launch is reported as LA2_ERR_LAUNCH.
 */
#ifndef LA2_H_
#define LA2_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LA2_OK = 0,
  LA2_ERR_NULL = 1,         /* a required pointer is NULL                                   */
  LA2_ERR_SHAPE = 2,        /* negative size, unsupported head_dim, or index range overflow */
  LA2_ERR_DTYPE = 3,        /* dtype is not a la2_dtype (or not one this entry point takes) */
  LA2_ERR_STRIDE_ALIGN = 4, /* pointer or stride not 16-byte aligned, or rows overlap       */
  LA2_ERR_WORKSPACE = 5,    /* workspace NULL or smaller than la2_workspace_bytes()         */
  LA2_ERR_LAUNCH = 6,       /* the HIP runtime refused a launch                             */
  LA2_ERR_VALUE = 7         /* a scalar argument is out of range (eps negative or not finite) */
} la2_status;

typedef enum { LA2_F32 = 0, LA2_BF16 = 1, LA2_F16 = 2 } la2_dtype;

typedef enum { LA2_OP_FWD = 0, LA2_OP_BWD = 1, LA2_OP_FWD_STATE = 2, LA2_OP_BWD_STATE = 3 } la2_op;

/* Host-side description of the sequence tensors. */
typedef struct {
  int32_t batch;
  int32_t heads;
  int32_t seqlen;
  int32_t head_dim; /* 64, 96, 128 or 256 */
  int32_t dtype;    /* la2_dtype */
  int32_t reserved; /* must be 0 */
  int64_t stride_b; /* elements between consecutive batches   */
  int64_t stride_h; /* elements between consecutive heads     */
  int64_t stride_n; /* elements between consecutive positions */
} la2_desc;

/* Fills strides for a dense [batch, heads, seqlen, head_dim] tensor. */
void la2_desc_dense(la2_desc* desc, int32_t batch, int32_t heads, int32_t seqlen, int32_t head_dim,
                    la2_dtype dtype);

/*
 * Bytes of device workspace la2_fwd / la2_bwd need for this problem (op is a la2_op).  The
 * workspace holds the d x d states of the sequence chunks that are processed in parallel when
 * batch*heads alone cannot fill the GPU (their start states; for a plan of at most four chunks their local
 * states, from which every workgroup forms its own start state); it may be 0.  Returns 0 for an invalid descriptor.
 * The value depends on the device's compute-unit count and on la2_set_chunk_tokens().
 */
size_t la2_workspace_bytes(const la2_desc* desc, int32_t op);

/*
 * How la2_fwd / la2_bwd cut this problem's sequences into chunks that run in parallel (host query, launches
 * nothing): *nchunks chunks of *chunk_tokens positions each (the last one may be shorter); 1 chunk = the block
 * loop of Algorithm 1 / 2 runs over the whole sequence in one workgroup per (batch, head).  The workspace
 * holds one d x d fp32 start state per (batch, head, chunk) when nchunks > 1.  Depends on the device's
 * compute-unit count and on la2_set_chunk_tokens(), like la2_workspace_bytes().
 * One case it does not describe: a batch with a few more chains than a whole number (one to four) per compute unit,
 * which as one launch gives some units a workgroup more than the others and takes nearly as long as the next whole round (fp32:
 * twice the time of one chain per unit for anything between one and two).  Every entry point that takes a dense
 * batch (la2_fwd, la2_bwd, their _state, _saved, _norm and _noalloc forms) runs it as two calls on the given
 * stream: the first floor(rounds * units / heads) batch rows by the plan of that many rows (one chunk), the
 * remaining rows, with their rows of the states and of rstd, by the plan of a descriptor with that many rows
 * (several chunks); la2_workspace_bytes() answers for both, and what either part would refuse is refused before the
 * first launch.  A forward call's workspace then holds the chunk states of its second part, which is what
 * la2_bwd_saved reads.  Which shapes: seqlen >= 2048 (fp32: 1024), no la2_set_chunk_tokens(), and a partial round
 * of at most 1/8 to 4/8 of the unit count, by dtype and head_dim, as measured.  Results are those of the same block
 * loop either way, up to the rounding of the chunk states.
 */
la2_status la2_chunk_plan(const la2_desc* desc, int32_t* nchunks, int32_t* chunk_tokens);

/*
 * Forward pass, Algorithm 1:  o = LA2(q, k, v; lambda).
 *   q, k, v   in   device, [batch, heads, seqlen, head_dim] with the descriptor's strides
 *   lambda    in   device, fp32 [heads]
 *   o         out  device, same layout as q
 *   workspace      device scratch of at least la2_workspace_bytes(desc, LA2_OP_FWD) bytes, 256-byte
 *                  aligned; may be NULL when that size is 0
 */
la2_status la2_fwd(const la2_desc* desc, const void* q, const void* k, const void* v,
                   const float* lambda, void* o, void* workspace, size_t workspace_bytes,
                   void* hip_stream);

/*
 * la2_fwd for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * la2_fwd, without the workspace: the chunk start states live in LA2_NOALLOC_SCRATCH_BYTES of device memory
 * that is part of the library's code object (each GPU the library runs on holds that much until the process
 * ends).  The call allocates nothing and frees nothing; its first use on a device looks up the scratch
 * address there (which may load the code object on that device), later calls only enqueue kernels.
 *   - A problem whose la2_workspace_bytes(desc, LA2_OP_FWD) exceeds LA2_NOALLOC_SCRATCH_BYTES is refused with
 *     LA2_ERR_WORKSPACE before anything is launched (the sweep's (4, 16K) and (1, 64K) points need exactly
 *     that much on a 256-CU device; problems whose chains fill the device in whole rounds need none).  One
 *     exception: a batch that la2_fwd would run as two calls (see la2_chunk_plan) and whose second part's chunk
 *     states exceed the scratch runs here as one call, which needs none.
 *   - All calls on one GPU share that GPU's scratch, whatever their stream: calls that overlap in time on one
 *     GPU race on it.  Calls on one stream, or otherwise ordered, are fine; the scratch keeps the previous
 *     call's contents and every call overwrites what it reads, so nothing needs clearing in between.
 *   - LA2_ERR_LAUNCH if the current device cannot be determined or holds no copy of the scratch.
 */
#define LA2_NOALLOC_SCRATCH_BYTES (16u << 20)
la2_status la2_fwd_noalloc(const la2_desc* desc, const void* q, const void* k, const void* v,
                           const float* lambda, void* o, void* hip_stream);

/*
 * Backward pass, Algorithm 2:  (dq, dk, dv) from (q, k, v, d_o).  dq comes from an ascending pass
 * with the running KV state, dk and dv from a descending pass with the running dKV state.  The
 * forward output o is not needed (Algorithm 2 lists it as loaded, but no formula uses it).
 *   workspace: at least la2_workspace_bytes(desc, LA2_OP_BWD) bytes.
 */
la2_status la2_bwd(const la2_desc* desc, const void* q, const void* k, const void* v,
                   const void* d_o, const float* lambda, void* dq, void* dk, void* dv,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Forward and backward pass of one SEGMENT of a longer sequence: the recursion of Sec. 3.2.1
 * (kv_t = lambda kv_{t-1} + k_t^T v_t, o_t = q_t kv_t) started from a given state kv_0 = kv_init
 * instead of zero, with the state after the last position handed out; Algorithm 1's KV and
 * Algorithm 2's dKV carried across calls.  Uses: chunked prefill followed by la2_decode_step,
 * sequences processed in pieces, sequence parallelism.
 *   kv_init     in   device fp32 [batch, heads, head_dim, head_dim] dense (key feature = row, value
 *                    feature = column; the layout of la2_decode_step's kv_state), or NULL for zero
 *   kv_final    out  same layout: kv_seqlen, or NULL if not wanted
 *   d_kv_final  in   gradient of the loss with respect to kv_final, or NULL for zero
 *   d_kv_init   out  gradient with respect to kv_init, or NULL if not wanted
 * la2_bwd_state needs the kv_init the forward pass was given (dq depends on it).  All other arguments
 * as for la2_fwd / la2_bwd, which are these functions with NULL states.  State pointers are 16-byte
 * aligned.  Workspace: la2_workspace_bytes(desc, LA2_OP_FWD_STATE / LA2_OP_BWD_STATE).  Any seqlen: the 16-bit
 * kernels form the state right after (and take the gradient right behind) the last position inside their block
 * loop, whatever the length; for LA2_F32 at head_dim 64 and 128, when kv_final / d_kv_final is given and seqlen
 * is not a multiple of 32, the last seqlen % 32 positions run in a short-run kernel (those block kernels form
 * states after whole blocks only).  seqlen == 0 copies the state through (kv_final = kv_init,
 * d_kv_init = d_kv_final; zero if the input is NULL).
 */
la2_status la2_fwd_state(const la2_desc* desc, const void* q, const void* k, const void* v,
                         const float* lambda, const float* kv_init, void* o, float* kv_final,
                         void* workspace, size_t workspace_bytes, void* hip_stream);
la2_status la2_bwd_state(const la2_desc* desc, const void* q, const void* k, const void* v,
                         const void* d_o, const float* lambda, const float* kv_init,
                         const float* d_kv_final, void* dq, void* dk, void* dv, float* d_kv_init,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The operator with its output normalisation, eq. (2): O = Norm(Q (K^T V)) with the decay and the causal
 * mask of Sec. 3.2.1 inside.  The paper names Norm without defining it and drops it from its derivations
 * (Sec. 3.2.1); here it is the root-mean-square normalisation of every output row over the head's
 * features, without a gain:
 *     u_t = sum_{s<=t} lambda^(t-s) (q_t . k_s) v_s,   r_t = 1 / sqrt(mean_j u_tj^2 + eps),   o_t = r_t u_t
 * Forward: Algorithm 1 with the normalisation applied to each finished output tile in registers (u never
 * goes to memory); r is kept for the backward pass.  Backward: one pass over the rows forms
 *     d_u_t = r_t (d_o_t - o_t mean_j(d_o_tj o_tj))
 * (the gradient with respect to u; this is where Algorithm 2's load of O_i is used), then Algorithm 2 runs
 * on d_u.
 *   eps   in   host scalar, >= 0 and finite, else LA2_ERR_VALUE.  With eps == 0 a row whose u_t is all
 *              zero yields NaN.
 *   rstd  out (forward) / in (backward)   device fp32 [batch, heads, seqlen] dense: r_t; 4-byte aligned
 *   o     out (forward) / in (backward)   the normalised output
 *   d_u   out  device, same layout as d_o: the gradient with respect to u (also the scratch that
 *              Algorithm 2 reads; fully overwritten; must not alias any other argument)
 * Everything else, the workspace included, as for la2_fwd (LA2_OP_FWD) and la2_bwd (LA2_OP_BWD).
 */
la2_status la2_fwd_norm(const la2_desc* desc, const void* q, const void* k, const void* v,
                        const float* lambda, float eps, void* o, float* rstd, void* workspace,
                        size_t workspace_bytes, void* hip_stream);
la2_status la2_bwd_norm(const la2_desc* desc, const void* q, const void* k, const void* v, const void* o,
                        const float* rstd, const void* d_o, const float* lambda, void* d_u, void* dq,
                        void* dk, void* dv, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The normalised operator on one SEGMENT of a longer sequence: la2_fwd_norm / la2_bwd_norm with the state
 * arguments of la2_fwd_state / la2_bwd_state (same meaning, layout and workspace: LA2_OP_FWD_STATE /
 * LA2_OP_BWD_STATE).  The state carries the un-normalised recurrence of Sec. 3.2.1; only the output rows are
 * normalised (eq. (2)), so kv_final and the state gradients are those of the un-normalised operator for d_u.
 * rstd, o, d_u as in la2_fwd_norm / la2_bwd_norm.  An empty sequence passes the state (its gradient) through.
 */
la2_status la2_fwd_state_norm(const la2_desc* desc, const void* q, const void* k, const void* v,
                              const float* lambda, const float* kv_init, float eps, void* o, float* rstd,
                              float* kv_final, void* workspace, size_t workspace_bytes, void* hip_stream);
la2_status la2_bwd_state_norm(const la2_desc* desc, const void* q, const void* k, const void* v, const void* o,
                              const float* rstd, const void* d_o, const float* lambda, const float* kv_init,
                              const float* d_kv_final, void* d_u, void* dq, void* dk, void* dv,
                              float* d_kv_init, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Algorithm 1 / Algorithm 2 over PACKED sequences of different lengths (a batch without padding): the
 * tensors are [total_positions, heads, head_dim]; sequence b occupies positions cu_seqlens[b] ..
 * cu_seqlens[b + 1] - 1 and is a chain of its own (zero start state, no interaction with its neighbours).
 *   desc             batch = number of sequences, seqlen = an upper bound of the sequence lengths (the launch is
 *                    planned for it: pass the longest length), stride_n / stride_h = elements between consecutive
 *                    positions / heads (dense packing: heads * head_dim and head_dim), stride_b ignored
 *   cu_seqlens       in   device, int32 [batch + 1], non-decreasing, cu_seqlens[0] = offset of the first
 *                    sequence; lengths above desc->seqlen are a precondition violation (not read on the host)
 *   total_positions  host scalar: the number of positions in all sequences together (the packed tensors' first
 *                    extent), or 0 if not known; negative: LA2_ERR_SHAPE.  It sizes the plan and the workspace
 *                    (a value below the real sum of the lengths is safe but leaves sequences that do not fit
 *                    the workspace planned from it uncomputed); the lengths
 *                    stay on the device, and with it the host can tell a batch of about equal lengths from one
 *                    whose longest sequence would run long after all the others have finished.  Such a batch is
 *                    cut into sequence chunks (a quarter of desc->seqlen) although it has chains enough to
 *                    fill the device; the short sequences are single chunks and pay nothing for it.
 * Everything else as for la2_fwd / la2_bwd.  Workspace: la2_varlen_workspace_bytes(desc, total_positions, op) with
 * op = LA2_OP_FWD or LA2_OP_BWD (with total_positions = 0: la2_workspace_bytes(desc, op)).
 * A sequence of length 0 is fine.
 */
size_t la2_varlen_workspace_bytes(const la2_desc* desc, int64_t total_positions, int32_t op);
la2_status la2_fwd_varlen(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions,
                          const void* q, const void* k, const void* v, const float* lambda, void* o,
                          void* workspace, size_t workspace_bytes, void* hip_stream);
la2_status la2_bwd_varlen(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions,
                          const void* q, const void* k, const void* v, const void* d_o, const float* lambda,
                          void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/*
 * Packed sequences as SEGMENTS of longer ones (Sec. 3.2.1, recursive form: what a sequence's past contributes is
 * its state): la2_fwd_varlen / la2_bwd_varlen with the state arguments of la2_fwd_state / la2_bwd_state, one state
 * per (sequence, head).  A prefill over a packed batch of prompts hands kv_final to la2_decode_step; a long
 * prompt can be fed in pieces, each call starting from the state the previous one left.
 *   kv_init     in   device fp32 [batch, heads, head_dim, head_dim] dense (sequence b, head h at
 *               ((b * heads + h) * head_dim + i) * head_dim + j, i = key feature, j = value feature), or NULL: zero
 *   kv_final    out  same layout, or NULL: the state right after each sequence's last position, whatever its length
 *   d_kv_final  in   gradient with respect to kv_final, or NULL: zero
 *   d_kv_init   out  gradient with respect to kv_init, or NULL: not wanted
 * All state pointers 16-byte aligned (LA2_ERR_STRIDE_ALIGN).  A sequence of length 0 passes its state (its state's
 * gradient) through.  Data types LA2_BF16 and LA2_F16 (LA2_ERR_DTYPE otherwise) at head_dim 64 and 128
 * (LA2_ERR_SHAPE otherwise): the kernels of these form the state at a sequence end that is not a block boundary
 * inside the block loop.  With every state pointer NULL the calls are la2_fwd_varlen / la2_bwd_varlen.
 * Workspace as for la2_fwd_varlen / la2_bwd_varlen.
 */
la2_status la2_fwd_varlen_state(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions,
                                const void* q, const void* k, const void* v, const float* lambda,
                                const float* kv_init, void* o, float* kv_final, void* workspace,
                                size_t workspace_bytes, void* hip_stream);
la2_status la2_bwd_varlen_state(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions,
                                const void* q, const void* k, const void* v, const void* d_o, const float* lambda,
                                const float* kv_init, const float* d_kv_final, void* dq, void* dk, void* dv,
                                float* d_kv_init, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The normalised operator (eq. (2), Norm read as in la2_fwd_norm) over packed sequences: la2_fwd_norm / la2_bwd_norm
 * with the packed layout and planning arguments of la2_fwd_varlen / la2_bwd_varlen.
 *   total_positions  here the packed tensors' first extent exactly (> 0, < 2^31; LA2_ERR_SHAPE otherwise): it is
 *                    the row length of rstd
 *   rstd   out (forward) / in (backward)   device fp32 [heads, total_positions] dense: r of packed position t and
 *          head h at rstd[h * total_positions + t]; entries of positions outside every sequence are not touched
 *   o, d_u, eps as in la2_fwd_norm / la2_bwd_norm; rows of d_u outside every sequence are not written
 * Workspace as for la2_fwd_varlen / la2_bwd_varlen.
 */
la2_status la2_fwd_varlen_norm(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions,
                               const void* q, const void* k, const void* v, const float* lambda, float eps,
                               void* o, float* rstd, void* workspace, size_t workspace_bytes, void* hip_stream);
la2_status la2_bwd_varlen_norm(const la2_desc* desc, const int32_t* cu_seqlens, int64_t total_positions,
                               const void* q, const void* k, const void* v, const void* o, const float* rstd,
                               const void* d_o, const float* lambda, void* d_u, void* dq, void* dk, void* dv,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * One step of the recurrent form (Sec. 3.2.1, recursive form), for every (batch, head):
 *     kv <- lambda_h * kv + k^T v          (state updated IN PLACE)
 *     o   = q kv                           (uses the UPDATED state, i.e. includes this token)
 *   q, k, v   in      device, dense [batch, heads, head_dim], dtype qkv_dtype
 *   lambda    in      device, fp32 [heads]
 *   kv_state  in/out  device, dense fp32 [batch, heads, head_dim (key), head_dim (value)]
 *   o         out     device, dense [batch, heads, head_dim], dtype qkv_dtype
 * All pointers 16-byte aligned.  head_dim is 64, 96, 128 or 256.
 */
la2_status la2_decode_step(int32_t batch, int32_t heads, int32_t head_dim, int32_t qkv_dtype,
                           const void* q, const void* k, const void* v, const float* lambda,
                           float* kv_state, void* o, void* hip_stream);

/*
 * The decode step of the normalised operator (eq. (2) with Norm read as in la2_fwd_norm): the same state update,
 * and the output row divided by sqrt(mean_j o_j^2 + eps) before it is stored.  eps as for la2_fwd_norm
 * (LA2_ERR_VALUE).
 */
la2_status la2_decode_step_norm(int32_t batch, int32_t heads, int32_t head_dim, int32_t qkv_dtype,
                                const void* q, const void* k, const void* v, const float* lambda,
                                float* kv_state, float eps, void* o, void* hip_stream);

/*
 * la2_bwd_state for callers that kept the forward pass's workspace (a training step).  When the sequence is
 * processed in chunks that buffer holds the chunk states of the (K, V) scan, which are (transposed)
 * those of Algorithm 2's first loop, so the backward pass skips recomputing them (one pass over K and V less).
 *   fwd_workspace        in  the workspace buffer that la2_fwd / la2_fwd_state (or their _norm forms) used for
 *                            the SAME desc, k, v, lambda and kv_init, contents untouched since, distinct from
 *                            `workspace`; 256-byte aligned (LA2_ERR_WORKSPACE otherwise); only read.  NULL, or a
 *                            problem that needs no workspace: exactly la2_bwd_state.
 *   fwd_workspace_bytes      its size; smaller than what that forward call needed: LA2_ERR_WORKSPACE
 *   fwd_wrote_kv_final       non-zero if that forward call was given a kv_final pointer.  With LA2_F32 data such
 *                            a call plans its chunks for the whole blocks of a ragged seqlen only (see
 *                            la2_fwd_state); if that plan differs from this call's, the saved states are not used
 *                            and the result is that of la2_bwd_state.
 * The chunk plan also depends on la2_set_chunk_tokens() and the device: both calls must see the same.
 * A batch that runs as two calls (see la2_chunk_plan) left only its second part's chunk states in fwd_workspace; the
 * second part of this call reads them, the first part, should its own plan cut, recomputes.
 */
la2_status la2_bwd_saved(const la2_desc* desc, const void* q, const void* k, const void* v,
                         const void* d_o, const float* lambda, const float* kv_init,
                         const float* d_kv_final, void* dq, void* dk, void* dv, float* d_kv_init,
                         const void* fwd_workspace, size_t fwd_workspace_bytes, int32_t fwd_wrote_kv_final,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Comparison kernel, not part of the method: the same forward pass evaluated as the masked left product
 * O = [(Q K^T) * M] V over all earlier key blocks (Sec. 3.1 eq. (1) with the decay mask M of Sec. 3.2),
 * O(n^2 d) instead of O(n d^2), the way the predecessor of Algorithm 1 computes it.  For measuring where
 * the block recurrence overtakes it as n grows.  bf16 only (LA2_ERR_DTYPE otherwise), head_dim 64 or 128
 * (LA2_ERR_SHAPE otherwise); arguments as la2_fwd; no workspace.
 */
la2_status la2_left_product_fwd(const la2_desc* desc, const void* q, const void* k, const void* v,
                                const float* lambda, void* o, void* hip_stream);

/*
 * The backward pass of the same comparison: the gradients of Sec. 3.2.2 evaluated as masked products over all
 * earlier (dq) or all later (dk, dv) positions, dQ = [(dO V^T) * M] K, dK = [(dO V^T) * M]^T Q,
 * dV = [(Q K^T) * M]^T dO, O(n^2 d), three launches of the comparison kernel.  bf16 only, head_dim 64 or 128;
 * arguments as la2_bwd; no workspace.
 */
la2_status la2_left_product_bwd(const la2_desc* desc, const void* q, const void* k, const void* v,
                                const void* d_o, const float* lambda, void* dq, void* dk, void* dv,
                                void* hip_stream);

/*
 * ntokens consecutive decode steps in one launch (recursive form of Sec. 3.2.1): for t = 0 .. ntokens-1
 * kv_state <- lambda_h kv_state + k_t^T v_t, o_t = q_t kv_state.  The state is read and written once per
 * launch instead of once per token.
 *   q, k, v   in      device, dense [batch, heads, ntokens, head_dim], dtype qkv_dtype (la2_dtype)
 *   lambda    in      device, fp32 [heads]
 *   kv_state  in/out  device, fp32 dense [batch, heads, head_dim, head_dim], updated in place
 *   o         out     device, dense [batch, heads, ntokens, head_dim], dtype qkv_dtype
 * All pointers 16-byte aligned.  head_dim is 64, 96, 128 or 256; ntokens <= 65536.  Same result as ntokens calls of
 * la2_decode_step up to rounding.  16-bit data: block kernels with bf16 / fp16 matrix operands as in la2_fwd
 * (whole blocks through la2_fwd_state's kernels with the state in place when batch * heads fills the device
 * without a workspace; a shorter run or the rest in one launch of a small block kernel that hands out the exact
 * state after a partial block).  fp32 data: whole blocks as in la2_fwd_state, the rest token by token in fp32.
 */
la2_status la2_decode_multi(int32_t batch, int32_t heads, int32_t head_dim, int32_t ntokens,
                            int32_t qkv_dtype, const void* q, const void* k, const void* v,
                            const float* lambda, float* kv_state, void* o, void* hip_stream);

/*
 * la2_decode_multi for the normalised operator: every output row divided by sqrt(mean_j o_j^2 + eps) before it is
 * stored (the state keeps the un-normalised recurrence), r_t handed out as by la2_fwd_norm.
 *   eps    host scalar as for la2_fwd_norm (LA2_ERR_VALUE)
 *   rstd   out  device fp32 dense [batch, heads, ntokens]; required
 */
la2_status la2_decode_multi_norm(int32_t batch, int32_t heads, int32_t head_dim, int32_t ntokens,
                                 int32_t qkv_dtype, const void* q, const void* k, const void* v,
                                 const float* lambda, float* kv_state, float eps, void* o, float* rstd,
                                 void* hip_stream);

/*
 * Block size B (rows of the intra-block tile, Algorithm 1) of the scan kernel the library launches
 * for this descriptor under the current la2_set_scan_variant(); results do not depend on it beyond
 * rounding.  Returns 0 for an invalid descriptor.  Used to report FLOPs with the formula of
 * Algorithms 1 and 2.
 */
int32_t la2_block_size(const la2_desc* desc);

/*
 * Tuning / test knob: tokens per sequence chunk (rounded up to a multiple of the block size).
 * 0 restores the automatic choice.  Process-global (an atomic that every call reads once: setting it while
 * another thread is inside a call gives that call either value); changes the value returned by
 * la2_workspace_bytes().  Results do not depend on it beyond rounding.
 */
void la2_set_chunk_tokens(int32_t tokens);

/*
 * Test / tuning knob: which 16-bit scan kernel la2_fwd / la2_bwd launch at head_dim 64 and 128.
 *   0  automatic (currently the half-block kernel: blocks of 32 positions, up to two workgroups per
 *      compute unit; it measured faster than the full-block kernel at every launch size)
 *   1  the full-block kernel (blocks of 64 positions, one workgroup per compute unit)
 *   2  the half-block kernel
 * Other values are taken as 0.  Both kernels implement Algorithm 1's block recurrence (the block
 * size is the algorithm's free parameter B); results differ by rounding only.  Process-global, as
 * la2_set_chunk_tokens.  Ignored for fp32, for head_dim 96 / 256, and by calls that carry states or the Norm
 * epilogue (only the half-block kernel has those).  With 1 the backward pass of a sequence-chunked problem forms
 * the chunk states of its second loop in a pass of its own instead of inside the first loop's launch.
 */
void la2_set_scan_variant(int32_t variant);

/* Static, NUL-terminated description of a status code. */
const char* la2_status_string(la2_status status);

#ifdef __cplusplus
}
#endif
#endif /* LA2_H_ */
