/*
 * libmeft -- the sparse-adapter layer of MEFT (Memory-Efficient Fine-Tuning through Sparse
 * Adapter) for one AMD MI355X (gfx950).  Plain C ABI: pointers and sizes only.
 *
 * The layer (paper: Section 3.1 "Sparse Activation", Section 3.2 "Key-Experts Mechanism",
 * Algorithm 1 "MEFT FFN Layer", evaluated per token):
 *
 *   p[t,b]   = sum_c Wg[b,c] h[t,c] (+ bias[b])                 router score, Eq. 5 (no softmax)
 *   tau_t    = the top_e blocks (key experts) with the largest p[t,.]
 *   sc[t,j]  = sum_c h[t,c] K[j,c]   for every neuron j of the blocks in tau_t       Eq. 6
 *   I_t      = the top_k of those neurons with the largest sc[t,j]                    Eq. 1
 *   out[t,:] = sum_{j in I_t} max(sc[t,j],0) V[j,:]                                   Eq. 4
 *
 * and its backward, in which only the activated neurons receive gradient (last paragraph of
 * Section 3.1):
 *
 *   ds[t,j]  = (dOut[t,:] . V[j,:])  if sc[t,j] > 0 else 0
 *   dh[t,:]  = sum_{j in I_t} ds[t,j] K[j,:]
 *   dK[j,:]  = sum_{t: j in I_t} ds[t,j] h[t,:]      dV[j,:] = sum_{t: j in I_t} max(sc[t,j],0) dOut[t,:]
 *
 * Naming: T tokens, hidden size d, N = n_blocks*block_size adapter neurons (the paper's r), K[N,d]
 * the keys (row j = column j of the paper's W_A), V[N,d] the values (row j of W_B), Wg[n_blocks,d]
 * the router.  Block b owns the contiguous neurons [b*block_size, (b+1)*block_size).
 * Ties in both selections go to the lower index; +0 and -0 tie.  The router score only selects
 * (no gate multiply), so there is no router gradient.
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers owned by the caller, row-major, contiguous, 16-byte
 *    aligned.  With MEFT_FLAG_HOST_KV set, K, V, dK, dV are pinned HOST pointers instead (see the flag).
 *  - `ws` is a device workspace of at least meft_workspace_bytes(shape) bytes, 256-byte aligned,
 *    owned by the caller; its contents are scratch and carry nothing from call to call.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued on
 *    it; the library never synchronises the stream, allocates no device memory per call and keeps
 *    no state between calls.  Calls that share a workspace must be ordered on one stream.
 *  - Arguments are validated on the host before anything is enqueued; a non-zero status means
 *    nothing was enqueued.  Faults that happen on the device later surface at the caller's next
 *    synchronisation.  Inputs must be finite (the ordering of NaN is unspecified).
 *  - dtype applies to h, Wg, K, V, out, dOut, dh, dK, dV.  Every sum is accumulated in fp32 and a result is
 *    rounded (to nearest even) when it is stored.  With MEFT_F32, and for bf16 shapes that run on the per-pair
 *    kernels (see "Precision" below), that is the only rounding.  bf16 shapes that run on the matrix cores round at
 *    these further points, each to bf16, nearest even:
 *      - the activation max(score, 0) when it enters a contraction as an operand (the value sum of Eq. 4 and dV);
 *        `act` itself is returned in fp32, unrounded;
 *      - the masked activation gradient ds when it enters a contraction as an operand (dh and dK);
 *      - a token's output row and input-gradient row are each the sum of top_e per-block partial rows; a partial
 *        row is rounded to bf16 when stored, the partial rows are summed in fp32 (blocks in ascending id) and
 *        the sum is rounded again.  out and dh therefore see three roundings (operand, partial row, result),
 *        dK and dV two (operand, result); each rounding has relative size at most 2^-9.
 *      A block that the batch routes at most min(16, top_e * block_size / top_k) tokens to is computed pair by pair
 *      instead (the paper's router is not balanced): for its entries the two operand roundings do not happen
 *      (act and ds stay fp32); the partial-row and result roundings are the same.
 *    Precision: a bf16 shape runs on the matrix cores when d is a multiple of 64, block_size >= 16,
 *    64 * top_k >= top_e * block_size and top_e * block_size <= 12288; otherwise on the per-pair kernels.
 *  - Host threads: the entry points may be called from several host threads; their host side (validation, launches,
 *    the library's few pieces of process-wide state) is serialised by a lock inside the library.  Ordering of the
 *    enqueued work is the caller's, through the streams.
 */
#ifndef MEFT_H
#define MEFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MEFT_OK = 0,
  MEFT_ERR_INVALID_ARG = 1, /* NULL pointer, misaligned pointer, inconsistent or non-positive sizes */
  MEFT_ERR_UNSUPPORTED = 2, /* a valid problem this build has no kernel for (see limits below)      */
  MEFT_ERR_WORKSPACE = 3,   /* ws is NULL, misaligned or smaller than meft_workspace_bytes()        */
  MEFT_ERR_DEVICE = 4       /* a HIP call (launch, copy) reported an error                          */
} meft_status;

typedef enum { MEFT_F32 = 0, MEFT_BF16 = 1 } meft_dtype;

/*
 * MEFT_FLAG_HOST_KV: the paper's placement of the adapter (Section 1 and Figure "Overview": parameters in CPU
 * memory, activated parts moved to the GPU on demand).  K, V (forward, backward) and dK, dV (backward) are
 * then PINNED HOST pointers (hipHostMalloc or equivalent).  The forward copies the blocks that some token
 * was routed to, the backward the blocks that hold a selected neuron, with hipMemcpyAsync on a stream of the
 * library's own, overlapped with the dispatch kernels (K) and with scoring and selection (V); the backward
 * computes dK, dV into device staging and a kernel then writes only the touched rows over the host link.
 * The workspace grows by four [N, d] matrices.  Differences from the conventions below, for these calls only:
 * the host blocks once per call until the routing result (which blocks are in use) is known; the library
 * creates one side stream, four events and a small pinned buffer on first use and keeps them; two such calls
 * must not be in flight at the same time on different streams.
 */
enum {
  MEFT_FLAG_HOST_KV = 1u,
  /*
   * With MEFT_FLAG_HOST_KV: the device copies of the K and V blocks that meft_sparse_fwd staged in the workspace
   * are kept for the meft_sparse_bwd of the same step, which then fetches nothing (and does not block the host):
   * K and V cross the host link once per step, not twice.  This is the one exception to "the workspace carries
   * nothing from call to call".  The caller promises that the backward uses the same workspace, shape, K and V
   * as the forward that produced `idx`, on the same stream, with no other call on that workspace in between.
   * The flag has no effect on the forward.
   */
  MEFT_FLAG_KEEP_STAGED = 2u,
  /*
   * With MEFT_FLAG_HOST_KV, for meft_sparse_fwd only: the K and V blocks this call needs were already requested
   * by meft_hostkv_stage on the same workspace with the same block_idx; the forward fetches nothing, does not block
   * the host, and waits (on the device) for those copies where it needs them.  See meft_hostkv_stage.
   */
  MEFT_FLAG_PRESTAGED = 4u,
  /*
   * For meft_sparse_bwd (ignored by the other calls): the meft_sparse_fwd of this step ran on this workspace with
   * this shape and wrote the idx and act that the backward is given, unchanged since, and no other call has used
   * the workspace in between.  The backward then takes the grouping of the (token, block) entries and the
   * activation rows from the workspace, where the forward left them, instead of rebuilding both from (idx, act):
   * same results, about 0.1 ms less at the LLaMA-7B-shaped configuration.  Like MEFT_FLAG_KEEP_STAGED this is an
   * exception to "the workspace carries nothing from call to call", and the promise is the caller's: the library
   * cannot check it.  Shapes that run on the per-pair kernels rebuild nothing and ignore the flag.
   */
  MEFT_FLAG_REUSE_FWD = 8u
};

/*
 * Problem shape.  Requirements (else MEFT_ERR_INVALID_ARG):
 *   T >= 0; d, n_blocks, block_size >= 1; N == n_blocks*block_size; 1 <= top_e <= n_blocks;
 *   1 <= top_k <= top_e*block_size; T*top_k and T*top_e*block_size below 2^31; activation == 0.
 * Limits of this build (else MEFT_ERR_UNSUPPORTED):
 *   d a multiple of 8 and at most 16384; top_e*block_size at most 4194304 (up to 12288
 *   candidates a token's scores are selected from LDS, beyond that from global memory); n_blocks at most 16384.
 */
typedef struct {
  int32_t T, d, N, n_blocks, block_size;
  int32_t top_e, top_k;
  int32_t dtype;      /* meft_dtype */
  int32_t activation; /* 0 = ReLU, the paper's choice and the only value */
  uint32_t flags;
} meft_shape;

/* Bytes of workspace that any of the three calls below needs for this shape (0 if the shape is
 * invalid or unsupported). */
size_t meft_workspace_bytes(const meft_shape* shape);

/* MEFT_OK if the shape is valid and supported, else the status the entry points would return. */
meft_status meft_check_shape(const meft_shape* shape);

const char* meft_status_string(meft_status status);

/*
 * Router scores and expert selection (Section 3.2, Eq. 5 and the top-K that follows it;
 * Algorithm 1, the two statements at the head of the token loop).
 *   h           [T, d]          in   hidden states
 *   Wg          [n_blocks, d]   in   router
 *   bias        [n_blocks] f32  in   added to the score, or NULL (NULL is the paper's router)
 *   block_idx   [T, top_e] i32  out  chosen blocks, ordered by (score descending, id ascending)
 *   block_score [T, top_e] f32  out  their scores, or NULL
 */
meft_status meft_route(const meft_shape* shape, const void* h, const void* Wg, const float* bias,
                       int32_t* block_idx, float* block_score, void* ws, size_t ws_bytes,
                       void* stream);

/*
 * meft_route for callers that cannot allocate or hand over a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, results and kernels as meft_route, without
 * `ws`: the partial router scores go to a fixed array of MEFT_ROUTE_STATIC_BYTES bytes of device memory that is
 * part of the library's image (every GPU the library runs on holds its own copy until the process ends; its
 * address is looked up once per device, on the first call with that device current).  The call allocates nothing,
 * on the host or on the device, and creates no events (per-kernel timing is off inside it).
 *   Limit: 16 * T * n_blocks <= MEFT_ROUTE_STATIC_BYTES (four partial score matrices of T x n_blocks floats);
 *   beyond it MEFT_ERR_WORKSPACE and nothing is enqueued.
 *   All calls on one GPU share that array: calls that overlap in time on one GPU (different streams, or host
 *   threads on different streams) race; order them on one stream or with events.  Nothing in the array has to
 *   start from zero and nothing in it is read after the call's kernels have finished.
 */
#define MEFT_ROUTE_STATIC_BYTES ((size_t)16 << 20)
meft_status meft_route_static(const meft_shape* shape, const void* h, const void* Wg, const float* bias,
                              int32_t* block_idx, float* block_score, void* stream);

/*
 * Key scores inside the chosen blocks, top-k neuron selection, gather of the selected value rows
 * and the activation-weighted sum (Section 3.2 Eq. 6-7; Section 3.1 Eq. 1-4; Algorithm 1, inner
 * loop, TopK and the returned adapter term).
 *   h         [T, d]           in
 *   K, V      [N, d]           in   keys, values
 *   block_idx [T, top_e] i32   in   distinct block ids per token, any order (as meft_route writes)
 *   out       [T, d]           out  adapter output (the frozen FFN term is the caller's); NULL: the call stops
 *                                   after the selection (S2'-S4) and writes only idx and act
 *   idx       [T, top_k] i32   out  selected neuron ids (global), distinct per token, ascending
 *   act       [T, top_k] f32   out  max(score, 0) of idx[t, i]
 * A block id outside [0, n_blocks) or repeated within a token is a caller error; such ids are
 * clamped into range so that no access leaves the tensors, and the results for that token are
 * unspecified.
 */
meft_status meft_sparse_fwd(const meft_shape* shape, const void* h, const void* K, const void* V,
                            const int32_t* block_idx, void* out, int32_t* idx, float* act, void* ws,
                            size_t ws_bytes, void* stream);

/*
 * Backward of meft_sparse_fwd for the saved selection (Section 3.1, last paragraph).
 *   h, K, V             in   as in the forward
 *   idx, act            in   as the forward wrote them (any order inside a token; ids distinct
 *                            per token and in [0, N))
 *   dOut   [T, d]       in   gradient of the loss with respect to out
 *   dh     [T, d]       out  or NULL
 *   dK, dV [N, d]       out  ONLY the rows listed in `touched` are written (overwritten, not
 *                            accumulated); every other row is neither read nor written
 *   touched [min(N, T*top_k)] i32  out  ascending ids of the neurons some token selected
 *   n_touched [1] i32   out  their number (device memory, like touched)
 * Pairs of one neuron are summed in ascending token order, so results are identical run to run.
 * Ids outside [0, N) are clamped into range (caller error, results unspecified).
 */
meft_status meft_sparse_bwd(const meft_shape* shape, const void* h, const void* K, const void* V,
                            const int32_t* idx, const float* act, const void* dOut, void* dh,
                            void* dK, void* dV, int32_t* touched, int32_t* n_touched, void* ws,
                            size_t ws_bytes, void* stream);

/*
 * Per-kernel timing for benchmarks (not part of the paper's method).  While enabled, every kernel
 * the library launches is bracketed by HIP events on the caller's stream.  meft_profile_read
 * synchronises those events and returns, for up to `cap` distinct kernel names in first-launch
 * order, the name, the number of launches and the summed milliseconds since the last
 * meft_profile_enable(1).  Returns the number of entries written.  Host memory; not thread-safe.
 */
void meft_profile_enable(int on);
int meft_profile_read(const char** names, int32_t* launches, float* total_ms, int cap);

/*
 * Layer pipeline for host-resident keys and values (the paper's Appendix A: retrieval and transfer of one layer's
 * rows run while the GPU computes, so that the GPU does not wait for them).  The call finds the blocks that
 * block_idx uses (the host blocks once until the work queued on `stream` so far has produced that list) and
 * requests their copies from the pinned host matrices K, V into this workspace on the library's side stream; it
 * returns without waiting for the copies.  A later meft_sparse_fwd with MEFT_FLAG_PRESTAGED on the same workspace
 * (same shape, block_idx, K, V) then finds them there; one stage call serves one forward.  Calling it for layer l+1 before enqueuing layer l's forward
 * overlaps l+1's transfer with l's compute; each layer in flight needs a workspace of its own.
 *   shape     with MEFT_FLAG_HOST_KV set (other flags are ignored)
 *   block_idx [T, top_e] device, as written by meft_route
 *   K, V      [N, d] pinned host
 *   ws        device workspace of meft_workspace_bytes(shape) bytes; the library remembers up to 16 workspaces
 *             with copies in flight (the oldest is forgotten first)
 * Errors as for meft_sparse_fwd; MEFT_ERR_INVALID_ARG without MEFT_FLAG_HOST_KV.
 */
meft_status meft_hostkv_stage(const meft_shape* shape, const int32_t* block_idx, const void* K, const void* V, void* ws,
                              size_t ws_bytes, void* stream);

/*
 * Batch-union evaluation: Algorithm 1 as printed gathers the selections of all tokens of the batch into one
 * set S and evaluates the adapter densely over S for every token (the per-token reading of Eq. 1-4 is what
 * meft_sparse_fwd computes; the two agree when one token is processed, or when everything is selected):
 *     S = sorted unique ids in idx;   out[t, :] = sum_{j in S} max(h[t,:].K[j,:], 0) V[j, :]
 * and, in the backward, the rules of Section 3.1 applied to every (token, neuron of S) pair:
 *     g = dOut[t,:].V[j,:], ds = g if h[t,:].K[j,:] > 0 else 0,
 *     dV[j,:] = sum_t a dOut[t,:],  dK[j,:] = sum_t ds h[t,:],  dh[t,:] = sum_{j in S} ds K[j,:].
 * bf16 with d % 64 == 0 only (MEFT_ERR_UNSUPPORTED otherwise, and with MEFT_FLAG_HOST_KV); the activations
 * enter the matrix cores rounded to bf16.
 *   idx       [T, top_k] device: the selection (meft_sparse_fwd with out == NULL computes just that)
 *   out       [T, d] device
 *   S, n_S    device; forward: outputs, capacity min(N, T*top_k), ascending ids and their count (|S| / top_k
 *             is the paper's sparsity statistic of Section 3.3); backward: inputs, as the forward wrote them
 *   dK, dV    [N, d] device: only the rows listed in S are written;  dh [T, d] or NULL
 *   ws        device workspace of at least meft_union_workspace_bytes(shape) bytes, 256-byte aligned
 * The backward recomputes the activations from h and K[S]; nothing is carried over in the workspace.
 * Same conventions as the calls above: caller-owned memory, work enqueued on `stream`, no allocation, no
 * synchronisation, arguments validated on the host first.  meft_union_workspace_bytes returns 0 for a shape
 * the variant does not support.
 */
size_t meft_union_workspace_bytes(const meft_shape* shape);
meft_status meft_union_fwd(const meft_shape* shape, const void* h, const void* K, const void* V, const int32_t* idx,
                           void* out, int32_t* S, int32_t* n_S, void* ws, size_t ws_bytes, void* stream);
meft_status meft_union_bwd(const meft_shape* shape, const void* h, const void* K, const void* V, const int32_t* S,
                           const int32_t* n_S, const void* dOut, void* dh, void* dK, void* dV, void* ws,
                           size_t ws_bytes, void* stream);

/*
 * Test aid (not part of the paper's method): the matrix-core kernels read operand matrices below 4 GB through
 * buffer resources and larger ones through 64-bit global pointers.  on != 0 selects the global-pointer kernels at
 * any size, so that a test reaches them with small inputs; on == 0 restores the choice by size.  The initial state
 * is that of the environment variable MEFT_GLOBAL_LOADS ("1" = on), read once when the library is loaded.
 */
void meft_debug_global_loads(int on);

/*
 * Diagnostics: the runtime's description of the launch failure behind the calling thread's most recent
 * MEFT_ERR_DEVICE from a launch ("no error" if there was none).  Static string, never NULL.
 */
const char* meft_last_device_error(void);

/*
 * Hyper-parameters of one optimizer step.  The paper trains with Adam (Section 4.3, "Implementation
 * Details"); the learning-rate schedule is the caller's, `lr` is the rate of this step.  `step` counts the
 * optimizer steps of the layer from 1 and drives both bias corrections.
 */
typedef struct {
  float lr, beta1, beta2, eps;   /* 0 <= beta < 1, eps >= 0 */
  int32_t step;                  /* >= 1 */
} meft_adam;

/*
 * Row-sparse Adam step on one parameter matrix of the adapter (K with G = dK, or V with G = dV).
 * Section 3.1, last paragraph: only the activated parameters have a gradient; those rows, as listed by
 * meft_sparse_bwd in `touched`, are updated, every other row keeps its weights and both moments unchanged
 * (a row without a gradient takes no part in the step).  For each listed row j and column c:
 *     m = beta1 m + (1 - beta1) g;   v = beta2 v + (1 - beta2) g^2
 *     w = w - lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 * computed in fp32.
 *   W       [N, d] of shape->dtype, device, updated in place on the listed rows
 *   G       [N, d] of shape->dtype, device, read on the listed rows only
 *   m, v    [N, d] float, device: first and second moment, updated in place on the listed rows
 *   master  [N, d] float or NULL, device: if given, it holds the weights in fp32; the step reads and updates
 *           it and writes its rounding to W (so steps smaller than a bf16 ulp are not lost)
 *   touched, n_touched   device, as written by meft_sparse_bwd (ascending ids; ids outside [0, N) are skipped)
 * Uses shape->N, d, dtype (and T, top_k for the launch size); no workspace; enqueues on `stream`, allocates
 * and synchronises nothing.  All matrices row-major, 16-byte aligned.
 * Errors: MEFT_ERR_INVALID_ARG (null or misaligned pointer, bad hyper-parameter, bad shape),
 * MEFT_ERR_UNSUPPORTED (MEFT_FLAG_HOST_KV: host-resident parameters are updated by the host),
 * MEFT_ERR_DEVICE (launch failure).
 */
meft_status meft_adam_rows(const meft_shape* shape, const meft_adam* hp, void* W, const void* G, float* m, float* v,
                           float* master, const int32_t* touched, const int32_t* n_touched, void* stream);

/*
 * Measurement aid (not part of the paper's method): a plain streaming copy of `bytes` bytes
 * (a multiple of 16; both pointers 16-byte aligned device memory) as one kernel on `stream`.
 * Gives the copy bandwidth of the machine and a dispatch of known traffic against which hardware
 * byte counters can be scaled.  It appears in meft_profile_read as "probe_copy".
 */
meft_status meft_probe_copy(void* dst, const void* src, size_t bytes, void* stream);

/*
 * Measurement aid (not part of the paper's method): a loop of bf16 matrix instructions and nothing else, as one
 * kernel on `stream`: `workgroups` workgroups of four waves, each wave issuing 8 * iters instructions
 * v_mfma_f32_32x32x16_bf16 (32768 flop each) on pseudo-random finite operands.  The rate it reaches is what the
 * matrix cores of this machine sustain, to set beside the published peak.  `out`: device memory for
 * workgroups * 256 floats (written, content of no interest).  It appears in meft_profile_read as "probe_mfma".
 * Errors: MEFT_ERR_INVALID_ARG (null pointer, workgroups outside 1..65536, iters < 1), MEFT_ERR_DEVICE.
 */
meft_status meft_probe_mfma(float* out, int workgroups, int iters, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MEFT_H */
