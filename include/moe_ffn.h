/*
 * moe_ffn.h -- C ABI of the MI355X (gfx950) Dispatch-to-Combine MoE-FFN library.
 *
 * One GPU's expert-parallel share of a top-k Mixture-of-Experts feed-forward
 * layer, as decomposed in the paper's Section 2.2 (Figure 2): Dispatch (permute
 * tokens into expert-contiguous order), grouped GEMM-1 (gate and up
 * projections), SwiGLU, grouped GEMM-2 (down projection), Combine (accumulate
 * the top-k contributions weighted by the routing scores), and the seven-node
 * backward graph.  The layer can run as one kernel launch per operator
 * ("serialized", the paper's kernel-by-kernel baseline of Section 2.3) or with
 * everything from Dispatch to Combine (the interval the paper times, Section 5.2)
 * as a single persistent launch that executes a static tile task list with
 * event-counter dependencies (the paper's Sections 4.3-4.4); routing runs ahead
 * of that launch as two small kernels.
 *
 * Conventions
 *   - Every pointer named d_* or documented "device" is device (HBM) memory on
 *     the current HIP device; everything else is host memory.
 *   - All tensors are row-major and contiguous.  Device pointers must be
 *     16-byte aligned.  MOE_MODE_PERSISTENT additionally requires 128-byte
 *     alignment of the workspace and of MoeSaved.Xp and MoeSaved.A (tiles of
 *     these buffers change hands between compute units inside the launch, and
 *     no cache line may be shared by two tiles); MOE_ERR_INVALID_ARG otherwise.
 *   - The library never allocates or frees device memory, never synchronises
 *     the stream and never reads results back: all work is enqueued on
 *     `stream`.  The caller owns every buffer and the stream.
 *   - Every function returns MOE_OK (0) or a negative MoeStatus.  Argument
 *     errors are detected on the host before anything is enqueued.
 *   - Calls that share a workspace must be ordered on one stream.
 *
 * Symbols: T tokens, H hidden size, I per-expert intermediate size, E global
 * experts, E_local experts owned by this device (global ids expert_base ..
 * expert_base+E_local-1), k experts per token, R = number of (token, slot)
 * pairs whose expert is local, R_max = T*min(k, E_local).
 */
#ifndef MOE_FFN_H_
#define MOE_FFN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum MoeStatus {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = -1,       /* null pointer, misaligned pointer, bad enum */
  MOE_ERR_UNSUPPORTED_SHAPE = -2, /* shape outside the limits listed at MoeShape */
  MOE_ERR_WORKSPACE_TOO_SMALL = -3,
  MOE_ERR_LAUNCH = -4,            /* a HIP launch or API call failed */
  MOE_ERR_SCHED_TIMEOUT = -5,     /* persistent scheduler: a bounded wait expired */
  MOE_ERR_XCD_PLACEMENT = -6      /* microbenchmark modes 1 and 3: workgroups of one class (id % 8) span several XCDs */
} MoeStatus;

typedef enum MoeDtype { MOE_F32 = 0, MOE_BF16 = 1 } MoeDtype;

typedef enum MoeMode {
  MOE_MODE_SERIALIZED = 0, /* one launch per operator, stream ordered */
  MOE_MODE_PERSISTENT = 1  /* Dispatch to Combine as one launch: tile tasks + event counters */
} MoeMode;

/*
 * Problem shape.  Limits: 1 <= k <= 16, k <= E <= 256, 1 <= E_local <= 256,
 * 0 <= expert_base, expert_base + E_local <= E, H and I multiples of 64 and at most 262144,
 * T >= 0 (T == 0 is a no-op).  dtype is the storage type of x, the weights,
 * the activations and the outputs; router logits and routing weights are
 * always fp32.  bf16 computes with fp32 accumulation (MFMA); f32 computes in
 * fp32 throughout.
 */
typedef struct MoeShape {
  int32_t T, H, I, E, E_local, expert_base, k;
  int32_t dtype; /* MoeDtype */
} MoeShape;

/*
 * Routing results and saved activations: caller-owned DEVICE buffers that the
 * forward fills.  They are the parity outputs of the routing / Dispatch steps
 * and the tensors the backward consumes.
 *   topk_idx [T,k]  i32  selected experts, ordered by (logit desc, id asc)
 *   topk_w   [T,k]  f32  softmax over the k selected logits
 *   counts   [E_local]   i32 rows per local expert
 *   offsets  [E_local+1] i32 exclusive prefix sum of counts; offsets[E_local]=R
 *   row_of   [T,k]  i32  row of slot (t,j) in expert-contiguous order, -1 if
 *                        the slot's expert is not local
 *   token_of [R_max] i32, slot_of [R_max] i32  inverse maps (first R entries)
 *   Xp [R_max,H]  dispatched tokens          (dtype)  may be NULL: no permuted copy is
 *                        kept; bf16 GEMM-1 and the backward's w1_grad then read x through
 *                        token_of (Section 4.4: no extra trip through HBM), other cases
 *                        make the copy in workspace memory
 *   H1 [R_max,2I] GEMM-1 output, gate|up     (dtype)  may be NULL: not stored
 *   A  [R_max,I]  SwiGLU output              (dtype)
 *   Yp [R_max,H]  GEMM-2 output              (dtype)
 * Only the first R rows of Xp/H1/A/Yp are written.  Rows of one expert are in
 * ascending token order.
 */
typedef struct MoeSaved {
  int32_t* topk_idx;
  float* topk_w;
  int32_t* counts;
  int32_t* offsets;
  int32_t* row_of;
  int32_t* token_of;
  int32_t* slot_of;
  void* Xp;
  void* H1;
  void* A;
  void* Yp;
} MoeSaved;

/* Human-readable name of a status code (static string, never NULL). */
const char* moe_status_string(int status);

/*
 * Bytes of device workspace the forward and the backward need for `shape`
 * (either pointer may be NULL).  The workspace holds the per-chunk expert
 * histograms, the tile map, the event counters and the scheduler's status
 * word; when `saved` is passed as NULL to moe_ffn_forward it also holds the
 * routing results and activations.  Host-only call.
 */
int moe_ffn_workspace_bytes(const MoeShape* shape, size_t* fwd_bytes, size_t* bwd_bytes);

/*
 * Forward layer (paper Section 2.2, Figure 2a; routing rule: top-k of the raw
 * logits, ties to the lowest expert id, softmax over the k selected logits):
 *   out[t,:] = sum over local slots j of topk_w[t,j] * FFN_e(x[t,:]),
 *   FFN_e(v) = (silu(v W_gate_up[e][:, :I]) * (v W_gate_up[e][:, I:])) W_down[e]
 * Tokens without a local slot get a zero row.
 *   d_x        [T,H]            dtype
 *   d_logits   [T,E]            f32
 *   d_w_gate_up[E_local,H,2I]   dtype, gate = columns 0..I-1, up = I..2I-1
 *   d_w_down   [E_local,I,H]    dtype
 *   d_out      [T,H]            dtype (overwritten)
 *   saved      nullable; if non-NULL every member except H1 and Xp must be non-NULL.
 *              NULL (inference): only `out` is produced.  Without a caller's Xp (saved
 *              NULL or saved->Xp NULL) the first grouped bf16 GEMM reads the token rows
 *              of x through the permutation and the permuted copy is not made at all
 *   d_workspace, workspace_bytes  >= moe_ffn_workspace_bytes(...).fwd_bytes
 *   mode       MoeMode.  MOE_MODE_PERSISTENT: the router and the prefix-sum / rank step run as two
 *              launches, then ONE launch runs every Dispatch, GEMM-1, GEMM-2 and Combine tile task.
 *              Its workers hand tiles over through the L2 of the accelerator die (XCD) they share;
 *              they verify at run time (hardware XCC id) that the workers of a queue all sit on one die
 *              and use device-wide fences for that queue otherwise.
 * Returns after enqueueing.  A scheduler timeout (MOE_MODE_PERSISTENT only) is
 * reported by moe_ffn_last_status().
 */
int moe_ffn_forward(const MoeShape* shape, const void* d_x, const float* d_logits,
                    const void* d_w_gate_up, const void* d_w_down, void* d_out,
                    const MoeSaved* saved, void* d_workspace, size_t workspace_bytes,
                    int mode, void* stream);

/*
 * Backward layer (paper Section 2.2, Figure 2b: backward Dispatch, act_grad,
 * w2_grad, SwiGLU_grad, gate_grad, w1_grad, backward Combine) plus the
 * gradient of the routing weights.  `saved` must come from a forward call with
 * H1 stored, on the same inputs.
 *   d_x           [T,H]  dtype   the forward's input; read only if saved->Xp is NULL
 *                                (then required, as is saved->token_of)
 *   d_dy          [T,H]  dtype   upstream gradient
 *   d_dx          [T,H]  dtype   overwritten; zero rows for tokens with no local slot
 *   d_dw_gate_up  [E_local,H,2I] dtype, overwritten (zeros for experts with no rows)
 *   d_dw_down     [E_local,I,H]  dtype, overwritten
 *   d_dtopk_w     [T,k]  f32     <dY[t], Yp[row_of[t,j]]>, 0 for non-local slots
 *   d_workspace, workspace_bytes  >= moe_ffn_workspace_bytes(...).bwd_bytes
 *   mode   MOE_MODE_SERIALIZED: one launch per operator.  MOE_MODE_PERSISTENT (bf16 only, else
 *          MOE_ERR_INVALID_ARG): act_grad + SwiGLU_grad and gate_grad, a producer-consumer pair of
 *          grouped GEMMs like the forward's, run as one launch of tile tasks with event counters
 *          (Sections 4.2-4.4), the other operators as launches of their own; results are
 *          bit-identical; a wait that expires is reported by moe_ffn_last_status() on this workspace.
 */
int moe_ffn_backward(const MoeShape* shape, const void* d_dy, const void* d_x,
                     const void* d_w_gate_up, const void* d_w_down, const MoeSaved* saved,
                     void* d_dx, void* d_dw_gate_up, void* d_dw_down, float* d_dtopk_w,
                     void* d_workspace, size_t workspace_bytes, int mode, void* stream);

/*
 * The same backward with its two branches on two streams (paper Section 2.2, Figure 2b: behind the backward
 * Dispatch the weight gradients w2_grad, w1_grad and the data gradients act_grad -> gate_grad -> backward
 * Combine only share inputs; Section 4.5 runs such branches side by side).  The weight-gradient launches are
 * enqueued on `wgrad_stream` (w2_grad behind the backward Dispatch, w1_grad behind the launch that completes
 * dH1), everything else on `stream`; their workgroups then take the CUs that the last tiles of the other
 * branch's kernels leave idle.  The call forks from `stream` and joins back into it with events before it
 * returns: work enqueued on `stream` afterwards sees every output, and `wgrad_stream` needs no
 * synchronisation by the caller.  Results are bit-identical to moe_ffn_backward's.
 *   wgrad_stream  a stream of the same device with the default priority; NULL or equal to `stream`:
 *                 exactly moe_ffn_backward.  While `stream` is being captured into a graph the other
 *                 stream joins the capture (fork / join through events); it must not be capturing already.
 * Everything else as for moe_ffn_backward.  The events are the library's (three per device, created at
 * the first such call on a device and kept); calls of this entry point are serialised against each other
 * while they enqueue.  MOE_ERR_LAUNCH if an event cannot be created or recorded.
 */
int moe_ffn_backward_two_streams(const MoeShape* shape, const void* d_dy, const void* d_x,
                                 const void* d_w_gate_up, const void* d_w_down, const MoeSaved* saved,
                                 void* d_dx, void* d_dw_gate_up, void* d_dw_down, float* d_dtopk_w,
                                 void* d_workspace, size_t workspace_bytes, int mode, void* stream,
                                 void* wgrad_stream);

/*
 * Reads the scheduler status word of a forward or backward workspace after the caller has
 * synchronised the stream (host-blocking 4-byte copy).  MOE_OK or
 * MOE_ERR_SCHED_TIMEOUT.
 */
int moe_ffn_last_status(const MoeShape* shape, const void* d_workspace);

/*
 * Test hook for the persistent scheduler's failure path (paper Section 4.3: a
 * task starts only once its dependent event has reached the threshold).  Sets
 * how many polls a wait may spend before it gives up; the default is about
 * one million (about a second).  With a tiny limit waits expire, the affected tasks
 * are skipped, every workgroup still drains its queues and exits, and
 * moe_ffn_last_status() reports MOE_ERR_SCHED_TIMEOUT.  Host-only, process-wide.
 */
int moe_ffn_debug_set_spin_limit(uint32_t polls);

/*
 * Test hook for the schedulers' fallback (paper Section 4.3: an event is triggered only once the task's
 * outputs are readable by the consumer).  Nonzero makes the single-launch forward and backward behave as
 * if every queue's workers had reported several XCDs: every tile hand-off uses device-wide release / acquire fences
 * instead of the XCD-local ones.  Results are unchanged.  Host-only, process-wide.
 */
int moe_ffn_debug_force_device_scope(int on);

/*
 * Test hook for checking the device-built schedule itself (paper Section 4.3: thresholds equal producer
 * counts, queue order is topological): byte offsets of the scheduler's tables inside the forward
 * (backward = 0) or backward (backward != 0) workspace and the constants needed to decode them.
 * out[0..6]  = offsets of: meta words, tile_expert, tile_row0, tile_rows (int32 per M tile), event counters
 *              (uint32), queue heads, task descriptors ([8 queues][max_tasks_per_queue] x {type | 0x80 if the index counts
 *              128-column halves of a wide GEMM-2 tile (a queue's halved last round) | index << 8,
 *              M tile, dependent event (-1: none), threshold}, int32 each)
 * out[7..9]  = max M tiles, max tasks per queue, number of event counters
 * out[10,11] = first per-tile event (Xp rows of M tile m ready: +m; A rows ready: + max M tiles + m), the
 *              event counting finished GEMM-2 tiles
 * out[12..14] = meta word indices: number of M tiles, first of the 8 queue lengths, GEMM-2 tile total
 * out[15..22] = queues, rows per PERMUTE task, GEMM-1 N tiles, GEMM-2 N tiles, wide tile rows, tall tile rows
 *              (0: none), lag (in tile pairs, clamped to a queue's
 *              pairs) of GEMM-2 tasks behind GEMM-1 tasks, bytes per descriptor
 * out[23]    = backward: N tiles of act_grad (the chain's first GEMM)
 * out[24]    = meta word index: workers of the last single launch that fell back to device-wide fences
 * n_out must be at least MOE_LAYOUT_WORDS.  Host-only.
 */
#define MOE_LAYOUT_WORDS 25
int moe_ffn_debug_layout(const MoeShape* shape, int backward, int64_t* out, int n_out);

/* ---- Stage entry points (the serialized path's operators, one launch each;
 *      used by the unit tests and the benchmark).  Same buffers as above. ---- */

/* Routing + Dispatch bookkeeping (paper Section 2.2, routing; Section 5.1,
 * tile offsets derived from the routing result at run time): fills topk_idx, topk_w, counts, offsets, row_of,
 * token_of, slot_of of `saved`, the tile map in the workspace and the tile scheduler's task tables (built for
 * this `saved`: with or without Dispatch tasks, depending on saved->Xp). */
int moe_route(const MoeShape* shape, const float* d_logits, const MoeSaved* saved,
              void* d_workspace, size_t workspace_bytes, void* stream);

/* Dispatch permute: Xp[r,:] = x[token_of[r],:] for r < R (Section 2.2 Dispatch). */
int moe_permute(const MoeShape* shape, const void* d_x, const MoeSaved* saved,
                void* d_workspace, size_t workspace_bytes, void* stream);

/* Grouped GEMM-1 with the SwiGLU epilogue: A = silu(Xp W[:, :I]) * (Xp W[:, I:])
 * per expert segment; also stores H1 if saved->H1 != NULL (Section 2.2). */
int moe_grouped_gemm_swiglu(const MoeShape* shape, const void* d_w_gate_up, const MoeSaved* saved,
                            void* d_workspace, size_t workspace_bytes, void* stream);

/* Grouped GEMM-2: Yp = A W_down[e] per expert segment (Section 2.2). */
int moe_grouped_gemm(const MoeShape* shape, const void* d_w_down, const MoeSaved* saved,
                     void* d_workspace, size_t workspace_bytes, void* stream);

/* Combine: out[t,:] = sum_j topk_w[t,j] * Yp[row_of[t,j],:] over local slots in
 * slot order, fp32 accumulation, no atomics (Section 2.2 Combine). */
int moe_combine(const MoeShape* shape, const MoeSaved* saved, void* d_out,
                void* d_workspace, size_t workspace_bytes, void* stream);

/* Grouped GEMM-2 with Combine in its epilogue (Section 4.4: the expert outputs reach their destination rows
 * from the epilogue of the tile that made them, without a trip through HBM as a permuted tensor): zeroes
 * out [T,H], then adds topk_w[t,j] * (A W_down[e])[r,:] to out[t,:] for every row r = row_of[t,j] with
 * packed-bf16 atomic adds (device scope).  Two launches (fill, GEMM).  saved->Yp is NOT written, so a backward
 * cannot follow (d_topk_w needs Yp): an inference path.  Rows of one token meet in no fixed order and every add
 * rounds to bf16: the result equals moe_grouped_gemm + moe_combine up to bf16 rounding of the partial sums, not
 * bit for bit, and is not reproducible bit for bit between runs for tokens with several local slots.
 * bf16 only (MOE_ERR_INVALID_ARG for MOE_F32). */
int moe_grouped_gemm_scatter(const MoeShape* shape, const void* d_w_down, const MoeSaved* saved, void* d_out,
                             void* d_workspace, size_t workspace_bytes, void* stream);

/* The forward pass with that epilogue: routing (whose second launch also zeroes out), Dispatch (or GEMM-1
 * reading x through the permutation when saved is NULL or saved->Xp is NULL), GEMM-1 + SwiGLU, GEMM-2 adding
 * into out; no Combine.  mode MOE_MODE_SERIALIZED: one launch per operator; MOE_MODE_PERSISTENT: Dispatch to
 * GEMM-2 as one launch of tile tasks without COMBINE tasks, so no task waits for the whole chip (alignment
 * rule and moe_ffn_last_status as for moe_ffn_forward).  Other arguments as moe_ffn_forward; same limits as
 * moe_grouped_gemm_scatter. */
int moe_ffn_forward_scatter(const MoeShape* shape, const void* d_x, const float* d_logits, const void* d_w_gate_up,
                            const void* d_w_down, void* d_out, const MoeSaved* saved, void* d_workspace,
                            size_t workspace_bytes, int mode, void* stream);

/* Dispatch to Combine, the interval the paper times (Section 5.2), on the routing results moe_route left in the
 * SAME `saved` and workspace: Dispatch permute, GEMM-1 + SwiGLU, GEMM-2, Combine.  mode MOE_MODE_SERIALIZED: one
 * launch per operator (Section 2.3's kernel-by-kernel execution); MOE_MODE_PERSISTENT: exactly one launch of
 * tile tasks with event counters (Sections 4.3-4.4; alignment rule at the top of this file), which consumes
 * the counters and queues moe_route prepared: one call per moe_route call (a second one finds every ticket
 * taken and does nothing).  Results are bit-identical.  moe_ffn_forward(mode) = moe_route + this, except that
 * its routing launches leave the counters and queues out when mode is MOE_MODE_SERIALIZED (nobody reads them
 * then): MOE_MODE_PERSISTENT here needs a moe_route call, or a MOE_MODE_PERSISTENT forward's routing, in front. */
int moe_dispatch_to_combine(const MoeShape* shape, const void* d_x, const void* d_w_gate_up, const void* d_w_down,
                            void* d_out, const MoeSaved* saved, void* d_workspace, size_t workspace_bytes, int mode,
                            void* stream);

/* ---- SwiGLU + Add microbenchmark (paper Section 6: tile interleaving and L2 reuse, Section 6.1;
 *      static against dynamic scheduling, Section 6.2) ----
 *   S[m,j]   = silu(X[m,j]) * X[m,N+j]      X [M,2N] bf16, S [M,N] bf16 (intermediate, written)
 *   Out[m,j] = S[m,j] + Y[m,j]              Y, Out [M,N] bf16
 * mode 0: two launches, one per operator; mode 1: one launch, row tiles in a static order with the Add
 * tile close behind its SwiGLU tile, event counters; mode 2: one launch, the same tiles pulled from a
 * shared ready queue that finished SwiGLU tiles feed; mode 3: as mode 2 with one ready queue per XCD (a
 * tile's two tasks stay on the XCD that owns the tile).  Results are bit-identical in all modes.
 * tile_rows (1..64) is the number of rows of one tile task (modes 1-3; mode 0 uses it as its loop granule).
 * N must be a multiple of 8, all pointers device and 16-byte aligned; d_workspace >=
 * moe_microbench_workspace_bytes(M).  Modes 1 and 3 hand S tiles over between compute units behind one
 * L2: they require d_s 128-byte aligned and tiles of whole 128-byte lines (tile_rows * N * 2 a multiple
 * of 128), MOE_ERR_INVALID_ARG otherwise, and their workers check (hardware XCC id) that the workgroups of
 * one class (id % 8), which hand tiles to each other, all run on one XCD.
 * The status word reports what went wrong inside a launch: moe_microbench_last_status() (host-blocking
 * 4-byte copy) returns MOE_OK, MOE_ERR_SCHED_TIMEOUT (a bounded wait expired) or MOE_ERR_XCD_PLACEMENT. */
size_t moe_microbench_workspace_bytes(int M);
int moe_microbench_swiglu_add(int M, int N, const void* d_x, const void* d_y, void* d_s, void* d_out, int mode,
                              int tile_rows, void* d_workspace, size_t workspace_bytes, void* stream);
int moe_microbench_last_status(const void* d_workspace);

/*
 * moe_microbench_swiglu_add for callers that cannot allocate device memory or pass a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the event counters and ready
 * rings live in a device array inside the library (394 KB per GPU, held until the process ends) instead
 * of a caller's workspace.  Same arguments, checks, kernels and results as moe_microbench_swiglu_add.
 *   M         at most 32768 (MOE_ERR_UNSUPPORTED_SHAPE beyond)
 *   d_status  nullable device word, 4-byte aligned, caller-owned: receives the launch's status word
 *             (0 ok, bit 0 a bounded wait expired, bit 1 wrong XCD placement); it is zeroed by the call
 * Calls no hipMalloc / hipFree or any allocating routine; only enqueues kernels on `stream`.  The first call
 * on a device looks up the array's address (make it outside graph capture).  All calls on one GPU share the
 * array: each call clears what it needs, and calls that overlap in time on one GPU (two streams) race.
 */
int moe_microbench_swiglu_add_static_scratch(int M, int N, const void* d_x, const void* d_y, void* d_s, void* d_out,
                                             int mode, int tile_rows, uint32_t* d_status, void* stream);

/* ---- Ceiling probes (measurement aids for the benchmark; no step of the layer) ----
 * What this GPU sustains on the two resources the grouped GEMMs and the permute / combine steps are
 * priced against (Section 2.3 judges the operators by hardware utilisation), with nothing
 * else in the way; each only enqueues one kernel on `stream`.
 * moe_probe_mfma_bf16: n_workgroups x 4 waves, each issuing mfma_per_wave (a multiple of 8)
 *   32x32x16 bf16 MFMAs on registers only = n_workgroups * 4 * mfma_per_wave * 32768 flop;
 *   random_operands != 0 uses pseudo-random values in [1, 2) instead of all ones (the sustained rate
 *   depends on the data).  d_sink: 4 bytes of device memory, 4-byte aligned, never written.
 * moe_probe_copy: streaming copy of `bytes` (a multiple of 16; pointers device, 16-byte aligned,
 *   not overlapping).
 * moe_probe_read: the same stream without the stores (read-only); d_sink: 4 bytes of device memory,
 *   4-byte aligned, left unchanged.
 * moe_probe_write: a write-only stream (4 KB per workgroup, plain stores: the fastest pattern found): every
 *   32-bit word of the `bytes` (a multiple of 16, below 8 TB) at d_dst (device, 16-byte aligned) becomes `word`.
 * All return MOE_OK, MOE_ERR_INVALID_ARG or MOE_ERR_LAUNCH. */
int moe_probe_mfma_bf16(int n_workgroups, int mfma_per_wave, int random_operands, void* d_sink, void* stream);
int moe_probe_copy(const void* d_src, void* d_dst, size_t bytes, void* stream);
int moe_probe_read(const void* d_src, size_t bytes, void* d_sink, void* stream);
int moe_probe_write(void* d_dst, size_t bytes, uint32_t word, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_FFN_H_ */
