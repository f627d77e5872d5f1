/*
 * moe_ffn.h -- C ABI of the MI355X (gfx950) Dispatch-to-Combine MoE-FFN library.
 *
 * One GPU's expert-parallel share of a top-k Mixture-of-Experts feed-forward
 * layer, as decomposed in the paper's Section 2.2 (Figure 2): Dispatch (permute
 * tokens into expert-contiguous order), grouped GEMM-1 (gate and up
 * projections), SwiGLU, grouped GEMM-2 (down projection), Combine (accumulate
 * the top-k contributions weighted by the routing scores), and the seven-node
 * backward graph.  The layer can run as one kernel launch per operator
 * ("serialized", the paper's kernel-by-kernel baseline of Section 2.3) or as a
 * single persistent launch that executes a static tile task list with
 * event-counter dependencies (the paper's Sections 4.3-4.4).
 *
 * Conventions
 *   - Every pointer named d_* or documented "device" is device (HBM) memory on
 *     the current HIP device; everything else is host memory.
 *   - All tensors are row-major and contiguous.  Device pointers must be
 *     16-byte aligned.
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
  MOE_ERR_SCHED_TIMEOUT = -5      /* persistent scheduler: a bounded wait expired */
} MoeStatus;

typedef enum MoeDtype { MOE_F32 = 0, MOE_BF16 = 1 } MoeDtype;

typedef enum MoeMode {
  MOE_MODE_SERIALIZED = 0, /* one launch per operator, stream ordered */
  MOE_MODE_PERSISTENT = 1  /* one launch, tile tasks + event counters  */
} MoeMode;

/*
 * Problem shape.  Limits: 1 <= k <= 16, k <= E <= 256, 1 <= E_local <= 256,
 * 0 <= expert_base, expert_base + E_local <= E, H and I multiples of 64,
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
 *                        token_of (Section 4.2: no extra trip through HBM), other cases
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
 *   mode       MoeMode
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

/* ---- Stage entry points (the serialized path's operators, one launch each;
 *      used by the unit tests and the benchmark).  Same buffers as above. ---- */

/* Routing + Dispatch bookkeeping (paper Section 2.2, routing; Section 5.1,
 * tile offsets derived from the routing result at run time): fills topk_idx, topk_w, counts, offsets, row_of,
 * token_of, slot_of of `saved` and the tile map in the workspace. */
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
 * moe_microbench_workspace_bytes(M).  A bounded wait that expires is reported by the status word:
 * moe_microbench_last_status() (host-blocking 4-byte copy) returns MOE_OK or MOE_ERR_SCHED_TIMEOUT. */
size_t moe_microbench_workspace_bytes(int M);
int moe_microbench_swiglu_add(int M, int N, const void* d_x, const void* d_y, void* d_s, void* d_out, int mode,
                              int tile_rows, void* d_workspace, size_t workspace_bytes, void* stream);
int moe_microbench_last_status(const void* d_workspace);

/* ---- Ceiling probes (measurement aids for the benchmark; no step of the layer) ----
 * What this GPU sustains on the two resources the grouped GEMMs and the permute / combine steps are
 * priced against (Section 5.1 evaluates the operators against hardware utilisation), with nothing
 * else in the way; both only enqueue one kernel on `stream`.
 * moe_probe_mfma_bf16: n_workgroups x 4 waves, each issuing mfma_per_wave (a multiple of 8)
 *   32x32x16 bf16 MFMAs on registers only = n_workgroups * 4 * mfma_per_wave * 32768 flop;
 *   random_operands != 0 uses pseudo-random values in [1, 2) instead of all ones (the sustained rate
 *   depends on the data).  d_sink: 4 bytes of device memory, 4-byte aligned, never written.
 * moe_probe_copy: streaming copy of `bytes` (a multiple of 16; pointers device, 16-byte aligned,
 *   not overlapping).
 * Both return MOE_OK, MOE_ERR_INVALID_ARG or MOE_ERR_LAUNCH. */
int moe_probe_mfma_bf16(int n_workgroups, int mfma_per_wave, int random_operands, void* d_sink, void* stream);
int moe_probe_copy(const void* d_src, void* d_dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_FFN_H_ */
