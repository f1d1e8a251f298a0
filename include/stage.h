/*
 * stage.h -- C ABI of the MI355X pipeline-stage F/B/W engine.
 *
 * One pipeline stage = a stack of identical pre-norm transformer decoder
 * layers living on one GPU.  Following the paper's block decomposition
 * (section 3.1 "Computation Blocks"; Appendix B "Weight Gradient Separation"),
 * the work of a microbatch is exposed as three separately schedulable ops:
 *
 *   F  forward,                          stashes activations
 *   B  input-gradient backward (the paper's D / DGrad: dX = dY W^T per linear)
 *   W  weight-gradient backward (WGrad: dW += X^T dY per linear), frees the stash
 *
 * and a schedule is a per-stage ordered list of such ops (the "per-stage
 * schedule S_d" that the paper's generators emit, Alg. 1; section 3.3 "schedule
 * dependencies").  Activations are cached in F and released after B and W
 * (section 3.2); the number of microbatches whose stash is live is bounded by
 * `stash_cap`, the on-device memory constraint of section 4.1.  With
 * `enforce_mb_order` the list must also satisfy the paper's "Microbatch Order
 * within Stage and Type" constraint (section 4.1), which makes accumulated
 * gradients bit-reproducible across schedules.
 *
 * Conventions
 *   - Every pointer named *_dev is DEVICE memory owned by the caller; the
 *     library never allocates or frees device memory.  `ops`, config structs
 *     and all out-parameters are HOST memory.
 *   - All device work is enqueued on the HIP stream given to stage_init and the
 *     calls return without synchronising (no host synchronisation and no device
 *     allocation inside any call, so a schedule can be captured into a HIP graph).  The caller synchronises that stream
 *     before reading y / dx / gradients.  x and dy are copied into the stash
 *     when their op is enqueued (stream order), so they may be reused after
 *     the op's position in the stream has been reached.
 *   - Row-major everywhere.  A boundary tensor of one microbatch is
 *     [mb_size, seq, hidden] contiguous in the compute dtype (fp32 or bf16).
 *   - Threads: calls that use the same stage_t (or stages sharing one stash) must not
 *     overlap.  Different stages may be driven from different threads; the one-time
 *     per-kernel set-up (raising a kernel's LDS limit, reading the CU count) is
 *     done once, thread-safely.  One process drives one GPU.
 *   - Return value: 0 on success, a negative STAGE_E_* code otherwise.  A call
 *     that returns STAGE_E_INVAL / _ORDER / _STASH_FULL has enqueued nothing
 *     and changed no state.  STAGE_E_HIP (a failed launch) is sticky.
 */
#ifndef PAPER_2507_00217_STAGE_H
#define PAPER_2507_00217_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct stage stage_t; /* opaque */

enum { STAGE_F = 0, STAGE_B = 1, STAGE_W = 2 };                 /* op kinds */
enum { STAGE_NORM_LAYERNORM = 0, STAGE_NORM_RMSNORM = 1 };
enum { STAGE_ACT_GELU = 0, STAGE_ACT_SWIGLU = 1 };               /* GELU is the exact erf form */
enum { STAGE_DTYPE_FP32 = 0, STAGE_DTYPE_BF16 = 1 };

enum {
  STAGE_OK = 0,
  STAGE_E_INVAL = -1,      /* null pointer, bad shape, unsupported head_dim, mb out of range */
  STAGE_E_ORDER = -2,      /* F twice, B before F or twice, W before B or twice, mb-order violation */
  STAGE_E_STASH_FULL = -3, /* F while stash_cap microbatches are live; B while recompute_cap hold a rebuilt stash */
  STAGE_E_HIP = -4         /* a kernel launch or runtime call failed */
};

/* Parameter ids of one layer, in storage order. */
enum {
  STAGE_P_NORM1_GAMMA = 0, STAGE_P_NORM1_BETA = 1, STAGE_P_WQKV = 2, STAGE_P_WO = 3,
  STAGE_P_NORM2_GAMMA = 4, STAGE_P_NORM2_BETA = 5, STAGE_P_WIN = 6, STAGE_P_WOUT = 7,
  STAGE_P_BQKV = 8, STAGE_P_BO = 9, STAGE_P_BIN = 10, STAGE_P_BOUT = 11,   /* linear biases, present when cfg.bias */
  STAGE_P_COUNT = 12
};

/* One op of a per-stage schedule: (type, microbatch) -- the paper's compute-op
 * id (stage, chunk, type, microbatch) reduced to one stage and one chunk. */
typedef struct { int32_t kind; int32_t mb; } stage_op_t;

typedef struct {
  int32_t n_layers;
  int32_t hidden;          /* d; multiple of 64 */
  int32_t n_heads;         /* h; head_dim (d / h unless given below) must be 64 or 128 */
  int32_t n_kv_heads;      /* divides n_heads (grouped-query attention when smaller) */
  int32_t ffn;             /* f; multiple of 64 */
  int32_t seq;             /* s */
  int32_t mb_size;         /* b sequences per microbatch; attention never mixes them */
  int32_t n_microbatches;
  int32_t norm;            /* STAGE_NORM_* */
  int32_t act;             /* STAGE_ACT_*  */
  int32_t causal;          /* 1: token t attends to tokens <= t of its own sequence */
  int32_t dtype;           /* STAGE_DTYPE_*; weight-gradient accumulators are fp32 in both */
  int32_t stash_cap;       /* max microbatches live (F started, W not finished); 0 = n_microbatches */
  int32_t enforce_mb_order;/* 1: ops of one kind must come in increasing microbatch index */
  float   norm_eps;        /* e.g. 1e-5 */
  int32_t n_sub;           /* sub-blocks per op (the paper's n_sub, section 4.2.1): each covers n_layers / n_sub
                              consecutive layers; 0 or 1 = whole ops only; must divide n_layers; at most 32 */
  int32_t recompute;       /* 1: layer-wise activation recomputation (section 7.2, Case 2 of the memory / batch-size
                              trade-off): F keeps only every layer's fp32 input; B runs a layer's forward again
                              (minus its last GEMM) right before that layer's backward, into a full-size slot that
                              the microbatch holds from its first B sub-block to its last W.  Results are bit-identical
                              to recompute = 0. */
  int32_t recompute_cap;   /* recompute = 1: max microbatches holding such a full-size slot (B started, W not
                              finished); 0 = stash_cap; at most stash_cap.  Must be 0 when recompute = 0. */
  int32_t head_dim;        /* width of one head, 64 or 128; 0 = hidden / n_heads.  With n_heads * head_dim != hidden the
                              stage computes one tensor-parallel share of a layer (the paper's per-GPU shapes at TP > 1:
                              fewer heads and a narrower ffn against the full hidden width): WQKV is
                              [d, (h + 2 h_kv) head_dim] and WO [h head_dim, d].  Summing the shares' outputs is the
                              caller's collective. */
  float   rope_theta;      /* > 0: rotary position embedding on q and k (Llama-style layers, which is what the paper
                              trains): pairs (2p, 2p+1) of a head turn by position * rope_theta^(-2p / head_dim),
                              position = index in the sequence; 0 = none */
  int32_t bias;            /* 1: every linear map carries a bias vector (GPT-style layers; Llama-style ones, which the
                              paper trains, have none): y = x W + b.  The bias gradients -- column sums of the dZ
                              tensors -- are accumulated by B, like the norm parameters'. */
} stage_config_t;

typedef struct { size_t weights, grads, stash, workspace; } stage_sizes_t; /* bytes */

/* Host only (no GPU needed). Bytes the caller must allocate for stage_init.
 * stash = stash_cap slots of equal size; under recomputation stash_cap small slots (layer inputs) followed by
 * recompute_cap full-size ones. */
int stage_query_sizes(const stage_config_t* cfg, stage_sizes_t* out);

/* Host only. Checks an op list against the microbatch state machine
 *   EMPTY --F--> FWD --B--> BWD --W--> EMPTY
 * starting from all-EMPTY, the stash cap and (if enabled) the microbatch-order
 * rule.  On failure *first_bad_index is the offending position.  *peak_live is
 * the largest number of live microbatches reached by the legal prefix.
 * The list need not be complete. Either out-pointer may be NULL. */
int stage_validate_schedule(const stage_config_t* cfg, const stage_op_t* ops, int n_ops,
                            int* first_bad_index, int* peak_live);

/* Host only. Where parameter `param_id` of `layer` lives inside the flat
 * weights buffer (compute dtype) and the flat grads buffer (fp32): same element
 * offset in both.  Linear weights are stored [in, out] row-major so that
 * forward is A.W:  WQKV [d, d_q+2*d_kv] (columns q | k | v; d_q = h*head_dim),  WO [d_q, d],
 * WIN [d, f] (GELU) or [d, 2f] (SwiGLU, columns gate | up),  WOUT [f, d];
 * norm vectors have rows = 1, cols = d; bias vectors rows = 1, cols = the map's output width.  A parameter the
 * config does not have (beta under RMSNorm, biases without cfg.bias) reports rows = cols = 0. */
int stage_param_layout(const stage_config_t* cfg, int layer, int param_id,
                       size_t* offset_elems, int64_t* rows, int64_t* cols);

/* Creates a stage over caller-allocated device buffers of at least the
 * queried sizes (256-byte aligned) and a caller-owned hipStream_t (may be
 * NULL for the default stream).  Weights must already be in weights_dev (or be
 * written there, in stream order, before the first op).  Zeroes grads_dev. */
int stage_init(const stage_config_t* cfg, void* weights_dev, void* grads_dev, void* stash_dev,
               void* workspace_dev, void* hip_stream, stage_t** out);

/* F(mb): y = layers(x); stashes what B and W need. x_dev, y_dev: [mb_size, seq, hidden]. */
int stage_forward(stage_t* st, int mb, const void* x_dev, void* y_dev);
/* B(mb): dx = d<y,dy>/dx; accumulates norm-parameter (and bias) gradients; keeps the dZ
 * tensors W needs inside the stash slot. */
int stage_backward_input(stage_t* st, int mb, const void* dy_dev, void* dx_dev);
/* W(mb): grads += A^T dZ for the four linear maps of every layer; releases the slot. */
int stage_backward_weight(stage_t* st, int mb);

/* Runs an ordered op list.  The whole list is validated against the current
 * state before anything is enqueued.  *_all: [n_microbatches, mb_size, seq,
 * hidden]; op (kind, mb) uses slice mb.  Leftover live microbatches carry over
 * to the next call, so an iteration may be fed in pieces. */
int stage_run_schedule(stage_t* st, const stage_op_t* ops, int n_ops,
                       const void* x_all_dev, const void* dy_all_dev, void* y_all_dev, void* dx_all_dev);

/* Sub-block ops (paper section 4.2.1: each F / D / W block is cut into n_sub sub-blocks so that a schedule can fill
 * bubbles at a finer grain).  Sub-block `sub` covers layers [sub, sub+1) * n_layers / n_sub.  Per microbatch:
 *   F(mb, sub) in the order sub = 0, 1, ...; the first takes a stash slot (STAGE_E_STASH_FULL applies to it);
 *   B(mb, sub) after every F(mb, .), in the order sub = n_sub-1, ..., 0;
 *   W(mb, sub) any time after B(mb, sub), each once; the last one releases the slot.
 * A whole op (stage_forward, ...) equals its sub-blocks issued back to back in that order, bit for bit.
 * x is read by F(mb, 0) and y written by F(mb, n_sub-1); dy is read by B(mb, n_sub-1) and dx written by B(mb, 0);
 * the other pointer of a call may be NULL.  With enforce_mb_order the microbatch-order rule applies per (kind, sub). */
typedef struct { int32_t kind; int32_t mb; int32_t sub; } stage_subop_t;
int stage_validate_subschedule(const stage_config_t* cfg, const stage_subop_t* ops, int n_ops,
                               int* first_bad_index, int* peak_live);
int stage_forward_sub(stage_t* st, int mb, int sub, const void* x_dev, void* y_dev);
int stage_backward_input_sub(stage_t* st, int mb, int sub, const void* dy_dev, void* dx_dev);
int stage_backward_weight_sub(stage_t* st, int mb, int sub);
int stage_run_subschedule(stage_t* st, const stage_subop_t* ops, int n_ops,
                          const void* x_all_dev, const void* dy_all_dev, void* y_all_dev, void* dx_all_dev);

/* Several model chunks on one device (paper section 3.1: an op is identified by (stage, chunk, type, microbatch); looped
 * and V-shaped placements such as interleaved 1F1B or ZB-V put two chunks on a device).  A chunk is a stage_t of its
 * own -- own weights, gradients and microbatch states -- that shares the stash of the stage it is attached to: slots come
 * from one pool and stash_cap (and recompute_cap) bound the live microbatches of all chunks together.  The chunk's config
 * must give the same slot size and caps as share_with's (in practice: the same shape); it uses share_with's stash and
 * stream.  workspace_dev is a workspace of the chunk's own (stage_query_sizes of ITS config), or share_with's when the
 * chunk needs no more than that one holds and uses the same rotary table (same seq, head_dim, rope_theta; one stream
 * orders all uses) -- anything else returns STAGE_E_INVAL.  Destroy in any order. */
int stage_init_chunk(const stage_config_t* cfg, void* weights_dev, void* grads_dev, void* workspace_dev, stage_t* share_with,
                     stage_t** out);
/* One op of a per-device schedule over chunks: sub = -1 for a whole op, else the sub-block. */
typedef struct { int32_t kind; int32_t mb; int32_t sub; int32_t chunk; } stage_chunkop_t;
/* Host only: like stage_validate_subschedule, for n_chunks chunks of the given config sharing its caps;
 * *peak_live counts live microbatches over all chunks. */
int stage_validate_chunk_schedule(const stage_config_t* cfg, int n_chunks, const stage_chunkop_t* ops, int n_ops,
                                  int* first_bad_index, int* peak_live);
/* Runs an op list over chunks[0..n_chunks) (all attached to one stash; op.chunk indexes this array).  The whole list is
 * validated first, shared caps included.  x_all_dev[c] ... dx_all_dev[c] are chunk c's boundary tensors, laid out as for
 * stage_run_schedule (HOST arrays of device pointers; an entry may be NULL if no op of the list needs it). */
int stage_run_chunk_schedule(stage_t* const* chunks, int n_chunks, const stage_chunkop_t* ops, int n_ops,
                             const void* const* x_all_dev, const void* const* dy_all_dev, void* const* y_all_dev,
                             void* const* dx_all_dev);

/* Borrowed pointer to the fp32 gradient buffer (== grads_dev) and its length.
 * After a full iteration it holds the SUM over microbatches of d<Y_m,dY_m>/dtheta.  A microbatch's contribution arrives
 * in two parts: B adds the norm-parameter (and bias) gradients, W the linear weights', so the buffer is complete for a
 * microbatch only after its W, and stage_zero_grads belongs between iterations (no microbatch between its B and its W). */
int stage_grads(stage_t* st, float** grads_dev, size_t* n_elems);
int stage_zero_grads(stage_t* st);

/* Counters: live microbatches now (of this chunk), their peak since init and the peak stash bytes in use (slots of both
 * kinds) -- over all chunks when the stash is shared. */
int stage_stats(stage_t* st, int* live, int* peak_live, size_t* peak_stash_bytes);

/* Kernel selection for debugging and A/B measurements: 0 = tuned gfx950 kernels
 * (MFMA GEMM / fused attention where the dtype has them), 1 = plain reference
 * HIP kernels for every step.  Both run on the GPU. */
int stage_set_kernel_set(stage_t* st, int which);

/* Per-launch timing by kernel class, with HIP events recorded on the stage's
 * stream around every launch while enabled (costs two event records per launch,
 * so use a separate, untimed pass).  stage_profile(st, 1) clears earlier records
 * and starts; stage_profile(st, 0) stops and clears.  stage_profile_read
 * synchronises the stream and returns, for one class, the summed duration in
 * ms, the number of launches, and the summed algorithmic work: FLOPs (2MNK per
 * GEMM; 2*b*s^2*d causal / 4*b*s^2*d full per attention forward, 2.5x that for
 * backward) for classes 0-4, bytes moved by definition for classes 5-10. */
enum {
  STAGE_K_GEMM_NN = 0, STAGE_K_GEMM_NT = 1, STAGE_K_GEMM_TN = 2, STAGE_K_ATTN_FWD = 3, STAGE_K_ATTN_BWD = 4,
  STAGE_K_NORM_FWD = 5, STAGE_K_NORM_BWD = 6, STAGE_K_ACT_FWD = 7, STAGE_K_ACT_BWD = 8, STAGE_K_COPY = 9,
  STAGE_K_ROPE = 10, STAGE_K_COUNT = 11
};
int stage_profile(stage_t* st, int enable);
int stage_profile_read(stage_t* st, int kernel_class, double* total_ms, int64_t* launches, double* work);

void stage_destroy(stage_t* st);
const char* stage_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif
