/*
 * monet.h -- C ABI of the schedule-executed training step for gfx950 (MI355X).
 *
 * The library runs one training step of a conv/BN/ReLU network under a given
 * joint schedule: per-tensor save / recompute bits (s, r) plus one
 * implementation choice per forward, recomputed and backward operator
 * (delta, delta^k, delta-hat).  The forward half is the paper's Algorithm 1
 * (forward pass with greedy freeing and checkpoint set S^N), the backward half
 * its Algorithm 2 (per backward operator k: start from S^k, recompute the
 * nodes with r_i^k = 1, keep S^{k-1}, run backward_k, prune the gradient set).
 * Feasibility is checked at load time against Eq. 7, Eq. 8 and the in-place
 * rules of Appendix C.3; the predicted peak is Eq. 1 / Eq. 5 / Eq. 6 with the
 * L-bar bound of Appendix B.  The schedule solver (Section 4's integer
 * program) is not part of the library: schedules are inputs.
 *
 * Conventions
 *   - All pointers named dev_* / marked "device" are device addresses owned by
 *     the caller; everything else is host memory.
 *   - The library allocates no device memory and never synchronises the
 *     stream: every kernel is enqueued on the stream handed to monet_step.
 *   - Functions returning int / int64_t return a negative monet_status on
 *     failure; monet_last_error() then holds a message naming the violated
 *     constraint or the failing call.  No C++ exception crosses this boundary.
 *   - A plan is not re-entrant: one monet_step at a time per plan.  Beyond that, one step at a
 *     time per process and GPU: convolution launches whose last round of tiles is cut count
 *     their arrivals in one table inside the library, so two steps (of one plan or of two) that
 *     overlap in time on different streams of one GPU would corrupt each other's results.
 *     monet_step zeroes that table at its start, so a step that was broken off by an error
 *     leaves nothing behind for the next one.
 *   - A BatchNorm backward implementation 'from_output' recovers the normalised input as
 *     (y - beta) / gamma (Section 4, "Backward Operator Optimization"): every gamma of such a layer
 *     must be non-zero, otherwise its gradients are not finite.  The library does not check the
 *     values (they live in device memory); a schedule for a model whose gamma may reach zero must
 *     choose 'from_input' for that layer.
 *   - Activations are N,H,W,C fp32; convolution weights K,R,S,C; linear
 *     weights out,in; the ReLU sign code is one bit per element, bit (e & 63) of
 *     little-endian 64-bit word (e >> 6), e = N,H,W,C linear index, tail bits
 *     zero; the max-pool code is one uint8 per output element, r*k+s of the
 *     first maximum of the window under a strict '>' scan.
 */
#ifndef MONET_H
#define MONET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct monet_plan monet_plan;   /* opaque, owned by the library */

enum monet_status {
    MONET_OK = 0,
    MONET_BAD_GRAPH = -1,        /* graph or schedule text does not parse / is inconsistent   */
    MONET_INFEASIBLE = -2,       /* a schedule constraint is violated (named in last_error)   */
    MONET_ARENA_TOO_SMALL = -3,  /* bound arena smaller than monet_plan_arena_bytes           */
    MONET_HIP_ERROR = -4,        /* a HIP call failed                                         */
    MONET_BAD_ARGUMENT = -5
};

/* One record of the alloc / free / run / save trace (all sizes are logical bytes,
 * i.e. element bytes rounded up to 256).
 *   kind   0 ALLOC 1 FREE 2 RUN_FWD 3 RUN_RECOMPUTE 4 RUN_BWD 5 SAVE 6 ALIAS
 *   stage  B+1 for the forward pass (B = number of backward operators), else k
 *   node   tensor's node id (ALLOC/FREE/SAVE/ALIAS), forward node (RUN_FWD/RUN_RECOMPUTE,
 *          forward workspace), backward operator k (RUN_BWD, backward workspace)
 *   impl   implementation index l of a RUN_* record, else -1
 *   aux    ALLOC/FREE: 0 forward tensor, 1 gradient tensor, 2 forward workspace,
 *          3 backward workspace; RUN_FWD/RUN_RECOMPUTE: bit0 in-place, bit1 writes its
 *          intermediate (mask / index) tensor; RUN_BWD: bit p set when the gradient of
 *          input p is accumulated into an existing tensor; ALIAS: the node whose buffer
 *          is taken over
 */
typedef struct monet_event {
    int32_t kind;
    int32_t stage;
    int32_t node;
    int32_t impl;
    int32_t aux;
    int32_t reserved;
    int64_t bytes;
    int64_t live_after;
} monet_event;

/* Parse, validate and lower a (graph, schedule) pair (Algorithms 1 and 2 run symbolically).
 * graph / schedule: host text in the `monet-graph 1` / `monet-schedule 1` formats, not
 * NUL-terminated necessarily (lengths given).  On success *out owns the plan. Host only. */
int monet_plan_load(const char *graph, size_t graph_len,
                    const char *schedule, size_t schedule_len,
                    monet_plan **out);

/* Peak logical live bytes of the step with the exact local sets (Eq. 1, Eq. 5, Eq. 3):
 * equals what monet_step reports. */
int64_t monet_plan_exact_peak(const monet_plan *plan);

/* Upper bound of the paper's memory constraints (Eq. 4 with the L-bar sets of Appendix B
 * and the no-recomputation term of Appendix C.2): always >= the exact peak. */
int64_t monet_plan_predicted_peak(const monet_plan *plan);

/* The same bound with Appendix B's tighter local sets L-dot (before backward stage k only operators up to
 * the stage's own node can be recomputed, so only their inputs count as local):
 * exact peak <= this <= monet_plan_predicted_peak. */
int64_t monet_plan_predicted_peak_tight(const monet_plan *plan);

/* Bytes of device memory the caller must bind: the physical high-water mark of the arena
 * (>= exact peak; the difference is fragmentation) plus the constant part (BatchNorm
 * statistics, loss scalar, reduction scratch). */
int64_t monet_plan_arena_bytes(const monet_plan *plan);

/* Constant part of monet_plan_arena_bytes (not counted in any peak). */
int64_t monet_plan_persistent_bytes(const monet_plan *plan);

/* Hand the plan its device memory: dev_base must be 256-byte aligned device memory of at
 * least monet_plan_arena_bytes bytes, owned by the caller and kept alive while the plan is
 * used. */
int monet_plan_bind_arena(monet_plan *plan, void *dev_base, size_t bytes);

/* Number of parameters / external inputs the graph declares. */
int monet_plan_num_params(const monet_plan *plan);
int monet_plan_num_inputs(const monet_plan *plan);

/* One training step: forward pass (Algorithm 1) then backward pass with recomputation
 * (Algorithm 2), all enqueued on `hip_stream` (a hipStream_t; NULL = default stream).
 *   inputs   host array of device pointers, one per `ext` record in declaration order
 *            (fp32 images N,H,W,C; int32 labels); read-only
 *   weights  host array of device pointers, one per `param` record; read-only
 *   grads    host array of device pointers, same shapes as weights; overwritten
 *   dev_loss device float that receives the loss, or NULL
 * Returns the peak logical live bytes seen by the arena accounting during this step
 * (>= 0), or a negative monet_status. */
int64_t monet_step(monet_plan *plan, void *hip_stream,
                   const void *const *inputs,
                   const float *const *weights,
                   float *const *grads,
                   float *dev_loss);

/* The trace of the last lowering (identical for every step of a plan).  The array is owned
 * by the plan and valid until monet_free. */
int monet_plan_trace(const monet_plan *plan, const monet_event **events, size_t *count);

/* Debug aids (host side, no extra device memory): when on, every freed arena block is
 * filled with a NaN pattern before it can be reused, so a read after free shows up in
 * the results. */
int monet_plan_set_poison(monet_plan *plan, int on);

/* Byte offset (from the bound base) and size of a forward tensor while RUN event
 * `event_index` executes, or -1 if it is not in memory then.  For tests that read
 * intermediate tensors back. */
int64_t monet_plan_tensor_offset(const monet_plan *plan, size_t event_index, int node, int is_grad);

/* Offset of the persistent mean / inverse-std vectors of BatchNorm node `node`
 * (2*C floats, mean first) from the bound base, or -1. */
int64_t monet_plan_bn_stats_offset(const monet_plan *plan, int node);

/* Stop after the event with this index (RUN events only count as executed if at or
 * before it); -1 runs the whole step.  Lets a test stop the step where a tensor it
 * wants to read is still in memory. */
int monet_plan_set_stop_after(monet_plan *plan, int64_t event_index);

/* ---- measurement aids ------------------------------------------------------------
 * One record per operator launch of the step, in execution order.  `flops` and `bytes`
 * are algorithmic figures (2*M*N*K of the contraction; bytes of the tensors the operator
 * must read and write once), used to place measured time against the roofline.
 *   kind  2 forward, 3 recomputation, 4 backward;  id = node (kind 2,3) or backward operator k
 *   label e.g. "conv_fwd", "conv_dgrad", "conv_wgrad" (implicit GEMM; "..._winograd" for the Winograd forms), "bn_fwd", "bn_apply", "bn_bwd",
 *         "relu_fwd", "relu_bwd", "maxpool_fwd", ... */
typedef struct monet_launch_info {
    int32_t kind;
    int32_t id;
    int32_t impl;
    uint32_t flags;
    double flops;            /* algorithmic: the direct form's 2 * multiply-adds */
    double bytes;
    double issued_flops;     /* what the kernels put on the matrix cores: less than `flops` for a Winograd implementation */
    char label[32];
} monet_launch_info;

/* Adjacent bandwidth-bound operators (BatchNorm-apply or add followed by ReLU; ReLU backward followed
 * by BatchNorm backward or by the add's backward) are launched as one fused kernel by default; the
 * trace and the results are the same either way.  Off: one kernel per operator.  The poison and
 * stop-after modes always run unfused. */
int monet_plan_set_fusion(monet_plan *plan, int on);

/* Launch records of the program monet_step currently runs (a fused pair counts once and carries a
 * combined label such as "bn_relu_fwd"). */
int monet_plan_num_launches(const monet_plan *plan);
int monet_plan_launch_info(const monet_plan *plan, size_t index, monet_launch_info *out);

/* When on, monet_step brackets every operator launch with a pair of HIP events on the
 * step's stream (events are created once and reused; no synchronisation is added). */
int monet_plan_set_timing(monet_plan *plan, int on);
/* Waits for the last timed step to finish and writes the elapsed milliseconds of each
 * launch of that step to ms[0..n) (n = monet_plan_num_launches).  Host array. */
int monet_plan_read_timing(monet_plan *plan, float *ms, size_t n);

const char *monet_last_error(void);     /* thread-local, static storage */
void monet_free(monet_plan *plan);

#ifdef __cplusplus
}
#endif
#endif /* MONET_H */
