/*
 * mtsched - staged, multi-stream forward pass of several CNN tenants on one MI355X.
 *
 * C ABI of the library.  The calls follow the problem statement of
 * "Automated Runtime-Aware Scheduling for Multi-Tenant DNN Inference on GPU"
 * (arXiv 2111.14255), Sec. III: N independent models, each a serial operator
 * sequence (Eq. 1) bound to its own GPU stream (Eq. 2); per-model pointers
 * (Eq. 3) split the sequences into stages (Eqs. 4-5) separated by
 * synchronisation barriers; the list of stages is the schedule (Eq. 6); a
 * profile-driven search over the pointer matrix (Eq. 8, Alg. 1) picks the
 * schedule with the lowest makespan (Sec. III-A: earliest start to latest end).
 *
 * Conventions
 *  - Every call returns an int32_t status: MT_OK (0) or a negative mt_status.
 *    After a failure mt_last_error() returns a description (thread-local).
 *  - Handles are opaque and owned by the library; destroy them with the
 *    matching *_destroy call.  Passing NULL where a handle is required is
 *    MT_ERR_INVALID_ARG.
 *  - "host" pointers are ordinary CPU memory, borrowed for the duration of the
 *    call and copied if needed.  "device" pointers are HIP device memory of
 *    the context's GPU, borrowed and never freed by the library.
 *  - Activations are NHWC.  Convolution weights are K-R-S-C (output channel,
 *    filter row, filter column, input channel); depthwise weights are C-R-S;
 *    fully-connected weights are K-J with J = H*W*C of the input flattened in
 *    H,W,C order.  Weights are given in the model's storage type, bias in fp32.
 *  - Arithmetic: products of storage-type values accumulated in fp32; bias,
 *    residual and activation applied in fp32; one round-to-nearest-even to the
 *    storage type on store.  The result of an operator does not depend on the
 *    schedule, stream, CU share or co-running operators: outputs are
 *    bit-identical across all schedules of the same tenants.
 *  - One context is used from one host thread at a time (the paper issues all
 *    operators from a single main thread, Sec. III-D).
 */
#ifndef MTSCHED_H
#define MTSCHED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MT_MAX_TENANTS 16
#define MT_MAX_STAGES 16

typedef struct mt_ctx mt_ctx;
typedef struct mt_model mt_model;
typedef struct mt_schedule mt_schedule;

typedef enum mt_status {
    MT_OK = 0,
    MT_ERR_INVALID_ARG = -1,
    MT_ERR_INVALID_SCHEDULE = -2,
    MT_ERR_SHAPE_MISMATCH = -3,
    MT_ERR_OUT_OF_MEMORY = -4,
    MT_ERR_HIP = -5,
    MT_ERR_NOT_FINALIZED = -6
} mt_status;

typedef enum mt_dtype { MT_F32 = 0, MT_F16 = 1, MT_BF16 = 2 } mt_dtype;

/* Operator kinds named by the paper's problem statement (Sec. III-A: conv, bn, relu, pooling);
 * bn is folded into the preceding convolution's weights and relu is an epilogue flag. */
typedef enum mt_op_kind {
    MT_CONV = 0,
    MT_DWCONV = 1,
    MT_MAXPOOL = 2,
    MT_AVGPOOL = 3,          /* divisor = number of in-bounds taps */
    MT_GLOBAL_AVGPOOL = 4,
    MT_FC = 5,
    MT_LRN = 6,              /* across-channel local response normalisation (the AlexNet paper's form, its Sec. 3.3) */
    MT_ADD = 7               /* out = act(in + res): a shortcut sum that is an operator of its own */
} mt_op_kind;

typedef enum mt_act { MT_ACT_NONE = 0, MT_ACT_RELU = 1, MT_ACT_RELU6 = 2 } mt_act;

typedef enum mt_issue_order { MT_ISSUE_BFS = 0, MT_ISSUE_DFS = 1 } mt_issue_order;

/* One operator of a model's serial sequence (Sec. III-B, Eq. 1).
 * Tensors are named by integers; tensor 0 is the model input.  out = floor((in + 2*pad - k)/stride) + 1. */
typedef struct mt_op_desc {
    int32_t kind;          /* mt_op_kind */
    int32_t in_tensor;     /* must have been written by an earlier operator (or be 0) */
    int32_t res_tensor;    /* CONV: tensor added before the activation, -1 = none; ADD: the second summand (required) */
    int32_t out_tensor;    /* >= 1 and at most 2 * (operators of the model) + 16 */
    int32_t out_c;         /* CONV / FC: output channels; ignored otherwise */
    int32_t out_c_offset;  /* first channel written inside out_tensor (channel concatenation without a copy) */
    int32_t out_c_total;   /* channel count of out_tensor; 0 = exactly the channels written */
    int32_t r, s;          /* window (CONV, DWCONV, pools); ignored for GLOBAL_AVGPOOL, FC, ADD; LRN: r = channels in the window (odd) */
    int32_t stride_h, stride_w;
    int32_t pad_h, pad_w;  /* symmetric per axis; max-pool padding is never selected */
    int32_t act;           /* mt_act; CONV, DWCONV, FC, ADD */
    int32_t groups;        /* CONV: independent channel groups (0 or 1 = ordinary convolution); group g maps input
                              channels [g*C/G, (g+1)*C/G) to output channels [g*K/G, (g+1)*K/G); weights are
                              [out_c][r][s][C/G].  One operator of the sequence, issued as G launches */
    float lrn_alpha;       /* LRN: out[c] = in[c] / (lrn_k + lrn_alpha * sum_{|j-c| <= r/2} in[j]^2) ^ lrn_beta; */
    float lrn_beta;        /*      lrn_alpha is not divided by the window size */
    float lrn_k;
} mt_op_desc;

/* What the library derived for one operator; lets a harness compute roofline figures
 * from the library's own view of the graph. */
typedef struct mt_op_info {
    int32_t kind;
    int32_t in_h, in_w, in_c;
    int32_t out_h, out_w, out_c;     /* channels written */
    int32_t kernel_id;               /* which device kernel family and tile runs it (see mt_kernel_name) */
    int32_t split_k;                 /* K-splits of the implicit GEMM (1 = none) */
    int32_t grid_blocks;             /* workgroups launched */
    double flops;                    /* 2 * multiply-accumulates, whole batch */
    double bytes;                    /* algorithmic traffic: inputs + weights + bias (+ residual) read once, output written once */
} mt_op_info;

typedef struct mt_device_info {
    int32_t cu_count;
    int32_t wavefront_size;
    int32_t lds_bytes_per_block;
    int32_t clock_khz;
    int64_t l2_bytes;
    int64_t hbm_bytes;
    char name[64];
    char arch[64];
} mt_device_info;

/* Timings of one mt_run, from HIP events recorded on the device.
 * makespan_ms: from the event recorded before the first operator of any tenant may start to the latest of the
 * events that the streams of the last stage record after their last operator (Sec. III-A objective: earliest start to
 * latest end); under MT_SCHED_GRAPH, the events around the graph launch.
 * stage_ms[s]: from the previous barrier (or the start) to the barrier that ends stage s.
 * host_issue_ms: wall time the issuing thread spent launching (Sec. III-D "invoking overhead").
 * first_op_done_ms[i]: only with MT_SCHED_TIME_FIRST_OP, else 0: from the start to the end of tenant i's first
 * operator, i.e. how long stream i was held back by the issue of the streams before it (Sec. III-D, Fig. 5).
 * tenant_done_ms[i]: only with MT_SCHED_TIME_TENANTS, else 0: from the start to the end of tenant i's last operator,
 * the latency of model i inside the multi-tenant run (the makespan is the largest of them, up to the final barrier). */
typedef struct mt_timings {
    float makespan_ms;
    float host_issue_ms;
    int32_t n_launches;
    int32_t n_stages;
    float stage_ms[MT_MAX_STAGES];
    float first_op_done_ms[MT_MAX_TENANTS];
    int32_t n_fused;       /* operators (of the n_launches issued) that ran inside another launch: a neighbouring operator's (fused pairs) or, under co-issue, the same operator of another tenant */
    float tenant_done_ms[MT_MAX_TENANTS];
} mt_timings;

/* ---- error reporting ---------------------------------------------------------------- */
const char *mt_last_error(void);
const char *mt_kernel_name(int32_t kernel_id);

/* ---- context ------------------------------------------------------------------------ */
/* Binds to HIP device `device`, creates the main stream and timing events. */
int32_t mt_create(int32_t device, mt_ctx **out);
int32_t mt_destroy(mt_ctx *ctx);
/* Destroys the pooled CU-masked streams that no schedule refers to (a share search leaves its winner's streams in the
 * pool for the schedule created next).  Synchronises the device. */
int32_t mt_release_idle_streams(mt_ctx *ctx);
int32_t mt_get_device_info(const mt_ctx *ctx, mt_device_info *out);

/* Diagnostic: which compute units a stream restricted to `share` units starting at unit `first_cu` (same rule as
 * mt_schedule_create's cu_share; share 0 = unmasked) really runs on.  Launches n_groups one-wavefront workgroups that
 * each record the hardware id registers of the unit they run on.  hw_ids: host [n_groups][2] = (HW_ID, XCC_ID) raw
 * register values (CU_ID = bits 8-11, SH_ID = bit 12, SE_ID = bits 13-15 of HW_ID; XCC_ID = low 4 bits). */
int32_t mt_probe_cu_mask(mt_ctx *ctx, int32_t share, int32_t first_cu, int32_t n_groups, uint32_t *hw_ids);

/* Diagnostic: what one stage barrier (Sec. III-B "Stage") costs on the tenant streams of this context.  n_streams
 * streams each run `rounds` rounds of one one-workgroup kernel; between rounds they are synchronised by
 *   kind 0  nothing (the reference: n_streams independent chains),
 *   kind 1  the barrier mt_run uses: every stream records an event and waits for the events of all others,
 *   kind 2  stream memory operations: every stream writes the round number to a word of its own
 *           (hipStreamWriteValue32) and waits until the words of all others have reached it (hipStreamWaitValue32, >=);
 *           all writes of a round are queued before any wait, so streams that share a hardware queue cannot block
 *           each other,
 *   kind 3  a counter: every stream launches a one-thread kernel that adds 1 to a shared word, then waits once until the
 *           word has reached round * n_streams (hipStreamWaitValue32, >=): 2 n runtime calls instead of n^2,
 *   kind 4  events through the main stream: every stream records an event, the main stream waits for all of them and
 *           records one, every stream waits for that: 3 n + 1 runtime calls.
 *   Kinds 2 and 3 give MT_ERR_HIP if the device does not support stream memory operations.
 * us_per_round: host float, the mean time of one round over all streams (the barrier's cost is the difference to
 * kind 0).  n_streams 1 .. MT_MAX_TENANTS, rounds 1 .. 4096. */
int32_t mt_probe_barrier_cost(mt_ctx *ctx, int32_t n_streams, int32_t kind, int32_t rounds, float *us_per_round);

/* Diagnostic: creates n_streams streams (each restricted to `share` units, 0 = unmasked), keeps them all alive, and
 * measures on each the mean time of `n_launches` dependent one-workgroup kernels issued while the context's main
 * stream waits for the stream's completion event (the pattern of a stage).  us_per_launch: host [n_streams]. */
int32_t mt_probe_dispatch_latency(mt_ctx *ctx, int32_t n_streams, int32_t share, int32_t n_launches, float *us_per_launch);

/* Diagnostic: which streams of this process can run side by side.  Creates n_streams unmasked streams (2 .. 32; they are
 * destroyed before the call returns) and measures the mean time per launch of `n_launches` (1 .. 256) dependent
 * one-workgroup kernels on each stream alone (single_us: host [n_streams]) and, for every pair, the mean time of a
 * round in which both streams launch one such kernel (pair_us: host [n_streams * n_streams], symmetric, the diagonal
 * repeats single_us).  A pair that takes about two single launches per round is served one stream at a time. */
int32_t mt_probe_stream_conflicts(mt_ctx *ctx, int32_t n_streams, int32_t n_launches, float *single_us, float *pair_us);

/* Diagnostic: what the chip sustains on a register-only loop of 32x32x16 matrix instructions (dtype MT_F16 or MT_BF16;
 * two workgroups of four waves per compute unit, four independent accumulators per wave, 4 * iters instructions per
 * wave; iters 1 .. 2^20).  tflops: host scalar, 2 * 32 * 32 * 16 flops per instruction over the kernel's event time.
 * Allocates and frees a small device buffer.  The figure to hold next to the published peak when a kernel's fraction
 * of the matrix-core roofline is read. */
int32_t mt_probe_peak_mfma(mt_ctx *ctx, int32_t dtype, int32_t iters, float *tflops);
/* Diagnostic: sustained device-memory rate of a plain kernel.  mode 0 copies `bytes` bytes (16-byte pieces, grid-stride,
 * eight pieces in flight per thread, groups_per_unit workgroups of 256 threads per compute unit, 1 .. 256) and counts
 * 2 * bytes per launch, mode 1 only reads them and counts bytes.  bytes: multiple of 16 between 1 MiB and 8 GiB (choose
 * it well above the last-level cache); reps launches (1 .. 1000) are timed after as many warm-up launches.
 * gbytes_per_s: host scalar.  Allocates and frees its buffers (MT_ERR_OUT_OF_MEMORY if it cannot). */
int32_t mt_probe_peak_stream(mt_ctx *ctx, int32_t mode, size_t bytes, int32_t groups_per_unit, int32_t reps, float *gbytes_per_s);

/* ---- model construction (host only; no GPU needed) ----------------------------------- */
/* Operators are added in the serial order that becomes the model's sequence M_i (Eq. 1). */
int32_t mt_model_begin(int32_t dtype, int32_t batch, int32_t in_h, int32_t in_w, int32_t in_c, mt_model **out);
int32_t mt_model_add_op(mt_model *m, const mt_op_desc *desc, int32_t *out_op_index);
/* Shape inference and validation: every input produced earlier, window fits, channel ranges agree. */
int32_t mt_model_end(mt_model *m);
int32_t mt_model_destroy(mt_model *m);
int32_t mt_model_num_ops(const mt_model *m, int32_t *out);
int32_t mt_model_op_info(const mt_model *m, int32_t op_index, mt_op_info *out);
int32_t mt_model_out_features(const mt_model *m, int64_t *out);
/* w: host, storage type, layout as above, exactly w_bytes bytes; bias: host fp32 [n_bias] or NULL (zeros). */
int32_t mt_model_set_weights(mt_model *m, int32_t op_index, const void *w, size_t w_bytes,
                             const float *bias, size_t n_bias);
/* Bytes of device memory a registered copy of the model needs (weights, activations, workspaces). */
int32_t mt_model_arena_bytes(const mt_model *m, size_t *out);

/* Batch-norm folding helper (graph-level fusion, Sec. II-A(b)); fp32, in place.
 * w: host [k][per_k]; gamma/beta/mean/var: host [k]; bias_out: host [k].
 * w[k][:] *= gamma[k]/sqrt(var[k]+eps);  bias_out[k] = beta[k] - mean[k]*gamma[k]/sqrt(var[k]+eps). */
int32_t mt_fold_bn(float *w, int64_t k, int64_t per_k, const float *gamma, const float *beta,
                   const float *mean, const float *var, float eps, float *bias_out);

/* Cast to the storage type (the numeric reading taken where the paper states no precision: values are stored as
 * fp16 or bf16 with one round-to-nearest-even, NaN kept quiet, or as fp32 unchanged).  Host only.
 * src: host [n] floats; dst: host [n] elements of the storage type (2 or 4 bytes each). */
int32_t mt_round_to_storage(const float *src, int64_t n, int32_t dtype, void *dst);

/* ---- registration -------------------------------------------------------------------- */
/* Uploads a finalised model with all weights set and makes it tenant `*out_tenant` (0, 1, ...)
 * of the context.  device_arena: device memory of at least mt_model_arena_bytes() bytes, 256-byte
 * aligned, borrowed until mt_destroy; NULL lets the library allocate.  The model handle may be
 * destroyed afterwards. */
int32_t mt_register(mt_ctx *ctx, const mt_model *m, void *device_arena, size_t arena_bytes, int32_t *out_tenant);
int32_t mt_num_tenants(const mt_ctx *ctx, int32_t *out);
int32_t mt_tenant_num_ops(const mt_ctx *ctx, int32_t tenant, int32_t *out);
int32_t mt_tenant_op_info(const mt_ctx *ctx, int32_t tenant, int32_t op_index, mt_op_info *out);
/* Debug aid: copies tensor `tensor_id` of a tenant (as left by the last run) to host memory. */
int32_t mt_tenant_read_tensor(mt_ctx *ctx, int32_t tenant, int32_t tensor_id, void *host_dst, size_t bytes);

/* ---- schedule (Sec. III-B) ----------------------------------------------------------- */
/* pointers: host [n_tenants][n_stages-1], row i non-decreasing, 0 <= value <= length of M_i.  A pointer is
 * the 1-based index of the last operator of a stage (Eq. 3); the last stage takes the remainder; equal
 * neighbours give an empty slice (Eq. 5, "None").  n_tenants must equal the number of registered tenants.
 * stage_concurrency: host [n_stages] or NULL (= n_tenants each).  In a stage with concurrency c at least as large
 * as the number of tenants that have work, every tenant is issued on its own stream (the paper's one stream per
 * model).  With a smaller c the streams of tenant indices 0 .. c - 1 are used and the tenants with work are dealt
 * to them longest first: in descending order of the operator count of their slice (ties: lower index) each goes to
 * the stream that holds the fewest operators so far (ties: lowest stream); a stream issues its tenants in tenant
 * order.  c = 1 runs them one after another on one stream (the sequential baseline).
 * cu_share: host [n_tenants] or NULL.  Number of compute units tenant i's stream may use; 0 = all.  The ranges are
 * laid out one after another (tenant i starts where tenant i-1 ended, modulo the unit count), so shares that sum to
 * at most the unit count are disjoint.  A share between 1 and 7 is rejected with MT_ERR_INVALID_SCHEDULE: consecutive
 * mask bits fall on the 8 XCDs in turn and the runtime refuses a mask that leaves an XCD without a unit.
 * issue_order: MT_ISSUE_BFS issues one operator per stream round-robin (Sec. III-D), MT_ISSUE_DFS stream by stream.
 * flags: MT_SCHED_GRAPH captures the whole schedule into a HIP graph on the first run and replays it
 * afterwards (CU shares are ignored in that mode: graph nodes do not inherit stream CU masks).  A replay has no issue
 * order, only the capture has one; a schedule of several tenants is captured in both orders on that first run, each
 * graph is replayed three times and the faster one is kept (on this runtime one of the two is sometimes several times
 * slower), so that run takes about ten passes. */
#define MT_SCHED_GRAPH 1
/* MT_SCHED_PARALLEL_ISSUE: one issuing host thread per tenant stream instead of the paper's single main thread
 * (Sec. III-D); the operators of a stage are launched by the threads of its streams concurrently, stage barriers and
 * results are unchanged.  Not combinable with MT_SCHED_GRAPH. */
#define MT_SCHED_PARALLEL_ISSUE 2
/* MT_SCHED_TIME_FIRST_OP: records one more event per tenant, after its first operator, and reports it in
 * mt_timings.first_op_done_ms.  Only with the single issuing thread on plain streams (neither flag above). */
#define MT_SCHED_TIME_FIRST_OP 4
/* MT_SCHED_SHARE_PER_STAGE: cu_share holds n_stages * n_tenants entries, row s = the shares of stage s; a tenant then
 * runs each stage on the pooled stream of that stage's share (the stage barrier orders them).  Without the flag
 * cu_share holds n_tenants entries used in every stage. */
#define MT_SCHED_SHARE_PER_STAGE 8
/* MT_SCHED_FUSE_DEPTHWISE: a 3x3 depthwise convolution whose consumer is a 1x1 convolution issued in the same stage
 * (on the 64x16 tile, unsplit) runs inside that convolution's launch: same arithmetic in the same order, so the
 * outputs, the intermediate tensor included, have the same bits as two launches.  Opt-in: one workgroup then computes
 * the depthwise output of its 16 pixels alone, which on small maps takes as long as the two launches it replaces. */
#define MT_SCHED_FUSE_DEPTHWISE 16
/* MT_SCHED_FUSE_EXPAND: a 1x1 convolution (stride 1, no residual, fp16 / bf16, output channels a multiple of 8) whose
 * output only the next operator reads, a 3x3 depthwise convolution with padding 1 and stride 1 or 2 issued in the same
 * stage, runs with it in one launch: the first two operators of the chain 1x1 -> depthwise -> 1x1 of an inverted
 * residual block.  Needs three rows of the map to fit one workgroup: width * 3 <= 512 pixels with at most 64 input
 * channels, <= 256 with at most 128, <= 64 with at most 256.  Same arithmetic in the same order as the two launches,
 * so every output, both intermediate tensors included, keeps its bits.  With MT_SCHED_FUSE_DEPTHWISE also set, a
 * depthwise operator joins its producer when it can and its consumer otherwise. */
#define MT_SCHED_FUSE_EXPAND 64
/* MT_SCHED_FUSE_POOL: a convolution on the matrix cores (fp16 / bf16, no residual, output channels a multiple of 8, even
 * output height and width) whose output only the next operator reads, a 2x2 max pooling with stride 2 issued in the
 * same stage, applies the pooling in its epilogue: the convolution walks its output pixels window by window and
 * writes the pooled tensor only.  The pooled tensor keeps its bits (activation and rounding are monotonic, so the
 * maximum commutes with them); the convolution's own output tensor is NOT written by such a launch. */
#define MT_SCHED_FUSE_POOL 128
/* MT_SCHED_PRIORITIZE_SHORT: the waves of short, latency-bound kernels (64x16-tile convolutions, depthwise, pooling,
 * normalisation, add, small matrix-vector layers, fused pairs of them) raise their issue priority on the SIMD to the
 * maximum; long kernels keep the default.  A short kernel of one tenant that shares a compute unit with a long kernel
 * of another then issues first.  Timing only, results unchanged.  (This is the priority of a wave among the waves of
 * its SIMD, set by the kernel itself; stream and queue priorities are never used.) */
#define MT_SCHED_PRIORITIZE_SHORT 256
/* MT_SCHED_TIME_TENANTS: records one more event per tenant, after its last operator, and reports it in
 * mt_timings.tenant_done_ms.  Works with the single issuing thread and with MT_SCHED_PARALLEL_ISSUE, with or without CU
 * shares; not with MT_SCHED_GRAPH or MT_SCHED_STREAM_GRAPHS (events inside a captured graph cannot be queried). */
#define MT_SCHED_TIME_TENANTS 512
/* MT_SCHED_HOST_BARRIER (only with MT_SCHED_PARALLEL_ISSUE): the barrier between stages is taken on the host.  The
 * issuing thread of a stream waits (hipEventSynchronize) for the events that the other streams recorded at the end of
 * the stage before and launches its operators of the stage after that, instead of queueing a device-side wait in
 * front of them.  Same ordering, same results; the launches of a stage can no longer be queued while the stage before
 * still runs, but no queue sits in a wait, which on this machine slows the dispatch of the queues that still work. */
#define MT_SCHED_HOST_BARRIER 1024
/* MT_SCHED_STREAM_GRAPHS: the launches of one stream in one stage are captured (on that stream, on the first run
 * and again when a buffer pointer changes) into a graph of their own and replayed on that stream: the short gaps
 * between kernels of a replayed graph, with CU shares still in force (the replay runs on the masked stream) and with
 * per-stage timings (the stage barriers stay ordinary events).  Not combinable with MT_SCHED_GRAPH,
 * MT_SCHED_PARALLEL_ISSUE or MT_SCHED_TIME_FIRST_OP. */
#define MT_SCHED_STREAM_GRAPHS 32
/* MT_SCHED_COUNTER_BARRIER: the barrier between stages (Sec. III-B "Stage") is taken with one counter word per run instead
 * of events: at the end of a stage every stream of the stage launches a one-thread kernel that adds 1 to the word, and a
 * stream of a later stage waits, with one hipStreamWaitValue32 packet on its queue, until the word has reached the number
 * of streams that ended the stages before.  2 n runtime calls per barrier instead of n + n (n - 1) event records and
 * waits; the stage's events are still recorded for the timings.  Same ordering, same results.  Works with the single
 * issuing thread and with MT_SCHED_PARALLEL_ISSUE (the arrivals of a stage are queued before any wait for them, so
 * streams that share a hardware queue cannot block each other); not with MT_SCHED_GRAPH, MT_SCHED_STREAM_GRAPHS or
 * MT_SCHED_HOST_BARRIER.  MT_ERR_HIP from mt_schedule_create if the device has no stream memory operations. */
#define MT_SCHED_COUNTER_BARRIER 2048
/* Co-issue (an issue mechanism of this runtime; the paper issues one launch per operator, Sec. III-D): where a stage
 * puts several tenants on one stream (stage_concurrency below the number of tenants with work), the stream would run
 * the first tenant's slice, then the second's, and so on.  With this flag up to four neighbouring tenants of a stream
 * whose slices cover the same operator range are walked together: operator i of all of them runs as ONE launch whose
 * workgroups are split between the tenants, wherever the operators have the same kernel and launch shape as the first
 * tenant's (same architecture and batch: everything in their kernel arguments but the buffers is equal) and the kernel
 * has a several-operator form (every kernel of the 16-bit storage types that works on 16-byte vectors; not grouped
 * convolutions, and not operators that run as a fused pair of their own tenant); the other operators are launched
 * one tenant after the other inside the same walk.  Every operator computes exactly what it computes alone (same tile
 * program, same split, same summation order), so outputs are bit-identical; what changes is the number of launches the
 * command processor has to dispatch and complete, which is what bounds many small kernels on several streams.  Such a
 * launch runs at the wave priority of the first of its tenants.  mt_timings.n_fused counts the operators that ran
 * inside another tenant's launch.  Not with MT_SCHED_GRAPH, MT_SCHED_STREAM_GRAPHS or MT_SCHED_TIME_FIRST_OP. */
#define MT_SCHED_COISSUE 4096
int32_t mt_schedule_create(mt_ctx *ctx, int32_t n_tenants, int32_t n_stages, const int32_t *pointers,
                           const int32_t *stage_concurrency, const int32_t *cu_share,
                           int32_t issue_order, int32_t flags, mt_schedule **out);
/* Wave priority per tenant (host array of n_tenants entries): 0..3 = every kernel of that tenant raises its waves to
 * that issue priority, -1 = the rule of MT_SCHED_PRIORITIZE_SHORT for that tenant.  Replaces what the flags set;
 * graphs captured so far are dropped and captured again on the next run.  Timing only. */
int32_t mt_schedule_set_wave_priority(mt_schedule *s, const int32_t *prio);
int32_t mt_schedule_destroy(mt_schedule *s);

/* Host-only views of the schedule generation function T(G, rho) (Eq. 8) and of the launch order (Sec. III-D).
 * lens: host [n_tenants] sequence lengths.  slices_out: host [n_stages][n_tenants][2], 0-based half-open. */
int32_t mt_expand_pointers(int32_t n_tenants, const int32_t *lens, int32_t n_stages, const int32_t *pointers,
                           int32_t *slices_out);
/* slices: host [n_tenants][2] of one stage.  order_out: host [sum of slice lengths][3] = (stream, tenant, op). */
int32_t mt_issue_order_of_stage(int32_t n_tenants, const int32_t *slices, int32_t concurrency,
                                int32_t issue_order, int32_t *order_out, int32_t *n_out);

/* ---- run ----------------------------------------------------------------------------- */
/* inputs: host array of n_tenants device pointers, tenant i's [batch,H,W,C] input in its storage type
 * (may alias).  outputs: host array of n_tenants device pointers receiving the last operator's tensor.
 * Blocks until every tenant has finished.  t may be NULL. */
int32_t mt_run(mt_ctx *ctx, mt_schedule *s, const void *const *inputs, void *const *outputs, mt_timings *t);

/* mt_run for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): the same pass on the same streams with the same kernels, but the partial-sum workspaces and
 * arrival counters of every operator whose reduction is split over workgroups are taken from a fixed array of
 * MT_STATIC_SCRATCH_BYTES bytes of device memory that the library's code object holds on every GPU it is loaded on,
 * instead of from the tenants' arenas.  The call allocates nothing on the device: no hipMalloc, no hipFree, no graph
 * instantiation, no stream creation; the schedule must have been created without MT_SCHED_GRAPH,
 * MT_SCHED_STREAM_GRAPHS and MT_SCHED_PARALLEL_ISSUE (their first run captures graphs or starts threads):
 * MT_ERR_INVALID_ARG otherwise.  The counters' part of the array is cleared by a fill kernel at the start of each call
 * (not a memset node, so that a caller may capture the call); workspaces need no clearing.  If the tenants together
 * need more than the array holds the call fails with MT_ERR_OUT_OF_MEMORY before anything is launched, and
 * mt_last_error states both figures.  Outputs have the bits of mt_run.  All calls on one GPU share the array, which
 * keeps the last call's contents: two calls that overlap in time on one GPU (from two contexts or two host threads)
 * race on it and must be serialised by the caller.  inputs / outputs / t as for mt_run. */
#define MT_STATIC_SCRATCH_BYTES (16u << 20)
int32_t mt_run_static_scratch(mt_ctx *ctx, mt_schedule *s, const void *const *inputs, void *const *outputs, mt_timings *t);

/* Measurement aid: runs each operator of one tenant `repeats` times back to back on one stream between
 * two events and reports the mean duration per launch.  op_ms: host [num ops]. */
int32_t mt_profile_ops(mt_ctx *ctx, int32_t tenant, const void *input, void *output, int32_t repeats, float *op_ms);

/* ---- search (Sec. III-C, Alg. 1) ------------------------------------------------------ */
typedef enum mt_search_algo { MT_SEARCH_COORDINATE = 0, MT_SEARCH_RANDOM = 1 } mt_search_algo;

typedef struct mt_search_opts {
    int32_t algo;          /* mt_search_algo */
    int32_t n_stages;      /* P + 1 */
    int32_t rounds;        /* R.  Random search evaluates rounds * n_tenants * candidates matrices. */
    int32_t candidates;    /* M candidate rows per (round, model) */
    int32_t runs;          /* timed runs per candidate (the profiling step of Alg. 1's inner loop); the cost is their median */
    int32_t warmup;        /* untimed runs per candidate */
    int32_t issue_order;   /* mt_issue_order */
    int32_t flags;         /* schedule flags used while profiling */
    int32_t seed_baselines; /* non-zero: before Alg. 1 starts, also profile and record (a) the matrix whose pointers all equal
                              len_i (every operator in stage 1: the stream-parallel baseline) and (b) the even split
                              (Alg. 1's start point).  An addition to the printed algorithm; with it the returned schedule is
                              never worse than stream-parallel under the same profiler. */
    int32_t cu_share_rounds; /* mt_search only: > 0 runs that many rounds of the CU-share descent (below) after the pointer search */
    int32_t wave_priority_rounds; /* mt_search only: > 0 runs that many rounds of the wave-priority descent (below) last */
    int32_t search_concurrency; /* mt_search only: non-zero also tries 2 .. n_tenants - 1 streams per stage (the same in every
                                   stage) under the pointers found, before shares and priorities */
    int32_t playoff_top;   /* mt_search only: > 0 ends the pointer search with a play-off (mt_playoff_pointers) over that many
                              of the best records plus the one-stage matrix, each measured again with playoff_runs runs */
    int32_t playoff_runs;  /* timed runs per play-off candidate (median); values below 1 mean 21 */
    uint64_t seed;
} mt_search_opts;

/* cost callback: pointers is host [n_tenants][n_stages-1]; returns the latency to minimise. */
typedef double (*mt_cost_fn)(const int32_t *pointers, void *user);

/* The search itself, on any cost function (host only).  Candidate rows are n_stages-1 draws, uniform on
 * [0, len_i], sorted; draws come from a counter-based generator keyed by (seed, round, model, candidate, j).
 * best_pointers: host [n_tenants][n_stages-1].  rec_pointers / rec_cost: optional host buffers for the record
 * memory D (every evaluated matrix and its cost, in evaluation order), capacity max_records. */
int32_t mt_search_pointers(int32_t n_tenants, const int32_t *lens, const mt_search_opts *opts,
                           mt_cost_fn cost, void *user, int32_t *best_pointers, double *best_cost,
                           int32_t *rec_pointers, double *rec_cost, int32_t max_records, int32_t *n_records);

/* Play-off over a record memory (an addition: Alg. 1 ends by returning the best record as it was profiled once, and two
 * schedules a few percent apart cannot be told apart by one short measurement).  Host only, any cost function.
 * Candidates, in this order: the top_k distinct matrices of the records by (cost, position), then the matrix whose
 * pointers all equal len_i (every operator in stage 1) unless it is one of them.  Each candidate is measured with
 * `cost` (meant to be a longer measurement than the one that filled the records); the lowest wins, the earlier
 * candidate on ties.  rec_pointers: host [n_records][n_tenants][n_stages-1]; rec_cost: host [n_records];
 * best_pointers: host [n_tenants][n_stages-1]; n_evaluated (optional): number of candidates measured. */
int32_t mt_playoff_pointers(int32_t n_tenants, const int32_t *lens, int32_t n_stages, const int32_t *rec_pointers,
                            const double *rec_cost, int32_t n_records, int32_t top_k, mt_cost_fn cost, void *user,
                            int32_t *best_pointers, double *best_cost, int32_t *n_evaluated);

/* Per-tenant CU share as one more coordinate per tenant (an extension; the paper leaves resource sharing to the
 * hardware, Sec. III-A(b)).  Host only, any cost function.  Start: the share vector passed in best_share (all zeros =
 * every tenant on all units).  Each round visits the tenants in order; for a tenant the candidates k * cu_count / 8,
 * k = 1..7, are evaluated with the other shares fixed, and the candidate replaces the tenant's share if its cost is
 * lower than the best cost so far.
 * share_cost: cost of a share vector (host [n_tenants]).  best_share: host [n_tenants], in = start, out = best found;
 * *best_cost: in = cost of the start vector, out = best cost found. */
typedef double (*mt_share_cost_fn)(const int32_t *cu_share, void *user);
int32_t mt_search_cu_share(int32_t n_tenants, int32_t cu_count, int32_t rounds, mt_share_cost_fn share_cost, void *user,
                           int32_t *best_share, double *best_cost);

/* Wave priority per tenant as one more coordinate per tenant (an extension, see mt_schedule_set_wave_priority).  Host
 * only, any cost function of the same shape as for the shares.  Start: the vector passed in best_prio.  Each round
 * visits the tenants in order; for a tenant the values -1, 0, 1, 2, 3 other than its current one are evaluated with the
 * other entries fixed, and a value replaces the tenant's entry if its cost is lower than the best cost so far; the
 * search stops after a round that changed nothing.  best_prio: host [n_tenants], in = start, out = best found;
 * *best_cost: in = cost of the start vector, out = best cost found. */
int32_t mt_search_wave_priority(int32_t n_tenants, int32_t rounds, mt_share_cost_fn prio_cost, void *user,
                                int32_t *best_prio, double *best_cost);

/* A disjoint start vector for the share search: the units are dealt out in eighths of cu_count; every tenant owns one eighth,
 * the 8 - n_tenants spare eighths go to the tenants in proportion to weight[] (host [n_tenants], >= 0, e.g. the serial
 * latency of each tenant) by largest remainder, lower index first on ties; with more than 8 tenants every share is one
 * eighth (the ranges then overlap).  share: host [n_tenants]. */
int32_t mt_proportional_cu_share(int32_t n_tenants, int32_t cu_count, const double *weight, int32_t *share);

/* The same searches with the profiled makespan of mt_run as cost (median of opts->runs timed runs after opts->warmup
 * untimed ones), all tenants on their own stream.  With opts->playoff_top > 0 the pointer search ends with
 * mt_playoff_pointers over its records (cost = median of opts->playoff_runs runs), and the play-off's winner and cost
 * replace the best record; the records returned to the caller are those of the search itself.
 * best_cu_share: host [n_tenants] or NULL; filled with zeros unless opts->cu_share_rounds > 0.  With
 * opts->cu_share_rounds > 0 three phases run: the pointer search on unmasked streams (the only phase written to the
 * records); the share descent under those pointers, started from the best of all-zero shares,
 * mt_proportional_cu_share of the tenants' serial latencies and two uniform vectors (every tenant one half, or three
 * quarters, of the units: overlapping shares); and, if a share came out non-zero and n_stages > 1, the
 * pointer search once more under those shares, kept only when its best cost is lower.  A masked result is measured
 * again on fresh streams before it is returned (they stay in the context's pool, so a schedule created next with the
 * same shares runs on exactly those streams); if it does not beat the unmasked result there, the unmasked pointers and
 * all-zero shares are returned.
 * best_wave_priority: host [n_tenants] or NULL; with opts->wave_priority_rounds > 0 the priority descent runs last,
 * under the pointers and shares found, from the vector the flags give (all 0, or all -1 with
 * MT_SCHED_PRIORITIZE_SHORT); if shares were found, a second descent runs under the unmasked result of the pointer
 * search, and that result (all-zero shares) is returned when it ends lower.  Without the descent the vector the flags
 * give is returned as it is.
 * best_concurrency: host [n_stages] or NULL; the stage concurrency the result was measured with (n_tenants in every
 * stage unless opts->search_concurrency found fewer streams faster); pass it to mt_schedule_create. */
int32_t mt_search(mt_ctx *ctx, const mt_search_opts *opts, const void *const *inputs, void *const *outputs,
                  int32_t *best_pointers, int32_t *best_concurrency, int32_t *best_cu_share, int32_t *best_wave_priority, double *best_cost,
                  int32_t *rec_pointers, double *rec_cost, int32_t max_records, int32_t *n_records);

#ifdef __cplusplus
}
#endif
#endif /* MTSCHED_H */
