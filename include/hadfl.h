/*
 * hadfl.h -- C-ABI of libhadfl.so: one HADFL aggregation cycle over N model
 * replicas held in one GPU's memory (Cao et al., "HADFL: Heterogeneity-aware
 * Decentralized Federated Learning Framework", arXiv 2111.08274).
 *
 * A cycle is   hadfl_local_steps -> hadfl_select -> hadfl_aggregate
 * after one    hadfl_init_replicas.
 *
 * Conventions
 *   - Every call returns a hadfl_status; nothing throws or aborts.  Output
 *     arguments are written only on HADFL_OK.  hadfl_last_error() gives text.
 *   - "dev" pointers are device memory owned by the CALLER (allocate them
 *     with any allocator, e.g. PyTorch tensors) and must outlive the context.
 *     "host" pointers are ordinary host memory, read or written during the
 *     call only.  The library owns the host-side context and a few small
 *     pinned staging buffers, nothing else.
 *   - All device work is enqueued on the hipStream_t given at init, in call
 *     order, asynchronously.  The calls that synchronise that stream say so:
 *     every hadfl_get_* and hadfl_set_params / hadfl_set_momentum /
 *     hadfl_set_steps (host arrays cross the boundary), hadfl_aggregate_group,
 *     and hadfl_profile_*.  hadfl_select* with a host mask waits only for the
 *     selection that last used the same staging slot (two calls back).
 *   - No global state and no environment variables; several contexts may
 *     coexist.  Calls on one context must not overlap in time.
 *
 * Data layout
 *   - Activations are channels-last: a batch is [B][H][W][C].
 *   - The parameter vector of a network lists its layers in order; a
 *     convolution contributes weights [kh][kw][Cin][Cout] then bias [Cout]
 *     (if it has one); a dense layer weights [in][out] (in = flattened
 *     H,W,C of its input) then bias; batch normalisation gamma [C] then
 *     beta [C].  After all trainable values come, for every batch-norm layer
 *     in order, running mean [C] and running variance [C].  m_train counts
 *     the trainable values, m_total includes the running statistics.
 *   - Replica k's vector starts at replicas_dev + k*row_stride floats;
 *     row_stride >= m_total is a multiple of 64 (hadfl_param_count); the
 *     padding is kept zero.
 */
#ifndef HADFL_H
#define HADFL_H

#include <stddef.h>
#include <stdint.h>

#ifdef HADFL_BUILD
#define HADFL_API __attribute__((visibility("default")))
#else
#define HADFL_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hadfl_ctx hadfl_ctx;   /* opaque; host memory owned by the library */

typedef enum {
    HADFL_OK = 0,
    HADFL_EINVAL = 1,        /* bad argument: null/misaligned pointer, size out of range, ... */
    HADFL_ENOMEM = 2,        /* host allocation failed */
    HADFL_EDEVICE = 3,       /* a HIP call failed; text in hadfl_last_error */
    HADFL_ESTATE = 4,        /* call out of order (e.g. aggregate before select) */
    HADFL_EUNSUPPORTED = 5   /* valid request the library has no kernel for */
} hadfl_status;

typedef enum {
    HADFL_NET_MLP = 0,       /* 784-128-10, ReLU */
    HADFL_NET_CNN2 = 1,      /* conv3x3(3->32) ReLU pool conv3x3(32->64) ReLU pool FC(4096->10) */
    HADFL_NET_RESNET18 = 2,  /* ResNet-18 for 32x32 inputs (paper Sec. 4.1) */
    HADFL_NET_VGG16 = 3,     /* VGG-16 with batch norm for 32x32 inputs (paper Sec. 4.1) */
    HADFL_NET_NONE = 4,      /* no training: bare parameter rows of m_none values (aggregation only) */
    HADFL_NET_CUSTOM = 5     /* layer list given in custom_ops */
} hadfl_net;

typedef enum {
    HADFL_OP_CONV = 0, HADFL_OP_DENSE = 1, HADFL_OP_RELU = 2, HADFL_OP_MAXPOOL = 3,
    HADFL_OP_BN = 4, HADFL_OP_ADD = 5, HADFL_OP_GAP = 6
} hadfl_op_type;

/* One layer of a custom network.  Layer i reads tensor in0 (and in1 for ADD) and writes tensor i+1;
 * tensor 0 is the input batch.  k/stride/pad: convolution geometry; cout: output channels/features;
 * bias: nonzero if the layer has a bias.  MAXPOOL is 2x2 stride 2; GAP averages over H,W. */
typedef struct { int32_t type, in0, in1, k, stride, pad, cout, bias; } hadfl_op;

typedef struct {
    int32_t n_replicas;      /* K: devices simulated as replicas (Algorithm 1's available set at most) */
    int32_t n_select;        /* N_p: replicas drawn per aggregation (Sec. 3.3) */
    int32_t net;             /* hadfl_net */
    int32_t bf16;            /* 0: fp32 everywhere; 1: bf16 weights/activations, fp32 master + accumulate */
    int32_t batch;           /* B, the same on every replica (Sec. 2.1) */
    int32_t n_samples;       /* samples per replica shard; multiple of batch */
    int32_t in_dim[3];       /* H, W, C of one sample */
    int32_t n_classes;
    float lr;                /* learning rate of the local update (Sec. 2.2) */
    float momentum;          /* 0 gives exactly the paper's update */
    int32_t t_sync;          /* aggregation every t_sync hyperperiods (Sec. 2.3) */
    int32_t steps_per_unit;  /* mini-batch steps per unit of the step-count rule */
    int32_t weight_mode;     /* 0: a_k = Flag_k / sum Flag (the paper's aggregate with unit weight sum);
                                1: extension, a_k = Flag_k f_k / sum Flag f with f of the selection function */
    int32_t n_custom_ops;    /* HADFL_NET_CUSTOM only */
    uint64_t seed;           /* key of the counter-based generator that drives the selection */
    int64_t m_none;          /* HADFL_NET_NONE only: values per replica */
    const hadfl_op *custom_ops;   /* host; copied at init */
} hadfl_config;

typedef struct { int64_t offset, count; int32_t kind, fan_in; } hadfl_tensor_info;
/* kind: 0 weight, 1 bias, 2 gamma, 3 beta, 4 running mean, 5 running variance */

/* Sizes of the parameter vector of cfg's network (layout described at the top). */
HADFL_API hadfl_status hadfl_param_count(const hadfl_config *cfg, int64_t *m_train, int64_t *m_total, int64_t *row_stride);

/* Parameter tensors in vector order.  Writes at most cap rows to out (host) and the full count to *n. */
HADFL_API hadfl_status hadfl_param_layout(const hadfl_config *cfg, hadfl_tensor_info *out, int32_t cap, int32_t *n);

/* Bytes the caller must provide: params_bytes for replicas_dev (n_replicas rows of row_stride floats),
 * scratch_bytes for scratch_dev (momentum, gradients, activations, the aggregate, small state). */
HADFL_API hadfl_status hadfl_workspace_bytes(const hadfl_config *cfg, size_t *params_bytes, size_t *scratch_bytes);

/* Algorithm 1, first line: every replica starts from the same model w0; momentum, batch cursors and versions
 * start at zero.  Also fixes the local step count of every replica (Sec. 2.3, Sec. 3.3):
 *   E_k = t_sync * steps_per_unit * ratio[k] / gcd(ratio), ratio[k] > 0 the computing-power ratio of
 * device k (larger = faster, Sec. 4.1).
 *   w0_dev        dev, [m_total] floats in the layout above; NULL keeps replicas_dev as the caller filled it
 *   replicas_dev  dev, params_bytes, 256-byte aligned
 *   scratch_dev   dev, scratch_bytes, 256-byte aligned; contents need not be initialised
 *   x_dev         dev, [n_replicas][n_samples][H][W][C] floats (NULL for HADFL_NET_NONE)
 *   y_dev         dev, [n_replicas][n_samples] int32 labels in [0, n_classes)
 *   ratio_host    host, [n_replicas] int32
 *   stream        hipStream_t (NULL = the default stream)
 * Errors: EINVAL for null/misaligned pointers, n_select outside [1, n_replicas], ratio <= 0,
 * n_samples % batch != 0, sizes out of range; EUNSUPPORTED for layer shapes without a kernel. */
HADFL_API hadfl_status hadfl_init_replicas(const hadfl_config *cfg, const void *w0_dev, void *replicas_dev,
                                 void *scratch_dev, const void *x_dev, const int32_t *y_dev,
                                 const int32_t *ratio_host, void *stream, hadfl_ctx **out);

/* Algorithm 1, inner loop, for all replicas at once: replica k runs E_k steps, each = next batch of its shard
 * (rows [(c_k*B) mod n_samples, +B), c_k counts its steps since init), forward, softmax cross-entropy averaged
 * over the batch, backward, buf = momentum*buf + g, w = w - lr*buf (local-update equation of Sec. 2.2).
 * The version of replica k becomes the number of steps it completed in this call.
 * Enqueues on the context's stream and returns without waiting.  Weight-gradient kernels run on a second stream the
 * context owns (default priority), forked from and joined back into the context's stream inside the call, so work
 * enqueued on that stream afterwards is ordered after the whole call.  hadfl_set_option(HADFL_OPT_SIDE_STREAM, 0)
 * keeps every launch on the context's stream. */
HADFL_API hadfl_status hadfl_local_steps(hadfl_ctx *ctx);

/* Sec. 3.3, probability-based selection: mu = third quartile of the available replicas' versions,
 * f_k = exp(-(v_k-mu)^2/2), P_k = f_k / sum f; n_select distinct replicas are drawn one after another in
 * proportion to f over those remaining, with uniforms from Philox4x32-10 keyed by cfg.seed at counter
 * (cycle, draw).  The result stays on the device for hadfl_aggregate.
 *   versions_dev  dev, [n_replicas] int32, or NULL for the versions hadfl_local_steps recorded
 *   avail_host    host, [n_replicas] bytes (0 = device absent this round, never selected), or NULL = all; copied
 *                 during the call into one of two pinned staging slots used in turn, so the call waits (on an event,
 *                 not on the whole stream) only if the selection two calls back has not started yet
 * Errors: EINVAL if fewer than n_select replicas are available. */
HADFL_API hadfl_status hadfl_select(hadfl_ctx *ctx, const int32_t *versions_dev, const uint8_t *avail_host, uint64_t cycle);

/* The step-count rule on its own (Sec. 2.3, Sec. 3.3; the rule hadfl_init_replicas applies):
 *   steps_host[k] = t_sync * steps_per_unit * ratio_host[k] / gcd(ratio_host[0..n)).
 * Host arrays only; no context and no GPU work.  EINVAL on a null pointer, n < 1, a non-positive ratio, t_sync or
 * steps_per_unit, or a step count above 2^20. */
HADFL_API hadfl_status hadfl_step_counts(const int32_t *ratio_host, int32_t n, int32_t t_sync, int32_t steps_per_unit,
                                         int32_t *steps_host);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc: the selection of hadfl_select without a context and without a workspace.  The kernel's
 * working memory (the selection function's values and the ascending list of the selected) is a static device array of
 * 16 KiB inside the library, enough for 1024 replicas; the call allocates nothing, on the host or on the device, and
 * creates no stream or event.  It enqueues one kernel on `stream` and returns without waiting.
 *   versions_dev  dev, [n_replicas] int32
 *   avail_dev     dev, [n_replicas] bytes (0 = absent this round), or NULL = all present.  A device array, unlike
 *                 hadfl_select's host mask: there is no staging copy.  If fewer than n_select replicas are present,
 *                 the surplus entries of selected_dev are -1 (the host cannot check a device mask).
 *   n_replicas    in [1, 1024]; EINVAL beyond that, with the limit in hadfl_last_error(NULL)
 *   n_select      in [1, n_replicas]; weight_mode as hadfl_config.weight_mode; seed, cycle as hadfl_select
 *   selected_dev  dev out, [n_select] int32, draw order
 *   flag_dev      dev out, [n_replicas] bytes
 *   weights_dev   dev out, [n_replicas] floats, the aggregation weights a_k
 *   stream        hipStream_t (NULL = the default stream)
 * Every call on one GPU uses that GPU's one array: calls that overlap in time on one GPU (two streams, two threads)
 * race and must be serialised by the caller.  Nothing in the array has to survive between calls and nothing has to be
 * cleared: the kernel writes every entry before it reads it. */
HADFL_API hadfl_status hadfl_select_static(const int32_t *versions_dev, const uint8_t *avail_dev, int32_t n_replicas,
                                           int32_t n_select, int32_t weight_mode, uint64_t seed, uint64_t cycle,
                                           int32_t *selected_dev, uint8_t *flag_dev, float *weights_dev, void *stream);

/* Sec. 3.2 (mutual-negotiation phase) with Sec. 3.3 (hyperperiod): step counts from measured calculation times.
 * Device k reports the time times_host[k] it needed for e_warmup warm-up units.  Its time per unit,
 * times_host[k] / e_warmup, is rounded to the nearest whole number q_k >= 1 of `quantum`; the hyperperiod is
 * H = lcm(q_1..q_n) quanta, and in t_sync hyperperiods device k completes
 *   steps_host[k] = t_sync * steps_per_unit * H / q_k
 * units -- the same counts as hadfl_init_replicas derives from computing-power ratios r_k when times are
 * proportional to 1/r_k.  Host arrays only; no context and no GPU work.
 * Errors: EINVAL on a null pointer, n < 1, a non-positive time, quantum, e_warmup, t_sync or steps_per_unit, or when
 * a step count would exceed 2^20 (quantum too fine for these times). */
HADFL_API hadfl_status hadfl_steps_from_times(const double *times_host, int32_t n, int32_t e_warmup, double quantum,
                                              int32_t t_sync, int32_t steps_per_unit, int32_t *steps_host);

/* Learning rate of the following hadfl_local_steps calls (the warm-up of Sec. 3.2 uses a small one).  EINVAL unless
 * lr > 0; ESTATE for a context without a trainable network. */
HADFL_API hadfl_status hadfl_set_lr(hadfl_ctx *ctx, float lr);

/* Sec. 3.2, a device may complete fewer (or more) local steps in a round than the step-count rule planned: replace
 * every replica's step count E_k for the following hadfl_local_steps calls.
 *   steps_host    host, [n_replicas] int32, each in [0, 2^20]; 0 = the replica sits the round out (version 0)
 * Synchronises the stream.  EINVAL on a value out of range. */
HADFL_API hadfl_status hadfl_set_steps(hadfl_ctx *ctx, const int32_t *steps_host);

/* Sec. 3.2, runtime version forecast by double exponential smoothing: feeds one observation per replica -- the
 * versions recorded by the last hadfl_local_steps, or versions_dev -- into the per-replica states
 *   s1 <- alpha*v + (1-alpha)*s1,  s2 <- alpha*s1 + (1-alpha)*s2   (both start at the first observation)
 * and leaves the forecast `horizon` rounds ahead, (2*s1 - s2) + alpha/(1-alpha)*(s1 - s2)*horizon, on the device
 * (fp64, every operation rounded on its own).
 *   versions_dev  dev, [n_replicas] int32, or NULL
 *   alpha         smoothing factor in (0, 1); horizon in [0, 2^20]
 * Errors: EINVAL on alpha or horizon out of range. */
HADFL_API hadfl_status hadfl_predict_versions(hadfl_ctx *ctx, const int32_t *versions_dev, double alpha, int32_t horizon);

/* Sec. 3.1 step 2 with Sec. 3.3: the selection of the next round drawn from real-valued (forecast) versions; the
 * same rule as hadfl_select with v_k real.
 *   versions_dev  dev, [n_replicas] fp64, or NULL for the forecast left by hadfl_predict_versions
 *   avail_host    as in hadfl_select
 * Errors: ESTATE if versions_dev is NULL and no forecast exists; EINVAL as hadfl_select. */
HADFL_API hadfl_status hadfl_select_real(hadfl_ctx *ctx, const double *versions_dev, const uint8_t *avail_host, uint64_t cycle);

/* Read-back of the last forecast (synchronises the stream).  predicted: host, [n_replicas] fp64.  ESTATE if none. */
HADFL_API hadfl_status hadfl_get_predicted(hadfl_ctx *ctx, double *predicted);

/* Sec. 2.3, partial aggregation over the replicas flagged by the last hadfl_select:
 *   w_agg[j] = sum_k a_k * w_k[j], added in ascending k in fp32,
 * then, if resync != 0, Algorithm 1's global synchronisation: every replica's parameters become w_agg
 * (optimiser state and batch cursors are local and stay).  ESTATE without a preceding hadfl_select. */
HADFL_API hadfl_status hadfl_aggregate(hadfl_ctx *ctx, int32_t resync);

/* Sec. 3.3, last paragraph (many devices are divided into groups; intra-group rounds run separately, the
 * inter-group round -- hadfl_select / hadfl_aggregate over everybody -- every integer multiple of them).
 * hadfl_select_group: the rule of hadfl_select among the members of one group.
 *   member_host   host, [n_replicas] bytes, nonzero = member of the group (and present this round)
 *   n_select      devices to draw, in [1, cfg.n_select]; EINVAL if the group has fewer members; hadfl_get_selected
 *                 then returns them in the first n_select entries
 * hadfl_aggregate_group: the aggregate of the last selection, written to the rows of the given members only
 * (pass the same mask to synchronise the group; synchronises the stream once to stage the row list). */
HADFL_API hadfl_status hadfl_select_group(hadfl_ctx *ctx, const int32_t *versions_dev, const uint8_t *member_host,
                                          int32_t n_select, uint64_t cycle);
HADFL_API hadfl_status hadfl_aggregate_group(hadfl_ctx *ctx, const uint8_t *member_host);

/* Read-back; each synchronises the stream.  All outputs are host arrays. */
HADFL_API hadfl_status hadfl_get_steps(hadfl_ctx *ctx, int32_t *steps /* [n_replicas] E_k */);
HADFL_API hadfl_status hadfl_get_versions(hadfl_ctx *ctx, int32_t *versions /* [n_replicas] */, int64_t *cursors /* [n_replicas] or NULL */);
/* The last selection: its size to *count (cfg.n_select, or the n_select of the last hadfl_select_group) and its
 * members in draw order to selected[0..*count); entries of selected beyond that are left untouched.  selected must
 * have room for cfg.n_select entries; count may be NULL.  ESTATE before the first selection. */
HADFL_API hadfl_status hadfl_get_selected(hadfl_ctx *ctx, int32_t *selected /* [cfg.n_select] */, int32_t *count,
                                uint8_t *flag /* [n_replicas] or NULL */, float *weights /* [n_replicas] a_k or NULL */);
/* replica in [0, n_replicas), or -1 for the last aggregate; n values (<= m_total) in the vector layout */
HADFL_API hadfl_status hadfl_get_params(hadfl_ctx *ctx, int32_t replica, float *out, size_t n);

/* Sec. 3.1, step 4 (model backup): the model manager fetches the latest model (hadfl_get_params, and
 * hadfl_get_momentum for the local optimiser state of Sec. 2.2's update with momentum) and can put it back.
 * hadfl_set_params: the first n values (<= m_total, vector layout) of replica's parameters <- in (host).
 * hadfl_get_momentum / hadfl_set_momentum: the momentum buffer of replica, n <= m_train values in the order of the
 * trainable part of the vector; ESTATE when the context trains without momentum or has no trainable network.
 * replica in [0, n_replicas).  Each synchronises the stream; the next hadfl_local_steps starts from the new state. */
HADFL_API hadfl_status hadfl_set_params(hadfl_ctx *ctx, int32_t replica, const float *in, size_t n);
HADFL_API hadfl_status hadfl_get_momentum(hadfl_ctx *ctx, int32_t replica, float *out, size_t n);
HADFL_API hadfl_status hadfl_set_momentum(hadfl_ctx *ctx, int32_t replica, const float *in, size_t n);

/* Execution options of one context (they change how the work is issued, never a bit of the result):
 *   HADFL_OPT_SIDE_STREAM  1 (default): weight-gradient kernels of hadfl_local_steps run on a second stream owned by
 *                          the context; 0: every launch goes to the context's stream
 *   HADFL_OPT_TILE_HINT    0 (default): tile shapes chosen per launch; 1: the bf16 / fp32 lean convolution kernels take
 *                          their 256-row tiles wherever the layer shape allows, whatever the launch size; 2: layers on
 *                          16- and 32-pixel-wide images stay on the general kernels
 * Takes effect from the next hadfl_local_steps.  EINVAL for an unknown option or value; ESTATE without a
 * trainable network. */
typedef enum { HADFL_OPT_SIDE_STREAM = 0, HADFL_OPT_TILE_HINT = 1 } hadfl_option;
HADFL_API hadfl_status hadfl_set_option(hadfl_ctx *ctx, int32_t option, int32_t value);
HADFL_API hadfl_status hadfl_get_losses(hadfl_ctx *ctx, float *loss /* [n_replicas] batch-mean loss of each replica's last step */);

/* Per-kernel timing with HIP events on the context's stream.  While enabled, every kernel launch is bracketed
 * by events (this serialises nothing but adds overhead: use a separate pass from throughput timing).  on = 2
 * additionally tags every name with the layer index and the number of active replicas ("conv_fwd:L12:n16").
 * hadfl_profile_read synchronises, then writes up to cap rows: name (<= 47 chars), launches, total ms, and the
 * algorithmic work of those launches: flops (2 per multiply-add of the layer's definition; 0 for memory-bound
 * kernels) and bytes (each operand and result counted once per launch). */
typedef struct { char name[48]; int64_t launches; double total_ms; double flops; double bytes; } hadfl_kernel_time;
HADFL_API hadfl_status hadfl_profile_enable(hadfl_ctx *ctx, int32_t on);
HADFL_API hadfl_status hadfl_profile_read(hadfl_ctx *ctx, hadfl_kernel_time *out, int32_t cap, int32_t *n);

HADFL_API const char *hadfl_last_error(const hadfl_ctx *ctx);   /* ctx may be NULL: error of the last failed init on this thread */
HADFL_API void hadfl_destroy(hadfl_ctx *ctx);                   /* frees host state only; NULL is a no-op */

#ifdef __cplusplus
}
#endif
#endif /* HADFL_H */
