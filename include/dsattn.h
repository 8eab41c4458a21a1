/*
 * dsattn — Dual-scope temporal self-attention for gfx950 (MI355X), C ABI.
 *
 * The operation is the DualScope attention of Video-Infinity (arXiv 2406.16260,
 * Section 4.2) under the clip split of Section 4 / 4.1, with all clips of the
 * long video resident in one device buffer: the context a clip needs from its
 * neighbours (c_pre, c_post) and from the whole video (c_global) is gathered by
 * frame index instead of being exchanged between devices (Section 4.1,
 * three-round context communication; Appendix, Algorithm 1).
 *
 * Notation (the paper's): N clips of F_clip frames, F = N * F_clip; per layer
 * the latent is [F, H', W', C'] (Section 3), here flattened to [F, P, C] with
 * P = H' * W' spatial positions and C = heads * head_dim, C fastest, contiguous.
 * Q, K, V (already projected) and O all have this layout.
 *
 * Clip i's key/value frame list ("context list") is
 *     local  = frames [i*F_clip - w, (i+1)*F_clip + w) intersected with [0, F), ascending
 *     global = global_idx[0 .. n_global), in the caller's order
 *     ctx(i) = Concat(local, global)          (duplicates are kept and count twice)
 * and every query frame of clip i, at every position and head, performs plain
 * softmax attention (scale * q.k, no mask) over exactly the frames of ctx(i).
 *
 * Conventions for every entry point
 *   - returns DSATTN_OK (0) or a negative dsattn_status; never throws or aborts;
 *   - pointers marked "host" are host memory, "device" are device memory of the
 *     plan's device; the caller owns all tensors, the library owns the plan;
 *   - work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call does not synchronise;
 *   - arguments are validated before anything is launched.
 */
#ifndef DSATTN_H
#define DSATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum dsattn_status {
    DSATTN_OK = 0,
    DSATTN_EINVAL = -1,       /* null pointer, non-positive size, index out of range, aliasing */
    DSATTN_EUNSUPPORTED = -2, /* no kernel for this combination */
    DSATTN_ENOMEM = -3,       /* host or device allocation failed */
    DSATTN_EHIP = -4,         /* a HIP runtime call failed; see dsattn_last_error() */
    DSATTN_ENODEVICE = -5     /* the plan was made host-only (device = -1) */
} dsattn_status;

typedef enum dsattn_dtype { DSATTN_F32 = 0, DSATTN_BF16 = 1 } dsattn_dtype;

/* dsattn_desc.flags */
#define DSATTN_FLAG_FORCE_GENERIC 1u /* planner must pick the generic vector-ALU kernel */
#define DSATTN_FLAG_SLIDING_WINDOW 2u /* local keys are also limited to |frame - query frame| <=
                                         dsattn_desc.window (Section 4.2: the local context as the
                                         neighbouring frames of the query frame) */

#define DSATTN_FLAG_DEDUP_GLOBAL 4u   /* set union instead of concatenation (Section 4.2 writes the
                                         key set of a query as the union of its local neighbours and
                                         the global frames): a global entry whose frame the query
                                         already sees, as a visible local key or as an earlier
                                         global entry, is dropped, so that no frame counts twice */

/* Problem statement, in the paper's terms. */
typedef struct dsattn_desc {
    int32_t clip_len;   /* F_clip >= 1                              (Section 4) */
    int32_t n_clips;    /* N >= 1; F = N * clip_len                  (Section 4) */
    int32_t local_ctx;  /* w >= 0: frames taken from each neighbouring side,
                           |c_pre| = |c_post| = w                    (Section 4.2) */
    int32_t spatial;    /* P = H' * W' >= 1                          (Section 3) */
    int32_t heads;      /* h >= 1 */
    int32_t head_dim;   /* D >= 1; C = h * D */
    int32_t io_dtype;   /* dsattn_dtype of Q, K, V; accumulation is always fp32 */
    int32_t out_dtype;  /* dsattn_dtype of O (F32 input requires F32 output) */
    float scale;        /* softmax scale; <= 0 selects 1/sqrt(D) */
    uint32_t flags;     /* DSATTN_FLAG_* */
    float bias_local;   /* scope weights (Section 5.1: the weights of the frames of N and of G are */
    float bias_global;  /* adjusted per timestep), as additive logit biases of the local / global
                           keys: logit_j = scale * q.k_j + bias; finite; 0 = the plain method */
    int32_t window;     /* with DSATTN_FLAG_SLIDING_WINDOW: radius r >= 0; a local key frame f is
                           visible to the query of frame a iff |f - a| <= r (global keys always
                           are); ignored without the flag */
} dsattn_desc;

typedef struct dsattn_plan_s dsattn_plan_t; /* opaque; made by dsattn_plan() */

/* What the launch planner decided for dsattn_forward (read-only report). */
typedef struct dsattn_launch_info {
    int32_t kernel;          /* 0 = generic vector-ALU kernel, 1 = bf16 MFMA streaming kernel */
    int32_t heads_per_wave;  /* MFMA kernel: heads handled by one wavefront */
    int32_t local_tiles;     /* MFMA kernel: 16-key tiles covering the local scope of a query tile */
    int32_t global_tiles;    /* MFMA kernel: 16-key tiles covering the global set */
    int32_t clips_per_task;  /* consecutive 16-frame query tiles walked by one wavefront (whole clips
                                when clip_len is 16; the generic kernel: 1 clip) */
    int32_t n_tasks;         /* wavefront tasks = grid size */
    int32_t block_threads;   /* threads per workgroup */
    int32_t lds_bytes;       /* LDS bytes per workgroup */
    int64_t algorithmic_bytes; /* Q + K + V read once, O written once */
    int32_t variant;         /* MFMA kernel: index of the kernel variant in the library's table,
                                resolved once by dsattn_plan (a launch searches nothing);
                                -1 for the generic kernel */
    int32_t ring_reach;      /* MFMA kernel: frames kept on chip beyond a query tile on each side
                                (local_ctx for 16-frame clips; the window radius or the rest of
                                the clip's local range for longer clips) */
} dsattn_launch_info;

/*
 * Build a plan: validates the descriptor, builds the per-clip context index
 * table (Section 4.1 c^i; Section 4.2 local + global), picks launch shapes for
 * this level's (P, h, D) (the latent's H', W', C' vary per U-Net level,
 * Section 3), and, unless device == -1, uploads the tables to that HIP device.
 *   global_idx : host, [n_global] int32, each in [0, F); may be NULL iff n_global == 0;
 *                duplicates and any order are legal.
 *   device     : HIP device ordinal, or -1 for a host-only plan (index queries only).
 *   out        : receives the plan; destroy with dsattn_plan_destroy.
 * Errors: EINVAL, ENOMEM, EHIP.
 */
int dsattn_plan(const dsattn_desc *desc, const int32_t *global_idx, int32_t n_global,
                int device, dsattn_plan_t **out);

/* Frees host and device tables. NULL is allowed. Does not synchronise: the caller
 * must have finished all work enqueued with this plan. */
void dsattn_plan_destroy(dsattn_plan_t *plan);

/* lk_max = max over clips of the context list length. */
int dsattn_plan_ctx_max(const dsattn_plan_t *plan, int32_t *lk_max);

/* Copies the context table to host arrays: ctx_idx [N * lk_max] (-1 padded),
 * ctx_len [N]. Either may be NULL to skip it. */
int dsattn_plan_ctx_indices(const dsattn_plan_t *plan, int32_t *ctx_idx, int32_t *ctx_len);

/* Reports the launch planner's choice. */
int dsattn_plan_launch_info(const dsattn_plan_t *plan, dsattn_launch_info *info);

/*
 * Context gather (Section 4.1: the context c^i delivered to clip i; Section 4.2:
 * K = Concat(K_local, K_global), V likewise), materialised:
 *   Kctx[i][j][p][c] = K[ctx_idx[i][j]][p][c]  for j < ctx_len[i], else 0   (same for V)
 *   K, V      : device, [F, P, C] of io_dtype
 *   Kctx, Vctx: device, [N, lk_max, P, C] of io_dtype, written entirely
 * Either pair (K,Kctx) or (V,Vctx) may be NULL/NULL to skip it.
 * Errors: EINVAL, ENODEVICE, EHIP.
 */
int dsattn_gather_context(const dsattn_plan_t *plan, const void *K, const void *V, void *Kctx,
                          void *Vctx, void *stream);

/*
 * Fused Dual-scope attention (Section 4.2), gathering K/V by index from the
 * original buffers; outputs are concatenated along frames (Section 4.1, v_out).
 *   Q, K, V : device, [F, P, C] of io_dtype, 16-byte aligned
 *   O       : device, [F, P, C] of out_dtype, 16-byte aligned, must not overlap Q, K or V
 * Errors: EINVAL, ENODEVICE, EUNSUPPORTED, EHIP.
 */
int dsattn_forward(const dsattn_plan_t *plan, const void *Q, const void *K, const void *V, void *O,
                   void *stream);

/*
 * Same attention, consuming the materialised context of dsattn_gather_context:
 * clip i attends over Kctx[i][0 .. ctx_len[i]).  Runs the kernel the plan chose for
 * dsattn_forward (the matrix-core kernel takes one clip per work item here, reading the clip's
 * slab of Kctx / Vctx); the result is identical to dsattn_forward's.
 */
int dsattn_forward_ctx(const dsattn_plan_t *plan, const void *Q, const void *Kctx, const void *Vctx,
                       void *O, void *stream);

/*
 * Plain device-to-device copy kernel of `bytes` bytes (multiple of 16, both
 * pointers 16-byte aligned).  Not part of the method: it is the known-traffic
 * yardstick that achieved bandwidth and profiler byte counters are scaled by.
 */
int dsattn_copy_probe(void *dst, const void *src, int64_t bytes, void *stream);

/*
 * Clip-parallel group normalisation (Section 4.2, "Group normalization"): the second temporal
 * module of the paper that needs context from every clip.  X is [F, P, C] with F = n_clips *
 * clip_len; the C channels form `groups` contiguous groups.  The statistics of a group are those
 * of the whole video, which is what the paper's exchange yields (per-clip means -> global mean =
 * mean of the clip means -> per-clip mean squared deviation about the GLOBAL mean -> global
 * variance = mean of those); then  y = (x - mean[g]) / sqrt(var[g] + eps) * gamma[c] + beta[c].
 * Here they are gathered in one pass: every part reports its count, mean and squared deviations
 * about its own mean, and the parts are merged pairwise (Chan et al.), which gives the same
 * global mean and (biased) variance.
 */
typedef struct dsattn_gn_desc {
    int32_t clip_len;  /* F_clip >= 1 */
    int32_t n_clips;   /* N >= 1 */
    int32_t spatial;   /* P >= 1 */
    int32_t channels;  /* C >= 1 */
    int32_t groups;    /* divides C; C a multiple of 8 (bf16) / 4 (fp32) and at least that many
                          channels per group (a 16-byte lane may straddle two groups, not more) */
    int32_t io_dtype;  /* dsattn_dtype of X and Y; statistics are fp32/fp64 */
    float eps;         /* >= 0 */
} dsattn_gn_desc;

/* Bytes of device workspace dsattn_groupnorm needs for this shape (per-workgroup moments). */
int dsattn_groupnorm_workspace(const dsattn_gn_desc *desc, size_t *bytes);

/*
 *   X, Y      : device, [F, P, C] of io_dtype, 16-byte aligned; Y may be X (in place)
 *   gamma,beta: device, [C] fp32, or NULL for 1 / 0
 *   stats     : device, [2 * groups] fp32 receiving mean[g] then 1/sqrt(var[g] + eps), or NULL
 *   workspace : device, at least dsattn_groupnorm_workspace() bytes, 16-byte aligned; contents
 *               are overwritten; calls sharing a workspace must not overlap
 * Enqueues three kernels on `stream`; allocates nothing.  Errors: EINVAL, EUNSUPPORTED, EHIP.
 */
int dsattn_groupnorm(const dsattn_gn_desc *desc, const void *X, const float *gamma,
                     const float *beta, void *Y, float *stats, void *workspace,
                     size_t workspace_bytes, void *stream);

/*
 * dsattn_groupnorm for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels
 * and the same result as dsattn_groupnorm; the per-workgroup moments go to a file-scope device
 * array of dsattn_groupnorm_static_max_bytes() = 4 MiB that every device the library runs on
 * holds until the process ends.  Runs on the current device.  The call allocates nothing (no
 * hipMalloc, hipFree or allocating library routine); the first call on a device looks the
 * array's address up once (make that call outside a graph capture).
 *   - a shape whose dsattn_groupnorm_workspace() exceeds the array is rejected with
 *     DSATTN_EUNSUPPORTED before anything is enqueued;
 *   - every call on a device shares that device's array: calls that overlap in time on one
 *     device (different streams, or graph replays running concurrently) race; calls on one
 *     stream are ordered and safe.  Nothing in the array has to start at zero: every entry a
 *     call reads was written earlier in the same call.
 * Arguments as for dsattn_groupnorm, without the workspace.  Errors: EINVAL, EUNSUPPORTED, EHIP.
 */
size_t dsattn_groupnorm_static_max_bytes(void);
int dsattn_groupnorm_static(const dsattn_gn_desc *desc, const void *X, const float *gamma,
                            const float *beta, void *Y, float *stats, void *stream);

/*
 * Clip-parallel temporal convolution (Section 4.2, "Convolution module"): the third temporal
 * module of the paper.  X is [F, P, c_in] with F = n_clips * clip_len; the module convolves
 * along the frame axis only, at every position separately, mixing channels densely:
 *   Y[f][p][co] = bias[co] + sum_{t = 0 .. 2n} sum_{ci} W[t][co][ci] * X[f + t - n][p][ci]
 * with frames outside [0, F) read as zeros.  This is what the paper's scheme computes clip by
 * clip: clip i is padded with c_pre = the last n frames of clip i-1 and c_post = the first n
 * frames of clip i+1 (zero frames at the two ends of the video), which is why n <= clip_len is
 * required.  Tap t looks at frame f + t - n (cross-correlation, the deep-learning convention).
 */
typedef struct dsattn_conv_desc {
    int32_t clip_len;  /* F_clip >= 1 */
    int32_t n_clips;   /* N >= 1 */
    int32_t spatial;   /* P >= 1 */
    int32_t c_in;      /* input channels >= 1 */
    int32_t c_out;     /* output channels >= 1 */
    int32_t reach;     /* n: frames the kernel reaches to each side (2n + 1 taps), 0 <= n <= F_clip */
    int32_t io_dtype;  /* dsattn_dtype of X and W; products are accumulated in fp32 */
    int32_t out_dtype; /* dsattn_dtype of Y; DSATTN_F32 is allowed with bf16 inputs */
    uint32_t flags;    /* DSATTN_FLAG_FORCE_GENERIC or 0 */
} dsattn_conv_desc;

/* The launch the library would make for this shape (host only; for tests and benchmarks). */
typedef struct dsattn_conv_info {
    int32_t kernel;        /* 0 = generic vector-ALU kernel, 1 = bf16 MFMA implicit-GEMM kernel */
    int32_t tile_m;        /* output rows (frame, position) per workgroup, 0 for the generic kernel */
    int32_t tile_n;        /* output channels per workgroup */
    int32_t tile_k;        /* contraction depth per step */
    int32_t n_blocks;      /* output tiles, counted in units the 8 XCDs share evenly (the matrix-core
                              kernel is launched with at most one persistent workgroup per compute
                              unit, which walk them); workgroups launched for the generic kernel */
    int32_t block_threads;
    int32_t lds_bytes;
    int32_t reserved;
    int64_t useful_flops;  /* 2 * P * c_in * c_out * (number of (frame, tap) pairs inside the video) */
    int64_t algorithmic_bytes; /* X read once + W read once + Y written once */
} dsattn_conv_info;

int dsattn_temporal_conv_info(const dsattn_conv_desc *desc, dsattn_conv_info *info);

/*
 *   X    : device, [F, P, c_in] of io_dtype, 16-byte aligned
 *   W    : device, [2n + 1][c_out][c_in] of io_dtype, 16-byte aligned (c_in fastest)
 *   bias : device, [c_out] fp32, or NULL for none
 *   Y    : device, [F, P, c_out] of out_dtype, 16-byte aligned; must not overlap X
 * Runs on the current device; enqueues one kernel on `stream`; allocates nothing.  bf16 inputs
 * with c_in a multiple of 8 run on the matrix cores, everything else on a plain vector kernel.
 * Errors: EINVAL (bad shape, null or misaligned pointer, overlap), EHIP.
 */
int dsattn_temporal_conv(const dsattn_conv_desc *desc, const void *X, const void *W,
                         const float *bias, void *Y, void *stream);

/*
 * The token-wise linear projections around the temporal attention (Section 4.2 derives the
 * queries, keys and values from the tokens and gives no formula beyond that; these are the
 * usual  Y_k = X W_k^T + b_k).  n_out weight sets are applied to the same X in one launch (3 for
 * Q, K, V: X is read from HBM once for all of them; 1 for the output projection).  Because the
 * projection is per token, projecting before or after a clip's context is gathered is the same.
 * Runs the temporal convolution's matrix-core kernel as its one-tap case.
 */
typedef struct dsattn_linear_desc {
    int64_t rows;      /* M >= 1 tokens (F * P), at most 2^31 - 1 */
    int32_t c_in;      /* >= 1 */
    int32_t c_out;     /* >= 1, the same for every weight set */
    int32_t n_out;     /* 1 .. 4 weight sets */
    int32_t io_dtype;  /* dsattn_dtype of X and W; products are accumulated in fp32 */
    int32_t out_dtype; /* dsattn_dtype of every Y */
    uint32_t flags;    /* DSATTN_FLAG_FORCE_GENERIC or 0 */
} dsattn_linear_desc;

/* The launch the library would make (host only); flops and bytes are those of all n_out sets. */
int dsattn_linear_info(const dsattn_linear_desc *desc, dsattn_conv_info *info);

/*
 *   X    : device, [rows, c_in] of io_dtype, 16-byte aligned
 *   W    : HOST array of n_out device pointers, each [c_out][c_in] of io_dtype, 16-byte aligned
 *   bias : NULL, or HOST array of n_out device pointers, each [c_out] fp32 or NULL
 *   Y    : HOST array of n_out device pointers, each [rows, c_out] of out_dtype, 16-byte aligned;
 *          the outputs must not overlap X or each other
 * The pointer arrays are read during the call only.  Runs on the current device; enqueues one
 * kernel on `stream` (n_out kernels on the vector path); allocates nothing.
 * Errors: EINVAL, EUNSUPPORTED (too large for the vector kernel), EHIP.
 */
int dsattn_linear(const dsattn_linear_desc *desc, const void *X, const void *const *W,
                  const float *const *bias, void *const *Y, void *stream);

/*
 * One whole temporal-attention layer on the caller's stream (Section 4.2, "Attention module":
 * queries, keys and values are computed from the tokens, each clip attends to its local and
 * global context, and the result is projected back):
 *   Q, K, V = X Wq^T + bq, X Wk^T + bk, X Wv^T + bv     one launch, X read once
 *   A       = Dual-scope attention(Q, K, V)              dsattn_forward of `plan`
 *   Y       = A Wo^T + bo                                one launch
 * Three kernels enqueued back to back with no host work and no allocation in between; the
 * intermediate tensors live in the caller's workspace (Q, K, V, A in that order, each [F, P, C]
 * of io_dtype at a 256-byte aligned offset).  The three stages are not merged into one kernel:
 * a workgroup of the projection needs all C channels of 256 tokens, a workgroup of the attention
 * all frames of one position.
 *   plan      : for a device; out_dtype must equal io_dtype (EUNSUPPORTED otherwise)
 *   X         : device, [F, P, C] of io_dtype, C = heads * head_dim, 16-byte aligned
 *   W         : HOST array of 4 device pointers Wq, Wk, Wv, Wo, each [C][C] of io_dtype
 *               (output channel major, as for dsattn_linear), 16-byte aligned
 *   bias      : NULL, or HOST array of 4 device pointers (entries may be NULL), each [C] fp32
 *   workspace : device, at least dsattn_temporal_layer_workspace() bytes, 256-byte aligned,
 *               overlapping neither X nor Y; contents on return: Q, K, V, A
 *   Y         : device, [F, P, C] of io_dtype; may be X itself (X is consumed by the first
 *               stage), must not overlap it otherwise
 * Errors: those of dsattn_linear and dsattn_forward; EINVAL for a short or misaligned workspace.
 * After a failure in a later stage the earlier stages stay enqueued.
 */
int dsattn_temporal_layer_workspace(const dsattn_plan_t *plan, size_t *bytes);
int dsattn_temporal_layer(const dsattn_plan_t *plan, const void *X, const void *const *W,
                          const float *const *bias, void *workspace, size_t workspace_bytes,
                          void *Y, void *stream);

/* Static description of a status code; never NULL. */
const char *dsattn_strerror(int code);

/* Detail of the calling thread's most recent failure (e.g. the HIP error string);
 * empty string if none. The pointer stays valid until the thread's next failing call. */
const char *dsattn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DSATTN_H */
