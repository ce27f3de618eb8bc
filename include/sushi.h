/*
 * sushi.h — C ABI of the SubGraph-Stationary (SGS) SubNet inference library for AMD MI355X (gfx950).
 *
 * The library serves a stream of SubNet queries drawn from one weight-shared SuperNet
 * (arXiv 2306.17266, "SUSHI").  The three calls of the paper's problem statement (Section 3.1:
 * the accelerator receives the selected SubNet, the next SubGraph to cache and the query data,
 * returns the result and enacts the caching decision) are
 *
 *     sushi_load_supernet        once      pack the SuperNet's weights on the device
 *     sushi_set_subgraph_cache   every Q   make a SubGraph's weights resident
 *     sushi_infer                per query run one SubNet, logits out
 *
 * plus the host-side scheduler of Algorithm 1 (sushi_sched_*) and counters (sushi_get_stats).
 *
 * Conventions
 *   - Plain C types only.  Every pointer is marked HOST or DEVICE below.
 *   - The library copies what it needs from HOST pointers before returning and never frees or
 *     keeps a caller's pointer.  DEVICE input/output buffers stay caller-owned and must stay
 *     alive until the stream has executed the enqueued work.
 *   - Every function returns a sushi_status (0 = ok, negative = error); on error nothing has
 *     been enqueued and sushi_last_error() gives a message.  Nothing aborts or throws.
 *   - A context is bound to one device and one HIP stream; calls on one context must not
 *     overlap in time.
 */
#ifndef SUSHI_H
#define SUSHI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SUSHI_MAX_STAGES 8
#define SUSHI_MAX_CHOICES 4
#define SUSHI_MAX_BLOCKS 32

typedef struct sushi_ctx sushi_ctx; /* opaque */

typedef enum {
    SUSHI_OK = 0,
    SUSHI_EINVAL = -1,  /* bad argument / SubNet choice not offered by the SuperNet */
    SUSHI_ENOMEM = -2,  /* host or device allocation failed                          */
    SUSHI_ESTATE = -3,  /* call out of order (e.g. infer before load)                */
    SUSHI_EBUDGET = -4, /* SubGraph larger than the stated cache budget              */
    SUSHI_EDEVICE = -5  /* a HIP call failed                                         */
} sushi_status;

typedef enum { SUSHI_FP32 = 0, SUSHI_BF16 = 1 } sushi_dtype;
typedef enum { SUSHI_FAMILY_TINY = 0, SUSHI_FAMILY_RESNET = 1, SUSHI_FAMILY_MBV3 = 2 } sushi_family;
typedef enum { SUSHI_ACT_NONE = 0, SUSHI_ACT_RELU = 1, SUSHI_ACT_HSWISH = 2 } sushi_act;
typedef enum { SUSHI_STRICT_ACCURACY = 0, SUSHI_STRICT_LATENCY = 1 } sushi_policy;

/* Kinds of SuperNet tensors in the weight blob (see sushi_describe_supernet). */
typedef enum {
    SUSHI_T_CONV = 0,     /* [K][C][R][R] dense convolution                      */
    SUSHI_T_DWCONV = 1,   /* [K][1][R][R] depthwise convolution                  */
    SUSHI_T_FC = 2,       /* [K][C] fully connected                              */
    SUSHI_T_BIAS = 3,     /* [K]                                                 */
    SUSHI_T_SCALE = 4,    /* [K] per-channel scale (batch norm folded to a pair) */
    SUSHI_T_SHIFT = 5,    /* [K] per-channel shift                               */
    SUSHI_T_SCALE_RES = 6 /* [K] scale that ends a residual branch               */
} sushi_tensor_kind;

/*
 * A weight-shared SuperNet (Section 2.1: stages of repeated blocks; elastic depth, width /
 * expand ratio and kernel size).  Three families:
 *   TINY    n_stages conv3x3+ReLU layers (one per "stage"), global average, FC.  Elastic width per
 *           layer, elastic depth = number of leading layers.
 *   RESNET  three 3x3 stem convs (first stride 2), 3x3/2 max-pool, n_stages stages of bottleneck
 *           blocks (1x1, 3x3 with the stage stride in its first block, 1x1, shortcut; the first
 *           block of a stage has a 1x1 projection shortcut), global average, FC.  Width multiplier
 *           per stage and for the stem, expand ratio per block.
 *   MBV3    3x3/2 stem (h-swish), one depthwise-separable block, n_stages stages of inverted
 *           residual blocks (1x1 expand, k x k depthwise, optional squeeze-excite, 1x1 project,
 *           skip when stride 1 and equal widths), 1x1 head conv, global average, two FCs.
 *           Expand ratio and kernel size per block.
 * Channel counts follow ch(x) = max(8, floor(x/8 + 0.5) * 8), plus 8 if that is below 0.9 x.
 */
typedef struct sushi_arch {
    int32_t family;
    int32_t n_classes;
    int32_t in_channels;
    int32_t n_stages;
    int32_t stage_base_out[SUSHI_MAX_STAGES]; /* channels at width multiplier 1 */
    int32_t stage_stride[SUSHI_MAX_STAGES];
    int32_t stage_max_depth[SUSHI_MAX_STAGES]; /* TINY: 1 each */
    int32_t stage_act[SUSHI_MAX_STAGES];       /* sushi_act of the stage's blocks (MBV3) */
    int32_t stage_se[SUSHI_MAX_STAGES];        /* squeeze-excite in the stage's blocks (MBV3) */
    int32_t n_depth_drop, depth_drop_choices[SUSHI_MAX_CHOICES]; /* a stage may run max_depth - d blocks */
    int32_t n_width;
    double width_choices[SUSHI_MAX_CHOICES];
    int32_t n_expand;
    double expand_choices[SUSHI_MAX_CHOICES];
    int32_t n_kernel, kernel_choices[SUSHI_MAX_CHOICES]; /* odd sizes; the largest is the stored one */
    int32_t n_res, res_choices[SUSHI_MAX_CHOICES];
    int32_t stem_mid, stem_out; /* RESNET: both; MBV3: stem_out */
    int32_t head_mid, head_feat; /* MBV3 */
} sushi_arch;

/*
 * One SubNet: which elastic choice is taken where.  Block slots are numbered stage by stage at
 * maximum depth (slot = sum of max depths of earlier stages + block index).
 *   depth[s]        active blocks of stage s (TINY: depth[0] = active layers); the FIRST depth[s]
 *                   blocks run ("top k blocks per stage", Section 2.1)
 *   width_idx[0]    stem, width_idx[1+s] stage s (TINY: layer s): index into width_choices
 *   expand_idx[b]   index into expand_choices for block slot b
 *   kernel_idx[b]   index into kernel_choices for block slot b (MBV3)
 */
typedef struct sushi_subnet_cfg {
    int32_t resolution;
    int32_t depth[SUSHI_MAX_STAGES];
    int32_t width_idx[SUSHI_MAX_STAGES + 1];
    int32_t expand_idx[SUSHI_MAX_BLOCKS];
    int32_t kernel_idx[SUSHI_MAX_BLOCKS];
} sushi_subnet_cfg;

typedef struct sushi_tensor_desc {
    char name[32];
    int32_t kind; /* sushi_tensor_kind */
    int32_t ndim;
    int32_t shape[4];
} sushi_tensor_desc;

/* Active slice of one weight-bearing layer: K leading filters, C leading input channels
 * (1 for depthwise), centred r x r taps (1 for FC).  K = 0: layer not used. */
typedef struct sushi_layer_dims {
    int32_t K, C, r;
} sushi_layer_dims;

/* A cacheable SubGraph (footnote 1 of the paper: any connected subset of weights; here, as in
 * the scheduler's encoding of Section 3.3, one prefix box (K, C, r) per SuperNet layer, in the
 * order sushi_subnet_layers reports).  Its size is sum K*C*r*r*sizeof(weight). */
typedef struct sushi_subgraph_cfg {
    int32_t n_layers;
    const sushi_layer_dims *layers; /* HOST */
} sushi_subgraph_cfg;

/* Inputs of the scheduler (Algorithm 1).  All arrays HOST, copied.
 *   subnet_vecs   [n_subnets][vec_len]   vectors [K_1,C_1,...,K_N,C_N] of the serving SubNets
 *   accuracy      [n_subnets]
 *   subgraph_vecs [n_subgraphs][vec_len] vectors of the candidate SubGraphs (the set S)
 *   table         [n_subnets][n_subgraphs+1] latency of SubNet i with SubGraph j cached; the last
 *                 column is "nothing cached"
 *   initial_cache index into the candidates, or -1 for an empty cache state */
typedef struct sushi_sched_desc {
    int32_t n_subnets, n_subgraphs, vec_len;
    const int32_t *subnet_vecs;
    const float *accuracy;
    const int32_t *subgraph_vecs;
    const float *table;
    int32_t Q;
    int32_t policy; /* sushi_policy */
    int32_t initial_cache;
} sushi_sched_desc;

typedef struct sushi_stats {
    uint64_t queries;                /* sushi_infer calls that enqueued work                          */
    uint64_t weight_bytes_total;     /* sum over queries of the SubNet's weight bytes                 */
    uint64_t weight_bytes_in_subgraph; /* of those, bytes that lie inside the cached SubGraph G (the
                                        closed form bytes(SN ∩ G) the scheduler's table reasons with; a
                                        nominal figure: what of G really sits on chip is the next but
                                        one counter)                                                   */
    uint64_t last_weight_bytes;      /* the same two figures for the last query                       */
    uint64_t last_in_subgraph_bytes;
    uint64_t cache_installs;         /* sushi_set_subgraph_cache calls that installed a SubGraph      */
    uint64_t cache_bytes_installed;  /* sum of bytes(G) over them (nominal, as above)                 */
    uint64_t cache_bytes;            /* bytes(G) of the SubGraph cached now                           */
    double last_hit_ratio;           /* ||SN ∩ G||_2 / ||SN||_2 on the [K,C] vectors (Appendix A.4)   */
    double sum_hit_ratio;            /* summed over queries                                           */
    uint64_t plan_cache_hits, plan_cache_misses;
    uint64_t weight_bytes_lds;       /* team kernel: weight bytes the queries took from resident LDS slabs
                                        instead of memory, counted on the host from the residency table
                                        each query ran under (the only bytes that are never fetched)   */
    uint64_t last_lds_bytes;         /* the same for the last query                                    */
    uint64_t cache_bytes_lds;        /* bytes of the cached SubGraph that sit in a team's LDS stores    */
    uint64_t residency_changes;      /* cache changes that altered what a team's LDS stores hold (a new residency
                                        table was published; the others changed the SubGraph outside the stores) */
    uint64_t install_bytes_lds;      /* slab bytes those changes make valid that were not valid under the table
                                        before: what ONE team copies into its LDS if it serves a query under
                                        every table (a team that skips tables copies less)               */
} sushi_stats;

/* ---------------------------------------------------------------- host-only helpers (no GPU needed) */

/* Lists the SuperNet's tensors in the order the weight blob must hold them (each tensor contiguous,
 * float32, row-major over its shape).  Writes min(n, cap) entries to out (HOST, may be NULL when
 * cap = 0) and the full count to *n_out.  SUSHI_EINVAL for an inconsistent arch. */
int sushi_describe_supernet(const sushi_arch *arch, sushi_tensor_desc *out, int cap, int *n_out);

/* For every weight-bearing SuperNet layer, in blob order, the slice (K, C, r) that SubNet cfg uses
 * (Section 2.1); skipped layers report K = 0.  The scheduler's vector of Section 3.3 is
 * [K_1, C_1, ..., K_N, C_N] of this list.  SUSHI_EINVAL if cfg is not a SubNet of arch. */
int sushi_subnet_layers(const sushi_arch *arch, const sushi_subnet_cfg *cfg, sushi_layer_dims *out, int cap,
                        int *n_out);

/* What a SubNet has in common with a cached SubGraph (both as per-layer boxes of n layers, K = 0: layer unused):
 * the SubNet's weight bytes, the bytes inside the intersection (per layer the elementwise minimum of the
 * boxes), and the hit ratio of Appendix A.4, ||min(v_SN, v_G)||_2 / ||v_SN||_2 on the [K_1, C_1, ..., K_n, C_n]
 * vectors.  Host only.  Any output pointer may be NULL. */
int sushi_subgraph_overlap(const sushi_layer_dims *subnet, const sushi_layer_dims *subgraph, int n, int bytes_per_weight,
                           uint64_t *subnet_bytes, uint64_t *common_bytes, double *hit_ratio);

/* Where one weight-bearing layer sits in the packed image of the SuperNet's weights (sushi_pack_supernet). */
typedef struct sushi_packed_layer {
    uint64_t offset;      /* element offset of the layer's packed weights */
    int32_t depthwise;    /* 1: [tap in ring order][filter < Kpad]; 0: [tap][channel group < CG][filter < Kpad][8 channels] */
    int32_t K, C, R;      /* the SuperNet layer: filters, input channels (1 for depthwise), taps per side */
    int32_t Kpad, CG;     /* filters padded to a multiple of 16; channel groups of 8 (0 for depthwise) */
} sushi_packed_layer;

/* The weight packer on its own (Section 2.1: a SubNet is a slice of the SuperNet's weights; the packed layout makes
 * every slice a set of contiguous prefixes).  Host only.  Produces the image that sushi_load_supernet copies to the
 * device for compute_dtype SUSHI_BF16 (uint16 bit patterns, values rounded to nearest even) or SUSHI_FP32 (float32):
 *   dense / FC layer  element ((tap * CG + c / 8) * Kpad + k) * 8 + c % 8 holds W[k][c][tap]: for every tap and channel
 *                     group below C' / 8 the slice (K', C') is the run of the first K' * 8 elements
 *   depthwise layer   element t * Kpad + k holds W[k][tap t], the taps in ring order: the 9 taps of the centre 3 x 3,
 *                     then the 16 of the 5 x 5 ring, then the 24 of the 7 x 7 ring, so that a centred r x r crop is the
 *                     first r * r taps
 * Elements the SuperNet does not define (filters K .. Kpad - 1, channels beyond C in the last group, gaps between
 * layers) are zero.  weights / nbytes: as for sushi_load_supernet.  packed: HOST buffer of cap_bytes bytes, may be NULL
 * with cap_bytes = 0; *n_bytes receives the image's size.  layers: HOST array of cap_layers entries (may be NULL with
 * cap_layers = 0), one per weight-bearing layer in the order of sushi_subnet_layers; *n_layers receives their number.
 * SUSHI_EINVAL for an inconsistent arch, a blob of the wrong size, an unknown dtype or a packed buffer that is too
 * small (sizes are still reported). */
int sushi_pack_supernet(const sushi_arch *arch, const void *weights, size_t nbytes, int compute_dtype, void *packed,
                        size_t cap_bytes, size_t *n_bytes, sushi_packed_layer *layers, int cap_layers, int *n_layers);

/* How exec mode 3 cuts one op of a SubNet's per-query plan (Section 3.1: a query activates one SubNet; Section 4.2:
 * its layers run one after the other) into units for a team of workgroups.  kind: 0 dense conv, 1 depthwise conv,
 * 2 max-pool, 3 global average pool, 4 fully connected, 5 channel gate; 6 a whole squeeze-excite block (pooling, two
 * fully connected layers, gating: the team kernel runs the four ops as one, without barriers between them; H, W, C
 * describe the gated map, K the width between the two FC layers), 7 the slot of an op that the kind-6 op before it
 * has done (skipped; the list keeps one entry per op of the plan).  layer: SuperNet layer (order of
 * sushi_subnet_layers) or -1.  wk selects the unit variant (> 0: split units, that many waves per unit; 0: tiled units;
 * -1: stem units; -2 depthwise through LDS; -3 tiled units with resident weights; -4 depthwise from memory), ft / pt its
 * tile shape, n_units / n_p the unit counts, lds_bytes what the variant takes of the 32 KiB LDS scratch. */
typedef struct sushi_team_op {
    int32_t kind, layer;
    int32_t B, H, W, C, P, Q, K, R, stride;
    int32_t ft, pt, wk, n_units, n_p;
    int32_t lds_bytes;
    int32_t res, out_f32; /* the op adds a residual of the output's shape / stores float32 (gates, logits) */
} sushi_team_op;

/* The ops of SubNet cfg at the given batch size as a team of team_wgs workgroups (2 .. 32) would run them, in order.
 * Host only: needs no device and no weights.  Writes min(n, cap) entries to out (HOST, may be NULL when cap = 0) and
 * the full count to *n_out.  SUSHI_EINVAL for an inconsistent arch or cfg, batch < 1 or team_wgs outside 1 .. 32;
 * SUSHI_ESTATE if a layer does not fit the team kernel. */
int sushi_team_plan(const sushi_arch *arch, const sushi_subnet_cfg *cfg, int batch, int team_wgs, sushi_team_op *out,
                    int cap, int *n_out);

/* ---------------------------------------------------------------- context */

/* device_id: HIP device ordinal, or -1 for a host-only context (scheduler calls only; load and
 * infer return SUSHI_ESTATE).  hip_stream: a hipStream_t created by the caller (e.g. PyTorch's
 * current stream), borrowed for the life of the context; NULL = the default stream. */
int sushi_create(sushi_ctx **out, int device_id, void *hip_stream);
void sushi_destroy(sushi_ctx *ctx);
/* Library-owned string, valid until the next call on ctx (ctx = NULL: last error of create). */
const char *sushi_last_error(const sushi_ctx *ctx);

/* ---------------------------------------------------------------- the SGS data path */

/* weights: HOST float32 blob in sushi_describe_supernet order, nbytes = its exact size.
 * compute_dtype: SUSHI_FP32 keeps float32 weights and activations (fp32 FMA); SUSHI_BF16 stores
 * weights and activations as bf16 (values rounded to nearest even), multiplies on the bf16 matrix
 * cores, accumulates and applies scale/shift in float32.  Packs the tensors so that every SubNet
 * slice is a prefix per (tap, 8-channel group) and copies them to the device.  Synchronous. */
int sushi_load_supernet(sushi_ctx *ctx, const sushi_arch *arch, const void *weights, size_t nbytes,
                        int compute_dtype);

/* The paper's own precision (Section 5.1, footnote on number formats: int8 weights, input activations and zero
 * points, int32 scale; Section 4.2.2, the zero-point / scale buffer).  Families SUSHI_FAMILY_TINY and
 * SUSHI_FAMILY_RESNET; exec mode 0 (sushi_infer with another mode set returns SUSHI_ESTATE); SubGraph caching is
 * accounted at one byte per weight.
 *   weights  HOST int8: the weight tensors of sushi_describe_supernet (conv [K][C][R][R], fc [K][C]) in that
 *            order, nothing else; n_weights = their exact total element count
 *   qparams  HOST int32: for every weight tensor, in the same order: mult[K], rshift[K], bias[K], then eight
 *            scalars [z_x, z_y, m_res, sh_res, z_res, 0, 0, 0]; n_qparams = sum of 3 K + 8
 * Arithmetic of a conv layer, all integers (x_q, w_q int8; acc int32; products int64):
 *   acc[k]   = sum over taps inside the image and active channels of w_q * (x_q - z_x)
 *   t        = rr((acc[k] + bias[k]) * mult[k], rshift[k]),  rr(v, s) = (v + 2^(s-1)) >> s (arithmetic shift)
 *   t       += rr((res_q - z_res) * m_res, sh_res)           where the layer adds a residual
 *   y_q      = clamp(z_y + t, lo, 127),  lo = z_y after a ReLU, else -128
 * 3x3/2 max-pool: maximum of the codes.  Global pooling: exact int32 sums of (x_q - z_x), z_x = first scalar of the
 * classifier.  Classifier: acc64[k] = sum_c w_q[k][c] * sum[c] + HW * bias[k];
 * logit[k] = (float)((double)acc64[k] * ((double)base[k] / (double)HW)), base[k] = the float32 whose bit pattern
 * is mult[k], HW = pixels pooled over.  rshift must lie in 1 .. 62 for conv layers.
 * sushi_infer then takes int8 input [batch][resolution][resolution][in_channels] (zero point z_x of the first
 * layer) and returns float32 logits.  Synchronous.  SUSHI_EINVAL for a family without an int8 path, wrong sizes
 * or a shift out of range. */
int sushi_load_supernet_int8(sushi_ctx *ctx, const sushi_arch *arch, const int8_t *weights, size_t n_weights,
                             const int32_t *qparams, size_t n_qparams);

/* Makes SubGraph g the cached one ("enacts the caching decision", Section 3.1).  g = NULL or
 * g->n_layers = 0 empties the cache (SGS off).  g->n_layers must equal the SuperNet's layer
 * count, every box must lie inside its layer, and the SubGraph's bytes must not exceed
 * budget_bytes (SUSHI_EBUDGET).  Ordered before later sushi_infer calls. */
int sushi_set_subgraph_cache(sushi_ctx *ctx, const sushi_subgraph_cfg *g, size_t budget_bytes);

/* Runs SubNet cfg on one batch.
 *   input_dev   DEVICE, [batch][resolution][resolution][in_channels], float32 (SUSHI_FP32),
 *               bf16 (SUSHI_BF16) or int8 (after sushi_load_supernet_int8)
 *   logits_dev  DEVICE, float32 [batch][n_classes]
 * Enqueues on the context's stream and returns; results are bit-identical whatever SubGraph is
 * cached.  SUSHI_EINVAL (nothing enqueued) if cfg is not a SubNet of the loaded SuperNet. */
int sushi_infer(sushi_ctx *ctx, const sushi_subnet_cfg *cfg, const void *input_dev, int batch, void *logits_dev);

/* For callers that must not allocate device memory while they run (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): sushi_infer as exec mode 0 does it (one launch per layer on
 * the context's stream, float32 or bf16), with the activation buffers of the query in a static device array
 * of the library instead of the context's arena.  Calls no hipMalloc / hipFree and no allocating library
 * routine; same arguments, results and error behaviour as sushi_infer.
 *   - The array holds SUSHI_STATIC_SCRATCH_BYTES per GPU for as long as the library is loaded.  A query whose
 *     SubNet needs more at its batch size and resolution (six feature-map buffers of its largest layer output
 *     plus four vector buffers) is refused with SUSHI_ENOMEM and nothing is enqueued.
 *   - Every call on a GPU, from any context, uses the same array: calls whose work overlaps in time on one
 *     GPU (two contexts, two streams) race.  Nothing in it has to start at zero; a call leaves its
 *     activations behind.
 *   - The SubGraph cache has no effect on this path (as in exec mode 0); the counters are kept. */
#define SUSHI_STATIC_SCRATCH_BYTES (16u << 20)
int sushi_infer_static(sushi_ctx *ctx, const sushi_subnet_cfg *cfg, const void *input_dev, int batch, void *logits_dev);

/* Waits until every query enqueued or posted through ctx has finished and its logits are visible
 * to the host and to later work on any stream. */
int sushi_synchronize(sushi_ctx *ctx);

/* sushi_synchronize, then makes the persistent team kernel (mode 3) leave, so that the GPU is free
 * for other work; the next query starts it again (and refills the LDS stores). */
int sushi_quiesce(sushi_ctx *ctx);

/* Team-kernel diagnostics.  enable = 1: from the next start of the team kernel, each team leader
 * stamps a 100 MHz clock before the first op of a query and after the barrier of every op
 * (slot 0, then slot i+1 for op i; 256 slots per team, 128 teams: team = XCD * teams per XCD + its number there).  Each call first waits for all
 * queries, stops the team kernel and, if out is not null, copies up to cap stamps to out (HOST). */
int sushi_team_trace(sushi_ctx *ctx, int enable, uint64_t *out, int cap);

/* ---------------------------------------------------------------- scheduler (Algorithm 1, Section 3.3) */

int sushi_sched_init(sushi_ctx *ctx, const sushi_sched_desc *desc);
/* One query (A_t, L_t): *subnet_idx_out = SubNet to serve under the current cache state;
 * *new_cache_idx_out = candidate to cache next if this is a Q-th query, else -1.  The caller
 * enacts it with sushi_set_subgraph_cache; the scheduler's own cache state changes here. */
int sushi_sched_step(sushi_ctx *ctx, float acc_target, float lat_target, int *subnet_idx_out, int *new_cache_idx_out);
/* For streams that name the SubNet themselves: accounts vector vec (HOST, vec_len ints) as the
 * served SubNet and makes the every-Q cache choice only. */
int sushi_sched_record(sushi_ctx *ctx, const int32_t *vec, int *new_cache_idx_out);

/* ---------------------------------------------------------------- counters and options */

int sushi_get_stats(sushi_ctx *ctx, sushi_stats *out);

typedef enum {
    SUSHI_OPT_EXEC_MODE = 0,    /* 0 = one launch per layer (default), 1 = replay a HIP graph per SubNet,
                                   2 = stream kernel: one launch per query, layers separated by grid
                                   barriers (bf16 mode only; a barrier wait that runs out is reported
                                   by the next sushi_infer as SUSHI_EDEVICE),
                                   3 = team kernel: a persistent kernel whose workgroups form 1 to 16 teams per
                                   XCD (SUSHI_OPT_TEAMS_PER_XCD); each team serves one query at a time inside
                                   its XCD, so 8 to 128 queries are in flight.  bf16 mode only.  sushi_infer then waits
                                   for the context's stream (the input must be complete), posts the
                                   query to a team and returns; the logits are valid after
                                   sushi_synchronize.  The kernel runs on a private stream and leaves by
                                   itself when no query arrives for SUSHI_OPT_IDLE_US. */
    SUSHI_OPT_KERNEL_TIMING = 1,/* 1 = bracket every launch with HIP events on the context's stream and
                                   accumulate per kernel family (modes 0, 2, 3); setting 1 clears the totals */
    SUSHI_OPT_SPIN_LIMIT = 2,   /* polls a stream-/team-kernel workgroup makes at one barrier before it
                                   gives up (default 400000, about a second) */
    SUSHI_OPT_STREAM_WGS = 4,   /* workgroups of the stream kernel (multiple of 16; default: one per
                                   compute unit); only before the first query in mode 2 */
    SUSHI_OPT_TEAM_WGS_PER_CU = 5, /* workgroups of the team kernel per compute unit, 1 or 2 (default 2);
                                   only before the first query in mode 3 */
    SUSHI_OPT_TEAMS_PER_XCD = 6, /* mode 3: teams the workgroups of one XCD are dealt to: 1 (default), 2, 4, 8 or 16.
                                   More, smaller teams serve more queries at a time, each more slowly:
                                   more queries per second, longer latency of a lone query.
                                   Only before the first query in mode 3 */
    SUSHI_OPT_IDLE_US = 3,      /* microseconds without a query after which the team kernel leaves
                                   (default 2000); the next query starts it again */
    SUSHI_OPT_COLD_SWEEP_MIB = 7, /* modes 0 - 2, measurement aid: before every query a kernel streams a scratch
                                   buffer of this many MiB (0 = off, at most 4096) through the caches, so the
                                   query finds none of its weights on chip: a device that loses its caches
                                   between queries, the premise the paper's SGS starts from (Section 4.3) */
    SUSHI_OPT_PATCH_CONV_MIN_PIXELS = 8 /* modes 0 - 1, bf16: dense 1x1 / 3x3 layers with at least this many output
                                   pixels (batch x rows x columns) run in the kernel that stages a tile's input
                                   patch in LDS (large batches); below four times this many only if the layer's
                                   reduction (input channels x taps) is at least 1024 long.  0 = never.
                                   Default 3136.  In mode 1 it applies to SubNets recorded afterwards */
} sushi_option;
int sushi_set_option(sushi_ctx *ctx, int option, int64_t value);

/* Per kernel family: launches timed, their summed duration, and the algorithmic bytes and flops
 * they processed (every input, output, residual, weight and scale/shift element of the active
 * slice counted once).  One launch of the stream kernel is one query; one launch of the persistent
 * team kernel lasts from its start to its exit and covers every query posted meanwhile.  Waits for
 * outstanding timed launches (and makes the team kernel leave).  Writes min(n, cap) entries. */
typedef struct sushi_kernel_stats {
    char name[32];
    uint64_t launches;
    double total_ms;
    double bytes;
    double flops;
} sushi_kernel_stats;
int sushi_get_kernel_stats(sushi_ctx *ctx, sushi_kernel_stats *out, int cap, int *n_out);

/* One timed launch of exec mode 0 (SUSHI_OPT_KERNEL_TIMING = 1): which op of the query's plan it ran (the order
 * sushi_team_plan lists them in), the kernel family (index into sushi_get_kernel_stats), its duration by HIP
 * events and its algorithmic bytes and flops.  The library keeps the records of the launches since timing was
 * switched on, at most 65536.  Waits for outstanding timed launches.  Writes min(n, cap) entries. */
typedef struct sushi_launch_record {
    int32_t op_index, kernel_class;
    float ms;
    float pad;
    double bytes, flops;
} sushi_launch_record;
int sushi_get_launch_records(sushi_ctx *ctx, sushi_launch_record *out, int cap, int *n_out);

#ifdef __cplusplus
}
#endif
#endif /* SUSHI_H */
