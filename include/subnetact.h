/*
 * subnetact.h -- C ABI of the SubNetAct forward path on one MI355X (gfx950).
 *
 * SubNetAct (paper section "SubNetAct: Instantaneous Model Actuation") keeps ONE
 * max-size, weight-shared SuperNet resident on the GPU and serves any subnet of
 * it in place.  A worker receives a batch of requests plus, per request, the
 * control tuple (D, E, W) chosen by a scheduling policy, actuates that subnet
 * and runs its forward pass (section "System Architecture", worker paragraph).
 * Three operators do the actuation:
 *   LayerSelect  blocks beyond the per-stage depth D are skipped; the input of a
 *                skipped block goes unchanged to the next one.
 *   WeightSlice  E / W fix how many channels a conv / linear layer uses; the
 *                layer runs on a slice of the shared weights, with no copy.
 *   SubnetNorm   normalisation layer j of subnet i uses statistics stored for
 *                (i, j); those statistics are the only non-shared state.
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses, "host" pointers host addresses.
 *   - The caller owns every buffer.  The library borrows `weights_dev`,
 *     `stats_dev` and `workspace_dev` from sna_supernet_load() until
 *     sna_supernet_free(); it never allocates device memory and never copies or
 *     repacks weights per subnet.
 *   - All functions return SNA_OK (0) or a negative sna_status; the text of the
 *     last error on the calling thread is available from sna_last_error().
 *     Argument and cfg validation comes first: a validation error (every status
 *     except SNA_E_HIP) means nothing has been enqueued.  SNA_E_HIP reports a
 *     failed HIP call, possibly in the middle of the launch list: outputs may
 *     then be partly written.  The handle stays usable either way.
 *   - Activations are NHWC, channel-fastest, densely packed.
 */
#ifndef SUBNETACT_H
#define SUBNETACT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SNA_MAX_STAGES 8
#define SNA_MAX_DEPTH 16
#define SNA_MAX_GROUPS 16   /* distinct subnet cfgs with at least one request in one call */
#define SNA_NAME_LEN 48

typedef enum {
  SNA_OK = 0,
  SNA_E_NULL = -1,        /* a required pointer is NULL */
  SNA_E_ARCH = -2,        /* architecture description invalid or unsupported */
  SNA_E_CFG_RANGE = -3,   /* depth / channels / kernel / resolution outside the SuperNet */
  SNA_E_CFG_ALIGN = -4,   /* channel count not a multiple of 8 */
  SNA_E_SUBNET_ID = -5,   /* subnet_id outside the statistics table */
  SNA_E_BATCH = -6,       /* n_requests < 0 or > max_batch, bad req_cfg entry, too many groups */
  SNA_E_WORKSPACE = -7,   /* workspace / weights / stats buffer too small or misaligned */
  SNA_E_HIP = -8          /* a HIP call failed */
} sna_status;

typedef enum { SNA_FAMILY_TINY = 0, SNA_FAMILY_RESNET = 1, SNA_FAMILY_MBV3 = 2,
               SNA_FAMILY_TRANSFORMER = 3 } sna_family;
typedef enum { SNA_DTYPE_FP32 = 0, SNA_DTYPE_BF16 = 1 } sna_dtype;
typedef enum { SNA_ACT_NONE = 0, SNA_ACT_RELU = 1, SNA_ACT_HSWISH = 2, SNA_ACT_GELU = 3 } sna_act;

/*
 * Max-size shape of one SuperNet family.  The paper names the families only
 * (ResNet- and MobileNet-style OFA supernets, transformer supernets in related
 * work); the block wiring each value feeds is fixed by this library:
 *   TINY         stem 3x3 conv -> SubnetNorm -> ReLU; per stage up to
 *                stage_max_depth blocks of 3x3 conv -> SubnetNorm -> ReLU, the
 *                first with stride 2, later ones with a residual add; global
 *                average pool; linear + bias.  fp32 throughout.
 *   RESNET       7x7/2 stem -> SubnetNorm -> ReLU -> 3x3/2 max pool; bottleneck
 *                blocks 1x1 -> 3x3 (stride in block 0) -> 1x1, each followed by
 *                SubnetNorm, ReLU after the first two and after the residual
 *                add; block 0 of a stage has a 1x1 strided projection shortcut;
 *                global average pool; linear + bias.
 *   MBV3         3x3/2 stem + hardswish; one fixed depthwise-separable block;
 *                inverted-residual blocks 1x1 expand -> k x k depthwise (centre
 *                slice of a stored 7x7) -> optional squeeze-excite -> 1x1
 *                project; 1x1 tail conv, pool, two linear layers.
 *   TRANSFORMER  post-LayerNorm encoder blocks with leading-head and leading-FFN
 *                column slices; logits from token 0.
 */
typedef struct {
  int32_t family;                 /* sna_family */
  int32_t dtype;                  /* sna_dtype: storage type of weights, inputs and activations */
  int32_t n_classes;
  int32_t in_ch;                  /* image channels (conv families) */
  int32_t stem_ch;                /* max stem width */
  int32_t n_stages;
  int32_t stage_ch[SNA_MAX_STAGES];          /* max output channels of each stage */
  int32_t stage_stride[SNA_MAX_STAGES];      /* stride of block 0 of each stage */
  int32_t stage_max_depth[SNA_MAX_STAGES];
  int32_t block_max_mid[SNA_MAX_STAGES][SNA_MAX_DEPTH]; /* max bottleneck / expanded channels (MBV3 stages with SE: <= 2048) */
  int32_t block_max_aux[SNA_MAX_STAGES][SNA_MAX_DEPTH]; /* max squeeze channels (MBV3 SE) */
  int32_t stage_se[SNA_MAX_STAGES];          /* MBV3: 1 if the stage's blocks carry squeeze-excite */
  int32_t stage_act[SNA_MAX_STAGES];         /* MBV3: sna_act of the stage */
  int32_t tail_ch, fc_ch;                    /* MBV3 head widths */
  int32_t hidden, n_heads, head_dim, ffn, seq_len, max_layers;   /* TRANSFORMER */
  int32_t max_res;                /* largest input height = width any cfg may ask for */
} sna_arch_desc;

/*
 * One resolved subnet: the control tuple of the paper (Depth D, Expand ratio E,
 * Width multiplier W; section "Weight-Shared Supernets") already turned into
 * integers by the caller, so that no rounding rule lives inside the library.
 * Kernel size and input resolution are extra knobs of the MBV3 / ResNet
 * workloads, not part of the paper's tuple.
 */
typedef struct {
  int32_t subnet_id;              /* row i of the SubnetNorm table */
  int32_t n_stages;               /* must equal the architecture's */
  int32_t depth[SNA_MAX_STAGES];  /* LayerSelect: blocks kept per stage, 1..stage_max_depth */
  int32_t stage_out_ch[SNA_MAX_STAGES + 1];  /* WeightSlice W: [0] stem, [1+s] stage s */
  int32_t block_mid_ch[SNA_MAX_STAGES][SNA_MAX_DEPTH]; /* WeightSlice E: bottleneck / expanded
                                      channels; TRANSFORMER: heads*head_dim of layer j */
  int32_t block_aux_ch[SNA_MAX_STAGES][SNA_MAX_DEPTH]; /* MBV3: SE squeeze channels;
                                      TRANSFORMER: FFN width of layer j; else 0 */
  int32_t block_kernel[SNA_MAX_STAGES][SNA_MAX_DEPTH]; /* MBV3 depthwise kernel 3|5|7; else 0 */
  int32_t in_h, in_w;             /* input resolution of requests using this cfg
                                     (TRANSFORMER: in_h = tokens per request, in_w = 1) */
} sna_subnet_cfg;

/* Layout of one weight tensor inside the weight blob, or of one SubnetNorm layer
 * inside a statistics row. */
typedef struct {
  char    name[SNA_NAME_LEN];
  int32_t kind;        /* 0 conv [K][R][S][C], 1 depthwise [R][S][C], 2 linear [K][C], 3 fp32 vector [C] */
  int32_t dtype;       /* sna_dtype of the stored elements */
  int32_t dims[4];     /* logical max-size dims, unused trailing dims = 1 */
  int32_t c_pad;       /* stored innermost extent (>= dims' innermost; extra entries must be 0) */
  int64_t offset;      /* byte offset in the weight blob */
  int64_t bytes;
} sna_tensor_info;

typedef struct {
  char    name[SNA_NAME_LEN];
  int32_t channels;    /* C_max of the layer */
  int32_t offset;      /* first column of the layer inside a statistics row */
} sna_norm_info;

typedef struct sna_supernet sna_supernet;     /* opaque handle */

/* ---- layout queries (host only, no GPU needed) ------------------------------------------- */

/* Number of weight tensors / SubnetNorm layers of `arch`, or a negative sna_status. */
int32_t sna_tensor_count(const sna_arch_desc* arch);
int32_t sna_norm_count(const sna_arch_desc* arch);
/* Fill *out for tensor / norm layer `index` (forward order). */
sna_status sna_tensor_info_get(const sna_arch_desc* arch, int32_t index, sna_tensor_info* out);
sna_status sna_norm_info_get(const sna_arch_desc* arch, int32_t index, sna_norm_info* out);
/* Bytes of the weight blob; columns of one statistics row (sum of C_max over norm layers).
 * The statistics table is fp32 [n_subnets][4][row_len], fields mean, var, gamma, beta. */
int64_t sna_weights_bytes(const sna_arch_desc* arch);
int64_t sna_stats_row_len(const sna_arch_desc* arch);
/* Workspace the handle needs for up to `max_batch` requests per call: folded
 * normalisation tables for n_subnets plus the activation arena at the largest cfg. */
int64_t sna_workspace_bytes(const sna_arch_desc* arch, int32_t n_subnets, int32_t max_batch);

/* ---- the two calls of the path ------------------------------------------------------------ */

/*
 * Make a SuperNet resident ("the supernet is submitted to the system", section
 * "System Architecture").  weights_dev: the max-size weights in the blob layout
 * reported above (shared by all subnets, SubNetAct "Reduced Memory Requirements").
 * stats_dev: SubnetNorm statistics for n_subnets subnets (SubnetNorm paragraph:
 * mu_{i,j}, sigma_{i,j} per subnet i and layer j; here with gamma, beta per
 * (i, j) as well).  The statistics are folded once, on `hip_stream`, into
 * per-channel scale = gamma / sqrt(var + 1e-5) and shift = beta - mean * scale
 * inside the workspace.  All three buffers must be 256-byte aligned.
 */
sna_status sna_supernet_load(const sna_arch_desc* arch,
                             const void* weights_dev, size_t weights_bytes,
                             const void* stats_dev, size_t stats_bytes,
                             int32_t n_subnets, int32_t max_batch,
                             void* workspace_dev, size_t workspace_bytes,
                             void* hip_stream,
                             sna_supernet** out);

/*
 * Forward pass of n_requests requests, request r through subnet cfgs[req_cfg[r]]
 * (worker paragraph of "System Architecture"; LayerSelect / WeightSlice /
 * SubnetNorm paragraphs).  The paper's worker runs one subnet per batch
 * (n_cfgs = 1); several cfgs in one call is this library's extension and gives
 * every request exactly the logits of its single-subnet run.
 *   cfgs, req_cfg  host memory, read before the call returns
 *   inputs_dev     requests concatenated in order; request r is
 *                  [in_h][in_w][in_ch] (TRANSFORMER: [in_h][hidden]) of the
 *                  architecture's dtype, sizes taken from its cfg
 *   logits_dev     fp32 [n_requests][n_classes]
 *   hidden_dev     TRANSFORMER only, may be NULL: final hidden states
 *                  [n_requests][seq][hidden] in the architecture's dtype
 *   hip_stream     hipStream_t; everything is enqueued on it, no host sync
 * Validation happens on the host first; on a validation error nothing is enqueued
 * (see the conventions above for SNA_E_HIP).
 * Calls on one handle must not overlap (they share the workspace).
 */
sna_status sna_subnet_forward(sna_supernet* net,
                              const sna_subnet_cfg* cfgs, int32_t n_cfgs,
                              const int32_t* req_cfg, int32_t n_requests,
                              const void* inputs_dev, float* logits_dev,
                              void* hidden_dev, void* hip_stream);

/*
 * sna_subnet_forward for callers that cannot allocate device memory or hand over a
 * large workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same kernels, same bits in the results.
 * The per-call scratch (activation buffers, request gather, pooled vectors, fp32
 * partial sums of split reductions) is taken from a static device array inside the
 * library instead of the handle's workspace; only the folded SubnetNorm tables
 * written by sna_supernet_load are still read from the workspace.  The array holds
 * sna_static_scratch_bytes() = 256 MiB per GPU, from library load until the process
 * ends: 224 MiB for activations, sized like the workspace (per request, at the
 * architecture's max_res), which is 8 requests of a ResNet-50-shaped SuperNet with
 * max_res 224, 11 of the MBV3-shaped one, 36 128-token requests of the 12 x 768
 * transformer; 32 MiB for split-reduction partial sums (a layer whose partial sums
 * do not fit is reduced inside its blocks instead: same bits).  A call whose requests need more returns
 * SNA_E_WORKSPACE with the sizes in sna_last_error(), before anything is enqueued.
 * Makes no hipMalloc / hipFree and calls no allocating library routine; the array's
 * device address is resolved once per device (by sna_supernet_load on that device,
 * else by the first call).  Nothing in the array needs a defined initial value, and
 * nothing is kept in it between calls.  All calls on one GPU share the one array:
 * calls that overlap in time on a GPU (two streams, two handles, two threads) race;
 * serialise them.  Not available while sna_profile_enable is on (SNA_E_BATCH).
 * Other errors: as sna_subnet_forward.
 */
sna_status sna_subnet_forward_static(sna_supernet* net,
                                     const sna_subnet_cfg* cfgs, int32_t n_cfgs,
                                     const int32_t* req_cfg, int32_t n_requests,
                                     const void* inputs_dev, float* logits_dev,
                                     void* hidden_dev, void* hip_stream);
int64_t sna_static_scratch_bytes(void);

/* Same arguments and result as sna_subnet_forward, but every conv / linear layer
 * shape met for the first time on this handle gets a measured tile variant of the
 * matrix kernel, remembered for later sna_subnet_forward calls with that shape.
 * Two steps: each new shape alone, launched back to back with every variant (this
 * also decides whether a long reduction is split over blocks); then, if the call
 * met any new shape, the whole forward is run with every launch forced to one
 * variant, for each variant in turn, every launch timed between two events, and a
 * new shape keeps the variant with the least time inside the forward (operands
 * come from HBM there, not from caches warmed by the previous repeat).  Step 2 is
 * skipped while sna_profile_enable is on.  The paper's serving system profiles
 * each subnet offline before serving; this is the same step for the kernels.
 * Tile variants do not change a bit of the result.  Synchronises on the stream
 * many times; returns after it has drained.  Not for use under stream capture.
 * Errors: as sna_subnet_forward. */
sna_status sna_subnet_tune(sna_supernet* net,
                           const sna_subnet_cfg* cfgs, int32_t n_cfgs,
                           const int32_t* req_cfg, int32_t n_requests,
                           const void* inputs_dev, float* logits_dev,
                           void* hidden_dev, void* hip_stream);

/* SubnetNorm calibration of one subnet (the paper computes every subnet's
 * normalisation statistics by forward passes over data before serving; section
 * "SubNetAct", SubnetNorm paragraph).  Runs cfg on n_requests inputs; every
 * SubnetNorm layer the subnet executes takes the per-channel mean and population
 * variance of its own input (the layer's convolution output in fp32, over all
 * requests and pixels), writes them as fp32 into row cfg->subnet_id of stats_dev
 * (fields mean and var, the layer's leading active channels; gamma, beta, other
 * rows and the layers of skipped blocks are left alone), refreshes the folded
 * scale / shift kept in the workspace, and normalises with the values as stored,
 * so that a later sna_subnet_forward of the same cfg on the same inputs returns
 * the same logits (to summation order where the calibration pass runs a layer
 * on another kernel than serving does: the squeeze-excite pool, the 7x7 stem).  stats_dev must be the device table given to
 * sna_supernet_load (the caller still owns it; this is the one call that writes
 * it).  logits_dev [n_requests][n_classes] receives that forward's logits.
 * The fp32 outputs of the layers launched together (a block's last convolution
 * and its projection shortcut) must fit the 64 MiB scratch region of the
 * workspace: SNA_E_WORKSPACE otherwise, before anything runs (use a smaller batch).  SNA_E_ARCH for families
 * without SubnetNorm.  Not for use concurrently with other calls on the handle. */
sna_status sna_subnet_calibrate(sna_supernet* net, const sna_subnet_cfg* cfg,
                                int32_t n_requests, const void* inputs_dev,
                                void* stats_dev, float* logits_dev, void* hip_stream);

/* Number of layer shapes with a measured tile variant on this handle. */
int32_t sna_tuned_count(const sna_supernet* net);

/* The measured choices as text, one per line ("v M K C RS stride parts twins variant" for a tile
 * variant, "s M K C RS stride 0 twins flag" for the K-split decision; twins = problems of this
 * shape that share the launch, e.g. 3 for a layer's Q, K and V projections; a line without the
 * twins field is read as twins = 1), so that a deployment can ship them instead of measuring at
 * every start.  Export writes at most `cap` bytes (host memory,
 * NUL-terminated when it fits) and returns the size needed, excluding the NUL.  Import adds
 * the lines of `text` (host memory, `len` bytes) to the handle's tables, replacing entries for
 * the same shape; lines it cannot parse or that name an unknown variant give SNA_E_CFG_RANGE and
 * nothing is imported.  Choices are hints: a wrong one costs time, never correctness. */
int64_t sna_tuning_export(const sna_supernet* net, char* buf, int64_t cap);
sna_status sna_tuning_import(sna_supernet* net, const char* text, int64_t len);

void sna_supernet_free(sna_supernet* net);

/* How long reductions are laid out over blocks.  A conv / linear whose reduction is
 * longer than 1536 elements is summed in 2 or 4 chunks (a function of the layer's
 * active shape only), chunk sums added in order in fp32.  mode 0 (default): when a
 * layer has too few output tiles to fill the GPU (or a measured table entry says
 * so), each chunk gets its own blocks, which leave fp32 chunk sums in the
 * workspace; the block that arrives last at a tile adds them in chunk order and
 * finishes the layer inside the same launch.  Otherwise one block walks all
 * chunks.  mode 1: never spread chunks over blocks.  mode 2: always, when the
 * layer is chunked.  mode 3: as 2, but the chunk sums are added by a separate
 * reduction launch (the fall-back used when a launch has more tiles than the
 * workspace has tile counters, 16384).  The logits have the same bits in all
 * modes; the knob exists for timing and for checking that property.
 * Errors: SNA_E_NULL, SNA_E_CFG_RANGE. */
sna_status sna_set_k_split(sna_supernet* net, int32_t mode);

/* Test / timing knob: force every conv / linear launch of the matrix kernel onto tile variant
 * `variant` (0 <= variant < sna_tile_variant_count()), or back to the measured / heuristic choice
 * with -1.  A variant that cannot run a layer (some take 3x3 stride-1 convolutions only) leaves that
 * layer on its usual choice.  The result does not depend on the variant.  Errors: SNA_E_NULL,
 * SNA_E_CFG_RANGE. */
int32_t sna_tile_variant_count(void);
sna_status sna_set_tile_variant(sna_supernet* net, int32_t variant);

/* Multiply-accumulate count and launch count of the last successful forward on
 * this handle (host bookkeeping for reports). */
sna_status sna_last_forward_info(const sna_supernet* net, int64_t* macs, int32_t* launches);

/* Per-launch timing: when enabled, every kernel launch of sna_subnet_forward is
 * bracketed by HIP events on the caller's stream; sna_profile_read() syncs them
 * and returns, per kernel class, total milliseconds, launch count, algorithmic
 * flops and algorithmic bytes accumulated since the last read.  Classes are
 * listed by sna_profile_class_name(). */
#define SNA_N_KCLASS 12
sna_status sna_profile_enable(sna_supernet* net, int32_t on);
sna_status sna_profile_read(sna_supernet* net, double ms[SNA_N_KCLASS], int64_t launches[SNA_N_KCLASS],
                            double flops[SNA_N_KCLASS], double bytes[SNA_N_KCLASS]);
const char* sna_profile_class_name(int32_t kclass);
/* The launches recorded since the last sna_profile_read(), one text line each in
 * launch order: microseconds between the launch's two events, class name,
 * "flops=" and "bytes=" (the launch's algorithmic work, active sizes only), then
 * for the grouped kernels the tile variant and every problem's active shape.
 * Syncs the events; does not clear them (sna_profile_read() does).  Writes at most
 * cap - 1 bytes plus a NUL into buf (host memory, may be NULL) and returns the
 * full length, or -1 on error. */
int64_t sna_profile_read_launches(sna_supernet* net, char* buf, int64_t cap);

const char* sna_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SUBNETACT_H */
