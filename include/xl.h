/*
 * xl -- cross-layer fused CNN blocks for AMD MI355X (gfx950 / CDNA4).
 *
 * C ABI of libxl.so.  Plain C types only: no C++ objects, no torch types, no
 * HIP types (a stream is passed as `void*` holding a hipStream_t).
 *
 * What the library does.  A convolutional network is given as a small layer
 * graph plus a list of fusion blocks.  Each block is one of the paper's three
 * fusion modes (section 3.1, Fig. 4): straight (Layer1 -> Layer2), split
 * (Layer1 -> {Layer2, Layer3}) or merge (two producers -> one consumer).  For
 * every block `xl_plan_create` picks an output tile and the halo ("redundant
 * data", section 3.2) each workgroup must recompute so that the block's
 * intermediate feature map can stay in LDS, against the LDS capacity of one
 * compute unit (section 3.2: shared memory is the bottleneck resource, keep the
 * share per block well below the whole).  `xl_run` then executes the network:
 * one fused kernel per block (intermediate in LDS, section 2.2 Fig. 3b:
 * LD.G, CONV1, ST.S, barrier, LD.S, CONV2, ST.G) or, for comparison, one
 * kernel per layer with every intermediate written to and re-read from HBM
 * (Fig. 3a).  Both paths use the same tiled implicit-GEMM convolution
 * (section 3.2) on the fp32 matrix cores, or, when xl_options.precision asks
 * for it, on the bf16 matrix cores with every operand split into two bf16
 * numbers.
 *
 * Data.  All tensors are dense fp32 NCHW in DEVICE memory owned by the caller
 * (e.g. allocated by PyTorch).  Filters are [Cout, Cin, K, K] fp32 (section 4.1
 * notation), per-channel scale/shift/bias vectors are [Cout] fp32.  The library
 * allocates no device memory; intermediates and re-laid-out filters live in a
 * caller-provided workspace of `xl_plan_workspace_bytes` bytes, 256-byte
 * aligned.  A plan owns host metadata only.
 *
 * Calls never throw or abort.  `xl_prepare` and `xl_run` only enqueue work on
 * the given stream and return without synchronising.  Every function returns
 * XL_OK (0) or a negative xl_status; `xl_strerror` names it, and
 * `xl_plan_last_error` gives a longer message for the last failure on a plan
 * handle (or of the last failed `xl_plan_create` when passed NULL).
 */
#ifndef XL_H
#define XL_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int xl_status;
#define XL_OK              0
#define XL_E_NULL        (-1)   /* a required pointer was NULL                          */
#define XL_E_SHAPE       (-2)   /* tensor shapes do not fit the layer parameters        */
#define XL_E_UNSUPPORTED (-3)   /* layer or fusion block outside what the kernels cover */
#define XL_E_LDS_BUDGET  (-4)   /* no tile fits the LDS budget (paper section 3.2: the
                                   kernel would fail for resource limitation)           */
#define XL_E_DEVICE      (-5)   /* device is not gfx950 or cannot be queried            */
#define XL_E_ALIGN       (-6)   /* workspace or tensor pointer not aligned              */
#define XL_E_LAUNCH      (-7)   /* a kernel launch was rejected by the runtime          */
#define XL_E_GRAPH       (-8)   /* graph wiring invalid (ids, order, group membership)  */
#define XL_E_STATE       (-9)   /* xl_run before xl_prepare on this workspace           */
#define XL_E_SCRATCH     (-10)  /* plan needs more workspace than xl_run_static holds   */

/* Layer kinds (paper section 2.2: convolution, pooling, activation, element-wise
 * addition and concatenation are the basic operations; activation rides in the
 * producing layer's epilogue). */
enum { XL_CONV = 0, XL_MAXPOOL = 1, XL_GLOBAL_AVGPOOL = 2, XL_ADD = 3, XL_CONCAT = 4 };

/* Fusion modes (paper section 3.1, Fig. 4).  XL_SINGLE is a block of one layer. */
enum { XL_SINGLE = 0, XL_STRAIGHT = 1, XL_SPLIT = 2, XL_MERGE = 3 };

typedef struct xl_shape { int n, c, h, w; } xl_shape;        /* dense NCHW fp32 */

/*
 * One layer.  `in` / `out` are tensor ids (indices into the shapes array);
 * in[1] is used by XL_ADD and XL_CONCAT only (-1 otherwise).
 * XL_CONV:   y = act(scale * corr(x, filter) + shift); square K x K filter with
 *            K = 1, 3 or 5, zero padding.  groups is 1, or equal to cin == cout
 *            (depthwise, K = 3, filter [C, 1, K, K]; paper Table 1 case a.2).
 *            Slots index the `weights` array of xl_prepare; scale_slot /
 *            shift_slot may be -1 (scale 1 / shift 0).  A bias is a shift with no
 *            scale; a folded batch-norm is both.
 * XL_MAXPOOL: K x K window, stride, pad; out-of-image taps are ignored.
 * XL_GLOBAL_AVGPOOL: mean over H x W -> [N, C, 1, 1].
 * XL_ADD:    y = act(in[0] + in[1]).
 * XL_CONCAT: channels of in[0] then in[1]; costs nothing: the producers write
 *            straight into the concatenated tensor at their channel offset.
 */
typedef struct xl_layer {
    int op;
    int in[2];
    int out;
    int cin, cout;
    int k, stride, pad, groups;
    int relu;
    int w_slot, scale_slot, shift_slot;
} xl_layer;

/* A fusion block: `mode` and the layer indices it covers, in graph order.
 *   XL_STRAIGHT: conv -> conv, conv -> maxpool, conv -> global average pooling
 *                (the image must fit one workgroup tile), depthwise conv -> conv
 *   XL_SPLIT:    conv -> {conv, conv} [-> concat [-> maxpool]]; the max pooling (with or without
 *                padding) is applied to the concatenated result before it leaves the chip, so
 *                only the pooled tensor is written
 *   XL_MERGE:    conv -> conv -> add(., block input)          (residual block), or
 *                {conv, conv}(block input) -> add -> conv      (two producers, all 1x1)
 *   XL_SINGLE:   any one layer
 * Layers not listed in any block are planned as XL_SINGLE. */
typedef struct xl_group {
    int mode;
    int nlayers;
    const int *layer_ids;
} xl_group;

/* Planner knobs; zero-initialise for defaults. */
typedef struct xl_options {
    int lds_budget_bytes;   /* LDS one workgroup may use; 0 = device limit (160 KB on gfx950) */
    int num_cus;            /* compute units to fill; 0 = query device (256 when device < 0)  */
    int force_tile_h;       /* >0: fix the output tile of every fused block (tests, tuning)   */
    int force_tile_w;
    int force_cout_split;   /* >0: fix how many workgroups share one tile's output channels   */
    int paper_tuner_only;   /* 1: restrict candidates to the paper's square common-factor
                               (tile, grid) pairs (section 3.2)                               */
    int force_threads;      /* >0: fix the workgroup size (256 or 512) of every block         */
    int precision;          /* XL_PRECISION_FP32 (0, default): fp32 matrix operations.
                               XL_PRECISION_BF16X3: every operand of a convolution is split into
                               two bf16 numbers, hi = bf16(x) and lo = bf16(x - hi), and a product
                               is hi*hi + hi*lo + lo*hi on the bf16 matrix cores, accumulated in
                               fp32 (error at most 3 * 2^-16 of |a||b| per product, about 4e-6 rms; operands must be
                               finite and below 2^127 in magnitude).  The error of an output is therefore
                               relative to sum(|a||b|) over its reduction, not to the output itself: the
                               library's bar |err| <= 1e-4 + 1e-4 |out| holds for data of the benchmark's
                               scale (activations and filter sums of order 1, where 3 * 2^-16 * sum|a||b|
                               stays under 1e-4); on inputs scaled by s the absolute part of the bar has to
                               scale with s as well, i.e. the guarantee is |err| <= 1e-4 * max|out| there.
                               Tensors in memory stay fp32.
                               A depthwise first layer stays on the vector ALU in fp32; xl_tune may
                               keep an fp32 kernel for a block where it measures faster. */
    int keep_blocks_fused;  /* 1: xl_tune never switches a block to layer-by-layer execution (see
                               xl_plan_set_block_fused)                                            */
} xl_options;
#define XL_PRECISION_FP32   0
#define XL_PRECISION_BF16X3 1

/* What the planner decided for one block (all sizes in elements unless named bytes). */
typedef struct xl_group_info {
    int mode;
    int first_layer, nlayers;
    int tile_h, tile_w;         /* output tile of the block's last spatial layer            */
    int mid_h, mid_w;           /* on-chip intermediate tile incl. halo (0 for XL_SINGLE)   */
    int in_h, in_w;             /* input tile incl. halo                                    */
    int tiles_y, tiles_x;       /* grid over the output image (paper: "grid size")          */
    int cout_split;             /* workgroups sharing a tile, each a slice of Cout          */
    int workgroups;             /* tiles_y * tiles_x * cout_split * N                       */
    int threads;                /* workgroup size                                           */
    int lds_bytes;              /* LDS per workgroup                                        */
    int workgroups_per_cu;      /* co-resident workgroups the LDS share allows              */
    int chunk_channels;         /* input channels staged through LDS per pipeline step      */
    long long bytes_fused;      /* algorithmic HBM bytes: block input + filters + output    */
    long long bytes_unfused;    /* same with every layer reading/writing HBM                */
    long long stores_fused;     /* elements written to HBM, fused   (paper Table 2)         */
    long long stores_unfused;   /* elements written to HBM, unfused (paper Table 2)         */
    long long flops;            /* 2*MAC, no halo recompute                                 */
    long long flops_executed;   /* 2*MAC the fused kernel issues incl. halo and tile padding */
    double redundancy;          /* intermediate elements computed / unique elements         */
    int precision;              /* arithmetic of the block's kernel: XL_PRECISION_*         */
} xl_group_info;

typedef struct xl_plan xl_plan;

/*
 * Validate the graph and blocks, choose tiles, build launch descriptors.
 * Host only; touches the device solely to query its properties when
 * device >= 0 (device < 0 plans for a nominal gfx950: 256 CUs, 160 KB LDS,
 * and works on a machine without a GPU).  `opts` may be NULL.
 * On success *out holds a plan to be freed with xl_plan_destroy.
 */
xl_status xl_plan_create(const xl_layer *layers, int nlayers,
                         const xl_shape *shapes, int ntensors,
                         const xl_group *groups, int ngroups,
                         int device, const xl_options *opts, xl_plan **out);

/* Frees the host metadata of a plan (NULL is allowed).  No device memory is touched. */
void xl_plan_destroy(xl_plan *plan);

/* Number of fusion blocks of the plan in graph order (paper section 3.1, Fig. 5: the dotted
 * boxes of the compute graph); layers outside every listed block count as XL_SINGLE blocks. */
int xl_plan_num_groups(const xl_plan *plan);

/* What was decided for block `group` (0 .. xl_plan_num_groups - 1): the output tile and grid
 * (paper section 3.2: "tiling size" and "grid size"), the halo-extended intermediate and input
 * tiles (section 3.2: redundant data), the LDS share of one workgroup (section 3.2: shared memory
 * is the bottleneck resource) and the block's algorithmic traffic, fused and unfused (section 2.2
 * Fig. 3; stored elements as counted in Table 2).  XL_E_GRAPH for a group out of range. */
xl_status xl_plan_query(const xl_plan *plan, int group, xl_group_info *out);

/* Bytes of caller-provided device workspace: the filters re-laid out for the matrix cores (the
 * counterpart of the paper's filters and bias placed in constant memory, section 3.3) plus every
 * tensor that one kernel writes and a later one reads -- in the unfused path each layer's output
 * (section 2.2 Fig. 3a), in the fused path only tensors between blocks. */
size_t xl_plan_workspace_bytes(const xl_plan *plan);

/*
 * Upload step before the first launch (paper section 2.1: read-only data is copied to the device
 * and placed where the kernels read it fastest before a kernel runs; section 3.3: filters and bias
 * are read-only and get a placement of their own).
 * Re-lay the filters into `workspace` (device) for the matrix-core kernels: the
 * per-channel scale is multiplied into the re-laid-out filter (one more fp32
 * rounding per weight), the shift is re-laid out in accumulator order.  `weights[slot]` are DEVICE pointers indexed
 * by the slots named in xl_layer; they must stay valid and unchanged until the
 * last xl_run that uses this workspace has finished.  Call once per workspace,
 * and again whenever filter values change; a plan remembers every workspace it
 * has prepared.  The plan's device must be the current HIP device (XL_E_DEVICE
 * otherwise).  Enqueues on `stream`; returns without synchronising.  Not
 * thread-safe against other calls on the same plan.
 */
xl_status xl_prepare(xl_plan *plan, const void *const *weights, int nweights,
                     void *workspace, void *stream);

/*
 * Execute the network once.  `tensors[id]` are DEVICE pointers by tensor id;
 * only tensors that no layer produces (graph inputs) and tensors that no layer
 * consumes (graph outputs) are read from this array -- every other entry may be
 * NULL and lives in the workspace.  fused = 1: one kernel per fusion block;
 * fused = 0: one kernel per layer (concat still free).  Stream-ordered,
 * asynchronous; results are complete when the stream reaches this point.
 * Two xl_run calls that share a workspace must be ordered on one stream.
 * The call enqueues kernel launches only (no allocation, no copy, no memset, no
 * synchronisation), so it may be recorded into a HIP graph by a capturing stream.
 * Every tensor pointer read from `tensors` must be 16-byte aligned (XL_E_ALIGN); the plan's device
 * must be the current HIP device (XL_E_DEVICE).  The plan is not modified: several threads may run
 * one plan at the same time (on workspaces of their own); the message of a failure is kept per
 * thread and returned by xl_plan_last_error on that thread.
 */
xl_status xl_run(const xl_plan *plan, const void *const *tensors, int ntensors,
                 void *workspace, void *stream, int fused);

/*
 * Measured tuning (paper section 3.2: a tuning tool searches tile sizes because the best one is a
 * trade-off the data dependency alone does not settle).  For every convolution block, in both
 * execution modes, times the planner's ranked candidates (tile, workgroup size, wave layout,
 * output-channel split) on the device with the caller's buffers and keeps the fastest; afterwards
 * xl_plan_query reports the adopted tiles.  Needs xl_prepare on this workspace first.  Contents of
 * the tensors do not matter but every graph input/output pointer must be valid; outputs and the
 * workspace intermediates are overwritten.  Unlike xl_run this call SYNCHRONISES the stream
 * repeatedly; call it once, outside any timed region.  Every candidate is timed three times (fastest
 * kept) and the six fastest again `reps` times each (reps < 5 means 5), ranked by their MEDIAN
 * time; ties go to the lower candidate index.  xl_plan_candidate_info(.., -1, ..) names the winner.
 * Last, a block whose layers, run back to back one kernel each, take less than 0.97 of the time of its fused
 * kernel (both medians of this call) is switched to layer-by-layer execution inside the fused path, as by
 * xl_plan_set_block_fused(.., 0), and every other block is (re)set to fused; options.keep_blocks_fused = 1
 * leaves that step out.
 */
xl_status xl_tune(xl_plan *plan, const void *const *tensors, int ntensors,
                  void *workspace, void *stream, int reps);

/*
 * xl_prepare + xl_run for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The workspace is not the caller's but a
 * static device array inside the library, XL_STATIC_SCRATCH_BYTES long, which every GPU the library
 * runs on holds from the first call on that GPU until the process ends.  The call allocates no
 * device memory and frees none; it enqueues kernels on `stream` and returns without synchronising.
 *   - XL_E_SCRATCH when xl_plan_workspace_bytes(plan) exceeds XL_STATIC_SCRATCH_BYTES (configs 1-4 at
 *     their full sizes fit; config 5 up to batch 4).
 *   - relayout != 0: the filters are re-laid out into the array first (as xl_prepare does), from
 *     `weights` / `nweights`; needed on the first call and whenever filter values change.
 *     relayout == 0: the filters are re-laid out only if the array's last user on this GPU was another
 *     plan (then `weights` must be given: XL_E_STATE if it is NULL); otherwise `weights` may be NULL.
 *   - `tensors`, `fused`: as xl_run.  Graph inputs and outputs stay the caller's buffers.
 * All calls on one GPU share that GPU's array, and the array keeps what the last call left: nothing in
 * it has to start at zero (filters are rewritten, every intermediate is written before it is read), but
 * two calls that overlap in time on one GPU -- different streams, different threads -- race on it.
 * Order them on one stream.  The current device must be the plan's.
 */
#define XL_STATIC_SCRATCH_BYTES (64u << 20)
xl_status xl_run_static(xl_plan *plan, const void *const *weights, int nweights, const void *const *tensors,
                        int ntensors, void *stream, int fused, int relayout);

/*
 * Per-launch timing of one execution mode (paper section 4.1: every measurement is run several times and
 * averaged, with timers on the GPU side).  Runs the network `reps` times (reps < 1 means 5) like xl_run,
 * with an event before and after every kernel launch on `stream`, then SYNCHRONISES the stream and writes the
 * average duration of each launch in microseconds to launch_us[0 .. xl_plan_num_launches(plan, fused) - 1]
 * (host memory, `cap` entries available; XL_E_GRAPH if cap is too small).  One untimed run comes first.
 * Tensors and workspace as for xl_run; outputs and workspace intermediates are overwritten.
 */
xl_status xl_profile(const xl_plan *plan, const void *const *tensors, int ntensors, void *workspace, void *stream,
                     int fused, int reps, float *launch_us, int cap);

/*
 * What this GPU sustains, measured, to put next to the published peaks the roofline fractions are quoted
 * against (paper section 4.1 lists the peaks of its two GPUs the same way):
 *   copy_gbs          a plain copy kernel over `bytes` bytes from `src` to `dst` (both DEVICE buffers of at
 *                     least `bytes` bytes, 16-byte aligned; use more than the 256 MB last-level cache):
 *                     bytes read + bytes written per second, in GB/s
 *   mfma_f32_tflops   a loop of independent V_MFMA_F32_32X32X2_F32 operations on registers, every compute unit busy
 *   mfma_bf16_tflops  the same with V_MFMA_F32_32X32X16_BF16
 *   valu_f32_tflops   a loop of independent (not packed) v_fma_f32 operations
 * Any output pointer may be NULL.  `dst` is overwritten (its first 2 MiB also serve the arithmetic loops as a
 * sink: bytes must be at least 2 MiB).  SYNCHRONISES the stream; allocates nothing.
 */
xl_status xl_measure_peaks(void *dst, const void *src, size_t bytes, void *stream, double *copy_gbs,
                           double *mfma_f32_tflops, double *mfma_bf16_tflops, double *valu_f32_tflops);

/* Number of kernel launches one xl_run issues in the given mode (paper section 2.2, Fig. 3: one
 * kernel per layer unfused, one per fusion block fused). */
int xl_plan_num_launches(const xl_plan *plan, int fused);

/*
 * The tuner's search space made visible (paper section 3.2: the tuning tool searches (tile, grid)
 * candidates and must not change results).  Every launch of a plan (index 0 ..
 * xl_plan_num_launches(plan, fused) - 1, in launch order) has a ranked list of candidate launch
 * configurations: kernel variant, output tile, workgroup size, wave layout, chunk length and
 * output-channel split.  Candidate 0 is the cost model's choice; xl_tune adopts the one it measures
 * fastest; xl_plan_select_candidate adopts one by index, so that a caller can time or check each.
 * Element-wise launches (pooling, add, depthwise, global pooling of the unfused path) have exactly
 * one candidate.
 */
typedef struct xl_launch_info {
    int group;              /* fusion block the launch belongs to (fused mode), -1 in unfused mode  */
    int first_layer;        /* first layer the launch executes                                     */
    int nlayers;            /* layers the launch executes (1 in unfused mode)                      */
    int is_block_kernel;    /* 1: a convolution block kernel; 0: an element-wise kernel            */
    int candidate;          /* index of this configuration in the launch's candidate list          */
    int variant;            /* id of the compiled kernel variant (block kernels)                   */
    int tile_h, tile_w;     /* output tile                                                         */
    int threads;            /* workgroup size                                                      */
    int cout_split;         /* workgroups sharing a tile, each a slice of the output channels      */
    int waves_cout_1, waves_cout_2;   /* waves along the output-channel direction, stage 1 / 2    */
    int chunk_channels;     /* input channels staged per pipeline step of stage 1                  */
    int lds_bytes;          /* LDS per workgroup                                                   */
    int workgroups;         /* workgroups launched (logical: tiles * cout_split * N)               */
    int precision;          /* XL_PRECISION_*                                                      */
    double model_cost_us;   /* the cost model's estimate for this candidate                        */
} xl_launch_info;

/* Number of candidates of a launch; 0 when plan is NULL or the launch index is out of range. */
int xl_plan_num_candidates(const xl_plan *plan, int fused, int launch);

/* Describes candidate `candidate` of a launch; candidate = -1 describes the adopted one.
 * XL_E_GRAPH for an index out of range. */
xl_status xl_plan_candidate_info(const xl_plan *plan, int fused, int launch, int candidate, xl_launch_info *out);

/* Adopts candidate `candidate` for a launch: later xl_run calls use it, and xl_plan_query reports
 * its tiles for the launch's block.  Host only; must not race with xl_run on the same plan. */
xl_status xl_plan_select_candidate(xl_plan *plan, int fused, int launch, int candidate);

/*
 * Fused or layer by layer.  Cross-layer reuse pays when the intermediate tensor would otherwise travel
 * through off-chip memory (paper section 3.1); where it would not -- images of a few hundred pixels at a
 * batch that cannot fill the chip with whole tiles, a batch of 1 -- the halo recomputation and the
 * larger workgroups of a fused block (paper section 3.2: the tile size is a trade-off) can cost more than
 * the reuse saves.  fused = 0 makes xl_run(.., fused = 1) execute the layers of block `group` one kernel each,
 * exactly as the unfused path does, in the block's place; fused = 1 restores the block's kernel.  Blocks of
 * one layer ignore the call.  The launch list of the fused path changes with it: xl_plan_num_launches,
 * the launch indices of the candidate functions and of xl_profile follow the current list.
 * xl_plan_block_is_fused: 1 if the block (of at least two layers) currently runs as one kernel, else 0.
 * Not thread-safe against concurrent xl_run on the same plan.  XL_E_GRAPH for an unknown block.
 */
xl_status xl_plan_set_block_fused(xl_plan *plan, int group, int fused);
int xl_plan_block_is_fused(const xl_plan *plan, int group);

/*
 * The paper's tuner search space (section 3.2): square tiles whose size and
 * grid are complementary non-trivial factors of the output size; a prime size
 * is replaced by the next larger non-prime.  Writes up to `cap` (tile, grid)
 * pairs into tile[] / grid[] and returns how many exist.
 */
int xl_tuner_candidates(int out_size, int *tile, int *grid, int cap);

/* Halo arithmetic of section 3.2: input extent needed for `t` outputs of a
 * K-wide, stride-s window: (t - 1) * s + K. */
int xl_required_extent(int t, int k, int stride);

const char *xl_strerror(xl_status st);
const char *xl_plan_last_error(const xl_plan *plan);

/* Version / build string, e.g. "xl 0.1 gfx950". */
const char *xl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* XL_H */
