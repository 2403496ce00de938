// C ABI of libxl (see include/xl.h).
#include <cstdint>
#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "plan.h"

namespace xl {
xl_status build_plan(xl_plan &pl, const xl_group *groups, int ngroups);
int tuner_candidates(int out_size, int *tile, int *grid, int cap);
int required_extent(int t, int k, int s);
}  // namespace xl

static thread_local std::string g_create_error;
// xl_run leaves the plan untouched: the message of a failed run lives with the calling thread
static thread_local std::string g_run_error;
static thread_local const xl_plan *g_run_error_plan = nullptr;

static xl_status run_fail(const xl_plan *plan, xl_status st, const std::string &msg)
{
    g_run_error = msg;
    g_run_error_plan = plan;
    return st;
}

static constexpr int GFX950_LDS_BYTES = 160 * 1024;
static constexpr int GFX950_CUS = 256;

extern "C" {

const char *xl_version(void) { return "xl 0.1 gfx950"; }

const char *xl_strerror(xl_status st)
{
    switch (st) {
    case XL_OK: return "ok";
    case XL_E_NULL: return "null pointer";
    case XL_E_SHAPE: return "tensor shapes do not fit the layer parameters";
    case XL_E_UNSUPPORTED: return "layer or fusion block not supported";
    case XL_E_LDS_BUDGET: return "no tile fits the LDS budget";
    case XL_E_DEVICE: return "device is not gfx950 or cannot be queried";
    case XL_E_ALIGN: return "pointer not aligned";
    case XL_E_LAUNCH: return "kernel launch failed";
    case XL_E_GRAPH: return "invalid graph wiring";
    case XL_E_STATE: return "xl_prepare has not been called for this workspace";
    case XL_E_SCRATCH: return "the plan needs more workspace than the static scratch array holds";
    }
    return "unknown status";
}

const char *xl_plan_last_error(const xl_plan *plan)
{
    if (!plan) return g_create_error.c_str();
    if (g_run_error_plan == plan && !g_run_error.empty()) return g_run_error.c_str();
    return plan->error.c_str();
}

int xl_tuner_candidates(int out_size, int *tile, int *grid, int cap) { return xl::tuner_candidates(out_size, tile, grid, cap); }

int xl_required_extent(int t, int k, int stride) { return xl::required_extent(t, k, stride); }

xl_status xl_plan_create(const xl_layer *layers, int nlayers, const xl_shape *shapes, int ntensors,
                         const xl_group *groups, int ngroups, int device, const xl_options *opts, xl_plan **out)
{
    g_create_error.clear();
    if (!out) return XL_E_NULL;
    *out = nullptr;
    if (!layers || !shapes || (ngroups > 0 && !groups)) {
        g_create_error = "layers, shapes or groups is NULL";
        return XL_E_NULL;
    }
    if (nlayers < 1 || ntensors < 1 || ngroups < 0) {
        g_create_error = "empty graph";
        return XL_E_GRAPH;
    }
    xl_plan *pl = new (std::nothrow) xl_plan;
    if (!pl) return XL_E_NULL;
    pl->layers.assign(layers, layers + nlayers);
    pl->shapes.assign(shapes, shapes + ntensors);
    if (opts) pl->opts = *opts;
    if (pl->opts.precision != XL_PRECISION_FP32 && pl->opts.precision != XL_PRECISION_BF16X3) {
        delete pl;
        return XL_E_UNSUPPORTED;
    }
    static std::atomic<unsigned long long> next_serial{1};
    pl->serial = next_serial.fetch_add(1);
    pl->device = device;
    pl->lds_per_cu = GFX950_LDS_BYTES;
    pl->num_cus = GFX950_CUS;
    if (device >= 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, device) != hipSuccess || strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
            g_create_error = "device is not a gfx950 GPU";
            delete pl;
            return XL_E_DEVICE;
        }
        pl->num_cus = prop.multiProcessorCount;
    }
    if (pl->opts.num_cus > 0) pl->num_cus = pl->opts.num_cus;
    pl->lds_budget = pl->lds_per_cu;
    if (pl->opts.lds_budget_bytes > 0) pl->lds_budget = std::min(pl->opts.lds_budget_bytes, pl->lds_per_cu);
    xl_status st = xl::build_plan(*pl, groups, ngroups);
    if (st != XL_OK) {
        g_create_error = pl->error;
        delete pl;
        return st;
    }
    *out = pl;
    return XL_OK;
}

void xl_plan_destroy(xl_plan *plan) { delete plan; }

int xl_plan_num_groups(const xl_plan *plan) { return plan ? (int)plan->groups.size() : 0; }

xl_status xl_plan_query(const xl_plan *plan, int group, xl_group_info *out)
{
    if (!plan || !out) return XL_E_NULL;
    if (group < 0 || group >= (int)plan->groups.size()) return XL_E_GRAPH;
    *out = plan->groups[group].info;
    return XL_OK;
}

size_t xl_plan_workspace_bytes(const xl_plan *plan) { return plan ? plan->workspace_bytes : 0; }

int xl_plan_num_launches(const xl_plan *plan, int fused)
{
    if (!plan) return 0;
    return (int)(fused ? plan->fused_active.size() : plan->unfused_steps.size());
}

// The launches of one execution mode, in order.
static std::vector<const xl::Step *> launches_of(const xl_plan *plan, int fused)
{
    std::vector<const xl::Step *> v;
    if (fused) {
        v.assign(plan->fused_active.begin(), plan->fused_active.end());
    } else {
        v.reserve(plan->unfused_steps.size());
        for (const xl::Step &st : plan->unfused_steps) v.push_back(&st);
    }
    return v;
}

// Fusion block a layer belongs to (-1: none).
static int group_of_layer(const xl_plan *plan, int layer)
{
    for (size_t g = 0; g < plan->groups.size(); ++g)
        for (int l : plan->groups[g].layers)
            if (l == layer) return (int)g;
    return -1;
}

int xl_plan_block_is_fused(const xl_plan *plan, int group)
{
    if (!plan || group < 0 || group >= (int)plan->groups.size()) return 0;
    return plan->groups[group].layers.size() > 1 && !plan->layerwise[group];
}

xl_status xl_plan_set_block_fused(xl_plan *plan, int group, int fused)
{
    if (!plan) return XL_E_NULL;
    if (group < 0 || group >= (int)plan->groups.size()) return XL_E_GRAPH;
    plan->layerwise[group] = (fused || plan->groups[group].layers.size() < 2) ? 0 : 1;
    xl::refresh_fused_path(*plan);
    return XL_OK;
}

// The plan was sized for one device (compute units, LDS): that device must be the current one.
static bool on_plan_device(const xl_plan *plan)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    return plan->device < 0 || dev == plan->device;
}

static xl_status configure_once(xl_plan *plan)
{
    static std::mutex mu;
    static bool done[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        plan->error = "no current HIP device";
        return XL_E_DEVICE;
    }
    if (!on_plan_device(plan)) {
        plan->error = "the plan was made for device " + std::to_string(plan->device) + ", which is not the current device";
        return XL_E_DEVICE;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!done[dev]) {
        hipError_t e = xl::configure_kernels(GFX950_LDS_BYTES);
        if (e != hipSuccess) {
            plan->error = std::string("cannot raise the dynamic LDS limit: ") + hipGetErrorString(e);
            return XL_E_DEVICE;
        }
        done[dev] = true;
    }
    return XL_OK;
}

xl_status xl_prepare(xl_plan *plan, const void *const *weights, int nweights, void *workspace, void *stream)
{
    if (!plan || !weights || !workspace) return XL_E_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) % 256) {
        plan->error = "workspace must be 256-byte aligned";
        return XL_E_ALIGN;
    }
    xl_status st = configure_once(plan);
    if (st != XL_OK) return st;
    const int nl = (int)plan->layers.size();
    plan->scale_ptr.assign(nl, nullptr);
    plan->shift_ptr.assign(nl, nullptr);
    auto slot = [&](int s, const void **p) -> bool {
        *p = nullptr;
        if (s < 0) return true;
        if (s >= nweights || !weights[s]) return false;
        *p = weights[s];
        return true;
    };
    for (int li = 0; li < nl; ++li) {
        const xl_layer &L = plan->layers[li];
        if (L.op != XL_CONV) continue;
        const void *w, *sc, *sh;
        if (!slot(L.w_slot, &w) || !w || !slot(L.scale_slot, &sc) || !slot(L.shift_slot, &sh)) {
            plan->error = "layer " + std::to_string(li) + ": weight slot missing or NULL";
            return XL_E_NULL;
        }
        plan->scale_ptr[li] = static_cast<const float *>(sc);
        plan->shift_ptr[li] = static_cast<const float *>(sh);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    for (const xl::PackedFilter &p : plan->packed) {
        const xl_layer &L = plan->layers[p.layer];
        hipError_t e;
        if (p.mf < 0) {
            e = xl::launch_pack_thin(static_cast<const float *>(weights[L.w_slot]), plan->scale_ptr[p.layer],
                                     plan->shift_ptr[p.layer], reinterpret_cast<float *>(ws + p.offset),
                                     reinterpret_cast<float *>(ws + p.aff_offset), L.cout, L.cin * L.k * L.k, s);
            if (e != hipSuccess) {
                plan->error = std::string("filter re-layout launch failed: ") + hipGetErrorString(e);
                return XL_E_LAUNCH;
            }
            continue;
        }
        if (p.mf == 0) {
            e = xl::launch_pack_depthwise(static_cast<const float *>(weights[L.w_slot]), plan->scale_ptr[p.layer],
                                          plan->shift_ptr[p.layer], reinterpret_cast<xl::f32x4 *>(ws + p.offset),
                                          reinterpret_cast<xl::f32x4 *>(ws + p.aff_offset), L.cout, L.k, s);
            if (e != hipSuccess) {
                plan->error = std::string("filter re-layout launch failed: ") + hipGetErrorString(e);
                return XL_E_LAUNCH;
            }
            continue;
        }
        e = xl::launch_pack_filter(static_cast<const float *>(weights[L.w_slot]), plan->scale_ptr[p.layer],
                                   reinterpret_cast<xl::f32x4 *>(ws + p.offset), L.cout, L.cin, L.k, p.mf,
                                   p.nkg, p.nrt, s, p.pairs ? 1 : 0, p.pr);
        if (e == hipSuccess)
            e = xl::launch_pack_affine(plan->shift_ptr[p.layer], reinterpret_cast<xl::f32x4 *>(ws + p.aff_offset), L.cout,
                                       p.mf, p.nrt, s);
        if (e != hipSuccess) {
            plan->error = std::string("filter re-layout launch failed: ") + hipGetErrorString(e);
            return XL_E_LAUNCH;
        }
    }
    plan->prepared.insert(workspace);
    plan->error.clear();
    return XL_OK;
}

// Enqueue one step.  Shared by xl_run and xl_tune.  Failures are reported through run_fail.
static xl_status launch_step(const xl_plan *plan, const xl::Step &st, const void *const *tensors, char *ws,
                             hipStream_t s)
{
    if (plan->shapes[st.x_id].n == 0) return XL_OK;  // empty batch: nothing to do, pointers may be NULL
    auto base = [&](int t) -> char * {
        const xl::Storage &sg = plan->storage[t];
        if (sg.external) return static_cast<char *>(const_cast<void *>(tensors[sg.root]));
        return ws + sg.offset;
    };
    char *x = base(st.x_id), *y = base(st.y_id);
    char *sc = st.type == xl::STEP_BLOCK && st.sc_id >= 0 ? base(st.sc_id) : x;
    char *b = st.type == xl::STEP_ADD ? base(st.b_id) : x;
    if (!x || !y || !sc || !b) return run_fail(plan, XL_E_NULL, "a graph input or output pointer is NULL");
    // every tensor is read and written with 16-byte accesses
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y) | reinterpret_cast<uintptr_t>(sc) |
         reinterpret_cast<uintptr_t>(b)) % 16)
        return run_fail(plan, XL_E_ALIGN, "tensor pointers must be 16-byte aligned");
    hipError_t e = hipSuccess;
    if (st.type == xl::STEP_BLOCK) {
        xl::BlockParams p = st.bp;
        p.x = reinterpret_cast<const float *>(x);
        p.y = reinterpret_cast<float *>(y);
        p.sc = st.sc_id >= 0 ? reinterpret_cast<const float *>(sc) : nullptr;
        xl::ConvW *cw[4] = {&p.c1, &p.c2[0], &p.c2[1], &p.c1b};
        for (int i = 0; i < 4; ++i) {
            if (st.conv_layer[i] < 0) continue;
            cw[i]->wp = reinterpret_cast<const xl::f32x4 *>(ws + plan->packed[st.packed[i]].offset);
            cw[i]->aff = reinterpret_cast<const xl::f32x4 *>(ws + plan->packed[st.packed[i]].aff_offset);
        }
        e = xl::launch_block(st.variant, p, st.threads, (size_t)st.lds_bytes, s);
    } else if (st.type == xl::STEP_MAXPOOL) {
        const xl::Storage &ys = plan->storage[st.y_id];
        e = xl::launch_maxpool(reinterpret_cast<const float *>(x), reinterpret_cast<float *>(y), st.N, st.C, st.H,
                               st.W, st.Ho, st.Wo, st.k, st.stride, st.pad, ys.ctot, ys.coff, s);
    } else if (st.type == xl::STEP_ADD) {
        if (plan->storage[st.y_id].root != st.y_id)
            return run_fail(plan, XL_E_UNSUPPORTED, "add writing into a concat slice is not supported");
        e = xl::launch_add(reinterpret_cast<const float *>(x), reinterpret_cast<const float *>(b),
                           reinterpret_cast<float *>(y), st.count, st.relu, s);
    } else if (st.type == xl::STEP_DEPTHWISE) {
        const xl::Storage &ys = plan->storage[st.y_id];
        const xl::PackedFilter &pf = plan->packed[st.packed[0]];
        e = xl::launch_depthwise(reinterpret_cast<const float *>(x), reinterpret_cast<float *>(y),
                                 reinterpret_cast<const xl::f32x4 *>(ws + pf.offset),
                                 reinterpret_cast<const xl::f32x4 *>(ws + pf.aff_offset), st.N, st.C, st.H, st.W, st.Ho,
                                 st.Wo, st.k, st.stride, st.pad, st.relu, ys.ctot, ys.coff, s);
    } else if (st.type == xl::STEP_GAP) {
        if (plan->storage[st.y_id].root != st.y_id)
            return run_fail(plan, XL_E_UNSUPPORTED, "global pooling writing into a concat slice is not supported");
        e = xl::launch_gap(reinterpret_cast<const float *>(x), reinterpret_cast<float *>(y), st.N * st.C,
                           st.H * st.W, s);
    }
    if (e != hipSuccess) return run_fail(plan, XL_E_LAUNCH, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return XL_OK;
}

static xl_status check_run_args(const xl_plan *plan, const void *const *tensors, int ntensors, const void *workspace)
{
    if (!plan || !tensors || !workspace) return XL_E_NULL;
    if (!plan->prepared.count(workspace)) return run_fail(plan, XL_E_STATE, "xl_prepare has not been called for this workspace");
    if (ntensors < (int)plan->shapes.size()) return run_fail(plan, XL_E_GRAPH, "the tensors array is shorter than the plan's tensor list");
    if (!on_plan_device(plan)) return run_fail(plan, XL_E_DEVICE, "the plan's device is not the current device");
    return XL_OK;
}

xl_status xl_run(const xl_plan *plan, const void *const *tensors, int ntensors, void *workspace, void *stream,
                 int fused)
{
    xl_status rc = check_run_args(plan, tensors, ntensors, workspace);
    if (rc != XL_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    if (fused) {
        for (const xl::Step *st : plan->fused_active) {
            rc = launch_step(plan, *st, tensors, ws, s);
            if (rc != XL_OK) return rc;
        }
    } else {
        for (const xl::Step &st : plan->unfused_steps) {
            rc = launch_step(plan, st, tensors, ws, s);
            if (rc != XL_OK) return rc;
        }
    }
    return XL_OK;
}

xl_status xl_profile(const xl_plan *plan, const void *const *tensors, int ntensors, void *workspace, void *stream,
                     int fused, int reps, float *launch_us, int cap)
{
    xl_status rc = check_run_args(plan, tensors, ntensors, workspace);
    if (rc != XL_OK) return rc;
    if (!launch_us) return XL_E_NULL;
    const std::vector<const xl::Step *> steps = launches_of(plan, fused);
    const int n = (int)steps.size();
    if (cap < n) return run_fail(plan, XL_E_GRAPH, "launch_us has fewer entries than the mode has launches");
    if (reps < 1) reps = 5;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    rc = xl_run(plan, tensors, ntensors, workspace, stream, fused);     // untimed: code and filters warm
    if (rc != XL_OK) return rc;
    std::vector<hipEvent_t> ev((size_t)reps * (n + 1));
    size_t made = 0;
    for (; made < ev.size(); ++made)
        if (hipEventCreate(&ev[made]) != hipSuccess) break;
    if (made < ev.size()) rc = run_fail(plan, XL_E_DEVICE, "cannot create timing events");
    for (int r = 0; r < reps && rc == XL_OK; ++r) {
        hipEvent_t *e = &ev[(size_t)r * (n + 1)];
        (void)hipEventRecord(e[0], s);
        for (int i = 0; i < n && rc == XL_OK; ++i) {
            rc = launch_step(plan, *steps[i], tensors, ws, s);
            (void)hipEventRecord(e[i + 1], s);
        }
    }
    if (rc == XL_OK && hipStreamSynchronize(s) != hipSuccess) rc = run_fail(plan, XL_E_LAUNCH, "a kernel failed while profiling");
    if (rc == XL_OK) {
        for (int i = 0; i < n; ++i) {
            double sum = 0;
            for (int r = 0; r < reps; ++r) {
                float ms = 0.f;
                (void)hipEventElapsedTime(&ms, ev[(size_t)r * (n + 1) + i], ev[(size_t)r * (n + 1) + i + 1]);
                sum += ms;
            }
            launch_us[i] = (float)(sum / reps * 1e3);
        }
    }
    for (size_t i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
    return rc;
}

xl_status xl_measure_peaks(void *dst, const void *src, size_t bytes, void *stream, double *copy_gbs,
                           double *mfma_f32_tflops, double *mfma_bf16_tflops, double *valu_f32_tflops)
{
    if (!dst || !src) return XL_E_NULL;
    if (bytes < (2u << 20) || (reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) % 16) return XL_E_ALIGN;
    int dev = 0, cus = GFX950_CUS;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return XL_E_DEVICE;
    cus = prop.multiProcessorCount;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return XL_E_DEVICE;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return XL_E_DEVICE;
    }
    double *out[4] = {copy_gbs, mfma_f32_tflops, mfma_bf16_tflops, valu_f32_tflops};
    xl_status rc = XL_OK;
    for (int what = 0; what < 4 && rc == XL_OK; ++what) {
        if (!out[what]) continue;
        double work = 0, best = 0;
        for (int r = 0; r < 6 && rc == XL_OK; ++r) {        // first launch untimed, then the fastest of 5
            if (r > 0) (void)hipEventRecord(e0, s);
            if (xl::launch_peak_probe(what, dst, src, bytes, cus, s, &work) != hipSuccess) rc = XL_E_LAUNCH;
            if (r > 0) (void)hipEventRecord(e1, s);
            if (hipStreamSynchronize(s) != hipSuccess) rc = XL_E_LAUNCH;
            if (r > 0 && rc == XL_OK) {
                float ms = 0.f;
                (void)hipEventElapsedTime(&ms, e0, e1);
                if (ms > 0.f) best = std::max(best, work / (ms * 1e-3));
            }
        }
        *out[what] = what == 0 ? best / 1e9 : best / 1e12;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}

// A block leaves the fused path for its layers' own kernels only when those measured this much faster.
static constexpr float LAYERWISE_MARGIN = 0.97f;

// Make candidate `idx` the configuration of step `st`; in the fused path the block's reported tiles follow.
static void adopt(xl_plan *plan, xl::Step &st, int idx, bool fused)
{
    std::vector<xl::Step> alts;
    std::vector<xl_group_info> infos;
    alts.swap(st.alts);
    infos.swap(st.alt_info);
    const int group = st.group, first_layer = st.first_layer, nlayers = st.nlayers;
    st = alts[idx];
    st.group = group;
    st.first_layer = first_layer;
    st.nlayers = nlayers;
    st.adopted = idx;
    st.alts.swap(alts);
    st.alt_info.swap(infos);
    if (fused && group >= 0 && group < (int)plan->groups.size()) {
        xl_group_info &gi = plan->groups[group].info;
        const xl_group_info &src = st.alt_info[idx];
        gi.tile_h = src.tile_h; gi.tile_w = src.tile_w;
        gi.mid_h = src.mid_h; gi.mid_w = src.mid_w;
        gi.in_h = src.in_h; gi.in_w = src.in_w;
        gi.tiles_y = src.tiles_y; gi.tiles_x = src.tiles_x;
        gi.cout_split = src.cout_split; gi.workgroups = src.workgroups;
        gi.threads = src.threads; gi.lds_bytes = src.lds_bytes;
        gi.workgroups_per_cu = src.workgroups_per_cu; gi.chunk_channels = src.chunk_channels;
        gi.flops_executed = src.flops_executed; gi.redundancy = src.redundancy;
        gi.precision = src.precision;
    }
}

static const xl::Step *find_launch(const xl_plan *plan, int fused, int launch)
{
    if (!plan) return nullptr;
    if (fused) return launch >= 0 && launch < (int)plan->fused_active.size() ? plan->fused_active[launch] : nullptr;
    return launch >= 0 && launch < (int)plan->unfused_steps.size() ? &plan->unfused_steps[launch] : nullptr;
}

int xl_plan_num_candidates(const xl_plan *plan, int fused, int launch)
{
    const xl::Step *st = find_launch(plan, fused, launch);
    if (!st) return 0;
    return st->alts.empty() ? 1 : (int)st->alts.size();
}

xl_status xl_plan_candidate_info(const xl_plan *plan, int fused, int launch, int candidate, xl_launch_info *out)
{
    if (!plan || !out) return XL_E_NULL;
    const xl::Step *st = find_launch(plan, fused, launch);
    if (!st) return XL_E_GRAPH;
    const int n = st->alts.empty() ? 1 : (int)st->alts.size();
    if (candidate < -1 || candidate >= n) return XL_E_GRAPH;
    if (candidate < 0) candidate = st->adopted;
    const xl::Step &c = st->alts.empty() ? *st : st->alts[candidate];
    memset(out, 0, sizeof *out);
    out->group = fused ? group_of_layer(plan, st->first_layer) : -1;
    out->first_layer = st->first_layer;
    out->nlayers = st->nlayers;
    out->candidate = candidate;
    out->is_block_kernel = c.type == xl::STEP_BLOCK ? 1 : 0;
    if (c.type == xl::STEP_BLOCK) {
        const xl::BlockParams &p = c.bp;
        const bool pooled = p.pth > 0;
        out->variant = c.variant;
        out->tile_h = pooled ? p.pth : p.th;
        out->tile_w = pooled ? p.ptw : p.tw;
        out->threads = c.threads;
        out->cout_split = p.csplit;
        out->waves_cout_1 = p.waves_r1;
        out->waves_cout_2 = p.waves_r2;
        out->lds_bytes = c.lds_bytes;
        out->workgroups = p.nblocks;
        out->model_cost_us = c.cost_us;
        if (!st->alt_info.empty()) {
            out->chunk_channels = st->alt_info[candidate].chunk_channels;
            out->precision = st->alt_info[candidate].precision;
        }
    }
    return XL_OK;
}

xl_status xl_plan_select_candidate(xl_plan *plan, int fused, int launch, int candidate)
{
    if (!plan) return XL_E_NULL;
    xl::Step *stp = const_cast<xl::Step *>(find_launch(plan, fused, launch));
    if (!stp) return XL_E_GRAPH;
    xl::Step &st = *stp;
    const int n = st.alts.empty() ? 1 : (int)st.alts.size();
    if (candidate < 0 || candidate >= n) return XL_E_GRAPH;
    if (!st.alts.empty()) adopt(plan, st, candidate, fused != 0);
    return XL_OK;
}

xl_status xl_tune(xl_plan *plan, const void *const *tensors, int ntensors, void *workspace, void *stream, int reps)
{
    xl_status rc = check_run_args(plan, tensors, ntensors, workspace);
    if (rc != XL_OK) {
        if (plan) plan->error = g_run_error;
        return rc;
    }
    if (reps < 5) reps = 5;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) {
        plan->error = "cannot create timing events";
        return XL_E_DEVICE;
    }
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        plan->error = "cannot create timing events";
        return XL_E_DEVICE;
    }
    for (int pass = 0; pass < 2 && rc == XL_OK; ++pass) {
        std::vector<xl::Step> &steps = pass == 0 ? plan->fused_steps : plan->unfused_steps;
        for (xl::Step &st : steps) {
            if (st.type != xl::STEP_BLOCK || st.alts.size() < 2) {
                // nothing to choose, but the step is timed (the fused-or-not decision below needs it) and later
                // blocks time on the data it produces
                std::vector<float> t1;
                for (int r = 0; r < reps && rc == XL_OK; ++r) {
                    (void)hipEventRecord(e0, s);
                    rc = launch_step(plan, st, tensors, ws, s);
                    (void)hipEventRecord(e1, s);
                    if (hipEventSynchronize(e1) != hipSuccess) {
                        if (rc == XL_OK) rc = run_fail(plan, XL_E_LAUNCH, "a kernel failed while tuning");
                        break;
                    }
                    float ms = 0.f;
                    (void)hipEventElapsedTime(&ms, e0, e1);
                    t1.push_back(ms);
                }
                if (rc != XL_OK) break;
                std::sort(t1.begin(), t1.end());
                st.tuned_us = t1[t1.size() / 2] * 1e3f;
                continue;
            }
            // n timed launches of one candidate, sorted
            auto time_alt = [&](size_t a, int n, std::vector<float> &t) {
                t.clear();
                for (int r = 0; r < n && rc == XL_OK; ++r) {
                    (void)hipEventRecord(e0, s);
                    rc = launch_step(plan, st.alts[a], tensors, ws, s);
                    (void)hipEventRecord(e1, s);
                    if (hipEventSynchronize(e1) != hipSuccess) {
                        if (rc == XL_OK) rc = run_fail(plan, XL_E_LAUNCH, "a candidate kernel failed while tuning");
                        break;
                    }
                    float ms = 0.f;
                    (void)hipEventElapsedTime(&ms, e0, e1);
                    t.push_back(ms);
                }
                std::sort(t.begin(), t.end());
            };
            // a quick look at every candidate (fastest of 3 after a warm-up launch) ...
            std::vector<std::pair<float, int>> quick;
            std::vector<float> t;
            for (size_t a = 0; a < st.alts.size() && rc == XL_OK; ++a) {
                rc = launch_step(plan, st.alts[a], tensors, ws, s);         // warm-up (code, filters in L2)
                if (rc != XL_OK) break;
                time_alt(a, 3, t);
                if (rc == XL_OK) quick.push_back({t.front(), (int)a});
            }
            // ... then the six fastest again, ranked by the median of `reps` launches (ties: lower index)
            int best = 0;
            float best_ms = 1e30f;
            if (rc == XL_OK) {
                std::sort(quick.begin(), quick.end());
                for (size_t i = 0; i < quick.size() && i < 6 && rc == XL_OK; ++i) {
                    time_alt((size_t)quick[i].second, reps, t);
                    if (rc != XL_OK) break;
                    const float med = t[t.size() / 2];
                    if (med < best_ms || (med == best_ms && quick[i].second < best)) {
                        best_ms = med;
                        best = quick[i].second;
                    }
                }
            }
            if (rc != XL_OK) break;
            adopt(plan, st, best, pass == 0);
            st.tuned_us = best_ms * 1e3f;
        }
    }
    // A block whose layers, one kernel each and back to back, were measured faster than its fused kernel runs
    // layer by layer in the fused path (small images at a batch that cannot fill the chip with whole tiles, a
    // batch of 1): the tuner only ever trades speed, and the fused path is then not the slower one.  The margin
    // covers what timings on warm buffers cannot see (intermediates that stay in cache here reach HBM in a long
    // pipeline).
    if (rc == XL_OK && !plan->opts.keep_blocks_fused) {
        for (const xl::Step &st : plan->fused_steps) {
            if (st.nlayers < 2 || st.group < 0 || st.tuned_us <= 0.f) continue;
            const std::vector<int> &ls = plan->groups[st.group].layers;
            std::vector<const xl::Step *> seq;
            for (const xl::Step &u : plan->unfused_steps)
                if (std::find(ls.begin(), ls.end(), u.first_layer) != ls.end()) seq.push_back(&u);
            // the layers as they would run: back to back, one pair of events around the sequence
            std::vector<float> t;
            for (int r = 0; r < reps + 1 && rc == XL_OK; ++r) {
                (void)hipEventRecord(e0, s);
                for (const xl::Step *u : seq) {
                    rc = launch_step(plan, *u, tensors, ws, s);
                    if (rc != XL_OK) break;
                }
                (void)hipEventRecord(e1, s);
                if (hipEventSynchronize(e1) != hipSuccess) {
                    if (rc == XL_OK) rc = run_fail(plan, XL_E_LAUNCH, "a kernel failed while tuning");
                    break;
                }
                float ms = 0.f;
                (void)hipEventElapsedTime(&ms, e0, e1);
                if (r > 0) t.push_back(ms);         // (the first run warms code and caches)
            }
            if (rc != XL_OK) break;
            std::sort(t.begin(), t.end());
            const float seq_us = t[t.size() / 2] * 1e3f;
            plan->layerwise[st.group] = !seq.empty() && seq_us < LAYERWISE_MARGIN * st.tuned_us;
        }
        xl::refresh_fused_path(*plan);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != XL_OK) plan->error = g_run_error;
    return rc;
}

}  // extern "C"
