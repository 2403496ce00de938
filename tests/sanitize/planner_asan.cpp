// Host-only build of the planner and the C ABI for AddressSanitizer / UBSan runs (no GPU, no HIP
// runtime): the device-side launchers and the few HIP runtime calls the C ABI makes are replaced by
// stubs, so that everything the planner does with a graph -- validation, storage map, tile search,
// launch descriptors, candidate lists, error paths -- runs under the sanitizers.
//
// Input (stdin): one or more workloads written by tests/test_sanitizers.py:
//   workload <name> <expected status> <nlayers> <ntensors> <ngroups> <8 option ints>
//   shape n c h w                       (ntensors lines)
//   layer op in0 in1 out cin cout k stride pad groups relu w_slot scale_slot shift_slot   (nlayers lines)
//   group mode n id...                  (ngroups lines)
// Output: one line per workload; exit status 0 when every plan came out with the expected status.
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "plan.h"

// ---- stubs for what lives in the HIP translation units ------------------------------------------
namespace xl {
hipError_t launch_block(int, const BlockParams &, int, size_t, hipStream_t) { return hipSuccess; }
hipError_t configure_kernels(int) { return hipSuccess; }
hipError_t launch_pack_filter(const float *, const float *, f32x4 *, int, int, int, int, int, int, hipStream_t, int, int) { return hipSuccess; }
hipError_t launch_peak_probe(int, void *, const void *, size_t, int, hipStream_t, double *w) { *w = 0; return hipSuccess; }
hipError_t launch_pack_thin(const float *, const float *, const float *, float *, float *, int, int, hipStream_t) { return hipSuccess; }
hipError_t launch_pack_affine(const float *, f32x4 *, int, int, int, hipStream_t) { return hipSuccess; }
hipError_t launch_maxpool(const float *, float *, int, int, int, int, int, int, int, int, int, int, int, hipStream_t) { return hipSuccess; }
hipError_t launch_add(const float *, const float *, float *, long long, int, hipStream_t) { return hipSuccess; }
hipError_t launch_gap(const float *, float *, int, int, hipStream_t) { return hipSuccess; }
hipError_t launch_pack_depthwise(const float *, const float *, const float *, f32x4 *, f32x4 *, int, int, hipStream_t) { return hipSuccess; }
hipError_t launch_depthwise(const float *, float *, const f32x4 *, const f32x4 *, int, int, int, int, int, int, int, int, int, int, int, int, hipStream_t) { return hipSuccess; }
}  // namespace xl

// ---- stubs for the HIP runtime calls of api.cpp (never reached with device < 0, except hipGetDevice) ----
extern "C" {
hipError_t hipGetDevicePropertiesR0600(hipDeviceProp_tR0600 *, int) { return hipErrorNoDevice; }
hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
const char *hipGetErrorString(hipError_t) { return "stub"; }
hipError_t hipEventCreate(hipEvent_t *) { return hipErrorNoDevice; }
hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.f; return hipSuccess; }
}

int main()
{
    char word[256], name[256];
    int failures = 0, count = 0;
    while (scanf("%255s", word) == 1) {
        if (strcmp(word, "workload") != 0) { fprintf(stderr, "expected 'workload', got '%s'\n", word); return 2; }
        int expect, nl, nt, ng, o[9];
        if (scanf("%255s %d %d %d %d %d %d %d %d %d %d %d %d %d", name, &expect, &nl, &nt, &ng, &o[0], &o[1], &o[2], &o[3], &o[4],
                  &o[5], &o[6], &o[7], &o[8]) != 14) return 2;
        std::vector<xl_shape> shapes(nt);
        std::vector<xl_layer> layers(nl);
        std::vector<std::vector<int>> ids(ng);
        std::vector<xl_group> groups(ng);
        for (int i = 0; i < nt; ++i)
            if (scanf("%255s %d %d %d %d", word, &shapes[i].n, &shapes[i].c, &shapes[i].h, &shapes[i].w) != 5) return 2;
        for (int i = 0; i < nl; ++i) {
            xl_layer &L = layers[i];
            if (scanf("%255s %d %d %d %d %d %d %d %d %d %d %d %d %d %d", word, &L.op, &L.in[0], &L.in[1], &L.out, &L.cin, &L.cout, &L.k,
                      &L.stride, &L.pad, &L.groups, &L.relu, &L.w_slot, &L.scale_slot, &L.shift_slot) != 15) return 2;
        }
        for (int g = 0; g < ng; ++g) {
            int n;
            if (scanf("%255s %d %d", word, &groups[g].mode, &n) != 3) return 2;
            ids[g].resize(n);
            for (int i = 0; i < n; ++i)
                if (scanf("%d", &ids[g][i]) != 1) return 2;
            groups[g].nlayers = n;
            groups[g].layer_ids = ids[g].data();
        }
        xl_options opts;
        memset(&opts, 0, sizeof opts);
        opts.lds_budget_bytes = o[0]; opts.num_cus = o[1]; opts.force_tile_h = o[2]; opts.force_tile_w = o[3];
        opts.force_cout_split = o[4]; opts.paper_tuner_only = o[5]; opts.force_threads = o[6]; opts.precision = o[7];
        opts.keep_blocks_fused = o[8];
        xl_plan *plan = nullptr;
        const xl_status st = xl_plan_create(layers.data(), nl, shapes.data(), nt, groups.data(), ng, -1, &opts, &plan);
        ++count;
        long long cands = 0;
        if (st == XL_OK) {
            // read everything a caller can read, and walk the candidate lists the way a tuner would
            for (int g = 0; g < xl_plan_num_groups(plan); ++g) {
                xl_group_info gi;
                if (xl_plan_query(plan, g, &gi) != XL_OK) ++failures;
            }
            (void)xl_plan_workspace_bytes(plan);
            for (int fused = 0; fused < 2; ++fused)
                for (int l = 0; l < xl_plan_num_launches(plan, fused); ++l) {
                    const int n = xl_plan_num_candidates(plan, fused, l);
                    for (int c = 0; c < n; ++c) {
                        xl_launch_info li;
                        if (xl_plan_candidate_info(plan, fused, l, c, &li) != XL_OK) ++failures;
                        ++cands;
                    }
                    if (xl_plan_select_candidate(plan, fused, l, n - 1) != XL_OK) ++failures;
                    if (xl_plan_select_candidate(plan, fused, l, 0) != XL_OK) ++failures;
                    if (xl_plan_select_candidate(plan, fused, l, n) != XL_E_GRAPH) ++failures;
                }
            // the run path up to the (stubbed) launches: a fake 256-byte aligned workspace and tensor pointers
            std::vector<const void *> weights(3 * nl, reinterpret_cast<const void *>(0x1000));
            std::vector<const void *> tensors(nt, reinterpret_cast<const void *>(0x2000));
            void *ws = reinterpret_cast<void *>(0x100000);
            if (xl_run(plan, tensors.data(), nt, ws, nullptr, 1) != XL_E_STATE) ++failures;
            if (xl_prepare(plan, weights.data(), 3 * nl, ws, nullptr) != XL_OK) ++failures;
            if (xl_run(plan, tensors.data(), nt, ws, nullptr, 1) != XL_OK) ++failures;
            if (xl_run(plan, tensors.data(), nt, ws, nullptr, 0) != XL_OK) ++failures;
            // every block layer by layer and back: the launch list follows, candidates stay addressable
            const int fused_launches = xl_plan_num_launches(plan, 1);
            for (int g = 0; g < xl_plan_num_groups(plan); ++g)
                if (xl_plan_set_block_fused(plan, g, 0) != XL_OK || xl_plan_block_is_fused(plan, g)) ++failures;
            if (xl_plan_num_launches(plan, 1) != xl_plan_num_launches(plan, 0)) ++failures;
            for (int l = 0; l < xl_plan_num_launches(plan, 1); ++l) {
                xl_launch_info li;
                if (xl_plan_candidate_info(plan, 1, l, -1, &li) != XL_OK || li.nlayers != 1) ++failures;
            }
            if (xl_run(plan, tensors.data(), nt, ws, nullptr, 1) != XL_OK) ++failures;
            for (int g = 0; g < xl_plan_num_groups(plan); ++g)
                if (xl_plan_set_block_fused(plan, g, 1) != XL_OK) ++failures;
            if (xl_plan_num_launches(plan, 1) != fused_launches) ++failures;
            if (xl_plan_set_block_fused(plan, xl_plan_num_groups(plan), 0) != XL_E_GRAPH) ++failures;
            tensors.assign(nt, reinterpret_cast<const void *>(0x2004));
            if (shapes[0].n > 0 && xl_run(plan, tensors.data(), nt, ws, nullptr, 1) != XL_E_ALIGN) ++failures;
        } else {
            (void)xl_plan_last_error(nullptr);
        }
        printf("%s status %d (%s) candidates %lld\n", name, st, xl_strerror(st), cands);
        if (st != expect) {
            fprintf(stderr, "%s: status %d, expected %d: %s\n", name, st, expect, xl_plan_last_error(nullptr));
            ++failures;
        }
        xl_plan_destroy(plan);
    }
    printf("%d workloads, %d failures\n", count, failures);
    return failures ? 1 : 0;
}
