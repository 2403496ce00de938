// Host-side plan: validated graph, storage map, and one launch descriptor per
// kernel for both execution modes.  Not part of the C ABI.
#pragma once

#include <set>
#include <string>
#include <vector>

#include "xl_internal.h"

namespace xl {

enum StepType { STEP_BLOCK = 0, STEP_MAXPOOL = 1, STEP_ADD = 2, STEP_GAP = 3, STEP_DEPTHWISE = 4 };

// A filter re-laid out for one matrix-core tile size.
struct PackedFilter {
    int layer;
    int mf;             // 32 or 16; 0 = depthwise tables ([channel group][tap], [channel group][scale, shift]);
                        // -1 = thin first layer ([Cout rounded up to 16][Cin*K*K] floats, as many shifts)
    int pr = 0;         // 1: split-bf16 form ([K step][tap][row tile][hi, lo][lane] of 8 bf16)
    bool pairs = false; // channels packed two per channel slot (c -> lane half c % 2, slot c / 2), one K step
    int nkg, nrt;
    size_t offset;      // bytes into the workspace
    size_t bytes;
    size_t aff_offset;  // scale / shift table in accumulator order
    size_t aff_bytes;
};

// Where a tensor lives: itself, or a channel slice of a concatenated tensor.
struct Storage {
    int root;           // tensor id that owns memory
    int coff;           // channel offset inside root
    int ctot;           // channels of root
    bool external;      // root pointer comes from the caller's tensors[] array
    size_t offset;      // bytes into the workspace when !external
};

struct Step {
    int type;
    // STEP_BLOCK
    int variant;
    BlockParams bp;     // pointers filled at run time
    int threads;
    int lds_bytes;
    int conv_layer[4];  // layer index of c1, c2[0], c2[1], c1b (-1 unused)
    int packed[4];      // index into Plan::packed
    // tensors
    int x_id, y_id, sc_id;
    // element-wise steps
    int N, C, H, W, Ho, Wo, k, stride, pad, relu;
    int b_id;
    long long count;
    // tuning: the planner's ranked candidates for this block (alts[0] is the model's choice) with
    // the tile facts each would report, and the fusion block whose info the selection updates
    int group = -1;
    int adopted = 0;        // index into alts of the configuration this step currently is
    double cost_us = 0;     // the cost model's estimate
    int first_layer = -1, nlayers = 1;
    float tuned_us = 0.f;   // median duration xl_tune measured for the adopted configuration (0: never timed)
    std::vector<Step> alts;
    std::vector<xl_group_info> alt_info;
};

struct GroupPlan {
    xl_group_info info;
    std::vector<int> layers;
};

}  // namespace xl

struct xl_plan;
namespace xl {
void refresh_fused_path(xl_plan &pl);
}

struct xl_plan {
    std::vector<xl_layer> layers;
    std::vector<xl_shape> shapes;
    std::vector<xl::GroupPlan> groups;
    std::vector<xl::Storage> storage;
    std::vector<xl::PackedFilter> packed;
    std::vector<xl::Step> fused_steps, unfused_steps;
    // What xl_run(fused = 1) launches: the step of every block, or -- for a block switched to layer-by-layer
    // execution (layerwise[block] != 0) -- the unfused steps of its layers.  Pointers into the two lists above,
    // rebuilt by xl::refresh_fused_path.
    std::vector<char> layerwise;
    std::vector<xl::Step *> fused_active;
    size_t workspace_bytes = 0;
    int device = -1;
    int lds_budget = 160 * 1024;
    int lds_per_cu = 160 * 1024;
    int num_cus = 256;
    xl_options opts{};
    unsigned long long serial = 0;                     // unique per created plan (never reused), from 1
    // bound by xl_prepare
    std::set<const void *> prepared;                   // workspaces that hold this plan's re-laid-out filters
    std::vector<const float *> scale_ptr, shift_ptr;   // per layer
    std::string error;
};
