// Execution plan: one kernel launch per fusion group (plus layout changes the
// planner inserts), buffers for intermediates carved from one workspace.
#pragma once
#include <map>
#include <string>
#include <vector>

#include "graph.h"
#include "kernels.h"

namespace rl {

enum StepKind { S_IGEMM = 0, S_ELTWISE, S_GATES, S_MAXPOOL, S_GAVG, S_TO_NHWC, S_TO_NCHW, S_STEM_PAD, S_STEM_POOL, S_PERMUTE, S_PACK, S_WGRAD, S_WGRAD_REDUCE, S_DILATE };
enum Slot { SL_X = 0, SL_X2, SL_W, SL_Y, SL_E0, SL_E1, SL_E2, SL_E3, SL_E4, SL_E5, SL_CIN, SL_COUT, SL_HOUT, SL_PART, SL_COUNT };

struct BufDesc {
    int bound_value = -1;     // >= 0: caller-bound pointer of that value id; -1: workspace
    size_t bytes = 0;
    size_t offset = 0;        // workspace offset
    int first = -1, last = -1;
};

struct Step {
    int kind = 0;
    int group = -1;
    std::string name, kernel;
    IgemmParams ig{};
    IgemmLaunch il{};
    EltwiseParams el{};
    GatesParams ga{};
    PoolParams po{};
    PermuteParams pe{};
    WgradParams wg{};                   // S_WGRAD (and the counts S_WGRAD_REDUCE adds up)
    GatherPack gp{};                    // S_PACK: an activation gathered into the K-contiguous rows a contraction reads
    int t_dtype = 0, t_N = 0, t_C = 0, t_P = 0;
    int st_H = 0, st_W = 0, st_Hp = 0, st_Wp = 0, st_ph = 0, st_pw = 0;   // S_STEM_PAD geometry (t_N, t_C: batch, channels)
    int stem = 0;                       // S_IGEMM: the few-channel stem form (padded 4-channel frame, regrouped taps)
    int sp_N = 0, sp_PH = 0, sp_PW = 0; // S_STEM_POOL: images and pooled size (ig: the stem contraction)
    int stem_kh = 0;                    // stem contractions: the filter's own height (ig.KH counts pairs of frame rows)
    int stem_direct = 0, stem_kw = 0;   // S_STEM_POOL reading the channel-first input itself (st_* and t_C: its geometry; stem_kw: filter width)
    int pair = 0;                       // S_IGEMM: 1: launched together with the next step (an independent contraction of the
                                        // same tile shape); 2: that next step, which launches nothing itself
    int chain = 0;                      // S_IGEMM: 1: a split dense contraction whose adding launch also runs the next step (a
                                        // small dense layer on its result); 2: that next step, which launches nothing itself
    int slot[SL_COUNT];
    double flops = 0, bytes = 0;
    Step() { for (int &s : slot) s = -1; }
};

struct PackSpec {
    int dtype = 0, O = 0, C = 0, T = 0, Kp = 0, perm_block = 0;   // perm_block -1: matrix, then the 64x64x3x3 fragment-order copy
    int stem = 0, KH = 0, KW = 0;      // stem = 1: few-channel stem layout (launch_pack_weight_stem); 2: launch_pack_weight_stem_direct
    int pw = 0;                         // stem = 2: the convolution's left padding (its parity shifts the filter inside the 8-pixel window)
    int gather = 0; GatherPack gp{};   // gather = 1: launch_pack_gather (operands of the gradient operators)
    size_t bytes = 0;
};

struct Plan {
    std::shared_ptr<ErrBox> err;
    std::vector<Value> values;
    std::vector<int> outputs;
    std::vector<BufDesc> bufs;
    std::vector<Step> steps;
    std::vector<int> bound_buf;          // value id -> buffer index of its bound pointer, or -1
    std::map<int, PackSpec> packs;       // param value id -> packing
    size_t workspace_bytes = 0;
    rl_plan_opts opts{};                 // the caller's plan-time switches, fixed at creation
};

rl_status build_plan(const Graph &g, Plan &plan, std::string &msg);
std::string describe_plan(const Plan &p);

// ptrs[buffer index] must be resolved; launches every step.
// events (optional): steps+1 events, events[i] recorded before step i, events[steps] after the last
rl_status run_steps(const Plan &p, void *const *ptrs, hipStream_t s, std::string &msg, hipEvent_t *events = nullptr);

}  // namespace rl
