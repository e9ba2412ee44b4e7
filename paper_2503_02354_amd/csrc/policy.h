// Expert-cache policy: which experts live on the device, what to load first, whom to evict.
// Paper: Section 4.1 "System initialization" (fill by descending usage probability) and Section 4.3
// "Dependency-aware Expert Management" (two-stage eviction).  Pure host code, no HIP.
#pragma once
#include <cstdint>
#include <vector>

namespace coe {

struct Switch {
    int32_t expert;                // expert loaded
    std::vector<int32_t> victims;  // experts evicted to make room, in eviction order
};

class Policy {
public:
    Policy(int32_t n_experts, const int64_t* nbytes, const float* prob, const int32_t* succ_off, const int32_t* succ,
           int32_t cap_experts, int64_t cap_bytes);

    // Initial fill: descending usage probability (ties: lower id), stopping at the first expert that does not fit.
    std::vector<int32_t> init_fill();

    // Plan one stage.  has_group[e] != 0: some pending request needs e.  Returns false if an expert cannot fit; the cache
    // state is then what it was before the call.
    // order: resident experts first, then missing ones, each by ascending id.  switches: one per missing expert.
    bool plan_stage(const uint8_t* has_group, std::vector<int32_t>& order, std::vector<Switch>& switches);

    bool resident(int32_t e) const { return resident_[e] != 0; }
    int32_t n_experts() const { return n_; }

    // Replacement rule: 0 = the two-stage rule of Section 4.3 (default); 1 = least recently used, 2 = first in first
    // out: the rules of the systems the paper compares with (Section 5.1), kept for measuring what the two-stage rule
    // buys.  Under all three an expert whose group has not run yet in the stage is never evicted.
    bool set_eviction(int32_t kind);

    // Loads are issued ahead of the groups that need them, so that the copy runs while earlier groups compute (paper
    // Section 4.2: an expert can be loaded during the processing of a preceding request).  The experts of the `depth`
    // groups that precede a missing one in the plan then still have kernels queued or running when its copy starts:
    // they count as in use and are not evicted for it.  0 (default): only groups that have not run yet are protected.
    bool set_in_use_depth(int32_t depth);

private:
    bool fits(int32_t e) const;
    void evict(int32_t v);

    int32_t n_;
    std::vector<int64_t> bytes_;
    std::vector<float> prob_;
    std::vector<std::vector<int32_t>> preds_;  // predecessors of each expert in the dependency graph
    int32_t cap_experts_;
    int64_t cap_bytes_;
    std::vector<uint8_t> resident_;
    int32_t n_res_ = 0;
    int64_t res_bytes_ = 0;
    int32_t eviction_ = 0;
    int32_t in_use_depth_ = 0;
    int64_t clock_ = 0;                        // counts loads and group executions, in plan order
    std::vector<int64_t> loaded_at_, used_at_;
};

// Dependency-graph check: ids in range (or -1), acyclic, n_route <= n_classes.  Returns 0 or COE_EGRAPH / COE_EINVAL.
int validate_graph(int32_t n_experts, const int32_t* succ_off, const int32_t* succ, const int32_t* n_classes);

}  // namespace coe
