// Expert-cache policy and dependency-graph validation (host only).
#include "policy.h"

#include <algorithm>
#include <numeric>

#include "../../include/coe.h"

namespace coe {

Policy::Policy(int32_t n_experts, const int64_t* nbytes, const float* prob, const int32_t* succ_off,
               const int32_t* succ, int32_t cap_experts, int64_t cap_bytes)
    : n_(n_experts), bytes_(nbytes, nbytes + n_experts), prob_(prob, prob + n_experts), preds_(n_experts),
      cap_experts_(cap_experts), cap_bytes_(cap_bytes), resident_(n_experts, 0), loaded_at_(n_experts, 0),
      used_at_(n_experts, 0)
{
    for (int32_t p = 0; p < n_; ++p)
        for (int32_t j = succ_off[p]; j < succ_off[p + 1]; ++j) {
            int32_t s = succ[j];
            if (s >= 0 && s < n_ && std::find(preds_[s].begin(), preds_[s].end(), p) == preds_[s].end())
                preds_[s].push_back(p);
        }
}

bool Policy::fits(int32_t e) const
{
    if (cap_experts_ > 0 && n_res_ >= cap_experts_) return false;
    if (cap_bytes_ > 0 && res_bytes_ + bytes_[e] > cap_bytes_) return false;
    return true;
}

void Policy::evict(int32_t v)
{
    resident_[v] = 0;
    --n_res_;
    res_bytes_ -= bytes_[v];
}

bool Policy::set_eviction(int32_t kind)
{
    if (kind < 0 || kind > 2) return false;
    eviction_ = kind;
    return true;
}

bool Policy::set_in_use_depth(int32_t depth)
{
    if (depth < 0) return false;
    in_use_depth_ = depth;
    return true;
}

std::vector<int32_t> Policy::init_fill()
{
    std::vector<int32_t> ids(n_);
    std::iota(ids.begin(), ids.end(), 0);
    std::stable_sort(ids.begin(), ids.end(), [&](int32_t a, int32_t b) { return prob_[a] > prob_[b]; });
    std::vector<int32_t> loaded;
    for (int32_t e : ids) {
        if (resident_[e]) continue;
        if (!fits(e)) break;
        resident_[e] = 1;
        ++n_res_;
        res_bytes_ += bytes_[e];
        loaded_at_[e] = used_at_[e] = ++clock_;
        loaded.push_back(e);
    }
    return loaded;
}

bool Policy::plan_stage(const uint8_t* has_group, std::vector<int32_t>& order, std::vector<Switch>& switches)
{
    order.clear();
    switches.clear();
    for (int32_t e = 0; e < n_; ++e)
        if (has_group[e] && resident_[e]) order.push_back(e);
    for (int32_t e = 0; e < n_; ++e)
        if (has_group[e] && !resident_[e]) order.push_back(e);

    std::vector<uint8_t> waiting(n_, 0);  // group not yet executed in this stage
    for (int32_t e : order) waiting[e] = 1;

    // a stage that cannot be planned leaves the cache as it was: the caller's device state stays the policy's state
    const std::vector<uint8_t> resident0 = resident_;
    const std::vector<int64_t> loaded0 = loaded_at_, used0 = used_at_;
    const int32_t n_res0 = n_res_;
    const int64_t res_bytes0 = res_bytes_, clock0 = clock_;
    auto give_up = [&]() {
        resident_ = resident0; loaded_at_ = loaded0; used_at_ = used0;
        n_res_ = n_res0; res_bytes_ = res_bytes0; clock_ = clock0;
        order.clear();
        switches.clear();
        return false;
    };

    for (size_t pos = 0; pos < order.size(); ++pos) {
        const int32_t e = order[pos];
        if (!resident_[e]) {
            Switch sw;
            sw.expert = e;
            // the groups right before this one are still running when the copy starts: their experts stay
            for (size_t q = pos > (size_t)in_use_depth_ ? pos - in_use_depth_ : 0; q < pos; ++q) waiting[order[q]] = 2;
            if (!fits(e) && eviction_ != 0) {
                // comparison rules: oldest use (LRU) or oldest load (FIFO) among everything that is not waiting to run
                const std::vector<int64_t>& key = eviction_ == 1 ? used_at_ : loaded_at_;
                while (!fits(e)) {
                    int32_t v = -1;
                    for (int32_t x = 0; x < n_; ++x)
                        if (resident_[x] && !waiting[x] && (v < 0 || key[x] < key[v])) v = x;
                    if (v < 0) break;
                    evict(v);
                    sw.victims.push_back(v);
                }
            }
            if (!fits(e)) {
                // Stage 1: dependent experts none of whose predecessors is resident or requested in this stage
                // (they cannot be reached soon), largest footprint first.
                std::vector<int32_t> cand;
                for (int32_t x = 0; x < n_; ++x) {
                    if (!resident_[x] || has_group[x] || preds_[x].empty()) continue;
                    bool around = false;
                    for (int32_t p : preds_[x]) around = around || resident_[p] || has_group[p];
                    if (!around) cand.push_back(x);
                }
                std::stable_sort(cand.begin(), cand.end(), [&](int32_t a, int32_t b) { return bytes_[a] > bytes_[b]; });
                for (int32_t v : cand) {
                    if (fits(e)) break;
                    // evicting an expert never makes another one's predecessor appear, so the candidate set only
                    // needs a re-check that v is still resident
                    evict(v);
                    sw.victims.push_back(v);
                }
            }
            if (!fits(e)) {
                // Stage 2: ascending usage probability among everything that is not waiting to run.
                std::vector<int32_t> cand;
                for (int32_t x = 0; x < n_; ++x)
                    if (resident_[x] && !waiting[x]) cand.push_back(x);
                std::stable_sort(cand.begin(), cand.end(), [&](int32_t a, int32_t b) { return prob_[a] < prob_[b]; });
                for (int32_t v : cand) {
                    if (fits(e)) break;
                    evict(v);
                    sw.victims.push_back(v);
                }
            }
            if (!fits(e)) return give_up();
            resident_[e] = 1;
            ++n_res_;
            res_bytes_ += bytes_[e];
            loaded_at_[e] = ++clock_;
            switches.push_back(std::move(sw));
            for (size_t q = pos > (size_t)in_use_depth_ ? pos - in_use_depth_ : 0; q < pos; ++q) waiting[order[q]] = 0;
        }
        used_at_[e] = ++clock_;
        waiting[e] = 0;
    }
    return true;
}

int validate_graph(int32_t n, const int32_t* succ_off, const int32_t* succ, const int32_t* n_classes)
{
    if (n <= 0 || !succ_off) return COE_EINVAL;
    if (succ_off[0] != 0) return COE_EGRAPH;
    for (int32_t e = 0; e < n; ++e) {
        if (succ_off[e + 1] < succ_off[e]) return COE_EGRAPH;
        if (n_classes && succ_off[e + 1] - succ_off[e] > n_classes[e]) return COE_EGRAPH;
    }
    if (succ_off[n] > 0 && !succ) return COE_EINVAL;
    for (int32_t j = 0; j < succ_off[n]; ++j)
        if (succ[j] < -1 || succ[j] >= n) return COE_EGRAPH;
    // Kahn's algorithm: every expert must be removable, else there is a cycle
    std::vector<int32_t> indeg(n, 0), stack;
    for (int32_t j = 0; j < succ_off[n]; ++j)
        if (succ[j] >= 0) ++indeg[succ[j]];
    for (int32_t e = 0; e < n; ++e)
        if (indeg[e] == 0) stack.push_back(e);
    int32_t seen = 0;
    while (!stack.empty()) {
        int32_t e = stack.back();
        stack.pop_back();
        ++seen;
        for (int32_t j = succ_off[e]; j < succ_off[e + 1]; ++j)
            if (succ[j] >= 0 && --indeg[succ[j]] == 0) stack.push_back(succ[j]);
    }
    return seen == n ? COE_OK : COE_EGRAPH;
}

}  // namespace coe

// ---- C ABI wrappers -------------------------------------------------------------------------------------------
struct coe_policy {
    coe::Policy impl;
};

extern "C" {

int coe_validate_graph(int32_t n_experts, const int32_t* succ_off, const int32_t* succ, const int32_t* n_classes)
{
    return coe::validate_graph(n_experts, succ_off, succ, n_classes);
}

coe_policy* coe_policy_create(int32_t n_experts, const int64_t* nbytes, const float* usage_prob, const int32_t* succ_off,
                              const int32_t* succ, int32_t cap_experts, int64_t cap_bytes)
{
    if (n_experts <= 0 || !nbytes || !usage_prob || !succ_off) return nullptr;
    if (coe::validate_graph(n_experts, succ_off, succ, nullptr) != COE_OK) return nullptr;
    return new (std::nothrow) coe_policy{coe::Policy(n_experts, nbytes, usage_prob, succ_off, succ, cap_experts, cap_bytes)};
}

void coe_policy_destroy(coe_policy* p) { delete p; }

int coe_policy_init_fill(coe_policy* p, int32_t* loaded)
{
    if (!p || !loaded) return COE_EINVAL;
    std::vector<int32_t> l = p->impl.init_fill();
    std::copy(l.begin(), l.end(), loaded);
    return (int)l.size();
}

int coe_policy_stage(coe_policy* p, const uint8_t* has_group, int32_t* order, int32_t* n_order, int32_t* log,
                     int32_t log_cap)
{
    if (!p || !has_group || !order || !n_order || (!log && log_cap > 0)) return COE_EINVAL;
    std::vector<int32_t> ord;
    std::vector<coe::Switch> sw;
    if (!p->impl.plan_stage(has_group, ord, sw)) return COE_ENOMEM;
    std::copy(ord.begin(), ord.end(), order);
    *n_order = (int32_t)ord.size();
    int32_t n = 0;
    for (const auto& s : sw) {
        if (n + 2 + (int32_t)s.victims.size() > log_cap) return COE_ERANGE;
        log[n++] = s.expert;
        log[n++] = (int32_t)s.victims.size();
        for (int32_t v : s.victims) log[n++] = v;
    }
    return n;
}

int coe_policy_set_eviction(coe_policy* p, int32_t kind)
{
    if (!p) return COE_EINVAL;
    return p->impl.set_eviction(kind) ? COE_OK : COE_EINVAL;
}

int coe_policy_set_in_use_depth(coe_policy* p, int32_t depth)
{
    if (!p) return COE_EINVAL;
    return p->impl.set_in_use_depth(depth) ? COE_OK : COE_EINVAL;
}

int coe_policy_resident(const coe_policy* p, uint8_t* out)
{
    if (!p || !out) return COE_EINVAL;
    int n = 0;
    for (int32_t e = 0; e < p->impl.n_experts(); ++e) {
        out[e] = p->impl.resident(e) ? 1 : 0;
        n += out[e];
    }
    return n;
}

}  // extern "C"
