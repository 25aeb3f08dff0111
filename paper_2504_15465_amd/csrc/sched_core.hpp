// Spatial-scheduler policy core (LithOS Sections 4.2-4.4 and 4.7), free of
// any device call: launch queues, CU quotas, the outstanding-atom limit, atom
// sizing from predicted latency, idle-CU stealing with revocation at atom
// boundaries, and the online latency predictor.  The dispatcher/tracker
// threads drive it with the real clock; tests drive it with their own.
//
// Not thread-safe: the owner serialises calls.
#pragma once
#include <cstdint>
#include <deque>
#include <map>
#include <unordered_map>
#include <vector>
#include "../../include/lithos.h"

namespace lithos {

// Section 4.7: per launch queue, keyed by the ordinal of the kernel since the
// last synchronisation and by the CU count; the value is an exponential
// moving average of microseconds per block.  An unseen CU count scales the
// nearest known one linearly.
class Predictor {
public:
    explicit Predictor(double alpha) : alpha_(alpha) {}
    bool us_per_block(int ordinal, int cus, double* out) const;
    bool measured(int ordinal, int cus, double* out) const;     // an entry of exactly this CU count
    void update(int ordinal, int cus, uint32_t blocks, double measured_us);
private:
    double alpha_;
    std::map<int, std::map<int, double>> table_;
};

struct CoreKernel {
    uint64_t id = 0;
    uint32_t total = 0;
    uint32_t wg_per_cu = 1;
    int ordinal = -1;
    bool is_sync = false;
};

struct CoreTenant {
    int cls = LITHOS_CLASS_BE;
    uint32_t quota = 0;                 // bit g = group g
    std::deque<CoreKernel> queue;
    bool has_cur = false;
    CoreKernel cur;
    uint32_t next_block = 0;
    int next_ordinal = 0;
    int outstanding = 0;
    int queued_kernels = 0;             // kernels (not sync marks) in `queue`
    uint32_t prev_mask = 0;             // groups of the current kernel's previous atom (0: none launched yet)
    bool cur_narrow = false;            // Section 4.5: the current kernel stays on the quota
    Predictor predictor;
    lithos_stats_t stats{};
    explicit CoreTenant(double alpha) : predictor(alpha) {}
    bool idle() const { return !has_cur && outstanding == 0 && queued_kernels == 0; }
};

struct InflightAtom {
    int tenant;
    int ordinal;
    int cus;
    uint32_t blocks;
    uint32_t group_mask;
    bool has_pred;
    double pred_us;
    bool last_of_kernel;
    uint64_t kernel_id;
};

class Core {
public:
    Core(const lithos_config_t& cfg, const std::vector<int>& group_cus);
    int add_group(int cus);                                     // returns group index or <0
    int add_tenant(int cls, uint32_t quota_groups);             // returns tenant index or <0
    uint64_t submit(int tenant, uint32_t total_blocks, uint32_t wg_per_cu);
    void sync_mark(int tenant);
    bool next_atom(int tenant, double now_us, lithos_core_atom_t* out);
    // returns false for an unknown atom id; *kernel_done = id of the kernel
    // this atom finished, or 0
    bool complete(uint64_t atom_id, double now_us, double measured_us, uint64_t* kernel_done);
    const lithos_stats_t& stats(int tenant) const { return tenants_[tenant].stats; }
    lithos_stats_t totals() const;
    int n_tenants() const { return (int)tenants_.size(); }
    int n_groups() const { return (int)group_cus_.size(); }
    int cus_of(uint32_t group_mask) const;
    const CoreTenant& tenant(int t) const { return tenants_[t]; }
    bool valid_tenant(int t) const { return t >= 0 && t < (int)tenants_.size(); }

private:
    uint32_t choose_mask(int tenant, double now_us, bool* stolen) const;
    bool keep_quota(const CoreTenant& t, const CoreKernel& k, int own_cus, int wide_cus) const;
    lithos_config_t cfg_;
    std::vector<int> group_cus_;
    std::vector<CoreTenant> tenants_;
    std::vector<double> busy_until_;
    std::vector<int> busy_by_;
    std::unordered_map<uint64_t, InflightAtom> inflight_;
    uint64_t next_kernel_id_ = 1;
    uint64_t next_atom_id_ = 1;
};

} // namespace lithos
