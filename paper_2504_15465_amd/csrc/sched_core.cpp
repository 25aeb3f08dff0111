#include "sched_core.hpp"

#include <algorithm>
#include <cmath>
#include <cstdlib>

namespace lithos {

static const double kMispredictUs = 50.0;   // Section 7.4: |error| above 50 us

bool Predictor::us_per_block(int ordinal, int cus, double* out) const
{
    auto row = table_.find(ordinal);
    if (row == table_.end() || row->second.empty()) return false;
    auto hit = row->second.find(cus);
    if (hit != row->second.end()) { *out = hit->second; return true; }
    int best = -1;
    for (const auto& kv : row->second) {
        if (best < 0) { best = kv.first; continue; }
        int d = std::abs(kv.first - cus), db = std::abs(best - cus);
        if (d < db || (d == db && kv.first > best)) best = kv.first;
    }
    *out = row->second.at(best) * (double)best / (double)cus;   // linear in CUs
    return true;
}

bool Predictor::measured(int ordinal, int cus, double* out) const
{
    auto row = table_.find(ordinal);
    if (row == table_.end()) return false;
    auto hit = row->second.find(cus);
    if (hit == row->second.end()) return false;
    *out = hit->second;
    return true;
}

void Predictor::update(int ordinal, int cus, uint32_t blocks, double measured_us)
{
    double v = measured_us / (double)blocks;
    auto& row = table_[ordinal];
    auto it = row.find(cus);
    if (it == row.end()) row[cus] = v;
    else it->second = (1.0 - alpha_) * it->second + alpha_ * v;
}

Core::Core(const lithos_config_t& cfg, const std::vector<int>& group_cus)
    : cfg_(cfg), group_cus_(group_cus), busy_until_(group_cus.size(), 0.0), busy_by_(group_cus.size(), -1)
{
}

int Core::add_group(int cus)
{
    if (group_cus_.size() >= 32 || cus <= 0) return -1;
    group_cus_.push_back(cus);
    busy_until_.push_back(0.0);
    busy_by_.push_back(-1);
    return (int)group_cus_.size() - 1;
}

int Core::add_tenant(int cls, uint32_t quota_groups)
{
    if (quota_groups == 0) return -1;
    if (group_cus_.size() < 32 && (quota_groups >> group_cus_.size()) != 0) return -1;
    for (const auto& t : tenants_)
        if (t.quota & quota_groups) return -1;          // quotas must be disjoint
    tenants_.emplace_back(cfg_.ema_alpha);
    tenants_.back().cls = cls;
    tenants_.back().quota = quota_groups;
    return (int)tenants_.size() - 1;
}

uint64_t Core::submit(int tenant, uint32_t total_blocks, uint32_t wg_per_cu)
{
    CoreKernel k;
    k.id = next_kernel_id_++;
    k.total = total_blocks;
    k.wg_per_cu = wg_per_cu ? wg_per_cu : 1;
    tenants_[tenant].queue.push_back(k);
    tenants_[tenant].queued_kernels++;
    return k.id;
}

void Core::sync_mark(int tenant)
{
    CoreKernel k;
    k.is_sync = true;
    tenants_[tenant].queue.push_back(k);
}

int Core::cus_of(uint32_t group_mask) const
{
    int n = 0;
    for (size_t g = 0; g < group_cus_.size(); ++g)
        if (group_mask >> g & 1u) n += group_cus_[g];
    return n;
}

// Quota, plus the whole quota of every other tenant that is idle and whose
// group timers have expired (or were set by this tenant's own atoms).
uint32_t Core::choose_mask(int tenant, double now_us, bool* stolen) const
{
    uint32_t mask = tenants_[tenant].quota;
    *stolen = false;
    if (!cfg_.steal) return mask;
    for (int o = 0; o < (int)tenants_.size(); ++o) {
        if (o == tenant || !tenants_[o].idle()) continue;
        bool all_free = true;
        for (size_t g = 0; g < group_cus_.size(); ++g)
            if (tenants_[o].quota >> g & 1u)
                if (!(busy_until_[g] <= now_us || busy_by_[g] == tenant)) { all_free = false; break; }
        if (all_free) { mask |= tenants_[o].quota; *stolen = true; }
    }
    return mask;
}

// Section 4.5 'Operation' on the two CU sets a kernel can get right now (its quota, or the quota
// plus borrowed CUs): true = the wider set is not worth taking.
bool Core::keep_quota(const CoreTenant& t, const CoreKernel& k, int own_cus, int wide_cus) const
{
    // 'Filtering Outliers': CUs the kernel can fill = blocks / resident blocks per CU
    const uint64_t bound = std::max<uint64_t>(1, ((uint64_t)k.total + k.wg_per_cu - 1) / k.wg_per_cu);
    if (bound < (uint64_t)wide_cus) return bound <= (uint64_t)own_cus;
    // 'Modeling Kernel Scaling': l = m/t + b through the kernel's latencies on the two sets
    // (the model needs the kernel's latency on both sets: the wider one is measured first, then the
    // quota once, after which the fit decides)
    double u1, u2;
    if (!t.predictor.measured(k.ordinal, wide_cus, &u2)) return false;
    if (!t.predictor.measured(k.ordinal, own_cus, &u1)) return true;
    const double l1 = u1 * k.total, l2 = u2 * k.total;
    const double m = (l1 - l2) / (1.0 / own_cus - 1.0 / wide_cus), b = l2 - m / wide_cus;
    const double target = cfg_.rightsize_slip * (m / wide_cus + b) * (1 + 1e-12);
    for (int c = 1; c <= own_cus; ++c)
        if (m / c + b <= target) return true;       // the minimum CU count within the slip fits in the quota
    return false;
}

static uint32_t atom_count(double predicted_us, double atom_us, uint32_t total)
{
    double n = predicted_us > 0 ? std::ceil(predicted_us / atom_us) : 1.0;
    if (n < 1.0) n = 1.0;
    if (n > (double)total) n = (double)total;
    return (uint32_t)n;
}

static uint32_t atom_size(uint32_t total, uint32_t n_atoms, uint64_t quantum)
{
    if (n_atoms <= 1) return total;
    uint64_t b = ((uint64_t)total + n_atoms - 1) / n_atoms;
    if (quantum > 1) b = (b + quantum - 1) / quantum * quantum;
    return (uint32_t)std::min<uint64_t>(b, total);
}

bool Core::next_atom(int ti, double now_us, lithos_core_atom_t* out)
{
    CoreTenant& t = tenants_[ti];
    int limit = cfg_.max_outstanding;
    if (t.cls == LITHOS_CLASS_HP && cfg_.max_outstanding_hp > 0) limit = cfg_.max_outstanding_hp;
    if (t.outstanding >= limit) return false;
    while (!t.has_cur) {
        if (t.queue.empty()) return false;
        CoreKernel head = t.queue.front();
        t.queue.pop_front();
        if (head.is_sync) { t.next_ordinal = 0; continue; }   // batch boundary (Section 4.7)
        t.queued_kernels--;
        t.cur = head;
        t.cur.ordinal = t.next_ordinal++;
        t.next_block = 0;
        t.has_cur = true;
        t.prev_mask = 0;
        t.stats.kernels++;
    }
    const CoreKernel& k = t.cur;
    bool stolen = false;
    uint32_t mask = choose_mask(ti, now_us, &stolen);
    if (t.next_block == 0) {
        // decided once per kernel; its atoms inherit the allocation (Section 4.5)
        t.cur_narrow = stolen && cfg_.rightsize_slip >= 1.0 && keep_quota(t, k, cus_of(t.quota), cus_of(mask));
        if (t.cur_narrow) t.stats.rightsized_kernels++;
    }
    if (t.cur_narrow) { mask = t.quota; stolen = false; }
    const int cus = cus_of(mask);
    const uint32_t remaining = k.total - t.next_block;
    uint32_t blocks = remaining;
    double upb = 0.0, pred = 0.0;
    const bool has_pred = t.predictor.us_per_block(k.ordinal, cus, &upb);
    if (has_pred) {
        if (!cfg_.atomize) {
            pred = upb * remaining;
        } else {
            // Section 4.4 'Operation': atoms = predicted duration / atom_duration
            const double pred_kernel = upb * k.total;
            const uint32_t n = atom_count(pred_kernel, cfg_.atom_duration_us, k.total);
            uint32_t b = atom_size(k.total, n, (uint64_t)cus * k.wg_per_cu);
            if (b >= k.total && pred_kernel > 2.0 * cfg_.atom_duration_us) b = atom_size(k.total, n, 1);
            blocks = std::min(b, remaining);
            pred = upb * blocks;
        }
    }
    out->atom_id = next_atom_id_++;
    out->tenant = ti;
    out->kernel_id = k.id;
    out->ordinal = k.ordinal;
    out->lo = t.next_block;
    out->hi = t.next_block + blocks;
    out->group_mask = mask;
    out->stolen = stolen ? 1 : 0;
    out->has_prediction = has_pred ? 1 : 0;
    out->predicted_us = has_pred ? pred : 0.0;

    InflightAtom a;
    a.tenant = ti; a.ordinal = k.ordinal; a.cus = cus; a.blocks = blocks; a.group_mask = mask;
    a.has_pred = has_pred; a.pred_us = pred; a.kernel_id = k.id;
    t.next_block += blocks;
    a.last_of_kernel = t.next_block >= k.total;
    if (a.last_of_kernel) t.has_cur = false;
    inflight_[out->atom_id] = a;
    t.outstanding++;
    t.stats.atoms++;
    if (stolen) t.stats.stolen_atoms++;
    // an atom boundary at which borrowed groups went back (Section 4.4 'Operation')
    if (t.prev_mask & ~mask) t.stats.revocations++;
    t.prev_mask = mask;
    // per-group timers from the prediction (unknown: one atom_duration)
    const double hold = has_pred ? pred : cfg_.atom_duration_us;
    for (size_t g = 0; g < group_cus_.size(); ++g)
        if (mask >> g & 1u) {
            busy_until_[g] = std::max(busy_until_[g], now_us) + hold;
            busy_by_[g] = ti;
        }
    return true;
}

lithos_stats_t Core::totals() const
{
    lithos_stats_t s{};
    for (const CoreTenant& t : tenants_) {
        s.kernels += t.stats.kernels;
        s.atoms += t.stats.atoms;
        s.stolen_atoms += t.stats.stolen_atoms;
        s.revocations += t.stats.revocations;
        s.rightsized_kernels += t.stats.rightsized_kernels;
        s.predictions += t.stats.predictions;
        s.mispredicts += t.stats.mispredicts;
        s.abs_err_sum_us += t.stats.abs_err_sum_us;
    }
    return s;
}

bool Core::complete(uint64_t atom_id, double now_us, double measured_us, uint64_t* kernel_done)
{
    auto it = inflight_.find(atom_id);
    if (it == inflight_.end()) return false;
    const InflightAtom a = it->second;
    inflight_.erase(it);
    CoreTenant& t = tenants_[a.tenant];
    t.outstanding--;
    if (a.has_pred) {
        t.stats.predictions++;
        double err = std::fabs(a.pred_us - measured_us);
        t.stats.abs_err_sum_us += err;
        if (err > kMispredictUs) t.stats.mispredicts++;
    }
    t.predictor.update(a.ordinal, a.cus, a.blocks, measured_us);
    if (t.outstanding == 0)
        for (size_t g = 0; g < group_cus_.size(); ++g)
            if ((a.group_mask >> g & 1u) && busy_by_[g] == a.tenant)
                busy_until_[g] = std::min(busy_until_[g], now_us);
    if (kernel_done) *kernel_done = a.last_of_kernel ? a.kernel_id : 0;
    return true;
}

} // namespace lithos

// ---- C ABI of the steppable core -------------------------------------------------

namespace lithos { int fail(int code, const char* fmt, ...); void default_config(lithos_config_t* c); }

struct lithos_core { lithos::Core* core; };

extern "C" {

int lithos_core_create(const lithos_config_t* cfg, int n_groups, int cus_per_group, lithos_core_t** out)
{
    if (!out || n_groups <= 0 || n_groups > 32 || cus_per_group <= 0)
        return lithos::fail(LITHOS_EINVAL, "lithos_core_create: need 1..32 groups of >0 CUs");
    lithos_config_t c;
    lithos::default_config(&c);
    if (cfg) c = *cfg;
    if (c.atom_duration_us <= 0 || c.max_outstanding <= 0 || c.ema_alpha <= 0 || c.ema_alpha > 1 ||
        (c.rightsize_slip != 0.0 && !(c.rightsize_slip >= 1.0)))
        return lithos::fail(LITHOS_EINVAL, "lithos_core_create: bad configuration");
    auto* h = new lithos_core();
    h->core = new lithos::Core(c, std::vector<int>(n_groups, cus_per_group));
    *out = h;
    return LITHOS_OK;
}

int lithos_core_destroy(lithos_core_t* c)
{
    if (!c) return lithos::fail(LITHOS_EINVAL, "lithos_core_destroy: null");
    delete c->core;
    delete c;
    return LITHOS_OK;
}

int lithos_core_add_tenant(lithos_core_t* c, int cls, uint32_t quota_groups, int* tenant_out)
{
    if (!c || !tenant_out) return lithos::fail(LITHOS_EINVAL, "lithos_core_add_tenant: null");
    int t = c->core->add_tenant(cls, quota_groups);
    if (t < 0) return lithos::fail(LITHOS_EMASK, "lithos_core_add_tenant: quota empty, out of range or overlapping");
    *tenant_out = t;
    return LITHOS_OK;
}

int lithos_core_submit(lithos_core_t* c, int tenant, uint32_t total_blocks, uint32_t wg_per_cu, uint64_t* kernel_id_out)
{
    if (!c || !c->core->valid_tenant(tenant) || total_blocks == 0)
        return lithos::fail(LITHOS_EINVAL, "lithos_core_submit: bad tenant or empty kernel");
    uint64_t id = c->core->submit(tenant, total_blocks, wg_per_cu);
    if (kernel_id_out) *kernel_id_out = id;
    return LITHOS_OK;
}

int lithos_core_sync_mark(lithos_core_t* c, int tenant)
{
    if (!c || !c->core->valid_tenant(tenant)) return lithos::fail(LITHOS_EINVAL, "lithos_core_sync_mark: bad tenant");
    c->core->sync_mark(tenant);
    return LITHOS_OK;
}

int lithos_core_next_atom(lithos_core_t* c, int tenant, double now_us, lithos_core_atom_t* atom_out, int* have_out)
{
    if (!c || !atom_out || !have_out || !c->core->valid_tenant(tenant))
        return lithos::fail(LITHOS_EINVAL, "lithos_core_next_atom: bad argument");
    *have_out = c->core->next_atom(tenant, now_us, atom_out) ? 1 : 0;
    return LITHOS_OK;
}

int lithos_core_complete(lithos_core_t* c, uint64_t atom_id, double now_us, double measured_us)
{
    if (!c) return lithos::fail(LITHOS_EINVAL, "lithos_core_complete: null");
    if (!c->core->complete(atom_id, now_us, measured_us, nullptr))
        return lithos::fail(LITHOS_ESTATE, "lithos_core_complete: atom %llu is not in flight", (unsigned long long)atom_id);
    return LITHOS_OK;
}

int lithos_core_stats(lithos_core_t* c, int tenant, lithos_stats_t* out)
{
    if (!c || !out || !c->core->valid_tenant(tenant)) return lithos::fail(LITHOS_EINVAL, "lithos_core_stats: bad argument");
    *out = c->core->stats(tenant);
    return LITHOS_OK;
}

} // extern "C"
