// Context, CU partitions, the atomized launch and the right-sizing sweep.
#include "runtime.hpp"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <fstream>
#include <map>
#include <sstream>
#include <vector>

namespace lithos {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

// ---- workspace for the entry point that allocates nothing ---------------------
// File-scope device array; each GPU holds its own copy at its own address.  In host code the
// array's name is only a stand-in for the symbol: its device address is asked for once per
// device (static_scratch_setup, called by lithos_init with that device current) and only that
// address is ever handed to kernels.
static __device__ __align__(256) __attribute__((used)) float scratch[LITHOS_STATIC_SCRATCH_FLOATS];
static const int kMaxDevices = 64;
static float* g_scratch_ptr[kMaxDevices] = {nullptr};
static std::mutex g_scratch_mu;

static int static_scratch_setup(int device)
{
    if (device < 0 || device >= kMaxDevices) return fail(LITHOS_ELIMIT, "device ordinal %d beyond %d", device, kMaxDevices);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (g_scratch_ptr[device]) return LITHOS_OK;
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(LITHOS_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", device, hipGetErrorString(e));
    g_scratch_ptr[device] = static_cast<float*>(p);
    return LITHOS_OK;
}

uint32_t cached_occupancy(const void* kernel, int threads, uint32_t fallback)
{
    struct Key { int dev; const void* fn; int threads; bool operator<(const Key& o) const { return std::tie(dev, fn, threads) < std::tie(o.dev, o.fn, o.threads); } };
    static std::mutex mu;
    static std::map<Key, uint32_t> cache;
    if (!kernel) return fallback ? fallback : 1u;
    int dev = 0;
    (void)hipGetDevice(&dev);
    const Key key{dev, kernel, threads};
    std::lock_guard<std::mutex> lk(mu);
    auto it = cache.find(key);
    if (it != cache.end()) return it->second;
    int occ = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kernel, threads, 0);
    if (e != hipSuccess) (void)hipGetLastError();
    const uint32_t v = (e == hipSuccess && occ > 0) ? (uint32_t)occ : (fallback ? fallback : 1u);
    cache[key] = v;
    return v;
}

// ---- probe kernel: which die / CU does each workgroup run on ---------------
__global__ __launch_bounds__(64) void probe_kernel(uint32_t* xcd, uint32_t* hwid, uint64_t ticks)
{
    uint32_t x, h;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(h));
    // hold the CU briefly so the workgroups of one launch spread over the mask
    const uint64_t t0 = wall_clock64();
    while (wall_clock64() - t0 < ticks) __builtin_amdgcn_s_sleep(4);
    if (threadIdx.x == 0) { xcd[blockIdx.x] = x & 0xf; hwid[blockIdx.x] = h; }
}

int probe_launch(uint32_t n_wg, uint32_t* dev_xcd, uint32_t* dev_hwid, hipStream_t s)
{
    LITHOS_HIP(launch_kernel(probe_kernel, dim3(n_wg), dim3(64), s, dev_xcd, dev_hwid, (uint64_t)2000));
    return LITHOS_OK;
}

// ---- operator dispatch -------------------------------------------------------
int op_plan(const lithos_op_t& op, OpPlan* plan)
{
    switch (op.kind) {
    case LITHOS_OP_GEMM: return gemm_plan(op, plan);
    case LITHOS_OP_ATTN_ENC:
    case LITHOS_OP_ATTN_MERGE:
    case LITHOS_OP_ATTN_DEC: return attn_plan(op, plan);
    case LITHOS_OP_ATTN_PREFILL: return attn_prefill_plan(op, plan);
    case LITHOS_OP_BIAS_ACT:
    case LITHOS_OP_LAYERNORM:
    case LITHOS_OP_SOFTMAX:
    case LITHOS_OP_RMSNORM:
    case LITHOS_OP_ROPE_KV:
    case LITHOS_OP_SILU_MUL:
    case LITHOS_OP_SUM_SLICES:
    case LITHOS_OP_SPIN: return rowops_plan(op, plan);
    default: return fail(LITHOS_EINVAL, "unknown operator kind %d", op.kind);
    }
}

int op_launch(const lithos_op_t& op, const OpPlan& plan, const AtomArgs& atom, hipStream_t s)
{
    if (atom.n == 0) return LITHOS_OK;
    switch (op.kind) {
    case LITHOS_OP_GEMM: return gemm_launch(op, plan, atom, s);
    case LITHOS_OP_ATTN_ENC:
    case LITHOS_OP_ATTN_MERGE:
    case LITHOS_OP_ATTN_DEC: return attn_launch(op, plan, atom, s);
    case LITHOS_OP_ATTN_PREFILL: return attn_prefill_launch(op, plan, atom, s);
    default: return rowops_launch(op, plan, atom, s);
    }
}

// ---- context -------------------------------------------------------------------

static int read_num_xcc(int device)
{
    // KFD topology: the GPU nodes list "num_xcc"; CPU nodes have simd_count 0.
    int gpu_index = 0;
    for (int node = 0; node < 64; ++node) {
        std::ostringstream path;
        path << "/sys/class/kfd/kfd/topology/nodes/" << node << "/properties";
        std::ifstream f(path.str());
        if (!f) break;
        std::string key;
        long long val, simd = 0, xcc = 0;
        while (f >> key >> val) {
            if (key == "simd_count") simd = val;
            if (key == "num_xcc") xcc = val;
        }
        if (simd > 0) {
            if (gpu_index == device) return (int)xcc;
            ++gpu_index;
        }
    }
    return 0;
}

// Find the driver's CU-mask bit numbering with one probe launch on a mask that
// leaves no die empty under either numbering: bits 0..15 plus every bit that
// is a multiple of cu_per_xcd.  Interleaved numbering puts 2 CUs of bits 0..15
// on every die (and the multiples of cu_per_xcd all on die 0); contiguous
// numbering puts 16 CUs on die 0 and one on each other die.
static int detect_mask_layout(lithos_ctx* ctx)
{
    ctx->mask_interleaved = true;
    const int nx = ctx->n_xcd, per = ctx->n_cu / nx;
    if (nx <= 1 || per < 16) return LITHOS_OK;
    uint32_t mask[LITHOS_MASK_WORDS] = {0};
    for (int i = 0; i < 16; ++i) mask[i / 32] |= 1u << (i % 32);
    for (int d = 1; d < nx; ++d) mask[(d * per) / 32] |= 1u << ((d * per) % 32);
    hipStream_t s = nullptr;
    LITHOS_HIP(hipExtStreamCreateWithCUMask(&s, (ctx->n_cu + 31) / 32, mask));
    const uint32_t n_wg = 2048;
    uint32_t* dev = nullptr;
    hipError_t e = hipMalloc(&dev, sizeof(uint32_t) * 2 * n_wg);
    if (e != hipSuccess) { (void)hipStreamDestroy(s); return fail(LITHOS_EHIP, "hipMalloc: %s", hipGetErrorString(e)); }
    std::vector<uint32_t> host(2 * n_wg);
    int rc = probe_launch(n_wg, dev, dev + n_wg, s);
    if (rc == LITHOS_OK) {
        e = hipStreamSynchronize(s);
        if (e == hipSuccess) e = hipMemcpy(host.data(), dev, sizeof(uint32_t) * 2 * n_wg, hipMemcpyDeviceToHost);
        if (e != hipSuccess) rc = fail(LITHOS_EHIP, "mask-layout probe: %s", hipGetErrorString(e));
    }
    (void)hipFree(dev);
    (void)hipStreamDestroy(s);
    if (rc != LITHOS_OK) return rc;
    // distinct (shader engine, array, CU) ids seen on each die
    std::vector<std::vector<uint32_t>> seen(16);
    for (uint32_t i = 0; i < n_wg; ++i) {
        uint32_t die = host[i] & 0xf, cu = (host[n_wg + i] >> 8) & 0xff;
        auto& v = seen[die];
        if (std::find(v.begin(), v.end(), cu) == v.end()) v.push_back(cu);
    }
    int max_other = 0, d0 = (int)seen[0].size(), covered = 0;
    for (int d = 0; d < 16; ++d) {
        if (!seen[d].empty()) ++covered;
        if (d > 0) max_other = std::max(max_other, (int)seen[d].size());
    }
    ctx->probe_d0 = d0;
    ctx->probe_other = max_other;
    if (covered == nx && max_other == 2 && d0 <= 2 + (nx - 1)) { ctx->mask_interleaved = true; return LITHOS_OK; }
    if (covered == nx && max_other == 1 && d0 > 2 + (nx - 1)) { ctx->mask_interleaved = false; return LITHOS_OK; }
    return fail(LITHOS_EMASK, "cannot tell the CU-mask bit numbering: %d dies seen, %d CUs on die 0, at most %d elsewhere",
                covered, d0, max_other);
}

void default_config(lithos_config_t* c)
{
    c->atom_duration_us = 250.0;
    c->max_outstanding = 2;
    c->max_outstanding_hp = 0;
    c->steal = 1;
    c->atomize = 1;
    c->xcd_remap = 1;
    c->prelude = 0;
    c->ema_alpha = 0.25;
    c->rightsize_slip = 0.0;
}

void retire_stream(lithos_ctx* ctx, hipStream_t s)
{
    if (!s) return;
    std::lock_guard<std::mutex> lk(ctx->park_mu);
    if (ctx->live_tenants.load() > 0) ctx->parked.push_back(s);
    else (void)hipStreamDestroy(s);
}

void drain_parked(lithos_ctx* ctx)
{
    std::lock_guard<std::mutex> lk(ctx->park_mu);
    // newest first: each removal then leaves the positions of the older queues alone
    for (auto it = ctx->parked.rbegin(); it != ctx->parked.rend(); ++it) { (void)hipStreamSynchronize(*it); (void)hipStreamDestroy(*it); }
    ctx->parked.clear();
}

} // namespace lithos

using namespace lithos;

extern "C" {

const char* lithos_last_error(void) { return g_err; }

int lithos_init(int device, const lithos_config_t* cfg, lithos_ctx_t** out)
{
    if (!out) return fail(LITHOS_EINVAL, "lithos_init: out is null");
    int count = 0;
    LITHOS_HIP(hipGetDeviceCount(&count));
    if (device < 0 || device >= count) return fail(LITHOS_EINVAL, "lithos_init: device %d of %d", device, count);
    LITHOS_HIP(hipSetDevice(device));
    auto* ctx = new lithos_ctx();
    ctx->device = device;
    default_config(&ctx->cfg);
    if (cfg) {
        ctx->cfg = *cfg;
        if (ctx->cfg.atom_duration_us <= 0) ctx->cfg.atom_duration_us = 250.0;
        if (ctx->cfg.max_outstanding <= 0) ctx->cfg.max_outstanding = 2;
        if (ctx->cfg.ema_alpha <= 0 || ctx->cfg.ema_alpha > 1) ctx->cfg.ema_alpha = 0.25;
        if (ctx->cfg.rightsize_slip != 0.0 && !(ctx->cfg.rightsize_slip >= 1.0)) {
            delete ctx;
            return fail(LITHOS_EINVAL, "lithos_init: rightsize_slip must be 0 (off) or >= 1");
        }
    }
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) { delete ctx; return fail(LITHOS_EHIP, "hipGetDeviceProperties: %s", hipGetErrorString(e)); }
    ctx->n_cu = prop.multiProcessorCount;
    ctx->n_xcd = read_num_xcc(device);
    if (ctx->n_xcd <= 0) ctx->n_xcd = (strncmp(prop.gcnArchName, "gfx95", 5) == 0 || strncmp(prop.gcnArchName, "gfx94", 5) == 0) ? 8 : 1;
    if (ctx->n_cu % ctx->n_xcd) ctx->n_xcd = 1;
    ctx->lds_per_cu = (int)prop.maxSharedMemoryPerMultiProcessor;
    ctx->clock_khz = prop.clockRate;
    snprintf(ctx->arch, sizeof ctx->arch, "%s", prop.gcnArchName);
    if (ctx->n_cu > 32 * LITHOS_MASK_WORDS) { delete ctx; return fail(LITHOS_ELIMIT, "device has %d CUs, more than %d", ctx->n_cu, 32 * LITHOS_MASK_WORDS); }
    e = hipStreamCreateWithFlags(&ctx->plain, hipStreamNonBlocking);
    if (e != hipSuccess) { delete ctx; return fail(LITHOS_EHIP, "hipStreamCreateWithFlags: %s", hipGetErrorString(e)); }
    e = hipEventCreateWithFlags(&ctx->ev_in, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_out, hipEventDisableTiming);
    if (e != hipSuccess) { delete ctx; return fail(LITHOS_EHIP, "hipEventCreateWithFlags: %s", hipGetErrorString(e)); }
    int rc = static_scratch_setup(device);
    if (rc == LITHOS_OK) rc = detect_mask_layout(ctx);
    if (rc != LITHOS_OK) {
        (void)hipStreamDestroy(ctx->plain);
        (void)hipEventDestroy(ctx->ev_in);
        (void)hipEventDestroy(ctx->ev_out);
        delete ctx;
        return rc;
    }
    *out = ctx;
    return LITHOS_OK;
}

int lithos_shutdown(lithos_ctx_t* ctx)
{
    if (!ctx) return fail(LITHOS_EINVAL, "lithos_shutdown: null context");
    if (ctx->live_tenants.load() != 0) return fail(LITHOS_ESTATE, "lithos_shutdown: %d tenants still exist", ctx->live_tenants.load());
    (void)hipSetDevice(ctx->device);
    sched_shutdown(ctx);
    drain_parked(ctx);
    (void)hipStreamSynchronize(ctx->plain);
    (void)hipStreamDestroy(ctx->plain);
    (void)hipEventDestroy(ctx->ev_in);
    (void)hipEventDestroy(ctx->ev_out);
    delete ctx;
    return LITHOS_OK;
}

int lithos_device_info(lithos_ctx_t* ctx, lithos_devinfo_t* out)
{
    if (!ctx || !out) return fail(LITHOS_EINVAL, "lithos_device_info: null argument");
    memset(out, 0, sizeof *out);
    out->n_cu = ctx->n_cu;
    out->n_xcd = ctx->n_xcd;
    out->cu_per_xcd = ctx->n_cu / ctx->n_xcd;
    out->wave_size = 64;
    out->lds_bytes_per_cu = ctx->lds_per_cu;
    out->clock_khz = ctx->clock_khz;
    out->mask_bits_interleaved = ctx->mask_interleaved ? 1 : 0;
    snprintf(out->arch, sizeof out->arch, "%s", ctx->arch);
    return LITHOS_OK;
}

// CU-mask bit numbering on multi-die parts.  Two numberings are possible for
// the mask words handed to hipExtStreamCreateWithCUMask:
//   interleaved: bit i addresses die (i % n_xcd), and its (i / n_xcd)-th CU;
//   contiguous:  bit i addresses die (i / cu_per_xcd), and its (i % cu_per_xcd)-th CU.
// lithos_init finds out which one the driver uses (detect_mask_layout) and
// every mask computation goes through these two helpers.
static inline int die_of_bit(const lithos_ctx* ctx, int bit)
{
    return ctx->mask_interleaved ? bit % ctx->n_xcd : bit / (ctx->n_cu / ctx->n_xcd);
}
static inline int bit_of(const lithos_ctx* ctx, int die, int cu)
{
    return ctx->mask_interleaved ? cu * ctx->n_xcd + die : die * (ctx->n_cu / ctx->n_xcd) + cu;
}

int lithos_make_mask(lithos_ctx_t* ctx, int n_cus, int policy, int first, uint32_t* mask_out)
{
    if (!ctx || !mask_out) return fail(LITHOS_EINVAL, "lithos_make_mask: null argument");
    if (n_cus <= 0 || first < 0 || first + n_cus > ctx->n_cu)
        return fail(LITHOS_EMASK, "lithos_make_mask: [%d, %d) is outside the %d CUs", first, first + n_cus, ctx->n_cu);
    memset(mask_out, 0, sizeof(uint32_t) * LITHOS_MASK_WORDS);
    const int nx = ctx->n_xcd, per = ctx->n_cu / nx;
    for (int i = first; i < first + n_cus; ++i) {
        int die, cu;
        if (policy == LITHOS_MASK_STRIPED) { die = i % nx; cu = i / nx; }          // walk across the dies first
        else if (policy == LITHOS_MASK_WHOLE_XCD) { die = i / per; cu = i % per; } // fill die after die
        else return fail(LITHOS_EINVAL, "lithos_make_mask: unknown policy %d", policy);
        int bit = bit_of(ctx, die, cu);
        mask_out[bit / 32] |= 1u << (bit % 32);
    }
    return LITHOS_OK;
}

int lithos_create_partition(lithos_ctx_t* ctx, const uint32_t* cu_mask, uint32_t mask_words, lithos_partition_t** out)
{
    if (!ctx || !cu_mask || !out) return fail(LITHOS_EINVAL, "lithos_create_partition: null argument");
    if (mask_words == 0 || mask_words > LITHOS_MASK_WORDS) return fail(LITHOS_EMASK, "lithos_create_partition: mask_words %u", mask_words);
    auto* p = new lithos_partition();
    p->ctx = ctx;
    memset(p->mask, 0, sizeof p->mask);
    int n = 0, dies = 0;
    uint32_t die_seen = 0;
    for (uint32_t w = 0; w < mask_words; ++w) {
        p->mask[w] = cu_mask[w];
        for (int b = 0; b < 32; ++b)
            if (cu_mask[w] >> b & 1u) {
                int bit = w * 32 + b;
                if (bit >= ctx->n_cu) { delete p; return fail(LITHOS_EMASK, "lithos_create_partition: bit %d beyond %d CUs", bit, ctx->n_cu); }
                ++n;
                die_seen |= 1u << die_of_bit(ctx, bit);
            }
    }
    if (n == 0) { delete p; return fail(LITHOS_EMASK, "lithos_create_partition: empty mask"); }
    for (int d = 0; d < ctx->n_xcd; ++d) dies += die_seen >> d & 1u;
    // Workgroups of a dispatch are handed to the dies in turn; a die that owns
    // no CU of the mask could not place its share, so such masks are refused.
    if (dies != ctx->n_xcd) { delete p; return fail(LITHOS_EMASK, "lithos_create_partition: the mask leaves %d of %d dies without a CU", ctx->n_xcd - dies, ctx->n_xcd); }
    p->n_cus = n;
    p->n_dies = dies;
    (void)hipSetDevice(ctx->device);
    uint32_t words = (ctx->n_cu + 31) / 32;
    hipError_t e = hipExtStreamCreateWithCUMask(&p->stream, words, p->mask);
    if (e != hipSuccess) { delete p; return fail(LITHOS_EHIP, "hipExtStreamCreateWithCUMask: %s", hipGetErrorString(e)); }
    *out = p;
    return LITHOS_OK;
}

int lithos_destroy_partition(lithos_partition_t* p)
{
    if (!p) return fail(LITHOS_EINVAL, "lithos_destroy_partition: null partition");
    (void)hipSetDevice(p->ctx->device);
    (void)hipStreamSynchronize(p->stream);
    retire_stream(p->ctx, p->stream);
    delete p;
    return LITHOS_OK;
}

int lithos_partition_cus(const lithos_partition_t* p, int* n_cus_out)
{
    if (!p || !n_cus_out) return fail(LITHOS_EINVAL, "lithos_partition_cus: null argument");
    *n_cus_out = p->n_cus;
    return LITHOS_OK;
}

int lithos_partition_stream(const lithos_partition_t* p, void** stream_out)
{
    if (!p || !stream_out) return fail(LITHOS_EINVAL, "lithos_partition_stream: null argument");
    *stream_out = (void*)p->stream;
    return LITHOS_OK;
}

int lithos_probe_partition(lithos_ctx_t* ctx, const lithos_partition_t* p, uint32_t n_wg, uint32_t* xcd_out, uint32_t* hwid_out)
{
    if (!ctx || !xcd_out || !hwid_out || n_wg == 0 || n_wg > 65536) return fail(LITHOS_EINVAL, "lithos_probe_partition: bad argument");
    (void)hipSetDevice(ctx->device);
    hipStream_t s = p ? p->stream : ctx->plain;
    uint32_t* dev = nullptr;
    LITHOS_HIP(hipMalloc(&dev, sizeof(uint32_t) * 2 * n_wg));
    int rc = probe_launch(n_wg, dev, dev + n_wg, s);
    hipError_t e = hipStreamSynchronize(s);
    if (rc == LITHOS_OK && e == hipSuccess) {
        e = hipMemcpy(xcd_out, dev, sizeof(uint32_t) * n_wg, hipMemcpyDeviceToHost);
        if (e == hipSuccess) e = hipMemcpy(hwid_out, dev + n_wg, sizeof(uint32_t) * n_wg, hipMemcpyDeviceToHost);
    }
    (void)hipFree(dev);
    if (rc != LITHOS_OK) return rc;
    if (e != hipSuccess) return fail(LITHOS_EHIP, "probe: %s", hipGetErrorString(e));
    return LITHOS_OK;
}

int lithos_op_grid(lithos_ctx_t* ctx, const lithos_op_t* op, lithos_dim3* grid_out, uint32_t* wg_per_cu_out)
{
    if (!ctx || !op) return fail(LITHOS_EINVAL, "lithos_op_grid: null argument");
    (void)hipSetDevice(ctx->device);
    OpPlan plan;
    int rc = op_plan(*op, &plan);
    if (rc != LITHOS_OK) return rc;
    if (grid_out) *grid_out = plan.grid;
    if (wg_per_cu_out) *wg_per_cu_out = plan.wg_per_cu;
    return LITHOS_OK;
}

int lithos_gemm_split_hint(const lithos_op_t* op, int32_t n_cus, int32_t* tile_out, int32_t* slices_out)
{
    if (!op || !tile_out || !slices_out || op->kind != LITHOS_OP_GEMM || n_cus <= 0)
        return fail(LITHOS_EINVAL, "lithos_gemm_split_hint: need a GEMM descriptor, a CU count and both outputs");
    const int64_t M = op->dim[0], N = op->dim[1], K = op->dim[2];
    if (M <= 0 || N <= 0 || K <= 0) return fail(LITHOS_EINVAL, "lithos_gemm_split_hint: M,N,K must be positive");
    *tile_out = 0;
    *slices_out = 1;
    // 256x256 tiles run one workgroup per CU.  With fewer than 3/4 of the CUs covered, cut K so
    // that tiles * slices just fits the CUs, keeping at least 8 k-tiles (512 of K) per slice.
    const int64_t tiles = ((M + 255) / 256) * ((N + 255) / 256), kt = (K + 63) / 64;
    if (M < 128 || N < 128 || tiles * 4 >= (int64_t)n_cus * 3) return LITHOS_OK;
    int64_t s = n_cus / tiles;
    if (s > kt / 8) s = kt / 8;
    if (s > LITHOS_GEMM_MAX_SLICES) s = LITHOS_GEMM_MAX_SLICES;
    if (s >= 2) { *tile_out = LITHOS_TILE_256; *slices_out = (int32_t)s; }
    return LITHOS_OK;
}

int lithos_debug_block_counters(lithos_ctx_t* ctx, uint32_t* dev_counters, uint32_t n)
{
    if (!ctx) return fail(LITHOS_EINVAL, "lithos_debug_block_counters: null context");
    ctx->counters = dev_counters;
    ctx->n_counters = dev_counters ? n : 0;
    return LITHOS_OK;
}

} // extern "C"

namespace lithos {

AtomArgs make_atom(const lithos_ctx* ctx, const OpPlan& plan, uint32_t lo, uint32_t hi, int n_dies)
{
    AtomArgs a;
    a.lo = lo;
    a.n = hi - lo;
    a.gx = plan.grid.x;
    a.gy = plan.grid.y;
    a.full = ctx->cfg.prelude ? plan.total : 0u;
    // Algorithm 1 as printed numbers blocks by their hardware index; the die-aware remap belongs to the
    // default form (over a whole grid it would hand an atom's contiguous range to one or two dies only)
    a.n_xcd = (ctx->cfg.xcd_remap && n_dies > 1 && !a.full) ? (uint32_t)n_dies : 1u;
    a.counters = ctx->counters;
    return a;
}

int check_counters(const lithos_ctx* ctx, const OpPlan& plan)
{
    if (ctx->counters && ctx->n_counters < plan.total)
        return fail(LITHOS_EINVAL, "block counters hold %u entries, the grid has %u blocks", ctx->n_counters, plan.total);
    return LITHOS_OK;
}

} // namespace lithos

extern "C" {

int lithos_launch_atom(lithos_ctx_t* ctx, const lithos_op_t* op, uint32_t lo, uint32_t hi, const lithos_partition_t* part)
{
    if (!ctx || !op) return fail(LITHOS_EINVAL, "lithos_launch_atom: null argument");
    (void)hipSetDevice(ctx->device);
    OpPlan plan;
    int rc = op_plan(*op, &plan);
    if (rc != LITHOS_OK) return rc;
    if (lo > hi || hi > plan.total) return fail(LITHOS_EINVAL, "lithos_launch_atom: range [%u,%u) outside [0,%u)", lo, hi, plan.total);
    if ((rc = check_counters(ctx, plan)) != LITHOS_OK) return rc;
    hipStream_t s = part ? part->stream : ctx->plain;
    return op_launch(*op, plan, make_atom(ctx, plan, lo, hi, part ? part->n_dies : ctx->n_xcd), s);
}

int lithos_launch_atomized(lithos_ctx_t* ctx, const lithos_op_t* op, lithos_dim3 grid, uint32_t atom_blocks,
                           const lithos_partition_t* part, void* stream)
{
    if (!ctx || !op) return fail(LITHOS_EINVAL, "lithos_launch_atomized: null argument");
    (void)hipSetDevice(ctx->device);
    OpPlan plan;
    int rc = op_plan(*op, &plan);
    if (rc != LITHOS_OK) return rc;
    if (grid.x || grid.y || grid.z) {
        // Atoms are ranges of the linear index z*gy*gx + y*gx + x, which covers [0, total) in the
        // same order for every factorisation: only the total has to agree.  The operator's own
        // grid (tile geometry, K slices on z) is what the kernels un-flatten that index with.
        uint64_t t = (uint64_t)grid.x * grid.y * grid.z;
        if (t != plan.total) return fail(LITHOS_EINVAL, "lithos_launch_atomized: grid has %llu blocks, the operator has %u", (unsigned long long)t, plan.total);
    }
    if ((rc = check_counters(ctx, plan)) != LITHOS_OK) return rc;
    hipStream_t s = part ? part->stream : ctx->plain;
    hipStream_t user = (hipStream_t)stream;
    const bool hop = user && user != s;
    std::lock_guard<std::mutex> lk(ctx->launch_mu);
    if (hop) {
        LITHOS_HIP(hipEventRecord(ctx->ev_in, user));
        LITHOS_HIP(hipStreamWaitEvent(s, ctx->ev_in, 0));
    }
    const uint32_t total = plan.total;
    const uint32_t B = (atom_blocks == 0 || atom_blocks >= total) ? total : atom_blocks;
    const int dies = part ? part->n_dies : ctx->n_xcd;
    for (uint32_t lo = 0; lo < total && rc == LITHOS_OK; lo += B)
        rc = op_launch(*op, plan, make_atom(ctx, plan, lo, std::min(lo + B, total), dies), s);
    if (hop) {
        // also after a failed launch: the caller's stream must not overtake the atoms already queued
        hipError_t e = hipEventRecord(ctx->ev_out, s);
        if (e == hipSuccess) e = hipStreamWaitEvent(user, ctx->ev_out, 0);
        if (e != hipSuccess && rc == LITHOS_OK) rc = fail(LITHOS_EHIP, "lithos_launch_atomized: %s", hipGetErrorString(e));
    }
    return rc;
}

int lithos_launch_attn_dec_static(lithos_ctx_t* ctx, const lithos_op_t* op, uint32_t atom_blocks,
                                  const lithos_partition_t* part, void* stream)
{
    if (!ctx || !op) return fail(LITHOS_EINVAL, "lithos_launch_attn_dec_static: null argument");
    if (op->kind != LITHOS_OP_ATTN_DEC) return fail(LITHOS_EINVAL, "lithos_launch_attn_dec_static: operator kind %d is not ATTN_DEC", op->kind);
    if (op->dim[6] < 2) return fail(LITHOS_EINVAL, "lithos_launch_attn_dec_static: needs splits >= 2 (an unsplit launch uses no workspace)");
    if (op->in[3]) return fail(LITHOS_EINVAL, "lithos_launch_attn_dec_static: in[3] must be NULL, the workspace is the library's");
    float* ws = g_scratch_ptr[ctx->device];
    if (!ws) return fail(LITHOS_ESTATE, "lithos_launch_attn_dec_static: no workspace address for device %d", ctx->device);
    (void)hipSetDevice(ctx->device);
    lithos_op_t dec = *op, merge{};
    dec.in[3] = ws;
    OpPlan pd, pm;
    int rc = op_plan(dec, &pd);             // validates shapes before the size is computed from them
    if (rc != LITHOS_OK) return rc;
    const uint64_t need = (uint64_t)dec.dim[0] * (uint64_t)dec.dim[1] * (uint64_t)dec.dim[6] * (uint64_t)(dec.dim[3] + 2);
    if (need > LITHOS_STATIC_SCRATCH_FLOATS)
        return fail(LITHOS_ELIMIT, "lithos_launch_attn_dec_static: batch*n_q*splits*(d+2) = %llu floats, the fixed workspace holds %u",
                    (unsigned long long)need, (unsigned)LITHOS_STATIC_SCRATCH_FLOATS);
    merge.kind = LITHOS_OP_ATTN_MERGE;
    merge.flags = dec.flags & LITHOS_F_OUT_F32;
    merge.op_id = dec.op_id;
    merge.dim[0] = dec.dim[0]; merge.dim[1] = dec.dim[1]; merge.dim[2] = dec.dim[2]; merge.dim[3] = dec.dim[3]; merge.dim[4] = dec.dim[6];
    merge.in[0] = ws;
    merge.out[0] = dec.out[0];
    if ((rc = op_plan(merge, &pm)) != LITHOS_OK) return rc;
    if ((rc = check_counters(ctx, pd)) != LITHOS_OK) return rc;
    hipStream_t s = part ? part->stream : ctx->plain;
    hipStream_t user = (hipStream_t)stream;
    const bool hop = user && user != s;
    const int dies = part ? part->n_dies : ctx->n_xcd;
    std::lock_guard<std::mutex> lk(ctx->launch_mu);
    if (hop) {
        LITHOS_HIP(hipEventRecord(ctx->ev_in, user));
        LITHOS_HIP(hipStreamWaitEvent(s, ctx->ev_in, 0));
    }
    const uint32_t total = pd.total;
    const uint32_t B = (atom_blocks == 0 || atom_blocks >= total) ? total : atom_blocks;
    for (uint32_t lo = 0; lo < total && rc == LITHOS_OK; lo += B)
        rc = op_launch(dec, pd, make_atom(ctx, pd, lo, std::min(lo + B, total), dies), s);
    if (rc == LITHOS_OK) {
        AtomArgs whole = make_atom(ctx, pm, 0, pm.total, dies);
        whole.counters = nullptr;           // the exactly-once counters, if set, describe the ATTN_DEC grid
        rc = op_launch(merge, pm, whole, s);
    }
    if (hop) {
        hipError_t e = hipEventRecord(ctx->ev_out, s);
        if (e == hipSuccess) e = hipStreamWaitEvent(user, ctx->ev_out, 0);
        if (e != hipSuccess && rc == LITHOS_OK) rc = fail(LITHOS_EHIP, "lithos_launch_attn_dec_static: %s", hipGetErrorString(e));
    }
    return rc;
}

int lithos_partition_sync(lithos_ctx_t* ctx, const lithos_partition_t* part)
{
    if (!ctx) return fail(LITHOS_EINVAL, "lithos_partition_sync: null context");
    (void)hipSetDevice(ctx->device);
    LITHOS_HIP(hipStreamSynchronize(part ? part->stream : ctx->plain));
    return LITHOS_OK;
}

// ---- right-sizing sweep ---------------------------------------------------------

int lithos_rightsize(lithos_ctx_t* ctx, const lithos_op_t* op, int cu_lo, int cu_hi, int cu_step,
                     int warmup, int reps, double slowdown, lithos_rightsize_result_t* out)
{
    if (!ctx || !op || !out) return fail(LITHOS_EINVAL, "lithos_rightsize: null argument");
    if (cu_lo <= 0 || cu_hi > ctx->n_cu || cu_lo > cu_hi || cu_step <= 0 || reps <= 0 || warmup < 0 || slowdown < 0)
        return fail(LITHOS_EINVAL, "lithos_rightsize: bad sweep [%d..%d step %d], reps %d", cu_lo, cu_hi, cu_step, reps);
    int n_points = (cu_hi - cu_lo) / cu_step + 1;
    if (n_points > LITHOS_MAX_SWEEP) return fail(LITHOS_ELIMIT, "lithos_rightsize: %d sweep points, at most %d", n_points, LITHOS_MAX_SWEEP);
    (void)hipSetDevice(ctx->device);
    OpPlan plan;
    int rc = op_plan(*op, &plan);
    if (rc != LITHOS_OK) return rc;
    if ((rc = check_counters(ctx, plan)) != LITHOS_OK) return rc;
    memset(out, 0, sizeof *out);
    hipEvent_t e0, e1;
    LITHOS_HIP(hipEventCreate(&e0));
    LITHOS_HIP(hipEventCreate(&e1));
    std::vector<float> ms(reps);
    for (int i = 0; i < n_points && rc == LITHOS_OK; ++i) {
        int cus = cu_lo + i * cu_step;
        uint32_t mask[LITHOS_MASK_WORDS];
        lithos_partition_t* p = nullptr;
        rc = lithos_make_mask(ctx, cus, LITHOS_MASK_STRIPED, 0, mask);
        if (rc == LITHOS_OK) rc = lithos_create_partition(ctx, mask, LITHOS_MASK_WORDS, &p);
        if (rc != LITHOS_OK) break;
        AtomArgs whole = make_atom(ctx, plan, 0, plan.total, p->n_dies);
        hipError_t e = hipSuccess;
        for (int w = 0; w < warmup && rc == LITHOS_OK; ++w) rc = op_launch(*op, plan, whole, p->stream);
        for (int r = 0; r < reps && rc == LITHOS_OK && e == hipSuccess; ++r) {
            e = hipEventRecord(e0, p->stream);
            rc = op_launch(*op, plan, whole, p->stream);
            if (e == hipSuccess) e = hipEventRecord(e1, p->stream);
            if (e == hipSuccess) e = hipEventSynchronize(e1);
            if (e == hipSuccess) e = hipEventElapsedTime(&ms[r], e0, e1);
        }
        lithos_destroy_partition(p);
        if (rc == LITHOS_OK && e != hipSuccess) rc = fail(LITHOS_EHIP, "lithos_rightsize timing: %s", hipGetErrorString(e));
        if (rc != LITHOS_OK) break;
        std::sort(ms.begin(), ms.end());
        double med = (reps & 1) ? ms[reps / 2] : 0.5 * (ms[reps / 2 - 1] + ms[reps / 2]);
        out->cus[i] = cus;
        out->median_us[i] = med * 1000.0;
        out->n_points = i + 1;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != LITHOS_OK) return rc;
    // selection: smallest CU count within (1+slowdown) of the largest count's latency
    const int last = out->n_points - 1;
    out->full_us = out->median_us[last];
    out->chosen_cus = out->cus[last];
    out->chosen_us = out->full_us;
    for (int i = 0; i <= last; ++i)
        if (out->median_us[i] <= (1.0 + slowdown) * out->full_us) { out->chosen_cus = out->cus[i]; out->chosen_us = out->median_us[i]; break; }
    out->occupancy_bound_cus = (int)std::max<uint32_t>(1u, (plan.total + plan.wg_per_cu - 1) / plan.wg_per_cu);
    // two-point model l = m/t + b through the smallest and the largest sweep point
    if (last >= 1) {
        double t1 = out->cus[0], t2 = out->cus[last], l1 = out->median_us[0], l2 = out->median_us[last];
        out->model_m = (l1 - l2) / (1.0 / t1 - 1.0 / t2);
        out->model_b = l2 - out->model_m / t2;
        double target = (1.0 + slowdown) * (out->model_m / t2 + out->model_b);
        out->model_cus = out->cus[last];
        for (int t = 1; t <= out->cus[last]; ++t)
            if (out->model_m / t + out->model_b <= target * (1 + 1e-12)) { out->model_cus = t; break; }
    }
    // Section 4.5 'Operation': the occupancy bound if the kernel cannot fill the allocation, else the model
    out->online_cus = out->occupancy_bound_cus < out->cus[last] ? out->occupancy_bound_cus
                                                                 : (last >= 1 ? out->model_cus : out->cus[last]);
    return LITHOS_OK;
}

} // extern "C"

// ---- timing of one (atomized) launch with device time stamps ---------------------

extern "C" int lithos_time_launch(lithos_ctx_t* ctx, const lithos_op_t* op, uint32_t atom_blocks,
                                  const lithos_partition_t* part, int warmup, int reps,
                                  double* mean_us_out, double* median_us_out)
{
    if (!ctx || !op || reps <= 0 || warmup < 0) return fail(LITHOS_EINVAL, "lithos_time_launch: bad argument");
    (void)hipSetDevice(ctx->device);
    OpPlan plan;
    int rc = op_plan(*op, &plan);
    if (rc != LITHOS_OK) return rc;
    if ((rc = check_counters(ctx, plan)) != LITHOS_OK) return rc;
    hipStream_t s = part ? part->stream : ctx->plain;
    const int dies = part ? part->n_dies : ctx->n_xcd;
    const uint32_t total = plan.total;
    const uint32_t B = (atom_blocks == 0 || atom_blocks >= total) ? total : atom_blocks;
    hipEvent_t e0, e1;
    LITHOS_HIP(hipEventCreate(&e0));
    LITHOS_HIP(hipEventCreate(&e1));
    std::vector<float> ms(reps);
    hipError_t e = hipSuccess;
    for (int r = -warmup; r < reps && rc == LITHOS_OK && e == hipSuccess; ++r) {
        if (r >= 0) e = hipEventRecord(e0, s);
        for (uint32_t lo = 0; lo < total && rc == LITHOS_OK; lo += B)
            rc = op_launch(*op, plan, make_atom(ctx, plan, lo, std::min(lo + B, total), dies), s);
        if (r >= 0) {
            if (e == hipSuccess) e = hipEventRecord(e1, s);
            if (e == hipSuccess) e = hipEventSynchronize(e1);
            if (e == hipSuccess) e = hipEventElapsedTime(&ms[r], e0, e1);
        }
    }
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != LITHOS_OK) return rc;
    if (e != hipSuccess) return fail(LITHOS_EHIP, "lithos_time_launch: %s", hipGetErrorString(e));
    double sum = 0;
    for (float v : ms) sum += v;
    std::sort(ms.begin(), ms.end());
    if (mean_us_out) *mean_us_out = sum / reps * 1000.0;
    if (median_us_out) *median_us_out = ((reps & 1) ? ms[reps / 2] : 0.5 * (ms[reps / 2 - 1] + ms[reps / 2])) * 1000.0;
    return LITHOS_OK;
}
