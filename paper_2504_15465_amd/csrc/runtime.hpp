// Library-internal object definitions behind the opaque C handles.
#pragma once
#include "common.hpp"
#include <atomic>
#include <mutex>
#include <vector>

namespace lithos { struct Scheduler; }

struct lithos_ctx {
    int device = 0;
    lithos_config_t cfg{};
    int n_cu = 0, n_xcd = 1, lds_per_cu = 0, clock_khz = 0;
    char arch[32] = "";
    bool mask_interleaved = true;         // CU-mask bit i -> die i % n_xcd (else i / cu_per_xcd)
    int probe_d0 = 0, probe_other = 0;    // what the numbering probe saw
    hipStream_t plain = nullptr;          // unmasked queue for part == NULL
    hipEvent_t ev_in = nullptr, ev_out = nullptr;   // ordering-stream hand-over of lithos_launch_atomized
    std::mutex launch_mu;                 // serialises lithos_launch_atomized (one event pair per context)
    std::atomic<uint64_t> pt_kernels{0};  // kernels of pass-through tenants (launched whole at submission)
    uint32_t* counters = nullptr;         // exactly-once instrumentation (device)
    uint32_t n_counters = 0;
    std::atomic<int> live_tenants{0};
    lithos::Scheduler* sched = nullptr;   // created with the first tenant
    std::mutex park_mu;
    std::vector<hipStream_t> parked;      // retired queues kept alive while tenants exist
};

struct lithos_partition {
    lithos_ctx* ctx = nullptr;
    uint32_t mask[LITHOS_MASK_WORDS] = {0};
    int n_cus = 0;
    int n_dies = 0;                       // dies that own at least one CU of the mask
    hipStream_t stream = nullptr;
};

namespace lithos {
void default_config(lithos_config_t* c);
AtomArgs make_atom(const lithos_ctx* ctx, const OpPlan& plan, uint32_t lo, uint32_t hi, int n_dies);
int check_counters(const lithos_ctx* ctx, const OpPlan& plan);
void sched_shutdown(lithos_ctx* ctx);
// Destroying a queue moves every queue created after it to another command-processor
// pipe, which can put two tenants' queues on one pipe.  While tenants exist a queue that
// is no longer needed is therefore parked; parked queues go when the last tenant does.
void retire_stream(lithos_ctx* ctx, hipStream_t s);
void drain_parked(lithos_ctx* ctx);
}
