// Host-side declarations shared by the library's translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <tuple>
#include <utility>
#include "../../include/lithos.h"
#include "atom_device.hpp"

namespace lithos {

template <typename Tuple, size_t... I>
inline void fill_ptrs(void** ptrs, Tuple& vals, std::index_sequence<I...>)
{
    ((ptrs[I] = (void*)&std::get<I>(vals)), ...);
}

void set_error(const char* fmt, ...);
int  fail(int code, const char* fmt, ...);

#define LITHOS_HIP(call)                                                                  \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess)                                                             \
            return ::lithos::fail(LITHOS_EHIP, "%s: %s (%s:%d)", #call,                   \
                                  hipGetErrorString(e_), __FILE__, __LINE__);             \
    } while (0)

// What an operator needs to be cut in atoms.
struct OpPlan {
    lithos_dim3 grid;       // logical grid
    uint32_t total;         // gx*gy*gz
    uint32_t threads;       // workgroup size
    uint32_t wg_per_cu;     // resident workgroups per CU (occupancy)
    int variant;            // kernel variant chosen by the validator
};

// Each operator family: validate + plan (no launch), and launch one atom.
int gemm_plan(const lithos_op_t& op, OpPlan* plan);
int gemm_launch(const lithos_op_t& op, const OpPlan& plan, const AtomArgs& atom, hipStream_t s);
int rowops_plan(const lithos_op_t& op, OpPlan* plan);
int rowops_launch(const lithos_op_t& op, const OpPlan& plan, const AtomArgs& atom, hipStream_t s);
int attn_plan(const lithos_op_t& op, OpPlan* plan);
int attn_launch(const lithos_op_t& op, const OpPlan& plan, const AtomArgs& atom, hipStream_t s);
int attn_prefill_plan(const lithos_op_t& op, OpPlan* plan);
int attn_prefill_launch(const lithos_op_t& op, const OpPlan& plan, const AtomArgs& atom, hipStream_t s);
int spin_plan(const lithos_op_t& op, OpPlan* plan);
int spin_launch(const lithos_op_t& op, const OpPlan& plan, const AtomArgs& atom, hipStream_t s);
int probe_launch(uint32_t n_wg, uint32_t* dev_xcd, uint32_t* dev_hwid, hipStream_t s);

int op_plan(const lithos_op_t& op, OpPlan* plan);
int op_launch(const lithos_op_t& op, const OpPlan& plan, const AtomArgs& atom, hipStream_t s);

// hipLaunchKernel with a status code (the <<< >>> form reports errors only
// through the thread's sticky last-error slot, which hipEventQuery also sets).
template <typename... Params, typename... Args>
inline hipError_t launch_kernel(void (*k)(Params...), dim3 grid, dim3 block, hipStream_t s, Args... args)
{
    std::tuple<Params...> vals{static_cast<Params>(args)...};
    void* ptrs[sizeof...(Params)];
    fill_ptrs(ptrs, vals, std::index_sequence_for<Params...>{});
    return hipLaunchKernel(reinterpret_cast<const void*>(k), grid, block, ptrs, 0, s);
}

// hipOccupancyMaxActiveBlocksPerMultiprocessor for a kernel and workgroup size (no dynamic LDS), asked
// once per (device, kernel, size) and remembered; `fallback` if the runtime cannot say.
uint32_t cached_occupancy(const void* kernel, int threads, uint32_t fallback);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

} // namespace lithos
