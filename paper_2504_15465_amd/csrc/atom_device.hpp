// Device-side half of kernel atomization (LithOS Section 4.4, Algorithm 1).
//
// The paper launches the full grid once per atom and lets blocks outside
// [lo,hi) exit early.  By default an atom here launches exactly hi-lo
// workgroups and each turns its hardware workgroup number into a logical block
// index, so no early-exit traffic exists; the paper's form is kept beside it
// (AtomArgs::full) so that its cost can be measured.  The logical index is numbered as in
// Algorithm 1: idx = z*gy*gx + y*gx + x.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Workgroups launched for an atom: its own blocks, or the whole grid in the Prelude form.
#define LITHOS_ATOM_LAUNCH_BLOCKS(a) ((a).full ? (a).full : (a).n)

namespace lithos {

struct AtomArgs {
    uint32_t lo;        // first logical block of this atom
    uint32_t n;         // blocks in this atom (= workgroups launched)
    uint32_t gx, gy;    // logical grid (gz is implied by the total)
    uint32_t n_xcd;     // >1: undo round-robin placement over that many dies
    uint32_t full;      // >0: Algorithm 1 as printed - this many workgroups (the whole grid) were launched
    uint32_t* counters; // exactly-once instrumentation, or nullptr
};

// Bijection of [0,n): hardware workgroup h runs on die h % n_xcd as that
// die's (h / n_xcd)-th workgroup; die x is given a contiguous run of logical
// slots (the first n % n_xcd dies hold one more than the rest), so
// neighbouring logical blocks share a die's L2.
__device__ __forceinline__ uint32_t atom_pi(uint32_t h, uint32_t n, uint32_t n_xcd)
{
    if (n_xcd <= 1) return h;
    uint32_t q = n / n_xcd, r = n % n_xcd;
    uint32_t x = h % n_xcd, s = h / n_xcd;
    return x * q + (x < r ? x : r) + s;
}

// Logical block index of the calling workgroup (uniform across the workgroup).
__device__ __forceinline__ uint32_t atom_logical_block(const AtomArgs& a)
{
    uint32_t L;
    if (a.full) {
        // the paper's Prelude: every block of the whole grid computes its index and leaves at once
        // when the index is outside the atom's range (uniform over the workgroup, before any barrier)
        L = atom_pi(blockIdx.x, a.full, a.n_xcd);
        if (L < a.lo || L - a.lo >= a.n) __builtin_amdgcn_endpgm();
    } else {
        L = a.lo + atom_pi(blockIdx.x, a.n, a.n_xcd);
    }
    if (a.counters != nullptr && threadIdx.x == 0) atomicAdd(&a.counters[L], 1u);
    return L;
}

struct Block3 { uint32_t x, y, z; };

// Inverse of Algorithm 1's linearisation.
__device__ __forceinline__ Block3 atom_delinearize(uint32_t L, const AtomArgs& a)
{
    Block3 b;
    b.x = L % a.gx;
    uint32_t t = L / a.gx;
    b.y = t % a.gy;
    b.z = t / a.gy;
    return b;
}

} // namespace lithos
