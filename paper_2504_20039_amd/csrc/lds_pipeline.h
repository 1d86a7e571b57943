// Device helpers shared by the LM-head kernels that stream operand tiles global -> LDS asynchronously.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aj {

// Asynchronous 16-byte-per-lane load global -> LDS: lane i's data lands at lds_base + 16*i.
// Written as inline assembly on purpose: with the compiler builtin, the compiler orders every later
// LDS read after ALL outstanding loads of this kind (s_waitcnt vmcnt(0)), which would drain the
// pipeline at every stage.  Here the kernel does its own accounting (wait_vm_and_barrier below); the
// compiler sees only a memory clobber.  lds_dst must be wave-uniform (it travels in M0).
__device__ __forceinline__ void load_to_lds_16(const char *base, uint32_t lane_off, uint32_t lds_dst)
{
    // base: wave-uniform global pointer; lane_off: this lane's unsigned byte offset from it
    uint32_t saved_m0;   // M0 is reserved for the compiler: keep its value across the statement
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0)
                 : "v"(lane_off), "s"(base), "s"(lds_dst)
                 : "memory");
}

// The same with the non-temporal hint, for an operand that is streamed from HBM exactly once (W_lm when
// a single row tile covers all verify rows): its lines are not kept in L2 at the expense of data that is
// re-read.  Measured: 6.19 -> 6.52 TB/s on the batch-1 streaming kernel.
__device__ __forceinline__ void load_to_lds_16_nt(const char *base, uint32_t lane_off, uint32_t lds_dst)
{
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0)
                 : "v"(lane_off), "s"(base), "s"(lds_dst)
                 : "memory");
}

// Same load for the hand-scheduled loop: two instructions, M0 not restored (nothing else in these
// kernels uses M0, and the compiler sets it itself before any use of its own).
__device__ __forceinline__ void lds_dma_16(const char *base, uint32_t lane_off, uint32_t lds_dst)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(lds_dst) : "memory");
}

__device__ __forceinline__ void lds_dma_16_nt(const char *base, uint32_t lane_off, uint32_t lds_dst)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(lane_off), "s"(base), "s"(lds_dst) : "memory");
}

__device__ __forceinline__ uint32_t lds_offset_of(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char *)p;
}

template <int N>
__device__ __forceinline__ void wait_vm_and_barrier()
{
    // wait until at most N of this wave's global loads are outstanding, then workgroup barrier.
    // The memory clobber keeps the compiler from moving LDS accesses across it.
    static_assert(N >= 0 && N <= 63, "vmcnt field");
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vm_lgkm_and_barrier()
{
    // as above, and this wave's LDS reads have returned (its buffer may be overwritten after the barrier)
    static_assert(N >= 0 && N <= 63, "vmcnt field");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}


// Tile order of the persistent kernels: groups of gm row tiles x all column tiles, row tile fastest
// inside a group, so that consecutive tiles share operand panels.
struct Sched {
    int tiles_m, tiles_n, gm, total;
};

__device__ __forceinline__ void tile_of(const Sched &sc, int T, int &mt, int &nt)
{
    const int per_group = sc.gm * sc.tiles_n;
    const int ngroups = (sc.tiles_m + sc.gm - 1) / sc.gm;
    int grp = T / per_group;
    if (grp > ngroups - 1) grp = ngroups - 1;
    const int within = T - grp * per_group;
    const int g = (grp == ngroups - 1) ? sc.tiles_m - grp * sc.gm : sc.gm;
    mt = grp * sc.gm + within % g;
    nt = within / g;
}

// grid of a persistent LM-head kernel: one workgroup per CU, a multiple of 8 (the XCD count), and no
// more workgroups than tiles (rounded up to a multiple of 8 so that the tile -> XCD mapping holds)
inline int persistent_grid(int num_cus, int total_tiles)
{
    int grid = (num_cus / 8) * 8;
    if (grid < 8) grid = 8;
    const int need = ((total_tiles + 7) / 8) * 8;
    return grid > need ? need : grid;
}

}  // namespace aj
