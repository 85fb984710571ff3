// Instantiates the forward kernel for one (element type, head dim) over the tile grid
// T_M in {64,128} x T_N in {32,64,128} (the paper's Table 1 knobs) and the 256 x 64 tile of this library's own,
// plus the general Sq x Skv / split-KV variant over T_M in {64,128} x T_N in {32,64} (and 256 x 64 on a dense cache),
// and provides its launcher.
// The kernel table is fixed at build time: there is no JIT step to cache (Section 4.2.2).
#pragma once
#include <mutex>

#include "sdpa_fwd_kernel.h"
#include "sdpa_fwd_launch.h"

namespace tsdpa {

constexpr int kLdsPerCU = 160 * 1024;

// Register budget of an instantiation, in wavefronts per SIMD (512 registers per lane divided among
// them).  Three for 32-row K/V tiles up to D = 128: the main loop then fits 168 registers without
// spilling and the third wavefront fills more of the phases in which the other two leave the matrix
// pipe idle (+4-6 % on the long workloads).  Two otherwise, also where the LDS admits only one: a
// budget of one wavefront per SIMD makes the compiler split accumulators between the VGPR and AGPR
// halves and move them back and forth (or to scratch) inside the loop.
template <int D, int NW, int TN> constexpr int waves_per_simd() { return (TN == 32 && D <= 128) ? 3 : 2; }

template <typename T, int D, int NW, int TN, int KV = 0>     // 0 square, 1 dense cache, 2 paged cache
int launch_one(const LaunchArgs &a)
{
    constexpr int WPS = waves_per_simd<D, NW, TN>();
    auto kern = sdpa_fwd_kernel<T, D, NW, TN, WPS, KV>;
    // K/V tile slots during the loop, one 32 x D block per wavefront for the output transpose after it
    constexpr int stage_bytes = NW * 32 * TileGeom<D, TN>::OROW;
    constexpr int lds_bytes = TileGeom<D, TN>::LDS_BYTES > stage_bytes ? TileGeom<D, TN>::LDS_BYTES : stage_bytes;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    });
    if (attr_err != hipSuccess) return (int)attr_err;
    constexpr int TM = NW * 32;
    const int nQ = (a.S + TM - 1) / TM;
    const int N = a.BH * nQ * (KV ? a.splits : 1);
    hipLaunchKernelGGL(kern, dim3(N), dim3(NW * 64), lds_bytes, a.stream,
                       (const T *)a.q, (const T *)a.k, (const T *)a.v, (T *)a.o, a.lse,
                       a.S, nQ, N, a.c, a.tau, a.qsign, a.linear_grid, a.causal,
                       a.Skv, a.splits, a.ws, a.rows_per_head, a.kv_lens, a.heads_per_batch,
                       a.block_table, a.max_blocks, a.block_shift, a.tile_rot);
    return (int)hipGetLastError();
}

// The 64-row K/V tile instantiations live in translation units of their own (sdpa_fwd_*_tn64.hip): the
// build compiles those with another machine scheduler, which gains 3-5 % there and loses badly on the
// 32-row tile kernels, and a scheduler is chosen per compiler invocation.
template <typename T, int D>
int launch_dispatch_tn64(int tile_m, const LaunchArgs &a)
{
    if (tile_m != 64 && tile_m != 128 && tile_m != 256) return (int)hipErrorInvalidValue;
    // 256 query rows per workgroup (eight wavefronts, one workgroup per CU): the square problem and the dense cache
    if (tile_m == 256) {
        if (a.kv && a.block_table != nullptr) return (int)hipErrorInvalidValue;
        return a.kv ? launch_one<T, D, 8, 64, 1>(a) : launch_one<T, D, 8, 64>(a);
    }
    if (a.kv && a.block_table != nullptr)
        return tile_m == 64 ? launch_one<T, D, 2, 64, 2>(a) : launch_one<T, D, 4, 64, 2>(a);
    if (a.kv)
        return tile_m == 64 ? launch_one<T, D, 2, 64, 1>(a) : launch_one<T, D, 4, 64, 1>(a);
    return tile_m == 64 ? launch_one<T, D, 2, 64>(a) : launch_one<T, D, 4, 64>(a);
}

using LaunchTn64 = int (*)(int tile_m, const LaunchArgs &a);

template <typename T, int D>
int launch_dispatch(int tile_m, int tile_n, const LaunchArgs &a, LaunchTn64 tn64)
{
    if (tile_n == 64) return tn64(tile_m, a);
    const int key = tile_m * 1000 + tile_n;
    if (a.kv && a.block_table != nullptr) {
        switch (key) {
            case 64032: return launch_one<T, D, 2, 32, 2>(a);
            case 128032: return launch_one<T, D, 4, 32, 2>(a);
            default: return (int)hipErrorInvalidValue;
        }
    }
    if (a.kv) {
        switch (key) {
            case 64032: return launch_one<T, D, 2, 32, 1>(a);
            case 128032: return launch_one<T, D, 4, 32, 1>(a);
            default: return (int)hipErrorInvalidValue;
        }
    }
    switch (key) {
        case 64032: return launch_one<T, D, 2, 32>(a);
        case 64128:
            if constexpr (D <= 128) return launch_one<T, D, 2, 128>(a);
            else return (int)hipErrorInvalidValue;   // four 128-row slots of 320-byte rows are all of a CU's LDS
        case 128032: return launch_one<T, D, 4, 32>(a);
        case 128128:
            if constexpr (D <= 128) return launch_one<T, D, 4, 128>(a);
            else return (int)hipErrorInvalidValue;
        default: return (int)hipErrorInvalidValue;
    }
}

}  // namespace tsdpa
