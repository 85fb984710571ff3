// Instantiates the forward kernel for one (element type, head dim) over the schedule grid
// (Table 1 of the paper: T_M query rows per workgroup, T_N key/value rows per tile, staging depth)
// and provides its launcher.  The kernel table is fixed at build time: there is no JIT step to
// cache (Section 4.2.2).
#pragma once
#include <mutex>

#include "sdpa_fwd_kernel.h"
#include "sdpa_fwd_launch.h"

namespace tsdpa {

constexpr int kLdsPerCU = 160 * 1024;

// Shape of one schedule: NW wavefronts x QB query blocks of 32 rows each, NS LDS ring slots.
// Wide wavefronts (QB = 2) reuse every K/V fragment read from LDS for two MFMAs and are sized for
// one wavefront per SIMD (512 registers); narrow ones (QB = 1) for two.
template <int D, int NW, int QB, int TN> struct Shape {
    static constexpr int kTile = TN * D * 2;
    static constexpr int kWgPerCU = (QB == 2 ? 4 : 8) / NW;               // by the register budget (>= 1 for every NW used)
    static constexpr int kBudget = kLdsPerCU / kWgPerCU;                   // LDS bytes per workgroup at that occupancy
    static constexpr int kFit = kBudget / (2 * kTile);
    static constexpr int NS = kFit < 2 ? 2 : (kFit > 4 ? 4 : kFit);
    static constexpr int kLds = 2 * NS * kTile;
    static constexpr int kWgByLds = kLdsPerCU / kLds;
    static constexpr int kWaves = (kWgByLds < kWgPerCU ? kWgByLds : kWgPerCU) * NW / 4;
    static constexpr int WPS = kWaves < 1 ? 1 : kWaves;
};

template <typename T, int D, int NW, int QB, int TN>
int launch_one(const LaunchArgs &a)
{
    using Sh = Shape<D, NW, QB, TN>;
    auto kern = sdpa_fwd_kernel<T, D, NW, QB, TN, Sh::NS, Sh::WPS>;
    constexpr int lds_bytes = TileGeom<D, TN, Sh::NS>::LDS_BYTES;
    static_assert(lds_bytes <= kLdsPerCU, "schedule does not fit the LDS");
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    });
    if (attr_err != hipSuccess) return (int)attr_err;
    constexpr int TM = NW * QB * 32;
    const int nQ = (a.S + TM - 1) / TM;
    const int N = a.BH * nQ;
    hipLaunchKernelGGL(kern, dim3(N), dim3(NW * 64), lds_bytes, a.stream,
                       (const T *)a.q, (const T *)a.k, (const T *)a.v, (T *)a.o, a.lse,
                       a.S, nQ, N, a.c, a.tau, a.qsign, a.linear_grid);
    return (int)hipGetLastError();
}

template <typename T, int D, int NW, int QB>
int launch_tn(int tile_n, const LaunchArgs &a)
{
    switch (tile_n) {
        case 32:
            if constexpr (32 * (D / 8) >= NW * 64) return launch_one<T, D, NW, QB, 32>(a);
            else return (int)hipErrorInvalidValue;   // fewer 16-byte chunks per tile than lanes in the workgroup
        case 64: return launch_one<T, D, NW, QB, 64>(a);
        case 128: return launch_one<T, D, NW, QB, 128>(a);
        default: return (int)hipErrorInvalidValue;
    }
}

// tile_m 64: 2 wavefronts x 32 rows; 128: 4 x 32 (2 x 64 when `wide`); 256: 8 x 32 (4 x 64 when `wide`).
template <typename T, int D>
int launch_dispatch(int tile_m, int tile_n, bool wide, const LaunchArgs &a)
{
    switch (tile_m) {
        case 64: return launch_tn<T, D, 2, 1>(tile_n, a);
        case 128: return wide ? launch_tn<T, D, 2, 2>(tile_n, a) : launch_tn<T, D, 4, 1>(tile_n, a);
        case 256: return wide ? launch_tn<T, D, 4, 2>(tile_n, a) : launch_tn<T, D, 8, 1>(tile_n, a);
        default: return (int)hipErrorInvalidValue;
    }
}

}  // namespace tsdpa
