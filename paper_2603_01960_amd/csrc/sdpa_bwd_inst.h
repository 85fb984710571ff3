// Instantiates the backward kernels for one (element type, head dim) and provides their launcher.
#pragma once
#include <mutex>

#include "sdpa_bwd_kernel.h"
#include "sdpa_fwd_launch.h"

namespace tsdpa {

// Tile shapes (resident rows = 32*NW per workgroup, TS streamed rows per tile) and the wavefronts per
// SIMD the register budget is sized for.  The keys-resident pass keeps two operand sets and two output
// accumulators in registers: at D = 128 that needs more than 256 registers per lane, so one wavefront per SIMD.
template <int D> struct BwdShape;
template <> struct BwdShape<64>  { static constexpr int NW = 4, TS_Q = 64, WPS_Q = 2, TS_K = 64, WPS_K = 2; };
template <> struct BwdShape<128> { static constexpr int NW = 4, TS_Q = 64, WPS_Q = 2, TS_K = 32, WPS_K = 1; };

template <typename T, int D, bool KEYS_RES>
int launch_bwd_pass(const BwdLaunchArgs &a)
{
    using Sh = BwdShape<D>;
    constexpr int NW = Sh::NW;
    constexpr int TS = KEYS_RES ? Sh::TS_K : Sh::TS_Q;
    constexpr int WPS = KEYS_RES ? Sh::WPS_K : Sh::WPS_Q;
    auto kern = sdpa_bwd_kernel<T, D, NW, TS, WPS, KEYS_RES>;
    constexpr int lds_bytes = BwdGeom<D, TS>::LDS_BYTES;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    });
    if (attr_err != hipSuccess) return (int)attr_err;
    const int nR = (a.S + NW * 32 - 1) / (NW * 32);
    const int N = a.BH * nR;
    hipLaunchKernelGGL(kern, dim3(N), dim3(NW * 64), lds_bytes, a.stream,
                       (const T *)a.q, (const T *)a.k, (const T *)a.v, (const T *)a.dout, a.lse2, a.delta,
                       (T *)(KEYS_RES ? a.dk : a.dq), (T *)(KEYS_RES ? a.dv : nullptr),
                       a.S, nR, N, a.c, a.scale, a.rsign, a.causal, a.stat_bytes);
    return (int)hipGetLastError();
}

template <typename T, int D>
int launch_bwd(const BwdLaunchArgs &a)
{
    const long long rows = (long long)a.BH * a.S;
    const long long threads = (rows + kBwdStatPad) * 16;
    hipLaunchKernelGGL((sdpa_bwd_prepare_kernel<T, D>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, a.stream,
                       (const T *)a.o, (const T *)a.dout, a.lse, a.delta, a.lse2, rows);
    int err = (int)hipGetLastError();
    if (err != 0) return err;
    err = launch_bwd_pass<T, D, true>(a);
    if (err != 0) return err;
    return launch_bwd_pass<T, D, false>(a);
}

}  // namespace tsdpa
