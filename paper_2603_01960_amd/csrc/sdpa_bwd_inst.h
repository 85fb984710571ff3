// Instantiates the backward kernels for one (element type, head dim) and provides their launcher.
#pragma once
#include <mutex>

#include "sdpa_bwd_kernel.h"
#include "sdpa_fwd_launch.h"

namespace tsdpa {

// Tile shapes, from timings on MI355X: 32*NW resident rows per workgroup, TS streamed rows per tile for
// the dQ / dK / dV pass, and the wavefronts per SIMD the register budget of each is sized for.  At D = 128 the
// dK pass (two resident operand sets, one output, per-row statistics) is the tightest on registers
// and runs best on 32-row tiles; the dQ pass on 64-row tiles spilled ten registers that it touched on
// every tile (108 MB of scratch traffic per call on B=2 H=32 S=8192) and is 2 % faster on 32-row tiles.
// FUSED_DKV: dK and dV in one keys-resident pass (seven S x S x D products per call instead of eight,
// one launch fewer); its two accumulators and two resident operand sets fit 256 registers at D = 64.
template <int D> struct BwdShape;
template <> struct BwdShape<64>  { static constexpr int NW = 4, WPS[4] = {2, 2, 2, 2}, TS[4] = {64, 64, 64, 64}; static constexpr bool FUSED_DKV = true; };
template <> struct BwdShape<96>  { static constexpr int NW = 4, WPS[4] = {2, 2, 2, 2}, TS[4] = {64, 32, 64, 32}; static constexpr bool FUSED_DKV = false; };
template <> struct BwdShape<128> { static constexpr int NW = 4, WPS[4] = {2, 2, 2, 2}, TS[4] = {32, 32, 64, 32}; static constexpr bool FUSED_DKV = false; };
// D = 160 (512-byte LDS rows): at two wavefronts per SIMD the dK and dQ passes spill 55-65 registers; with the
// whole register file of a SIMD for one wavefront (the compiler then places accumulators in AGPRs) nothing
// spills and the pass is 38 % faster although only one workgroup fits a CU.  The dV pass (one product fewer,
// no dP) does fit 256 registers on 32-row tiles, whose 64 KB of LDS admit a second workgroup: +12 % per call.
template <> struct BwdShape<160> { static constexpr int NW = 4, WPS[4] = {1, 1, 2, 1}, TS[4] = {64, 32, 32, 32}; static constexpr bool FUSED_DKV = false; };

template <typename T, int D, int MODE, bool GRP, int NW>
int launch_bwd_pass_nw(const BwdLaunchArgs &a)
{
    using Sh = BwdShape<D>;
    constexpr int TS = Sh::TS[MODE], WPS = Sh::WPS[MODE];
    auto kern = sdpa_bwd_kernel<T, D, NW, TS, WPS, MODE, GRP>;
    // tile and statistics slots during the loop, one 32 x D block per wavefront for the output transpose after it
    constexpr int stage_bytes = NW * 32 * BwdGeom<D, TS>::ROW;
    constexpr int lds_bytes = BwdGeom<D, TS>::LDS_BYTES > stage_bytes ? BwdGeom<D, TS>::LDS_BYTES : stage_bytes;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    });
    if (attr_err != hipSuccess) return (int)attr_err;
    const int nR = (a.S + NW * 32 - 1) / (NW * 32);
    // one workgroup per (head of the resident side, tile of its rows): query heads in the dQ pass, key/value heads otherwise
    const int N = (MODE == BWD_DQ ? a.BH : a.BH / a.group) * nR;
    void *out = MODE == BWD_DQ ? a.dq : (MODE == BWD_DV ? a.dv : a.dk);
    hipLaunchKernelGGL(kern, dim3(N), dim3(NW * 64), lds_bytes, a.stream,
                       (const T *)a.q, (const T *)a.k, (const T *)a.v, (const T *)a.dout, a.delta,
                       (T *)out, (T *)(MODE == BWD_DKV ? a.dv : nullptr), a.S, nR, N, a.c, a.scale, a.rsign, a.causal, a.stat_bytes, a.group);
    return (int)hipGetLastError();
}

// Eight wavefronts per workgroup (256 resident rows, one workgroup per CU) at D = 128 without the causal mask, once
// that gives every CU a workgroup: each streamed tile is then loaded once for twice the rows, half the load
// instructions per wavefront (3-4 % on the whole call from S = 2048 to 16384; with the mask the coarser tiles lose 3-12 %,
// at D = 96 and 64 the gain is 0.5-2 %, and the D = 160 passes have no registers for it).
template <typename T, int D, int MODE, bool GRP>
int launch_bwd_pass(const BwdLaunchArgs &a)
{
    if constexpr (D == 128) {
        const long long heads = MODE == BWD_DQ ? a.BH : a.BH / a.group;
        if (!a.causal && heads * ((a.S + 255) / 256) >= 256) return launch_bwd_pass_nw<T, D, MODE, GRP, 8>(a);
    }
    return launch_bwd_pass_nw<T, D, MODE, GRP, BwdShape<D>::NW>(a);
}

template <typename T, int D, bool GRP>
int launch_bwd_passes(const BwdLaunchArgs &a)
{
    int err;
    if constexpr (BwdShape<D>::FUSED_DKV) {
        err = launch_bwd_pass<T, D, BWD_DKV, GRP>(a);
    } else {
        err = launch_bwd_pass<T, D, BWD_DV, GRP>(a);
        if (err != 0) return err;
        err = launch_bwd_pass<T, D, BWD_DK, GRP>(a);
    }
    if (err != 0) return err;
    return launch_bwd_pass<T, D, BWD_DQ, GRP>(a);
}

template <typename T, int D>
int launch_bwd(const BwdLaunchArgs &a)
{
    const long long rows = (long long)a.BH * a.S;
    const long long threads = (rows + kBwdStatPad) * (D <= 128 ? 16 : 32);
    hipLaunchKernelGGL((sdpa_bwd_prepare_kernel<T, D>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, a.stream,
                       (const T *)a.o, (const T *)a.dout, a.lse, a.delta, a.lse2, rows);
    int err = (int)hipGetLastError();
    if (err != 0) return err;
    // rows that see at most 64 keys get Delta from its definition (see the kernel)
    const int short_rows = a.causal ? (a.S < kBwdShortRow ? a.S : kBwdShortRow) : (a.S <= kBwdShortRow ? a.S : 0);
    if (short_rows > 0) {
        hipLaunchKernelGGL((sdpa_bwd_delta_short_kernel<T, D>), dim3((unsigned)a.BH), dim3(256), 0, a.stream,
                           (const T *)a.q, (const T *)a.k, (const T *)a.v, (const T *)a.dout, a.lse2, a.delta,
                           a.S, short_rows, a.group, a.scale * 1.44269504088896340736f, a.causal);
        err = (int)hipGetLastError();
        if (err != 0) return err;
    }
    // one query head per key/value head keeps the kernels without the loop over a group
    return a.group == 1 ? launch_bwd_passes<T, D, false>(a) : launch_bwd_passes<T, D, true>(a);
}

}  // namespace tsdpa
