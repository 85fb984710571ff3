// Measurement aids: what the matrix pipe of this GPU sustains with nothing else in the way.
// The attention kernel is judged against the published dense MFMA peak; these loops show how much of
// that peak a pure register-resident MFMA stream reaches, and how much the operand DATA matters:
// with random mantissas and signs the chip runs into its power limit and lowers the shader clock,
// with constant operands it does not.  See include/tiled_sdpa.h (tiled_sdpa_probe_mfma).
#include "tiled_sdpa.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kGrid = 512;          // two workgroups of four wavefronts per CU: two wavefronts per SIMD
constexpr int kMfmaPerIter = 64;    // fully unrolled body

__device__ __forceinline__ uint32_t mix(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

template <bool BF16>
__global__ void __launch_bounds__(256) mfma_stream(float *sink, int iters, int random_operands)
{
#if defined(__HIP_DEVICE_COMPILE__)
    // eight A and eight B fragments per lane; exponent fields fixed so nothing overflows
    u32x4 ra[8], rb[8];
    const uint32_t expo = BF16 ? 0x3f003f00u : 0x38003800u;
    const uint32_t keep = BF16 ? 0x807f807fu : 0x83ff83ffu;
#pragma unroll
    for (int f = 0; f < 8; ++f)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t h = mix((blockIdx.x * 256u + threadIdx.x) * 64u + f * 8u + e);
            ra[f][e] = random_operands ? ((h & keep) | expo) : (BF16 ? 0x3f803f80u : 0x3c003c00u);
            rb[f][e] = random_operands ? ((mix(h) & keep) | expo) : (BF16 ? 0x3f803f80u : 0x3c003c00u);
        }
    f32x16 acc[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int f = 0; f < 8; ++f) {
                if constexpr (BF16)
                    acc[f & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ra[f]),
                                                                        __builtin_bit_cast(bf16x8, rb[(f + u) & 7]),
                                                                        acc[f & 3], 0, 0, 0);
                else
                    acc[f & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, ra[f]),
                                                                       __builtin_bit_cast(f16x8, rb[(f + u) & 7]),
                                                                       acc[f & 3], 0, 0, 0);
            }
    }
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[n][i];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
#endif
}

// The same MFMA stream with the other work of the attention kernel's loop mixed in at the kernel's own
// ratios (C4 profile: per MFMA one 16-byte-per-lane LDS operand read and 3.7 vector instructions, a
// quarter of them exponentials), all of it independent of the MFMAs: what the chip sustains for that
// instruction mix when nothing ever waits.  Operands are random as above; the LDS holds random data.
template <bool BF16>
__global__ void __launch_bounds__(256) mfma_mix_stream(float *sink, int iters)
{
#if defined(__HIP_DEVICE_COMPILE__)
    __shared__ __attribute__((aligned(16))) uint32_t tile[4096];      // 16 KiB, one K tile's worth
    for (int i = threadIdx.x; i < 4096; i += 256) tile[i] = mix(i * 977u + blockIdx.x);
    __syncthreads();
    const uint32_t lds_addr = (uint32_t)(size_t)(__attribute__((address_space(3))) uint32_t *)tile + (threadIdx.x & 63) * 16;
    u32x4 ra[8], rb[8];
    const uint32_t expo = BF16 ? 0x3f003f00u : 0x38003800u;
    const uint32_t keep = BF16 ? 0x807f807fu : 0x83ff83ffu;
#pragma unroll
    for (int f = 0; f < 8; ++f)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t h = mix((blockIdx.x * 256u + threadIdx.x) * 64u + f * 8u + e);
            ra[f][e] = (h & keep) | expo;
            rb[f][e] = (mix(h) & keep) | expo;
        }
    f32x16 acc[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
    u32x4 d0 = {0u, 0u, 0u, 0u}, d1 = d0, d2 = d0, d3 = d0;   // landing registers of the LDS reads
    float x0 = 0.3f + (threadIdx.x & 63), x1 = 0.7f, x2 = 1.1f + 0.01f * (threadIdx.x & 63), x3 = 0.1f;   // x0 -> x2 / (1 - x1)
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
#pragma unroll
            for (int r = 0; r < 8; r += 4)            // 8 reads of 1 KiB per 8 MFMAs, walking the tile
                asm volatile("ds_read_b128 %0, %4 offset:%5\n ds_read_b128 %1, %4 offset:%6\n"
                             "ds_read_b128 %2, %4 offset:%7\n ds_read_b128 %3, %4 offset:%8"
                             : "+v"(d0), "+v"(d1), "+v"(d2), "+v"(d3)
                             : "v"(lds_addr), "n"(((u * 8 + r) % 16) * 1024), "n"(((u * 8 + r + 1) % 16) * 1024),
                               "n"(((u * 8 + r + 2) % 16) * 1024), "n"(((u * 8 + r + 3) % 16) * 1024));
#pragma unroll
            for (int f = 0; f < 8; ++f) {
                if constexpr (BF16)
                    acc[f & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ra[f]),
                                                                        __builtin_bit_cast(bf16x8, rb[(f + u) & 7]),
                                                                        acc[f & 3], 0, 0, 0);
                else
                    acc[f & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, ra[f]),
                                                                       __builtin_bit_cast(f16x8, rb[(f + u) & 7]),
                                                                       acc[f & 3], 0, 0, 0);
#pragma unroll
                for (int v = f * 30 / 8; v < (f + 1) * 30 / 8; ++v) {      // 30 vector instructions per 8 MFMAs
                    if ((v & 3) == 0) asm volatile("v_exp_f32 %0, %1" : "+v"(x3) : "v"(x0));
                    else asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x0) : "v"(x1), "v"(x2));
                }
            }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // every read has landed before its register dies
    float s = x0 + x3 + (float)(d0[0] ^ d1[0] ^ d2[0] ^ d3[0]);
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[n][i];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
#endif
}

// Read-only stream: every workgroup walks a contiguous run of 16-byte words, four loads per lane in
// flight, and keeps an XOR of what it read so that the loads cannot be dropped.
constexpr int kReadGrid = 8192;
constexpr int kReadStep = 1024;               // 16-byte words a workgroup reads per loop trip (256 lanes x 4)

__global__ void __launch_bounds__(256)
hbm_read_stream(const uint4 *__restrict__ src, float *__restrict__ sink, int words_per_group)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const uint4 *p = src + (size_t)blockIdx.x * words_per_group;
    uint4 acc = {0u, 0u, 0u, 0u};
    for (int i = threadIdx.x; i < words_per_group; i += kReadStep) {      // words_per_group is a multiple of kReadStep
        const uint4 a = p[i], b = p[i + 256], c = p[i + 512], d = p[i + 768];
        acc.x ^= a.x ^ b.x ^ c.x ^ d.x;
        acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
        acc.z ^= a.z ^ b.z ^ c.z ^ d.z;
        acc.w ^= a.w ^ b.w ^ c.w ^ d.w;
    }
    if (threadIdx.x == 0) sink[blockIdx.x % (512 * 256)] = (float)((acc.x ^ acc.y ^ acc.z ^ acc.w) & 0xFFFFu);
#endif
}

}  // namespace

extern "C" int tiled_sdpa_probe_mfma(int dtype, int random_operands, int iters, float *sink,
                                     double *flops, void *stream)
{
    if (dtype != TSDPA_F16 && dtype != TSDPA_BF16) return TSDPA_ERR_BAD_DTYPE;
    if (iters < 0) return TSDPA_ERR_BAD_SHAPE;
    if (flops) *flops = (double)kGrid * 4.0 * (double)iters * kMfmaPerIter * 32768.0;
    if (iters == 0) return TSDPA_OK;    // nothing is launched, so no sink is needed
    if (!sink) return TSDPA_ERR_NULL_PTR;
    if (random_operands == 2) {
        if (dtype == TSDPA_BF16)
            hipLaunchKernelGGL(mfma_mix_stream<true>, dim3(kGrid), dim3(256), 0, (hipStream_t)stream, sink, iters);
        else
            hipLaunchKernelGGL(mfma_mix_stream<false>, dim3(kGrid), dim3(256), 0, (hipStream_t)stream, sink, iters);
    } else if (dtype == TSDPA_BF16)
        hipLaunchKernelGGL(mfma_stream<true>, dim3(kGrid), dim3(256), 0, (hipStream_t)stream, sink, iters, random_operands);
    else
        hipLaunchKernelGGL(mfma_stream<false>, dim3(kGrid), dim3(256), 0, (hipStream_t)stream, sink, iters, random_operands);
    return hipGetLastError() == hipSuccess ? TSDPA_OK : TSDPA_ERR_LAUNCH;
}

extern "C" int tiled_sdpa_probe_hbm_read(const void *src, unsigned long long bytes, float *sink,
                                         double *bytes_read, void *stream)
{
    if (!src || !sink) return TSDPA_ERR_NULL_PTR;
    if (((uintptr_t)src & 15u) != 0) return TSDPA_ERR_MISALIGNED;
    // whole loop trips only, so that no access needs a bounds check: the tail that does not fill one is not read
    const unsigned long long per_group = bytes / 16 / kReadGrid / kReadStep * kReadStep;
    if (per_group == 0 || per_group > 0x7FFFFFFFull) return TSDPA_ERR_BAD_SHAPE;
    if (bytes_read) *bytes_read = (double)per_group * 16.0 * kReadGrid;
    hipLaunchKernelGGL(hbm_read_stream, dim3(kReadGrid), dim3(256), 0, (hipStream_t)stream,
                       (const uint4 *)src, sink, (int)per_group);
    return hipGetLastError() == hipSuccess ? TSDPA_OK : TSDPA_ERR_LAUNCH;
}
