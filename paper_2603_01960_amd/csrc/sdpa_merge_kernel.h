// Merge of split-KV partial states into the final output.
//
// Each split s of a query row holds the state of the online-softmax recurrence (Section 4.1.2,
// Eqs. 2-4) after its own run of key tiles: a reference m_s (log2 units of the scaled scores), the
// normaliser l_s and the unnormalised output o_s, both taken against m_s.  Because Eqs. 3-4 only ever
// rescale by e^{m_old - m_new}, states over disjoint key ranges combine the same way:
//     M = max_s m_s,   w_s = 2^(m_s - M),   L = sum_s w_s l_s,   O = (sum_s w_s o_s) / L,
// and O_i = o_i / l_i as at the end of Section 4.1.2; LSE = (M + log2 L) ln 2.  A split that saw no
// key of the row has (o, m, l) = (0, -inf, 0) and weight 0.
//
// Workspace layout (written by sdpa_fwd_kernel<..., KV = true>): o as float [BH][splits][S][D],
// then (m, l) pairs as float [BH][splits][S][2].
//
// Two kernels.  sdpa_merge_kernel: one thread produces 4 consecutive output columns and walks the
// splits itself, eight loads in flight at a time; right for up to eight splits, and for any split count
// when the rows are many (a long prefill chunk), where the other threads hide the waiting.
// sdpa_merge_wide_kernel: one workgroup per output row, kMergeLanes threads per column group that
// take every kMergeLanes-th split each and combine through the LDS; for the many splits of a decoding
// step, where rows are few and a walk over 32 splits would be a chain of load latencies longer than
// the attention kernel itself.  Both sum in a fixed order (results do not depend on timing).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tsdpa {

template <typename T>
__global__ void __launch_bounds__(256)
sdpa_merge_kernel(const float *__restrict__ ws, T *__restrict__ o, float *__restrict__ lse,
                  int BH, int S, int D, int splits)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef T vec4 __attribute__((ext_vector_type(4)));
    const int d4n = D / 4;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t rows = (size_t)BH * S;
    if (idx >= rows * d4n) return;
    const size_t r = idx / d4n;                   // bh * S + row
    const int d4 = (int)(idx - r * d4n);
    const size_t bh = r / S, row = r - bh * S;
    const float *ml = ws + rows * splits * D;
    const size_t first = (bh * splits) * S + row; // split s sits s*S rows further on

    // both loops are chains of independent loads: unrolled so that eight of them are in flight at a time
    // (with many splits and few rows this kernel is pure load latency)
    float M = -INFINITY;
#pragma unroll 8
    for (int s = 0; s < splits; ++s) M = fmaxf(M, ml[(first + (size_t)s * S) * 2]);
    float L = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
    for (int s = 0; s < splits; ++s) {
        const size_t p = first + (size_t)s * S;
        // 0 for a split with m = -inf; M itself is -inf only for a row that no key reaches (an empty
        // cache entry, or a causal limit before the first key): all weights 0, O = 0, LSE = -inf
        const float w = M == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ml[p * 2] - M);
        L += w * ml[p * 2 + 1];
        const f32x4 part = *(const f32x4 *)(ws + p * D + d4 * 4);
        acc += w * part;
    }
    const float inv = L > 0.f ? 1.0f / L : 0.f;
    vec4 out;
#pragma unroll
    for (int e = 0; e < 4; ++e) out[e] = (T)(acc[e] * inv);
    *(vec4 *)(o + r * D + d4 * 4) = out;
    if (lse != nullptr && d4 == 0)
        lse[r] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * 0.69314718055994530942f : -INFINITY;
#endif
}

constexpr int kMergeLanes = 8;                  // threads that share one column group's splits
constexpr int kMergePerLane = 16;               // splits per such thread: 8 * 16 = TSDPA_MAX_SPLITS
constexpr int kMergeMaxCols = 40;               // D / 4 at D = 160

// blockDim = (D / 4, kMergeLanes); gridDim.x = BH * S rows.
template <typename T>
__global__ void __launch_bounds__(kMergeMaxCols * kMergeLanes)
sdpa_merge_wide_kernel(const float *__restrict__ ws, T *__restrict__ o, float *__restrict__ lse,
                       int BH, int S, int D, int splits)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef T vec4 __attribute__((ext_vector_type(4)));
    __shared__ f32x4 acc_sh[kMergeLanes][kMergeMaxCols];
    __shared__ f32x2 ml_sh[kMergeLanes];
    const int d4 = threadIdx.x, lane = threadIdx.y;
    const size_t rows = (size_t)BH * S;
    const size_t r = blockIdx.x;                  // bh * S + row
    const size_t bh = r / S, row = r - bh * S;
    const float *ml = ws + rows * splits * D;
    const size_t first = (bh * splits) * S + row; // split s sits s*S rows further on

    // every load of this thread is issued before anything waits: splits lane, lane + 8, ...
    f32x2 st[kMergePerLane];
    f32x4 part[kMergePerLane];
#pragma unroll
    for (int i = 0; i < kMergePerLane; ++i) {
        const int s = lane + i * kMergeLanes;
        st[i] = f32x2{-INFINITY, 0.f};
        part[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (s < splits) {
            const size_t p = first + (size_t)s * S;
            st[i] = *(const f32x2 *)(ml + p * 2);
            part[i] = *(const f32x4 *)(ws + p * D + d4 * 4);
        }
    }
    // this thread's splits combined against their own maximum
    float m_own = -INFINITY;
#pragma unroll
    for (int i = 0; i < kMergePerLane; ++i) m_own = fmaxf(m_own, st[i][0]);
    float l_own = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < kMergePerLane; ++i) {
        // weight 0 for a split with m = -inf (it saw no key of the row, or does not exist)
        const float w = st[i][0] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(st[i][0] - m_own);
        l_own += w * st[i][1];
        acc += w * part[i];
    }
    acc_sh[lane][d4] = acc;
    if (d4 == 0) ml_sh[lane] = f32x2{m_own, l_own};
    __syncthreads();
    if (lane != 0) return;
    // the kMergeLanes states of this column group, in lane order
    float M = -INFINITY;
#pragma unroll
    for (int y = 0; y < kMergeLanes; ++y) M = fmaxf(M, ml_sh[y][0]);
    float L = 0.f;
    f32x4 out_acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int y = 0; y < kMergeLanes; ++y) {
        const float w = ml_sh[y][0] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ml_sh[y][0] - M);
        L += w * ml_sh[y][1];
        out_acc += w * acc_sh[y][d4];
    }
    // M is -inf only for a row that no key reaches: all weights 0, O = 0, LSE = -inf
    const float inv = L > 0.f ? 1.0f / L : 0.f;
    vec4 out;
#pragma unroll
    for (int e = 0; e < 4; ++e) out[e] = (T)(out_acc[e] * inv);
    *(vec4 *)(o + r * D + d4 * 4) = out;
    if (lse != nullptr && d4 == 0)
        lse[r] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * 0.69314718055994530942f : -INFINITY;
#endif
}

}  // namespace tsdpa
