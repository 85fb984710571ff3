// Tiled SDPA forward kernel for gfx950 (MI355X): Eq. 1 of the paper evaluated with the
// online-softmax recurrence of Section 4.1.2 (Eqs. 2-4), FP32 accumulation (Section 4.1.3).
//
// Work split (Section 4.1.2: one workgroup per block of T_M query rows, K/V streamed in
// tiles of T_N rows):
//   * a workgroup has NW wavefronts; each wavefront owns 32 query rows (T_M = 32*NW) and keeps
//     its Q rows in registers as MFMA B-operands for the whole loop;
//   * K and V tiles are staged global -> registers -> LDS, double buffered, one barrier per tile;
//     K runs one tile ahead of V so the scores of tile j+1 (matrix pipe) overlap the softmax of
//     tile j (vector ALU) inside every wavefront;
//   * scores are computed TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16: in the 32x32
//     accumulator layout a lane then owns ONE query column and 16 of the 32 key rows, so the row
//     maximum / sum of Eqs. 2-3 are in-lane reductions plus one exchange with lane^32, and m, l and
//     the rescale factor are per-lane scalars;
//   * O^T = V^T P^T: P^T is taken straight from the score accumulators as the MFMA B-operand (the
//     k-slot <-> key-row permutation this implies is mirrored on the A side), and V^T is fetched
//     from the row-major V tile in LDS with the transposing read ds_read_b64_tr_b16;
//   * exp is v_exp_f32 on (s*c - m) with c = |scale|*log2(e); a negative scale is folded into the
//     sign of Q so the running maximum is always a maximum.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace tsdpa {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef short i16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define TSDPA_LDS __attribute__((address_space(3)))
typedef TSDPA_LDS unsigned char *lds_ptr;

template <typename T> struct Elem;
template <> struct Elem<_Float16> {
    using vec8 = f16x8;
    using vec4 = f16x4;
    static __device__ __forceinline__ f32x16 mfma(vec8 a, vec8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};
template <> struct Elem<__bf16> {
    using vec8 = bf16x8;
    using vec4 = bf16x4;
    static __device__ __forceinline__ f32x16 mfma(vec8 a, vec8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};

__device__ __forceinline__ u32x4 lds_read128(lds_ptr p) { return *(TSDPA_LDS u32x4 *)p; }
__device__ __forceinline__ void lds_write128(lds_ptr p, u32x4 x) { *(TSDPA_LDS u32x4 *)p = x; }
// 16 lanes x 4 consecutive 16-bit values, transposed across the 16 lanes: lane i receives, as
// element e, the value that lane 4*e + i/4 addressed at position i%4.
__device__ __forceinline__ i16x4 lds_read_tr16(lds_ptr p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((TSDPA_LDS i16x4 *)p);
}

// Exchange between lane and lane^32 with v_permlane32_swap: for operands (a, b) the instruction
// leaves {a[0:31], b[0:31]} in the first and {a[32:63], b[32:63]} in the second result, so with
// a == b == x every lane ends up holding both its own and its partner's x.  The two results are
// copied to scalars before the bit casts (a bit cast applied to a vector-element expression reads
// element 0 whatever the index).
__device__ __forceinline__ float pair_max(float x) {
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const u32x2 r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const uint32_t r0 = r[0], r1 = r[1];
    return fmaxf(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));
}
__device__ __forceinline__ float pair_sum(float x) {
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const u32x2 r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const uint32_t r0 = r[0], r1 = r[1];
    return __builtin_bit_cast(float, r0) + __builtin_bit_cast(float, r1);
}

// LDS geometry shared by host (dynamic LDS size) and device.
template <int D, int TN> struct TileGeom {
    static constexpr int KS = D * 2 + 16;  // K row stride (bytes): +4 banks per row -> 128-bit row reads spread
    static constexpr int VS = D * 2 + 64;  // V row stride: 4 consecutive rows x 64 B tile the 64 banks (tr reads)
    static constexpr int KBYTES = TN * KS;
    static constexpr int VBYTES = TN * VS;
    static constexpr int LDS_BYTES = 2 * (KBYTES + VBYTES);   // two K slots, then two V slots
};

// Workgroup -> (head, query tile).  Hardware deals consecutive workgroup ids round-robin over the
// 8 XCDs (each with its own L2).  Regroup so that each XCD walks a contiguous range of
// (head, tile) pairs: the workgroups resident on one XCD then share one head's K/V in that L2.
__device__ __forceinline__ int remap_workgroup(int id, int N, bool linear) {
    if (linear) return id;
    const int x = id & 7, y = id >> 3;
    const int base = N >> 3, rem = N & 7;
    return x * base + (x < rem ? x : rem) + y;
}

template <typename T, int D, int NW, int TN, int WPS>
__global__ void __launch_bounds__(NW * 64, WPS)  // WPS = wavefronts per SIMD the register budget is sized for
sdpa_fwd_kernel(const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v,
                T *__restrict__ o, float *__restrict__ lse, int S, int nQ, int N, float c,
                float tau, uint32_t qsign, int linear_grid)
{
    using E = Elem<T>;
    using vec8 = typename E::vec8;
    using vec4 = typename E::vec4;
    using G = TileGeom<D, TN>;
    constexpr int NT = NW * 64, TM = NW * 32;
    constexpr int CPR = D / 8;            // 16-byte chunks per row
    constexpr int NLD = TN * CPR / NT;    // chunks per thread per tensor per tile
    static_assert(NLD >= 1 && (TN * CPR) % NT == 0, "tile does not divide over the workgroup");
    constexpr int NB = TN / 32, KK = D / 16, DB = D / 32;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const lds_ptr lds = (lds_ptr)smem;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, l32 = lane & 31;

    const int wg = remap_workgroup(blockIdx.x, N, linear_grid != 0);
    const int head = wg / nQ, qt = wg - head * nQ;
    const size_t head_off = (size_t)head * (size_t)S * D;
    const T *qh = q + head_off, *kh = k + head_off, *vh = v + head_off;

    // ---- Q rows of this wavefront as MFMA B-operands: lane holds Q[row l32][kk*16 + g*8 .. +7]
    const int qrow = qt * TM + wave * 32 + l32;
    const int qrow_c = qrow < S ? qrow : S - 1;
    vec8 qf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        u32x4 raw = *(const u32x4 *)(qh + (size_t)qrow_c * D + kk * 16 + g * 8);
        raw ^= qsign;
        qf[kk] = __builtin_bit_cast(vec8, raw);
    }

    const int nT = (S + TN - 1) / TN;

    // ---- staging of one [TN x D] tile: HBM -> registers (128-bit, coalesced) -> LDS rows
    struct Stage { u32x4 r[NLD]; };
    auto load_tile = [&](const T *base, int j, Stage &st) {
#pragma unroll
        for (int it = 0; it < NLD; ++it) {
            const int ci = tid + it * NT;
            const int row = ci / CPR, cc = ci % CPR;
            int key = j * TN + row;
            key = key < S ? key : S - 1;   // rows past S re-read the last row: finite data, masked later
            st.r[it] = *(const u32x4 *)(base + (size_t)key * D + cc * 8);
        }
    };
    auto store_tile = [&](lds_ptr dst, int stride, const Stage &st) {
#pragma unroll
        for (int it = 0; it < NLD; ++it) {
            const int ci = tid + it * NT;
            const int row = ci / CPR, cc = ci % CPR;
            lds_write128(dst + row * stride + cc * 16, st.r[it]);
        }
    };
    auto kslot = [&](int j) { return lds + (j & 1) * G::KBYTES; };
    auto vslot = [&](int j) { return lds + 2 * G::KBYTES + (j & 1) * G::VBYTES; };

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    // Online-softmax state (Eqs. 2-4), all in the log2 domain of s*c.  m_ref is the reference the
    // exponentials are taken against: it is raised to the tile maximum only when that exceeds it by
    // more than tau (tau = 0 is Eq. 2 literally).  With a stale reference the weights are merely
    // scaled by a common factor <= 2^tau per row, which cancels in o/l and in m_ref + log2(l).
    float m_ref = -INFINITY;
    float l_run = 0.f;         // this lane's share of the normaliser (lane^32 holds the rest)

    // per-lane constant parts of the LDS read addresses
    const int k_lane_off = l32 * G::KS + g * 16;
    const int v_lane_off = (g * 4 + ((lane & 15) >> 2)) * G::VS + (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;

    // scores, transposed: sacc[nb][i] = <k_row, q_col>, row = nb*32 + (i/4)*8 + g*4 + i%4, col = l32
    auto scores = [&](lds_ptr kb, f32x16 (&sacc)[NB]) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[nb][i] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                u32x4 raw = lds_read128(kb + k_lane_off + nb * 32 * G::KS + kk * 32);
                sacc[nb] = E::mfma(__builtin_bit_cast(vec8, raw), qf[kk], sacc[nb]);
            }
        }
    };

    // Eqs. 2-3 on one tile of scores; leaves the 16-bit weights (MFMA B-operands) in pb
    auto softmax = [&](f32x16 (&sacc)[NB], int j, vec8 (&pb)[NB][2], auto tail_tag) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        const int key0 = j * TN + g * 4;
        if constexpr (TAIL) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (key0 + nb * 32 + (i >> 2) * 8 + (i & 3) >= S) sacc[nb][i] = -INFINITY;
        }
        float mx = sacc[0][0];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[nb][i]);
        mx = pair_max(mx);
        const float m_tile = mx * c;
        const bool grow = m_tile > m_ref + tau;     // always true on the first tile (m_ref = -inf)
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {  // wavefront-uniform: rescale only when some row needs it
            const float m_new = grow ? m_tile : m_ref;
            const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);   // exactly 1 for rows that keep m_ref
            m_ref = m_new;
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
        }
        // p = 2^(s*c - m_ref); Eq. 3 sums the unrounded FP32 p, the PV product uses the 16-bit rounded p
        float psum = 0.f;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[nb][i], c, -m_ref));
                if constexpr (TAIL) {
                    if (key0 + nb * 32 + (i >> 2) * 8 + (i & 3) >= S) p = 0.f;
                }
                psum += p;
                pb[nb][i >> 3][i & 7] = (T)p;
            }
        l_run += psum;
    };

    // Eq. 4: O^T += V^T P^T
    auto accumulate = [&](lds_ptr vb, const vec8 (&pb)[NB][2]) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    // k-slots 0..3 / 4..7 of this lane <-> key rows base+g*4+0..3 / base+8+g*4+0..3
                    const lds_ptr p0 = vb + v_lane_off + (nb * 32 + ks * 16) * G::VS + db * 64;
                    i16x4 lo = lds_read_tr16(p0);
                    i16x4 hi = lds_read_tr16(p0 + 8 * G::VS);
                    i16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    oacc[db] = E::mfma(__builtin_bit_cast(vec8, a), pb[nb][ks], oacc[db]);
                }
    };

    // ---- software pipeline.  K runs one tile ahead of V: while the VALU does the softmax of tile j,
    // the matrix pipe already computes the scores of tile j+1.  In iteration j the LDS holds K(j+1)
    // and V(j); K(j+2) and V(j+1) travel HBM -> registers and are written to the slots that K(j) and
    // V(j-1) occupied, whose last readers finished before the barrier that ended iteration j-1.
    Stage sk, sv;
    load_tile(kh, 0, sk);
    load_tile(vh, 0, sv);
    store_tile(kslot(0), G::KS, sk);
    store_tile(vslot(0), G::VS, sv);
    if (nT > 1) {
        load_tile(kh, 1, sk);
        store_tile(kslot(1), G::KS, sk);
    }
    __syncthreads();
    f32x16 s_cur[NB], s_nxt[NB];
    vec8 pb[NB][2];
    scores(kslot(0), s_cur);
    __syncthreads();   // iteration 0 overwrites K slot 0: every wavefront must have read it first
    for (int j = 0; j + 1 < nT; ++j) {
        const int jk = j + 2 < nT ? j + 2 : nT - 1;   // past the end: reload the last tile (never read)
        load_tile(kh, jk, sk);
        load_tile(vh, j + 1, sv);
        scores(kslot(j + 1), s_nxt);
        softmax(s_cur, j, pb, std::false_type{});
        accumulate(vslot(j), pb);
        store_tile(kslot(j + 2), G::KS, sk);
        store_tile(vslot(j + 1), G::VS, sv);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) s_cur[nb] = s_nxt[nb];
        __syncthreads();
    }
    if (nT * TN != S)
        softmax(s_cur, nT - 1, pb, std::true_type{});
    else
        softmax(s_cur, nT - 1, pb, std::false_type{});
    accumulate(vslot(nT - 1), pb);

    // ---- O_i = o_i / l_i (Section 4.1.2), rounded once to the 16-bit output type
    const float l_tot = pair_sum(l_run);
    const float inv = 1.0f / l_tot;
    if (qrow < S) {
        T *orow = o + head_off + (size_t)qrow * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                vec4 out;
#pragma unroll
                for (int e = 0; e < 4; ++e) out[e] = (T)(oacc[db][q4 * 4 + e] * inv);
                *(vec4 *)(orow + db * 32 + q4 * 8 + g * 4) = out;
            }
        if (lse != nullptr && g == 0)
            lse[(size_t)head * S + qrow] = (m_ref + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
    }
}

}  // namespace tsdpa
