// Tiled SDPA forward kernel for gfx950 (MI355X): Eq. 1 of the paper evaluated with the
// online-softmax recurrence of Section 4.1.2 (Eqs. 2-4), FP32 accumulation (Section 4.1.3).
//
// Work split (Section 4.1.2: one workgroup per block of T_M query rows, K/V streamed in
// tiles of T_N rows):
//   * a workgroup has NW wavefronts; each wavefront owns 32 query rows (T_M = 32*NW) and keeps
//     its Q rows in registers as MFMA B-operands for the whole loop;
//   * K and V tiles go HBM -> LDS directly (buffer_load_dwordx4 ... lds: no staging registers, no
//     LDS write instructions), double buffered, one barrier per tile.  Such a load writes 64 lanes x
//     16 B contiguously, so rows cannot be padded; bank conflicts are avoided by an XOR swizzle of
//     the 16-byte chunks within each row, applied through the choice of the global address each
//     lane fetches.  Rows past S are never fetched: the buffer descriptor's range check returns 0;
//   * K runs one tile ahead of V so the scores of tile j+1 (matrix pipe) overlap the softmax of
//     tile j (vector ALU) inside every wavefront.  The overlap is written out by hand: a step is a
//     sequence of slots, one MFMA each, with that slot's share of the exponentials / maxima and the
//     LDS reads of a later slot, fenced so the compiler keeps the order (two wavefronts of a SIMD that
//     run matrix and vector phases in lockstep do not overlap by themselves: issue is in order);
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
#include <utility>

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
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

template <> struct Elem<_Float16> {
    using vec8 = f16x8;
    using vec4 = f16x4;
    using vec2 = f16x2;

    static __device__ __forceinline__ f32x16 mfma(vec8 a, vec8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};
template <> struct Elem<__bf16> {
    using vec8 = bf16x8;
    using vec4 = bf16x4;
    using vec2 = bf16x2;

    static __device__ __forceinline__ f32x16 mfma(vec8 a, vec8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};

__device__ __forceinline__ u32x4 lds_read128(lds_ptr p) { return *(TSDPA_LDS u32x4 *)p; }
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

// LDS geometry shared by host (dynamic LDS size) and device.  A tile is TN rows of D 16-bit values,
// unpadded; within a row the 16-byte chunks are XOR-swizzled:
//   K: chunk c of row r sits at c ^ kswz(r).  The score MFMA's A-operand read has 16 lanes fetch the
//      same chunk of 16 consecutive rows; the swizzle spreads them over all 64 banks.
//   V: 64-byte block b of row r sits at b ^ vswz(r).  The transposing read has 32 lanes fetch one
//      64-byte block of 4 consecutive rows; the swizzle puts those on 4 x 16 distinct banks.
// NS slots per tensor form a ring: tile j lives in slot j % NS.
template <int D, int TN, int NS> struct TileGeom {
    static constexpr int ROW = D * 2;               // bytes per row
    static constexpr int TILE = TN * ROW;           // bytes per K or V tile
    static constexpr int LDS_BYTES = 2 * NS * TILE; // K slots 0..NS-1, then V slots 0..NS-1
    static __host__ __device__ constexpr int kswz(int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); }
    static __host__ __device__ constexpr int vswz(int r) { return D == 128 ? (r & 3) : ((r >> 1) & 1); }
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

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F> __device__ __forceinline__ void static_for(F &&f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Order of the matrix instructions of one pipeline step and where the vector work sits between them.
// A slot is one operand fragment fetched from LDS and the QB MFMAs (one per 32-row query block of the
// wavefront) that consume it.
//   QK q (q = kk*NB + nb): scores of the NEXT tile, accumulator nb, depth slice kk.
//   PV p (p = group*DB + db, group = nb*2 + ks): output block db += V^T P^T over the 16 keys of group.
// The step starts with half of the QK slots, then alternates PV groups with the remaining QK chunks,
// so the exponentials (needed group by group) can be spread evenly over the whole step.
template <int NB, int KK, int DB, int QB> struct StepSchedule {
    static constexpr int NQK = NB * KK, NG = 2 * NB, NPV = NG * DB, NM = NQK + NPV;
    static constexpr int H = NQK / 2, Q = NQK / NG;
    static constexpr int NPAIR = 8 * NB * QB;   // pairs of weights per lane per tile, ordered (group, qb, e2)
    static constexpr int NMAX = 8 * NB;         // v_max3 operations for one query block's tile maximum
    struct Op { int pv; int idx; };
    static constexpr Op op(int t) {
        if (t < H) return {0, t};
        int u = t - H, qk = H;
        for (int gi = 0; gi < NG; ++gi) {
            if (u < DB) return {1, gi * DB + u};
            u -= DB;
            if (gi < NG / 2) {
                if (u < Q) return {0, qk + u};
                u -= Q;
                qk += Q;
            }
        }
        return {-1, -1};
    }
    static constexpr int first_pv_slot(int gi) { return H + gi * DB + (gi < NG / 2 ? gi : NG / 2) * Q; }
    static constexpr int last_qk_slot() {
        int last = 0;
        for (int t = 0; t < NM; ++t) if (op(t).pv == 0) last = t;
        return last;
    }
    // slot in which pair pr of the exponentials is computed: the pairs of group gi are spread evenly
    // over the slots from the first PV slot of group gi-1 up to the slot before their own PV
    static constexpr int pair_slot(int pr) {
        const int gi = pr / (4 * QB), r = pr % (4 * QB);
        const int lo = gi == 0 ? 0 : first_pv_slot(gi - 1), hi = first_pv_slot(gi) - 1;
        return lo + r * (hi - lo + 1) / (4 * QB);
    }
    // first slot that may read the finished scores of the next tile, and v_max3 operations per slot
    static constexpr int max_first_slot() { return last_qk_slot() + 2 < NM ? last_qk_slot() + 2 : NM; }
    static constexpr int max_per_slot() {
        return NM - max_first_slot() > 0 ? (NMAX + (NM - max_first_slot()) - 1) / (NM - max_first_slot()) : NMAX;
    }
    static constexpr bool valid() {
        for (int gi = 0; gi < NG; ++gi)
            if (pair_slot((gi + 1) * 4 * QB - 1) >= first_pv_slot(gi)) return false;   // weights ready before their PV
        int nqk = 0, npv = 0;
        for (int t = 0; t < NM; ++t) {
            if (op(t).pv == 0) { if (op(t).idx != nqk) return false; ++nqk; }
            else if (op(t).pv == 1) { if (op(t).idx != npv) return false; ++npv; }
            else return false;
        }
        return nqk == NQK && npv == NPV;
    }
};

// s_waitcnt vmcnt(n) with the other counters left at their maxima (gfx9 encoding: vmcnt is split
// over bits 3:0 and 15:14)
#define TSDPA_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt((((n) & 15) | (((n) >> 4) << 14)) | 0x0F70)
// nothing is scheduled across this point
#define TSDPA_FENCE() __builtin_amdgcn_sched_barrier(0)

// T: element type; D: head dim; NW wavefronts per workgroup; QB 32-row query blocks per wavefront
// (T_M = 32*NW*QB); TN key/value rows per tile; NS LDS ring slots per tensor; WPS wavefronts per SIMD
// the register budget is sized for.
template <typename T, int D, int NW, int QB, int TN, int NS, int WPS>
__global__ void __launch_bounds__(NW * 64, WPS)
sdpa_fwd_kernel(const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v,
                T *__restrict__ o, float *__restrict__ lse, int S, int nQ, int N, float c,
                float tau, uint32_t qsign, int linear_grid)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses device-only types
    using E = Elem<T>;
    using vec8 = typename E::vec8;
    using vec4 = typename E::vec4;
    using vec2 = typename E::vec2;
    using G = TileGeom<D, TN, NS>;
    constexpr int WROWS = 32 * QB, TM = NW * WROWS;
    constexpr int CPR = D / 8;                    // 16-byte chunks per row
    constexpr int NLD = TN * CPR / (NW * 64);     // direct-to-LDS load instructions per wavefront per tile
    static_assert(NLD >= 1 && (TN * CPR) % (NW * 64) == 0, "tile does not divide over the workgroup");
    static_assert(NS >= 2, "need at least a double buffer");
    constexpr int NB = TN / 32, KK = D / 16, DB = D / 32;
    using Sch = StepSchedule<NB, KK, DB, QB>;
    static_assert(Sch::valid(), "step schedule violates a dependency");
    constexpr int PF = 3;                         // LDS operand reads run this many slots ahead
    constexpr int RING = PF + 1;
    // loads that may stay in flight across the barrier that ends a step: those of the NS-2 latest steps
    constexpr int INFLIGHT = 2 * NLD * (NS - 2);
    static_assert(INFLIGHT < 64, "vmcnt is a 6-bit counter");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const lds_ptr lds = (lds_ptr)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, l32 = lane & 31;

    const int wg = remap_workgroup(blockIdx.x, N, linear_grid != 0);
    const int head = wg / nQ, qt = wg - head * nQ;
    const size_t head_off = (size_t)head * (size_t)S * D;
    const T *qh = q + head_off;

    // ---- Q rows of this wavefront as MFMA B-operands: lane holds Q[row qb*32 + l32][kk*16 + g*8 .. +7]
    int qrow[QB];
    vec8 qf[QB][KK];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        qrow[qb] = qt * TM + wave * WROWS + qb * 32 + l32;
        const int qrow_c = qrow[qb] < S ? qrow[qb] : S - 1;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            u32x4 raw = *(const u32x4 *)(qh + (size_t)qrow_c * D + kk * 16 + g * 8);
            raw ^= qsign;
            qf[qb][kk] = __builtin_bit_cast(vec8, raw);
        }
    }

    const int nT = (S + TN - 1) / TN;
    const bool ragged = nT * TN != S;

    // ---- K/V tiles: HBM -> LDS.  One buffer descriptor per tensor covers exactly this head's S rows,
    // so a row index >= S reads as zeros instead of touching memory.  Load instruction `it` of this
    // wavefront fills LDS chunks [(it*NW + wave)*64, +64) of the tile; lane `lane` fills chunk p of
    // that range and therefore fetches the global chunk that the swizzle maps to position p.
    const auto k_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(k + head_off), (short)0, S * G::ROW, 0x00020000);
    const auto v_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(v + head_off), (short)0, S * G::ROW, 0x00020000);
    int k_goff[NLD], v_goff[NLD];
#pragma unroll
    for (int it = 0; it < NLD; ++it) {
        const int p = (it * NW + wave) * 64 + lane;
        const int r = p / CPR, cp = p % CPR;
        k_goff[it] = r * G::ROW + ((cp ^ G::kswz(r)) << 4);
        v_goff[it] = r * G::ROW + ((cp ^ (G::vswz(r) << 2)) << 4);
    }
    // tile j -> ring slot j % NS; byte offsets of the K ring and the V ring
    auto load_tile = [&](decltype(k_rsrc) rsrc, const int (&goff)[NLD], int j, int slot_byte) {
        const int soff = j * G::TILE;     // wavefront-uniform; rows >= S fall outside the descriptor
#pragma unroll
        for (int it = 0; it < NLD; ++it)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (TSDPA_LDS void *)(lds + slot_byte + (it * NW + wave) * 1024),
                                                     16, goff[it], soff, 0, 0);
    };
    auto k_slot = [&](int j) { return (j % NS) * G::TILE; };
    auto v_slot = [&](int j) { return (NS + j % NS) * G::TILE; };

    f32x16 oacc[QB][DB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[qb][db][i] = 0.f;
    // Online-softmax state (Eqs. 2-4) per query block, all in the log2 domain of s*c.  m_ref is the
    // reference the exponentials are taken against: it is raised to the tile maximum only when that
    // exceeds it by more than tau (tau = 0 is Eq. 2 literally).  With a stale reference the weights are
    // merely scaled by a common factor <= 2^tau per row, which cancels in o/l and in m_ref + log2(l).
    float m_ref[QB], l_even[QB], l_odd[QB];   // l: this lane's share of the normaliser, in two partial sums
    float m_tile[QB];                         // maximum of the tile about to be consumed
    bool grow[QB];                            // ... and whether it forces m_ref up
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_ref[qb] = -INFINITY;
        l_even[qb] = l_odd[qb] = 0.f;
        m_tile[qb] = -INFINITY;
        grow[qb] = false;
    }

    // ---- per-lane LDS read addresses within a tile (loop invariant; nb, group enter as immediates)
    // K: row l32 (+32*nb), chunk (2*kk + g) ^ kswz(row)
    int k_roff[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) k_roff[kk] = l32 * G::ROW + (((2 * kk + g) ^ G::kswz(l32)) << 4);
    // V (transposing read): row g*4 + (lane%16)/4 (+ multiples of 8), 64-byte block db ^ vswz(row),
    // then 32 B for the upper 16 lanes of each 32 and 8 B per lane%4
    const int v_row = g * 4 + ((lane & 15) >> 2);
    int v_roff[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
        v_roff[db] = v_row * G::ROW + ((db ^ G::vswz(v_row)) << 6) + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;

    // operand fetches from the tile at byte address `base` (ring slot + per-lane offset, per step).
    // K fragment for QK q: rows nb*32 + l32, depth slice kk.  V fragment for PV p: k-slots 0..3 / 4..7 of
    // this lane <-> key rows base+g*4+0..3 / base+8+g*4+0..3 (base = 16*group), which is exactly where
    // the score accumulator layout put the matching weights.
    auto read_k = [&](const int (&kaddr)[KK], int qidx) -> u32x4 {
        const int kk = qidx / NB, nb = qidx % NB;
        return lds_read128(lds + kaddr[kk] + nb * 32 * G::ROW);
    };
    auto read_v = [&](const int (&vaddr)[DB], int pidx) -> u32x4 {
        const int gi = pidx / DB, db = pidx % DB;
        const lds_ptr p0 = lds + vaddr[db] + gi * 16 * G::ROW;
        const i16x4 lo = lds_read_tr16(p0);
        const i16x4 hi = lds_read_tr16(p0 + 8 * G::ROW);
        const i16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(u32x4, a);
    };

    // weights of one pair of score elements: p = 2^(s*c - m_ref).  The normaliser (Eq. 3) sums the
    // unrounded FP32 p; the PV product takes p rounded to the 16-bit type.
    // pr = (group*QB + qb)*4 + e2, group = nb*2 + ks <-> accumulator elements ks*8 + 2*e2, +1 of block nb.
    auto weight_pair = [&](f32x16 (&sacc)[QB][NB], vec8 (&pb)[QB][NB][2], int pr, bool tail, int j) {
        const int gi = pr / (4 * QB), qb = (pr / 4) % QB, e2 = pr & 3;
        const int nb = gi / 2, ks = gi % 2;
        const int i0 = ks * 8 + 2 * e2;
        float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[qb][nb][i0], c, -m_ref[qb]));
        float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[qb][nb][i0 + 1], c, -m_ref[qb]));
        if (tail) {
            const int key = j * TN + g * 4 + nb * 32 + (i0 >> 2) * 8 + (i0 & 3);
            if (key >= S) p0 = 0.f;
            if (key + 1 >= S) p1 = 0.f;
        }
        const vec2 pp = {(T)p0, (T)p1};
        pb[qb][nb][ks][2 * e2] = pp[0];
        pb[qb][nb][ks][2 * e2 + 1] = pp[1];
        l_even[qb] += p0;
        l_odd[qb] += p1;
    };

    // Eq. 2, first half: maximum of one tile of scores (log2 domain) and whether it forces m_ref up.
    auto mask_tail = [&](f32x16 (&sacc)[QB][NB], int j) {
        const int key0 = j * TN + g * 4;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (key0 + nb * 32 + (i >> 2) * 8 + (i & 3) >= S) sacc[qb][nb][i] = -INFINITY;
    };
    auto full_max = [&](f32x16 (&sacc)[QB][NB], float (&mx)[QB]) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx[qb] = fmaxf(mx[qb], sacc[qb][nb][i]);
    };
    auto finish_max = [&](float (&mx)[QB]) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            m_tile[qb] = pair_max(mx[qb]) * c;
            grow[qb] = m_tile[qb] > m_ref[qb] + tau;     // always true on the first tile (m_ref = -inf)
        }
    };
    // Eq. 2, second half, with the rescale of Eqs. 3-4: runs at the start of the step that consumes the
    // tile, after the previous tile's PV product has been issued.  Wavefront-uniform branch, rarely taken.
    auto raise_reference = [&]() {
        bool any = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) any = any || grow[qb];
        if (__builtin_amdgcn_ballot_w64(any) != 0) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const float m_new = grow[qb] ? m_tile[qb] : m_ref[qb];
                const float alpha = __builtin_amdgcn_exp2f(m_ref[qb] - m_new);   // exactly 1 for rows that keep m_ref
                m_ref[qb] = m_new;
                l_even[qb] *= alpha;
                l_odd[qb] *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[qb][db][i] *= alpha;
            }
        }
    };

    f32x16 s_a[QB][NB], s_b[QB][NB];
    vec8 pb[QB][NB][2];
    int kaddr[KK], vaddr[DB];
    auto set_read_slots = [&](int kbyte, int vbyte) {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kaddr[kk] = k_roff[kk] + kbyte;
#pragma unroll
        for (int db = 0; db < DB; ++db) vaddr[db] = v_roff[db] + vbyte;
    };

    // ---- one pipeline step.  On entry the LDS holds K(j+1) and V(j) (and later tiles already landed
    // or in flight); the step issues the loads of K(j+NS) and V(j+NS-1) into the slots that K(j) and
    // V(j-1) occupied, whose last readers finished before the barrier that ended step j-1.
    // `cur` holds the scores of tile j, `nxt` receives those of tile j+1.
    auto step = [&](int j, f32x16 (&cur)[QB][NB], f32x16 (&nxt)[QB][NB], auto next_tail_tag) {
        constexpr bool NEXT_TAIL = decltype(next_tail_tag)::value; // tile j+1 is the ragged last tile
        raise_reference();
        load_tile(k_rsrc, k_goff, j + NS, k_slot(j + NS));
        load_tile(v_rsrc, v_goff, j + NS - 1, v_slot(j + NS - 1));
        set_read_slots(k_slot(j + 1), v_slot(j));
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int i = 0; i < 16; ++i) nxt[qb][nb][i] = 0.f;
        u32x4 frag[RING];
        auto fetch = [&](auto t_tag) {
            constexpr int t = decltype(t_tag)::value;
            if constexpr (t < Sch::NM) {
                constexpr auto op = Sch::op(t);
                if constexpr (op.pv) frag[t % RING] = read_v(vaddr, op.idx);
                else                 frag[t % RING] = read_k(kaddr, op.idx);
            }
        };
        static_for<PF>([&](auto t) { fetch(t); });
        float mx[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) mx[qb] = -INFINITY;
        TSDPA_FENCE();
        static_for<Sch::NM>([&](auto t_tag) {
            constexpr int t = decltype(t_tag)::value;
            constexpr auto op = Sch::op(t);
            fetch(std::integral_constant<int, t + PF>{});
            const vec8 a = __builtin_bit_cast(vec8, frag[t % RING]);
            if constexpr (op.pv) {
                constexpr int gi = op.idx / DB, db = op.idx % DB;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) oacc[qb][db] = E::mfma(a, pb[qb][gi / 2][gi % 2], oacc[qb][db]);
            } else {
                constexpr int kk = op.idx / NB, nb = op.idx % NB;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) nxt[qb][nb] = E::mfma(a, qf[qb][kk], nxt[qb][nb]);
            }
            static_for<Sch::NPAIR>([&](auto pr_tag) {
                constexpr int pr = decltype(pr_tag)::value;
                if constexpr (Sch::pair_slot(pr) == t) weight_pair(cur, pb, pr, false, j);
            });
            if constexpr (!NEXT_TAIL && t >= Sch::max_first_slot()) {
                constexpr int first = (t - Sch::max_first_slot()) * Sch::max_per_slot();
                static_for<Sch::max_per_slot()>([&](auto u_tag) {
                    constexpr int u = first + decltype(u_tag)::value;
                    if constexpr (u < Sch::NMAX) {
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb)
                            mx[qb] = fmaxf(fmaxf(mx[qb], nxt[qb][u / 8][2 * (u % 8)]), nxt[qb][u / 8][2 * (u % 8) + 1]);
                    }
                });
            }
            TSDPA_FENCE();
        });
        if constexpr (NEXT_TAIL || Sch::max_first_slot() >= Sch::NM) {
            if constexpr (NEXT_TAIL) mask_tail(nxt, j + 1);
            full_max(nxt, mx);
        }
        finish_max(mx);
        TSDPA_WAIT_VMCNT(INFLIGHT);
        __syncthreads();
    };
    // the last tile: weights (masked if ragged) and PV product, nothing to overlap with
    auto last = [&](f32x16 (&cur)[QB][NB]) {
        raise_reference();
        set_read_slots(0, v_slot(nT - 1));
        static_for<Sch::NPAIR>([&](auto pr_tag) { weight_pair(cur, pb, decltype(pr_tag)::value, ragged, nT - 1); });
        static_for<Sch::NPV>([&](auto p_tag) {
            constexpr int pi = decltype(p_tag)::value;
            constexpr int gi = pi / DB, db = pi % DB;
            const vec8 a = __builtin_bit_cast(vec8, read_v(vaddr, pi));
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) oacc[qb][db] = E::mfma(a, pb[qb][gi / 2][gi % 2], oacc[qb][db]);
        });
    };

    // ---- prologue: K(0), V(0), K(1) must have landed; K(2..NS-1), V(1..NS-2) are left in flight so
    // that every step finds the same number of outstanding loads.  Tiles past the end read as zeros.
    load_tile(k_rsrc, k_goff, 0, k_slot(0));
    load_tile(v_rsrc, v_goff, 0, v_slot(0));
    load_tile(k_rsrc, k_goff, 1, k_slot(1));
#pragma unroll
    for (int t = 2; t < NS; ++t) {
        load_tile(v_rsrc, v_goff, t - 1, v_slot(t - 1));
        load_tile(k_rsrc, k_goff, t, k_slot(t));
    }
    TSDPA_WAIT_VMCNT(INFLIGHT);
    __syncthreads();
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) s_a[qb][nb][i] = 0.f;
    set_read_slots(k_slot(0), v_slot(0));
    static_for<Sch::NQK>([&](auto q_tag) {
        constexpr int qi = decltype(q_tag)::value;
        const vec8 a = __builtin_bit_cast(vec8, read_k(kaddr, qi));
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) s_a[qb][qi % NB] = E::mfma(a, qf[qb][qi / NB], s_a[qb][qi % NB]);
    });
    {
        if (nT == 1 && ragged) mask_tail(s_a, 0);
        float mx[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) mx[qb] = -INFINITY;
        full_max(s_a, mx);
        finish_max(mx);
    }
    __syncthreads();   // step 0 overwrites K slot 0: every wavefront must have read it first

    // ---- main loop, unrolled by two so that the two score register sets alternate by name
    int j = 0;
    for (; j + 3 < nT; j += 2) {          // both next tiles are full tiles
        step(j, s_a, s_b, std::false_type{});
        step(j + 1, s_b, s_a, std::false_type{});
    }
    // 1, 2 or 3 tiles left, j even
    if (j + 3 == nT) {
        step(j, s_a, s_b, std::false_type{});
        if (ragged) step(j + 1, s_b, s_a, std::true_type{});
        else        step(j + 1, s_b, s_a, std::false_type{});
        last(s_a);
    } else if (j + 2 == nT) {
        if (ragged) step(j, s_a, s_b, std::true_type{});
        else        step(j, s_a, s_b, std::false_type{});
        last(s_b);
    } else {
        last(s_a);
    }

    // ---- O_i = o_i / l_i (Section 4.1.2), rounded once to the 16-bit output type
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l_tot = pair_sum(l_even[qb] + l_odd[qb]);
        const float inv = 1.0f / l_tot;
        if (qrow[qb] < S) {
            T *orow = o + head_off + (size_t)qrow[qb] * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    vec4 out;
#pragma unroll
                    for (int e = 0; e < 4; ++e) out[e] = (T)(oacc[qb][db][q4 * 4 + e] * inv);
                    *(vec4 *)(orow + db * 32 + q4 * 8 + g * 4) = out;
                }
            if (lse != nullptr && g == 0)
                lse[(size_t)head * S + qrow[qb]] =
                    (m_ref[qb] + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
        }
    }
#endif
}

}  // namespace tsdpa
