// Backward pass of tiled SDPA for gfx950 (MI355X).  The paper leaves it as future work (Section 7);
// what is computed is the derivative of its Eq. 1 (Section 3.1), with P recomputed tile by tile from
// the forward pass's log-sum-exp instead of being stored, in the spirit of Section 4.1.2:
//
//     P_ij  = exp(scale * <q_i, k_j> - LSE_i)          (0 for masked keys)
//     dV_j  = sum_i P_ij dO_i
//     dP_ij = <dO_i, v_j>
//     dS_ij = P_ij (dP_ij - Delta_i),   Delta_i = <dO_i, O_i>   (= sum_j P_ij dP_ij)
//     dQ_i  = scale * sum_j dS_ij k_j,  dK_j = scale * sum_i dS_ij q_i
//
// Three passes over the S x S score plane, all instances of ONE kernel template, so that no sum
// crosses workgroups (no atomics, deterministic results) and every pass fits 256 registers per lane
// (two wavefronts per SIMD):
//   * BWD_DQ: a workgroup owns 32*NW query rows (Q and dO rows in registers), streams K and V tiles;
//   * BWD_DK: a workgroup owns 32*NW key rows (K and V rows in registers), streams Q and dO tiles;
//   * BWD_DV: a workgroup owns 32*NW key rows (K rows in registers), streams Q and dO tiles.
// With R the resident and T the streamed rows, a pass computes, per streamed tile,
//     acc[t][r]  = <T1_t, R1_r>  (scores)        acc2[t][r] = <T2_t, R2_r>  (dP; not in BWD_DV)
//     out^T[d][r] += sum_t T1[t][d] dS[t][r]     (dQ^T or dK^T)
//     out^T[d][r] += sum_t T2[t][d] P[t][r]      (dV^T, BWD_DV)
// (T1, T2, R1, R2) = (K, V, Q, dO) or (Q, dO, K, V).  The scores are thus computed three times and dP
// twice (8 S x S x D products against the 5 of the formulas): the price of keeping dK and dV out of
// one register file.  The MFMA formulation is the forward kernel's:
// transposed accumulators (a lane owns one resident row), P and dS handed to the second product
// straight from the accumulator registers as B-operands, the streamed tile read row-wise for the
// first product and through the transposing LDS read for the second.  Since one LDS tile now serves
// both kinds of read, its 16-byte chunks are XOR-swizzled by a function of the row under which
// both are bank-conflict free (BwdGeom::swz).
#pragma once
#include "sdpa_fwd_kernel.h"
#include "sdpa_fwd_launch.h"

namespace tsdpa {

// LDS geometry of a streamed tile: TS rows of D 16-bit values, rows DG*2 bytes apart (DG = D rounded up
// to a power of two; the chunks past D are never fetched, as in the forward kernel).  Chunk c of row
// r sits at c ^ swz(r).  Row-wise reads have 16 lanes fetch one chunk index of 16 consecutive rows:
// swz is a bijection of the row bits that select the bank group, so they spread over all banks.
// Transposing reads have 32 lanes fetch one 64-byte block (4 chunks) of 4 consecutive rows: bits
// 3:2 of swz (bit 2 when a row has only two blocks) come from the low row bits, so the four rows
// land in different blocks.
template <int D, int TS> struct BwdGeom {
    static_assert(D == 64 || D == 96 || D == 128 || D == 160, "head dims of the paper's grid");
    static constexpr int DG = D <= 64 ? 64 : (D <= 128 ? 128 : 256);   // LDS row geometry: next power of two
    static constexpr int ROW = DG * 2;              // bytes per LDS row
    static constexpr int GROW = D * 2;              // bytes per row in global memory
    static constexpr int TILE = TS * ROW;
    static constexpr int GTILE = TS * GROW;
    static constexpr int STATS = 2 * TS * 4;        // LSE then Delta of a tile's rows (keys-resident passes)
    static constexpr int LDS_BYTES = 4 * TILE + 2 * STATS;   // T1 slots 0,1, T2 slots 0,1, statistics slots 0,1
    static __host__ __device__ constexpr int swz(int r) {
        return DG == 64 ? ((((r >> 1) & 1) << 2) | ((r >> 2) & 3)) : (((r & 3) << 2) | ((r >> 2) & 3));
    }
};

// Delta_i = <dO_i, O_i> and LSE_i in log2 units, one row per group of 16 (D <= 128) or 32 lanes; the
// kBwdStatPad entries after the last row are set to zero.
template <typename T, int D>
__global__ void __launch_bounds__(256)
sdpa_bwd_prepare_kernel(const T *__restrict__ o, const T *__restrict__ dout, const float *__restrict__ lse,
                        float *__restrict__ delta, float *__restrict__ lse2, long long rows)
{
#if defined(__HIP_DEVICE_COMPILE__)
    using vec8 = typename Elem<T>::vec8;
    constexpr int LPR = D <= 128 ? 16 : 32;        // lanes per row; lanes >= D/8 idle
    const long long row = ((long long)blockIdx.x * 256 + threadIdx.x) / LPR;
    const int part = threadIdx.x % LPR;
    float sum = 0.f;
    if (row < rows && part < D / 8) {
        const vec8 a = *(const vec8 *)(o + row * D + part * 8);
        const vec8 b = *(const vec8 *)(dout + row * D + part * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) sum += (float)a[e] * (float)b[e];
    }
#pragma unroll
    for (int w = LPR / 2; w >= 1; w >>= 1) sum += __shfl_xor(sum, w, LPR);
    if (part == 0) {
        if (row < rows) {
            delta[row] = sum;
            lse2[row] = lse[row] * 1.44269504088896340736f;
        } else if (row < rows + kBwdStatPad) {
            delta[row] = 0.f;
            lse2[row] = 0.f;
        }
    }
#endif
}

// Delta_i for the query rows that see at most 64 keys (the first rows under the causal mask; every row of
// a sequence of up to 64), recomputed from its definition  Delta_i = sum_j P_ij dP_ij  in FP32, which
// replaces what sdpa_bwd_prepare_kernel left there.  <dO_i, O_i> equals it only in exact arithmetic: O
// arrives rounded to 16 bits, and the rounding error of the D-term sum goes into dS_ij = P_ij (dP_ij -
// Delta_i) scaled by P_ij, which is of order 1 exactly on such rows (on a row of n comparable keys it is of
// order 1/n).  Rows of more than 64 keys keep the <dO_i, O_i> form.
// One workgroup per query head covers its first 64 rows against its first 64 keys: each of the four
// wavefronts takes a 32-key x 32-query block of the scores and of dP (the forward kernel's transposed MFMA
// formulation, operands straight from global memory), weights and sums its block, and the two key blocks
// of a query meet in the LDS.  (A first form with one wavefront per row and a lane per key took half of a
// causal backward call on short sequences.)
constexpr int kBwdShortRow = 64;

template <typename T, int D>
__global__ void __launch_bounds__(256)
sdpa_bwd_delta_short_kernel(const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v,
                            const T *__restrict__ dout, const float *__restrict__ lse2, float *__restrict__ delta,
                            int S, int rows, int group, float scale_log2, int causal)
{
#if defined(__HIP_DEVICE_COMPILE__)
    using E = Elem<T>;
    using vec8 = typename E::vec8;
    constexpr int KK = D / 16;
    __shared__ float part[2][kBwdShortRow];
    const int head = blockIdx.x;                          // query head
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, l32 = lane & 31;
    const int kb = wave & 1, qb = wave >> 1;              // this wavefront's 32-key block and 32-query block
    const int krow = kb * 32 + l32, qrow = qb * 32 + l32;
    // rows past the end are read as the last row and left out of the sums below
    const size_t kbase = ((size_t)(head / group) * S + (krow < S ? krow : S - 1)) * D + g * 8;
    const size_t qbase = ((size_t)head * S + (qrow < S ? qrow : S - 1)) * D + g * 8;
    f32x16 s, dp;
#pragma unroll
    for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const vec8 ka = *(const vec8 *)(k + kbase + kk * 16), qa = *(const vec8 *)(q + qbase + kk * 16);
        const vec8 va = *(const vec8 *)(v + kbase + kk * 16), da = *(const vec8 *)(dout + qbase + kk * 16);
        s = E::mfma(ka, qa, s);        // s[i] = <k_row, q_col>: key kb*32 + (i/4)*8 + g*4 + i%4, query qrow
        dp = E::mfma(va, da, dp);      // dP likewise
    }
    const float l2 = lse2[(size_t)head * S + (qrow < S ? qrow : S - 1)];
    const int klim = causal ? (qrow < S - 1 ? qrow : S - 1) : S - 1;      // the keys 0 ... klim reach this query
    float x = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int key = kb * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
        if (key <= klim) x += __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], scale_log2, -l2)) * dp[i];
    }
    x += __shfl_xor(x, 32, 64);                           // the two lanes that share a query column
    if (g == 0) part[kb][qrow] = x;
    __syncthreads();
    if (tid < rows) delta[(size_t)head * S + tid] = part[0][tid] + part[1][tid];
#endif
}

// BWD_DKV is the dK and dV passes in one (scores and P computed once for both): two output
// accumulators and both resident operand sets, which fits 256 registers per lane at D = 64 only.
enum { BWD_DQ = 0, BWD_DK = 1, BWD_DV = 2, BWD_DKV = 3 };

// GRP: grouped heads, G query heads reading one key/value head (query head h the head h / G).  The
// dQ pass then streams the K and V of its query head's group; the keys-resident passes run one
// workgroup per (key/value head, key tile) and stream the Q and dO tiles of the G query heads of the
// group one head after the other into the same accumulators, which is the sum over the group that dK
// and dV are.  GRP = false is G = 1 with that loop gone.
template <typename T, int D, int NW, int TS, int WPS, int MODE, bool GRP = false>
__global__ void __launch_bounds__(NW * 64, WPS)
sdpa_bwd_kernel(const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v,
                const T *__restrict__ dout, const float *__restrict__ stats,   // Delta [B*H*S + slack], then LSE likewise
                T *__restrict__ out,   // dQ, dK or dV
                T *__restrict__ out2,  // dV of the fused dK + dV pass, else unused
                int S, int nR, int N, float c, float scale, uint32_t rsign, int causal, unsigned stat_bytes,
                int group)
{
#if defined(__HIP_DEVICE_COMPILE__)
    using E = Elem<T>;
    using vec8 = typename E::vec8;
    using vec4 = typename E::vec4;
    using G = BwdGeom<D, TS>;
    constexpr bool KEYS_RES = MODE != BWD_DQ;
    constexpr bool NEED_DP = MODE != BWD_DV;      // dP product and Delta
    constexpr bool FUSED = MODE == BWD_DKV;       // P kept next to dS, second accumulator for dV
    constexpr int RM = NW * 32;                   // resident rows per workgroup
    constexpr int CPR = G::DG / 8;                // 16-byte chunks per LDS row
    constexpr int GCPR = D / 8;                   // ... of which this many hold data
    constexpr int NLD = TS * CPR / (NW * 64);     // direct-to-LDS load instructions per wavefront per tile
    static_assert(NLD >= 1 && (TS * CPR) % (NW * 64) == 0, "tile does not divide over the workgroup");
    constexpr int NB = TS / 32, KK = D / 16, DB = D / 32;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const lds_ptr lds = (lds_ptr)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, l32 = lane & 31;

    const int wg = remap_workgroup(blockIdx.x, N, false);
    const int head = wg / nR;                     // head of the resident side: a query head (dQ pass) or a key/value head
    const int Gn = GRP ? group : 1;              // query heads per key/value head
    // causal: query tiles get longer with their index, key tiles shorter; start the long ones first
    const int rt = (causal && !KEYS_RES) ? nR - 1 - (wg - head * nR) : wg - head * nR;
    const size_t head_off = (size_t)head * (size_t)S * D;
    const T *r1 = (KEYS_RES ? k : q) + head_off;       // resident operands
    const T *r2 = (KEYS_RES ? v : dout) + head_off;
    // streamed operands: the key/value head of this query head, or the first query head of this key/value head
    const size_t shead0 = KEYS_RES ? (size_t)head * Gn : (size_t)(head / Gn);
    const T *t1 = (KEYS_RES ? q : k) + shead0 * (size_t)S * D;
    const T *t2 = (KEYS_RES ? dout : v) + shead0 * (size_t)S * D;

    // ---- resident rows as MFMA B-operands: lane holds R[row l32][kk*16 + g*8 .. +7]; the sign of a
    // negative scale is folded into R1 so that c = |scale| * log2(e) applies to the scores
    const int r0 = rt * RM;
    const int rrow = r0 + wave * 32 + l32;
    const int rrow_c = rrow < S ? rrow : S - 1;
    vec8 rf1[KK], rf2[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        u32x4 raw = *(const u32x4 *)(r1 + (size_t)rrow_c * D + kk * 16 + g * 8);
        raw ^= rsign;
        rf1[kk] = __builtin_bit_cast(vec8, raw);
        if constexpr (NEED_DP) rf2[kk] = *(const vec8 *)(r2 + (size_t)rrow_c * D + kk * 16 + g * 8);
    }

    // ---- range of streamed tiles, and the streamed rows [tlo, thi] that pair with this lane's row
    const int nT = (S + TS - 1) / TS;
    const int last_row = (r0 + RM < S ? r0 + RM : S) - 1;
    int j0 = 0, j1 = nT;
    int tlo = 0, thi = S - 1;
    if (causal) {
        if (KEYS_RES) { j0 = r0 / TS; tlo = rrow; }                       // queries at or after the key
        else { j1 = last_row / TS + 1; thi = rrow < S ? rrow : S - 1; }   // keys up to the query
    }

    // per-row statistics of the query side, LSE (log2 units) and Delta: scalars of this lane's row, or
    // (keys-resident pass) streamed into the LDS with each tile.  The descriptor spans both arrays,
    // slack included; rows >= S of a head pick up the next head's or the slack's values and are masked.
    const float *delta = stats, *lse2 = (const float *)((const char *)stats + stat_bytes);
    float lse_r = 0.f, delta_r = 0.f;
    if (!KEYS_RES) { lse_r = lse2[(size_t)head * S + rrow_c]; delta_r = delta[(size_t)head * S + rrow_c]; }
    const auto stat_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)stats, (short)0, (int)(2 * stat_bytes), 0x00020000);
    constexpr int NST = 2 * TS / 64;              // 4-byte direct-to-LDS loads (wavefront 0) per tile: LSE rows, then Delta rows
    int stat_goff[NST];
#pragma unroll
    for (int it = 0; it < NST; ++it) {
        const int e = it * 64 + lane;             // element of the tile's statistics block
        stat_goff[it] = (e / TS == 0 ? (int)stat_bytes : 0) + ((int)shead0 * S + e % TS) * 4;
    }

    // ---- streamed tiles HBM -> LDS, as in the forward kernel: a descriptor per tensor covers this
    // head's S rows (rows >= S read as zeros), lane `lane` of load `it` fills LDS chunk
    // (it*NW + wave)*64 + lane with the global chunk the swizzle maps there
    auto t1_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)t1, (short)0, S * G::GROW, 0x00020000);
    auto t2_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)t2, (short)0, S * G::GROW, 0x00020000);
    constexpr int kNoFetch = 0x60000000;          // beyond any descriptor (one head holds < 2^30 bytes)
    int goff[NLD];
#pragma unroll
    for (int it = 0; it < NLD; ++it) {
        const int p = (it * NW + wave) * 64 + lane;
        const int r = p / CPR, cp = p % CPR;
        const int gc = cp ^ G::swz(r);            // global chunk that belongs at LDS chunk cp
        goff[it] = gc < GCPR ? r * G::GROW + (gc << 4) : kNoFetch;
    }
    // load instruction `it` (of NLD) of tile j of a streamed tensor
    auto load_part = [&](decltype(t1_rsrc) rsrc, int j, lds_ptr dst, int it) __attribute__((always_inline)) {
        const int soff = (j < j1 ? j : nT) * G::GTILE;    // a tile past the range: outside the descriptor, zeros
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (TSDPA_LDS void *)(dst + (it * NW + wave) * 1024), 16,
                                                 goff[it], soff, 0, 0);
    };
    auto load_tile = [&](decltype(t1_rsrc) rsrc, int j, lds_ptr dst) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < NLD; ++it) load_part(rsrc, j, dst, it);
    };
    constexpr int T2BASE = 2 * G::TILE;           // T1 slot s at s*TILE, T2 slot s at T2BASE + s*TILE
    constexpr int STBASE = 4 * G::TILE;           // statistics slot s at STBASE + s*STATS
    auto stat_slot = [](int slot) { return STBASE + slot / G::TILE * G::STATS; };
    auto load_stats = [&](int j, int slot) __attribute__((always_inline)) {
        if constexpr (KEYS_RES) {
            if (wave == 0) {
#pragma unroll
                for (int it = 0; it < NST; ++it)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(stat_rsrc, (TSDPA_LDS void *)(lds + stat_slot(slot) + it * 256), 4,
                                                             stat_goff[it], j * TS * 4, 0, 0);
            }
        }
    };

    f32x16 oacc[DB], oacc2[FUSED ? DB : 1];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            oacc[db][i] = 0.f;
            if constexpr (FUSED) oacc2[db][i] = 0.f;
        }

    // ---- per-lane LDS read pointers (tile slot, nb, ks enter as immediate offsets)
    // row-wise: row l32 (+32*nb), chunk (2*kk + g) ^ swz(row)
    lds_ptr row_ptr[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        row_ptr[kk] = lds + l32 * G::ROW + (((2 * kk + g) ^ G::swz(l32)) << 4);
        TSDPA_OPAQUE(row_ptr[kk]);
    }
    // transposing: row g*4 + (lane%16)/4 (+ multiples of 8), bytes db*64 + ((lane/16)%2)*32 + (lane%4)*8
    // of the row, i.e. chunk db*4 + ((lane/16)%2)*2 + (lane%4)/2, swizzled.  Adding 8 to the row flips
    // bit 1 of swz (bit 5 of the byte offset); adding 16 or 32 leaves swz alone.
    const int t_row = g * 4 + ((lane & 15) >> 2);
    lds_ptr tr_lo[DB], tr_hi[DB];                 // rows t_row (+16k) and t_row + 8 (+16k)
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        const int chunk = db * 4 + ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
        const int off = t_row * G::ROW + ((chunk ^ G::swz(t_row)) << 4) + (lane & 1) * 8;
        tr_lo[db] = lds + off;
        tr_hi[db] = lds + 8 * G::ROW + (off ^ 32);
        TSDPA_OPAQUE(tr_lo[db]);
        TSDPA_OPAQUE(tr_hi[db]);
    }

    // acc[i] = <T_row, R_col>, row = nb*32 + (i/4)*8 + g*4 + i%4 of the tile, col = this lane's row
    auto products = [&](int slot, int nb, const vec8 (&rf)[KK], f32x16 &acc, auto &&after_mfma) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            u32x4 raw = lds_read128(row_ptr[kk] + slot + nb * 32 * G::ROW);
            acc = E::mfma(__builtin_bit_cast(vec8, raw), rf[kk], acc);
            after_mfma(kk);
        }
    };
    // out^T += T^T X, X taken from accumulator layout as B-operands (k-slots 0..3 / 4..7 of a lane <->
    // tile rows base+g*4+0..3 / base+8+g*4+0..3, mirrored on the A side by the two transposing reads)
    auto accumulate = [&](int slot, const vec8 (&xb)[NB][2], f32x16 (&out)[DB]) __attribute__((always_inline)) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const int tile_off = slot + (nb * 32 + ks * 16) * G::ROW;
                    i16x4 lo = lds_read_tr16(tr_lo[db] + tile_off);
                    i16x4 hi = lds_read_tr16(tr_hi[db] + tile_off);
                    i16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    out[db] = E::mfma(__builtin_bit_cast(vec8, a), xb[nb][ks], out[db]);
                }
    };

    // One streamed tile: P (and dS) from the first products, rounded to 16 bits as B-operands of the
    // second product.  The next tile's loads are issued first and land while this one is computed.
    vec8 xb[NB][2], pb[FUSED ? NB : 1][2];
    auto tile = [&](int j, auto par_tag, auto mask_tag) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_tag)::value;
        constexpr bool MASK = decltype(mask_tag)::value;
        constexpr int cur = PAR * G::TILE, nxt = (1 - PAR) * G::TILE;
        load_stats(j + 1, nxt);
        // Where a SIMD holds one wavefront, the next tile's loads go out one at a time behind the MFMAs of the
        // first products: back to back they hold the wavefront at the issue stage while the CU's address unit
        // works through them, and nothing else is there to run (D = 160: 4-6 % of the whole call; with two
        // wavefronts per SIMD the spread-out form is level without the causal mask and 4-6 % slower with it)
        constexpr bool SPREAD = WPS == 1;
        constexpr int HOOKS = NB * (NEED_DP ? 2 : 1) * KK, L = 2 * NLD;
        if constexpr (!SPREAD) {
            load_tile(t1_rsrc, j + 1, lds + nxt);
            load_tile(t2_rsrc, j + 1, lds + T2BASE + nxt);
        }
        auto spread = [&](int h) __attribute__((always_inline)) {
            if constexpr (SPREAD) {
#pragma unroll
                for (int i = h * L / HOOKS; i < (h + 1) * L / HOOKS; ++i) {
                    if (i < NLD) load_part(t1_rsrc, j + 1, lds + nxt, i);
                    else         load_part(t2_rsrc, j + 1, lds + T2BASE + nxt, i - NLD);
                }
                __builtin_amdgcn_sched_barrier(0x786);      // MFMAs and loads keep this order
            }
        };
        const int trow0 = j * TS + g * 4;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {       // one 32-row block at a time: only its accumulators are live
            f32x16 sacc, dpacc;
            products(cur, nb, rf1, sacc, [&](int kk) __attribute__((always_inline)) { spread(nb * (NEED_DP ? 2 : 1) * KK + kk); });
            if constexpr (NEED_DP)
                products(T2BASE + cur, nb, rf2, dpacc, [&](int kk) __attribute__((always_inline)) { spread((nb * 2 + 1) * KK + kk); });
            // the 16 streamed rows this lane meets in the block come in 4 runs of 4 consecutive rows; in the
            // keys-resident passes their statistics are read from the LDS run by run (in the dK pass
            // scheduling barriers keep the compiler from fetching all of them ahead, which costs 32 registers)
            const lds_ptr sp = lds + stat_slot(cur) + (nb * 32 + g * 4) * 4;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                f32x4 st_lse, st_delta;
                if constexpr (KEYS_RES) {
                    st_lse = *(TSDPA_LDS f32x4 *)(sp + r4 * 32);
                    if constexpr (NEED_DP) st_delta = *(TSDPA_LDS f32x4 *)(sp + TS * 4 + r4 * 32);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = r4 * 4 + e;
                    const float l2 = KEYS_RES ? st_lse[e] : lse_r;
                    float x = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[i], c, -l2));        // P
                    if constexpr (MASK) {
                        const int trow = trow0 + nb * 32 + r4 * 8 + e;
                        if (trow < tlo || trow > thi) x = 0.f;
                    }
                    if constexpr (FUSED) pb[nb][i >> 3][i & 7] = (T)x;
                    if constexpr (NEED_DP) {
                        const float dl = KEYS_RES ? st_delta[e] : delta_r;
                        x *= dpacc[i] - dl;                                                   // dS
                    }
                    xb[nb][i >> 3][i & 7] = (T)x;
                }
                if constexpr (MODE == BWD_DK || FUSED) __builtin_amdgcn_sched_barrier(0);
            }
        }
        accumulate(MODE == BWD_DV ? T2BASE + cur : cur, xb, oacc);
        if constexpr (FUSED) accumulate(T2BASE + cur, pb, oacc2);       // dV^T += dO^T P
        TSDPA_WAIT_VMCNT0();
        __syncthreads();
    };

    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    // a tile needs the masked path if it reaches past row S-1 or (causal) crosses the diagonal of any
    // of this workgroup's rows
    auto needs_mask = [&](int j) __attribute__((always_inline)) -> bool {
        if ((j + 1) * TS > S) return true;
        if (!causal) return false;
        return KEYS_RES ? j * TS < r0 + RM - 1 : (j + 1) * TS - 1 > r0;
    };
    for (int gq = 0; gq < (KEYS_RES ? Gn : 1); ++gq) {
    if (GRP && KEYS_RES && gq > 0) {
        // next query head of the group: its Q, dO and statistics (the last barrier of the previous head's
        // loop has every wavefront past its last LDS read and every outstanding load landed)
        t1 += (size_t)S * D;
        t2 += (size_t)S * D;
        t1_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)t1, (short)0, S * G::GROW, 0x00020000);
        t2_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)t2, (short)0, S * G::GROW, 0x00020000);
#pragma unroll
        for (int it = 0; it < NST; ++it) stat_goff[it] += S * 4;
    }
    if (j0 < j1) {
        load_stats(j0, 0);
        load_tile(t1_rsrc, j0, lds);
        load_tile(t2_rsrc, j0, lds + T2BASE);
        TSDPA_WAIT_VMCNT0();
        __syncthreads();
        int j = j0;
        while (j < j1) {
            const bool even = ((j - j0) & 1) == 0;
            if (even && j + 1 < j1 && !needs_mask(j) && !needs_mask(j + 1)) {
                tile(j, P0{}, std::false_type{});
                tile(j + 1, P1{}, std::false_type{});
                j += 2;
            } else {
                if (even) tile(j, P0{}, std::true_type{});
                else      tile(j, P1{}, std::true_type{});
                ++j;
            }
        }
    }
    }

    // ---- store: out^T tiles are turned through LDS (as the forward kernel's O) and written as whole
    // rows; dQ and dK carry the factor `scale` of the score, dV none.  The last barrier of the loop has
    // every wavefront past its last LDS read.
    auto store = [&](const f32x16 (&acc)[DB], float factor, T *dst) __attribute__((always_inline)) {
        constexpr int CMASK = CPR - 1;
        const lds_ptr ow = lds + wave * (32 * G::ROW);
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                vec4 val;
#pragma unroll
                for (int e = 0; e < 4; ++e) val[e] = (T)(acc[db][q4 * 4 + e] * factor);
                const int chunk = db * 4 + q4;
                *(TSDPA_LDS vec4 *)(ow + l32 * G::ROW + ((chunk ^ (l32 & CMASK)) << 4) + g * 8) = val;
            }
        constexpr int RPI = 64 / CPR;
        const int row0 = r0 + wave * 32;
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int r = i * RPI + lane / CPR, cc = lane % CPR;
            const u32x4 val = lds_read128(ow + r * G::ROW + ((cc ^ (r & CMASK)) << 4));
            if (row0 + r < S && cc < GCPR) *(u32x4 *)(dst + head_off + (size_t)(row0 + r) * D + cc * 8) = val;
        }
    };
    // (the launcher sizes the dynamic LDS for the larger of the tile slots and this staging area)
    store(oacc, MODE == BWD_DV ? 1.0f : scale, out);
    if constexpr (FUSED) store(oacc2, 1.0f, out2);   // same staging region: it is private to the wavefront, whose LDS operations complete in order
#endif
}

}  // namespace tsdpa
