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
typedef float f32x4 __attribute__((ext_vector_type(4)));

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

// LDS geometry shared by host (dynamic LDS size) and device.  A tile is TN rows of D 16-bit values,
// unpadded; within a row the 16-byte chunks are XOR-swizzled:
//   K: chunk c of row r sits at c ^ kswz(r).  The score MFMA's A-operand read has 16 lanes fetch the
//      same chunk of 16 consecutive rows; the swizzle spreads them over all 64 banks.
//   V: 64-byte block b of row r sits at b ^ vswz(r).  The transposing read has 32 lanes fetch one
//      64-byte block of 4 consecutive rows; the swizzle puts those on 4 x 16 distinct banks.
// Head dims that are not a power of two (96 and 160: 12 and 20 chunks per row) keep their rows unpadded
// as well (COMPACT): rows 192 or 320 bytes apart start 3 or 5 quarters of the 64 banks after one another, so
//   V needs no swizzle: 4 consecutive rows put the same 64-byte block on 4 different quarters;
//   K: row r = 4a + b starts on quarter +-b (mod 4), and chunk c = 4*ch + cl stored at c ^ (a & 3) lands on
//      16-byte slot 4*(ch +- b) + (cl ^ a) of the 16 that make up the 64 banks: 16 consecutive rows, 16 slots.
// A tile in the LDS is then as long as in memory, every lane of every load instruction carries data (padded
// to 128 or 256 columns, 25 % or 37.5 % of them would fetch nothing), and the four tile slots of D = 160 take
// 80 KiB instead of 128 at 64 rows.  The output transpose after the loop keeps the power-of-two rows (OROW).
template <int D, int TN> struct TileGeom {
    static constexpr bool COMPACT = (D & (D - 1)) != 0;
    static constexpr int DG = D <= 64 ? 64 : (D <= 128 ? 128 : 256);
    static constexpr int ROW = COMPACT ? D * 2 : DG * 2;   // bytes per LDS row of a K or V tile
    static constexpr int OROW = DG * 2;             // bytes per LDS row of the output transpose
    static constexpr int GROW = D * 2;              // bytes per row in global memory
    static constexpr int TILE = TN * ROW;           // bytes per K or V tile in LDS
    static constexpr int GTILE = TN * GROW;         // ... and in global memory
    static constexpr int LDS_BYTES = 4 * TILE;      // K slots 0,1 then V slots 0,1
    static __host__ __device__ constexpr int kswz(int r) { return COMPACT ? ((r >> 2) & 3) : DG == 64 ? ((r >> 1) & 7) : (r & 15); }
    static __host__ __device__ constexpr int vswz(int r) { return COMPACT ? 0 : DG == 64 ? ((r >> 1) & 1) : (r & 3); }
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

// Hides how a register value was computed from the optimiser.  Used on loop-invariant LDS pointers:
// left transparent, the compiler splits them into a common base and per-pointer offsets and re-adds the
// two in front of every LDS read of the loop (one vector-ALU instruction per read).
#define TSDPA_OPAQUE(x) asm volatile("" : "+v"(x))

// s_waitcnt vmcnt(0) with the other counters left at their maxima (gfx9 encoding)
#define TSDPA_WAIT_VMCNT0() __builtin_amdgcn_s_waitcnt(0x0F70)

// KV = false is the paper's problem: S query rows against the same S key rows, one workgroup per
// (head, query tile), final output.  KV = true generalises it for the decoding shapes of the paper's
// roadmap (Section 7): S query rows against Skv key rows (under the causal mask the queries are the
// last S positions of the sequence), and the key range of every (head, query tile) cut into `splits`
// contiguous runs of tiles, one workgroup each.  With splits > 1 a workgroup writes its unnormalised
// state (o, m, l of Eqs. 2-4) to `ws` instead of O: o as float [BH][splits][S][D], followed by
// (m, l) pairs as float [BH][splits][S][2]; sdpa_merge_kernel combines them.
// Grouped heads (G query heads reading one key/value head) arrive folded: a "head" of the KV = true
// kernel is one key/value head and its S = G * Sp rows are the Sp positions of each of the G query
// heads in turn, so only the causal limit has to know Sp (`rows_per_head`; equal to S when nothing is
// folded).  With `kv_lens` every batch entry has its own number of valid key rows (a KV cache of
// capacity Skv_arg rows per head, filled to kv_lens[b]): everything below uses that length, only the
// distance between heads in memory stays the capacity.  With `block_table` the cache is paged: K and V
// are [pages][heads_per_batch][block_rows][D], block_table[b][i] names the page that holds key rows
// i * block_rows ... of batch entry b, and every K/V tile (block_rows is a multiple of the tile) gets a
// buffer descriptor of its own, based at its page and as long as the tile has valid rows.
// KVM: 0 = the paper's square problem, 1 = the general kernel over a dense cache, 2 = over a paged cache
// (an instantiation of its own: the per-tile descriptors cost scalar registers in the loop, which the
// latency-bound small decoding shapes of the dense path would pay for too).
template <typename T, int D, int NW, int TN, int WPS, int KVM>
__global__ void __launch_bounds__(NW * 64, WPS)  // WPS = wavefronts per SIMD the register budget is sized for
sdpa_fwd_kernel(const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v,
                T *__restrict__ o, float *__restrict__ lse, int S, int nQ, int N, float c,
                float tau, uint32_t qsign, int linear_grid, int causal,
                int Skv_arg, int splits_arg, float *__restrict__ ws, int rows_per_head,
                const int *__restrict__ kv_lens, int heads_per_batch,
                const int *__restrict__ block_table, int max_blocks, int block_shift, int tile_rot)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses device-only types
    constexpr bool KV = KVM != 0, PAGED = KVM == 2;
    using E = Elem<T>;
    using vec8 = typename E::vec8;
    using vec4 = typename E::vec4;
    using G = TileGeom<D, TN>;
    constexpr int TM = NW * 32;
    constexpr bool COMPACT = G::COMPACT;
    constexpr int CPR = G::ROW / 16;              // 16-byte chunks per LDS row
    constexpr int GCPR = D / 8;                   // (all of them hold data; the rows of the output transpose may be longer)
    // A direct-to-LDS load instruction fills one unit: 64 consecutive chunks (1 KiB) of a tile slot.
    constexpr int U = TN * CPR / 64;              // units per K or V tile
    constexpr int NLD = U / NW;                   // units of one tensor's tile per wavefront (where that divides)
    constexpr int L = 2 * U / NW;                 // load instructions per wavefront per K/V tile pair
    static_assert((TN * CPR) % 64 == 0 && L >= 1 && (2 * U) % NW == 0, "tile pair does not divide over the workgroup");
    static_assert(COMPACT || U % NW == 0, "tile does not divide over the workgroup");
    // A 128-row K/V tile above D = 64 is filled and released as one tile (one barrier per 128 rows) but
    // worked through in two halves of 64 rows, each a complete step of Eqs. 2-4: four 32-row score
    // accumulators at once do not fit the registers beside the output accumulator of these head dims.
    constexpr int TNS = (TN == 128 && D > 64) ? 64 : TN;   // key rows per pass through scores / softmax / PV
    constexpr int NSUB = TN / TNS;
    constexpr int NB = TNS / 32, KK = D / 16, DB = D / 32;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const lds_ptr lds = (lds_ptr)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, l32 = lane & 31;

    const int splits = KV ? splits_arg : 1;
    const int Sp = KV ? rows_per_head : S;        // query positions per query head (S = G * Sp rows when folded)
    const bool folded = KV && Sp != S;
    const int wg = remap_workgroup(blockIdx.x, N, linear_grid != 0);
    // query tile fastest, then split, then head: neighbours share one run of K/V tiles
    const int hs = wg / nQ;
    const int head = KV ? hs / splits : hs;
    const int sp = KV ? hs - head * splits : 0;
    // under the causal mask the work of a query tile grows with its index: start the long ones first
    const int qt = causal ? nQ - 1 - (wg - hs * nQ) : wg - hs * nQ;
    const size_t head_off = (size_t)head * (size_t)S * D;
    const size_t kv_off = (size_t)head * (size_t)(KV ? Skv_arg : S) * D;
    // key rows of this head; S is the number of query rows
    int Skv = KV ? Skv_arg : S;
    if (KV && kv_lens != nullptr) {
        const int len = kv_lens[head / heads_per_batch];
        Skv = len < 0 ? 0 : (len < Skv_arg ? len : Skv_arg);
    }
    const int koff = Skv - Sp;                    // position of a head's query row 0 in the key sequence (causal)
    // paged cache: this batch entry's row of the block table, and the head's index within a page
    const int *pages = nullptr;
    int page_head = 0;
    if constexpr (PAGED) {
        const int b = head / heads_per_batch;
        page_head = head - b * heads_per_batch;
        pages = block_table + (size_t)b * max_blocks;
    }
    const T *qh = q + head_off;

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

    // Tiles this workgroup streams, and how many leading ones need no mask for any of its rows.
    // A key j contributes to query row i iff j <= klim(i): klim = Skv-1 (only the ragged tail is cut
    // off), or the query's own position min(i, S-1) + koff under the causal mask of Section 4.1.3,
    // where tiles strictly above the diagonal of the workgroup's last row are neither read nor computed.
    const int nT = (Skv + TN - 1) / TN;
    const int r0 = qt * TM;
    int page_now = 0, page_next = 0;              // paged cache: pages of the tile being loaded and of the one after it
    const int last_row = (r0 + TM < S ? r0 + TM : S) - 1;
    // least and greatest position among the workgroup's rows, and this lane's own
    int pos_lo = r0, pos_hi = last_row, pos_own = qrow_c;
    if (folded) {
        const int g0 = r0 / Sp, g1 = last_row / Sp;
        if (g0 == g1) { pos_lo -= g0 * Sp; pos_hi -= g0 * Sp; }
        else          { pos_lo = 0; pos_hi = Sp - 1; }        // the tile crosses into the next query head
        pos_own = qrow_c % Sp;
    }
    // (a cache entry shorter than the query block leaves the first rows without any key: reach < 0)
    const int reach = pos_hi + koff;
    const int nTw = causal ? ((KV && reach < 0) ? 0 : reach / TN + 1) : nT;
    const int klim = causal ? pos_own + koff : Skv - 1;
    const int nfull = ((causal ? pos_lo + koff : Skv - 1) + 1) / TN;
    // this workgroup's run of tiles [t0, t1): all nTw of them unless the key range is split
    const int per_split = (nTw + splits - 1) / splits;
    const int t0 = KV ? sp * per_split : 0;
    const int t1 = KV ? (t0 + per_split < nTw ? t0 + per_split : nTw) : nTw;

    // ---- K/V tiles: HBM -> LDS.  One buffer descriptor per tensor covers exactly this head's Skv rows,
    // so a row index >= Skv reads as zeros instead of touching memory.  Load instruction `it` of this
    // wavefront fills LDS chunks [(it*NW + wave)*64, +64) of the tile; lane `lane` fills chunk p of
    // that range and therefore fetches the global chunk that the swizzle maps to position p.
    const auto k_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(k + kv_off), (short)0, Skv * G::GROW, 0x00020000);
    const auto v_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(v + kv_off), (short)0, Skv * G::GROW, 0x00020000);
    // Rows of a power of two.  The swizzles repeat every 16 rows and a load instruction of the workgroup's sweep lands
    // NW * RPI rows after the previous one, so the per-lane offsets repeat with period NG in `it`: only NG of them are
    // kept in vector registers, the rest of the distance travels in the scalar offset.
    constexpr int RPI = COMPACT ? 1 : 64 / CPR;   // tile rows filled by one load instruction
    constexpr int PER = 16 / (NW * RPI) > 1 ? 16 / (NW * RPI) : 1;
    constexpr int NG = COMPACT ? 1 : (NLD < PER ? NLD : PER);
    constexpr int GSTEP = NG * NW * RPI * G::GROW; // global bytes between load instructions it and it + NG
    static_assert(COMPACT || NLD <= NG || (NG * NW * RPI) % 16 == 0, "offsets must repeat with the swizzle period");
    int k_goff[NG], v_goff[NG];
    if constexpr (!COMPACT) {
#pragma unroll
        for (int it = 0; it < NG; ++it) {
            const int p = (it * NW + wave) * 64 + lane;
            const int r = p / CPR, cp = p % CPR;
            const int kc = cp ^ G::kswz(r), vc = cp ^ (G::vswz(r) << 2);   // global chunk that belongs at LDS chunk cp
            k_goff[it] = r * G::GROW + (kc << 4);
            v_goff[it] = r * G::GROW + (vc << 4);
        }
    }
    // Compact rows.  The units of a tile pair, K's U then V's U, are dealt round-robin: load i of this wavefront is
    // unit i * NW + wave.  A V unit is a plain copy (chunk p of the tile in memory to chunk p of the slot); a K unit
    // has its chunks permuted within each row, and 16 rows being CP = CPR / 4 units, the per-lane offsets of K repeat
    // every CP units.  Where U is a multiple of NW (EVEN) a load is a K or a V load for all wavefronts alike: CP
    // registers serve K and one serves V, the rest of the distance travels in the scalar offset.  Otherwise one load
    // of the L is a K load for the first wavefronts and a V load for the others; then L = CP and each load has a
    // register of its own, filled for whatever this wavefront loads there.
    constexpr int CP = CPR / 4;
    constexpr bool EVEN = U % NW == 0;
    constexpr int NCG = !COMPACT ? 1 : EVEN ? (NLD < CP ? NLD : CP) : L;
    static_assert(!COMPACT || EVEN || L <= 6, "a register per load is meant for a few loads");
    static_assert(!COMPACT || !EVEN || NLD <= CP || (CP * NW * 64) % (16 * CPR) == 0, "offsets must repeat with the swizzle period");
    int c_goff[NCG], cv_goff = 0;
    if constexpr (COMPACT) {
#pragma unroll
        for (int i = 0; i < NCG; ++i) {
            const int u = i * NW + wave;
            const int p = (EVEN || u < U ? u : u - U) * 64 + lane;
            const int r = p / CPR, cp = p % CPR;
            const int kg = r * G::GROW + ((cp ^ G::kswz(r)) << 4);
            c_goff[i] = (EVEN || u < U) ? kg : p * 16;
        }
        cv_goff = (wave * 64 + lane) * 16;
    }
    struct TileSrc { decltype(k_rsrc) rsrc; int soff; };
    // where tile j of a tensor is fetched from: descriptor and wavefront-uniform offset
    auto tile_src = [&](const T *tensor, decltype(k_rsrc) whole, int j) __attribute__((always_inline)) {
        auto rsrc = whole;
        // wavefront-uniform (scalar) offset.  On gfx950 the descriptor's range check takes the scalar
        // offset into account (a parity test surrounds K and V with NaN to pin this): rows >= S fall
        // outside the descriptor and read as zeros without a memory access, and so does a tile this
        // workgroup does not need (its index is moved past the end)
        int soff = (j < t1 ? j : nT) * G::GTILE;
        if constexpr (PAGED) {
            // the tile lies within one page: a descriptor from the page's rows of this head, covering
            // the tile's valid rows only (none for a tile this workgroup does not need)
            const int row0 = j * TN;
            int valid = j < t1 ? Skv - row0 : 0;
            valid = valid < 0 ? 0 : (valid < TN ? valid : TN);
            const int blk = row0 >> block_shift;
            // tiles are loaded in increasing order, K before V: the K load takes the page looked up while the
            // previous tile was loaded and starts the lookup for the next tile, so that the scalar load's
            // latency is not paid in front of every tile
            if (tensor == k) {
                page_now = page_next;
                const int nblk = (row0 + TN) >> block_shift;
                // (the value is the same in every lane; said explicitly, or the descriptor built from it is
                // taken for lane-dependent and every load is wrapped in a loop over distinct descriptors)
                page_next = nblk == blk ? page_now : __builtin_amdgcn_readfirstlane(pages[nblk < max_blocks ? nblk : 0]);
            }
            const int page = page_now;
            const size_t first = (((size_t)page * heads_per_batch + page_head) << block_shift) + (row0 - (blk << block_shift));
            // every input of the descriptor is the same in all lanes; stated for the two the compiler cannot
            // see through (loaded values), or each load below becomes a loop over distinct descriptors
            const unsigned long long byte0 = (unsigned long long)first * (unsigned long long)(D * sizeof(T));
            const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)byte0);
            const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(byte0 >> 32));
            const char *base = (const char *)tensor + (((unsigned long long)hi << 32) | lo);
            rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)base, (short)0,
                                                     __builtin_amdgcn_readfirstlane(valid * G::GROW), 0x00020000);
            soff = 0;
        }
        return TileSrc{rsrc, soff};
    };
    // load instruction `it` (of NLD) of a tile in rows of a power of two
    auto load_part = [&](const TileSrc &src, const int (&goff)[NG], lds_ptr dst, int it) __attribute__((always_inline)) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(src.rsrc, (TSDPA_LDS void *)(dst + (it * NW + wave) * 1024), 16,
                                                 goff[it % NG], src.soff + (it / NG) * GSTEP, 0, 0);
    };
    // unit `unit` of a tile in compact rows
    auto load_unit = [&](const TileSrc &src, lds_ptr dst, int unit, int goff, int soff) __attribute__((always_inline)) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(src.rsrc, (TSDPA_LDS void *)(dst + unit * 1024), 16, goff, src.soff + soff, 0, 0);
    };
    // load instruction i (of L) of the tile pair (K, V): K's come first
    auto issue = [&](const TileSrc &ksrc, const TileSrc &vsrc, lds_ptr kdst, lds_ptr vdst, int i) __attribute__((always_inline)) {
        if constexpr (!COMPACT) {
            if (i < NLD) load_part(ksrc, k_goff, kdst, i);
            else         load_part(vsrc, v_goff, vdst, i - NLD);
        } else if constexpr (EVEN) {
            // K: NCG units on, the offsets repeat NCG * NW units = NW * 16 rows further down (NCG = CP whenever i >= NCG)
            if (i < NLD) load_unit(ksrc, kdst, i * NW + wave, c_goff[i % NCG], (i / NCG) * (NW * 16 * G::GROW));
            else         load_unit(vsrc, vdst, (i - NLD) * NW + wave, cv_goff, (i - NLD) * NW * 1024);
        } else {
            const int u = i * NW + wave;
            if ((i + 1) * NW <= U)  load_unit(ksrc, kdst, u, c_goff[i], 0);
            else if (i * NW >= U)   load_unit(vsrc, vdst, u - U, c_goff[i], 0);
            else {
                // K for the first wavefronts, V for the others: chosen by scalar selects (a branch here would cut
                // the chain of score MFMAs that the loads are issued between in two)
                const bool is_k = u < U;
                const TileSrc src{is_k ? ksrc.rsrc : vsrc.rsrc, is_k ? ksrc.soff : vsrc.soff};
                load_unit(src, is_k ? kdst : vdst, is_k ? u : u - U, c_goff[i], 0);
            }
        }
    };
    // tile j of K and of V into the slots kdst, vdst
    auto load_tiles = [&](int j, lds_ptr kdst, lds_ptr vdst) __attribute__((always_inline)) {
        const TileSrc ksrc = tile_src(k, k_rsrc, j), vsrc = tile_src(v, v_rsrc, j);
#pragma unroll
        for (int i = 0; i < L; ++i) issue(ksrc, vsrc, kdst, vdst, i);
    };
    constexpr int KSLOT0 = 0, KSLOT1 = G::TILE, VSLOT0 = 2 * G::TILE, VSLOT1 = 3 * G::TILE;

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    // Online-softmax state (Eqs. 2-4), all in the log2 domain of s*c.  m_ref is the reference the
    // exponentials are taken against.  It is not the running maximum of Eq. 2 but a stale one: a tile's
    // weights p = 2^(s*c - m_ref) are computed first, and only if this lane's sum of them exceeds
    // 2^tau (some score lies far above the reference; always so on a row's first tile, where m_ref is
    // -inf) is the tile maximum taken, the reference raised to it, the state rescaled (Eqs. 3-4) and
    // the weights recomputed.  With a stale reference the weights of a row are merely scaled by a common
    // factor <= 2^tau, which cancels in o/l and in m_ref + log2(l); in return the common case needs
    // neither the maximum nor the rescale.  tau = 0 raises the reference on every new maximum (any
    // weight above 1 makes the sum exceed 1), which is Eq. 2 literally, at the price of recomputing
    // most tiles.
    float m_ref = -INFINITY;
    const float lazy_limit = __builtin_amdgcn_exp2f(tau);
    float l_run = 0.f;         // this lane's share of the normaliser (lane^32 holds the rest)

    // ---- per-lane LDS read pointers (loop invariant; tile slot, nb, ks enter as immediate offsets)
    // K: row l32 (+32*nb), chunk (2*kk + g) ^ kswz(row)
    lds_ptr k_rptr[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        k_rptr[kk] = lds + l32 * G::ROW + (((2 * kk + g) ^ G::kswz(l32)) << 4);
        TSDPA_OPAQUE(k_rptr[kk]);
    }
    // V (transposing read): row g*4 + (lane%16)/4 (+ multiples of 8), 64-byte block db ^ vswz(row),
    // then 32 B for the upper 16 lanes of each 32 and 8 B per lane%4
    const int v_row = g * 4 + ((lane & 15) >> 2);
    lds_ptr v_rptr[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        v_rptr[db] = lds + v_row * G::ROW + ((db ^ G::vswz(v_row)) << 6) + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;
        TSDPA_OPAQUE(v_rptr[db]);
    }

    // scores, transposed: sacc[nb][i] = <k_row, q_col>, row = nb*32 + (i/4)*8 + g*4 + i%4, col = l32
    auto scores = [&](int kslot, f32x16 (&sacc)[NB], auto &&after_kstep) __attribute__((always_inline)) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[nb][i] = 0.f;
        if constexpr (NB == 1 && KK <= 8) {
            // 32-row tiles (the register-lean instantiations): all operand reads first, then the MFMA
            // chain.  The scheduling barrier keeps the compiler from sinking each read next to its MFMA,
            // where the LDS latency would be paid once per MFMA instead of once per tile (+2-4 %).
            u32x4 kb[KK];
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) kb[kk] = lds_read128(k_rptr[kk] + kslot);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                sacc[0] = E::mfma(__builtin_bit_cast(vec8, kb[kk]), qf[kk], sacc[0]);
                after_kstep(kk);
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {   // nb innermost: independent accumulators alternate
                    u32x4 raw = lds_read128(k_rptr[kk] + kslot + nb * 32 * G::ROW);
                    sacc[nb] = E::mfma(__builtin_bit_cast(vec8, raw), qf[kk], sacc[nb]);
                }
                after_kstep(kk);
            }
        }
    };

    // Eq. 2 on one tile of scores, for the rows whose weights overflowed the limit (`over`; the two lanes
    // that share a row decide together): tile maximum, new reference and the rescale of Eqs. 3-4.
    auto raise_reference = [&](f32x16 (&sacc)[NB], int row0, auto mask_tag, bool over) __attribute__((always_inline)) {
        constexpr bool MASK = decltype(mask_tag)::value;
        const int key0 = row0 + g * 4;
        if constexpr (MASK) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (key0 + nb * 32 + (i >> 2) * 8 + (i & 3) > klim) sacc[nb][i] = -INFINITY;
        }
        float mx = sacc[0][0];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[nb][i]);
        mx = pair_max(mx);
        const float m_tile = mx * c;
        const bool row_over = pair_max(over ? 1.f : 0.f) > 0.f;
        // rows that keep m_ref are left alone (also one whose keys so far were all masked: m_ref = -inf,
        // m_tile = -inf or NaN)
        const bool grow = row_over && m_tile > m_ref;
        const float alpha = grow ? __builtin_amdgcn_exp2f(m_ref - m_tile) : 1.0f;
        m_ref = grow ? m_tile : m_ref;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
    };
    // p = 2^(s*c - m_ref); Eq. 3 sums the unrounded FP32 p (this lane's share of the tile is returned),
    // the PV product uses the 16-bit rounded p, left in pb as MFMA B-operands
    auto exponentials = [&](f32x16 (&sacc)[NB], int row0, vec8 (&pb)[NB][2], auto mask_tag) __attribute__((always_inline)) {
        constexpr bool MASK = decltype(mask_tag)::value;
        const int key0 = row0 + g * 4;
        float psum[4];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[nb][i], c, -m_ref));
                if constexpr (MASK) {
                    if (key0 + nb * 32 + (i >> 2) * 8 + (i & 3) > klim) p = 0.f;
                }
                if (nb == 0 && i < 4) psum[i] = p;        // four partial sums: short dependency chains
                else psum[i & 3] += p;
                pb[nb][i >> 3][i & 7] = (T)p;
            }
        return (psum[0] + psum[1]) + (psum[2] + psum[3]);
    };

    // Eq. 4: O^T += V^T P^T
    auto accumulate = [&](int vslot, const vec8 (&pb)[NB][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    // k-slots 0..3 / 4..7 of this lane <-> key rows base+g*4+0..3 / base+8+g*4+0..3
                    const lds_ptr p0 = v_rptr[db] + vslot + (nb * 32 + ks * 16) * G::ROW;
                    i16x4 lo = lds_read_tr16(p0);
                    i16x4 hi = lds_read_tr16(p0 + 8 * G::ROW);
                    i16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    oacc[db] = E::mfma(__builtin_bit_cast(vec8, a), pb[nb][ks], oacc[db]);
                }
    };

    f32x16 sacc[NB];
    vec8 pb[NB][2];
    // weights of the key rows row0 ... row0 + TNS - 1 (with the lazy reference), this lane's share of their
    // sum added to l_run
    auto softmax_tile = [&](int row0, auto mask_tag) __attribute__((always_inline)) {
        float ps = exponentials(sacc, row0, pb, mask_tag);
        const bool over = !(ps <= lazy_limit);               // also catches inf (first tile) and NaN
        if (__builtin_amdgcn_ballot_w64(over) != 0) {        // wavefront-uniform and rare
            raise_reference(sacc, row0, mask_tag, over);
            ps = exponentials(sacc, row0, pb, mask_tag);
        }
        l_run += ps;
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    // ---- main loop, unrolled by two so that the LDS slots alternate by name.  In step j the LDS holds
    // K(j) and V(j); K(j+1) and V(j+1) are in flight into the other slots, whose last readers finished
    // before the barrier that ended step j-1.  Overlap of matrix and vector work comes from the
    // wavefronts that share a SIMD (an in-wavefront software pipeline that ran the scores one tile
    // ahead cost 32 registers and measured 4 % slower).
    // tiles below nfull need no mask: they run in pairs through the unmasked step; the few tiles
    // left (the diagonal band under the causal mask, the ragged tail, an odd one out) take the
    // masked path, which is also correct for a tile that turns out to need no mask
    const int fast_n = (t1 < nfull ? t1 : nfull) - t0;
    const int fast_end = t0 + (fast_n > 0 ? fast_n & ~1 : 0);
    // Dense cache with one query tile per head (decoding): every workgroup streams another head, and
    // heads lie a power of two apart, so workgroups that all start at their tile 0 and advance in step
    // keep hitting the same memory channels.  The order of the unmasked tiles is free (Eqs. 2-4 do not
    // care), so each workgroup starts its sweep at a tile of its own and wraps around.
    int rot = 0;
    if constexpr (KVM == 1) {
        const int nf = fast_end - t0;
        if (tile_rot != 0 && nf > 2) rot = (int)((((unsigned)hs * 2654435761u) >> 12) % (unsigned)nf);
    }
    if (!KV || t0 < t1) {   // a split past the diagonal has no tile: its state stays (o, m, l) = (0, -inf, 0)
    if constexpr (PAGED) {
        const int blk0 = (t0 * TN) >> block_shift;
        page_next = __builtin_amdgcn_readfirstlane(pages[blk0 < max_blocks ? blk0 : 0]);
    }
    if constexpr (KVM == 0) {
        // A wavefront whose 32 rows all lie past the end of the sequence (the last query tile of a ragged S)
        // has nothing to compute or store: it only takes its share of the tile loads and keeps the
        // workgroup's barriers, leaving its SIMD's matrix and vector slots to the wavefronts that have rows.
        if (r0 + wave * 32 >= S) {
            load_tiles(t0, lds + KSLOT0, lds + VSLOT0);
            TSDPA_WAIT_VMCNT0();
            __syncthreads();
            for (int jj = t0; jj < t1; ++jj) {
                if (jj + 1 < t1) {
                    const int odd = (jj + 1 - t0) & 1;            // slot of tile jj + 1
                    load_tiles(jj + 1, lds + (odd ? KSLOT1 : KSLOT0), lds + (odd ? VSLOT1 : VSLOT0));
                }
                TSDPA_WAIT_VMCNT0();
                __syncthreads();
            }
            return;
        }
    }
    load_tiles(t0 + rot, lds + KSLOT0, lds + VSLOT0);
    TSDPA_WAIT_VMCNT0();
    __syncthreads();

    // tile j, followed by tile jn: PAR (alternating) selects the slots, MASK the masked code path
    auto step = [&](int j, int jn, auto par_tag, auto mask_tag) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_tag)::value;
        // The loads of tile jn go out one at a time between the score MFMAs: direct-to-LDS loads issued back
        // to back hold the wavefront at the issue stage while the CU's one address unit works through
        // them, and a SIMD with one resident wavefront has nothing else to run meanwhile (one workgroup
        // per CU: -12 % time; two or three per CU: -0.5 to -2 %; the 32-row tile at D = 160 alone is 6 %
        // slower that way and keeps its loads at the start of the step).  A tile this workgroup does not
        // need is fetched from past the end of the descriptor: no memory access, zeros written to a slot
        // that nobody reads before the wait that ends the step.
        constexpr bool SPREAD = NB >= 2 || D <= 128;
        const lds_ptr kdst = lds + (PAR ? KSLOT0 : KSLOT1), vdst = lds + (PAR ? VSLOT0 : VSLOT1);
        const TileSrc ksrc = tile_src(k, k_rsrc, jn), vsrc = tile_src(v, v_rsrc, jn);
        if constexpr (!SPREAD) {
            if (jn < t1) {
#pragma unroll
                for (int i = 0; i < L; ++i) issue(ksrc, vsrc, kdst, vdst, i);
            }
        }
        // the MFMAs of a step form chains fed by LDS reads: a raised wavefront priority lets them go
        // ahead of the other wavefronts' vector work whenever their operands are ready (+1-3 %), and
        // the PV chain, whose end releases the workgroup's barrier, goes ahead of other score chains
        // (+0.5-2 % more)
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub) {
            // (halves strictly one after the other: the scheduler would otherwise start the scores of the
            // second beside the softmax of the first and hold both sets of score accumulators)
            if (sub > 0) __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(1);
            scores((PAR ? KSLOT1 : KSLOT0) + sub * TNS * G::ROW, sacc, [&](int kk) __attribute__((always_inline)) {
                if constexpr (SPREAD) {
                    constexpr int HOOKS = NSUB * KK;
                    const int h = sub * KK + kk;
#pragma unroll
                    for (int i = h * L / HOOKS; i < (h + 1) * L / HOOKS; ++i) issue(ksrc, vsrc, kdst, vdst, i);
                    // MFMAs and loads keep this order (LDS reads, vector and scalar instructions may still move)
                    __builtin_amdgcn_sched_barrier(0x786);
                }
            });
            __builtin_amdgcn_s_setprio(0);
            softmax_tile(j * TN + sub * TNS, mask_tag);
            __builtin_amdgcn_s_setprio(2);
            accumulate((PAR ? VSLOT1 : VSLOT0) + sub * TNS * G::ROW, pb);
            __builtin_amdgcn_s_setprio(0);
        }
        TSDPA_WAIT_VMCNT0();
        __syncthreads();
    };
    int j = t0;
    if constexpr (KVM == 1) {
        // unmasked tiles in rotated order: t0+rot ... fast_end-1, t0 ... t0+rot-1, then on to fast_end
        int cur = t0 + rot;
        for (; j < fast_end; j += 2) {
            int n1 = cur + 1;
            if (n1 == fast_end) n1 = t0;
            int n2 = n1 + 1;
            if (n2 == fast_end) n2 = t0;
            if (j + 2 >= fast_end) n2 = fast_end;
            step(cur, n1, P0{}, std::false_type{});
            step(n1, n2, P1{}, std::false_type{});
            cur = n2;
        }
    } else {
        for (; j < fast_end; j += 2) {
            step(j, j + 1, P0{}, std::false_type{});
            step(j + 1, j + 2, P1{}, std::false_type{});
        }
    }
    for (; j < t1; ++j) {
        if ((j - t0) & 1) step(j, j + 1, P1{}, std::true_type{});
        else              step(j, j + 1, P0{}, std::true_type{});
    }
    }

    // ---- O_i = o_i / l_i (Section 4.1.2), rounded once to the 16-bit output type.  The accumulators
    // hold O^T (a lane owns one query row and scattered groups of 4 columns), so the tile is turned
    // through LDS: each wavefront writes its 32 x D block into its own LDS region (16-byte chunks
    // XOR-swizzled by row against bank conflicts) and reads it back as whole rows, so that every global
    // store instruction writes complete, contiguous rows (16 B per lane) instead of 8-byte pieces.
    const float l_tot = pair_sum(l_run);
    if (KV && splits > 1) {
        // partial state of this split: the accumulators as they are (a lane owns query row qrow and
        // groups of 4 consecutive columns), then the reference m and the normaliser l
        const size_t prow = (size_t)(head * splits + sp) * S + qrow;
        if (qrow < S) {
            float *po = ws + prow * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4 part;
#pragma unroll
                    for (int e = 0; e < 4; ++e) part[e] = oacc[db][q4 * 4 + e];
                    *(f32x4 *)(po + db * 32 + q4 * 8 + g * 4) = part;
                }
            if (g == 0) {
                float *pml = ws + (size_t)(N / nQ) * S * D + prow * 2;   // N / nQ = BH * splits
                pml[0] = m_ref;
                pml[1] = l_tot;
            }
        }
        return;
    }
    // a row that no key reaches (empty cache entry, causal limit before the first key) has l = 0: O = 0, LSE = -inf
    // (only the cache variants can have such a row: in the square problem every row sees key 0)
    const bool no_key = KV && !(l_tot > 0.f);
    const float inv = no_key ? 0.f : 1.0f / l_tot;
    if (lse != nullptr && g == 0 && qrow < S)
        lse[(size_t)head * S + qrow] = no_key ? -INFINITY : (m_ref + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
    // (the launcher sizes the dynamic LDS for the larger of the tile slots and this staging area)
    {
        constexpr int OCPR = G::OROW / 16, CMASK = OCPR - 1;   // chunks per staging row: a power of two
        const lds_ptr ow = lds + wave * (32 * G::OROW);
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                vec4 out;
#pragma unroll
                for (int e = 0; e < 4; ++e) out[e] = (T)(oacc[db][q4 * 4 + e] * inv);
                const int chunk = db * 4 + q4;        // columns chunk*8 .. +7 (< D); this lane owns half g of it
                *(TSDPA_LDS vec4 *)(ow + l32 * G::OROW + ((chunk ^ (l32 & CMASK)) << 4) + g * 8) = out;
            }
        // the region is private to this wavefront: LDS operations of one wavefront complete in order
        constexpr int ORPI = 64 / OCPR;               // rows per store instruction
        const int qrow0 = qt * TM + wave * 32;
#pragma unroll
        for (int i = 0; i < 32 / ORPI; ++i) {
            const int r = i * ORPI + lane / OCPR, cc = lane % OCPR;
            const u32x4 val = lds_read128(ow + r * G::OROW + ((cc ^ (r & CMASK)) << 4));
            if (qrow0 + r < S && cc < GCPR)
                *(u32x4 *)(o + head_off + (size_t)(qrow0 + r) * D + cc * 8) = val;
        }
    }
#endif
}

}  // namespace tsdpa
