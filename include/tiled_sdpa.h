/*
 * tiled_sdpa.h -- C-ABI of the MI355X (gfx950) tiled scaled-dot-product-attention
 * forward library.
 *
 * The operation is the paper's Eq. 1 (Section 3.1) with no mask,
 *
 *     O = softmax(Q K^T * scale) V        per (batch, head),
 *
 * evaluated blockwise with the online-softmax recurrence of Section 4.1.2
 * (Eqs. 2-4: running row maximum m, normaliser l and accumulator o over streamed
 * K/V tiles, final O_i = o_i / l_i), so the S x S score matrix never exists in
 * memory.  Numerics follow Section 4.1.3: FP16 or BF16 inputs and output, FP32
 * accumulation of the dot products, the softmax statistics and the output.
 * The call surface mirrors the functional API of Section 4.2.1,
 * sdpa(q, k, v, causal, scale) -> o; causal = true is TSDPA_FLAG_CAUSAL of tiled_sdpa_fwd_ex.
 *
 * All pointers are DEVICE pointers owned by the caller.  The library allocates
 * and frees nothing, keeps no state besides its kernel table, never
 * synchronises, and is thread-safe.  Work is enqueued on `stream`.
 */
#ifndef TILED_SDPA_H
#define TILED_SDPA_H

#ifdef __cplusplus
extern "C" {
#endif

/* element types (Section 4.1.3) */
enum { TSDPA_F16 = 0, TSDPA_BF16 = 1 };

/* status codes: every entry point returns one of these and never throws or aborts */
enum {
    TSDPA_OK = 0,
    TSDPA_ERR_NULL_PTR = 1,      /* q, k, v or o is NULL while B*H*S > 0                    */
    TSDPA_ERR_BAD_SHAPE = 2,     /* negative B, H or S; B*H*ceil(S/64) overflows int; (S+1024)*D*2 >= 2^30 */
    TSDPA_ERR_BAD_DTYPE = 3,     /* dtype is neither TSDPA_F16 nor TSDPA_BF16               */
    TSDPA_ERR_UNSUPPORTED_D = 4, /* D is not 64, 96, 128 or 160                             */
    TSDPA_ERR_MISALIGNED = 5,    /* a tensor base is not 16-byte aligned / lse not 4-byte   */
    TSDPA_ERR_BAD_TILE = 6,      /* (tile_m, tile_n) neither (256,64) nor in {64,128} x {32,64,128},
                                    tile_n = 128 at D = 160 (four such slots fill the LDS), or a
                                    tile the entry point does not offer                       */
    TSDPA_ERR_BAD_SCALE = 7,     /* scale is +-infinity                                     */
    TSDPA_ERR_LAUNCH = 8,        /* the HIP runtime refused the launch                      */
    TSDPA_ERR_WORKSPACE = 9,     /* tiled_sdpa_fwd_kv with more than one split, tiled_sdpa_bwd: workspace NULL,
                                    not 16-byte aligned, or smaller than the matching *_workspace_bytes reports */
    TSDPA_ERR_BAD_SPLITS = 10,   /* splits < 0 or > TSDPA_MAX_SPLITS                         */
    TSDPA_ERR_STATIC_SCRATCH = 11 /* tiled_sdpa_fwd_kvcache_static: the split states need more than
                                    TSDPA_STATIC_SCRATCH_BYTES, or the buffer's address cannot be obtained */
};

enum { TSDPA_MAX_SPLITS = 128 };
enum { TSDPA_TUNE_TILES = 7 };      /* candidates of tiled_sdpa_tune_tile */

/* size of the library-owned device buffer behind tiled_sdpa_fwd_kvcache_static (32 MiB per GPU) */
enum { TSDPA_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024 };

/* flags for tiled_sdpa_fwd_ex */
enum {
    TSDPA_FLAG_LINEAR_GRID = 1u, /* workgroup i handles tile i (no per-XCD regrouping); for measurements */
    TSDPA_FLAG_EXACT_MAX = 2u,   /* raise the softmax reference m on every new row maximum (Eq. 2 literally).
                                    Default: the weights of a tile are taken against the current reference
                                    first, and it is raised (to the tile maximum, with the rescale of
                                    Eqs. 3-4) only when their sum exceeds 2^8; this gives the same O and lse
                                    up to rounding and spares most tiles the maximum and the rescale.  With
                                    the flag most tiles are computed twice: for checking, not for speed. */
    TSDPA_FLAG_CAUSAL = 8u       /* causal mask (Section 4.1.3; Eq. 1 with M_ij = -inf for j > i): key j
                                    contributes to query row i only if j <= i.  K/V tiles strictly above
                                    the diagonal of a workgroup's rows are neither read nor computed. */
};

/*
 * Forward pass, Eq. 1 via Eqs. 2-4.
 *
 *   q, k, v : [B, H, S, D] contiguous row-major, element type `dtype`, device memory,
 *             16-byte aligned (Section 4.1.1 layout; viewed as [B*H, S, D] and tiled along S).
 *   o       : [B, H, S, D], same type; every element is overwritten.  Must not alias q, k, v.
 *   lse     : optional (NULL to skip) FP32 [B, H, S]; receives m_i + ln(l_i), the natural-log
 *             normaliser of row i, which is what merging partial results over key ranges needs.
 *   S       : any length >= 0; key columns beyond S contribute nothing and rows beyond S are
 *             neither computed into memory nor read past the tensor end.
 *   D       : 64, 96, 128 or 160 (the head dims of the paper's grid, Section 4.3).
 *   scale   : multiplies Q K^T; any finite value.  NaN selects the default 1/sqrt(D)
 *             (Section 4.2.1), since C has no default arguments.
 *   stream  : hipStream_t (NULL = default stream).  The call returns once the kernel is enqueued.
 *
 * Validation order: dtype, D, shape, empty problem (B*H*S == 0 returns TSDPA_OK without
 * touching memory), null pointers, alignment, tile, scale, launch.
 */
int tiled_sdpa_fwd(const void *q, const void *k, const void *v, void *o, float *lse,
                   int B, int H, int S, int D, float scale, int dtype, void *stream);

/*
 * Same operation with the schedule exposed (Table 1 of the paper: T_M query rows per
 * workgroup, T_N key/value rows per streamed tile).  tile_m in {64,128}, tile_n in
 * {32,64,128} (128 not at D = 160), or (tile_m, tile_n) = (256, 64), which is not in the paper's grid: eight
 * wavefronts share every K/V tile, the fastest schedule on this GPU for long sequences at D >= 96 without the
 * causal mask.
 * tile_m = tile_n = 0 selects the built-in shape heuristic, which is what tiled_sdpa_fwd uses.  The
 * result does not depend on the tile choice beyond rounding order.
 */
int tiled_sdpa_fwd_ex(const void *q, const void *k, const void *v, void *o, float *lse,
                      int B, int H, int S, int D, float scale, int dtype, void *stream,
                      int tile_m, int tile_n, unsigned flags);

/* The (tile_m, tile_n) the heuristic picks for a shape and flags (only TSDPA_FLAG_CAUSAL matters);
 * returns a status code. */
int tiled_sdpa_default_tile(int B, int H, int S, int D, int dtype, unsigned flags, int *tile_m, int *tile_n);

/*
 * Schedule search (the tuning policy of Table 1 and Sections 5.5-5.6: a small set of tile candidates, the
 * best one kept per problem shape): runs the forward pass of tiled_sdpa_fwd_ex with every legal
 * (tile_m, tile_n) on the caller's tensors -- one untimed launch, then `launches` (1..1000) timed
 * ones between two HIP events on `stream` -- and reports the fastest in *tile_m, *tile_n.  Unlike
 * every other entry point this one WAITS for the stream (once per candidate); it keeps no record, the
 * caller passes the result to tiled_sdpa_fwd_ex.  o is overwritten (with the correct result).
 * ms_per_launch: NULL, or host array of TSDPA_TUNE_TILES (7) floats that receives the time per launch of
 * (64,32) (64,64) (64,128) (128,32) (128,64) (128,128) (256,64) in that order, -1 for a tile that is not
 * offered at this D.  An empty problem returns the heuristic's tile and measures nothing.
 * Validation as tiled_sdpa_fwd_ex; launches out of range is TSDPA_ERR_BAD_SHAPE; tile_m or tile_n
 * NULL is TSDPA_ERR_NULL_PTR.  Timings are only meaningful on an otherwise idle GPU (Section 4.2.3).
 */
int tiled_sdpa_tune_tile(const void *q, const void *k, const void *v, void *o,
                         int B, int H, int S, int D, float scale, int dtype, void *stream, unsigned flags,
                         int launches, int *tile_m, int *tile_n, float *ms_per_launch);

/*
 * Forward pass for Sq query rows against Skv key/value rows, with the key range optionally split
 * over several workgroups: the KV-cache / decoding shapes that the paper names as future work
 * (Section 7), and the cure for shapes whose B*H*ceil(Sq/tile_m) workgroups cannot fill the GPU.
 * Each split runs the recurrence of Section 4.1.2 (Eqs. 2-4) over its own contiguous run of K/V
 * tiles and leaves its state (o, m, l) in the workspace; a second kernel combines the states with
 * the rescaling of Eqs. 3-4 and applies the final O_i = o_i / l_i.
 *
 *   q        : [B, H, Sq, D];  k, v : [B, H, Skv, D];  o : [B, H, Sq, D];  lse : NULL or FP32 [B, H, Sq].
 *              Layout, alignment, D, scale, dtype, stream as for tiled_sdpa_fwd.
 *   flags    : TSDPA_FLAG_CAUSAL takes the Sq queries to be the LAST Sq positions of the Skv-long
 *              sequence (the paper defines the mask for Sq = Skv only): key j contributes to query
 *              row i only if j <= i + Skv - Sq.  It needs Skv >= Sq.  The other flags as above.
 *   tile_m   : 64 or 128;  tile_n : 32 or 64;  or (256, 64) (not with a paged cache);  both 0 = heuristic.
 *   splits   : workgroups per (head, query tile) along the key axis, 1..TSDPA_MAX_SPLITS; 0 = the
 *              value tiled_sdpa_kv_default_splits reports for this shape and these flags.
 *   workspace: device memory for the split states, 16-byte aligned, at least
 *              tiled_sdpa_kv_workspace_bytes(B, H, Sq, D, n) bytes, n being `splits` or, for splits = 0,
 *              the heuristic's value; ignored (may be NULL) when n = 1, where O is written directly.
 *              Owned by the caller; the library uses it only between the two kernels of this call, so
 *              calls that may overlap on the GPU need distinct workspaces.  Its contents afterwards
 *              are unspecified.  More splits than there are K/V tiles are allowed (the surplus ones
 *              contribute nothing) but waste workspace.
 *
 * Skv = 0 with Sq > 0 is TSDPA_ERR_BAD_SHAPE (a softmax over no keys).  Validation order: dtype, D,
 * shape, empty problem (B*H*Sq == 0), null pointers, alignment, tile, scale, splits, workspace, launch.
 */
int tiled_sdpa_fwd_kv(const void *q, const void *k, const void *v, void *o, float *lse,
                      int B, int H, int Sq, int Skv, int D, float scale, int dtype, void *stream,
                      int tile_m, int tile_n, unsigned flags,
                      int splits, void *workspace, unsigned long long workspace_bytes);

/*
 * tiled_sdpa_fwd_kv with grouped heads: H query heads read Hkv key/value heads, query head h the
 * key/value head h / (H / Hkv) -- the layout of multi-query and grouped-query KV caches.  The paper
 * has one key/value head per query head (Section 3.1); per query head this computes the same Eq. 1,
 * with the causal limit of tiled_sdpa_fwd_kv for each head's Sq rows.
 *
 *   q, o : [B, H, Sq, D];  lse : NULL or FP32 [B, H, Sq];  k, v : [B, Hkv, Skv, D];  H % Hkv == 0.
 *   Everything else as for tiled_sdpa_fwd_kv, which is this call with Hkv = H.  The heuristics see
 *   B * Hkv heads of (H / Hkv) * Sq rows each: tiled_sdpa_kv_default_splits(B, Hkv, (H / Hkv) * Sq, ...)
 *   without the causal flag reports the split count used for splits = 0, and the workspace size is
 *   tiled_sdpa_kv_workspace_bytes(B, H, Sq, D, n).
 *
 * The query heads of a group are adjacent in memory, so a group's (H / Hkv) * Sq rows form one run of
 * rows that streams the group's keys and values once (instead of once per query head): on a
 * decoding step the otherwise empty rows of the 32-row MFMA tile carry the other heads of the
 * group.  Hkv <= 0 with H > 0, or H not a multiple of Hkv, is TSDPA_ERR_BAD_SHAPE (checked right
 * after the shape checks of tiled_sdpa_fwd_kv).
 */
int tiled_sdpa_fwd_gqa(const void *q, const void *k, const void *v, void *o, float *lse,
                       int B, int H, int Hkv, int Sq, int Skv, int D, float scale, int dtype, void *stream,
                       int tile_m, int tile_n, unsigned flags,
                       int splits, void *workspace, unsigned long long workspace_bytes);

/*
 * tiled_sdpa_fwd_gqa over a KV cache whose batch entries are filled to different lengths (the
 * serving form of the KV-cache variants the paper names as future work, Section 7): k and v are
 * [B, Hkv, Skv, D] with Skv the CAPACITY of the cache, and batch entry b holds kv_lens[b] valid key
 * rows at the front of each of its heads.
 *
 *   kv_lens : device pointer to B 32-bit integers, 4-byte aligned, read by the kernels when they run
 *             (not by this call); values are clamped to [0, Skv].  NULL = every entry holds Skv rows,
 *             which is tiled_sdpa_fwd_gqa.
 *
 * Entry b is computed as tiled_sdpa_fwd_gqa would compute it on its first kv_lens[b] key rows: rows
 * past the length are never fetched, and under TSDPA_FLAG_CAUSAL the Sq queries are the last Sq
 * positions of the kv_lens[b]-long sequence (key j contributes to query row i only if
 * j <= i + kv_lens[b] - Sq).  A query row that no key reaches -- an empty entry, or under the causal
 * flag an entry shorter than Sq for its first Sq - kv_lens[b] rows -- gets O = 0 and LSE = -infinity
 * (a softmax over no keys has no value; zero is what leaves a residual stream untouched).  Shapes are
 * validated against the capacity; the split heuristic sees the capacity too, so workspace sizes do not
 * depend on the lengths.  Everything else as for tiled_sdpa_fwd_gqa.
 */
int tiled_sdpa_fwd_kvcache(const void *q, const void *k, const void *v, void *o, float *lse, const int *kv_lens,
                           int B, int H, int Hkv, int Sq, int Skv, int D, float scale, int dtype, void *stream,
                           int tile_m, int tile_n, unsigned flags,
                           int splits, void *workspace, unsigned long long workspace_bytes);

/*
 * tiled_sdpa_fwd_kvcache for callers that cannot allocate device memory and so have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The split
 * states go to a buffer of TSDPA_STATIC_SCRATCH_BYTES that is part of the library's device code (a
 * file-scope __device__ array: every GPU the library runs on holds its own copy from the first use of
 * the library on it until the process ends).  The call itself allocates and frees nothing and does not
 * synchronise; the first call on a device looks the buffer's address up once.
 *
 *   All arguments as for tiled_sdpa_fwd_kvcache (kv_lens NULL = a full cache, Hkv = H = plain heads),
 *   minus the workspace.  Results are bit-identical to tiled_sdpa_fwd_kvcache with the same tile and
 *   split count: the same kernels run.
 *   Limit: tiled_sdpa_kv_workspace_bytes(B, H, Sq, D, n) <= TSDPA_STATIC_SCRATCH_BYTES, n being `splits`
 *   or the heuristic's count for splits = 0; beyond it the call enqueues nothing and returns
 *   TSDPA_ERR_STATIC_SCRATCH (pass fewer splits, or use tiled_sdpa_fwd_kvcache).  n = 1 needs no scratch.
 *   Nothing in the buffer has to start at zero: every word the second kernel reads is written by the
 *   first kernel of the same call; its contents after a call are unspecified.
 *   ALL calls on one GPU share that GPU's buffer: calls that may overlap on the GPU (different streams,
 *   or graphs replayed concurrently) race on it and must be serialised by the caller; calls on one
 *   stream are ordered and safe.
 *
 * Validation order: dtype, D, shape, empty problem, splits, tile (when the heuristic split count needs
 * it), static-scratch size, then everything tiled_sdpa_fwd_kvcache checks.
 */
int tiled_sdpa_fwd_kvcache_static(const void *q, const void *k, const void *v, void *o, float *lse,
                                  const int *kv_lens, int B, int H, int Hkv, int Sq, int Skv, int D, float scale,
                                  int dtype, void *stream, int tile_m, int tile_n, unsigned flags, int splits);

/*
 * tiled_sdpa_fwd_kvcache over a PAGED cache (the KV-cache variants of the paper's roadmap, Section 7,
 * in the form serving systems store them): keys and values live in pages of block_rows rows that any
 * batch entry may own in any order.
 *
 *   k_pages, v_pages : [P, Hkv, block_rows, D], P pages (P is not passed: the table names the pages);
 *                      16-byte aligned.  block_rows is 64, 128, 256, ... (a power of two >= 64, so that a
 *                      K/V tile of 32 or 64 rows lies within one page).
 *   block_table      : device, int32 [B, max_blocks], 4-byte aligned: block_table[b][i] is the page
 *                      holding key rows i*block_rows ... (i+1)*block_rows - 1 of batch entry b.  Only
 *                      the entries below ceil(kv_lens[b] / block_rows) are used; the others may hold
 *                      anything.  The pages named must exist; the library cannot check that.
 *   kv_lens          : device, int32 [B]: valid key rows of entry b, clamped to
 *                      [0, max_blocks * block_rows].  Required (not NULL).
 *   q, o, lse, H, Hkv, Sq, D, scale, dtype, stream, tiles, flags, splits, workspace: as for
 *                      tiled_sdpa_fwd_kvcache with capacity Skv = max_blocks * block_rows (that is
 *                      what shapes are validated against and what the split heuristic sees).
 *
 * Both arrays are read by the kernels when they run.  Every K/V tile is fetched through a buffer
 * descriptor of its own that starts at the tile's rows within its page and is as long as the tile has
 * valid rows, so neither rows past kv_lens[b] nor pages past the last one are touched.  Results are
 * those of tiled_sdpa_fwd_kvcache on the same rows gathered into a dense cache.  block_rows not a
 * power of two >= 64, max_blocks < 0 or max_blocks * block_rows overflowing an int is
 * TSDPA_ERR_BAD_SHAPE; kv_lens or block_table NULL with B*H*Sq > 0 is TSDPA_ERR_NULL_PTR.
 */
int tiled_sdpa_fwd_paged(const void *q, const void *k_pages, const void *v_pages, void *o, float *lse,
                         const int *kv_lens, const int *block_table,
                         int B, int H, int Hkv, int Sq, int max_blocks, int block_rows, int D,
                         float scale, int dtype, void *stream, int tile_m, int tile_n, unsigned flags,
                         int splits, void *workspace, unsigned long long workspace_bytes);

/* Splits the heuristic picks (1 when the query tiles alone fill the GPU); returns a status code. */
int tiled_sdpa_kv_default_splits(int B, int H, int Sq, int Skv, int D, int dtype, unsigned flags, int *splits);

/* Workspace bytes tiled_sdpa_fwd_kv needs for `splits` >= 1 (a value from tiled_sdpa_kv_default_splits,
 * or the caller's own): B*H*splits*Sq*(D+2) floats.  0 for splits <= 1 or negative arguments. */
unsigned long long tiled_sdpa_kv_workspace_bytes(int B, int H, int Sq, int D, int splits);

/*
 * Backward pass: gradients of a scalar loss with respect to q, k and v, given dout = d(loss)/d(o).
 * The paper leaves the backward pass as future work (Section 7); this is the derivative of its
 * Eq. 1 (Section 3.1), evaluated tile by tile with the probabilities recomputed from the forward
 * pass's log-sum-exp (never stored), in FP32 with 16-bit MFMA operands as in Section 4.1.3:
 *     P = exp(scale * Q K^T [+ causal mask] - lse),  dV = P^T dO,  dP = dO V^T,
 *     dS = P * (dP - rowsum(dO * O)),  dQ = scale * dS K,  dK = scale * dS^T Q.
 *
 *   q, k, v, o, dout : [B, H, S, D] as for tiled_sdpa_fwd; o and lse are that call's outputs for the
 *                      same q, k, v, scale and flags (lse is required here).
 *   dq, dk, dv       : [B, H, S, D], same type; every element is overwritten.  Must not alias inputs.
 *   flags            : TSDPA_FLAG_CAUSAL or 0.
 *   workspace        : device memory, 16-byte aligned, at least tiled_sdpa_bwd_workspace_bytes(B, H, S)
 *                      bytes (two FP32 values per query row); caller-owned, used only during this call's
 *                      kernels, so calls that may overlap on the GPU need distinct workspaces.
 * Kernels enqueued on `stream`: row statistics (Delta_i = <dO_i, O_i> and LSE_i in log2 units); for query
 * rows that see at most 64 keys (S <= 64, or the first 64 rows under the causal mask) a second small
 * kernel that replaces Delta_i by its definition sum_j P_ij dP_ij in FP32 (on such rows the rounding of
 * the 16-bit o inside <dO_i, O_i> is not attenuated by small P_ij); then the keys-resident gradients (one
 * fused dK + dV pass at D = 64, a dV pass and a dK pass at D = 96, 128, 160), then dQ.  No sum crosses
 * workgroups, so results are deterministic.  Validation order: dtype, D, shape, empty problem, null
 * pointers, alignment, scale, workspace, launch.
 */
int tiled_sdpa_bwd(const void *q, const void *k, const void *v, const void *o, const void *dout,
                   const float *lse, void *dq, void *dk, void *dv,
                   int B, int H, int S, int D, float scale, int dtype, unsigned flags,
                   void *workspace, unsigned long long workspace_bytes, void *stream);

/*
 * tiled_sdpa_bwd with grouped heads (the backward pass of tiled_sdpa_fwd_gqa at Sq = Skv = S): H query
 * heads read Hkv key/value heads, query head h the head h / (H / Hkv).  q, o, dout, dq : [B, H, S, D];
 * lse : [B, H, S];  k, v, dk, dv : [B, Hkv, S, D].  dq is the gradient of each query head against the
 * keys and values of its group; dk and dv are the gradients summed over the query heads of the group
 * (the chain rule of sharing one head among them), accumulated in FP32 inside one workgroup per
 * (key/value head, key tile), in a fixed order: results are deterministic.  Workspace as for
 * tiled_sdpa_bwd(B, H, S).  Everything else, validation included, as tiled_sdpa_bwd, which is this call
 * with Hkv = H; Hkv <= 0 with H > 0 or H not a multiple of Hkv is TSDPA_ERR_BAD_SHAPE.
 */
int tiled_sdpa_bwd_gqa(const void *q, const void *k, const void *v, const void *o, const void *dout,
                       const float *lse, void *dq, void *dk, void *dv,
                       int B, int H, int Hkv, int S, int D, float scale, int dtype, unsigned flags,
                       void *workspace, unsigned long long workspace_bytes, void *stream);

/* Workspace bytes tiled_sdpa_bwd needs: 2 * (B*H*S + 128) floats.  0 for negative arguments. */
unsigned long long tiled_sdpa_bwd_workspace_bytes(int B, int H, int S);

/*
 * Measurement aid, not part of the attention path: enqueue a register-resident stream of
 * v_mfma_f32_32x32x16 (FP16 or BF16 per `dtype`) on every SIMD of the GPU -- 512 workgroups of four
 * wavefronts, `iters` x 64 MFMAs per wavefront -- so the caller can time what the matrix pipe
 * sustains with no memory traffic.  random_operands != 0 fills the operand registers with random
 * signs and mantissas (the switching activity of real data, under which the chip lowers its
 * clock); 0 uses constant ones; 2 is the random-operand stream with the rest of the attention
 * loop's instruction mix added at the loop's own ratios and independent of the MFMAs (per MFMA one
 * 16-byte-per-lane LDS read and 3.7 vector instructions, a quarter of them exponentials): the rate
 * that mix sustains when nothing ever waits for anything.  sink: device buffer of at least 512*256 floats, overwritten.
 * flops (host pointer, may be NULL) receives the flop count of the launch.  The Section 4.2.3
 * policy of measuring on an otherwise idle GPU applies.  Returns a status code; iters = 0 only
 * reports flops (nothing is launched and sink may then be NULL; with iters > 0 a NULL sink is
 * TSDPA_ERR_NULL_PTR).
 */
int tiled_sdpa_probe_mfma(int dtype, int random_operands, int iters, float *sink, double *flops,
                          void *stream);

/*
 * Measurement aid, not part of the attention path: enqueue a kernel that reads `bytes` of device memory at
 * `src` once (8192 workgroups, each a contiguous run, four 16-byte loads per lane in flight) and writes
 * nothing but one word per workgroup into `sink` (device, at least 512*256 floats).  What a decoding step
 * (Section 7: reading the K/V cache once is all it does) can be compared with besides the published
 * HBM figure: the rate a pure read stream sustains on this GPU.  src: device, 16-byte aligned; bytes: at
 * least 128 MiB (smaller is refused as a bad shape), the part that does not fill a whole loop trip of every
 * workgroup is not read; bytes_read (host pointer, may be NULL) receives the bytes the launch does read.
 * Returns a status code.
 */
int tiled_sdpa_probe_hbm_read(const void *src, unsigned long long bytes, float *sink, double *bytes_read,
                              void *stream);

/* Human-readable text for a status code (static storage, never NULL). */
const char *tiled_sdpa_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int tiled_sdpa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TILED_SDPA_H */
