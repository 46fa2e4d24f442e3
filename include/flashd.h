/*
 * libflashd -- the FlashAttention forward pass in the FLASH-D form, for AMD MI355X (gfx950).
 *
 * What is computed (Sec. II-A, problem statement): for every batch b, query head h and
 * query row i,
 *
 *     s_j = scale * dot(q[b,h,i,:], k[b,kvh,j,:])          kvh = h / (Hq / Hkv)
 *     o[b,h,i,:] = sum_j softmax_j(s)_j * v[b,kvh,j,:]      over the keys j visible to i
 *
 * How it is computed (Sec. III, Alg. 3): the output is built key by key as the blend
 * o_i = o_{i-1} + (v_i - o_{i-1}) w_i with w_1 = 1 and
 * w_i = sigmoid(s_i - s_{i-1} + ln w_{i-1}); there is no running maximum, no running sum of
 * exponentials and no division of the output.  Runs of keys (tiles, split-K partitions) are
 * folded by the same rule, a run acting as one key whose score is s_last - ln w_last.
 * That is literally what PER_KEY does per key and TILE_BLEND per tile of keys.  The default
 * matrix-core variant TILE does not apply the (1 - W) factor of each tile to the accumulator
 * but carries their product as one scalar beta per row and multiplies it in at the store; in
 * that form 1/beta is a sum of exponentials 2^(s_j - R) against a reference R that moves only
 * when a score would overflow, so compared with Alg. 2 it drops the running maximum and the
 * per-tile rescaling of the accumulator, not the sum.
 *
 * Conventions shared by every entry point
 *   - q, k, v, o and workspace are DEVICE pointers owned by the caller; the library never
 *     frees or keeps them beyond the work it enqueues.  They must be 16-byte aligned.
 *   - Layout, row-major and contiguous: q, o: [B][Hq][Lq][d];  k, v: [B][Hkv][Lk][d];
 *     all four in the storage type named by `dtype`.  o must not overlap an input.
 *   - B, Hq, Hkv, Lq, Lk >= 1; Hq % Hkv == 0; d is 64 or 128.  B and Hq are at most 65535,
 *     Lq and Lk at most 10^9 and a tensor has at most 10^12 elements (else FLASHD_E_SHAPE).
 *   - causal != 0: key j is visible to query i iff j <= i + (Lk - Lq) (the last query sees
 *     every key).  A query row with no visible key yields zeros.  causal == 0: all keys.
 *   - `scale` multiplies the dot product in fp32; any finite value is taken as it is (zero
 *     weighs every visible key the same, a negative one turns the ranking of the keys
 *     round).  State and accumulation are fp32 for all storage types.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work and return; they do not synchronise.
 *   - Every function returns a flashd_status (0 = success, negative = error).  Argument errors
 *     are detected before any GPU call and leave nothing enqueued.  FLASHD_E_HIP can also come
 *     from a kernel launch that the runtime refuses after an earlier kernel of the same call
 *     (the fp8 widening, the main kernel before the merge of key splits) has been enqueued:
 *     the output is then undefined, the inputs untouched.
 *   - The entry points that take scratch memory from the cache allocate on first use and
 *     cannot be recorded into a HIP graph before that; flashd_attn_fwd_ex and
 *     flashd_attn_fwd_static never allocate.
 *   - For fixed inputs, variant and splits the output is bitwise reproducible.
 */
#ifndef FLASHD_H
#define FLASHD_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { FLASHD_F32 = 0, FLASHD_F16 = 1, FLASHD_BF16 = 2 } flashd_dtype;

typedef enum {
    FLASHD_OK = 0,
    FLASHD_E_NULL = -1,       /* q, k, v or o is NULL                                   */
    FLASHD_E_SHAPE = -2,      /* a dimension is < 1 or beyond the limits stated above   */
    FLASHD_E_DTYPE = -3,      /* dtype is not a flashd_dtype                            */
    FLASHD_E_HEADDIM = -4,    /* d is not 64 or 128                                     */
    FLASHD_E_GQA = -5,        /* Hq is not a multiple of Hkv                            */
    FLASHD_E_ALIGN = -6,      /* a pointer is not 16-byte aligned                       */
    FLASHD_E_WORKSPACE = -7,  /* workspace missing or smaller than flashd_workspace_bytes */
    FLASHD_E_HIP = -8,        /* a HIP call (allocation, launch) failed                 */
    FLASHD_E_ARCH = -9,       /* the current device is not gfx950                       */
    FLASHD_E_VARIANT = -10    /* variant/splits not valid for this problem              */
} flashd_status;

/* How the recurrence is evaluated.  All variants compute the same result. */
typedef enum {
    FLASHD_VARIANT_AUTO = 0,     /* TILE (or TILE_256) for f16/bf16, PER_KEY for f32        */
    FLASHD_VARIANT_TILE = 1,     /* Alg. 3 lifted to key tiles on the matrix cores (f16/bf16),
                                    the (1 - W) factors of the blend deferred to the store   */
    FLASHD_VARIANT_PER_KEY = 2,  /* Alg. 3 literally, one sigmoid per key (any dtype)       */
    FLASHD_VARIANT_ONLINE_SOFTMAX = 3, /* ablation: Alg. 2 (running max, sum, final division)
                                          on the same tiling as TILE (f16/bf16)             */
    FLASHD_VARIANT_TILE_BLEND = 4,     /* Alg. 3 on key tiles with the blend of Sec. III-A applied
                                          on every tile: o <- (1 - W) o + sum_j c_j v_j with
                                          W = sigmoid(Lam_tile - Lam) and c_j <= 1 (f16/bf16)  */
    FLASHD_VARIANT_TILE_256 = 5        /* TILE on the kernel with 256 query rows per workgroup
                                          (one wavefront per SIMD, matrix and vector work
                                          interleaved by hand) where it can serve the call:
                                          f16/bf16, d = 128, no splits, no state; any other
                                          call runs as TILE.  Same
                                          arithmetic; measured 6 to 16 % ahead of TILE on
                                          long inputs, level with it at 2048 causal keys
                                          and behind it on shorter ones: the automatic
                                          choice takes it where it is ahead
                                          (flashd_auto_variant)                            */
} flashd_variant;

/*
 * Attention forward, Alg. 3 (Sec. III-C).  Picks the variant and the number of key splits
 * itself (for decode shapes in f16/bf16 the kernel of flashd_attn_fwd_skipv, which leaves out
 * the value fetch of key blocks whose weights have all saturated at 0) and takes split-K
 * scratch memory from a grow-only cache kept per (device, stream);
 * the first call that needs a larger cache allocates (hipMalloc), later calls do not.
 * Safe to call from several host threads; calls that share a stream share its cache and are
 * ordered by the stream.
 */
int flashd_attn_fwd(const void* q, const void* k, const void* v, void* o,
                    int B, int Hq, int Hkv, int Lq, int Lk, int d,
                    int causal, float scale, int dtype, void* stream);

/*
 * Same computation with explicit knobs.
 *   variant   a flashd_variant; TILE, TILE_BLEND and ONLINE_SOFTMAX need f16/bf16 (else FLASHD_E_VARIANT).
 *   splits    number of consecutive key ranges reduced independently and then merged with
 *             the sigmoid rule; 0 = choose, 1 = no split; at most FLASHD_MAX_SPLITS and at
 *             most Lk (else FLASHD_E_VARIANT).
 *   workspace device memory of at least flashd_workspace_bytes(..., splits) bytes, used only
 *             while the enqueued work runs; may be NULL when that size is 0.  With
 *             splits == 0 pass the size for splits = 0, which covers whatever is chosen.
 * Never allocates.
 */
int flashd_attn_fwd_ex(const void* q, const void* k, const void* v, void* o,
                       int B, int Hq, int Hkv, int Lq, int Lk, int d,
                       int causal, float scale, int dtype, void* stream,
                       int variant, int splits, void* workspace, size_t workspace_bytes);

#define FLASHD_MAX_SPLITS 64

/*
 * Bytes of workspace flashd_attn_fwd_ex needs: one partial state (o[d], s, ln w) in fp32 per
 * (split, b, h, i) when more than one split is used (the state of Alg. 3, Sec. III-C), else 0.
 * splits == 0 returns the bound for the automatic choice.  Returns 0 for invalid arguments.
 */
size_t flashd_workspace_bytes(int B, int Hq, int Hkv, int Lq, int Lk, int d, int dtype,
                              int variant, int splits);

/* The number of splits the automatic choice takes for this problem (>= 1). */
int flashd_auto_splits(int B, int Hq, int Hkv, int Lq, int Lk, int d, int dtype, int variant);

/*
 * The variant flashd_attn_fwd (FLASHD_VARIANT_AUTO) runs for this problem: PER_KEY for f32,
 * else TILE, or TILE_256 for calls that kernel can serve and was measured faster on (d = 128,
 * one split, at least a workgroup per compute unit, from 1536 keys on
 * without a mask, and with one where a row sees 1536 keys on average, or 1024 if the row
 * tiles come in whole rounds of the compute units).  Host-only; -1 for invalid arguments.  (Decode shapes,
 * (Hq / Hkv) * Lq <= 32, report TILE: they run the tile form on the split-K decode kernel.)
 */
int flashd_auto_variant(int B, int Hq, int Hkv, int Lq, int Lk, int d, int dtype, int causal);

/*
 * Attention forward over one chunk of keys with the state of Alg. 3 handed in and out
 * (Sec. III-C: the state after a run of keys is (o, s_last, ln w_last), and only
 * s_last - ln w_last enters later steps).  Processes this call's Lk keys after the keys
 * that state_in stands for; chunked prefill, appended KV blocks and merging the results of
 * key ranges held by different devices are all sequences of such calls.
 *   state_in   DEVICE pointer or NULL (no earlier keys): [B][Hq][Lq][d + 2] fp32, per query
 *              row (o[0..d), s, ln w).  A row that has seen no key has s = -inf, ln w = 0.
 *   state_out  DEVICE pointer or NULL: same layout, receives the state after this call's keys,
 *              normalised to (o, s = s_last - ln w_last, ln w = 0); with fp32 storage ln w
 *              holds what s - ln w needs beyond one float instead of 0 (only the difference
 *              enters later steps).  May equal state_in.
 *   o          DEVICE pointer or NULL: the attention output after this call's keys in the
 *              storage type (what the state's o holds).  o and state_out must not both be NULL.
 *   causal_shift  with causal != 0, key j of THIS call is visible to query i iff
 *              j <= i + causal_shift; for a chunk that starts at key offset k0 of Lk_total
 *              keys that is (Lk_total - Lq) - k0.  Any int is valid (Lk or more shows every
 *              key, less than -Lq none).  Ignored when causal == 0.
 * Other arguments, conventions and errors as for flashd_attn_fwd (all pointers 16-byte aligned).
 * Takes scratch memory for partial states from the same grow-only cache as flashd_attn_fwd.
 */
int flashd_attn_fwd_state(const void* q, const void* k, const void* v, void* o,
                          const float* state_in, float* state_out,
                          int B, int Hq, int Hkv, int Lq, int Lk, int d,
                          int causal, int causal_shift, float scale, int dtype, void* stream);

/*
 * Attention forward with K and V stored as fp8 (the paper's second storage format, Sec. IV:
 * FP8-E4M3; here the OCP encoding, no infinities, 0x7f / 0xff = NaN), one byte per element,
 * same [B][Hkv][Lk][d] layout.  The real key and value are kscale * k8 and vscale * v8; q and
 * o are in the storage type `dtype` (FLASHD_F16 or FLASHD_BF16).  K and V cross HBM as fp8
 * and are widened exactly to `dtype` inside the kernel; everything else is the arithmetic
 * of flashd_attn_fwd (kscale joins the score scale, vscale the output).
 * For decode shapes ((Hq / Hkv) * Lq <= 32) the kernel reads the fp8 data itself; for other
 * shapes K and V are first widened into scratch memory (2 * B * Hkv * Lk * d * 2 bytes from the
 * grow-only cache) and the f16/bf16 kernel runs on that.  FLASHD_F32 gives FLASHD_E_VARIANT.
 * Other conventions and errors as for flashd_attn_fwd.
 */
int flashd_attn_fwd_kv8(const void* q, const void* k8, const void* v8, void* o,
                        int B, int Hq, int Hkv, int Lq, int Lk, int d,
                        int causal, float scale, float kscale, float vscale, int dtype,
                        void* stream);

/*
 * Decode with the saturation skip of Sec. III-C (a weight that has saturated at 0 leaves the
 * output as it is, so the value vector need not be loaded), for decode shapes only:
 * (Hq / Hkv) * Lq <= 32 and f16/bf16 storage, else FLASHD_E_VARIANT.  Variant TILE's
 * arithmetic; per 32-key block the scores are formed first, and the block's V is fetched only
 * if, for some query row of the kv group, the block's top score lies within 2^200 of the
 * largest s_last - ln w_last that row has reached so far (the test is on the full argument of
 * the sigmoid, where the weight is exactly 0 in fp32, not on the paper's static range of score
 * differences, which is an approximation).  K is always read.  The result is that of
 * flashd_attn_fwd_ex(..., FLASHD_VARIANT_TILE, splits, ...) to the last bit on inputs where
 * nothing is skipped, and within rounding of the fp32 accumulator otherwise.
 *   splits, workspace, workspace_bytes   as for flashd_attn_fwd_ex (variant TILE).
 *   counts   DEVICE pointer to two 64-bit unsigned integers, 8-byte aligned, or NULL: the
 *            enqueued work ADDS the number of 32-key blocks it visited to counts[0] and the
 *            number whose V it did not fetch to counts[1] (clear them yourself).
 * Never allocates.  Other conventions and errors as for flashd_attn_fwd.
 */
int flashd_attn_fwd_skipv(const void* q, const void* k, const void* v, void* o,
                          int B, int Hq, int Hkv, int Lq, int Lk, int d,
                          int causal, float scale, int dtype, void* stream,
                          int splits, void* workspace, size_t workspace_bytes,
                          unsigned long long* counts);

/*
 * flashd_attn_fwd for callers that cannot allocate: work recorded into a HIP graph, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same choice of variant and
 * splits, same result bit for bit; the split-K partial states go into a fixed array of
 * FLASHD_STATIC_SCRATCH_BYTES that is part of the library's code object (each GPU the library
 * runs on holds one copy until the process ends) instead of the grow-only cache.  Calls no
 * hipMalloc, hipFree or other allocating routine.  A problem whose partial states
 * (flashd_workspace_bytes(..., FLASHD_VARIANT_AUTO, 0)) exceed that size is refused with
 * FLASHD_E_WORKSPACE and nothing is enqueued: use flashd_attn_fwd_ex with memory of your own
 * for it.  All calls on one GPU share the array, whatever their stream, and it keeps the last
 * call's contents (every partial state a call reads it has written first, so nothing needs
 * clearing): calls that overlap in time on one GPU race; order them on one stream or by events.
 * The first call on a device looks up the array's device address (which may load the code
 * object); make that call outside a graph capture.
 */
#define FLASHD_STATIC_SCRATCH_BYTES (32u << 20)
int flashd_attn_fwd_static(const void* q, const void* k, const void* v, void* o,
                           int B, int Hq, int Hkv, int Lq, int Lk, int d,
                           int causal, float scale, int dtype, void* stream);

/*
 * Static skip statistics (Sec. III-C; the quantity reported in Table I).  Over every query
 * row and every step i >= 2 of Alg. 3 on that row's visible keys (same layout, head mapping
 * and causal rule as above; v is not needed), counts
 *     counts[0] = steps,
 *     counts[1] = steps with s_i - s_{i-1} <= lo   (weight ~ 0, the step could be skipped),
 *     counts[2] = steps with s_i - s_{i-1} >= hi   (weight ~ 1, the output becomes v_i).
 * The paper's static range is lo = -6, hi = 11.  Score arithmetic (fixed, so that the counts
 * are reproducible bit for bit): acc = fma(q[t], k[t], acc) over t = 0 .. d-1 in fp32,
 * s = acc * scale, the difference in fp32.
 * counts: DEVICE pointer to three 64-bit unsigned integers, 8-byte aligned, overwritten by
 * the enqueued work.  Errors as for flashd_attn_fwd.  Never allocates.
 */
int flashd_skip_stats(const void* q, const void* k, int B, int Hq, int Hkv, int Lq, int Lk, int d,
                      int causal, float scale, int dtype, float lo, float hi,
                      unsigned long long* counts, void* stream);

/*
 * Frees the split-K / fp8 scratch memory that flashd_attn_fwd, flashd_attn_fwd_state and
 * flashd_attn_fwd_kv8 have cached for the CURRENT device: the live buffer of every stream
 * that has been used and the buffers those streams have outgrown (which are kept until this
 * call, since work enqueued earlier may still read them).  The frees wait for the device, so
 * work already enqueued is not disturbed; do not call it while another host thread is inside
 * one of those entry points for this device.  A host that creates and destroys streams should
 * call it now and then: the cache is keyed by stream handle and forgets nothing by itself.
 * Returns FLASHD_OK, or FLASHD_E_HIP if a free failed.
 */
int flashd_release_workspace(void);

/* Static, NUL-terminated description of a status code. */
const char* flashd_status_string(int status);

/* major * 10000 + minor * 100 + patch */
int flashd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FLASHD_H */
