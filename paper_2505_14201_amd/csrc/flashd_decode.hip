// Split-K decode (few query rows per kv head, long key range): HBM-bound streaming of K
// and V, each element read once for all Hq/Hkv query heads of a kv group.
//
// A workgroup owns one (b, kv head, key split).  The g * Lq <= 32 query rows that share
// the kv head become the 32 columns of the score tile S^T = K Q^T, so the register layout
// and the per-row FLASH-D update are those of the prefill kernel (one lane pair per row).
// The four wavefronts of the workgroup do not share keys: wavefront w takes the 32-key
// blocks w, w + 4, ... of the split, stages them through its own LDS region (no workgroup
// barrier in the loop) and keeps its own state (U, Lam).  At the end the four states are
// folded with the sigmoid rule -- a run of keys acts as one key of score Lam -- and the
// result is either the output (splits == 1) or a partial state (o, s, ln w) for the merge
// kernel.
//
// Memory pipeline: each lane fetches the next block's K and V with fully coalesced 16-byte
// loads (a block is one contiguous 32 * d * 2 byte range) into registers while the
// current block is being multiplied; V stays row-major in LDS and is read through the
// transposing LDS load.
//
// KV8: K and V are stored as fp8 (e4m3, the paper's second format, Sec. IV), one byte per
// element, with one scale each.  They cross HBM in that form (half the bytes per key) and
// are widened exactly to the storage type of Q on the way from registers into the LDS
// stage, so everything after the stage is the same arithmetic; kscale joins the score scale
// and vscale the output.
#include "flashd_common.h"
#include "flashd_kernels.h"
#include "flashd_mma.h"

#include <type_traits>

namespace flashd {

constexpr int kDecWaves = 4;
constexpr int kDecThreads = kDecWaves * kWave;
constexpr int kDecBlock = 32;      // keys per wavefront step

// Issue the coalesced 16-byte loads of one 32-key block of K and V into registers.  Every
// byte of K and V is read exactly once per launch, so the loads are marked as streaming
// (non-temporal): on this part the same access pattern reads 7.0 TB/s that way and 6.15 TB/s
// with ordinary loads, which fill the caches with lines that are never used again.
template <int D, int CH>
__device__ __forceinline__ void fetch_block(const uint16_t* kg, const uint16_t* vg, int j0, int Lk,
                                            int lane, u32x4 (&kreg)[CH], u32x4 (&vreg)[CH]) {
#pragma unroll
    for (int n = 0; n < CH; ++n) {
        const int c = n * kWave + lane;            // chunk index inside the block
        const int key = c / (D / 8);
        const int part = c % (D / 8);
        const size_t off = (size_t)min(j0 + key, Lk - 1) * D + 8 * part;
        kreg[n] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kg + off));
        vreg[n] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vg + off));
    }
}

// The same for fp8 storage: 16 elements (16 bytes) per chunk.
template <int D, int CH8>
__device__ __forceinline__ void fetch_block8(const uint8_t* kg, const uint8_t* vg, int j0, int Lk,
                                             int lane, u32x4 (&kreg)[CH8], u32x4 (&vreg)[CH8]) {
#pragma unroll
    for (int n = 0; n < CH8; ++n) {
        const int c = n * kWave + lane;            // 16-element chunk index inside the block
        const int key = c / (D / 16);
        const int part = c % (D / 16);
        const size_t off = (size_t)min(j0 + key, Lk - 1) * D + 16 * part;
        kreg[n] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kg + off));
        vreg[n] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vg + off));
    }
}

// 16 fp8 values -> 16 values of the storage type T (two 16-byte LDS chunks)
template <typename T>
__device__ __forceinline__ void widen16(u32x4 raw, u32x4& lo, u32x4& hi) {
    lo = u32x4{Mma<T>::from_fp8_lo(raw[0]), Mma<T>::from_fp8_hi(raw[0]),
               Mma<T>::from_fp8_lo(raw[1]), Mma<T>::from_fp8_hi(raw[1])};
    hi = u32x4{Mma<T>::from_fp8_lo(raw[2]), Mma<T>::from_fp8_hi(raw[2]),
               Mma<T>::from_fp8_lo(raw[3]), Mma<T>::from_fp8_hi(raw[3])};
}

// Fold the four wavefront states of a workgroup with the sigmoid rule (a run of keys acts as
// one key of score Lam) and store the output, or the partial state of this key split.
// U, fin, lam_out: the lane's accumulator, the factor that turns it into the run's output, and
// the run's Lam in log2 units (-inf: the wavefront saw no key for this row).
template <typename T, int D>
__device__ __forceinline__ void decode_fold(const Problem& p, uint16_t* lds,
                                            const f32x16 (&U)[D / 32], float fin, float lam_out,
                                            bool row_ok, int nrows) {
    constexpr int NDB = D / 32;
    const float ninf = -__builtin_inff();
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31;
    const int hh = lane >> 5;
    const int sp = blockIdx.x;
    const int kvh = blockIdx.y;
    const int b = blockIdx.z;
    const int g = p.Hq / p.Hkv;
    __syncthreads();                                   // stages are dead, reuse the LDS
    float* fold = reinterpret_cast<float*>(lds);       // [wave][row][D + 1]
    constexpr int SROW = D + 1;
    if (row_ok) {
        float* dst = fold + ((size_t)wave * 32 + col) * SROW;
#pragma unroll
        for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                dst[32 * i + 8 * (r >> 2) + 4 * hh + (r & 3)] = U[i][r] * fin;
        if (hh == 0) dst[D] = lam_out;
    }
    __syncthreads();
    for (int idx = tid; idx < nrows * D; idx += kDecThreads) {
        const int row = idx / D;
        const int t = idx % D;
        float o = 0.0f;
        float lm = ninf;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) {
            const float* src = fold + ((size_t)w * 32 + row) * SROW;
            const float lb = src[D];
            if (lb == ninf) continue;                  // empty run: identity
            if (lm == ninf) { o = src[t]; lm = lb; continue; }
            // W = sigmoid(Lam_b - Lam_a) in log2 units; o += (o_b - o) W; Lam = lse
            const float dlt = lb - lm;
            const float e = exp2_fast(-fabsf(dlt));
            const float r1 = __builtin_amdgcn_rcpf(1.0f + e);
            const float W = dlt >= 0.0f ? r1 : e * r1;
            o = fmaf(src[t] - o, W, o);
            lm = fmaxf(lm, lb) + log2_fast(1.0f + e);
        }
        const int hq = kvh * g + row / p.Lq;
        const int i = row % p.Lq;
        const size_t orow = ((size_t)b * p.Hq + hq) * (size_t)p.Lq + i;
        if (!p.partial) {
            Store<T>::store(p.o, orow * D + t, o);
        } else {
            float* dst = p.ws + ((size_t)sp * p.B * p.Hq * p.Lq + orow) * (D + 2);
            dst[t] = o;
            if (t == 0) { dst[D] = lm * kLn2; dst[D + 1] = 0.0f; }
        }
    }
}

// MODE: how a block's scores update a row (kTileModeLazy / Online / Blend).  TL: the state
// is handed out and the coefficient sums are those of the rounded coefficients, so the
// unrounded sum is carried as well (the Lam handed out is then the true log-sum-exp).
template <typename T, int D, int MODE, bool KV8, bool TL>
__global__ __launch_bounds__(kDecThreads, 2)
void decode_kernel(Problem p) {
    constexpr bool kTL = TL && Mma<T>::kRoundedSum && MODE == kTileModeLazy;
    constexpr int KROW = D + 8;                 // padded LDS rows (elements)
    constexpr int VROW = D + 32;                // conflict-free for the transposing read
    constexpr int NKK = D / 16;
    constexpr int NDB = D / 32;
    constexpr int CH = kDecBlock * D / 8 / kWave;      // 16-byte chunks per lane per block
    constexpr int STAGE = kDecBlock * (KROW + VROW);   // elements per wavefront
    __shared__ __align__(16) uint16_t lds[kDecWaves * STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31;
    const int hh = lane >> 5;
    const int sp = blockIdx.x;
    const int kvh = blockIdx.y;
    const int b = blockIdx.z;
    const int g = p.Hq / p.Hkv;
    const int nrows = g * p.Lq;                 // <= 32, checked by the launcher

    // query row of this lane's column: head kvh * g + col / Lq, position col % Lq
    const bool row_ok = col < nrows;
    const int head = kvh * g + (row_ok ? col / p.Lq : 0);
    const int qi = row_ok ? col % p.Lq : 0;
    const uint16_t* qg = static_cast<const uint16_t*>(p.q) +
                         (((size_t)b * p.Hq + head) * (size_t)p.Lq + qi) * D;
    u32x4 qf[NKK];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
        qf[kk] = row_ok ? *reinterpret_cast<const u32x4*>(qg + 16 * kk + 8 * hh)
                        : u32x4{0u, 0u, 0u, 0u};
    }
    // position 0 sees the fewest keys, position Lq - 1 the most; unused columns (zero
    // query, output discarded) mimic the last position so they never leave the fast path
    const int nvis_min = visible_count(p, 0);
    const int nvis_max = visible_count(p, p.Lq - 1);
    const int nvis = row_ok ? visible_count(p, qi) : nvis_max;

    const size_t kv_off = ((size_t)b * p.Hkv + kvh) * (size_t)p.Lk * D;       // elements
    const uint16_t* kg = static_cast<const uint16_t*>(p.k) + kv_off;
    const uint16_t* vg = static_cast<const uint16_t*>(p.v) + kv_off;
    const uint8_t* kg8 = static_cast<const uint8_t*>(p.k) + kv_off;
    const uint8_t* vg8 = static_cast<const uint8_t*>(p.v) + kv_off;

    // 32-key blocks of this split; wavefront w takes blk_begin + w, + 4, ...
    const int nblk = (nvis_max + kDecBlock - 1) / kDecBlock;
    const int nblk_all = (p.Lk + kDecBlock - 1) / kDecBlock;
    const int per_split = (nblk_all + p.splits - 1) / p.splits;
    const int blk_begin = sp * per_split;
    const int blk_end = min(nblk, blk_begin + per_split);

    uint16_t* ks = lds + wave * STAGE;
    uint16_t* vs = ks + kDecBlock * KROW;

    const float c_log2 = (KV8 ? p.scale * p.kscale : p.scale) * kLog2e;
    const float ninf = -__builtin_inff();
    f32x16 U[NDB];
#pragma unroll
    for (int i = 0; i < NDB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) U[i][r] = 0.0f;
    LazyRow st = {0.0f, 1.0f, 0.0f, 0.0f};      // FLASH-D state of the lane's row (lazy form)
    BlendRow bl = {0.0f, 0.0f};            // FLASH-D state, literal per-block blend
    float lam = ninf, beta = 0.0f;         // Alg. 2 state: running max, running sum
    bool first = true;
    Wary wary = {0, kWaryTiles};     // wavefront-uniform, see lazy_spec_pack

    constexpr int CHR = KV8 ? CH / 2 : CH;     // 16-byte loads per lane, block and tensor
    // One block per wavefront is in flight while the previous one is multiplied.  (Two
    // register sets for the half-sized fp8 blocks were tried and were slower: the kernel is
    // bound by instruction issue there, not by memory latency.)
    u32x4 kreg[CHR], vreg[CHR];    // native vectors: HIP's uint4 struct would live in scratch
    auto fetch = [&](int blk_) __attribute__((always_inline)) {
        if constexpr (KV8)
            fetch_block8<D, CHR>(kg8, vg8, blk_ * kDecBlock, p.Lk, lane, kreg, vreg);
        else
            fetch_block<D, CHR>(kg, vg, blk_ * kDecBlock, p.Lk, lane, kreg, vreg);
    };
    int blk = blk_begin + wave;
    if (blk < blk_end) fetch(blk);
    while (blk < blk_end) {
        const int j0 = blk * kDecBlock;
        // registers -> this wavefront's LDS stage
#pragma unroll
        for (int n = 0; n < CHR; ++n) {
            const int c = n * kWave + lane;
            if constexpr (KV8) {
                const int key = c / (D / 16);
                const int part = c % (D / 16);
                u32x4 lo, hi;
                widen16<T>(kreg[n], lo, hi);
                *reinterpret_cast<u32x4*>(&ks[key * KROW + 16 * part]) = lo;
                *reinterpret_cast<u32x4*>(&ks[key * KROW + 16 * part + 8]) = hi;
                widen16<T>(vreg[n], lo, hi);
                *reinterpret_cast<u32x4*>(&vs[key * VROW + 16 * part]) = lo;
                *reinterpret_cast<u32x4*>(&vs[key * VROW + 16 * part + 8]) = hi;
            } else {
                const int key = c / (D / 8);
                const int part = c % (D / 8);
                *reinterpret_cast<u32x4*>(&ks[key * KROW + 8 * part]) = kreg[n];
                *reinterpret_cast<u32x4*>(&vs[key * VROW + 8 * part]) = vreg[n];
            }
        }
        if (blk + kDecWaves < blk_end) fetch(blk + kDecWaves);     // in flight during the math
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // S^T = K Q^T for the block's 32 keys
        f32x16 acc[1];
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][r] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            const u32x4 a = *reinterpret_cast<const u32x4*>(&ks[col * KROW + 16 * kk + 8 * hh]);
            acc[0] = Mma<T>::mfma(a, qf[kk], acc[0]);
        }
        // Coefficients of the block and the per-row state update (flashd_mma.h): the blend
        // factor is carried as a scalar per row, U is only scaled on the rare overflow path.
        // general: keys may be masked, or rows may still be empty (the wavefront's first block).
        const bool general = first || j0 + kDecBlock > nvis_min;
        first = false;
        const int jb = j0 + 4 * hh;
        u32x4 bfrag[2];
        auto scale_u = [&](float f) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < NDB; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) U[i][r] *= f;
        };
        if (MODE == kTileModeLazy) {
            bool risky;
            LazySpec spec;
            if (general) risky = lazy_spec_pack<T, 1, true, true, TL>(acc, bfrag, st, c_log2, jb, nvis, lane, spec, wary);
            else risky = lazy_spec_pack<T, 1, false, false, TL>(acc, bfrag, st, c_log2, jb, nvis, lane, spec, wary);
            if (spec.any_moved) scale_u(spec.fu);
            if (!spec.checked && __builtin_amdgcn_ballot_w64(risky) != 0) {
                // rare: bf16 with a sum that is still a number moves the reference by a power
                // of two in place; everything else takes the checked step on the raw scores
                const bool lost = risky && !(spec.psum <= kLazyShiftMax);
                float f;
                bool moved;
                if (std::is_same<T, BF16>::value && __builtin_amdgcn_ballot_w64(lost) == 0)
                    f = lazy_shift_inplace_bf16<TL>(bfrag, 2, st, risky, spec);
                else if (general)
                    f = lazy_checked_pack<T, 1, true, TL>(acc, bfrag, st, risky, c_log2, jb, nvis, moved);
                else
                    f = lazy_checked_pack<T, 1, false, TL>(acc, bfrag, st, risky, c_log2, jb, nvis, moved);
                wary.failed();
                scale_u(f);
            }
        } else if (MODE == kTileModeOnline) {
            float f;
            if (general) f = online_pack<T, 1, true>(acc, bfrag, lam, beta, c_log2, jb, nvis);
            else f = online_pack<T, 1, false>(acc, bfrag, lam, beta, c_log2, jb, nvis);
            if (__builtin_amdgcn_ballot_w64(f != 1.0f) != 0) scale_u(f);
        } else {
            float f;
            if (general) f = blend_pack<T, 1, true>(acc, bfrag, bl, c_log2, jb, nvis);
            else f = blend_pack<T, 1, false>(acc, bfrag, bl, c_log2, jb, nvis);
            scale_u(f);
        }
#pragma unroll
        for (int g2 = 0; g2 < 2; ++g2) {
#pragma unroll
            for (int i = 0; i < NDB; ++i) {
                const u32x4 a = lds_read_v_operand(&vs[(16 * g2) * VROW + 32 * i], VROW, lane);
                U[i] = Mma<T>::mfma(a, bfrag[g2], U[i]);
            }
        }
        // the next stage write must not overtake these LDS reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        blk += kDecWaves;
    }

    // ---- fold the four wavefront states (sigmoid rule on runs of keys) --------------
    float fin, lam_out;
    if (MODE == kTileModeLazy) {
        fin = st.beta;                     // the state is the output: o = beta U
        lam_out = st.one == 0.0f ? ninf
                  : kTL ? st.R + log2_fast(st.ltrue) : st.R - log2_fast(st.beta);
    } else if (MODE == kTileModeBlend) {
        fin = 1.0f;
        lam_out = bl.one == 0.0f ? ninf : bl.lam;
    } else {
        row_finish<true>(lam, beta, fin, lam_out);
    }
    if (KV8) fin *= p.vscale;
    decode_fold<T, D>(p, lds, U, fin, lam_out, row_ok, nrows);
}

// The decode kernel with the saturation skip of Sec. III-C ("a weight that has saturated at 0
// leaves the output as it is: the value need not be loaded"), in the lazy form, f16/bf16
// storage.  The skip is taken per 32-key block and only where it is exact in fp32, on the full
// argument of the sigmoid rather than on the paper's static range of score differences: a
// block's V is not fetched (and its output product not issued) when, for every query row of
// the group, the block's top score lies more than kSkipMarginLog2 below a lower bound of the
// row's final Lam.  Lam only grows, so any Lam seen so far is such a bound; the four
// wavefronts of the workgroup, which walk interleaved blocks with states of their own, share
// the largest Lam any of them has reached per row through LDS (a stale value is still a
// bound).  The margin covers three things at once: a wavefront whose own Lam ends up more
// than 2^150 below the workgroup's has weight exactly 0 in the fold, so what it left out
// does not matter; otherwise its own Lam is within 2^150 of the bound and a skipped key
// weighs less than 2^-(margin - 150) of what the wavefront holds, 2^-37 even with every key
// of the longest split skipped, far below the fp32 accumulator's rounding.
//
// To skip a fetch the scores must exist before the fetch is issued, so V runs one block
// behind K: iteration b stages K(b), requests K(b + 4), forms the scores of block b, then
// multiplies block b - 4's coefficients with its V (requested an iteration ago), updates the
// rows with block b's coefficients and only then decides whether to request V(b).  The order
// of the operations on the accumulator is that of decode_kernel.
constexpr float kSkipMarginLog2 = 200.0f;

template <typename T, int D, bool TL>
__global__ __launch_bounds__(kDecThreads, 2)
void decode_vskip_kernel(Problem p) {
    constexpr bool kTL = TL && Mma<T>::kRoundedSum;
    constexpr int KROW = D + 8;
    constexpr int VROW = D + 32;
    constexpr int NKK = D / 16;
    constexpr int NDB = D / 32;
    constexpr int CH = kDecBlock * D / 8 / kWave;
    constexpr int STAGE = kDecBlock * (KROW + VROW);
    __shared__ __align__(16) uint16_t lds[kDecWaves * STAGE];
    __shared__ float lam_seen[32];             // per row: the largest Lam any wavefront has reached

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31;
    const int hh = lane >> 5;
    const int sp = blockIdx.x;
    const int kvh = blockIdx.y;
    const int b = blockIdx.z;
    const int g = p.Hq / p.Hkv;
    const int nrows = g * p.Lq;

    const bool row_ok = col < nrows;
    const int head = kvh * g + (row_ok ? col / p.Lq : 0);
    const int qi = row_ok ? col % p.Lq : 0;
    const uint16_t* qg = static_cast<const uint16_t*>(p.q) +
                         (((size_t)b * p.Hq + head) * (size_t)p.Lq + qi) * D;
    u32x4 qf[NKK];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
        qf[kk] = row_ok ? *reinterpret_cast<const u32x4*>(qg + 16 * kk + 8 * hh)
                        : u32x4{0u, 0u, 0u, 0u};
    const int nvis_min = visible_count(p, 0);
    const int nvis_max = visible_count(p, p.Lq - 1);
    const int nvis = row_ok ? visible_count(p, qi) : nvis_max;

    const size_t kv_off = ((size_t)b * p.Hkv + kvh) * (size_t)p.Lk * D;
    const uint16_t* kg = static_cast<const uint16_t*>(p.k) + kv_off;
    const uint16_t* vg = static_cast<const uint16_t*>(p.v) + kv_off;

    const int nblk = (nvis_max + kDecBlock - 1) / kDecBlock;
    const int nblk_all = (p.Lk + kDecBlock - 1) / kDecBlock;
    const int per_split = (nblk_all + p.splits - 1) / p.splits;
    const int blk_begin = sp * per_split;
    const int blk_end = min(nblk, blk_begin + per_split);

    uint16_t* ks = lds + wave * STAGE;
    uint16_t* vs = ks + kDecBlock * KROW;

    const float c_log2 = p.scale * kLog2e;
    const float ninf = -__builtin_inff();
    if (tid < 32) lam_seen[tid] = ninf;
    __syncthreads();

    f32x16 U[NDB];
#pragma unroll
    for (int i = 0; i < NDB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) U[i][r] = 0.0f;
    LazyRow st = {0.0f, 1.0f, 0.0f, 0.0f};
    bool first = true;
    Wary wary = {0, kWaryTiles};
    unsigned visited = 0, skipped = 0;         // wavefront-uniform

    u32x4 kreg[CH], vreg[CH];
    u32x4 bprev[2] = {u32x4{0u, 0u, 0u, 0u}, u32x4{0u, 0u, 0u, 0u}};
    bool pending = false;                      // wavefront-uniform: vreg / bprev hold a block
    auto fetch_k = [&](int blk_) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < CH; ++n) {
            const int c = n * kWave + lane;
            const size_t off = (size_t)min(blk_ * kDecBlock + c / (D / 8), p.Lk - 1) * D + 8 * (c % (D / 8));
            kreg[n] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kg + off));
        }
    };
    auto fetch_v = [&](int blk_) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < CH; ++n) {
            const int c = n * kWave + lane;
            const size_t off = (size_t)min(blk_ * kDecBlock + c / (D / 8), p.Lk - 1) * D + 8 * (c % (D / 8));
            vreg[n] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vg + off));
        }
    };
    // U += (coefficients of the pending block) x (its V, staged through LDS)
    auto flush_pending = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < CH; ++n) {
            const int c = n * kWave + lane;
            *reinterpret_cast<u32x4*>(&vs[(c / (D / 8)) * VROW + 8 * (c % (D / 8))]) = vreg[n];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int g2 = 0; g2 < 2; ++g2)
#pragma unroll
            for (int i = 0; i < NDB; ++i) {
                const u32x4 a = lds_read_v_operand(&vs[(16 * g2) * VROW + 32 * i], VROW, lane);
                U[i] = Mma<T>::mfma(a, bprev[g2], U[i]);
            }
        // the next stage write must not overtake these LDS reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    auto scale_u = [&](float f) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) U[i][r] *= f;
    };

    int blk = blk_begin + wave;
    if (blk < blk_end) fetch_k(blk);
    while (blk < blk_end) {
        const int j0 = blk * kDecBlock;
#pragma unroll
        for (int n = 0; n < CH; ++n) {
            const int c = n * kWave + lane;
            *reinterpret_cast<u32x4*>(&ks[(c / (D / 8)) * KROW + 8 * (c % (D / 8))]) = kreg[n];
        }
        if (blk + kDecWaves < blk_end) fetch_k(blk + kDecWaves);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        f32x16 acc[1];
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][r] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            const u32x4 a = *reinterpret_cast<const u32x4*>(&ks[col * KROW + 16 * kk + 8 * hh]);
            acc[0] = Mma<T>::mfma(a, qf[kk], acc[0]);
        }
        // the previous block's output product: its V has been in flight since that block's
        // coefficients were known
        if (pending) flush_pending();

        const bool general = first || j0 + kDecBlock > nvis_min;
        first = false;
        const int jb = j0 + 4 * hh;
        u32x4 bfrag[2];
        bool risky;
        LazySpec spec;
        float top;
        if (general) {
            risky = lazy_spec_pack<T, 1, true, true, TL>(acc, bfrag, st, c_log2, jb, nvis, lane, spec, wary);
            top = row_top_score<1, true>(acc, c_log2, jb, nvis);
        } else {
            risky = lazy_spec_pack<T, 1, false, false, TL>(acc, bfrag, st, c_log2, jb, nvis, lane, spec, wary);
            top = row_top_score<1, false>(acc, c_log2, jb, nvis);
        }
        if (spec.any_moved) scale_u(spec.fu);
        if (!spec.checked && __builtin_amdgcn_ballot_w64(risky) != 0) {
            const bool lost = risky && !(spec.psum <= kLazyShiftMax);
            float f;
            bool moved;
            if (std::is_same<T, BF16>::value && __builtin_amdgcn_ballot_w64(lost) == 0)
                f = lazy_shift_inplace_bf16<TL>(bfrag, 2, st, risky, spec);
            else if (general)
                f = lazy_checked_pack<T, 1, true, TL>(acc, bfrag, st, risky, c_log2, jb, nvis, moved);
            else
                f = lazy_checked_pack<T, 1, false, TL>(acc, bfrag, st, risky, c_log2, jb, nvis, moved);
            wary.failed();
            scale_u(f);
        }
        // The skip decision.  own: this wavefront's Lam for the row after the block.
        const float own = st.one == 0.0f ? ninf
                          : kTL ? st.R + log2_fast(st.ltrue) : st.R - log2_fast(st.beta);
        // (volatile: the other wavefronts' stores must be looked at on every block)
        volatile float* shared_lam = lam_seen;
        const float seen = shared_lam[col];
        if (hh == 0 && row_ok && own > seen) shared_lam[col] = own;    // a lost race leaves a bound
        const float bound = fmaxf(own, seen);
        const bool matters = row_ok && !(top < bound - kSkipMarginLog2);   // false for top = -inf
        ++visited;
        if (__builtin_amdgcn_ballot_w64(matters) != 0) {
            fetch_v(blk);
            bprev[0] = bfrag[0];
            bprev[1] = bfrag[1];
            pending = true;
        } else {
            pending = false;
            ++skipped;
        }
        blk += kDecWaves;
    }
    if (pending) flush_pending();
    if (p.vskip_counts != nullptr && lane == 0) {
        atomicAdd(p.vskip_counts, (unsigned long long)visited);
        atomicAdd(p.vskip_counts + 1, (unsigned long long)skipped);
    }

    const float fin = st.beta;
    const float lam_out = st.one == 0.0f ? ninf
                          : kTL ? st.R + log2_fast(st.ltrue) : st.R - log2_fast(st.beta);
    decode_fold<T, D>(p, lds, U, fin, lam_out, row_ok, nrows);
}

template <typename T, int D>
static hipError_t launch_decode_t(const Problem& p, int mode, hipStream_t st) {
    dim3 grid((unsigned)p.splits, (unsigned)p.Hkv, (unsigned)p.B);
    const dim3 block(kDecThreads);
    // the true log-sum-exp is wanted wherever the state leaves the kernel
    const bool tl = p.partial != 0;
    if (mode == kTileModeLazySkipV) {
        if (p.kv8) return hipErrorInvalidValue;
        if (tl) hipLaunchKernelGGL((decode_vskip_kernel<T, D, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((decode_vskip_kernel<T, D, false>), grid, block, 0, st, p);
    } else if (p.kv8) {
        if (mode != kTileModeLazy) return hipErrorInvalidValue;
        if (tl) hipLaunchKernelGGL((decode_kernel<T, D, kTileModeLazy, true, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((decode_kernel<T, D, kTileModeLazy, true, false>), grid, block, 0, st, p);
    } else if (mode == kTileModeOnline) {
        hipLaunchKernelGGL((decode_kernel<T, D, kTileModeOnline, false, false>), grid, block, 0, st, p);
    } else if (mode == kTileModeBlend) {
        hipLaunchKernelGGL((decode_kernel<T, D, kTileModeBlend, false, false>), grid, block, 0, st, p);
    } else if (mode == kTileModeLazy) {
        if (tl) hipLaunchKernelGGL((decode_kernel<T, D, kTileModeLazy, false, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((decode_kernel<T, D, kTileModeLazy, false, false>), grid, block, 0, st, p);
    } else {
        return hipErrorInvalidValue;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !p.merge) return e;
    return launch_merge_splits(p, st);
}

bool decode_applies(int Hq, int Hkv, int Lq) {
    return (long)(Hq / Hkv) * Lq <= 32;
}

long decode_workgroups(int B, int Hkv) { return (long)B * Hkv; }

hipError_t launch_decode(const Problem& p, int mode, hipStream_t st) {
    if (!decode_applies(p.Hq, p.Hkv, p.Lq)) return hipErrorInvalidValue;
    if (p.dtype == 1 && p.d == 64) return launch_decode_t<F16, 64>(p, mode, st);
    if (p.dtype == 1 && p.d == 128) return launch_decode_t<F16, 128>(p, mode, st);
    if (p.dtype == 2 && p.d == 64) return launch_decode_t<BF16, 64>(p, mode, st);
    if (p.dtype == 2 && p.d == 128) return launch_decode_t<BF16, 128>(p, mode, st);
    return hipErrorInvalidValue;
}

}  // namespace flashd
