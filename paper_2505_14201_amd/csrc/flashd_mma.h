// Matrix-core building blocks shared by the tiled prefill and the decode kernels:
// the v_mfma_f32_32x32x16 wrappers per storage type, and the per-row update of the
// FLASH-D state for one tile of keys (plus the Alg. 2 update used by the ablation).
//
// Register layout this file assumes (checked on gfx950 with an integer-valued probe):
// for D = A B with A 32xK, B Kx32 (K = 16), lane l = (c, hh) = (l % 32, l / 32) supplies
// A[c][8 hh .. 8 hh + 7] and B[8 hh .. 8 hh + 7][c], and receives D[8 (r / 4) + 4 hh + r % 4][c]
// in accumulator register r = 0..15.
#pragma once

#include "flashd_common.h"

namespace flashd {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));


constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <typename T> struct Mma;
template <> struct Mma<BF16> {
    static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ u32x4 pack8(f32x8 x) {
        return __builtin_bit_cast(u32x4, __builtin_convertvector(x, bf16x8));
    }
    static constexpr bool kRoundedSum = true;
    // Sum of the 8 coefficients of a group.  bf16: of the ROUNDED coefficients, two per
    // v_dot2c_f32_bf16 with a pair of ones (one rounding per instruction): half the
    // instructions of adding the fp32 values, and the sum that normalises a row is the sum of
    // exactly the weights the output product uses, so a weight of nearly 1 carries no
    // rounding error of its own into the output.
    static __device__ __forceinline__ void sum8(const f32x8& x, u32x4 packed, f32x4& acc) {
        (void)x;
        // the pair of ones in a scalar register rather than as a 32-bit literal in each of
        // the instructions
        unsigned one_bits = 0x3f803f80u;
        asm volatile("" : "+s"(one_bits));
        const bf16x2 ones = __builtin_bit_cast(bf16x2, one_bits);
        const bf16x8 v = __builtin_bit_cast(bf16x8, packed);
        // four independent chains: one long one would wait on every instruction's latency
        acc[0] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(v, v, 0, 1), ones, acc[0], false);
        acc[1] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(v, v, 2, 3), ones, acc[1], false);
        acc[2] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(v, v, 4, 5), ones, acc[2], false);
        acc[3] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(v, v, 6, 7), ones, acc[3], false);
    }
    // the same for one packed pair: acc + the two rounded coefficients (ones: a pair of ones in
    // the storage type, kOnes, which the caller keeps in a scalar register)
    static constexpr uint32_t kOnes = 0x3f803f80u;
    static __device__ __forceinline__ float sum2(float a, float b, uint32_t packed, uint32_t ones,
                                                 float acc) {
        (void)a; (void)b;
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed),
                                               __builtin_bit_cast(bf16x2, ones), acc, false);
    }
    static __device__ __forceinline__ u32x2 pack4(f32x4 x) {
        return __builtin_bit_cast(u32x2, __builtin_convertvector(x, bf16x4));
    }
    static __device__ __forceinline__ uint32_t pack2(float a, float b) {
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
    }
    // two fp8 (e4m3) values of a dword -> two storage-type values, exact (scale 1)
    static __device__ __forceinline__ uint32_t from_fp8_lo(uint32_t w) {
        return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false));
    }
    static __device__ __forceinline__ uint32_t from_fp8_hi(uint32_t w) {
        return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true));
    }
};
template <> struct Mma<F16> {
    static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ u32x4 pack8(f32x8 x) {
        return __builtin_bit_cast(u32x4, __builtin_convertvector(x, f16x8));
    }
    static constexpr bool kRoundedSum = false;
    // fp16: of the fp32 values (a coefficient beyond the fp16 range must still give a finite
    // sum, which the reference-shift path works from; fp16 rounding is eight times finer)
    static __device__ __forceinline__ void sum8(const f32x8& x, u32x4 packed, f32x4& acc) {
        (void)packed;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[0] += x[e];
    }
    static constexpr uint32_t kOnes = 0x3c003c00u;
    static __device__ __forceinline__ float sum2(float a, float b, uint32_t packed, uint32_t ones,
                                                 float acc) {
        (void)packed; (void)ones;
        return (acc + a) + b;
    }
    static __device__ __forceinline__ u32x2 pack4(f32x4 x) {
        return __builtin_bit_cast(u32x2, __builtin_convertvector(x, f16x4));
    }
    static __device__ __forceinline__ uint32_t pack2(float a, float b) {
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, f16x2));
    }
    static __device__ __forceinline__ uint32_t from_fp8_lo(uint32_t w) {
        return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, false));
    }
    static __device__ __forceinline__ uint32_t from_fp8_hi(uint32_t w) {
        return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, true));
    }
};

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float log2_fast(float x) { return __builtin_amdgcn_logf(x); }

// log2(2^a + 2^b) through 2^{-|a-b|} <= 1 (the saturating side of the sigmoid);
// -inf is the empty run.  Branch-free: with one side -inf the correction term is
// log2(1 + 0) = 0 and the other side comes back unchanged; only (-inf, -inf), where
// a - b is NaN, needs the select.
__device__ __forceinline__ float lse2(float a, float b) {
    const float ninf = -__builtin_inff();
    const float m = fmaxf(a, b);
    const float r = m + log2_fast(1.0f + exp2_fast(-fabsf(a - b)));
    return m == ninf ? ninf : r;
}

// 8 keys x 1 column of a row-major [key][d] LDS tile as an MFMA operand, through the
// transposing LDS read: within each 16-lane group, lanes 4r .. 4r+3 address the four
// 8-byte pieces of row r (r = 0..3) and lane t receives column t of those four rows.
// `base` points at element [key0][dcol0]; rows are `row_elems` apart.  Lane (c, hh)
// receives keys key0 + 4 hh + {0..3} and key0 + 8 + 4 hh + {0..3} at column dcol0 + c,
// which is the key order of the score accumulator registers r = 0..7 (see above).
__device__ __forceinline__ u32x4 lds_read_v_operand(const uint16_t* base, int row_elems, int lane) {
    const int t = lane & 15;
    const int hh = lane >> 5;
    const int half = (lane >> 4) & 1;
    const uint16_t* p0 = base + (4 * hh + (t >> 2)) * row_elems + 16 * half + 4 * (t & 3);
    const uint16_t* p1 = p0 + 8 * row_elems;
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p1));
    const u32x2 l2 = __builtin_bit_cast(u32x2, lo);
    const u32x2 h2 = __builtin_bit_cast(u32x2, hi);
    return u32x4{l2[0], l2[1], h2[0], h2[1]};
}

// ---------------------------------------------------------------------------
// The tile rule of Alg. 3 as the matrix-core kernels apply it by default ("lazy blend"; the
// literal per-tile blend is blend_pack() further down).  After a run of keys the state of
// Alg. 3 is (o, s_last, ln w_last) and only Lam = s_last - ln w_last enters later steps; a tile
// of keys acts as one key.  A row's state here is (U, R, beta, one):
//     true output o = beta U,   Lam = R - log2 beta,   one = 0 until the row has seen a key.
// For a tile, with p_j = 2^{s_j - R} (R does not move on this path) and psum = sum_j p_j,
//     tot = one + beta psum,   1 - W = 1/tot   (W = sigmoid(S_tile - Lam), the tile's weight),
//     U <- U + sum_j p_j v_j,  beta <- beta (1 - W).
// This is o <- (1 - W)(o + sum_j 2^{s_j - Lam} v_j) with the vector multiplication by
// (1 - W) folded into the scalar beta: U is never rescaled here.  Said the other way round:
// 1/beta is the sum of 2^{s_j - R} over the keys seen so far, taken against a reference R that
// is not a running maximum and does not move unless it has to, and o = beta U at the store is
// the normalisation by that sum, applied once.  An empty row takes the score of the tile's
// first key as R (w_1 = 1 for that key).
//
// lazy_spec_pack() does that speculatively, branch-free, leaving the raw scores untouched,
// and reports rows whose psum left the safe range (some 2^{s_j - R} too large for the
// storage type: a score far above everything before it -- the case in which the sigmoid of
// the weight equation saturates at 1, Sec. III-C).  For bf16, whose coefficients have the
// range of fp32, a psum that is still an ordinary number is served by
// lazy_shift_inplace_bf16(): the reference moves up by a power of two and the coefficients are
// scaled as they are.  Everything else goes through lazy_checked_pack(): the row's top score
// of the tile is looked at BEFORE anything is exponentiated, and a row whose top score lies
// far above its reference takes that score as its new reference (the saturating key takes
// the weight to 1 and everything before it is scaled down by 2^{R - R'}, which underflows to
// zero where the sigmoid would).  A wavefront that has needed the checked step keeps using it
// (instead of speculating and forming the tile's scores a second time) until a run of tiles
// has left every reference where it was.
struct LazyRow {
    float R;      // exponent reference, log2 units
    float beta;   // o = beta * U
    float one;    // 0.0f while the row is empty, then 1.0f
    float ltrue;  // only where the coefficient sums are those of the rounded coefficients and
                  // the state is handed out: the sum of the unrounded 2^{s_j - R}, so that
                  // Lam = R + log2 ltrue is the true log-sum-exp
};

// What the speculative pass found for a row: the sum of its coefficients and the reference
// they were taken against (the row's R, or the tile's first visible score for an empty row).
struct LazySpec {
    float psum;
    float ref;
    float ptrue;  // sum of the unrounded coefficients (see LazyRow::ltrue)
    float fu;     // factor that what the row holds (U) still has to be scaled by; 1 as a rule
    bool any_moved;   // wavefront-uniform: some row's fu is not 1
    bool checked;     // wavefront-uniform: the top scores were looked at first, so no row can be
                      // risky (short of a sum that is not a number)
};

// psum above this is treated as overflowed.  Below it one + beta psum (beta <= 2) stays far
// under 2^126, so that its reciprocal is still a normal number (v_rcp_f32 returns zero where
// the result would be subnormal, and a beta of zero would poison the row).
constexpr float kLazyShiftMax = 1.0e30f;      // ~2^100

template <typename T> struct LazyLimit;
// kMaxPsum: the speculative pass trusts a tile whose coefficient sum stays below this.
// kMoveLog2: the checked step moves a row's reference once a score lies this far above it.
template <> struct LazyLimit<BF16> {
    static constexpr float kMaxPsum = 1.0e18f;       // ~2^60
    static constexpr float kMoveLog2 = 54.0f;
};
template <> struct LazyLimit<F16> {
    static constexpr float kMaxPsum = 16384.0f;      // each p_j < 2^14
    static constexpr float kMoveLog2 = 13.0f;
};

// x[lane] + x[lane ^ 32] without touching LDS: the swap returns {x_lo, x_lo} and {x_hi, x_hi}
__device__ __forceinline__ float pair_sum(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x),
                                                    false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float pair_max(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x),
                                                    false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
// the value held by the hh = 0 lane of the pair
__device__ __forceinline__ float pair_low(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x),
                                                    false, false);
    return __uint_as_float(r[0]);
}

// The largest scaled score (log2 units) of the lane pair's row over NB 32-key blocks; -inf
// if every key is masked.  Without a mask the raw dot products are compared and the result
// scaled once (a negative scale turns the order round).
template <int NB, bool MASK>
__device__ __forceinline__ float row_top_score(const f32x16 (&acc)[NB], float c_log2, int jb,
                                               int nvis) {
    const float ninf = -__builtin_inff();
    float m;
    if (!MASK) {
        if (c_log2 >= 0.0f) {
            m = acc[0][0];
#pragma unroll
            for (int kb = 0; kb < NB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) m = fmaxf(m, acc[kb][r]);
        } else {
            m = acc[0][0];
#pragma unroll
            for (int kb = 0; kb < NB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) m = fminf(m, acc[kb][r]);
        }
        m *= c_log2;
    } else {
        m = ninf;
#pragma unroll
        for (int kb = 0; kb < NB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float x = acc[kb][r] * c_log2;
                m = fmaxf(m, ((jb + 32 * kb + 8 * (r >> 2) + (r & 3)) >= nvis) ? ninf : x);
            }
    }
    return pair_max(m);
}

// acc: raw dot products of NB 32-key blocks in the accumulator layout (not modified).
// bfrag[g]: the coefficients of 16-key group g, rounded to the storage type, as the B
// operand of the output product.  jb = index of the key in register 0 of block 0 for this
// lane (tile start + 4 hh).  MASK = false: every key is visible to every row of the
// wavefront.  Returns true if the row is risky; its state is then left untouched.
// MAY_BE_EMPTY = false promises that no row of the wavefront is still empty (true from a
// row's second unit on); the code is then free of the first-key logic.
// TL: also carry the sum of the unrounded coefficients (LazyRow::ltrue).
// wary (wavefront-uniform) > 0: the wavefront has lately needed the checked step, so the
// rows' top scores are looked at before the exponentials (a few instructions, against a
// failed speculation that costs the tile's scores and exponentials a second time): a row
// whose top score lies more than LazyLimit::kMoveLog2 above its reference takes that score as
// its reference, what it holds is scaled by f = 2^{R - R'} (left to the caller: spec.fu,
// 1 for rows that stay, and spec.any_moved for the wavefront), and at least kWaryTiles more
// tiles are looked at; a tile that moves no reference counts wary.left down.  Every failed
// speculation multiplies the number of tiles the wavefront then stays wary for (wary.len) by
// 16: inputs whose scores keep jumping soon look at every tile (a failed speculation costs
// about one more tile, the look a percent of one), inputs of ordinary range never start.
// (Looking at every row's first tile as a matter of course was measured and lost 3-8 %: with
// the mask in play the look costs three instructions per score.)
constexpr int kWaryTiles = 64;
struct Wary {
    int left;     // > 0: look at the top scores before exponentiating
    int len;      // tiles to stay wary for after the next failed speculation
    __device__ __forceinline__ void failed() {
        left = len;
        len = len < (1 << 24) ? 16 * len : len;
    }
};

template <typename T, int NB, bool MASK, bool MAY_BE_EMPTY, bool TL>
__device__ __forceinline__ bool lazy_spec_pack(const f32x16 (&acc)[NB], u32x4 (&bfrag)[2 * NB],
                                               LazyRow& st, float c_log2, int jb, int nvis,
                                               int lane, LazySpec& spec, Wary& wary) {
    constexpr bool kTL = TL && Mma<T>::kRoundedSum;
    const float ninf = -__builtin_inff();
    bool empty = false;
    float ref = st.R;
    float fu = 1.0f;          // what the row holds (U, the carried sum) shrinks by this
    spec.any_moved = false;
    // a tile whose top scores have been looked at cannot hold a coefficient the storage type
    // does not: only a sum that is no number at all (NaN input) is then refused
    const float limit = (wary.left > 0) ? kLazyShiftMax : LazyLimit<T>::kMaxPsum;
    if (MAY_BE_EMPTY) {
        empty = st.one == 0.0f;
        // first key of the tile for this row: register 0 of block 0 in the hh = 0 lane
        const float s0 = pair_low(acc[0][0]) * c_log2;
        const float ref0 = ((jb - 4 * (lane >> 5)) < nvis) ? s0 : 0.0f;
        ref = empty ? ref0 : st.R;
    }
    spec.checked = wary.left > 0;
    if (spec.checked) {
        // branch-free apart from the wavefront-uniform test above: the few instructions
        // below cost less than waiting for a vector compare to reach a scalar branch
        const float m = row_top_score<NB, MASK>(acc, c_log2, jb, nvis);
        const bool move = !empty && (m - st.R > LazyLimit<T>::kMoveLog2);
        // an empty row starts from its top score rather than its first: no coefficient above 1
        if (MAY_BE_EMPTY) ref = (empty && m != ninf) ? m : ref;
        fu = move ? exp2_fast(st.R - m) : 1.0f;
        ref = move ? m : ref;
        spec.any_moved = __builtin_amdgcn_ballot_w64(move) != 0;
        wary.left = spec.any_moved ? (wary.left < kWaryTiles ? kWaryTiles : wary.left)
                                   : (wary.left > 0 ? wary.left - 1 : 0);
    }
    f32x4 ps4 = {0.0f, 0.0f, 0.0f, 0.0f};
    float pt0 = 0.0f, pt1 = 0.0f;
#pragma unroll
    for (int g = 0; g < 2 * NB; ++g) {
        f32x8 pv;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int r = 8 * (g & 1) + e;
            float x = fmaf(acc[g >> 1][r], c_log2, -ref);
            if (MASK) x = ((jb + 32 * (g >> 1) + 8 * (r >> 2) + (r & 3)) >= nvis) ? ninf : x;
            pv[e] = exp2_fast(x);
        }
        bfrag[g] = Mma<T>::pack8(pv);
        Mma<T>::sum8(pv, bfrag[g], ps4);
        if (kTL) {
#pragma unroll
            for (int e = 0; e < 8; e += 2) { pt0 += pv[e]; pt1 += pv[e + 1]; }
        }
        // Keep the groups apart: scheduled together, the 32 exponents and 32 results of a
        // tile are all live at once, and the register allocator then starts to move the
        // accumulators around.  Eight independent elements are enough to hide latencies.
        __builtin_amdgcn_sched_barrier(0);
    }
    float psum = pair_sum((ps4[0] + ps4[1]) + (ps4[2] + ps4[3]));
    spec.psum = psum;
    spec.ref = ref;
    spec.ptrue = kTL ? pair_sum(pt0 + pt1) : 0.0f;
    spec.fu = fu;
    const bool safe = psum <= limit;             // false for inf and NaN
    // 1/beta is the carried sum: beta' = 1 / (fu / beta + psum) = beta / (fu + beta psum)
    if (MAY_BE_EMPTY) {
        const bool upd = safe & !(empty & (psum == 0.0f));
        const float tot = fmaf(st.beta, psum, st.one * fu);
        const float nb = st.beta * __builtin_amdgcn_rcpf(tot);
        st.beta = upd ? nb : st.beta;
        st.R = upd ? ref : st.R;
        st.one = upd ? 1.0f : st.one;
        if (kTL) st.ltrue = upd ? fmaf(fu, st.ltrue, spec.ptrue) : st.ltrue;
    } else {
        const float nb = st.beta * __builtin_amdgcn_rcpf(fmaf(st.beta, psum, fu));
        st.beta = safe ? nb : st.beta;
        st.R = safe ? ref : st.R;
        if (kTL) st.ltrue = safe ? fmaf(fu, st.ltrue, spec.ptrue) : st.ltrue;
    }
    return !safe;
}

// Entered by the whole wavefront when some row is risky and every risky row's psum is an
// ordinary number, for a storage type whose coefficients have the range of fp32 (bf16): the
// coefficients of the speculative pass are still at hand and valid.  For a risky row the
// update of the state is the one of the common path (tot = one + beta psum); its reference
// moves up by e = exponent of psum (psum = m 2^e, 1/2 <= m < 1); what the row holds shrinks
// with it, U by 2^-e (the returned factor) and beta by 2^e the other way, o = beta U
// unchanged.  The coefficients are not formed again but scaled by 2^-e as they are, by taking
// e off the exponent field of each (two per instruction, saturating at zero), so that the
// coefficients the output product uses are bit for bit the ones whose sum went into the
// state (formed again at the new reference, one that sat on a rounding boundary could land
// on the other side).  Needs neither the raw scores nor an exponential, and no maximum.
template <bool TL>
__device__ __forceinline__ float lazy_shift_inplace_bf16(u32x4* bfrag, int ngroups, LazyRow& st,
                                                         bool risky, const LazySpec& spec) {
    typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
    float f = 1.0f;
    unsigned sub = 0u;                   // e in the position of the bf16 exponent field
    if (risky) {
        const int e = __builtin_amdgcn_frexp_expf(spec.psum);
        const bool empty = st.one == 0.0f;
        const float tot = fmaf(st.beta, spec.psum, st.one);
        const float nb = st.beta * __builtin_amdgcn_rcpf(tot);       // below 2^-e, then scaled up
        st.beta = __builtin_ldexpf(nb, e);
        st.R = spec.ref + (float)e;
        st.one = 1.0f;
        if (TL) st.ltrue = __builtin_ldexpf(st.ltrue + spec.ptrue, -e);
        f = empty ? 0.0f : __builtin_ldexpf(1.0f, -e);
        sub = (unsigned)e << 7;          // 0 < e <= 100: fits the field
    }
    // (whole vectors: a bit cast of a single vector element to a pair came out of this
    // compiler reading element 0 every time)
    const unsigned short s1 = (unsigned short)sub;
    const u16x8 s8 = {s1, s1, s1, s1, s1, s1, s1, s1};
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        if (g < ngroups) {
            const u16x8 x = __builtin_bit_cast(u16x8, bfrag[g]);
            bfrag[g] = __builtin_bit_cast(u32x4, __builtin_elementwise_sub_sat(x, s8));
        }
    }
    return f;
}

// The checked step.  Rows with update = true have not had this tile applied to their state
// yet; the others have (by lazy_spec_pack) and only get their coefficients formed again with
// the reference they used (same values).  For a row to update, the tile's top score m is
// compared with the reference first.  If m lies more than LazyLimit::kMoveLog2 above R (or
// the row is still empty) the reference moves to m: every coefficient is then 2^{s_j - m} <= 1,
// what the row holds is scaled by f = 2^{R - m} (the returned factor, for U; 1/beta, the
// carried sum, likewise), and a jump too large for fp32 simply makes f zero: the earlier keys'
// weight has saturated at 0 as the sigmoid's would (Sec. III-C).  Otherwise the reference
// stays and the coefficients are at most 2^kMoveLog2, which the storage type holds.  The sum
// can no longer overflow, so this step has no fallback of its own.  `moved` tells the caller
// whether this lane's U needs the factor.
template <typename T, int NB, bool MASK, bool TL>
__device__ __forceinline__ float lazy_checked_pack(const f32x16 (&acc)[NB], u32x4 (&bfrag)[2 * NB],
                                                   LazyRow& st, bool update, float c_log2, int jb,
                                                   int nvis, bool& moved) {
    constexpr bool kTL = TL && Mma<T>::kRoundedSum;
    const float ninf = -__builtin_inff();
    const float m = row_top_score<NB, MASK>(acc, c_log2, jb, nvis);
    const bool empty = st.one == 0.0f;
    float ref = st.R, f = 1.0f;
    moved = false;
    if (update) {
        const float mref = (m == ninf) ? 0.0f : m;
        const bool move = empty || (m - st.R > LazyLimit<T>::kMoveLog2);
        ref = move ? mref : st.R;
        f = empty ? 0.0f : (move ? exp2_fast(st.R - mref) : 1.0f);
        moved = move && !empty;
    }
    int nv = nvis;
    asm volatile("" : "+v"(nv));      // keep these compares apart from row_top_score's
    f32x4 ps4 = {0.0f, 0.0f, 0.0f, 0.0f};
    float pt0 = 0.0f, pt1 = 0.0f;
#pragma unroll
    for (int g = 0; g < 2 * NB; ++g) {
        f32x8 pv;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int r = 8 * (g & 1) + e;
            float x = fmaf(acc[g >> 1][r], c_log2, -ref);
            if (MASK) x = ((jb + 32 * (g >> 1) + 8 * (r >> 2) + (r & 3)) >= nv) ? ninf : x;
            pv[e] = exp2_fast(x);
        }
        bfrag[g] = Mma<T>::pack8(pv);
        Mma<T>::sum8(pv, bfrag[g], ps4);
        if (kTL) {
#pragma unroll
            for (int e = 0; e < 8; e += 2) { pt0 += pv[e]; pt1 += pv[e + 1]; }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    const float psum = pair_sum((ps4[0] + ps4[1]) + (ps4[2] + ps4[3]));
    const float ptrue = kTL ? pair_sum(pt0 + pt1) : 0.0f;
    if (update) {
        // 1/beta is the carried sum; against the new reference it shrinks by f
        const float carried = empty ? 0.0f : f * __builtin_amdgcn_rcpf(st.beta);
        const float tot = carried + psum;
        const bool has = tot > 0.0f;        // false only for an empty row that sees no key here
        st.beta = has ? __builtin_amdgcn_rcpf(tot) : st.beta;
        st.R = has ? ref : st.R;
        st.one = has ? 1.0f : st.one;
        if (kTL) st.ltrue = has ? fmaf(f, st.ltrue, ptrue) : st.ltrue;
    }
    return f;
}

// Alg. 2 on the same interface (ablation): m_i = max(m_{i-1}, s), l_i = l_{i-1}
// e^{m_{i-1}-m_i} + sum e^{s-m_i}; returns the factor e^{m_{i-1}-m_i} for the row's U, which
// is exactly 1 unless the maximum has moved (the caller skips the scaling of U while no row of
// the wavefront has a new maximum).
template <typename T, int NB, bool MASK>
__device__ __forceinline__ float online_pack(const f32x16 (&acc)[NB], u32x4 (&bfrag)[2 * NB],
                                             float& m, float& l, float c_log2, int jb, int nvis) {
    const float ninf = -__builtin_inff();
    const float mx = row_top_score<NB, MASK>(acc, c_log2, jb, nvis);
    const float m_new = fmaxf(m, mx);
    const float m_use = (m_new == ninf) ? 0.0f : m_new;
    const float resc = exp2_fast(m - m_use);
    int nv = nvis;
    asm volatile("" : "+v"(nv));
    f32x4 ps4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < 2 * NB; ++g) {
        f32x8 pv;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int r = 8 * (g & 1) + e;
            float x = fmaf(acc[g >> 1][r], c_log2, -m_use);
            if (MASK && (jb + 32 * (g >> 1) + 8 * (r >> 2) + (r & 3)) >= nv) x = ninf;
            pv[e] = exp2_fast(x);
        }
        bfrag[g] = Mma<T>::pack8(pv);
        Mma<T>::sum8(pv, bfrag[g], ps4);
        __builtin_amdgcn_sched_barrier(0);
    }
    const float psum = pair_sum((ps4[0] + ps4[1]) + (ps4[2] + ps4[3]));
    l = l * resc + psum;
    m = m_new;
    return resc;
}

// The blend of Sec. III-A applied literally per tile (variant TILE_BLEND): the row holds the
// output o itself (in U) and Lam; a tile of keys acts as one key of score
// Lam_tile = log2 sum_j 2^{s_j} and value o_tile = sum_j 2^{s_j - Lam_tile} v_j, its weight is
// W = sigmoid(Lam_tile - Lam) (weight equation of Sec. III-B on the run states), and
//     o <- (1 - W) o + W o_tile = (1 - W) o + sum_j c_j v_j,   c_j = 2^{s_j - Lam_new} <= 1,
//     Lam_new = Lam - log2(1 - W).
// Nothing is deferred: U is scaled by (1 - W) on every tile and the coefficients are final
// weights, so the stored row is U as it stands.  The sigmoid is evaluated from its saturating
// side, i.e. the exponentials are taken against ref = the larger of Lam and the tile's top
// score, where all of them are <= 1:  a = 2^{Lam - ref}, p_j = 2^{s_j - ref}, tot = a + sum p_j,
// 1 - W = a / tot, c_j = p_j / tot, Lam_new = ref + log2 tot.  No overflow is possible and
// there is no fallback path.  Where the coefficient sums are those of the rounded
// coefficients (bf16), 1 - W is taken as 1 - sum of the rounded c_j, so that the row stays a
// weighted mean of the values.  Returns 1 - W (the factor for U).
struct BlendRow {
    float lam;    // log2 units; meaningless while one == 0
    float one;    // 0.0f while the row is empty, then 1.0f
};

template <typename T, int NB, bool MASK>
__device__ __forceinline__ float blend_pack(const f32x16 (&acc)[NB], u32x4 (&bfrag)[2 * NB],
                                            BlendRow& st, float c_log2, int jb, int nvis) {
    const float ninf = -__builtin_inff();
    const float m = row_top_score<NB, MASK>(acc, c_log2, jb, nvis);
    const bool empty = st.one == 0.0f;
    const float mref = (m == ninf) ? 0.0f : m;
    const float ref = empty ? mref : fmaxf(st.lam, m);
    const float a = empty ? 0.0f : exp2_fast(st.lam - ref);
    int nv = nvis;
    asm volatile("" : "+v"(nv));
    f32x8 pv[2 * NB];
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
#pragma unroll
    for (int g = 0; g < 2 * NB; ++g) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int r = 8 * (g & 1) + e;
            float x = fmaf(acc[g >> 1][r], c_log2, -ref);
            if (MASK && (jb + 32 * (g >> 1) + 8 * (r >> 2) + (r & 3)) >= nv) x = ninf;
            pv[g][e] = exp2_fast(x);
        }
#pragma unroll
        for (int e = 0; e < 8; e += 4) {
            s0 += pv[g][e]; s1 += pv[g][e + 1]; s2 += pv[g][e + 2]; s3 += pv[g][e + 3];
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    const float psum = pair_sum((s0 + s1) + (s2 + s3));
    const float tot = a + psum;
    const bool has = tot > 0.0f;            // false only for an empty row that sees no key here
    const float cs = has ? __builtin_amdgcn_rcpf(tot) : 0.0f;
    f32x4 cs4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < 2 * NB; ++g) {
        f32x8 cv;
#pragma unroll
        for (int e = 0; e < 8; ++e) cv[e] = pv[g][e] * cs;
        bfrag[g] = Mma<T>::pack8(cv);
        if (Mma<T>::kRoundedSum) Mma<T>::sum8(cv, bfrag[g], cs4);
        __builtin_amdgcn_sched_barrier(0);
    }
    float omw = a * cs;                      // 1 - W = sigmoid(Lam - Lam_tile)
    if (Mma<T>::kRoundedSum) {
        const float csum = pair_sum((cs4[0] + cs4[1]) + (cs4[2] + cs4[3]));
        omw = fmaxf(1.0f - csum, 0.0f);
    }
    st.lam = has ? ref + log2_fast(tot) : st.lam;
    st.one = has ? 1.0f : st.one;
    return empty ? 0.0f : omw;
}

// What a finished row hands on: the factor that turns U into the output, and the row's
// Lam (log2 units) for a later merge with other key ranges.
template <bool ONLINE>
__device__ __forceinline__ void row_finish(float lam, float beta, float& fin, float& lam_out) {
    if (!ONLINE) {
        fin = beta;                 // FLASH-D: the state is the output
        lam_out = lam;
    } else {
        fin = beta > 0.0f ? 1.0f / beta : 0.0f;      // the one division of Alg. 2
        lam_out = beta > 0.0f ? lam + log2_fast(beta) : -__builtin_inff();
    }
}

// Keys visible to query position pos of a head (0 <= pos < Li.d).
__device__ __forceinline__ int visible_at(const Problem& p, int pos) {
    if (!p.causal) return p.Lk;
    return min(max(pos + p.shift + 1, 0), p.Lk);
}

// Keys visible to row i of a head as the kernel sees heads (Lq rows, row i standing for
// position i % Li.d); rows past the end see none.
__device__ __forceinline__ int visible_count(const Problem& p, int i) {
    if (i >= p.Lq) return 0;
    // i % Li, branch-free: the rule runs per lane
    return visible_at(p, i - (int)(fast_div((uint32_t)i, p.Li) * p.Li.d));
}

}  // namespace flashd
