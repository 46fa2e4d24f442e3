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
    static __device__ __forceinline__ u32x2 pack4(f32x4 x) {
        return __builtin_bit_cast(u32x2, __builtin_convertvector(x, bf16x4));
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
    static __device__ __forceinline__ u32x2 pack4(f32x4 x) {
        return __builtin_bit_cast(u32x2, __builtin_convertvector(x, f16x4));
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
// The tile rule of Alg. 3 with the blend factor kept as a scalar ("lazy blend"), used by the
// prefill and the decode kernel.  After a run of keys the state of Alg. 3 is
// (o, s_last, ln w_last) and only Lam = s_last - ln w_last enters later steps; a tile of keys
// acts as one key.  A row's state here is (U, R, beta, one):
//     true output o = beta U,   Lam = R - log2 beta,   one = 0 until the row has seen a key.
// For a tile, with p_j = 2^{s_j - R} (R does not move on this path) and psum = sum_j p_j,
//     tot = one + beta psum,   1 - W = 1/tot   (W = sigmoid(S_tile - Lam), the tile's weight),
//     U <- U + sum_j p_j v_j,  beta <- beta (1 - W).
// This is o <- (1 - W)(o + sum_j 2^{s_j - Lam} v_j) with the vector multiplication by
// (1 - W) folded into the scalar beta: U is never rescaled here.  An empty row takes the
// score of the tile's first key as R (w_1 = 1 for that key).
//
// lazy_spec_pack() does that speculatively, branch-free, leaving the raw scores untouched,
// and reports rows whose psum left the safe range (some 2^{s_j - R} too large for the
// storage type: a score far above everything before it).  If that psum is still an ordinary
// fp32 number the tile's total is known and only the coefficients do not fit:
// lazy_shift_pack() moves the row's reference up by a power of two and rounds the
// coefficients again.  If psum itself overflowed, lazy_redo_pack() redoes the tile from the
// raw scores with the key-by-key sigmoid recurrence, which saturates instead of overflowing,
// and moves R.
struct LazyRow {
    float R;      // exponent reference, log2 units
    float beta;   // o = beta * U
    float one;    // 0.0f while the row is empty, then 1.0f
};

// What the speculative pass found for a row: the sum of its coefficients and the reference
// they were taken against (the row's R, or the tile's first visible score for an empty row).
struct LazySpec {
    float psum;
    float ref;
};

// psum above this is treated as overflowed.  Below it one + beta psum (beta <= 2) stays far
// under 2^126, so that its reciprocal is still a normal number (v_rcp_f32 returns zero where
// the result would be subnormal, and a beta of zero would poison the row).
constexpr float kLazyShiftMax = 1.0e30f;      // ~2^100

template <typename T> struct LazyLimit;
template <> struct LazyLimit<BF16> { static constexpr float kMaxPsum = 1.0e18f; };   // ~2^60
template <> struct LazyLimit<F16> { static constexpr float kMaxPsum = 16384.0f; };   // each p_j < 2^14

// x[lane] + x[lane ^ 32] without touching LDS: the swap returns {x_lo, x_lo} and {x_hi, x_hi}
__device__ __forceinline__ float pair_sum(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x),
                                                    false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// the value held by the hh = 0 lane of the pair
__device__ __forceinline__ float pair_low(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x),
                                                    false, false);
    return __uint_as_float(r[0]);
}

// acc: raw dot products of NB 32-key blocks in the accumulator layout (not modified).
// bfrag[g]: the coefficients of 16-key group g, rounded to the storage type, as the B
// operand of the output product.  jb = index of the key in register 0 of block 0 for this
// lane (tile start + 4 hh).  MASK = false: every key is visible to every row of the
// wavefront.  Returns true if the row is risky; its state is then left untouched.
// MAY_BE_EMPTY = false promises that no row of the wavefront is still empty (true from a
// row's second unit on); the code is then free of the first-key logic and stays one
// basic block, which the caller needs to interleave it with matrix instructions.
template <typename T, int NB, bool MASK, bool MAY_BE_EMPTY>
__device__ __forceinline__ bool lazy_spec_pack(const f32x16 (&acc)[NB], u32x4 (&bfrag)[2 * NB],
                                               LazyRow& st, float c_log2, int jb, int nvis,
                                               int lane, LazySpec& spec) {
    const float ninf = -__builtin_inff();
    bool empty = false;
    float ref = st.R;
    if (MAY_BE_EMPTY) {
        empty = st.one == 0.0f;
        // first key of the tile for this row: register 0 of block 0 in the hh = 0 lane
        const float s0 = pair_low(acc[0][0]) * c_log2;
        const float ref0 = ((jb - 4 * (lane >> 5)) < nvis) ? s0 : 0.0f;
        ref = empty ? ref0 : st.R;
    }
    f32x4 ps4 = {0.0f, 0.0f, 0.0f, 0.0f};
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
        // Keep the groups apart: scheduled together, the 32 exponents and 32 results of a
        // tile are all live at once, and the register allocator then starts to move the
        // accumulators around.  Eight independent elements are enough to hide latencies.
        __builtin_amdgcn_sched_barrier(0);
    }
    float psum = pair_sum((ps4[0] + ps4[1]) + (ps4[2] + ps4[3]));
    spec.psum = psum;
    spec.ref = ref;
    const bool safe = psum <= LazyLimit<T>::kMaxPsum;             // false for inf and NaN
    if (MAY_BE_EMPTY) {
        const bool upd = safe & !(empty & (psum == 0.0f));
        const float tot = fmaf(st.beta, psum, st.one);
        const float nb = st.beta * __builtin_amdgcn_rcpf(tot);
        st.beta = upd ? nb : st.beta;
        st.R = upd ? ref : st.R;
        st.one = upd ? 1.0f : st.one;
    } else {
        const float nb = st.beta * __builtin_amdgcn_rcpf(fmaf(st.beta, psum, 1.0f));
        st.beta = safe ? nb : st.beta;
    }
    return !safe;
}

// Middle path, entered by the whole wavefront when some row is risky and every risky row's
// psum is an ordinary number.  For a risky row the update of the state is the one of the
// common path (tot = one + beta psum); its reference moves up by e = exponent of psum
// (psum = m 2^e, 1/2 <= m < 1), so that every coefficient 2^{s_j - R - e} <= m < 1 fits the
// storage type; what the row holds shrinks with it, U by 2^-e (the returned factor) and beta
// by 2^e the other way, o = beta U unchanged.  The other rows' coefficients are formed again
// with the reference they used (same values).  No maximum is taken and no key is looked at
// on its own.
template <typename T, int NB>
__device__ __forceinline__ float lazy_shift_pack(const f32x16 (&acc)[NB], u32x4 (&bfrag)[2 * NB],
                                                 LazyRow& st, bool risky, const LazySpec& spec,
                                                 float c_log2, bool need_mask, int jb, int nvis) {
    const float ninf = -__builtin_inff();
    float f = 1.0f;
    float ref = st.R;     // rows that were not risky: the reference lazy_spec_pack used
    if (risky) {
        const int e = __builtin_amdgcn_frexp_expf(spec.psum);
        const bool empty = st.one == 0.0f;
        const float tot = fmaf(st.beta, spec.psum, st.one);
        const float nb = st.beta * __builtin_amdgcn_rcpf(tot);       // below 2^-e, then scaled up
        st.beta = __builtin_ldexpf(nb, e);
        ref = spec.ref + (float)e;
        st.R = ref;
        st.one = 1.0f;
        f = empty ? 0.0f : __builtin_ldexpf(1.0f, -e);
    }
    int nv = nvis;
    asm volatile("" : "+v"(nv));      // see lazy_redo_pack
#pragma unroll
    for (int g = 0; g < 2 * NB; ++g) {
        f32x8 pv;
#pragma unroll
        for (int e8 = 0; e8 < 8; ++e8) {
            const int r = 8 * (g & 1) + e8;
            float x = fmaf(acc[g >> 1][r], c_log2, -ref);
            const bool masked = need_mask && (jb + 32 * (g >> 1) + 8 * (r >> 2) + (r & 3)) >= nv;
            if (masked) x = ninf;
            pv[e8] = exp2_fast(x);
        }
        bfrag[g] = Mma<T>::pack8(pv);
        __builtin_amdgcn_sched_barrier(0);
    }
    return f;
}

// The same middle path where the coefficients of the speculative pass are still at hand and
// have the range of fp32 (bf16): they are not formed again but scaled by 2^-e as they are,
// by taking e off the exponent field of each (two per instruction, saturating at zero), so
// that the coefficients the output product uses are bit for bit the ones whose sum went into
// the state (formed again at the new reference, one that sat on a rounding boundary could
// land on the other side).  Needs neither the raw scores nor an exponential.
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

// Rare path, entered by the whole wavefront when any of its rows is risky.  Key-by-key
// recurrence inside the lane over the raw scores: Lam_j = Lam_{j-1} + softplus(s_j -
// Lam_{j-1}), i.e. w_j = sigmoid(s_j - s_{j-1} + ln w_{j-1}) carried as Lam = s - ln w; the
// first visible key starts the run (w = 1); the lane pair and the carried state are folded
// by the same rule.  Risky rows get c_j = 2^{s_j - Lam_new} <= 1 and a new reference; the
// other rows' coefficients are recomputed with the reference they used (same values; a
// row that is still empty has every key masked, so its reference does not matter).
// Returns the factor for the row's U (1 for rows that were not risky).
template <typename T, int NB>
__device__ __forceinline__ float lazy_redo_pack(const f32x16 (&acc)[NB], u32x4 (&bfrag)[2 * NB],
                                                LazyRow& st, bool risky, float c_log2,
                                                bool need_mask, int jb, int nvis) {
    const float ninf = -__builtin_inff();
    // The mask compares are redone here from values the compiler cannot connect with the
    // ones of lazy_spec_pack (empty asm); shared, 32 compare results would stay live
    // across the branch into this rare path.
    int nv1 = nvis, nv2 = nvis;
    asm volatile("" : "+v"(nv1));
    float ll = ninf;
#pragma unroll
    for (int kb = 0; kb < NB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool masked = need_mask && (jb + 32 * kb + 8 * (r >> 2) + (r & 3)) >= nv1;
            ll = lse2(ll, masked ? ninf : acc[kb][r] * c_log2);
            // rare path: keep it sequential so that it does not add to the register need
            if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }
    ll = lse2(ll, __shfl_xor(ll, 32, 64));                  // partner lane's run
    const bool empty = st.one == 0.0f;
    const float lam_old = empty ? ninf : st.R - log2_fast(st.beta);
    const float lam_new = lse2(lam_old, ll);                  // the tile acts as one key
    const bool none = risky && lam_new == ninf;
    float f = 1.0f;
    float ref = st.R;     // rows that were not risky: the reference lazy_spec_pack used
    float w_old = 0.0f;   // 1 - W = 2^{Lam_old - Lam_new}: what is left of the old state
    if (risky) {
        ref = none ? 0.0f : lam_new;
        w_old = empty ? 0.0f : exp2_fast(lam_old - lam_new);
        f = st.beta * w_old;            // applied to U now
        st.R = ref;
        st.one = none ? 0.0f : 1.0f;
    }
    asm volatile("" : "+v"(nv2));
    f32x4 ps4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < 2 * NB; ++g) {
        f32x8 pv;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int r = 8 * (g & 1) + e;
            float x = fmaf(acc[g >> 1][r], c_log2, -ref);
            const bool masked =
                need_mask && (jb + 32 * (g >> 1) + 8 * (r >> 2) + (r & 3)) >= nv2;
            if (masked || none) x = ninf;
            pv[e] = exp2_fast(x);
        }
        bfrag[g] = Mma<T>::pack8(pv);
        if (Mma<T>::kRoundedSum) Mma<T>::sum8(pv, bfrag[g], ps4);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (risky) {
        // Exactly, w_old and the tile's coefficients sum to one and beta is 1.  Where the row
        // sums are those of the rounded coefficients (Mma::sum8) beta takes the sum they
        // really have, so that o = beta U stays a weighted mean of the values.
        float tot = 1.0f;
        if (Mma<T>::kRoundedSum) tot = w_old + pair_sum((ps4[0] + ps4[1]) + (ps4[2] + ps4[3]));
        st.beta = (none || !Mma<T>::kRoundedSum) ? 1.0f : __builtin_amdgcn_rcpf(tot);
    }
    return f;
}

// Alg. 2 on the same interface (ablation): m_i = max(m_{i-1}, s), l_i = l_{i-1}
// e^{m_{i-1}-m_i} + sum e^{s-m_i}; returns the factor e^{m_{i-1}-m_i} for the row's U.
template <typename T, int NB, bool MASK>
__device__ __forceinline__ float online_pack(const f32x16 (&acc)[NB], u32x4 (&bfrag)[2 * NB],
                                             float& m, float& l, float c_log2, int jb, int nvis) {
    const float ninf = -__builtin_inff();
    float mx = ninf;
#pragma unroll
    for (int kb = 0; kb < NB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float s = acc[kb][r] * c_log2;
            if (MASK && (jb + 32 * kb + 8 * (r >> 2) + (r & 3)) >= nvis) s = ninf;
            mx = fmaxf(mx, s);
        }
    {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx),
                                                         false, false);
        mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    }
    const float m_new = fmaxf(m, mx);
    const float m_use = (m_new == ninf) ? 0.0f : m_new;
    const float resc = exp2_fast(m - m_use);
    f32x4 ps4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < 2 * NB; ++g) {
        f32x8 pv;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int r = 8 * (g & 1) + e;
            float x = fmaf(acc[g >> 1][r], c_log2, -m_use);
            if (MASK && (jb + 32 * (g >> 1) + 8 * (r >> 2) + (r & 3)) >= nvis) x = ninf;
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
