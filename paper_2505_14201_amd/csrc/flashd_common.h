// Shared device-side pieces of libflashd: storage-type traits, the problem
// descriptor passed to kernels, and the sigmoid-rule primitives on a state.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace flashd {

constexpr int kWave = 64;

// Division of a 32-bit unsigned number by a divisor fixed at launch, without a division
// instruction (Granlund and Montgomery's round-up multiplier: with l = ceil(log2 d) and
// m = floor(2^32 (2^l - d) / d) + 1, the quotient of any n < 2^32 is
// (t + ((n - t) >> min(l, 1))) >> max(l - 1, 0), t = high word of m * n; exact for d >= 1).
struct FastDiv {
    uint32_t d, m;
    int s1, s2;
};

inline FastDiv make_fast_div(uint32_t d) {
    FastDiv f;
    f.d = d;
    int l = 0;
    while ((1ull << l) < (unsigned long long)d) ++l;
    f.m = (uint32_t)((((1ull << l) - (unsigned long long)d) << 32) / (unsigned long long)d + 1);
    f.s1 = l < 1 ? l : 1;
    f.s2 = l > 1 ? l - 1 : 0;
    return f;
}

__host__ __device__ __forceinline__ uint32_t fast_div(uint32_t n, const FastDiv& f) {
    const uint32_t t = (uint32_t)(((uint64_t)f.m * n) >> 32);       // one v_mul_hi_u32
    return (t + ((n - t) >> f.s1)) >> f.s2;
}

struct Problem {
    const void* q;
    const void* k;
    const void* v;
    void* o;
    float* ws;          // split-K partial states, [splits][B][Hq][Lq][d + 2] fp32
    int B, Hq, Hkv, Lq, Lk, d;
    int dtype;          // flashd_dtype: 0 f32, 1 f16, 2 bf16
    int causal;         // 0/1
    int splits;         // >= 1
    float scale;
    int shift;          // causal: key j is visible to query i iff j <= i + shift
    int partial;        // 1: the main kernel writes partial states to ws (always with splits > 1)
    int store_o;        // 1: the main kernel stores the output in the storage type
    int merge;          // 1: merge_splits_kernel runs after the main kernel
    int from_state;     // 1: the tile kernel starts every row from state_in (no merge needed)
    int kv8;            // 1: k and v hold fp8 (e4m3) elements, scaled by kscale / vscale
    float kscale, vscale;
    float oscale;       // factor on the output (and on the o of partial states); 1 unless kv8
    const float* state_in;   // optional state of earlier keys, [B][Hq][Lq][d + 2] fp32
    float* state_out;        // optional state after this call's keys, same layout
    int wide;           // 1: the tiled prefill takes the 256-row kernel where it can serve the call
    unsigned long long* vskip_counts;   // optional, decode kernel with saturation skips:
                                        // [0] += 32-key blocks visited, [1] += blocks whose V was not fetched
    FastDiv Li;         // causal rule: row r of a head stands for query position r % Li.d.  Li.d == Lq
                        // except where the tile kernel runs the heads of a kv group as one head
};

// ---- storage types -------------------------------------------------------

struct F32 { using raw = float; };
struct F16 { using raw = _Float16; };
struct BF16 { using raw = uint16_t; };

__device__ __forceinline__ float bf16_to_f32(uint16_t x) {
    return __uint_as_float(static_cast<uint32_t>(x) << 16);
}

// round-to-nearest-even; inputs here are finite or +-inf (NaN stays NaN)
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

template <typename T> struct Store;
template <> struct Store<F32> {
    static __device__ __forceinline__ float load(const void* p, size_t i) {
        return static_cast<const float*>(p)[i];
    }
    static __device__ __forceinline__ void store(void* p, size_t i, float x) {
        static_cast<float*>(p)[i] = x;
    }
    // 8 consecutive elements starting at element index i (i % 8 == 0)
    static __device__ __forceinline__ void load8(const void* p, size_t i, float (&out)[8]) {
        const float4* s = reinterpret_cast<const float4*>(static_cast<const float*>(p) + i);
        float4 a = s[0], b = s[1];
        out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
        out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
    }
};
template <> struct Store<F16> {
    static __device__ __forceinline__ float load(const void* p, size_t i) {
        return static_cast<float>(static_cast<const _Float16*>(p)[i]);
    }
    static __device__ __forceinline__ void store(void* p, size_t i, float x) {
        static_cast<_Float16*>(p)[i] = static_cast<_Float16>(x);
    }
    static __device__ __forceinline__ void load8(const void* p, size_t i, float (&out)[8]) {
        typedef _Float16 h8 __attribute__((ext_vector_type(8)));
        h8 a = *reinterpret_cast<const h8*>(static_cast<const _Float16*>(p) + i);
#pragma unroll
        for (int t = 0; t < 8; ++t) out[t] = static_cast<float>(a[t]);
    }
};
template <> struct Store<BF16> {
    static __device__ __forceinline__ float load(const void* p, size_t i) {
        return bf16_to_f32(static_cast<const uint16_t*>(p)[i]);
    }
    static __device__ __forceinline__ void store(void* p, size_t i, float x) {
        static_cast<uint16_t*>(p)[i] = f32_to_bf16(x);
    }
    static __device__ __forceinline__ void load8(const void* p, size_t i, float (&out)[8]) {
        uint4 a = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(p) + i);
        uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            out[2 * t] = __uint_as_float(w[t] << 16);
            out[2 * t + 1] = __uint_as_float(w[t] & 0xffff0000u);
        }
    }
};

// ---- the sigmoid rule ------------------------------------------------------
//
// Weight equation of Sec. III-B: w_i = sigmoid(x), x = s_i - s_{i-1} + ln w_{i-1}.
// The next step needs ln w_i; it is taken from x (ln sigmoid(x)), never from the
// rounded w_i, so a weight that rounds to 0 or 1 still carries its logarithm.
// Both are evaluated through e^{-|x|} <= 1, which cannot overflow: this is the
// saturation the paper's stability argument (Sec. III-C) relies on.
__device__ __forceinline__ void sigmoid_and_log(float x, float& w, float& lnw) {
    float e = __expf(-fabsf(x));          // in (0, 1]; 0 once |x| > ~104
    float t = 1.0f + e;
    float r = __frcp_rn(t);
    float lt = __logf(t);                 // ln(1 + e) in [0, ln 2]
    bool pos = x >= 0.0f;
    w = pos ? r : e * r;
    lnw = pos ? -lt : x - lt;
}

// The same step with the argument and the logarithm carried in fp64 (fp32 storage: scores of
// several hundred have an fp32 spacing of 6e-5, which as an error of s - ln w is a relative
// error of every later weight; the stated fp32 tolerance is 1e-5).  Only sums and differences
// of large terms are fp64; the exponential and the logarithm see a rounded argument whose
// error no longer matters (|x| <= 104 wherever e is not zero, and ln(1 + e) <= ln 2).
__device__ __forceinline__ void sigmoid_and_log(double x, float& w, double& lnw) {
    const float xf = static_cast<float>(x);
    float e = __expf(-fabsf(xf));
    float t = 1.0f + e;
    float r = __frcp_rn(t);
    float lt = __logf(t);
    bool pos = x >= 0.0;
    w = pos ? r : e * r;
    lnw = pos ? -static_cast<double>(lt) : x - static_cast<double>(lt);
}

// A run of keys is summarised by (o, lam) with lam = s_last - ln w_last; the empty
// run has lam = -inf.  Appending run B to run A treats B as one key of score lam_b
// and value o_b: W = sigmoid(lam_b - lam_a), o = o_a + (o_b - o_a) W (Sec. IV-A
// form of the blend), lam = lam_b - ln W.
__device__ __forceinline__ void merge_weight(float lam_a, float lam_b, float& W, float& lam) {
    const float ninf = -__builtin_inff();
    if (lam_b == ninf) { W = 0.0f; lam = lam_a; return; }
    if (lam_a == ninf) { W = 1.0f; lam = lam_b; return; }
    float lnW;
    sigmoid_and_log(lam_b - lam_a, W, lnW);
    lam = lam_b - lnW;
}
__device__ __forceinline__ void merge_weight(double lam_a, double lam_b, float& W, double& lam) {
    const double ninf = -__builtin_inf();
    if (lam_b == ninf) { W = 0.0f; lam = lam_a; return; }
    if (lam_a == ninf) { W = 1.0f; lam = lam_b; return; }
    double lnW;
    sigmoid_and_log(lam_b - lam_a, W, lnW);
    lam = lam_b - lnW;
}

// A state's (s, ln w) pair as two floats whose difference is lam: fp32 storage keeps what
// lam needs beyond one float in ln w (only s - ln w enters later steps).
__device__ __forceinline__ void split_lam(float lam, float& s, float& lnw) { s = lam; lnw = 0.0f; }
__device__ __forceinline__ void split_lam(double lam, float& s, float& lnw) {
    s = static_cast<float>(lam);
    lnw = (s == -__builtin_inff()) ? 0.0f : static_cast<float>(static_cast<double>(s) - lam);
}

}  // namespace flashd
