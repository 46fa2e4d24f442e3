// Alg. 3 taken literally: one sigmoid per key (variant PER_KEY), any storage type,
// fp32 arithmetic on the vector ALU.  This is the exact-by-construction path (fp32
// inputs use it) and the slow reference for the tiled kernels.
//
// Work split: a wavefront owns R query rows of one (b, h) and one key range
// (split); the 4 wavefronts of a workgroup share the K and V tiles in LDS.
// Lane t walks keys k0+t, k0+t+64, ... and runs the recurrence of Alg. 3
// over ITS subsequence with the state (s_prev, ln w_prev, o) in registers, exactly
// as the algorithm box states it.  The 64 lane states are then folded pairwise by
// the same sigmoid rule (a run of keys acts as one key with score
// s_last - ln w_last), and so are the split partials in a second kernel.
#include "flashd_common.h"
#include "flashd_kernels.h"

#include <type_traits>

namespace flashd {

template <int D> struct PerKeyCfg { static constexpr int R = (D <= 64) ? 2 : 1; };
constexpr int kPerKeyWaves = 4;
constexpr int kPerKeyTile = kWave;            // keys per tile: one per lane

typedef uint32_t pk_u32x4 __attribute__((ext_vector_type(4)));

// 16 bytes of storage -> fp32 values (4 for fp32 storage, 8 for the 16-bit types)
template <typename T> struct Chunk;
typedef __bf16 pk_bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 pk_f16x2 __attribute__((ext_vector_type(2)));

template <> struct Chunk<F32> {
    static constexpr int N = 4;
    static constexpr bool kPairs = false;        // scores by fma on the widened values
    // fp32 storage: the dot product, the score and s - ln w are carried in fp64 (same fma
    // rate as unpacked fp32 on this part), so that the stated 1e-5 holds whatever the size
    // of the scores; weights and the blend of Alg. 3 stay fp32
    using state_t = double;
    static __device__ __forceinline__ void unpack(pk_u32x4 w, float (&out)[4]) {
#pragma unroll
        for (int t = 0; t < 4; ++t) out[t] = __uint_as_float(w[t]);
    }
};
template <> struct Chunk<BF16> {
    static constexpr int N = 8;
    using state_t = float;
    // Scores of the 16-bit types: q and k stay packed, two products per v_dot2 (exact
    // products, fp32 accumulation, subnormals kept), no widening of K
    static constexpr bool kPairs = true;
    static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(pk_bf16x2, a),
                                               __builtin_bit_cast(pk_bf16x2, b), c, false);
    }
    static __device__ __forceinline__ void unpack(pk_u32x4 w, float (&out)[8]) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            out[2 * t] = __uint_as_float(w[t] << 16);
            out[2 * t + 1] = __uint_as_float(w[t] & 0xffff0000u);
        }
    }
};
template <> struct Chunk<F16> {
    static constexpr int N = 8;
    using state_t = float;
    static constexpr bool kPairs = true;
    static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(pk_f16x2, a),
                                      __builtin_bit_cast(pk_f16x2, b), c, false);
    }
    static __device__ __forceinline__ void unpack(pk_u32x4 w, float (&out)[8]) {
        typedef _Float16 h8 __attribute__((ext_vector_type(8)));
        const h8 a = __builtin_bit_cast(h8, w);
#pragma unroll
        for (int t = 0; t < 8; ++t) out[t] = static_cast<float>(a[t]);
    }
};

// A workgroup of 4 wavefronts owns 4 R query rows of one (b, h) and one key range.  K and V
// go through LDS in tiles of 64 keys, fetched once per workgroup in coalesced 16-byte chunks
// (each lane reading its own key row straight from global memory touches 64 cache lines per
// load instruction, and every row of the workgroup would fetch the tile again: that traffic,
// not the arithmetic, set the pace).  The next tile is requested into registers before the
// current one is worked on.  Chunk c of key row r sits at chunk position c ^ (r % 8), so that
// the 64 lanes, each reading chunk c of its own row, spread over all banks.
template <typename T, int D>
__global__ __launch_bounds__(kPerKeyWaves * kWave)
void perkey_kernel(Problem p) {
    constexpr int R = PerKeyCfg<D>::R;
    constexpr int ROWS_PER_BLOCK = R * kPerKeyWaves;
    constexpr int EPC = Chunk<T>::N;                     // elements per 16-byte chunk
    constexpr int CPR = D / EPC;                         // chunks per key row
    constexpr int kThreads = kPerKeyWaves * kWave;
    constexpr int NCH = kPerKeyTile * CPR / kThreads;    // chunks per thread, tensor and tile
    static_assert(kPerKeyTile * CPR % kThreads == 0 && CPR % 8 == 0, "tile does not divide");
    using state_t = typename Chunk<T>::state_t;
    constexpr bool kWide = std::is_same<state_t, double>::value;
    __shared__ float lds[ROWS_PER_BLOCK][D];
    __shared__ double qwide[kWide ? ROWS_PER_BLOCK : 1][kWide ? D : 1];   // q widened once
    __shared__ uint32_t qpairs[ROWS_PER_BLOCK][D / 2];      // q as stored, two per word (16-bit types)
    __shared__ __align__(16) pk_u32x4 kt[kPerKeyTile * CPR];
    __shared__ __align__(16) pk_u32x4 vt[kPerKeyTile * CPR];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int row_blocks = (p.Lq + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    const int rb = blockIdx.x % row_blocks;
    const int sp = blockIdx.x / row_blocks;
    const int h = blockIdx.y;
    const int b = blockIdx.z;
    const int kvh = h / (p.Hq / p.Hkv);
    const int i0 = rb * ROWS_PER_BLOCK + wave * R;

    const size_t qbase = ((size_t)b * p.Hq + h) * (size_t)p.Lq * D;
    const size_t kbase = ((size_t)b * p.Hkv + kvh) * (size_t)p.Lk * D;

    // query rows -> LDS (wave-private rows), read back as broadcasts
    float (*qs)[D] = &lds[wave * R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i = i0 + r;
        for (int t = lane; t < D; t += kWave)
            qs[r][t] = (i < p.Lq) ? Store<T>::load(p.q, qbase + (size_t)i * D + t) : 0.0f;
        if constexpr (kWide)
            for (int t = lane; t < D; t += kWave) qwide[wave * R + r][t] = (double)qs[r][t];
        if constexpr (Chunk<T>::kPairs) {
            const uint32_t* qw = static_cast<const uint32_t*>(p.q) + (qbase + (size_t)i * D) / 2;
            for (int t = lane; t < D / 2; t += kWave)
                qpairs[wave * R + r][t] = (i < p.Lq) ? qw[t] : 0u;
        }
    }
    const uint32_t (*qp)[D / 2] = &qpairs[wave * R];

    // key range of this split, and how many keys each row may see
    const int chunk = (p.Lk + p.splits - 1) / p.splits;
    const int k0 = sp * chunk;
    const int k1 = min(p.Lk, k0 + chunk);
    auto visible = [&](int i) {
        if (i >= p.Lq) return 0;
        return p.causal ? min(max(i + p.shift + 1, 0), p.Lk) : p.Lk;
    };
    int nvis[R];
#pragma unroll
    for (int r = 0; r < R; ++r) nvis[r] = min(visible(i0 + r), k1);
    // the workgroup walks the tiles that any of its rows can see (its last row sees the most)
    const int kend = min(visible(min(rb * ROWS_PER_BLOCK + ROWS_PER_BLOCK, p.Lq) - 1), k1);

    float o[R][D];
    state_t s_prev[R], lnw[R];
    bool has[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        s_prev[r] = 0; lnw[r] = 0; has[r] = false;
#pragma unroll
        for (int t = 0; t < D; ++t) o[r][t] = 0.0f;
    }

    const char* kg = static_cast<const char*>(p.k) + kbase * sizeof(typename T::raw);
    const char* vg = static_cast<const char*>(p.v) + kbase * sizeof(typename T::raw);
    pk_u32x4 kreg[NCH], vreg[NCH];
    auto fetch = [&](int jt) {
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
            const int ci = tid + kThreads * n;           // chunk of the tile, row-major
            const int row = ci / CPR;
            const int c = ci % CPR;
            const size_t off = ((size_t)min(jt + row, p.Lk - 1) * CPR + c) * 16;
            kreg[n] = *reinterpret_cast<const pk_u32x4*>(kg + off);
            vreg[n] = *reinterpret_cast<const pk_u32x4*>(vg + off);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
            const int ci = tid + kThreads * n;
            const int row = ci / CPR;
            const int c = ci % CPR;
            kt[row * CPR + (c ^ (row & 7))] = kreg[n];
            vt[row * CPR + (c ^ (row & 7))] = vreg[n];
        }
    };

    if (k0 < kend) fetch(k0);
    for (int jt = k0; jt < kend; jt += kPerKeyTile) {
        stash();
        __syncthreads();
        if (jt + kPerKeyTile < kend) fetch(jt + kPerKeyTile);
        const int j = jt + lane;                         // this lane's key
        if (i0 < p.Lq) {
            state_t s[R];
            if constexpr (Chunk<T>::kPairs) {
                float part[R][4];                // four chains per row, added at the end
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int t = 0; t < 4; ++t) part[r][t] = 0.0f;
#pragma unroll
                for (int c = 0; c < CPR; ++c) {
                    const pk_u32x4 kw = kt[lane * CPR + (c ^ (lane & 7))];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            part[r][t] = Chunk<T>::dot2(kw[t], qp[r][4 * c + t], part[r][t]);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int r = 0; r < R; ++r)
                    s[r] = (part[r][0] + part[r][1]) + (part[r][2] + part[r][3]);
            } else {
                const double (*qd)[kWide ? D : 1] = &qwide[kWide ? wave * R : 0];
#pragma unroll
                for (int r = 0; r < R; ++r) s[r] = 0;
#pragma unroll
                for (int c = 0; c < CPR; ++c) {
                    float kk[EPC];
                    Chunk<T>::unpack(kt[lane * CPR + (c ^ (lane & 7))], kk);
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int t = 0; t < EPC; ++t) {
                            if constexpr (kWide) s[r] = fma(qd[r][c * EPC + t], (double)kk[t], s[r]);
                            else s[r] = fmaf(qs[r][c * EPC + t], kk[t], s[r]);
                        }
                    // keep the chunks apart: scheduled together, all of a row's chunks are
                    // held in registers at once, beside the 128 of the output state
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            float w[R];
            bool vis[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                vis[r] = j < nvis[r];
                const state_t sj = (state_t)p.scale * s[r];
                float wi = 1.0f;
                state_t lw = 0;                             // first key: w_1 = 1
                if (has[r]) sigmoid_and_log(sj - s_prev[r] + lnw[r], wi, lw);
                if (vis[r]) { w[r] = wi; lnw[r] = lw; s_prev[r] = sj; has[r] = true; }
                else w[r] = 0.0f;                           // a masked key is not an iteration
            }
#pragma unroll
            for (int c = 0; c < CPR; ++c) {
                float vv[EPC];
                Chunk<T>::unpack(vt[lane * CPR + (c ^ (lane & 7))], vv);
#pragma unroll
                for (int r = 0; r < R; ++r)
                    if (vis[r]) {
#pragma unroll
                        for (int t = 0; t < EPC; ++t) {
                            float& acc = o[r][c * EPC + t];
                            acc = fmaf(vv[t] - acc, w[r], acc);   // o + (v - o) w
                        }
                    }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
    }
    if (i0 >= p.Lq) return;

    // fold the 64 lane states; the lower lane's keys come first
#pragma unroll
    for (int r = 0; r < R; ++r) {
        state_t lam = has[r] ? s_prev[r] - lnw[r] : (state_t)(-__builtin_inff());
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const bool upper = (lane & off) != 0;
            const state_t lam_x = __shfl_xor(lam, off, kWave);
            const state_t lam_a = upper ? lam_x : lam;
            const state_t lam_b = upper ? lam : lam_x;
            float W;
            state_t lam_n;
            merge_weight(lam_a, lam_b, W, lam_n);
#pragma unroll
            for (int t = 0; t < D; ++t) {
                const float ox = __shfl_xor(o[r][t], off, kWave);
                const float oa = upper ? ox : o[r][t];
                const float ob = upper ? o[r][t] : ox;
                o[r][t] = fmaf(ob - oa, W, oa);
            }
            lam = lam_n;
        }
        const int i = i0 + r;
        if (i >= p.Lq) continue;
        if (lane == 0) {
#pragma unroll
            for (int t = 0; t < D; ++t) qs[r][t] = o[r][t];
        }
        __builtin_amdgcn_wave_barrier();
        if (!p.partial) {
            const size_t obase = qbase + (size_t)i * D;
            for (int t = lane; t < D; t += kWave) Store<T>::store(p.o, obase + t, qs[r][t]);
        } else {
            // partial state (o, s, ln w): the run acts as one key of score lam, weight 1
            float* dst = p.ws + ((((size_t)sp * p.B + b) * p.Hq + h) * (size_t)p.Lq + i) * (D + 2);
            for (int t = lane; t < D; t += kWave) dst[t] = qs[r][t];
            if (lane == 0) split_lam(lam, dst[D], dst[D + 1]);
        }
    }
}

// Fold the split partials of each query row with the sigmoid rule, together with the state of
// earlier keys if one is given (p.state_in).  Writes the output (p.o, if not null) and the
// state (p.state_out, if not null) as the run seen as one key: (o, s = Lam, ln w = 0).
//
// One wavefront per row.  Folded one after the other, o <- o + (o_p - o) W_p with
// W_p = sigmoid(Lam_p - Lam) and Lam <- Lam_p - ln W_p, the partials end up with the weights
// e^{Lam_p - Lam_total} (the product of a partial's own W_p and the 1 - W of every later
// step), and the fold of the Lam alone does not need the o.  So: each lane takes the Lam of
// one partial (at most 64 splits), a butterfly of sigmoid merges gives every lane Lam_total
// (the rule is associative and commutative; no maximum is taken, and Lam_total >= Lam_p keeps
// every exponent at or below zero), and the output is one pass of independent loads,
// sum_p e^{Lam_p - Lam_total} o_p.  Left to right instead, a launch with 64 splits and few
// rows waits for memory 64 times in a row (43 us, against 22 us for the kernel that wrote
// the partials; a few us this way).
// state_out may be the buffer the single partial came from, or state_in: a wavefront reads
// all of its row before it writes.
template <typename T, int D, int kBatch>            // kBatch: partial rows in flight per lane
__global__ __launch_bounds__(256)
void merge_splits_kernel(Problem p) {
    constexpr int E = D / kWave;                   // output elements per lane
    using state_t = typename Chunk<T>::state_t;    // fp32 storage folds s - ln w in fp64
    const state_t ninf = (state_t)(-__builtin_inff());
    const size_t rows = (size_t)p.B * p.Hq * p.Lq;
    const int lane = threadIdx.x & (kWave - 1);
    const size_t row = (size_t)blockIdx.x * (256 / kWave) + (threadIdx.x >> 6);
    if (row >= rows) return;                       // the whole wavefront leaves together

    // the first batch of partial rows is requested before the weights are known: the loads
    // do not depend on them, and the fold of the Lam then runs while they are in flight
    float ob[kBatch][E];
    auto fetch = [&](int sp0) {
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int sp = min(sp0 + u, p.splits - 1);
            const float* src = p.ws + ((size_t)sp * rows + row) * (D + 2);
#pragma unroll
            for (int e = 0; e < E; ++e) ob[u][e] = src[lane * E + e];
        }
    };
    fetch(0);
    state_t lam_p = ninf;
    if (lane < p.splits) {
        const float* src = p.ws + ((size_t)lane * rows + row) * (D + 2);
        lam_p = (state_t)src[D] - (state_t)src[D + 1];               // s - ln w
    }
    state_t lam_in = ninf;
    float oin[E];
#pragma unroll
    for (int e = 0; e < E; ++e) oin[e] = 0.0f;
    if (p.state_in) {
        const float* sin = p.state_in + row * (D + 2);
        lam_in = (state_t)sin[D] - (state_t)sin[D + 1];
#pragma unroll
        for (int e = 0; e < E; ++e) oin[e] = sin[lane * E + e];
    }
    state_t tot = lam_p;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const state_t other = __shfl_xor(tot, off);
        const bool upper = (lane & off) != 0;      // both lanes of a pair fold (lower, upper)
        float W;
        merge_weight(upper ? other : tot, upper ? tot : other, W, tot);
    }
    {
        float W;
        merge_weight(lam_in, tot, W, tot);
    }
    const float w_p = lam_p == ninf ? 0.0f : __expf((float)(lam_p - tot));
    const float w_in = lam_in == ninf ? 0.0f : __expf((float)(lam_in - tot));

    float acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = w_in != 0.0f ? w_in * oin[e] : 0.0f;
    for (int sp0 = 0; sp0 < p.splits; sp0 += kBatch) {
        if (sp0 > 0) fetch(sp0);
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const float w = sp0 + u < p.splits ? __shfl(w_p, sp0 + u) : 0.0f;
            if (w != 0.0f) {                       // a partial of weight 0 may hold anything
#pragma unroll
                for (int e = 0; e < E; ++e) acc[e] = fmaf(w, ob[u][e], acc[e]);
            }
        }
    }
    if (p.o) {
#pragma unroll
        for (int e = 0; e < E; ++e) Store<T>::store(p.o, row * D + lane * E + e, acc[e]);
    }
    if (p.state_out) {
        float* dst = p.state_out + row * (D + 2);
#pragma unroll
        for (int e = 0; e < E; ++e) dst[lane * E + e] = acc[e];
        if (lane == 0) split_lam(tot, dst[D], dst[D + 1]);
    }
}

template <typename T, int D>
static hipError_t launch_merge_t(const Problem& p, hipStream_t st) {
    const size_t rows = (size_t)p.B * p.Hq * p.Lq;
    if ((rows + 3) / 4 > 0x7fffffffull) return hipErrorInvalidValue;
    const unsigned blocks = (unsigned)((rows + 3) / 4);
    // many splits come with few rows: more loads in flight per lane, fewer round trips
    if (p.splits > 8)
        hipLaunchKernelGGL((merge_splits_kernel<T, D, 32>), dim3(blocks), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL((merge_splits_kernel<T, D, 8>), dim3(blocks), dim3(256), 0, st, p);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_perkey_t(const Problem& p, hipStream_t st) {
    constexpr int ROWS_PER_BLOCK = PerKeyCfg<D>::R * kPerKeyWaves;
    const int row_blocks = (p.Lq + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    dim3 grid((unsigned)(row_blocks * p.splits), (unsigned)p.Hq, (unsigned)p.B);
    hipLaunchKernelGGL((perkey_kernel<T, D>), grid, dim3(kPerKeyWaves * kWave), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !p.merge) return e;
    return launch_merge_t<T, D>(p, st);
}

#define FLASHD_DISPATCH(FN, ...)                                                     \
    do {                                                                             \
        if (p.dtype == 0 && p.d == 64) return FN<F32, 64>(__VA_ARGS__);              \
        if (p.dtype == 0 && p.d == 128) return FN<F32, 128>(__VA_ARGS__);            \
        if (p.dtype == 1 && p.d == 64) return FN<F16, 64>(__VA_ARGS__);              \
        if (p.dtype == 1 && p.d == 128) return FN<F16, 128>(__VA_ARGS__);            \
        if (p.dtype == 2 && p.d == 64) return FN<BF16, 64>(__VA_ARGS__);             \
        if (p.dtype == 2 && p.d == 128) return FN<BF16, 128>(__VA_ARGS__);           \
        return hipErrorInvalidValue;                                                 \
    } while (0)

hipError_t launch_merge_splits(const Problem& p, hipStream_t st) {
    FLASHD_DISPATCH(launch_merge_t, p, st);
}

hipError_t launch_perkey(const Problem& p, hipStream_t st) {
    FLASHD_DISPATCH(launch_perkey_t, p, st);
}

}  // namespace flashd
