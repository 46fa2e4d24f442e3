// Alg. 3 lifted to key tiles on the gfx950 matrix cores (variant TILE), and the
// Alg. 2 ablation (running max, running sum, final division) on the same tiling
// (variant ONLINE_SOFTMAX).  Storage types f16 and bf16, fp32 state and accumulation.
//
// Tile form of the recurrence.  The state of Alg. 3 after a run of keys is
// (o, s_last, ln w_last); only Lam = s_last - ln w_last = ln sum_j e^{s_j} enters later
// steps (weight equation of Sec. III-B).  A tile of keys acts as one key: with
// p_j = e^{s_j - Lam} and tot = 1 + sum_j p_j,
//     1 - W = 1/tot   (W = sigmoid(S_tile - Lam) is the tile's weight),
//     o <- (1 - W) (o + sum_j p_j v_j),      Lam <- Lam + ln tot,
// which is the blend o <- (1 - W) o + W o_tile of Sec. III-A with the tile's own
// weighted value o_tile = sum_j p_j v_j / sum_j p_j.  No maximum is tracked and the
// output is never divided by a running sum.  Where a score exceeds Lam by more than
// kTheta (or Lam is still -inf: the first tile) e^{s_j - Lam} is not formed; the tile
// then runs the recurrence key by key inside each lane (sigmoid saturates instead of
// overflowing, Sec. III-C) and forms c_j = e^{s_j - Lam_new} <= 1 afterwards.
//
// Mapping.  A workgroup of 4 wavefronts owns 128 query rows of one (b, h); a
// wavefront owns 32 of them.  Keys stream through LDS in tiles of 64.  The score tile
// is produced transposed, S^T = K Q^T, by v_mfma_f32_32x32x16: lane (c, hh) =
// (lane % 32, lane / 32) then holds, for query row c, the 16 keys
// 8*(r/4) + 4*hh + r%4 (r = 0..15) of each 32-key block, so the whole per-row state
// lives in that lane and its partner lane ^ 32.  The same registers, rounded to the
// storage type, are the B operand of O^T = V^T P^T; V is transposed into LDS with the
// keys permuted to match that operand order.
#include "flashd_common.h"
#include "flashd_kernels.h"
#include "flashd_mma.h"

namespace flashd {

constexpr int kBM = 128;          // query rows per workgroup
constexpr int kBC = 64;           // keys per tile
constexpr int kTileThreads = 256;

template <typename T, int D, bool ONLINE>
__global__ __launch_bounds__(kTileThreads, 2)
void tile_kernel(Problem p) {
    constexpr int KROW = D + 8;       // padded LDS rows (elements)
    constexpr int VROW = kBC + 8;
    constexpr int NKK = D / 16;       // k-steps of the score product
    constexpr int NDB = D / 32;       // 32-wide blocks of the head dimension
    __shared__ __align__(16) uint16_t ks[kBC * KROW];
    __shared__ __align__(16) uint16_t vt[D * VROW];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31;
    const int hh = lane >> 5;

    const int m_tiles = (p.Lq + kBM - 1) / kBM;
    const int mt_raw = blockIdx.x % m_tiles;
    const int sp = blockIdx.x / m_tiles;
    const int mt = p.causal ? m_tiles - 1 - mt_raw : mt_raw;      // longest rows first
    const int h = blockIdx.y;
    const int b = blockIdx.z;
    const int kvh = h / (p.Hq / p.Hkv);
    const int m0 = mt * kBM;
    const int wrow0 = m0 + wave * 32;
    const int my_row = wrow0 + col;

    const uint16_t* qg = static_cast<const uint16_t*>(p.q) +
                         ((size_t)b * p.Hq + h) * (size_t)p.Lq * D;
    const uint16_t* kg = static_cast<const uint16_t*>(p.k) +
                         ((size_t)b * p.Hkv + kvh) * (size_t)p.Lk * D;
    const uint16_t* vg = static_cast<const uint16_t*>(p.v) +
                         ((size_t)b * p.Hkv + kvh) * (size_t)p.Lk * D;

    // Q fragments: B operand of S^T = K Q^T, kept for the whole kernel
    uint4 qf[NKK];
    {
        const int qr = min(my_row, p.Lq - 1);
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
            qf[kk] = *reinterpret_cast<const uint4*>(qg + (size_t)qr * D + 16 * kk + 8 * hh);
    }

    const int nvis = visible_count(p, my_row);
    const bool wave_live = wrow0 < p.Lq;
    const int wave_nvis_max = wave_live ? visible_count(p, min(wrow0 + 31, p.Lq - 1)) : 0;
    const int wave_nvis_min = (wrow0 + 31 < p.Lq) ? visible_count(p, wrow0) : 0;
    const int blk_nvis = visible_count(p, min(m0 + kBM - 1, p.Lq - 1));
    const int tiles_all = (p.Lk + kBC - 1) / kBC;
    const int per_split = (tiles_all + p.splits - 1) / p.splits;
    const int t_begin = sp * per_split;
    const int t_end = min((blk_nvis + kBC - 1) / kBC, t_begin + per_split);

    const float c_log2 = p.scale * kLog2e;        // scores are carried in log2 units
    const float ninf = -__builtin_inff();

    f32x16 U[NDB];
#pragma unroll
    for (int i = 0; i < NDB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) U[i][r] = 0.0f;
    float lam = ninf;      // FLASH-D: Lam in log2 units.  ONLINE: running max m.
    float beta = 1.0f;     // FLASH-D: factor still owed to U.  ONLINE: running sum l.
    if (ONLINE) beta = 0.0f;

    for (int kt = t_begin; kt < t_end; ++kt) {
        const int j0 = kt * kBC;
        __syncthreads();
        // ---- K tile: 16-byte chunks, row-major, padded rows
#pragma unroll
        for (int n = 0; n < (kBC * D / 8) / kTileThreads; ++n) {
            const int c = tid + n * kTileThreads;
            const int key = c / (D / 8);
            const int part = c % (D / 8);
            const int jr = min(j0 + key, p.Lk - 1);
            const uint4 x = *reinterpret_cast<const uint4*>(kg + (size_t)jr * D + 8 * part);
            *reinterpret_cast<uint4*>(&ks[key * KROW + 8 * part]) = x;
        }
        // ---- V tile: 4x4 blocks transposed in registers, keys permuted inside each
        // 16-key group to the operand order (group position 8*(quad%2) + 4*(quad/2))
#pragma unroll
        for (int n = 0; n < (kBC / 4) * (D / 4) / kTileThreads; ++n) {
            const int id = tid + n * kTileThreads;
            const int dq = id % (D / 4);
            const int kq = id / (D / 4);
            uint32_t lo[4], hi[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int jr = min(j0 + 4 * kq + i, p.Lk - 1);
                const uint2 x = *reinterpret_cast<const uint2*>(vg + (size_t)jr * D + 4 * dq);
                lo[i] = x.x;
                hi[i] = x.y;
            }
            const int quad = kq & 3;
            const int pos = 16 * (kq >> 2) + 8 * (quad & 1) + 4 * (quad >> 1);
            uint2 c0, c1, c2, c3;
            c0.x = __builtin_amdgcn_perm(lo[1], lo[0], 0x05040100u);
            c0.y = __builtin_amdgcn_perm(lo[3], lo[2], 0x05040100u);
            c1.x = __builtin_amdgcn_perm(lo[1], lo[0], 0x07060302u);
            c1.y = __builtin_amdgcn_perm(lo[3], lo[2], 0x07060302u);
            c2.x = __builtin_amdgcn_perm(hi[1], hi[0], 0x05040100u);
            c2.y = __builtin_amdgcn_perm(hi[3], hi[2], 0x05040100u);
            c3.x = __builtin_amdgcn_perm(hi[1], hi[0], 0x07060302u);
            c3.y = __builtin_amdgcn_perm(hi[3], hi[2], 0x07060302u);
            *reinterpret_cast<uint2*>(&vt[(4 * dq + 0) * VROW + pos]) = c0;
            *reinterpret_cast<uint2*>(&vt[(4 * dq + 1) * VROW + pos]) = c1;
            *reinterpret_cast<uint2*>(&vt[(4 * dq + 2) * VROW + pos]) = c2;
            *reinterpret_cast<uint2*>(&vt[(4 * dq + 3) * VROW + pos]) = c3;
        }
        __syncthreads();
        if (j0 >= wave_nvis_max) continue;       // nothing visible to this wavefront

        // ---- S^T = K Q^T for the two 32-key blocks
        f32x16 acc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[kb][r] = 0.0f;
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk) {
                const uint4 a = *reinterpret_cast<const uint4*>(
                    &ks[(32 * kb + col) * KROW + 16 * kk + 8 * hh]);
                acc[kb] = Mma<T>::mfma(a, qf[kk], acc[kb]);
            }
        }
        // ---- scale to log2 units; masked keys get -inf (not an iteration)
        const bool need_mask = j0 + kBC > wave_nvis_min;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float s = acc[kb][r] * c_log2;
                if (need_mask) {
                    const int j = j0 + 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
                    if (j >= nvis) s = ninf;
                }
                acc[kb][r] = s;
            }

        // ---- per-row state update; acc becomes the coefficients p_j
        const float f = row_step<T, 2, ONLINE>(acc, lam, beta);

        // ---- U <- f U + P V   (O^T = V^T P^T)
#pragma unroll
        for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) U[i][r] *= f;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            f32x8 pv;
#pragma unroll
            for (int e = 0; e < 8; ++e) pv[e] = acc[g4 >> 1][8 * (g4 & 1) + e];
            const uint4 bfrag = Mma<T>::pack8(pv);
#pragma unroll
            for (int i = 0; i < NDB; ++i) {
                const uint4 a = *reinterpret_cast<const uint4*>(
                    &vt[(32 * i + col) * VROW + 16 * g4 + 8 * hh]);
                U[i] = Mma<T>::mfma(a, bfrag, U[i]);
            }
        }
    }

    if (my_row >= p.Lq) return;
    // ---- epilogue.  FLASH-D: the output is the state (times the factor still owed);
    // ONLINE: the one division of Alg. 2.
    float fin, lam_out;
    row_finish<ONLINE>(lam, beta, fin, lam_out);
    if (p.splits == 1) {
        uint16_t* og = static_cast<uint16_t*>(p.o) +
                       (((size_t)b * p.Hq + h) * (size_t)p.Lq + my_row) * D;
#pragma unroll
        for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int dc = 32 * i + 8 * g + 4 * hh;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    Store<T>::store(og, dc + e, U[i][4 * g + e] * fin);
            }
    } else {
        // partial state (o, s, ln w) in natural-log units: the run is one key of score Lam
        float* dst = p.ws +
                     ((((size_t)sp * p.B + b) * p.Hq + h) * (size_t)p.Lq + my_row) * (D + 2);
#pragma unroll
        for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int dc = 32 * i + 8 * g + 4 * hh;
                float4 x;
                x.x = U[i][4 * g + 0] * fin; x.y = U[i][4 * g + 1] * fin;
                x.z = U[i][4 * g + 2] * fin; x.w = U[i][4 * g + 3] * fin;
                *reinterpret_cast<float4*>(dst + dc) = x;
            }
        if (hh == 0) { dst[D] = lam_out * kLn2; dst[D + 1] = 0.0f; }
    }
}

template <typename T, int D>
static hipError_t launch_tile_t(const Problem& p, bool online, hipStream_t st) {
    const int m_tiles = (p.Lq + kBM - 1) / kBM;
    dim3 grid((unsigned)(m_tiles * p.splits), (unsigned)p.Hq, (unsigned)p.B);
    if (online)
        hipLaunchKernelGGL((tile_kernel<T, D, true>), grid, dim3(kTileThreads), 0, st, p);
    else
        hipLaunchKernelGGL((tile_kernel<T, D, false>), grid, dim3(kTileThreads), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits == 1) return e;
    return launch_merge_splits(p, st);
}

long tile_workgroups(int B, int Hq, int Hkv, int Lq, int d) {
    (void)Hkv; (void)d;
    return (long)B * Hq * ((Lq + kBM - 1) / kBM);
}

hipError_t launch_tile(const Problem& p, bool online, hipStream_t st) {
    if (p.dtype == 1 && p.d == 64) return launch_tile_t<F16, 64>(p, online, st);
    if (p.dtype == 1 && p.d == 128) return launch_tile_t<F16, 128>(p, online, st);
    if (p.dtype == 2 && p.d == 64) return launch_tile_t<BF16, 64>(p, online, st);
    if (p.dtype == 2 && p.d == 128) return launch_tile_t<BF16, 128>(p, online, st);
    return hipErrorInvalidValue;
}

}  // namespace flashd
