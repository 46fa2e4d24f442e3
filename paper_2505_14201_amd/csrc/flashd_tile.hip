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
// output is not divided by a running sum of exponentials.  The product of the (1 - W)
// factors is carried as one scalar per row and multiplied in when the row is stored
// (flashd_mma.h, "lazy blend").  A score far above everything before it would overflow
// e^{s_j - Lam}; such rows redo the tile with the key-by-key sigmoid recurrence, which
// saturates instead (Sec. III-C).
//
// Mapping.  A workgroup of 4 wavefronts owns 128 query rows of one (b, h); a wavefront
// owns 32 of them.  Keys stream through LDS in tiles of 64, double-buffered: the next
// tile's global loads are issued before the current tile's math and land in LDS after
// it, one workgroup barrier per tile.  The score tile is produced transposed,
// S^T = K Q^T, by v_mfma_f32_32x32x16: lane (c, hh) = (lane % 32, lane / 32) then holds,
// for query row c, the 16 keys 8*(r/4) + 4*hh + r%4 (r = 0..15) of each 32-key block, so
// the whole per-row state lives in that lane and its partner lane ^ 32.  The same
// registers, rounded to the storage type, are the B operand of O^T = V^T P^T; V stays
// row-major in LDS and its operand comes from the transposing LDS read.  K and V tiles
// are copied global->LDS directly (no registers), with an XOR chunk swizzle instead of
// row padding.
//
// Launch order: workgroup ids run over (row tile, split, b*Hq + h) with the row tile
// slowest and, under a causal mask, longest first, so the short tiles fill the tail.
// Workgroups of one head are B*Hq*splits apart, a multiple of 8 for the usual shapes, and
// therefore land on the same XCD and share its L2 for K and V.
#include "flashd_common.h"
#include "flashd_kernels.h"
#include "flashd_mma.h"

#include <cstdlib>
#include <type_traits>

namespace flashd {

constexpr int kBC = 64;           // keys per tile

// LDS layout of one K or V tile: [64 keys][D] elements, rows unpadded (the direct
// global->LDS loads write 64 consecutive 16-byte chunks per instruction, so rows cannot
// be padded); bank conflicts are avoided by storing chunk c of row r at chunk position
// c ^ swz(r).  K is read as 16-byte operands by 16 consecutive keys at a time, V as 8-byte
// pieces of 4 consecutive keys by the transposing read; each gets the XOR pattern that
// spreads its access over all banks.
template <int D> struct TileCfg;
template <> struct TileCfg<128> {
    static constexpr int CPR = 16;                                   // chunks per row
    static __device__ __forceinline__ int swz_k(int row) { return row & 15; }
    static __device__ __forceinline__ int swz_v(int row) { return 4 * (row & 3); }
};
template <> struct TileCfg<64> {
    static constexpr int CPR = 8;
    static __device__ __forceinline__ int swz_k(int row) { return (row >> 1) & 7; }
    static __device__ __forceinline__ int swz_v(int row) { return 4 * ((row >> 1) & 1); }
};

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// Per-lane element offsets of the direct global->LDS copy.  Instruction n of a wavefront
// (n < CPR/NW, NW wavefronts) moves 64 chunks of 16 bytes into 1 KB of LDS: lane l fills
// chunk position cs = l % CPR of tile row (64/NW)*wave + n*(64/CPR) + l/CPR.  With the swizzles above the
// global chunk to fetch is cs ^ (l >> 4) ^ 4n for K and cs ^ swz_v for V (independent of
// n), so the offsets are (k0 ^ 32n) + 512n and v0 + 512n elements.
template <int D, int NW> struct DmaLane {
    int k0, v0;
    __device__ __forceinline__ DmaLane(int wave, int lane) {
        using C = TileCfg<D>;
        const int row = (kBC / NW) * wave + lane / C::CPR;     // row of this lane for n = 0
        const int cs = lane % C::CPR;
        k0 = row * D + 8 * (cs ^ C::swz_k(row));
        v0 = row * D + 8 * (cs ^ C::swz_v(row));
    }
};

// Start the copy of the K (or V) tile whose first key is j0.  A tile that sticks out past
// the last key takes the slow form with rows clamped to the last key (masked later).
template <int D, int NW>
__device__ __forceinline__ void tile_copy_k(const uint16_t* kg, int j0, int Lk,
                                            const DmaLane<D, NW>& dl, int wave, int lane,
                                            uint16_t* ks) {
    using C = TileCfg<D>;
    if (j0 + kBC <= Lk) {
        const uint16_t* kt = kg + (size_t)j0 * D;       // wavefront-uniform tile base
#pragma unroll
        for (int n = 0; n < C::CPR / NW; ++n)
            __builtin_amdgcn_global_load_lds((gptr_t)(kt + ((dl.k0 ^ (32 * n)) + 512 * n)),
                                             (lptr_t)(ks + (wave * (C::CPR / NW) + n) * 512), 16,
                                             0, 0);
    } else {
#pragma unroll 1
        for (int n = 0; n < C::CPR / NW; ++n) {
            const int inst = wave * (C::CPR / NW) + n;
            const int slot = inst * 64 + lane;
            const int row = slot / C::CPR;
            const int cs = slot % C::CPR;
            const size_t grow = (size_t)min(j0 + row, Lk - 1) * D;
            __builtin_amdgcn_global_load_lds((gptr_t)(kg + grow + 8 * (cs ^ C::swz_k(row))),
                                             (lptr_t)(ks + inst * 512), 16, 0, 0);
        }
    }
}

template <int D, int NW>
__device__ __forceinline__ void tile_copy_v(const uint16_t* vg, int j0, int Lk,
                                            const DmaLane<D, NW>& dl, int wave, int lane,
                                            uint16_t* vs) {
    using C = TileCfg<D>;
    if (j0 + kBC <= Lk) {
        const uint16_t* vt = vg + (size_t)j0 * D;
#pragma unroll
        for (int n = 0; n < C::CPR / NW; ++n)
            __builtin_amdgcn_global_load_lds((gptr_t)(vt + (dl.v0 + 512 * n)),
                                             (lptr_t)(vs + (wave * (C::CPR / NW) + n) * 512), 16,
                                             0, 0);
    } else {
#pragma unroll 1
        for (int n = 0; n < C::CPR / NW; ++n) {
            const int inst = wave * (C::CPR / NW) + n;
            const int slot = inst * 64 + lane;
            const int row = slot / C::CPR;
            const int cs = slot % C::CPR;
            const size_t grow = (size_t)min(j0 + row, Lk - 1) * D;
            __builtin_amdgcn_global_load_lds((gptr_t)(vg + grow + 8 * (cs ^ C::swz_v(row))),
                                             (lptr_t)(vs + inst * 512), 16, 0, 0);
        }
    }
}

// 8 keys x 1 column of V as an MFMA operand through the transposing LDS read (see
// flashd_mma.h for the lane roles); vaddr = this lane's element offset for the d-block,
// key0 = first key of the 16-key group.
template <int D>
__device__ __forceinline__ u32x4 tile_v_operand(const uint16_t* vs, int vaddr, int key0) {
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(vs + vaddr + key0 * D));
    const s16x4 hi =
        __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(vs + vaddr + (key0 + 8) * D));
    const u32x2 l2 = __builtin_bit_cast(u32x2, lo);
    const u32x2 h2 = __builtin_bit_cast(u32x2, hi);
    return u32x4{l2[0], l2[1], h2[0], h2[1]};
}

// State that stays in registers for the life of a workgroup's row tile.
template <int D> struct TileRegs {
    u32x4 qf[D / 16];
    int kaddr[D / 16];
    int vaddr[D / 32];
    f32x16 U[D / 32];
    LazyRow st;             // FLASH-D state
    float lam, beta;        // Alg. 2 state: running max m, running sum l
};

constexpr int kAhead = 8;         // operand reads in flight ahead of the matrix instructions

// Phase 1 of a tile: raw scores S^T = K Q^T (two 32-key blocks, chains interleaved).
// Operand reads run kAhead products ahead of the matrix instructions that consume them
// (LDS returns in order).
template <typename T, int D>
__device__ __forceinline__ void phase_scores(const uint16_t* ks, const TileRegs<D>& g,
                                             f32x16 (&acc)[2]) {
    constexpr int NK = 2 * (D / 16);      // K operands / score products per tile
    u32x4 ka[NK];
#pragma unroll
    for (int m = 0; m < kAhead; ++m)
        ka[m] = *reinterpret_cast<const u32x4*>(&ks[g.kaddr[m >> 1] + 32 * D * (m & 1)]);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[kb][r] = 0.0f;
#pragma unroll
    for (int m = 0; m < NK; ++m) {
        acc[m & 1] = Mma<T>::mfma(ka[m], g.qf[m >> 1], acc[m & 1]);
        if (m + kAhead < NK)
            ka[m + kAhead] = *reinterpret_cast<const u32x4*>(
                &ks[g.kaddr[(m + kAhead) >> 1] + 32 * D * ((m + kAhead) & 1)]);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
    for (int m = 0; m < NK - kAhead; ++m) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, kAhead, 0);
    __builtin_amdgcn_sched_barrier(0);
}

// Phase 2: coefficients of the tile from its raw scores (per-row state update) and, where
// the variant needs it, the scaling of U.  The raw scores are left untouched.
template <typename T, int D, bool ONLINE>
__device__ __forceinline__ void phase_coeffs(const f32x16 (&acc)[2], u32x4 (&bfrag)[4],
                                             TileRegs<D>& g, int j0, int hh, int lane, int nvis,
                                             bool need_mask, float c_log2) {
    constexpr int NDB = D / 32;
    const int jb = j0 + 4 * hh;
    if (!ONLINE) {
        bool risky;
        if (need_mask)
            risky = lazy_spec_pack<T, 2, true, true>(acc, bfrag, g.st, c_log2, jb, nvis, lane);
        else
            risky = lazy_spec_pack<T, 2, false, true>(acc, bfrag, g.st, c_log2, jb, nvis, lane);
        if (__builtin_amdgcn_ballot_w64(risky) != 0) {
            // rare: flagged rows redo the tile with the key-by-key sigmoid recurrence
            const float f =
                lazy_redo_pack<T, 2>(acc, bfrag, g.st, risky, c_log2, need_mask, jb, nvis);
#pragma unroll
            for (int i = 0; i < NDB; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) g.U[i][r] *= f;
        }
    } else {
        float f;
        if (need_mask) f = online_pack<T, 2, true>(acc, bfrag, g.lam, g.beta, c_log2, jb, nvis);
        else f = online_pack<T, 2, false>(acc, bfrag, g.lam, g.beta, c_log2, jb, nvis);
#pragma unroll
        for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) g.U[i][r] *= f;
    }
}

// Phase 3: U <- U + P V   (O^T = V^T P^T)
template <typename T, int D>
__device__ __forceinline__ void phase_output(const uint16_t* vs, TileRegs<D>& g,
                                             const u32x4 (&bfrag)[4]) {
    constexpr int NDB = D / 32;
    constexpr int NV = 4 * NDB;           // V operands / output products per tile
    u32x4 va[NV];
#pragma unroll
    for (int m = 0; m < kAhead; ++m)
        va[m] = tile_v_operand<D>(vs, g.vaddr[m % NDB], 16 * (m / NDB));
#pragma unroll
    for (int m = 0; m < NV; ++m) {
        g.U[m % NDB] = Mma<T>::mfma(va[m], bfrag[m / NDB], g.U[m % NDB]);
        if (m + kAhead < NV)
            va[m + kAhead] =
                tile_v_operand<D>(vs, g.vaddr[(m + kAhead) % NDB], 16 * ((m + kAhead) / NDB));
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAhead, 0);
    if (NV > kAhead) {
#pragma unroll
        for (int m = 0; m < NV - kAhead; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
    }
    __builtin_amdgcn_sched_group_barrier(0x008, kAhead, 0);
    __builtin_amdgcn_sched_barrier(0);
}

// NW wavefronts of 32 query rows each per workgroup, two wavefronts per SIMD either way.
//   NW = 4: two workgroups per compute unit; K and V tiles double-buffered, the copies of
//           tile t+1 run during the math of tile t.
//   NW = 8: one workgroup per compute unit (half the K/V traffic into LDS per unit of
//           work); three buffers each, the copies run two tiles ahead.
template <typename T, int D, bool ONLINE, int NW>
__global__ __launch_bounds__(NW * 64, 8 / NW)
void tile_kernel(Problem p) {
    using C = TileCfg<D>;
    constexpr int NBUF = NW == 8 ? 3 : 2;     // buffers per tensor
    constexpr int AHEAD = NBUF - 1;           // tiles the copies run ahead of the math
    constexpr int NCP = 2 * (C::CPR / NW);    // copy instructions per wavefront and tile
    constexpr int kBM = 32 * NW;      // query rows per workgroup
    constexpr int NKK = D / 16;       // k-steps of the score product
    constexpr int NDB = D / 32;       // 32-wide blocks of the head dimension
    constexpr int kTile = kBC * D;    // elements of one K or V tile
    // tile t lives in buffer t % NBUF of its tensor
    __shared__ __align__(1024) uint16_t lds[2 * NBUF * kTile];
    uint16_t* const kbuf = lds;
    uint16_t* const vbuf = lds + NBUF * kTile;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wavefront-uniform
    const int col = lane & 31;
    const int hh = lane >> 5;

    // workgroup id -> (row tile, split, b, h); the row tile is the slowest index
    const int m_tiles = (p.Lq + kBM - 1) / kBM;
    const int n_bh = p.B * p.Hq;
    const int per_rank = n_bh * p.splits;
    const int mt_rank = blockIdx.x / per_rank;
    const int rem = blockIdx.x % per_rank;
    const int sp = rem / n_bh;
    const int bh = rem % n_bh;
    const int b = bh / p.Hq;
    const int h = bh % p.Hq;
    const int mt = p.causal ? m_tiles - 1 - mt_rank : mt_rank;     // longest rows first
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

    const int nvis = visible_count(p, my_row);
    const bool wave_live = wrow0 < p.Lq;
    const int wave_nvis_max = wave_live ? visible_count(p, min(wrow0 + 31, p.Lq - 1)) : 0;
    const int wave_nvis_min = (wrow0 + 31 < p.Lq) ? visible_count(p, wrow0) : 0;
    const int blk_nvis = visible_count(p, min(m0 + kBM - 1, p.Lq - 1));
    const int tiles_all = (p.Lk + kBC - 1) / kBC;
    const int per_split = (tiles_all + p.splits - 1) / p.splits;
    const int t_begin = sp * per_split;
    const int t_end = min((blk_nvis + kBC - 1) / kBC, t_begin + per_split);
    const int n = max(t_end - t_begin, 0);          // tiles of this workgroup
    const int jbase = t_begin * kBC;                // first key of tile 0

    // prologue copies: the first AHEAD tiles
    const DmaLane<D, NW> dl(wave, lane);
#pragma unroll
    for (int t = 0; t < AHEAD; ++t)
        if (t < n) {
            tile_copy_k<D, NW>(kg, jbase + t * kBC, p.Lk, dl, wave, lane, kbuf + t * kTile);
            tile_copy_v<D, NW>(vg, jbase + t * kBC, p.Lk, dl, wave, lane, vbuf + t * kTile);
        }

    TileRegs<D> g;
    {
        // Q fragments: B operand of S^T = K Q^T, kept for the whole kernel
        const int qr = min(my_row, p.Lq - 1);
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
            g.qf[kk] = *reinterpret_cast<const u32x4*>(qg + (size_t)qr * D + 16 * kk + 8 * hh);
        // operand addresses inside a tile (elements)
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
            g.kaddr[kk] = col * D + 8 * ((2 * kk + hh) ^ C::swz_k(col));
        const int t = lane & 15;
        const int tq = t >> 2;
        const int half = (lane >> 4) & 1;
#pragma unroll
        for (int i = 0; i < NDB; ++i)
            g.vaddr[i] = (4 * hh + tq) * D +
                         8 * ((4 * i + 2 * half + ((t & 3) >> 1)) ^ C::swz_v(tq)) + 4 * (t & 1);
#pragma unroll
        for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) g.U[i][r] = 0.0f;
        g.st = {0.0f, 1.0f, 0.0f};
        g.lam = -__builtin_inff();
        g.beta = 0.0f;
    }

    const float c_log2 = p.scale * kLog2e;        // scores are carried in log2 units
    const float ninf = -__builtin_inff();

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // Period t: start the copies of tile t + AHEAD (its buffers were last read in period
    // t - 1), do the math of tile t, wait until tile t + 1 has landed (the copies started
    // in this period may stay in flight when AHEAD = 2), barrier.
    for (int t = 0; t < n; ++t) {
        const int j0 = jbase + t * kBC;
        const int ta = t + AHEAD;
        if (ta < n) {
            tile_copy_k<D, NW>(kg, jbase + ta * kBC, p.Lk, dl, wave, lane,
                               kbuf + (ta % NBUF) * kTile);
            tile_copy_v<D, NW>(vg, jbase + ta * kBC, p.Lk, dl, wave, lane,
                               vbuf + (ta % NBUF) * kTile);
        }
        if (j0 < wave_nvis_max) {
            f32x16 acc[2];
            u32x4 bfrag[4];
            phase_scores<T, D>(kbuf + (t % NBUF) * kTile, g, acc);
            phase_coeffs<T, D, ONLINE>(acc, bfrag, g, j0, hh, lane, nvis,
                                       j0 + kBC > wave_nvis_min, c_log2);
            phase_output<T, D>(vbuf + (t % NBUF) * kTile, g, bfrag);
        }
        if (AHEAD == 2 && ta < n) {
            if constexpr (NCP == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else if constexpr (NCP == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        __syncthreads();
    }

    // ---- epilogue.  FLASH-D: the output is the state, o = beta U; Alg. 2: one division.
    float fin, lam_out;
    if (!ONLINE) {
        fin = g.st.beta;
        lam_out = g.st.one == 0.0f ? ninf : g.st.R - log2_fast(g.st.beta);
    } else {
        row_finish<true>(g.lam, g.beta, fin, lam_out);
    }
    if (p.splits == 1) {
        // Stage the wavefront's 32 x D output block through LDS (the tile buffers are idle
        // after the last barrier; each wavefront uses its own 32 * D elements) so that the
        // global stores are 16 bytes per lane and whole rows are contiguous.  Chunk c of
        // row r sits at chunk position c ^ (r % CPR) to keep the 8-byte writes and the
        // 16-byte reads off each other's banks.
        uint16_t* stage = lds + wave * (32 * D);
#pragma unroll
        for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int dc = 32 * i + 8 * gq + 4 * hh;            // 4 consecutive columns
                uint16_t h4[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if constexpr (std::is_same<T, BF16>::value)
                        h4[e] = f32_to_bf16(g.U[i][4 * gq + e] * fin);
                    else
                        h4[e] = __builtin_bit_cast(uint16_t,
                                                   static_cast<_Float16>(g.U[i][4 * gq + e] * fin));
                }
                const int chunk = (dc >> 3) ^ (col % C::CPR);
                u32x2 w2;
                w2[0] = (uint32_t)h4[0] | ((uint32_t)h4[1] << 16);
                w2[1] = (uint32_t)h4[2] | ((uint32_t)h4[3] << 16);
                *reinterpret_cast<u32x2*>(&stage[col * D + 8 * chunk + (dc & 4)]) = w2;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint16_t* og = static_cast<uint16_t*>(p.o) + ((size_t)b * p.Hq + h) * (size_t)p.Lq * D;
#pragma unroll
        for (int n = 0; n < 32 * C::CPR / 64; ++n) {
            const int slot = n * 64 + lane;
            const int r = slot / C::CPR;
            const int c = slot % C::CPR;
            const u32x4 x =
                *reinterpret_cast<const u32x4*>(&stage[r * D + 8 * (c ^ (r % C::CPR))]);
            if (wrow0 + r < p.Lq)
                *reinterpret_cast<u32x4*>(og + (size_t)(wrow0 + r) * D + 8 * c) = x;
        }
    } else if (my_row < p.Lq) {
        // partial state (o, s, ln w) in natural-log units: the run is one key of score Lam
        float* dst = p.ws +
                     ((((size_t)sp * p.B + b) * p.Hq + h) * (size_t)p.Lq + my_row) * (D + 2);
#pragma unroll
        for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int dc = 32 * i + 8 * gq + 4 * hh;
                float4 x;
                x.x = g.U[i][4 * gq + 0] * fin; x.y = g.U[i][4 * gq + 1] * fin;
                x.z = g.U[i][4 * gq + 2] * fin; x.w = g.U[i][4 * gq + 3] * fin;
                *reinterpret_cast<float4*>(dst + dc) = x;
            }
        if (hh == 0) { dst[D] = lam_out * kLn2; dst[D + 1] = 0.0f; }
    }
}

template <typename T, int D, int NW>
static hipError_t launch_tile_nw(const Problem& p, bool online, hipStream_t st) {
    const long m_tiles = (p.Lq + 32 * NW - 1) / (32 * NW);
    const long total = m_tiles * p.splits * p.B * p.Hq;
    if (total > 0x7fffffffL) return hipErrorInvalidValue;
    dim3 grid((unsigned)total);
    if (online)
        hipLaunchKernelGGL((tile_kernel<T, D, true, NW>), grid, dim3(NW * 64), 0, st, p);
    else
        hipLaunchKernelGGL((tile_kernel<T, D, false, NW>), grid, dim3(NW * 64), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits == 1) return e;
    return launch_merge_splits(p, st);
}

// Rows per workgroup: 256 (8 wavefronts) halves the K/V traffic into LDS per unit of work
// and pays off once there are enough 256-row tiles to fill the chip; 128 otherwise.
static int tile_rows(int B, int Hq, int Lq) {
    static const int forced = [] {
        const char* e = getenv("FLASHD_TILE_ROWS");
        return e ? atoi(e) : 0;
    }();
    if (forced == 128 || forced == 256) return forced;
    return 128;
}

template <typename T, int D>
static hipError_t launch_tile_t(const Problem& p, bool online, hipStream_t st) {
    if (tile_rows(p.B, p.Hq, p.Lq) == 256) return launch_tile_nw<T, D, 8>(p, online, st);
    return launch_tile_nw<T, D, 4>(p, online, st);
}

long tile_workgroups(int B, int Hq, int Hkv, int Lq, int d) {
    (void)Hkv; (void)d;
    const int rows = tile_rows(B, Hq, Lq);
    return (long)B * Hq * ((Lq + rows - 1) / rows);
}

hipError_t launch_tile(const Problem& p, bool online, hipStream_t st) {
    if (p.dtype == 1 && p.d == 64) return launch_tile_t<F16, 64>(p, online, st);
    if (p.dtype == 1 && p.d == 128) return launch_tile_t<F16, 128>(p, online, st);
    if (p.dtype == 2 && p.d == 64) return launch_tile_t<BF16, 64>(p, online, st);
    if (p.dtype == 2 && p.d == 128) return launch_tile_t<BF16, 128>(p, online, st);
    return hipErrorInvalidValue;
}

}  // namespace flashd
