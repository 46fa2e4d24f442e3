// Alg. 3 lifted to key tiles on the gfx950 matrix cores (variants TILE and TILE_BLEND), and
// the Alg. 2 ablation (running max, running sum, final division) on the same tiling
// (variant ONLINE_SOFTMAX).  Storage types f16 and bf16, fp32 state and accumulation.
//
// Tile form of the recurrence.  The state of Alg. 3 after a run of keys is
// (o, s_last, ln w_last); only Lam = s_last - ln w_last = ln sum_j e^{s_j} enters later
// steps (weight equation of Sec. III-B).  A tile of keys acts as one key: with
// p_j = e^{s_j - Lam} and tot = 1 + sum_j p_j,
//     1 - W = 1/tot   (W = sigmoid(S_tile - Lam) is the tile's weight),
//     o <- (1 - W) (o + sum_j p_j v_j),      Lam <- Lam + ln tot,
// which is the blend o <- (1 - W) o + W o_tile of Sec. III-A with the tile's own
// weighted value o_tile = sum_j p_j v_j / sum_j p_j.
//   TILE_BLEND applies exactly that on every tile: U holds o, is scaled by (1 - W) per tile,
// and the coefficients are the final weights c_j = e^{s_j - Lam_new} <= 1 (blend_pack).
//   TILE, the default, defers the scaling: the product of the (1 - W) factors is carried as
// one scalar beta per row and multiplied in when the row is stored, and the coefficients are
// taken against a reference R that only moves when it has to (flashd_mma.h, "lazy blend").
// In that form 1/beta IS a sum of exponentials 2^{s_j - R} over the keys seen so far and
// o = beta U at the store is the normalisation by it: what TILE does without, compared with
// Alg. 2, is the running maximum and the per-tile rescaling of the accumulator, not the sum.
// A score far above everything before it would overflow e^{s_j - R}; the row's reference then
// moves to that score, which is the saturation of the sigmoid at 1 (Sec. III-C) in tile form.
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
// Work hand-out: see TileSched below (virtual workgroups, causal row tiles paired long
// with short, workgroups of a head kept on one XCD so that its K and V stay in that L2).
#include "flashd_common.h"
#include "flashd_kernels.h"
#include "flashd_mma.h"
#include "flashd_tile_parts.h"

#include <algorithm>
#include <type_traits>

namespace flashd {

// State that stays in registers for the life of a workgroup's row tile.
template <int D> struct TileRegs {
    u32x4 qf[D / 16];
    int kaddr[D / 16];
    int vaddr[D / 32];
    f32x16 U[D / 32];
    LazyRow st;             // FLASH-D state, lazy form
    BlendRow bl;            // FLASH-D state, literal per-tile blend
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
// the variant needs it, the scaling of U.  general = false promises that every key of the
// tile is visible to every row of the wavefront and that no row is still empty (not the
// first tile of a row); the common code path then carries neither the mask nor the
// first-key logic.  wary (wavefront-uniform): see lazy_spec_pack.
template <typename T, int D, int MODE, bool TL>
__device__ __forceinline__ void phase_coeffs(const uint16_t* ks, const f32x16 (&acc)[2],
                                             u32x4 (&bfrag)[4], TileRegs<D>& g, int j0, int hh,
                                             int lane, int nvis, bool general, float c_log2,
                                             Wary& wary) {
    constexpr int NDB = D / 32;
    const int jb = j0 + 4 * hh;
    auto scale_u = [&](float f) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) g.U[i][r] *= f;
    };
    if (MODE == kModeLazy) {
        bool risky;
        LazySpec spec;
        if (general)
            risky = lazy_spec_pack<T, 2, true, true, TL>(acc, bfrag, g.st, c_log2, jb, nvis, lane,
                                                         spec, wary);
        else
            risky = lazy_spec_pack<T, 2, false, false, TL>(acc, bfrag, g.st, c_log2, jb, nvis,
                                                           lane, spec, wary);
        if (spec.any_moved) scale_u(spec.fu);
        if (!spec.checked && __builtin_amdgcn_ballot_w64(risky) != 0) {
            // rare: a flagged row's coefficients do not fit the storage type.  bf16 with a
            // sum that is still a number: the reference moves up by a power of two and the
            // coefficients are scaled as they are.  Else the checked step on the raw scores,
            // which are formed again (K is still in LDS) rather than kept: holding them until
            // here would cost the common path 32 registers.  The wavefront then looks before
            // it exponentiates for a while (wary).
            const bool lost = risky && !(spec.psum <= kLazyShiftMax);
            const bool any_lost = __builtin_amdgcn_ballot_w64(lost) != 0;
            float f;
            if (std::is_same<T, BF16>::value && !any_lost) {
                f = lazy_shift_inplace_bf16<TL>(bfrag, 4, g.st, risky, spec);
            } else {
                f32x16 acc2[2];
                phase_scores<T, D>(ks, g, acc2);
                bool moved;
                if (general)
                    f = lazy_checked_pack<T, 2, true, TL>(acc2, bfrag, g.st, risky, c_log2, jb,
                                                          nvis, moved);
                else
                    f = lazy_checked_pack<T, 2, false, TL>(acc2, bfrag, g.st, risky, c_log2, jb,
                                                           nvis, moved);
                wary.failed();
            }
            scale_u(f);
        }
    } else if (MODE == kModeOnline) {
        float f;
        if (general) f = online_pack<T, 2, true>(acc, bfrag, g.lam, g.beta, c_log2, jb, nvis);
        else f = online_pack<T, 2, false>(acc, bfrag, g.lam, g.beta, c_log2, jb, nvis);
        // the accumulator is rescaled only when some row's maximum has moved
        if (__builtin_amdgcn_ballot_w64(f != 1.0f) != 0) scale_u(f);
    } else {
        float f;
        if (general) f = blend_pack<T, 2, true>(acc, bfrag, g.bl, c_log2, jb, nvis);
        else f = blend_pack<T, 2, false>(acc, bfrag, g.bl, c_log2, jb, nvis);
        scale_u(f);                      // o <- (1 - W) o, every tile
    }
}

// The first kAhead V operands of phase 3, requested before phase 2 so that they arrive
// while the coefficients are computed.
template <int D>
__device__ __forceinline__ void prefetch_v(const uint16_t* vs, const TileRegs<D>& g,
                                           u32x4 (&va)[kAhead]) {
    constexpr int NDB = D / 32;
#pragma unroll
    for (int m = 0; m < kAhead; ++m)
        va[m] = tile_v_operand<D>(vs, g.vaddr[m % NDB], 16 * (m / NDB));
    __builtin_amdgcn_sched_barrier(0);
}

// Phase 3: U <- U + P V   (O^T = V^T P^T); va0 = the operands prefetch_v() asked for.
template <typename T, int D>
__device__ __forceinline__ void phase_output(const uint16_t* vs, TileRegs<D>& g,
                                             const u32x4 (&bfrag)[4],
                                             const u32x4 (&va0)[kAhead]) {
    constexpr int NDB = D / 32;
    constexpr int NV = 4 * NDB;           // V operands / output products per tile
    static_assert(NV >= kAhead, "operand prefetch deeper than the phase");
    u32x4 va[NV];
#pragma unroll
    for (int m = 0; m < kAhead; ++m) va[m] = va0[m];
#pragma unroll
    for (int m = 0; m < NV; ++m) {
        g.U[m % NDB] = Mma<T>::mfma(va[m], bfrag[m / NDB], g.U[m % NDB]);
        if (m + kAhead < NV)
            va[m + kAhead] =
                tile_v_operand<D>(vs, g.vaddr[(m + kAhead) % NDB], 16 * ((m + kAhead) / NDB));
    }
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

// The three phases of one tile, with the LDS slot (PAR) a compile-time constant so that
// every operand address is a register plus an immediate.  general: keys may be masked or
// rows may still be empty.
template <typename T, int D, int MODE, bool TL, int PAR>
__device__ __forceinline__ void tile_math(const uint16_t* lds, TileRegs<D>& g, int j0, int hh,
                                          int lane, int nvis, bool general, float c_log2,
                                          Wary& wary) {
    constexpr int kTile = kBC * D;
    f32x16 acc[2];
    u32x4 bfrag[4];
    // D = 128: the first V operands are requested before phase 2.  D = 64 asks for them at
    // the start of phase 3 instead: the registers that early requests hold would cost it
    // the third resident workgroup per compute unit.
    constexpr bool kEarlyV = D == 128;
    u32x4 va0[kAhead];
    phase_scores<T, D>(lds + PAR * kTile, g, acc);
    // The copies of the next tile have landed by now as a rule; waiting for them here rather
    // than at the end of the period costs no time and keeps the workgroups that share a
    // head's K and V closer in step, which the L2 rewards: 271 MB instead of 350 MB fetched
    // from memory per launch of the headline workload.
    wait_copies();
    if (kEarlyV) prefetch_v<D>(lds + (2 + PAR) * kTile, g, va0);
    phase_coeffs<T, D, MODE, TL>(lds + PAR * kTile, acc, bfrag, g, j0, hh, lane, nvis,
                                          general, c_log2, wary);
    if (!kEarlyV) prefetch_v<D>(lds + (2 + PAR) * kTile, g, va0);
    phase_output<T, D>(lds + (2 + PAR) * kTile, g, bfrag, va0);
}

// 4 wavefronts of 32 query rows each per workgroup, two workgroups per compute unit.  K and
// V tiles are double-buffered in LDS ([K0 K1 V0 V1]); the copies of tile t+1 run during
// the math of tile t, one barrier per tile.  A workgroup may own two row tiles (a long and a
// short one under a causal mask, so that all workgroups carry the same work); the copy
// pipeline runs on across the change of row tile.
// TL: the state is handed out (partial states, state_out) and the coefficient sums are those
// of the rounded coefficients: also carry the unrounded sum, so that the Lam handed out is the
// true log-sum-exp.
template <typename T, int D, int MODE, bool TL>
__global__ __launch_bounds__(kNW * 64, 2)
void tile_kernel(Problem p, TileSched sc) {
    constexpr bool kTL = TL && Mma<T>::kRoundedSum && MODE == kModeLazy;
    using C = TileCfg<D>;
    constexpr int NKK = D / 16;       // k-steps of the score product
    constexpr int NDB = D / 32;       // 32-wide blocks of the head dimension
    constexpr int kTile = kBC * D;    // elements of one K or V tile
    __shared__ __align__(1024) uint16_t lds[4 * kTile];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wavefront-uniform
    const int col = lane & 31;
    const int hh = lane >> 5;

    const DmaLane<D> dl(wave, lane);
    int seq = 0;
    Item cur = next_item<D>(p, sc, seq, wave);
    if (!cur.valid) return;
    int nvis = visible_count(p, cur.wrow0 + col);      // keys visible to the lane's row
    bool have0 = false;          // tile 0 of the current item is in flight or has landed
    if (cur.n > 0) {
        tile_copy<D>(cur.kg, cur.vg, cur.jbase, p.Lk, dl, wave, lane, lds, lds + 2 * kTile);
        have0 = true;
    }

    TileRegs<D> g;
    {
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
        // Q fragments: B operand of S^T = K Q^T, kept for the whole row tile
        const int qr = min(cur.wrow0 + col, p.Lq - 1);
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
            g.qf[kk] =
                *reinterpret_cast<const u32x4*>(cur.qg + (size_t)qr * D + 16 * kk + 8 * hh);
    }

    const float c_log2 = p.scale * kLog2e;        // scores are carried in log2 units
    const float ninf = -__builtin_inff();
    Wary wary = {0, kWaryTiles};      // wavefront-uniform, see lazy_spec_pack

    for (bool first = true; cur.valid; first = false) {
        ++seq;
        const Item nxt = next_item<D>(p, sc, seq, wave);
#pragma unroll
        for (int i = 0; i < NDB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) g.U[i][r] = 0.0f;
        g.st = {0.0f, 1.0f, 0.0f, 0.0f};
        g.bl = {0.0f, 0.0f};
        g.lam = ninf;
        g.beta = 0.0f;
        if (MODE == kModeLazy && p.from_state) {
            // continue from the state of earlier keys: o = U with beta = 1, R = Lam
            const int row = min(cur.wrow0 + col, p.Lq - 1);
            const float* src = p.state_in +
                               ((size_t)cur.bh * (size_t)p.Lq + row) * (D + 2);
            const float lam_in = src[D] - src[D + 1];            // s - ln w, natural log
            if (cur.wrow0 + col < p.Lq && lam_in != ninf) {
#pragma unroll
                for (int i = 0; i < NDB; ++i)
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        const float4 x =
                            *reinterpret_cast<const float4*>(src + 32 * i + 8 * gq + 4 * hh);
                        g.U[i][4 * gq + 0] = x.x; g.U[i][4 * gq + 1] = x.y;
                        g.U[i][4 * gq + 2] = x.z; g.U[i][4 * gq + 3] = x.w;
                    }
                g.st = {lam_in * kLog2e, 1.0f, 1.0f, 1.0f};
            }
            // Have the state here before going on: left pending, these loads make the
            // compiler put a full wait in front of the epilogue's first use of U (a row tile
            // without key tiles gets there with no matrix instruction in between), and that
            // wait then also covers the Q fragments requested for the next row tile.
            wait_copies();
        }

        if (!have0 && cur.n > 0)
            tile_copy<D>(cur.kg, cur.vg, cur.jbase, p.Lk, dl, wave, lane, lds, lds + 2 * kTile);
        if (first || !have0) {
            wait_copies();
            __syncthreads();
        }
        have0 = false;

        // Period t: start the copies of the next tile into the other slot, which was last
        // read in period t - 1; do the math of tile t; wait for the copies; barrier.  Tile t
        // of a row tile lives in slot t % 2, and the loop body is two periods, one per slot,
        // so that each is compiled once with constant LDS addresses.  Tile 0 of the next
        // row tile is copied during this row tile's last period if that leaves slot 0 free
        // (an even number of tiles), else after it.
        auto period = [&](auto slot, int t) __attribute__((always_inline)) {
            constexpr int PAR = decltype(slot)::value;
            const int j0 = cur.jbase + t * kBC;
            uint16_t* kdst = lds + (PAR ^ 1) * kTile;
            if (t + 1 < cur.n) {
                if (sc.once)
                    tile_copy<D, true>(cur.kg, cur.vg, j0 + kBC, p.Lk, dl, wave, lane, kdst,
                                       kdst + 2 * kTile);
                else
                    tile_copy<D>(cur.kg, cur.vg, j0 + kBC, p.Lk, dl, wave, lane, kdst,
                                 kdst + 2 * kTile);
            } else if (PAR == 1 && nxt.n > 0) {
                tile_copy<D>(nxt.kg, nxt.vg, nxt.jbase, p.Lk, dl, wave, lane, kdst,
                             kdst + 2 * kTile);
                have0 = true;
            }
            if (j0 < cur.wmax)
                tile_math<T, D, MODE, TL, PAR>(lds, g, j0, hh, lane, nvis,
                                               t == 0 || j0 + kBC > cur.wmin, c_log2, wary);
            wait_copies();
            __syncthreads();
        };
        for (int t = 0; t < cur.n; t += 2) {
            period(IntC<0>{}, t);
            if (t + 1 < cur.n) period(IntC<1>{}, t + 1);
        }

        // The next row tile's Q fragments: requested now, needed after the epilogue.
        if (nxt.valid) {
            const int qr = min(nxt.wrow0 + col, p.Lq - 1);
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk)
                g.qf[kk] = *reinterpret_cast<const u32x4*>(nxt.qg + (size_t)qr * D + 16 * kk +
                                                           8 * hh);
        }

        // ---- epilogue.  FLASH-D: the output is the state, o = beta U; Alg. 2: one division.
        float fin, lam_out;
        if (MODE == kModeLazy) {
            fin = g.st.beta;
            lam_out = g.st.one == 0.0f ? ninf
                      : kTL ? g.st.R + log2_fast(g.st.ltrue) : g.st.R - log2_fast(g.st.beta);
        } else if (MODE == kModeBlend) {
            fin = 1.0f;                  // U is the output
            lam_out = g.bl.one == 0.0f ? ninf : g.bl.lam;
        } else {
            row_finish<true>(g.lam, g.beta, fin, lam_out);
        }
        // The epilogue's lane arithmetic is kept inside the loop over row tiles (the empty asm
        // hides that it is invariant): hoisted, its addresses would occupy registers during
        // the tile loop.
        int elane = lane;
        asm volatile("" : "+v"(elane));
        const int col = elane & 31;
        const int hh = elane >> 5;
        fin *= p.oscale;
        if (p.store_o) {
            // Stage the wavefront's 32 x D output block through LDS so that the global
            // stores are 16 bytes per lane and whole rows are contiguous.  Slot 1 is idle
            // after the last barrier and never the target of the copy of the next row
            // tile's first tile; the wavefront uses exactly the parts of it that its own
            // copies fill (its 16 rows of the K tile for output rows 0..15, of the V tile
            // for rows 16..31), so no other wavefront's copies or reads can touch them and
            // no barrier is needed.  Chunk c of row r sits at chunk position c ^ (r % CPR)
            // to keep the 8-byte writes and the 16-byte reads off each other's banks.
            uint16_t* stage_k = lds + kTile + wave * (16 * D);
            uint16_t* stage = col < 16 ? stage_k : stage_k + 2 * kTile;
            const int srow = col & 15;
#pragma unroll
            for (int i = 0; i < NDB; ++i)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int dc = 32 * i + 8 * gq + 4 * hh;            // 4 consecutive columns
                    f32x4 x4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x4[e] = g.U[i][4 * gq + e] * fin;
                    const u32x2 w2 = Mma<T>::pack4(x4);     // round to nearest even
                    const int chunk = (dc >> 3) ^ (col % C::CPR);
                    *reinterpret_cast<u32x2*>(&stage[srow * D + 8 * chunk + (dc & 4)]) = w2;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // all reads of the staged block first, then the stores: one read-wait-store
            // chain per row group leaves the wavefront waiting on LDS eight times in a row
            constexpr int NST = 32 * C::CPR / 64;
            u32x4 xs[NST];
#pragma unroll
            for (int n = 0; n < NST; ++n) {
                const int slot = n * 64 + elane;
                const int r = slot / C::CPR;                // output row within the wavefront
                const int c = slot % C::CPR;
                const uint16_t* src = (r < 16 ? stage_k : stage_k + 2 * kTile) +
                                      (r & 15) * D + 8 * (c ^ (r % C::CPR));
                xs[n] = *reinterpret_cast<const u32x4*>(src);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int n = 0; n < NST; ++n) {
                const int slot = n * 64 + elane;
                const int r = slot / C::CPR;
                const int c = slot % C::CPR;
                // written once and not read again by this launch: streaming stores
                if (cur.wrow0 + r < p.Lq)
                    __builtin_nontemporal_store(
                        xs[n],
                        reinterpret_cast<u32x4*>(cur.og + (size_t)(cur.wrow0 + r) * D + 8 * c));
            }
        }
        if (p.partial && cur.wrow0 + col < p.Lq) {
            // partial state (o, s, ln w) in natural-log units: the run is one key of score Lam
            float* dst = p.ws + ((size_t)cur.unit * (size_t)p.Lq + cur.wrow0 + col) * (D + 2);
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
        cur = nxt;
        nvis = visible_count(p, cur.wrow0 + col);
    }
}

// resident workgroups per compute unit of one kernel instantiation (asked once per kernel:
// the kernel is a template argument, so each has its own cached answer)
template <auto Kernel>
static int resident_per_cu() {
    static const int n = [] {
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, Kernel, kNW * 64, 0) != hipSuccess ||
            nb < 1)
            nb = 1;
        return nb;
    }();
    return n;
}

// Grouped-query attention with few query positions per head: the g query heads of a kv head
// read the same K and V, and in [B][Hq][Lq][d] their rows follow one another, so they can run
// as one head of g * Lq rows (the causal rule then looks at the row index modulo Lq).  Taken
// when that needs fewer row tiles than the heads one by one: 4 heads of 16 rows fill half a
// row tile instead of an eighth of four, and K and V are streamed once for the group.
static bool heads_as_one(int Hq, int Hkv, int Lq) {
    constexpr long kBM = 32 * kNW;
    const long g = Hq / Hkv;
    if (g <= 1 || g * Lq > (1L << 30)) return false;
    return (g * Lq + kBM - 1) / kBM < g * ((Lq + kBM - 1) / kBM);
}

template <typename T, int D>
static hipError_t launch_tile_t(const Problem& p_in, int mode, hipStream_t st) {
    Problem p = p_in;
    if (heads_as_one(p.Hq, p.Hkv, p.Lq)) {
        p.Li = make_fast_div((uint32_t)p.Lq);
        p.Lq *= p.Hq / p.Hkv;
        p.Hq = p.Hkv;
    }
    const long m_tiles = (p.Lq + 32 * kNW - 1) / (32 * kNW);
    if (m_tiles * p.splits * p.B * p.Hq > 0x7fffffffL) return hipErrorInvalidValue;
    const bool tl = mode == kModeLazy && p.partial && Mma<T>::kRoundedSum;
    const int per_cu = mode == kModeOnline  ? resident_per_cu<tile_kernel<T, D, kModeOnline, false>>()
                       : mode == kModeBlend ? resident_per_cu<tile_kernel<T, D, kModeBlend, false>>()
                       : tl                 ? resident_per_cu<tile_kernel<T, D, kModeLazy, true>>()
                                            : resident_per_cu<tile_kernel<T, D, kModeLazy, false>>();
    const TileSched sc = tile_sched(p, per_cu * kCusPerXcd);
    // One workgroup per virtual workgroup, handed out by the hardware as slots free up.
    // (The kernel can also walk several virtual workgroups per workgroup, but a fixed split
    // loses: of the two workgroups resident on a compute unit the older one is served first
    // and runs a third faster, and only dynamic hand-out evens that out.)
    const long wgs = sc.total;
    dim3 grid((unsigned)wgs);
    if (mode == kModeOnline)
        hipLaunchKernelGGL((tile_kernel<T, D, kModeOnline, false>), grid, dim3(kNW * 64), 0, st, p, sc);
    else if (mode == kModeBlend)
        hipLaunchKernelGGL((tile_kernel<T, D, kModeBlend, false>), grid, dim3(kNW * 64), 0, st, p, sc);
    else if (tl)
        hipLaunchKernelGGL((tile_kernel<T, D, kModeLazy, true>), grid, dim3(kNW * 64), 0, st, p, sc);
    else
        hipLaunchKernelGGL((tile_kernel<T, D, kModeLazy, false>), grid, dim3(kNW * 64), 0, st, p, sc);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !p.merge) return e;
    return launch_merge_splits(p, st);
}

long tile_workgroups(int B, int Hq, int Hkv, int Lq, int d) {
    (void)d;
    if (heads_as_one(Hq, Hkv, Lq)) {
        Lq *= Hq / Hkv;
        Hq = Hkv;
    }
    return (long)B * Hq * ((Lq + 32 * kNW - 1) / (32 * kNW));
}

hipError_t launch_tile(const Problem& p, int mode, hipStream_t st) {
    if (mode != kModeLazy && mode != kModeOnline && mode != kModeBlend) return hipErrorInvalidValue;
    if (p.wide && wide_applies(p, mode)) return launch_wide(p, mode, st);
    if (p.dtype == 1 && p.d == 64) return launch_tile_t<F16, 64>(p, mode, st);
    if (p.dtype == 1 && p.d == 128) return launch_tile_t<F16, 128>(p, mode, st);
    if (p.dtype == 2 && p.d == 64) return launch_tile_t<BF16, 64>(p, mode, st);
    if (p.dtype == 2 && p.d == 128) return launch_tile_t<BF16, 128>(p, mode, st);
    return hipErrorInvalidValue;
}

}  // namespace flashd
