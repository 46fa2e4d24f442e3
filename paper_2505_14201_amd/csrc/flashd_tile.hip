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

#include <algorithm>
#include <type_traits>

namespace flashd {

constexpr int kBC = 64;           // keys per tile

// How a tile's scores update a row (the kernel's MODE argument)
constexpr int kModeLazy = kTileModeLazy;        // variant TILE
constexpr int kModeOnline = kTileModeOnline;    // variant ONLINE_SOFTMAX (Alg. 2)
constexpr int kModeBlend = kTileModeBlend;      // variant TILE_BLEND

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

constexpr int kNW = 4;            // wavefronts per workgroup

// Per-lane byte offsets of the direct global->LDS copy.  Instruction n of a wavefront
// (n < NI = CPR/4) moves 64 chunks of 16 bytes into 1 KB of LDS: lane l fills chunk position
// cs = l % CPR of tile row 16*wave + n*(64/CPR) + l/CPR.  With the swizzles above the global
// chunk to fetch is cs ^ (l >> 4) ^ 4n for K and cs ^ swz_v for V (independent of n), so the
// element offsets are (k0 ^ 32n) + 512n and v0 + 512n.  The + 512n (1 KB) is the same on
// the global and on the LDS side and rides in the instruction's immediate offset, which is
// added to both addresses.
template <int D> struct DmaLane {
    static constexpr int NI = TileCfg<D>::CPR / kNW;
    uint32_t koff[NI], voff;
    __device__ __forceinline__ DmaLane(int wave, int lane) {
        using C = TileCfg<D>;
        const int row = (kBC / kNW) * wave + lane / C::CPR;     // row of this lane for n = 0
        const int cs = lane % C::CPR;
        const int k0 = row * D + 8 * (cs ^ C::swz_k(row));
#pragma unroll
        for (int n = 0; n < NI; ++n) koff[n] = 2u * (uint32_t)(k0 ^ (32 * n));
        voff = 2u * (uint32_t)(row * D + 8 * (cs ^ C::swz_v(row)));
    }
};

template <int N> struct IntC { static constexpr int value = N; };

// Wait until every global->LDS copy (and load) this wavefront has issued is complete.  The
// builtin rather than inline assembly, so that the compiler's own bookkeeping of outstanding
// copies sees the wait: after an assembly wait it still assumed copies in flight and put a
// full wait of its own before the first LDS write of the epilogue, which then also waited
// for the Q fragments just requested for the next row tile.
__device__ __forceinline__ void wait_copies() {
    __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0), the other counters not waited for
    asm volatile("" ::: "memory");
}


// Start the copy of the K and V tiles whose first key is j0 into ks / vs (the wavefront
// fills its own 16 rows of each).  A tile that sticks out past the last key takes the slow
// form with rows clamped to the last key (masked later).
template <int D, bool NT = false>
__device__ __forceinline__ void tile_copy(const uint16_t* kg, const uint16_t* vg, int j0, int Lk,
                                          const DmaLane<D>& dl, int wave, int lane,
                                          uint16_t* ks, uint16_t* vs) {
    // NT: the non-temporal cache policy, for K and V that no other workgroup will read
    constexpr int kAux = NT ? 2 : 0;
    using C = TileCfg<D>;
    constexpr int NI = DmaLane<D>::NI;
    uint16_t* kw = ks + wave * (NI * 512);
    uint16_t* vw = vs + wave * (NI * 512);
    if (j0 + kBC <= Lk) {
        // wavefront-uniform tile bases, 32-bit lane offsets
        const char* kt = reinterpret_cast<const char*>(kg + (size_t)j0 * D);
        const char* vt = reinterpret_cast<const char*>(vg + (size_t)j0 * D);
        // The empty asm keeps the 32-bit offsets from being widened outside the loop, so
        // that each copy is one instruction with a scalar base and a 32-bit lane offset.
        // (the immediate offset is a 13-bit signed field: 1024 N must stay below 4096)
        static_assert(1024 * (NI - 1) < 4096, "immediate offset of the copy out of range");
        auto issue = [&](auto n) {
            constexpr int N = decltype(n)::value;
            uint32_t off = dl.koff[N];
            asm volatile("" : "+v"(off));
            __builtin_amdgcn_global_load_lds((gptr_t)(kt + off), (lptr_t)kw, 16, 1024 * N, kAux);
        };
        uint32_t voff = dl.voff;
        asm volatile("" : "+v"(voff));
        auto issue_v = [&](auto n) {
            constexpr int N = decltype(n)::value;
            __builtin_amdgcn_global_load_lds((gptr_t)(vt + voff), (lptr_t)vw, 16, 1024 * N, kAux);
        };
        issue(IntC<0>{}); issue(IntC<1>{});
        if constexpr (NI == 4) { issue(IntC<2>{}); issue(IntC<3>{}); }
        issue_v(IntC<0>{}); issue_v(IntC<1>{});
        if constexpr (NI == 4) { issue_v(IntC<2>{}); issue_v(IntC<3>{}); }
    } else {
#pragma unroll 1
        for (int n = 0; n < NI; ++n) {
            const int inst = wave * NI + n;
            const int slot = inst * 64 + lane;
            const int row = slot / C::CPR;
            const int cs = slot % C::CPR;
            const size_t grow = (size_t)min(j0 + row, Lk - 1) * D;
            __builtin_amdgcn_global_load_lds((gptr_t)(kg + grow + 8 * (cs ^ C::swz_k(row))),
                                             (lptr_t)(kw + n * 512), 16, 0, kAux);
            __builtin_amdgcn_global_load_lds((gptr_t)(vg + grow + 8 * (cs ^ C::swz_v(row))),
                                             (lptr_t)(vw + n * 512), 16, 0, kAux);
        }
    }
}

// 8 keys x 1 column of V as an MFMA operand through the transposing LDS read (see
// flashd_mma.h for the lane roles); vaddr = this lane's element offset for the d-block,
// key0 = first key of the 16-key group.
template <int D>
__device__ __forceinline__ u32x4 tile_v_operand(const uint16_t* __restrict__ vs, int vaddr,
                                                int key0) {
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

// How workgroups map to work (set by the launcher).  The work is cut into "virtual
// workgroups" (one row tile of a unit, or a long and a short one under a causal mask);
// workgroup w of the launch runs the virtual workgroups w, w + gridDim.x, ... one after the
// other, with the copy pipeline running on from one to the next.
struct TileSched {
    int pair;          // 1: a virtual workgroup is row tiles (m_tiles - 1 - r) and r of its unit
    int wg_per_unit;   // virtual workgroups per (split, b, h) unit
    int nx_log2;       // 3: unit u runs on XCD u % 8 (ids go round-robin over the XCDs); 0: no such mapping
    int group;         // units of one XCD that are in flight together
    int total;         // virtual workgroups
    int once;          // 1: no two workgroups read the same K and V (one row tile per kv head)
    // fixed per launch, so that a workgroup finds its work without a division instruction
    int nux;           // units per XCD
    int per_split;     // key tiles per split
    FastDiv gw;        // virtual workgroups of a full group: group * wg_per_unit
    FastDiv gfull;     // units in a full group: group
    FastDiv glast;     // units in the last group of an XCD: nux % group (or group)
    FastDiv n_bh;      // units per split: B * Hq
    FastDiv g;         // query heads per kv head
};

// One row tile of one unit as seen by a wavefront.  All members are wavefront-uniform.
struct Item {
    bool valid;
    int sp, bh, unit;           // split, b * Hq + h, sp * B * Hq + bh
    const uint16_t* qg;         // this head's Q, K, V, O
    const uint16_t* kg;
    const uint16_t* vg;
    uint16_t* og;
    int wrow0;                  // first row of the wavefront
    int wmax, wmin;             // most / fewest keys visible to a row of the wavefront
    int n;                      // key tiles of this item (within its split)
    int jbase;                  // first key of tile 0
};

// Most and fewest keys visible to the rows r0 .. r1 (r0 <= r1 < Lq), or bounds of them.  With
// the heads of a kv group run as one head (Li.d < Lq) a range of rows may run over the end of a
// head; the bounds are then those of a whole head, its last and its first position (they only
// decide which tiles a wavefront may skip and which take the code path without the mask).
__device__ __forceinline__ void visible_range(const Problem& p, int r0, int r1, int& most,
                                              int& fewest) {
    const bool whole_head = (int)p.Li.d != p.Lq;
    most = visible_at(p, whole_head ? (int)p.Li.d - 1 : r1);
    fewest = visible_at(p, whole_head ? 0 : r0);
}

// Item number seq of this workgroup, or an invalid item when the workgroup has run out of
// work.  (A virtual workgroup that is a pair whose two row tiles coincide has one item; the
// caller skips the other.)
template <int D>
__device__ __forceinline__ Item make_item(const Problem& p, const TileSched& sc, int seq,
                                          int wave, bool& skip) {
    constexpr int kBM = 32 * kNW;
    Item it;
    it.valid = false;
    it.n = 0;
    skip = false;
    const int v = blockIdx.x + (seq >> sc.pair) * gridDim.x;
    if (v >= sc.total) return it;
    // virtual workgroup id -> (unit, rank of the row tile within the unit)
    const int m_tiles = (p.Lq + kBM - 1) / kBM;
    const int xcd = v & ((1 << sc.nx_log2) - 1);
    const int local = v >> sc.nx_log2;
    const int grp = (int)fast_div((uint32_t)local, sc.gw);
    const int within = local - grp * (int)sc.gw.d;
    const bool last = (grp + 1) * sc.group > sc.nux;             // the XCD's last, shorter group
    const int gsz = last ? (int)sc.glast.d : sc.group;
    const int rank = (int)(last ? fast_div((uint32_t)within, sc.glast)
                                : fast_div((uint32_t)within, sc.gfull));     // slowest inside a group
    const int unit = xcd + ((grp * sc.group + within - rank * gsz) << sc.nx_log2);
    int mt;
    if (sc.pair) {
        // the longer row tile first
        mt = (seq & 1) == 0 ? m_tiles - 1 - rank : rank;
        if ((seq & 1) == 1 && m_tiles - 1 - rank == rank) { skip = true; return it; }
    } else {
        mt = p.causal ? m_tiles - 1 - rank : rank;
    }
    it.valid = true;
    it.unit = unit;
    it.sp = (int)fast_div((uint32_t)unit, sc.n_bh);
    it.bh = unit - it.sp * (int)sc.n_bh.d;
    const size_t kv_unit = fast_div((uint32_t)it.bh, sc.g);     // b * Hkv + h / g
    it.qg = static_cast<const uint16_t*>(p.q) + (size_t)it.bh * (size_t)p.Lq * D;
    it.kg = static_cast<const uint16_t*>(p.k) + kv_unit * (size_t)p.Lk * D;
    it.vg = static_cast<const uint16_t*>(p.v) + kv_unit * (size_t)p.Lk * D;
    it.og = static_cast<uint16_t*>(p.o) + (size_t)it.bh * (size_t)p.Lq * D;
    const int m0 = mt * kBM;
    it.wrow0 = m0 + wave * 32;
    it.wmax = 0;
    it.wmin = 0;
    if (it.wrow0 < p.Lq) {
        int mn;
        visible_range(p, it.wrow0, min(it.wrow0 + 31, p.Lq - 1), it.wmax, mn);
        if (it.wrow0 + 31 < p.Lq) it.wmin = mn;      // a row past the end sees no key
    }
    int blk_nvis, blk_min;
    visible_range(p, m0, min(m0 + kBM - 1, p.Lq - 1), blk_nvis, blk_min);
    const int t_begin = it.sp * sc.per_split;
    const int t_end = min((blk_nvis + kBC - 1) / kBC, t_begin + sc.per_split);
    it.n = max(t_end - t_begin, 0);
    it.jbase = t_begin * kBC;
    return it;
}

// The first valid item at or after seq (seq is advanced to it), or an invalid one.
template <int D>
__device__ __forceinline__ Item next_item(const Problem& p, const TileSched& sc, int& seq,
                                          int wave) {
    bool skip;
    Item it = make_item<D>(p, sc, seq, wave, skip);
    if (skip) {
        ++seq;
        it = make_item<D>(p, sc, seq, wave, skip);
    }
    return it;
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

constexpr int kXcds = 8;
constexpr int kCusPerXcd = 32;

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

static TileSched tile_sched(const Problem& p, int slots_per_xcd) {
    const long m_tiles = (p.Lq + 32 * kNW - 1) / (32 * kNW);
    const long units = (long)p.splits * p.B * p.Hq;
    TileSched sc;
    // Pairing halves the number of virtual workgroups; it pays once there are at least
    // two rounds of them for all workgroup slots.  (Not with the heads of a kv group run
    // as one head: the row tiles of such a run do not grow in length from first to last.  Not
    // with split keys either: a split's share of a long and of a short row tile do not add up
    // to the same for every pair.)
    sc.pair = (p.causal && p.splits == 1 && (int)p.Li.d == p.Lq && m_tiles >= 2 &&
               m_tiles * units >= 2L * kXcds * slots_per_xcd) ? 1 : 0;
    sc.wg_per_unit = (int)(sc.pair ? (m_tiles + 1) / 2 : m_tiles);
    sc.nx_log2 = units % kXcds == 0 ? 3 : 0;
    static_assert(kXcds == 8, "the unit -> XCD mapping shifts by 3");
    const long nux = units >> sc.nx_log2;
    // Virtual workgroups that all carry the same work (paired, or no mask): run as few
    // units at a time as fill the XCD, so that their K/V stay in its L2.  Unpaired causal
    // tiles differ in length: all units together, longest tiles first.
    long group = nux;
    if (sc.pair || !p.causal) group = std::max(1L, (long)slots_per_xcd / sc.wg_per_unit);
    sc.group = (int)std::min(group, nux);
    sc.total = (int)(sc.wg_per_unit * units);
    sc.once = (m_tiles == 1 && p.Hq == p.Hkv) ? 1 : 0;
    sc.nux = (int)nux;
    const long tiles_all = (p.Lk + kBC - 1) / kBC;
    sc.per_split = (int)((tiles_all + p.splits - 1) / p.splits);
    sc.gw = make_fast_div((uint32_t)(sc.group * sc.wg_per_unit));
    sc.gfull = make_fast_div((uint32_t)sc.group);
    sc.glast = make_fast_div((uint32_t)(nux % sc.group != 0 ? nux % sc.group : sc.group));
    sc.n_bh = make_fast_div((uint32_t)(p.B * p.Hq));
    sc.g = make_fast_div((uint32_t)(p.Hq / p.Hkv));
    return sc;
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
    if (p.dtype == 1 && p.d == 64) return launch_tile_t<F16, 64>(p, mode, st);
    if (p.dtype == 1 && p.d == 128) return launch_tile_t<F16, 128>(p, mode, st);
    if (p.dtype == 2 && p.d == 64) return launch_tile_t<BF16, 64>(p, mode, st);
    if (p.dtype == 2 && p.d == 128) return launch_tile_t<BF16, 128>(p, mode, st);
    return hipErrorInvalidValue;
}

}  // namespace flashd
