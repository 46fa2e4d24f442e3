// Pieces shared by the matrix-core prefill kernels: the LDS layout of a K or V tile and the
// direct global->LDS copy that fills it, the transposing V operand read, and the hand-out of
// row tiles to workgroups (TileSched, Item).
#pragma once

#include "flashd_common.h"
#include "flashd_kernels.h"
#include "flashd_mma.h"

#include <algorithm>

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
template <int D, int BM = 32 * kNW>
__device__ __forceinline__ Item make_item(const Problem& p, const TileSched& sc, int seq,
                                          int wave, bool& skip) {
    constexpr int kBM = BM;             // rows per workgroup
    constexpr int kRW = BM / kNW;       // rows per wavefront
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
    it.wrow0 = m0 + wave * kRW;
    it.wmax = 0;
    it.wmin = 0;
    if (it.wrow0 < p.Lq) {
        int mn;
        visible_range(p, it.wrow0, min(it.wrow0 + kRW - 1, p.Lq - 1), it.wmax, mn);
        if (it.wrow0 + kRW - 1 < p.Lq) it.wmin = mn;      // a row past the end sees no key
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
template <int D, int BM = 32 * kNW>
__device__ __forceinline__ Item next_item(const Problem& p, const TileSched& sc, int& seq,
                                          int wave) {
    bool skip;
    Item it = make_item<D, BM>(p, sc, seq, wave, skip);
    if (skip) {
        ++seq;
        it = make_item<D, BM>(p, sc, seq, wave, skip);
    }
    return it;
}

constexpr int kXcds = 8;
constexpr int kCusPerXcd = 32;

// rows: query rows per workgroup
inline TileSched tile_sched(const Problem& p, int slots_per_xcd, int rows = 32 * kNW) {
    const long m_tiles = (p.Lq + rows - 1) / rows;
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

}  // namespace flashd
