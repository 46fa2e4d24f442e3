// The tiled FLASH-D prefill kernel with 256 query rows per workgroup (variant TILE_256).
//
// Same tile form of Alg. 3 (Sec. III-A/B lifted to key tiles, see flashd_tile.hip and
// flashd_mma.h), same LDS layout of a tile, same copies and work hand-out as the 128-row
// kernel.  What differs is the shape of a workgroup and the order of the work:
//
//   * A wavefront owns two 32-row blocks, a workgroup of 4 wavefronts 256 rows, and a compute
//     unit holds one workgroup (one wavefront per SIMD, up to 512 registers each).  Every K or V
//     operand read from LDS feeds two matrix instructions instead of one and a tile is copied
//     into LDS once per 256 rows: LDS traffic and copy instructions per matrix instruction halve.
//     (With 32 rows per wavefront the operand reads alone take 125 bytes per clock of LDS
//     bandwidth at the full matrix rate.)
//   * The unit of work is a block of 32 keys.  With one wavefront per SIMD nothing else fills
//     the matrix pipe while a wavefront does the exponentials, so the two kinds of work are
//     issued together by the wavefront itself ("fused steps", wide_h1 / wide_h2): the scores
//     of block b + 1 are formed while the coefficients of block b's first 16 keys are computed
//     (two score accumulators), and the output product of block b runs while the coefficients
//     of its last 16 keys, the update of the row state and the look at block b + 1's top scores
//     are computed.  A few vector instructions follow each matrix instruction and run in its
//     shadow; operand reads and copies are spread over the slots as well.
//   * Nothing is speculated: the output product of a block starts before all its coefficients
//     exist, so a coefficient that does not fit the storage type must be ruled out beforehand.
//     Every block takes the checked step of flashd_mma.h: the row's top score is looked at first
//     and the reference moves there if it lies more than LazyLimit::kMoveLog2 above it (the
//     saturation of Sec. III-C in tile form); the fused steps hand a block whose reference has
//     to move to the plain steps, which scale what the rows hold.
//   * The output accumulators, the Q fragments and the matrix operands live in fixed
//     accumulation registers that only inline assembly touches (flashd_wide_regs.h).
//
// Blocks on which a mask applies or a row may still be empty (the first block, the diagonal
// blocks of a causal mask, the tail), and any block under a negative scale, take the plain
// steps (wide_first_general / wide_second).
//
// Serves f16/bf16, d = 128, Lq a multiple of 256, unsplit calls without state in or out
// (wide_applies()); everything else stays with the 128-row kernel.
#include "flashd_common.h"
#include "flashd_kernels.h"
#include "flashd_mma.h"
#include "flashd_tile_parts.h"
#include "flashd_wide_regs.h"

#include <type_traits>

namespace flashd {

constexpr int kWideRB = 2;                      // 32-row blocks per wavefront
constexpr int kWideBM = 32 * kWideRB * kNW;     // query rows per workgroup
constexpr int kWideKB = 32;                     // keys per step of a wavefront (half a tile)

// (The output accumulators U and the Q fragments are not here: they live in fixed accumulation
// registers, see flashd_wide_regs.h.)
template <int D> struct WideRegs {
    int kaddr[D / 16];
    int vaddr[D / 32];
    LazyRow st[kWideRB];            // FLASH-D state, lazy form
};

// K (IS_V = false) or V rows of one tile into LDS: this wavefront's 16 rows.
template <int D, bool IS_V>
__device__ __forceinline__ void wide_copy(const uint16_t* src, int j0, int Lk, const DmaLane<D>& dl,
                                          int wave, int lane, uint16_t* dst) {
    using C = TileCfg<D>;
    constexpr int NI = DmaLane<D>::NI;
    uint16_t* w = dst + wave * (NI * 512);
    if (j0 + kBC <= Lk) {
        const char* t = reinterpret_cast<const char*>(src + (size_t)j0 * D);
        static_assert(1024 * (NI - 1) < 4096, "immediate offset of the copy out of range");
        uint32_t voff = dl.voff;
        asm volatile("" : "+v"(voff));
        auto issue = [&](auto n) {
            constexpr int N = decltype(n)::value;
            uint32_t off = IS_V ? voff : dl.koff[N];
            if (!IS_V) asm volatile("" : "+v"(off));
            __builtin_amdgcn_global_load_lds((gptr_t)(t + off), (lptr_t)w, 16, 1024 * N, 0);
        };
        issue(IntC<0>{}); issue(IntC<1>{});
        if constexpr (NI == 4) { issue(IntC<2>{}); issue(IntC<3>{}); }
    } else {
#pragma unroll 1
        for (int n = 0; n < NI; ++n) {
            const int inst = wave * NI + n;
            const int slot = inst * 64 + lane;
            const int row = slot / C::CPR;
            const int cs = slot % C::CPR;
            const size_t grow = (size_t)min(j0 + row, Lk - 1) * D;
            const int sw = IS_V ? C::swz_v(row) : C::swz_k(row);
            __builtin_amdgcn_global_load_lds((gptr_t)(src + grow + 8 * (cs ^ sw)),
                                             (lptr_t)(w + n * 512), 16, 0, 0);
        }
    }
}

// The matrix instructions of this kernel are inline assembly on fixed accumulation registers
// (flashd_wide_regs.h): the output accumulators U and the Q fragments never pass through the
// register allocator, which otherwise moves them between register files at every merge of
// control flow; the score accumulators are ordinary registers, where the vector instructions
// read them.  The functions below pick the instruction for a register index that is a
// constant once the loops around them are unrolled.  The compiler does not see these as
// matrix instructions, so a result is only read by vector instructions that are known to come
// at least 20 wait states later (mma_fence() where nothing else lies between).
__device__ __forceinline__ void wide_set_q_n(int n, u32x4 q) {
    switch (n) {
#define FLASHD_CASE(N) case N: wide_set_q<N>(q); break;
        FLASHD_CASE(0) FLASHD_CASE(1) FLASHD_CASE(2) FLASHD_CASE(3) FLASHD_CASE(4) FLASHD_CASE(5)
        FLASHD_CASE(6) FLASHD_CASE(7) FLASHD_CASE(8) FLASHD_CASE(9) FLASHD_CASE(10) FLASHD_CASE(11)
        FLASHD_CASE(12) FLASHD_CASE(13) FLASHD_CASE(14) FLASHD_CASE(15)
#undef FLASHD_CASE
    }
}
__device__ __forceinline__ f32x16 wide_get_u_n(int j) {
    switch (j) {
#define FLASHD_CASE(J) case J: return wide_get_u<J>();
        FLASHD_CASE(0) FLASHD_CASE(1) FLASHD_CASE(2) FLASHD_CASE(3) FLASHD_CASE(4) FLASHD_CASE(5)
        FLASHD_CASE(6) FLASHD_CASE(7)
#undef FLASHD_CASE
    }
    return f32x16{};
}
__device__ __forceinline__ void wide_put_u_n(int j, const f32x16& x) {
    switch (j) {
#define FLASHD_CASE(J) case J: wide_put_u<J>(x); break;
        FLASHD_CASE(0) FLASHD_CASE(1) FLASHD_CASE(2) FLASHD_CASE(3) FLASHD_CASE(4) FLASHD_CASE(5)
        FLASHD_CASE(6) FLASHD_CASE(7)
#undef FLASHD_CASE
    }
}

// The fused steps: operands in fixed registers too (flashd_wide_regs.h)
#define FLASHD_CASES16(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15)
#define FLASHD_CASES8(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7)
template <typename T>
__device__ __forceinline__ void ws_mma(int rb, int kk, f32x16& acc) {
    switch (8 * rb + kk) {
#define FLASHD_CASE(N) case N: WideS<T, N / 8, N % 8>::mma(acc); break;
        FLASHD_CASES16(FLASHD_CASE)
#undef FLASHD_CASE
    }
}
template <typename T>
__device__ __forceinline__ void wp_mma(int rb, int m, u32x4 b) {
    switch (8 * rb + m) {
#define FLASHD_CASE(N) case N: WideP<T, N / 8, N % 8>::mma(b); break;
        FLASHD_CASES16(FLASHD_CASE)
#undef FLASHD_CASE
    }
}
__device__ __forceinline__ void wide_read_k_n(int kk, uint32_t addr) {
    switch (kk) {
#define FLASHD_CASE(N) case N: wide_read_k<N>(addr); break;
        FLASHD_CASES8(FLASHD_CASE)
#undef FLASHD_CASE
    }
}
__device__ __forceinline__ void wide_read_v_n(int m, uint32_t addr) {
    switch (m) {
#define FLASHD_CASE(N) case N: wide_read_v<N>(addr); break;
        FLASHD_CASES8(FLASHD_CASE)
#undef FLASHD_CASE
    }
}
__device__ __forceinline__ void wide_wait_lds_n(int n) {
    switch (n) {
        case 0: wide_wait_lds<0>(); break;
        case 1: wide_wait_lds<1>(); break;
        case 2: wide_wait_lds<2>(); break;
        case 3: wide_wait_lds<3>(); break;
        default: wide_wait_lds<4>(); break;
    }
}
#undef FLASHD_CASES16
#undef FLASHD_CASES8
__device__ __forceinline__ uint32_t lds_byte_address(const uint16_t* p) {
    return (uint32_t)(uintptr_t)(lptr_t)p;
}
// K operand kk of a block whose K rows start at kb; V operand m of a block whose V rows start at vb
template <int D>
__device__ __forceinline__ void wide_req_k(int kk, const uint16_t* kb, const WideRegs<D>& g) {
    wide_read_k_n(kk, lds_byte_address(kb) + 2u * (uint32_t)g.kaddr[kk]);
}
template <int D>
__device__ __forceinline__ void wide_req_v(int m, const uint16_t* vb, const WideRegs<D>& g) {
    constexpr int NDB = D / 32;
    wide_read_v_n(m, lds_byte_address(vb) +
                         2u * (uint32_t)(g.vaddr[m % NDB] + 16 * (m / NDB) * D));
}

// Results of the matrix instructions before this point may be read by vector instructions
// after it (20 wait states cover the longest of these instructions).
__device__ __forceinline__ void mma_fence(f32x16 (&acc)[kWideRB]) {
    asm volatile("s_nop 15\n\ts_nop 7" : "+v"(acc[0]), "+v"(acc[1]));
}

// Copy instruction N (of DmaLane::NI) of the same, for a tile that lies wholly inside the keys:
// the fused steps issue the copies of a period one at a time, spread over the period (issued
// together by the four wavefronts of the workgroup, which run in step, 32 of these queue up in
// front of the one address unit), and without a branch in between.
template <int D, bool IS_V, int N>
__device__ __forceinline__ void wide_copy_one(const uint16_t* src, int j0, const DmaLane<D>& dl,
                                              int wave, uint16_t* dst) {
    constexpr int NI = DmaLane<D>::NI;
    static_assert(N < NI, "a tile takes NI copy instructions per wavefront");
    uint16_t* w = dst + wave * (NI * 512);
    const char* t = reinterpret_cast<const char*>(src + (size_t)j0 * D);
    uint32_t off = IS_V ? dl.voff : dl.koff[N];
    asm volatile("" : "+v"(off));
    __builtin_amdgcn_global_load_lds((gptr_t)(t + off), (lptr_t)w, 16, 1024 * N, 0);
}

// Raw scores of one 32-key block (kb: its rows in LDS) for both row blocks, by plain steps:
// all eight K operands into the operand ring, then the sixteen matrix instructions (every
// operand feeds two).
template <typename T, int D>
__device__ __forceinline__ void wide_scores(const uint16_t* kb, const WideRegs<D>& g,
                                            f32x16 (&acc)[kWideRB]) {
    constexpr int NKK = D / 16;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) wide_req_k<D>(kk, kb, g);
    wide_wait_lds<0>();
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
        for (int rb = 0; rb < kWideRB; ++rb) ws_mma<T>(rb, kk, acc[rb]);
    mma_fence(acc);
}

// Scaling what the rows of a row block hold (rare: their reference has moved).
template <int D>
__device__ __forceinline__ void wide_scale_u(int rb, float f) {
#pragma unroll
    for (int i = 0; i < D / 32; ++i) {
        f32x16 x = wide_get_u_n(4 * rb + i);
#pragma unroll
        for (int r = 0; r < 16; ++r) x[r] *= f;
        wide_put_u_n(4 * rb + i, x);
    }
}

// What the first half of a block's step leaves for the second: the coefficients of the first
// 16 keys packed, the exponentials of the last 16, the partial sums, and per row the reference
// used, the factor what the row held was scaled by, and whether the row was still empty.
struct WideCoef {
    u32x4 bf0[kWideRB];
    f32x8 pv1[kWideRB];
    f32x4 ps[kWideRB];
    float ref[kWideRB], f[kWideRB];
    bool empty[kWideRB];
};

// What one fused step hands to the next: the K operands of the next score product (requested
// while the output product runs) and whether the next block can be taken by a fused step at
// all: a row's reference (TILE) moves only if the block's top score lies more than
// LazyLimit::kMoveLog2 above it; what the rows hold would then have to be scaled, which the
// fused steps do not do (bail: the block goes through wide_first_general()).
struct WideAhead {
    bool bail;                  // wavefront-uniform
};

__device__ __forceinline__ float wide_top_part(const f32x16& a, int part, float top) {
    if (part == 0) {
        top = fmaxf(a[0], a[1]);
#pragma unroll
        for (int r = 2; r < 8; r += 2) top = fmaxf(fmaxf(top, a[r]), a[r + 1]);
    } else {
#pragma unroll
        for (int r = 8; r < 16; r += 2) top = fmaxf(fmaxf(top, a[r]), a[r + 1]);
    }
    return top;
}

// The look at the top scores of a block that a fused step may take next (all keys visible, no
// row empty, scale >= 0) and the request for its successor's K operands, on their own: used
// where a fused step follows a plain one.
template <typename T, int D>
__device__ __forceinline__ void wide_look_ahead(const uint16_t* kb, const WideRegs<D>& g,
                                                const f32x16 (&acc)[kWideRB], float c_log2,
                                                WideAhead& ah) {
#pragma unroll
    for (int kk = 0; kk < 3; ++kk) wide_req_k<D>(kk, kb, g);
    bool move = false;
#pragma unroll
    for (int rb = 0; rb < kWideRB; ++rb) {
        float top = wide_top_part(acc[rb], 0, 0.0f);
        top = wide_top_part(acc[rb], 1, top);
        move |= pair_max(top * c_log2) - g.st[rb].R > LazyLimit<T>::kMoveLog2;
    }
    ah.bail = __builtin_amdgcn_ballot_w64(move) != 0;
}

// First half of a fused step (an interior block: all 32 keys visible to all rows, no row
// empty, scale >= 0, no reference to move): the scores of the next block are formed (into
// accn, kb: that block's K rows in LDS) while the vector instructions compute the coefficients
// of this block's first 16 keys.  The vector work is a pipeline of its own, one key per slot:
// after matrix instruction s come the scaling of score s + 1, the exponential of score s and
// the summing and packing of coefficient s - 1, three instructions that do not wait for one
// another (with one wavefront per SIMD there is nobody else to fill a wait).
template <typename T, int D>
__device__ __forceinline__ void wide_h1(const WideAhead& ah, const uint16_t* kb,
                                        const uint16_t* vb, const WideRegs<D>& g,
                                        const f32x16 (&acc)[kWideRB], f32x16 (&accn)[kWideRB],
                                        float c_log2, WideCoef& c) {
    static_assert(D == 128 && kWideRB == 2, "the slots below are laid out for this shape");
    constexpr int NKK = D / 16;
    // The operands are read from LDS into fixed registers by inline assembly, one operand per
    // two slots and each six slots ahead of its use (the four wavefronts of the workgroup run
    // in step, and reads issued together by all of them queue up in front of the LDS while
    // the matrix pipe waits); K operands 0..2 were requested by the step before.  The waits
    // count the read instructions issued after the wanted one (a V operand takes two).
    (void)ah;
#pragma unroll
    for (int rb = 0; rb < kWideRB; ++rb) {
        c.ref[rb] = g.st[rb].R;
        c.f[rb] = 1.0f;
        c.empty[rb] = false;
        c.ps[rb] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
    // key i of the 16: row block i & 1, score register i >> 1
    float x[17], pe[16];
    auto F = [&](int i) __attribute__((always_inline)) {
        if (i < 16) x[i] = fmaf(acc[i & 1][i >> 1], c_log2, -c.ref[i & 1]);
    };
    auto X = [&](int i) __attribute__((always_inline)) { pe[i] = exp2_fast(x[i]); };
    auto A = [&](int i) __attribute__((always_inline)) {
        if (i < 0) return;
        const int rb = i & 1, e = i >> 1;
        c.ps[rb][e & 3] += pe[i];
        if (e & 1) c.bf0[rb][e >> 1] = Mma<T>::pack2(pe[i - 2], pe[i]);
    };
    F(0);
    __builtin_amdgcn_sched_barrier(0);
    // slot s = 2 kk + rb
#pragma unroll
    for (int s = 0; s < 2 * NKK; ++s) {
        const int kk = s >> 1, rb = s & 1;
        if ((s & 1) == 0) wide_wait_lds_n(s < 12 ? 2 : s == 12 ? 3 : 4);
        ws_mma<T>(rb, kk, accn[rb]);
        // K operand 3 + s / 2 (used in slot 6 + s), then V operands 0..2 of the second half
        if (s <= 8 && (s & 1) == 0) wide_req_k<D>(3 + (s >> 1), kb, g);
        if (s >= 10 && (s & 1) == 0) wide_req_v<D>((s - 10) >> 1, vb, g);
        F(s + 1);
        X(s);
        A(s - 1);
        __builtin_amdgcn_sched_barrier(0);
    }
    A(15);
}

// Second half of a fused step: the output product U <- U + P V over the block's 32 keys (vb: its
// V rows in LDS) while the vector instructions compute the coefficients of its last 16 keys
// (two per slot in the first eight slots: their products come in the last eight), update the
// row state,
//     1/beta' = 1/beta + psum,
// and look at the top scores of the next block (accn): ah.bail.  Pipelined like wide_h1.
// copy_hook(i), i = 0..3: called in slots 1, 5, 9, 13, for the caller's global->LDS copies.
template <typename T, int D, typename Hook>
__device__ __forceinline__ void wide_h2(const uint16_t* vb, const uint16_t* kb_ahead,
                                        WideRegs<D>& g, const f32x16 (&acc)[kWideRB],
                                        const f32x16 (&accn)[kWideRB], float c_log2, WideCoef& c,
                                        WideAhead& ah, const Hook& copy_hook) {
    static_assert(D == 128 && kWideRB == 2, "the slots below are laid out for this shape");
    constexpr int NDB = D / 32;
    constexpr int NV = 2 * NDB;
    u32x4 bf1[kWideRB];
    // pair q of the 8: row block q >> 2, score registers 8 + 2 (q & 3) and the next
    float x0[9], x1[9], p0[8], p1[8];
    auto F = [&](int q) __attribute__((always_inline)) {
        if (q >= 8) return;
        const int rb = q >> 2, e = 8 + 2 * (q & 3);
        x0[q] = fmaf(acc[rb][e], c_log2, -c.ref[rb]);
        x1[q] = fmaf(acc[rb][e + 1], c_log2, -c.ref[rb]);
    };
    auto X = [&](int q) __attribute__((always_inline)) {
        p0[q] = exp2_fast(x0[q]);
        p1[q] = exp2_fast(x1[q]);
    };
    auto A = [&](int q) __attribute__((always_inline)) {
        if (q < 0) return;
        const int rb = q >> 2, e = 2 * (q & 3);
        c.ps[rb][e & 3] += p0[q];
        c.ps[rb][(e + 1) & 3] += p1[q];
        bf1[rb][q & 3] = Mma<T>::pack2(p0[q], p1[q]);
    };
    float top[kWideRB], t2[kWideRB], sw[kWideRB], psum[kWideRB], tot[kWideRB], inv[kWideRB];
    float tm[kWideRB];
    bool move[kWideRB];
    F(0);
    __builtin_amdgcn_sched_barrier(0);
    // slot s = 2 m + rb; the products of key group m / NDB
#pragma unroll
    for (int s = 0; s < 2 * NV; ++s) {
        const int m = s >> 1, rb = s & 1;
        if ((s & 1) == 0) wide_wait_lds_n(s < 12 ? 4 : s == 12 ? 3 : 2);
        wp_mma<T>(rb, m, m / NDB == 0 ? c.bf0[rb] : bf1[rb]);
        // V operand 3 + s / 2 (used in slot 6 + s), then the first K operands of the next step
        if (s <= 8 && (s & 1) == 0) wide_req_v<D>(3 + (s >> 1), vb, g);
        if (s >= 10 && (s & 1) == 0) wide_req_k<D>((s - 10) >> 1, kb_ahead, g);
        if ((s & 3) == 1) copy_hook(s >> 2);
        if (s < 8) { F(s + 1); X(s); A(s - 1); }
        if (s == 8) A(7);
        // the look at the next block: two maxima per row block and slot
        if (s >= 8 && s < 12) {
            const int r0 = 4 * (s - 8);
#pragma unroll
            for (int rbb = 0; rbb < kWideRB; ++rbb) {
                if (s == 8) top[rbb] = fmaxf(accn[rbb][0], accn[rbb][1]);
                else top[rbb] = fmaxf(fmaxf(top[rbb], accn[rbb][r0]), accn[rbb][r0 + 1]);
                top[rbb] = fmaxf(fmaxf(top[rbb], accn[rbb][r0 + 2]), accn[rbb][r0 + 3]);
            }
        }
        // sums of the coefficients, state update and the rest of the look, a stage per slot
        if (s == 9) {
#pragma unroll
            for (int rbb = 0; rbb < kWideRB; ++rbb)
                t2[rbb] = (c.ps[rbb][0] + c.ps[rbb][1]) + (c.ps[rbb][2] + c.ps[rbb][3]);
        }
        if (s == 10) {
#pragma unroll
            for (int rbb = 0; rbb < kWideRB; ++rbb) psum[rbb] = pair_sum(t2[rbb]);
        }
        if (s == 11) {
#pragma unroll
            for (int rbb = 0; rbb < kWideRB; ++rbb) tot[rbb] = fmaf(g.st[rbb].beta, psum[rbb], 1.0f);
        }
        if (s == 12) {
#pragma unroll
            for (int rbb = 0; rbb < kWideRB; ++rbb) {
                inv[rbb] = __builtin_amdgcn_rcpf(tot[rbb]);
                sw[rbb] = top[rbb] * c_log2;
            }
        }
        if (s == 13) {
#pragma unroll
            for (int rbb = 0; rbb < kWideRB; ++rbb) {
                g.st[rbb].beta *= inv[rbb];
                tm[rbb] = pair_max(sw[rbb]);
            }
        }
        if (s == 14) {
#pragma unroll
            for (int rbb = 0; rbb < kWideRB; ++rbb)
                move[rbb] = tm[rbb] - g.st[rbb].R > LazyLimit<T>::kMoveLog2;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    ah.bail = __builtin_amdgcn_ballot_w64(move[0] | move[1]) != 0;
}

// First half of the step of any other block (a mask applies, rows may be empty, any scale, or
// a reference has to move), by plain steps: the checked step of flashd_mma.h.  For a row the
// block's top score m is compared with the reference first; if the row is still empty or m
// lies more than LazyLimit::kMoveLog2 above R the reference moves to m, every coefficient is
// then at most 1, and what the row holds is scaled by f = 2^{R - m} (here).  jb: index of the
// key in accumulator register 0 for this lane.
template <typename T, int D>
__device__ __forceinline__ void wide_first_general(const uint16_t* vb, WideRegs<D>& g,
                                                   const f32x16 (&acc)[kWideRB],
                                                   float c_log2, int jb,
                                                   const int (&nvis)[kWideRB], WideCoef& c) {
    const float ninf = -__builtin_inff();
#pragma unroll
    for (int rb = 0; rb < kWideRB; ++rb) {
        const f32x16 a1[1] = {acc[rb]};
        const float m = row_top_score<1, true>(a1, c_log2, jb, nvis[rb]);
        const bool empty = g.st[rb].one == 0.0f;
        const float mref = (m == ninf) ? 0.0f : m;
        const bool move = empty || (m - g.st[rb].R > LazyLimit<T>::kMoveLog2);
        c.ref[rb] = move ? mref : g.st[rb].R;
        c.f[rb] = empty ? 0.0f : (move ? exp2_fast(g.st[rb].R - mref) : 1.0f);
        c.empty[rb] = empty;
        if (__builtin_amdgcn_ballot_w64(c.f[rb] != 1.0f) != 0) wide_scale_u<D>(rb, c.f[rb]);
        int nv = nvis[rb];
        asm volatile("" : "+v"(nv));      // keep these compares apart from row_top_score's
        f32x8 pv0;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float x = fmaf(acc[rb][e], c_log2, -c.ref[rb]);
            x = ((jb + 8 * (e >> 2) + (e & 3)) >= nv) ? ninf : x;
            const float pe = exp2_fast(x);
            if (e < 8) pv0[e] = pe; else c.pv1[rb][e - 8] = pe;
        }
        c.bf0[rb] = Mma<T>::pack8(pv0);
        c.ps[rb] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int e = 0; e < 8; ++e) c.ps[rb][e & 3] += pv0[e];
    }
    (void)vb;
}

// Second half of a block's step by plain steps: the output product U <- U + P V over the
// block's 32 keys (vb: its V rows in LDS) for both row blocks, and the update of the row state,
//     1/beta' = f / beta + psum   (the carried sum of coefficients, against the reference used).
template <typename T, int D>
__device__ __forceinline__ void wide_second(const uint16_t* vb, WideRegs<D>& g, WideCoef& c) {
    constexpr int NDB = D / 32;
    constexpr int NV = 2 * NDB;
#pragma unroll
    for (int m = 0; m < NV; ++m) wide_req_v<D>(m, vb, g);
    u32x4 bf1[kWideRB];
#pragma unroll
    for (int rb = 0; rb < kWideRB; ++rb) {
        bf1[rb] = Mma<T>::pack8(c.pv1[rb]);
#pragma unroll
        for (int e = 0; e < 8; ++e) c.ps[rb][e & 3] += c.pv1[rb][e];
        const float psum = pair_sum((c.ps[rb][0] + c.ps[rb][1]) + (c.ps[rb][2] + c.ps[rb][3]));
        const float carried = c.empty[rb] ? 0.0f : c.f[rb] * __builtin_amdgcn_rcpf(g.st[rb].beta);
        const float tot = carried + psum;
        const bool has = tot > 0.0f;        // false only for an empty row that sees no key here
        g.st[rb].beta = has ? __builtin_amdgcn_rcpf(tot) : g.st[rb].beta;
        g.st[rb].R = has ? c.ref[rb] : g.st[rb].R;
        g.st[rb].one = has ? 1.0f : g.st[rb].one;
    }
    wide_wait_lds<0>();
    // the coefficients were packed by vector instructions just now: two wait states before the
    // first matrix instruction reads them
    asm volatile("s_nop 1");
#pragma unroll
    for (int m = 0; m < NV; ++m)
#pragma unroll
        for (int rb = 0; rb < kWideRB; ++rb) wp_mma<T>(rb, m, m / NDB == 0 ? c.bf0[rb] : bf1[rb]);
}

// LDS: four K slots and three V slots.  A wavefront forms the scores of block b + 1 while it
// works on block b, so during the period of tile t it reads K(t), K(t + 1) and V(t); the
// copies of K(t + 3) and V(t + 2) are started in that period and those started one period
// earlier, K(t + 2) and V(t + 1), are waited for at its end: a copy has two periods to land
// (a period of this kernel is half as long as one of the 128-row kernel, and one period is less
// than the latency of a copy).  One workgroup barrier per tile.
template <typename T, int D, int MODE>
__global__ __launch_bounds__(kNW * 64, 1)
void wide_kernel(Problem p, TileSched sc) {
    using C = TileCfg<D>;
    constexpr int NKK = D / 16;
    constexpr int NDB = D / 32;
    constexpr int kTile = kBC * D;
    __shared__ __align__(1024) uint16_t lds[7 * kTile];       // K0 K1 K2 K3 V0 V1 V2
    uint16_t* const vs0 = lds + 4 * kTile;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31;
    const int hh = lane >> 5;
    const DmaLane<D> dl(wave, lane);
    const float c_log2 = p.scale * kLog2e;
    WideRegs<D> g;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) g.kaddr[kk] = col * D + 8 * ((2 * kk + hh) ^ C::swz_k(col));
    {
        const int t = lane & 15;
        const int tq = t >> 2;
        const int half = (lane >> 4) & 1;
#pragma unroll
        for (int i = 0; i < NDB; ++i)
            g.vaddr[i] = (4 * hh + tq) * D +
                         8 * ((4 * i + 2 * half + ((t & 3) >> 1)) ^ C::swz_v(tq)) + 4 * (t & 1);
    }

    int seq = 0;
    bool first = true;
    for (Item cur = next_item<D, kWideBM>(p, sc, seq, wave); cur.valid;
         ++seq, cur = next_item<D, kWideBM>(p, sc, seq, wave), first = false) {
        // the staging reads of the row tile before must be over before its LDS is refilled
        if (!first) __syncthreads();
        const int n = cur.n;
        if (n > 0) {
            wide_copy<D, false>(cur.kg, cur.jbase, p.Lk, dl, wave, lane, lds);
            wide_copy<D, true>(cur.vg, cur.jbase, p.Lk, dl, wave, lane, vs0);
        }
        if (n > 1) {
            wide_copy<D, false>(cur.kg, cur.jbase + kBC, p.Lk, dl, wave, lane, lds + kTile);
            wide_copy<D, true>(cur.vg, cur.jbase + kBC, p.Lk, dl, wave, lane, vs0 + kTile);
        }
        if (n > 2)
            wide_copy<D, false>(cur.kg, cur.jbase + 2 * kBC, p.Lk, dl, wave, lane, lds + 2 * kTile);
        int nvis[kWideRB];
        u32x4 qload[kWideRB][NKK];
        wide_zero_u();
#pragma unroll
        for (int rb = 0; rb < kWideRB; ++rb) {
            const int row = cur.wrow0 + 32 * rb + col;
            nvis[rb] = visible_count(p, row);
            const int qr = min(row, p.Lq - 1);
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk)
                qload[rb][kk] =
                    *reinterpret_cast<const u32x4*>(cur.qg + (size_t)qr * D + 16 * kk + 8 * hh);
            g.st[rb] = {0.0f, 1.0f, 0.0f, 0.0f};
        }
        // 32-key blocks this wavefront takes part in: those that start before its rows' last
        // visible key
        const int nbw = min(2 * n, max(0, (cur.wmax - cur.jbase + kWideKB - 1) / kWideKB));
        wait_copies();
        __syncthreads();
        // the Q fragments go to their accumulation registers
#pragma unroll
        for (int rb = 0; rb < kWideRB; ++rb)
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk) wide_set_q_n(8 * rb + kk, qload[rb][kk]);

        f32x16 acc[2][kWideRB];          // scores of block b live in acc[b % 2]
        if (nbw > 0) wide_scores<T, D>(lds, g, acc[0]);

        // Block b = 2 t + KB of the row tile by plain steps: K rows in kcur (KB = 0: the scores
        // of the tile's second half come next) or knext's first half comes next.
        auto step = [&](auto kbc, int t, const uint16_t* kcur, const uint16_t* knext,
                        const uint16_t* vcur) __attribute__((always_inline)) {
            constexpr int KB = decltype(kbc)::value;
            const int b = 2 * t + KB;
            if (b >= nbw) return;
            const int j0 = cur.jbase + b * kWideKB;
            const uint16_t* kn = KB == 0 ? kcur + kWideKB * D : knext;
            const uint16_t* vb = vcur + KB * kWideKB * D;
            if (b + 1 < nbw) wide_scores<T, D>(kn, g, acc[KB ^ 1]);
            WideCoef c;
            wide_first_general<T, D>(vb, g, acc[KB], c_log2, j0 + 4 * hh, nvis, c);
            wide_second<T, D>(vb, g, c);
        };
        // The last block a fused step can take: every key visible to every row of the
        // wavefront, and a block after it whose scores it forms.  (Block 0 never: rows are
        // still empty.)
        const int b_fused = c_log2 >= 0.0f
                                ? min((cur.wmin - cur.jbase) / kWideKB - 1, nbw - 2) : -1;
        WideAhead ah;
        bool have_ah = false;       // ah belongs to the first block of the coming period
        // Period t: start the copies of K(t + 3) and V(t + 2) into the slots of K(t - 1) and
        // V(t - 1), which were last read in period t - 1; the two blocks of tile t; wait for
        // the copies started in period t - 1 (all but this period's); barrier.
        int vslot = 0;                      // t % 3
        for (int t = 0; t < n; ++t) {
            const int vslot1 = vslot == 2 ? 0 : vslot + 1;
            const int vslot2 = vslot1 == 2 ? 0 : vslot1 + 1;
            const int j0 = cur.jbase + t * kBC;
            // this period's copies: K(t + 3) and V(t + 2).  A fused period issues them one at
            // a time from its output-product slots, K from the first block's, V from the
            // second's; whatever has not gone out that way goes out in one piece after the blocks.
            const bool kcopy = t + 3 < n, vcopy = t + 2 < n;
            // (one at a time only for tiles that lie wholly inside the keys)
            const bool kspread = kcopy && j0 + 4 * kBC <= p.Lk;
            const bool vspread = vcopy && j0 + 3 * kBC <= p.Lk;
            bool kdone = false, vdone = false;
            uint16_t* const kdst = lds + ((t + 3) & 3) * kTile;
            uint16_t* const vdst = vs0 + vslot2 * kTile;
            auto khook = [&](int i) __attribute__((always_inline)) {
                switch (i) {
                    case 0: wide_copy_one<D, false, 0>(cur.kg, j0 + 3 * kBC, dl, wave, kdst); break;
                    case 1: wide_copy_one<D, false, 1>(cur.kg, j0 + 3 * kBC, dl, wave, kdst); break;
                    case 2: wide_copy_one<D, false, 2>(cur.kg, j0 + 3 * kBC, dl, wave, kdst); break;
                    default: wide_copy_one<D, false, 3>(cur.kg, j0 + 3 * kBC, dl, wave, kdst); break;
                }
            };
            auto vhook = [&](int i) __attribute__((always_inline)) {
                switch (i) {
                    case 0: wide_copy_one<D, true, 0>(cur.vg, j0 + 2 * kBC, dl, wave, vdst); break;
                    case 1: wide_copy_one<D, true, 1>(cur.vg, j0 + 2 * kBC, dl, wave, vdst); break;
                    case 2: wide_copy_one<D, true, 2>(cur.vg, j0 + 2 * kBC, dl, wave, vdst); break;
                    default: wide_copy_one<D, true, 3>(cur.vg, j0 + 2 * kBC, dl, wave, vdst); break;
                }
            };
            auto nohook = [](int) __attribute__((always_inline)) {};
            const uint16_t* kcur = lds + (t & 3) * kTile;
            const uint16_t* knext = lds + ((t + 1) & 3) * kTile;
            const uint16_t* vcur = vs0 + vslot * kTile;
            bool done = false;
            if (__builtin_expect(t >= 1 && 2 * t + 1 <= b_fused, 1)) {
                if (!have_ah) wide_look_ahead<T, D>(kcur + kWideKB * D, g, acc[0], c_log2, ah);
                if (__builtin_expect(!ah.bail, 1)) {
                    WideCoef c;
                    wide_h1<T, D>(ah, kcur + kWideKB * D, vcur, g, acc[0], acc[1], c_log2, c);
                    if (kspread) wide_h2<T, D>(vcur, knext, g, acc[0], acc[1], c_log2, c, ah, khook);
                    else wide_h2<T, D>(vcur, knext, g, acc[0], acc[1], c_log2, c, ah, nohook);
                    kdone = kspread;
                    if (__builtin_expect(!ah.bail, 1)) {
                        wide_h1<T, D>(ah, knext, vcur + kWideKB * D, g, acc[1], acc[0], c_log2, c);
                        if (vspread)
                            wide_h2<T, D>(vcur + kWideKB * D, knext + kWideKB * D, g, acc[1], acc[0],
                                          c_log2, c, ah, vhook);
                        else
                            wide_h2<T, D>(vcur + kWideKB * D, knext + kWideKB * D, g, acc[1], acc[0],
                                          c_log2, c, ah, nohook);
                        vdone = vspread;
                        have_ah = true;
                    } else {
                        step(IntC<1>{}, t, kcur, knext, vcur);
                        have_ah = false;
                    }
                    done = true;
                }
            }
            if (__builtin_expect(!done, 0)) {
                step(IntC<0>{}, t, kcur, knext, vcur);
                step(IntC<1>{}, t, kcur, knext, vcur);
                have_ah = false;
            }
            if (kcopy && !kdone) wide_copy<D, false>(cur.kg, j0 + 3 * kBC, p.Lk, dl, wave, lane, kdst);
            if (vcopy && !vdone) wide_copy<D, true>(cur.vg, j0 + 2 * kBC, p.Lk, dl, wave, lane, vdst);
            const int started = (kcopy ? 4 : 0) + (vcopy ? 4 : 0);   // copy instructions of this period
            static_assert(DmaLane<D>::NI == 4, "the waits below count 4 copies per tile and tensor");
            if (started == 8) __builtin_amdgcn_s_waitcnt(0x0F70 | 8);       // vmcnt(8)
            else if (started == 4) __builtin_amdgcn_s_waitcnt(0x0F70 | 4);  // vmcnt(4)
            else __builtin_amdgcn_s_waitcnt(0x0F70);                        // vmcnt(0)
            // the bare barrier: __syncthreads() would first wait for every copy in flight
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            vslot = vslot1;
        }

        // ---- epilogue: o = beta U (FLASH-D) or U / l (Alg. 2), staged through LDS so that the
        // global stores are 16 bytes per lane and whole rows are contiguous.  Every wavefront
        // is past the last barrier, so all of LDS is free; a wavefront stages its 64 rows in
        // its own 64 x D elements.  Chunk c of row r sits at chunk position c ^ (r % CPR).
        uint16_t* stage = lds + wave * (64 * D);
#pragma unroll
        for (int rb = 0; rb < kWideRB; ++rb) {
            float fin = g.st[rb].beta;
            fin *= p.oscale;
            const int srow = 32 * rb + col;
#pragma unroll
            for (int i = 0; i < NDB; ++i) {
                const f32x16 u = wide_get_u_n(4 * rb + i);
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int dc = 32 * i + 8 * gq + 4 * hh;
                    f32x4 x4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x4[e] = u[4 * gq + e] * fin;
                    const u32x2 w2 = Mma<T>::pack4(x4);
                    const int chunk = (dc >> 3) ^ (srow % C::CPR);
                    *reinterpret_cast<u32x2*>(&stage[srow * D + 8 * chunk + (dc & 4)]) = w2;
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        constexpr int NST = 64 * C::CPR / 64;
#pragma unroll
        for (int h = 0; h < NST; h += 8) {
            u32x4 xs[8];
#pragma unroll
            for (int n8 = 0; n8 < 8; ++n8) {
                const int slot = (h + n8) * 64 + lane;
                const int r = slot / C::CPR;
                const int c = slot % C::CPR;
                xs[n8] = *reinterpret_cast<const u32x4*>(stage + r * D + 8 * (c ^ (r % C::CPR)));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int n8 = 0; n8 < 8; ++n8) {
                const int slot = (h + n8) * 64 + lane;
                const int r = slot / C::CPR;
                const int c = slot % C::CPR;
                if (cur.wrow0 + r < p.Lq)
                    __builtin_nontemporal_store(
                        xs[n8],
                        reinterpret_cast<u32x4*>(cur.og + (size_t)(cur.wrow0 + r) * D + 8 * c));
            }
        }
    }
}

// Calls the 256-row kernel can serve.
bool wide_applies(const Problem& p, int mode) {
    if (p.d != 128 || (p.dtype != 1 && p.dtype != 2)) return false;
    if (mode != kModeLazy) return false;
    if (p.splits != 1 || p.partial || p.merge || p.from_state || !p.store_o) return false;
    if (p.state_out != nullptr || p.kv8) return false;
    if ((int)p.Li.d != p.Lq) return false;
    return p.Lq % kWideBM == 0;
}

template <typename T, int D>
static hipError_t launch_wide_t(const Problem& p, int mode, hipStream_t st) {
    const long m_tiles = (p.Lq + kWideBM - 1) / kWideBM;
    if (m_tiles * p.B * p.Hq > 0x7fffffffL) return hipErrorInvalidValue;
    const TileSched sc = tile_sched(p, kCusPerXcd, kWideBM);
    dim3 grid((unsigned)sc.total);
    hipLaunchKernelGGL((wide_kernel<T, D, kModeLazy>), grid, dim3(kNW * 64), 0, st, p, sc);
    return hipGetLastError();
}

hipError_t launch_wide(const Problem& p, int mode, hipStream_t st) {
    if (!wide_applies(p, mode)) return hipErrorInvalidValue;
    if (p.dtype == 1) return launch_wide_t<F16, 128>(p, mode, st);
    return launch_wide_t<BF16, 128>(p, mode, st);
}

}  // namespace flashd
