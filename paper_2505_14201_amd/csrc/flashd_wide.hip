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
//     issued together by the wavefront itself, and one block apart so that neither waits for
//     the other ("fused step", wide_step): while the vector instructions form the coefficients
//     of block b from its scores, the matrix pipe forms the scores of block b + 1 and multiplies
//     the coefficients of block b - 1 into U.  A few vector instructions follow each matrix
//     instruction; operand reads and copies are spread over the slots as well.
//   * The coefficients of a block are formed speculatively against the rows' present references
//     and used one step later, after the sum of each row's coefficients has been looked at: a
//     sum beyond LazyLimit::kMaxPsum means a score far above the row's reference, and the block
//     goes through the plain steps instead, which look at the row's top score first and move
//     the reference there if it lies more than LazyLimit::kMoveLog2 above it (the saturation of
//     Sec. III-C in tile form).  Nothing risky ever reaches U.
//   * The output accumulators, the Q fragments and the matrix operands live in fixed
//     accumulation registers that only inline assembly touches (flashd_wide_regs.h).
//
// A fused step also takes the blocks a mask applies to (a hidden key gets the score -inf where
// the scores are scaled), a wavefront's last block (the scores it forms beside it are nobody's)
// and a row tile's first (zero stands in for the rows' reference where their coefficients then
// add up to a trusted amount).  Blocks some row of which may still be empty afterwards (a row
// that sees no key of the first block), and any block under a negative scale, take the plain
// steps (wide_first_general / wide_second).
//
// Serves f16/bf16, d = 128, unsplit calls without state in or out (wide_applies()); everything
// else stays with the 128-row kernel.
#include "flashd_common.h"
#include "flashd_kernels.h"
#include "flashd_mma.h"
#include "flashd_tile_parts.h"
#include "flashd_wide_regs.h"

namespace flashd {

constexpr int kWideRB = 2;                      // 32-row blocks per wavefront
constexpr int kWideBM = 32 * kWideRB * kNW;     // query rows per workgroup
constexpr int kWideKB = 32;                     // keys per step of a wavefront (half a tile)
// The least a row's coefficients of block 0 must add up to when zero stood in for the row's
// reference (the largest of them is then at least 2^-8: far inside the range of either storage
// type, whose rounding of a coefficient is relative).
constexpr float kWideMinStart = 0.125f;

// A row's state in this kernel, the lazy form of flashd_mma.h with the blend factor kept as its
// reciprocal: o = U / l, where l = 1 / beta is the sum of 2^{s_j - R} over the keys seen so far.
// A lane holds the part of l that comes from the keys its own registers hold (the hh = 0 lane
// of a row keys 0-3, 8-11, ... of every 16, its partner the others); the two parts are added
// once, at the store.  Kept that way a fused step only adds the block's coefficients to l (no
// reciprocal, no exchange between lanes per block); the quotient is formed once per row.
struct WideRow {
    float R;      // exponent reference, log2 units
    float l;      // this lane's part of 1 / beta
    float one;    // 0.0f while the row is empty, then 1.0f
};

// (The output accumulators U and the Q fragments are not here: they live in fixed accumulation
// registers, see flashd_wide_regs.h.)
template <int D> struct WideRegs {
    int kaddr[D / 16];
    int vaddr[D / 32];
    WideRow st[kWideRB];            // FLASH-D state, lazy form
};

// The lane's index within its wavefront, formed afresh (opaque to the compiler, so that what
// is computed from it is computed where it is used).
__device__ __forceinline__ int wide_lane_id() {
    int l = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    asm volatile("" : "+v"(l));
    return l;
}

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
        // (the lane index afresh: this path is rare, and the index does not have to be kept for it)
        (void)lane;
        const int lane_now = wide_lane_id();
#pragma unroll 1
        for (int n = 0; n < NI; ++n) {
            const int inst = wave * NI + n;
            const int slot = inst * 64 + lane_now;
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
__device__ __forceinline__ void wide_read_q_n(int n, uint32_t addr) {
    switch (n) {
#define FLASHD_CASE(N) case N: wide_read_q<N>(addr); break;
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
#define FLASHD_CASE(N) case N: wide_wait_lds<N>(); break;
        FLASHD_CASES16(FLASHD_CASE)
#undef FLASHD_CASE
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
__device__ __forceinline__ void wide_copy_one(const uint16_t* src, int j0, DmaLane<D>& dl,
                                              int wave, uint16_t* dst) {
    constexpr int NI = DmaLane<D>::NI;
    static_assert(N < NI, "a tile takes NI copy instructions per wavefront");
    uint16_t* w = dst + wave * (NI * 512);
    const char* t = reinterpret_cast<const char*>(src + (size_t)j0 * D);
    // (the lane's offset is made opaque where it lives, not in a copy: the address stays a
    // scalar base plus this 32-bit register, and no instruction is spent on it)
    if (IS_V) {
        asm volatile("" : "+v"(dl.voff));
        __builtin_amdgcn_global_load_lds((gptr_t)(t + dl.voff), (lptr_t)w, 16, 1024 * N, 0);
    } else {
        asm volatile("" : "+v"(dl.koff[N]));
        __builtin_amdgcn_global_load_lds((gptr_t)(t + dl.koff[N]), (lptr_t)w, 16, 1024 * N, 0);
    }
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

// What the first half of a block's plain step leaves for the second, per row: the sum of the
// block's coefficients, the reference they were taken against, the factor what the row held was
// scaled by, and whether the row was still empty.  (The coefficients themselves go to a
// WidePacked.)
struct WideCoef {
    float psum[kWideRB], half[kWideRB], ref[kWideRB], f[kWideRB];   // half: this lane's part of psum
    bool empty[kWideRB];
};

// The coefficients of one 32-key block, rounded to the storage type, as operands of the output
// product: g0 the first 16 keys, g1 the last 16.  A fused step forms those of its block and
// multiplies those of the block before into U.
struct WidePacked {
    u32x4 g0[kWideRB], g1[kWideRB];
};

// How many operands ahead of their use the fused steps request them from LDS (the stream of a
// step's operands: K 0..7 of its score product, V 0..7 of its output product, then K 0.. of the
// next step).
#ifndef FLASHD_WIDE_LEAD
#define FLASHD_WIDE_LEAD 3
#endif
constexpr int kWideLead = FLASHD_WIDE_LEAD;
static_assert(kWideLead >= 1 && kWideLead <= 8, "the rings hold eight operands, lgkmcnt counts to 15");

// The request for the first K operands of a block on its own: a fused step expects them to be the
// last three reads issued (a fused step leaves its successor's behind; a plain step does not).
template <int D>
__device__ __forceinline__ void wide_request_first_k(const uint16_t* kb, const WideRegs<D>& g) {
#pragma unroll
    for (int kk = 0; kk < kWideLead; ++kk) wide_req_k<D>(kk, kb, g);
}

// A fused step, for an interior block b (all 32 keys visible to all rows, no row empty): three
// things at once, one block apart from each other so that none waits for another,
//   * the scores of block b + 1 (16 matrix instructions into accn; kb: its K rows in LDS),
//   * the coefficients of block b from its scores acc, by vector instructions, speculatively
//     against the rows' present references (cur),
//   * PENDING: the output product of block b - 1, U <- U + P V (16 matrix instructions; prev:
//     its coefficients, vb_prev: its V rows in LDS).
// The vector instructions follow the matrix instructions of the second half of the step, two
// keys per slot, as a pipeline of their own: the scaling of score k + 1, the exponential of
// score k, the packing of coefficient k - 1 and the summing of coefficient k - 2 do not wait for
// one another.  The operands are read from LDS into fixed registers by
// inline assembly, one operand per two slots and each six slots ahead of its use (the four
// wavefronts of the workgroup run in step, and reads issued together by all of them queue up
// in front of the LDS); K operands 0..2 were requested by the step before, and this step
// requests those of the next (kb_ahead).  The waits count the read instructions issued after
// the wanted one (a V operand takes two).
//
// Nothing this step does to block b is final before its end: the coefficients are used by the
// NEXT step, after the sum of each row's coefficients has been looked at here.  A sum beyond
// LazyLimit::kMaxPsum (or no number at all) means a score far above the row's reference: the
// step returns true, the row state is left as it was, and the caller takes block b through the
// plain steps, which move the reference (the saturation of Sec. III-C in tile form).  Otherwise
//     1/beta' = 1/beta + psum,
// which costs nothing here: the coefficients are summed straight onto the rows' l = 1 / beta.
// copy_hook(i), i = 0..3: called in slots 1, 5, 9, 13 (PENDING only: among the matrix
// instructions of the score product, away from the vector work), for the caller's global->LDS
// copies.
// MASKED: block b may be one a mask applies to.  lim[rb]: the lane's keys of the block are
// those at offsets 8 (r >> 2) + (r & 3), r = 0..15, from the key in its score register 0, and
// the ones at offsets >= lim[rb] are hidden from its row of row block rb: their score counts as
// -inf and their coefficient is 0.  (Two more vector instructions per key; no row may be empty
// as for any fused step.)
template <typename T, int D, bool PENDING, bool MASKED, typename Hook>
__device__ __forceinline__ bool wide_step(const uint16_t* kb, const uint16_t* kb_ahead,
                                          const uint16_t* vb_prev, WideRegs<D>& g,
                                          const f32x16 (&acc)[kWideRB], f32x16 (&accn)[kWideRB],
                                          float c_log2, uint32_t ones, const WidePacked& prev,
                                          WidePacked& cur, const int (&lim)[kWideRB],
                                          const Hook& copy_hook) {
    static_assert(D == 128 && kWideRB == 2, "the slots below are laid out for this shape");
    constexpr int NDB = D / 32;
    float ref[kWideRB], l[kWideRB];
#pragma unroll
    for (int rb = 0; rb < kWideRB; ++rb) {
        ref[rb] = g.st[rb].R;
        l[rb] = g.st[rb].l;
    }
    // key k of the 32: row block k & 1, score register k >> 1
    float x[33], pe[32];
    auto F = [&](int k) __attribute__((always_inline)) {
        if (k < 32) {
            x[k] = fmaf(acc[k & 1][k >> 1], c_log2, -ref[k & 1]);
            if (MASKED) {
                const int r = k >> 1;
                x[k] = (8 * (r >> 2) + (r & 3) >= lim[k & 1]) ? -__builtin_inff() : x[k];
            }
        }
    };
    auto X = [&](int k) __attribute__((always_inline)) {
        if (k < 32) pe[k] = exp2_fast(x[k]);
    };
    // pair of keys j of a row block's 8: the coefficients of score registers 2 j and 2 j + 1
    auto A = [&](int k) __attribute__((always_inline)) {        // pack
        if (k < 0 || k >= 32) return;
        const int rb = k & 1, e = k >> 1, j = e >> 1;
        if (e & 1) {
            const uint32_t w = Mma<T>::pack2(pe[k - 2], pe[k]);
            if (j < 4) cur.g0[rb][j] = w; else cur.g1[rb][j - 4] = w;
        }
    };
    auto B = [&](int k) __attribute__((always_inline)) {        // sum, an instruction later
        if (k < 0 || k >= 32) return;
        const int rb = k & 1, e = k >> 1, j = e >> 1;
        if (e & 1) {
            const uint32_t w = j < 4 ? cur.g0[rb][j] : cur.g1[rb][j - 4];
            l[rb] = Mma<T>::sum2(pe[k - 2], pe[k], w, ones, l[rb]);
        }
    };
    // key k passes through the pipeline
    auto tick = [&](int k) __attribute__((always_inline)) { F(k + 1); X(k); A(k - 1); B(k - 2); };
    // vector work of slot s
    auto valu = [&](int s) __attribute__((always_inline)) {
        if (PENDING) {
            if (s < 16 && (s & 3) == 1) copy_hook(s >> 2);
            // 32 keys through slots 15..30, two per slot, then the last coefficients.
            // (Measured: a wavefront's vector instructions do not run beside its own matrix
            // instructions whatever their order, and every change from one kind to the other
            // costs a little; one key per slot over the whole step ran 3.4 % slower than two
            // per slot from slot 14 on, all vector work in one piece between the two products
            // the same; starting at an odd slot, 11, 13 or 15, is another 3 % ahead of starting
            // at 12, 14 or 16.)
            if (s >= 15 && s < 31) { tick(2 * (s - 15)); tick(2 * (s - 15) + 1); }
            else if (s == 31) { A(31); B(30); B(31); }
        } else {
            tick(2 * s);
            tick(2 * s + 1);
        }
    };
    F(0);
    __builtin_amdgcn_sched_barrier(0);
    // The operands of this step in the order of their use: j < 8 is K operand j, then
    // (PENDING) V operand j - 8, then K operand j - 16 (or j - 8) of the next step.  A K operand
    // is one read instruction, a V operand two.
    constexpr int NOPS = PENDING ? 16 : 8;
    auto op_size = [](int j) { return (PENDING && (j % 16) >= 8) ? 2 : 1; };
    auto request = [&](int j) __attribute__((always_inline)) {
        if (j < 8) wide_req_k<D>(j, kb, g);
        else if (PENDING && j < 16) wide_req_v<D>(j - 8, vb_prev, g);
        else wide_req_k<D>(j - NOPS, kb_ahead, g);
    };
    // before operand j is used: the read instructions issued after it are those of operands
    // j + 1 .. j + kWideLead - 1
    auto wait_for = [&](int j) __attribute__((always_inline)) {
        int n = 0;
        for (int i = j + 1; i < j + kWideLead; ++i) n += op_size(i);
        wide_wait_lds_n(n);
    };
    // score product: slot s = 2 kk + rb
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        const int kk = s >> 1, rb = s & 1;
        if ((s & 1) == 0) wait_for(kk);
        ws_mma<T>(rb, kk, accn[rb]);
        if ((s & 1) == 0) request(kk + kWideLead);
        valu(s);
        __builtin_amdgcn_sched_barrier(0);
    }
    // output product of the block before: slot 16 + q, q = 2 m + rb, key group m / NDB
    if (PENDING) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int m = q >> 1, rb = q & 1;
            if ((q & 1) == 0) wait_for(8 + m);
            wp_mma<T>(rb, m, m / NDB == 0 ? prev.g0[rb] : prev.g1[rb]);
            if ((q & 1) == 0) request(8 + m + kWideLead);
            valu(16 + q);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (!PENDING) {
        A(31);
        B(30);
        B(31);
        // the scores just formed are read by vector instructions next
        mma_fence(accn);
    }
    // what the block added to this lane's part of the rows' sums: beyond the limit (or no
    // number) if any of its coefficients was
    const bool bad = !(l[0] - g.st[0].l <= LazyLimit<T>::kMaxPsum) ||
                     !(l[1] - g.st[1].l <= LazyLimit<T>::kMaxPsum);
    const bool risky = __builtin_amdgcn_ballot_w64(bad) != 0;
    if (!risky) {
#pragma unroll
        for (int rb = 0; rb < kWideRB; ++rb) g.st[rb].l = l[rb];
    }
    return risky;
}

// First half of the step of any other block (a mask applies, rows may be empty, any scale, or
// a reference has to move), by plain steps: the checked step of flashd_mma.h.  For a row the
// block's top score m is compared with the reference first; if the row is still empty or m
// lies more than LazyLimit::kMoveLog2 above R the reference moves to m, every coefficient is
// then at most 1, and what the row holds is scaled by f = 2^{R - m} (here).  jb: index of the
// key in accumulator register 0 for this lane.
template <typename T, int D>
__device__ __forceinline__ void wide_first_general(WideRegs<D>& g, const f32x16 (&acc)[kWideRB],
                                                   float c_log2, int jb,
                                                   const int (&nvis)[kWideRB], WideCoef& c,
                                                   WidePacked& out) {
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
        // (an empty row holds zeros: nothing to scale)
        if (__builtin_amdgcn_ballot_w64(c.f[rb] != 1.0f && !empty) != 0) wide_scale_u<D>(rb, c.f[rb]);
        int nv = nvis[rb];
        asm volatile("" : "+v"(nv));      // keep these compares apart from row_top_score's
        f32x4 ps = {0.0f, 0.0f, 0.0f, 0.0f};
        // 16 keys at a time, packed as they are formed
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            f32x8 pv;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int r = 8 * h + e;
                float x = fmaf(acc[rb][r], c_log2, -c.ref[rb]);
                x = ((jb + 8 * (r >> 2) + (r & 3)) >= nv) ? ninf : x;
                pv[e] = exp2_fast(x);
                ps[e & 3] += pv[e];
            }
            if (h == 0) out.g0[rb] = Mma<T>::pack8(pv); else out.g1[rb] = Mma<T>::pack8(pv);
            __builtin_amdgcn_sched_barrier(0);
        }
        c.half[rb] = (ps[0] + ps[1]) + (ps[2] + ps[3]);
        c.psum[rb] = pair_sum(c.half[rb]);
    }
}

// The output product of a block on its own, U <- U + P V over the block's 32 keys (vb: its V
// rows in LDS; b0, b1: the coefficients of its first and last 16 keys, packed).
template <typename T, int D>
__device__ __forceinline__ void wide_pv(const uint16_t* vb, const WideRegs<D>& g,
                                        const u32x4 (&b0)[kWideRB], const u32x4 (&b1)[kWideRB]) {
    constexpr int NDB = D / 32;
    constexpr int NV = 2 * NDB;
#pragma unroll
    for (int m = 0; m < NV; ++m) wide_req_v<D>(m, vb, g);
    wide_wait_lds<0>();
    // the coefficients may have been packed by vector instructions just now: two wait states
    // before the first matrix instruction reads them
    asm volatile("s_nop 1");
#pragma unroll
    for (int m = 0; m < NV; ++m)
#pragma unroll
        for (int rb = 0; rb < kWideRB; ++rb) wp_mma<T>(rb, m, m / NDB == 0 ? b0[rb] : b1[rb]);
}

// Second half of a block's step by plain steps: the update of the row state,
//     l' = f l + psum   (l = 1 / beta: the carried sum of coefficients, against the reference
//                        used; each lane of a row keeps its own part),
// and the output product.
template <typename T, int D>
__device__ __forceinline__ void wide_second(const uint16_t* vb, WideRegs<D>& g, const WideCoef& c,
                                            const WidePacked& pk) {
#pragma unroll
    for (int rb = 0; rb < kWideRB; ++rb) {
        // false only for an empty row that sees no key here (a row that is not empty has a sum
        // above zero against its reference, and the block's top score has coefficient 1 against
        // a reference that moves)
        const bool has = !c.empty[rb] || c.psum[rb] > 0.0f;
        g.st[rb].l = has ? fmaf(c.f[rb], g.st[rb].l, c.half[rb]) : g.st[rb].l;
        g.st[rb].R = has ? c.ref[rb] : g.st[rb].R;
        g.st[rb].one = has ? 1.0f : g.st[rb].one;
    }
    wide_pv<T, D>(vb, g, pk.g0, pk.g1);
}

// LDS: four K slots and four V slots, tile t in slot t % 4 of each, and a ninth slot that only
// the Q rows pass through at the start of a row tile (with three of the others).  In the period of tile t a
// wavefront forms the scores of the tile's second half and of the first half of tile t + 1, and
// the output products of the second half of tile t - 1 and the first half of tile t: it reads
// K(t), K(t + 1), V(t - 1) and V(t).  The copies of K(t + 3) and V(t + 2) are started in that
// period and those started one period earlier, K(t + 2) and V(t + 1), are waited for at its
// end: a copy has two periods to land (a period of this kernel is half as long as one of the
// 128-row kernel, and one period is less than the latency of a copy).  One workgroup barrier
// per tile.
template <typename T, int D, int MODE>
__global__ __launch_bounds__(kNW * 64, 1)
void wide_kernel(Problem p, TileSched sc) {
    using C = TileCfg<D>;
    constexpr int NKK = D / 16;
    constexpr int NDB = D / 32;
    constexpr int kTile = kBC * D;
    __shared__ __align__(1024) uint16_t lds[9 * kTile];       // K0 K1 K2 K3 V0 V1 V2 V3 X
    uint16_t* const vs0 = lds + 4 * kTile;
    // Where the Q rows of a row tile land, 64 rows (a wavefront's) per slot: the four slots that
    // the first copies of K and V do not fill (K3, V2, V3 and X, which has no other use).  Laid
    // out as a K tile, whose operand read is the read of a Q fragment (row = lane % 32, 16 bytes
    // at element 16 kk + 8 hh), and copied like one: whole rows per instruction.  (Fetched
    // straight into registers, 16 bytes per lane from 32 different rows per instruction, the
    // same bytes kept the address unit busy three times as long.)
    auto qslot = [&](int w) __attribute__((always_inline)) {
        return lds + (w == 0 ? 3 : w == 3 ? 8 : 5 + w) * kTile;
    };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31;
    const int hh = lane >> 5;
    DmaLane<D> dl(wave, lane);
    const float c_log2 = p.scale * kLog2e;
    // a pair of ones in the storage type, kept in a scalar register (not a literal in each of
    // the instructions that sum coefficients)
    uint32_t ones = Mma<T>::kOnes;
    asm volatile("" : "+s"(ones));
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
        {
            const int m0 = cur.wrow0 - 32 * kWideRB * wave;     // the row tile's first row
#pragma unroll
            for (int w = 0; w < kNW; ++w)
                wide_copy<D, false>(cur.qg, m0 + 32 * kWideRB * w, p.Lq, dl, wave, lane, qslot(w));
        }
        if (n > 0) {
            wide_copy<D, false>(cur.kg, cur.jbase, p.Lk, dl, wave, lane, lds);
            wide_copy<D, true>(cur.vg, cur.jbase, p.Lk, dl, wave, lane, vs0);
        }
        // (K of tile 1 is read in period 0 already; V of tile 1 and K of tile 2, which period 1
        // reads, follow once the Q fragments are in their registers: the row tile starts when
        // what it starts with has landed, and the copy path is the slowest part of that)
        if (n > 1) wide_copy<D, false>(cur.kg, cur.jbase + kBC, p.Lk, dl, wave, lane, lds + kTile);
        int nvis[kWideRB];
        wide_zero_u();
        // (the lane index afresh, here and in the epilogue: what is formed from it then does
        // not sit in registers across the tile loop)
        const int lane_q = wide_lane_id();
#pragma unroll
        for (int rb = 0; rb < kWideRB; ++rb) {
            // rows past the end stand in for the last row (the same arithmetic on the same
            // numbers; nothing of them is stored)
            const int row = min(cur.wrow0 + 32 * rb + (lane_q & 31), p.Lq - 1);
            nvis[rb] = visible_count(p, row);
            g.st[rb] = {0.0f, 0.0f, 0.0f};
        }
        // 32-key blocks this wavefront takes part in: those that start before its rows' last
        // visible key
        const int nbw = min(2 * n, max(0, (cur.wmax - cur.jbase + kWideKB - 1) / kWideKB));
        wait_copies();
        __syncthreads();
        // the Q fragments go to their accumulation registers; once every wavefront has read
        // its own, the slots they came from are free for the copies of the first period
        // (the slot's address is made opaque here, so that the sixteen addresses below are
        // formed here and not kept in registers from the start of the kernel on)
        uint32_t qbase = lds_byte_address(qslot(wave));
        asm volatile("" : "+v"(qbase));
#pragma unroll
        for (int rb = 0; rb < kWideRB; ++rb)
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk)
                wide_read_q_n(8 * rb + kk, qbase + 2u * (uint32_t)(g.kaddr[kk] + 32 * rb * D));
        wide_wait_lds<0>();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (n > 1) wide_copy<D, true>(cur.vg, cur.jbase + kBC, p.Lk, dl, wave, lane, vs0 + kTile);
        if (n > 2)
            wide_copy<D, false>(cur.kg, cur.jbase + 2 * kBC, p.Lk, dl, wave, lane, lds + 2 * kTile);

        f32x16 acc[2][kWideRB];          // scores of block b live in acc[b % 2]
        WidePacked pk[2];                // coefficients of block b (a fused step's) in pk[b % 2]
        if (nbw > 0) wide_scores<T, D>(lds, g, acc[0]);

        // The last block a fused step can take: the wavefront's last (the scores the step forms
        // beside it are then those of a block the wavefront has no part in, or of whatever the
        // next K slot holds, and nobody reads them; that costs less than a second kind of step
        // would cost the others in registers and code).  Blocks a mask applies to included, as
        // long as no row is still empty: not if some row of the wavefront sees no key in block 0
        // (nor under a negative scale).  Block 0 as well, with zero standing in for the rows'
        // reference: good if every row's coefficients then add up to something between
        // kWideMinStart and the limit of any fused step, else the plain steps take the block.
        const int nolim[kWideRB] = {64, 64};
        int wmin = cur.wmin;        // keys every row of the wavefront sees
        if (cur.wrow0 < p.Lq && cur.wrow0 + 32 * kWideRB > p.Lq) {
            // the wavefront's rows run past the end: those that exist decide
            int most;
            visible_range(p, cur.wrow0, p.Lq - 1, most, wmin);
        }
        const int b_nomask = (wmin - cur.jbase) / kWideKB - 1;    // the last block without a mask
        const int b_fused = (c_log2 >= 0.0f && wmin > cur.jbase) ? nbw - 1 : -1;
        bool pending = false;       // the output product of the block before is still to come
        bool k_ahead = false;       // K operands 0..2 of the next score product are on their way
        // Tile t sits in K slot t % 4 and V slot t % 4.  Period t: start the copies of K(t + 3)
        // and V(t + 2) into the slots of K(t - 1) and V(t - 2), which were last read in period
        // t - 1; the two blocks of tile t; wait for the copies started in period t - 1 (all but
        // this period's); barrier.
        int t = 0;
        auto kslot = [&](int i) __attribute__((always_inline)) { return lds + ((t + i) & 3) * kTile; };
        auto vslot = [&](int i) __attribute__((always_inline)) { return vs0 + ((t + i) & 3) * kTile; };
        auto khook = [&](int i) __attribute__((always_inline)) {
            const int j3 = cur.jbase + (t + 3) * kBC;
            switch (i) {
                case 0: wide_copy_one<D, false, 0>(cur.kg, j3, dl, wave, kslot(3)); break;
                case 1: wide_copy_one<D, false, 1>(cur.kg, j3, dl, wave, kslot(3)); break;
                case 2: wide_copy_one<D, false, 2>(cur.kg, j3, dl, wave, kslot(3)); break;
                default: wide_copy_one<D, false, 3>(cur.kg, j3, dl, wave, kslot(3)); break;
            }
        };
        auto vhook = [&](int i) __attribute__((always_inline)) {
            const int j2 = cur.jbase + (t + 2) * kBC;
            switch (i) {
                case 0: wide_copy_one<D, true, 0>(cur.vg, j2, dl, wave, vslot(2)); break;
                case 1: wide_copy_one<D, true, 1>(cur.vg, j2, dl, wave, vslot(2)); break;
                case 2: wide_copy_one<D, true, 2>(cur.vg, j2, dl, wave, vslot(2)); break;
                default: wide_copy_one<D, true, 3>(cur.vg, j2, dl, wave, vslot(2)); break;
            }
        };
        auto nohook = [](int) __attribute__((always_inline)) {};
        // The last period both of whose blocks fused steps can take while its copies (both
        // there, both of tiles that lie wholly inside the keys) go out one at a time.
        const int t_hi = min(min(min((b_fused - 1) >> 1, (b_nomask - 1) >> 1), n - 4),
                             (p.Lk - cur.jbase) / kBC - 4);
        // 0: nothing of period t is done; 1: a fused step found block 2 t risky (the scores of
        // the next block are there, the K copies are out); 2: the same for block 2 t + 1 (both
        // copies are out)
        int resume = 0;
        while (t < n) {
            // ---- the common case as a loop of its own: periods both of whose blocks are
            // taken by fused steps that find nothing risky
            if (pending) {
                while (t <= t_hi) {
                    if (__builtin_expect(wide_step<T, D, true, false>(
                                             kslot(0) + kWideKB * D, kslot(1),
                                             vslot(3) + kWideKB * D, g, acc[0], acc[1], c_log2,
                                             ones, pk[1], pk[0], nolim, khook), 0)) {
                        resume = 1;
                        break;
                    }
                    if (__builtin_expect(wide_step<T, D, true, false>(
                                             kslot(1), kslot(1) + kWideKB * D, vslot(0), g, acc[1],
                                             acc[0], c_log2, ones, pk[0], pk[1], nolim, vhook), 0)) {
                        resume = 2;
                        break;
                    }
                    __builtin_amdgcn_s_waitcnt(0x0F70 | 8);       // vmcnt(8)
                    asm volatile("" ::: "memory");
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                    ++t;
                }
                if (t >= n) break;
            }
            // ---- any other period
            const int j0 = cur.jbase + t * kBC;
            // this period's copies: K(t + 3) and V(t + 2), in one piece after the blocks
            const bool kcopy = t + 3 < n, vcopy = t + 2 < n;
            const uint16_t* kcur = kslot(0);
            const uint16_t* knext = kslot(1);
            const uint16_t* vcur = vslot(0);
            const uint16_t* vprev = vslot(3);
            // Block b = 2 t + KB by plain steps (have_next: the scores of block b + 1 are there
            // already, a fused step that found block b risky has formed them).
            auto plain = [&](auto kbc, bool have_next) __attribute__((always_inline)) {
                constexpr int KB = decltype(kbc)::value;
                const int b = 2 * t + KB;
                const uint16_t* kn = KB == 0 ? kcur + kWideKB * D : knext;
                const uint16_t* vb = vcur + KB * kWideKB * D;
                const int jb = cur.jbase + b * kWideKB;
                if (!have_next && b + 1 < nbw) wide_scores<T, D>(kn, g, acc[KB ^ 1]);
                WideCoef c;
                wide_first_general<T, D>(g, acc[KB], c_log2, jb + 4 * hh, nvis, c, pk[KB]);
                wide_second<T, D>(vb, g, c, pk[KB]);
                k_ahead = false;
            };
            // Block b = 2 t + KB of the row tile.  K rows of block b + 1 in kn, of block b + 2
            // in ka; V rows of block b - 1 in vp.
            auto block = [&](auto kbc) __attribute__((always_inline)) {
                constexpr int KB = decltype(kbc)::value;
                const int b = 2 * t + KB;
                const uint16_t* kn = KB == 0 ? kcur + kWideKB * D : knext;
                const uint16_t* ka = KB == 0 ? knext : knext + kWideKB * D;
                const uint16_t* vp = KB == 0 ? vprev + kWideKB * D : vcur;
                if (b >= nbw) {
                    // past the wavefront's last block: that one's output product, if a fused
                    // step has left it
                    if (pending) wide_pv<T, D>(vp, g, pk[KB ^ 1].g0, pk[KB ^ 1].g1);
                    pending = false;
                    return;
                }
                bool have_next = false;
                if (b <= b_fused) {
                    bool risky;
                    // offsets from the key in the lane's score register 0 at which its rows'
                    // hidden keys begin (none: 64)
                    int lim[kWideRB];
#pragma unroll
                    for (int rb = 0; rb < kWideRB; ++rb)
                        lim[rb] = b > b_nomask ? nvis[rb] - (cur.jbase + b * kWideKB + 4 * hh) : 64;
                    if (pending) {
                        risky = wide_step<T, D, true, true>(kn, ka, vp, g, acc[KB], acc[KB ^ 1],
                                                            c_log2, ones, pk[KB ^ 1], pk[KB], lim,
                                                            nohook);
                    } else {
                        if (!k_ahead) wide_request_first_k<D>(kn, g);
                        risky = wide_step<T, D, false, true>(kn, ka, vp, g, acc[KB], acc[KB ^ 1],
                                                             c_log2, ones, pk[KB ^ 1], pk[KB], lim,
                                                             nohook);
                    }
                    if (b == 0 && !risky) {
                        // the rows were empty and zero was their reference
                        bool low = false;
#pragma unroll
                        for (int rb = 0; rb < kWideRB; ++rb)
                            low = low || !(pair_sum(g.st[rb].l) >= kWideMinStart);
                        risky = __builtin_amdgcn_ballot_w64(low) != 0;
#pragma unroll
                        for (int rb = 0; rb < kWideRB; ++rb) {
                            g.st[rb].l = risky ? 0.0f : g.st[rb].l;
                            g.st[rb].one = risky ? 0.0f : 1.0f;
                        }
                    }
                    k_ahead = true;
                    have_next = true;
                    pending = !risky;
                    if (!risky) return;
                } else if (pending) {
                    wide_pv<T, D>(vp, g, pk[KB ^ 1].g0, pk[KB ^ 1].g1);
                    pending = false;
                }
                plain(kbc, have_next);
            };
            bool kdone = false, vdone = false;
            if (resume == 1) {
                pending = false;
                plain(IntC<0>{}, true);
                block(IntC<1>{});
                kdone = true;
            } else if (resume == 2) {
                pending = false;
                plain(IntC<1>{}, true);
                kdone = vdone = true;
            } else {
                block(IntC<0>{});
                block(IntC<1>{});
            }
            resume = 0;
            if (kcopy && !kdone)
                wide_copy<D, false>(cur.kg, j0 + 3 * kBC, p.Lk, dl, wave, lane, lds + ((t + 3) & 3) * kTile);
            if (vcopy && !vdone)
                wide_copy<D, true>(cur.vg, j0 + 2 * kBC, p.Lk, dl, wave, lane, vs0 + ((t + 2) & 3) * kTile);
            const int started = (kcopy ? 4 : 0) + (vcopy ? 4 : 0);   // copy instructions of this period
            static_assert(DmaLane<D>::NI == 4, "the waits below count 4 copies per tile and tensor");
            if (started == 8) __builtin_amdgcn_s_waitcnt(0x0F70 | 8);       // vmcnt(8)
            else if (started == 4) __builtin_amdgcn_s_waitcnt(0x0F70 | 4);  // vmcnt(4)
            else __builtin_amdgcn_s_waitcnt(0x0F70);                        // vmcnt(0)
            // the bare barrier: __syncthreads() would first wait for every copy in flight
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            ++t;
        }
        // the output product of the row tile's last block, if a fused step has left it
        if (pending) wide_pv<T, D>(vs0 + ((n - 1) & 3) * kTile + kWideKB * D, g, pk[1].g0, pk[1].g1);

        // ---- epilogue: o = U / l, staged through LDS so that the global stores are 16 bytes per
        // lane and cover whole 128-byte lines.  In four passes per wavefront, a row block's 32
        // rows by 64 columns each, so that the stores of one pass drain while the vector
        // instructions of the next scale and round (all in one piece, the 64 stores of a
        // wavefront came after 400 vector instructions and each kind waited for the other).
        // Every wavefront is past the last barrier and nobody reads K any more: a wavefront
        // stages in its own 4 KB of K slot 0.  Chunk c of row r sits at chunk position
        // c ^ ((r / 2) % 8) of the row's 128 bytes.
        uint16_t* stage = lds + wave * (32 * 64);
        const int lane_e = wide_lane_id();
        const int col_e = lane_e & 31, hh_e = lane_e >> 5;
        float fin[kWideRB];
#pragma unroll
        for (int rb = 0; rb < kWideRB; ++rb) {
            // beta = 1 / l, the two lanes' parts added; a row that saw no key stores zeros
            const float lrow = pair_sum(g.st[rb].l);
            fin[rb] = lrow > 0.0f ? p.oscale * __builtin_amdgcn_rcpf(lrow) : 0.0f;
        }
#pragma unroll
        for (int pass = 0; pass < 2 * kWideRB; ++pass) {
            const int rb = pass >> 1, hf = pass & 1;
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
                const f32x16 u = wide_get_u_n(4 * rb + 2 * hf + ii);
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int dc = 32 * ii + 8 * gq + 4 * hh_e;        // column within the pass's 64
                    f32x4 x4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x4[e] = u[4 * gq + e] * fin[rb];
                    const u32x2 w2 = Mma<T>::pack4(x4);
                    const int chunk = (dc >> 3) ^ ((col_e >> 1) & 7);
                    *reinterpret_cast<u32x2*>(&stage[col_e * 64 + 8 * chunk + (dc & 4)]) = w2;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            u32x4 xs[4];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const int slot = h * 64 + lane_e;
                const int r = slot >> 3, c = slot & 7;
                xs[h] = *reinterpret_cast<const u32x4*>(stage + r * 64 + 8 * (c ^ ((r >> 1) & 7)));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const int slot = h * 64 + lane_e;
                const int r = 32 * rb + (slot >> 3), c = slot & 7;
                if (cur.wrow0 + r < p.Lq)
                    __builtin_nontemporal_store(
                        xs[h], reinterpret_cast<u32x4*>(cur.og + (size_t)(cur.wrow0 + r) * D +
                                                        64 * hf + 8 * c));
            }
            // (the next pass writes where this one has read: one wavefront's LDS accesses are
            // served in the order it issued them)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

// Calls the 256-row kernel can serve.
bool wide_applies(const Problem& p, int mode) {
    if (p.d != 128 || (p.dtype != 1 && p.dtype != 2)) return false;
    if (mode != kModeLazy) return false;
    if (p.splits != 1 || p.partial || p.merge || p.from_state || !p.store_o) return false;
    if (p.state_out != nullptr || p.kv8) return false;
    return (int)p.Li.d == p.Lq;
}

template <typename T, int D>
static hipError_t launch_wide_t(const Problem& p, hipStream_t st) {
    const long m_tiles = (p.Lq + kWideBM - 1) / kWideBM;
    if (m_tiles * p.B * p.Hq > 0x7fffffffL) return hipErrorInvalidValue;
    const TileSched sc = tile_sched(p, kCusPerXcd, kWideBM);
    dim3 grid((unsigned)sc.total);
    hipLaunchKernelGGL((wide_kernel<T, D, kModeLazy>), grid, dim3(kNW * 64), 0, st, p, sc);
    return hipGetLastError();
}

hipError_t launch_wide(const Problem& p, int mode, hipStream_t st) {
    if (!wide_applies(p, mode)) return hipErrorInvalidValue;
    if (p.dtype == 1) return launch_wide_t<F16, 128>(p, st);
    return launch_wide_t<BF16, 128>(p, st);
}

}  // namespace flashd
