// Static skip statistics of Sec. III-C (the quantity of Table I): over every query row and
// every step i >= 2 of its visible keys, how often the score difference s_i - s_{i-1} lies
// at or below `lo` (weight ~ 0: the step could be skipped) or at or above `hi` (weight ~ 1:
// the output becomes v_i).
//
// The comparison decides an integer, so the score arithmetic is fixed and kept apart from
// the matrix-core kernels: acc = fma(q[t], k[t], acc) for t = 0 .. d-1 in this order in
// fp32, s = acc * scale, diff = s_i - s_{i-1}, all single IEEE operations.
//
// Mapping: a wavefront owns kStatRows consecutive query rows of one head and walks their
// keys 64 at a time, a key per lane, so that a key row is fetched once for all of them; the
// lane's predecessor score comes from the neighbouring lane (from lane 63 of the previous
// step for lane 0).  The query rows are read as fp32 from LDS (every lane the same address:
// a broadcast).  16-bit storage: the four wavefronts of a workgroup take 16 consecutive query
// rows and share the key tiles, which are copied global->LDS with coalesced 16-byte chunks
// (double-buffered, chunk c of key r at position c ^ swz(r)) and read back a key per lane;
// read straight from global memory, a key per lane touches 64 cache lines per load
// instruction and the address unit, not the arithmetic, sets the pace (fp32 storage, which
// only the small configuration uses, still does that).  Workgroups walk the row groups
// grid-stride and add their three counts to the global counters once at the end.
#include "flashd_common.h"
#include "flashd_kernels.h"

#include <type_traits>

namespace flashd {

__global__ void stats_clear_kernel(unsigned long long* counts) {
    if (threadIdx.x < 3) counts[threadIdx.x] = 0ull;
}

constexpr int kStatRows = 4;      // query rows per wavefront

template <typename T, int D>
__global__ __launch_bounds__(256)
void skip_stats_kernel(Problem p, float lo, float hi, unsigned long long* counts) {
    constexpr int R = kStatRows;
    __shared__ __align__(16) float qs[4][R][D];
    __shared__ unsigned long long part[4][3];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int g = p.Hq / p.Hkv;
    const long groups_per_head = (p.Lq + R - 1) / R;
    const long groups = (long)p.B * p.Hq * groups_per_head;
    unsigned long long steps = 0, low = 0, high = 0;     // this wavefront's counts (uniform)

    for (long grp = (long)blockIdx.x * 4 + wave; grp < groups; grp += (long)gridDim.x * 4) {
        const int i0 = (int)(grp % groups_per_head) * R;
        const long bh = grp / groups_per_head;
        const int h = (int)(bh % p.Hq);
        const int b = (int)(bh / p.Hq);
        const size_t qoff = (((size_t)b * p.Hq + h) * p.Lq + i0) * (size_t)D;
        const size_t koff = ((size_t)b * p.Hkv + h / g) * (size_t)p.Lk * D;
        // only this wavefront touches qs[wave]; the wave barriers order its own accesses
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        int nvis[R];
        int nmax = 0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int i = i0 + r;
            const bool ok = i < p.Lq;
            for (int t = lane; t < D; t += 64)
                qs[wave][r][t] = ok ? Store<T>::load(p.q, qoff + (size_t)r * D + t) : 0.0f;
            int n = p.Lk;
            if (p.causal) n = min(max(i + p.shift + 1, 0), p.Lk);
            nvis[r] = ok ? n : 0;
            nmax = max(nmax, nvis[r]);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        float carry[R];                                   // score of key j0 - 1, per row
#pragma unroll
        for (int r = 0; r < R; ++r) carry[r] = 0.0f;
        for (int j0 = 0; j0 < nmax; j0 += 64) {
            const int j = j0 + lane;
            const int jr = min(j, nmax - 1);              // clamped: loads stay in bounds
            float acc[R];
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r] = 0.0f;
#pragma unroll 2
            for (int t0 = 0; t0 < D; t0 += 8) {
                float kf[8];
                Store<T>::load8(p.k, koff + (size_t)jr * D + t0, kf);
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        acc[r] = __builtin_fmaf(qs[wave][r][t0 + e], kf[e], acc[r]);
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float s = __fmul_rn(acc[r], p.scale);    // never fused with the subtraction
                float prev = __shfl_up(s, 1, 64);
                if (lane == 0) prev = carry[r];
                const float diff = __fsub_rn(s, prev);
                const bool step = j < nvis[r] && j > 0;
                steps += __builtin_popcountll(__builtin_amdgcn_ballot_w64(step));
                low += __builtin_popcountll(__builtin_amdgcn_ballot_w64(step && diff <= lo));
                high += __builtin_popcountll(__builtin_amdgcn_ballot_w64(step && diff >= hi));
                carry[r] = __shfl(s, 63, 64);
            }
        }
    }
    if (lane == 0) { part[wave][0] = steps; part[wave][1] = low; part[wave][2] = high; }
    __syncthreads();
    if (threadIdx.x < 3) {
        const unsigned long long sum = part[0][threadIdx.x] + part[1][threadIdx.x] +
                                       part[2][threadIdx.x] + part[3][threadIdx.x];
        if (sum) atomicAdd(&counts[threadIdx.x], sum);
    }
}

typedef const __attribute__((address_space(1))) void* stat_gptr_t;
typedef __attribute__((address_space(3))) void* stat_lptr_t;

// 16-bit storage: key tiles staged through LDS and shared by the workgroup's 4 x kStatRows rows
template <typename T, int D>
__global__ __launch_bounds__(256)
void skip_stats_tiled_kernel(Problem p, float lo, float hi, unsigned long long* counts) {
    constexpr int R = kStatRows;
    constexpr int CPR = D / 8;                 // 16-byte chunks per key row
    constexpr int NI = CPR / 4;                // copy instructions per wavefront and tile
    constexpr int kTileEl = 64 * D;            // elements of a 64-key tile
    __shared__ __align__(1024) uint16_t kt[2][kTileEl];
    __shared__ __align__(16) float qs[4][R][D];
    __shared__ unsigned long long part[4][3];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = p.Hq / p.Hkv;
    const long groups_per_head = (p.Lq + 4 * R - 1) / (4 * R);
    const long groups = (long)p.B * p.Hq * groups_per_head;
    unsigned long long steps = 0, low = 0, high = 0;     // this wavefront's counts (uniform)
    // chunk c of key r sits at position c ^ swz(r): a key per lane then reads conflict-free
    auto swz = [](int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); };

    for (long grp = blockIdx.x; grp < groups; grp += gridDim.x) {
        const int i0 = (int)(grp % groups_per_head) * (4 * R) + wave * R;   // this wavefront's rows
        const long bh = grp / groups_per_head;
        const int h = (int)(bh % p.Hq);
        const int b = (int)(bh / p.Hq);
        const size_t qoff = (((size_t)b * p.Hq + h) * p.Lq + i0) * (size_t)D;
        const uint16_t* kg = static_cast<const uint16_t*>(p.k) +
                             ((size_t)b * p.Hkv + h / g) * (size_t)p.Lk * D;
        // keys that the last row of the workgroup's 16 sees: the tiles all four wavefronts walk
        const int ilast = min((int)(grp % groups_per_head) * (4 * R) + 4 * R - 1, p.Lq - 1);
        const int nwg = p.causal ? min(max(ilast + p.shift + 1, 0), p.Lk) : p.Lk;
        // everybody is done with the previous group's tiles and query rows
        __syncthreads();
        int nvis[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int i = i0 + r;
            const bool ok = i < p.Lq;
            for (int t = lane; t < D; t += 64)
                qs[wave][r][t] = ok ? Store<T>::load(p.q, qoff + (size_t)r * D + t) : 0.0f;
            int n = p.Lk;
            if (p.causal) n = min(max(i + p.shift + 1, 0), p.Lk);
            nvis[r] = ok ? n : 0;
        }
        // this wavefront's share of the copy of the tile that starts at key j0 (rows past the
        // last key are clamped to it; they are never counted)
        auto copy_tile = [&](int j0, uint16_t* dst) {
#pragma unroll
            for (int n = 0; n < NI; ++n) {
                const int inst = wave * NI + n;
                const int slot = inst * 64 + lane;
                const int row = slot / CPR;
                const int cs = slot % CPR;
                const size_t grow = (size_t)min(j0 + row, p.Lk - 1) * D;
                __builtin_amdgcn_global_load_lds((stat_gptr_t)(kg + grow + 8 * (cs ^ swz(row))),
                                                 (stat_lptr_t)(dst + inst * 512), 16, 0, 0);
            }
        };
        if (nwg > 0) copy_tile(0, kt[0]);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();

        float carry[R];                                   // score of key j0 - 1, per row
#pragma unroll
        for (int r = 0; r < R; ++r) carry[r] = 0.0f;
        int buf = 0;
        for (int j0 = 0; j0 < nwg; j0 += 64, buf ^= 1) {
            if (j0 + 64 < nwg) copy_tile(j0 + 64, kt[buf ^ 1]);
            const int j = j0 + lane;
            const uint16_t* krow = kt[buf] + lane * D;
            float acc[R];
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r] = 0.0f;
#pragma unroll 2
            for (int c = 0; c < CPR; ++c) {
                float kf[8];
                Store<T>::load8(krow, (size_t)(8 * (c ^ swz(lane))), kf);
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        acc[r] = __builtin_fmaf(qs[wave][r][8 * c + e], kf[e], acc[r]);
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float s = __fmul_rn(acc[r], p.scale);    // never fused with the subtraction
                float prev = __shfl_up(s, 1, 64);
                if (lane == 0) prev = carry[r];
                const float diff = __fsub_rn(s, prev);
                const bool step = j < nvis[r] && j > 0;
                steps += __builtin_popcountll(__builtin_amdgcn_ballot_w64(step));
                low += __builtin_popcountll(__builtin_amdgcn_ballot_w64(step && diff <= lo));
                high += __builtin_popcountll(__builtin_amdgcn_ballot_w64(step && diff >= hi));
                carry[r] = __shfl(s, 63, 64);
            }
            // the next tile has landed and this one is free for the copy after it
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
    }
    if (lane == 0) { part[wave][0] = steps; part[wave][1] = low; part[wave][2] = high; }
    __syncthreads();
    if (threadIdx.x < 3) {
        const unsigned long long sum = part[0][threadIdx.x] + part[1][threadIdx.x] +
                                       part[2][threadIdx.x] + part[3][threadIdx.x];
        if (sum) atomicAdd(&counts[threadIdx.x], sum);
    }
}

template <typename T, int D>
static hipError_t launch_stats_t(const Problem& p, float lo, float hi, unsigned long long* counts,
                                 hipStream_t st) {
    const long groups = (long)p.B * p.Hq * ((p.Lq + kStatRows - 1) / kStatRows);
    const long want = (groups + 3) / 4;
    const unsigned grid = (unsigned)(want < 4096 ? want : 4096);
    hipLaunchKernelGGL(stats_clear_kernel, dim3(1), dim3(64), 0, st, counts);
    if constexpr (std::is_same<T, F32>::value) {
        hipLaunchKernelGGL((skip_stats_kernel<T, D>), dim3(grid), dim3(256), 0, st, p, lo, hi,
                           counts);
    } else {
        const long tgroups = (long)p.B * p.Hq * ((p.Lq + 4 * kStatRows - 1) / (4 * kStatRows));
        const unsigned tgrid = (unsigned)(tgroups < 8192 ? tgroups : 8192);
        hipLaunchKernelGGL((skip_stats_tiled_kernel<T, D>), dim3(tgrid), dim3(256), 0, st, p, lo,
                           hi, counts);
    }
    return hipGetLastError();
}

hipError_t launch_skip_stats(const Problem& p, float lo, float hi, unsigned long long* counts,
                             hipStream_t st) {
    if (p.d == 64) {
        if (p.dtype == 0) return launch_stats_t<F32, 64>(p, lo, hi, counts, st);
        if (p.dtype == 1) return launch_stats_t<F16, 64>(p, lo, hi, counts, st);
        if (p.dtype == 2) return launch_stats_t<BF16, 64>(p, lo, hi, counts, st);
    } else if (p.d == 128) {
        if (p.dtype == 0) return launch_stats_t<F32, 128>(p, lo, hi, counts, st);
        if (p.dtype == 1) return launch_stats_t<F16, 128>(p, lo, hi, counts, st);
        if (p.dtype == 2) return launch_stats_t<BF16, 128>(p, lo, hi, counts, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace flashd
