// Static skip statistics of Sec. III-C (the quantity of Table I): over every query row and
// every step i >= 2 of its visible keys, how often the score difference s_i - s_{i-1} lies
// at or below `lo` (weight ~ 0: the step could be skipped) or at or above `hi` (weight ~ 1:
// the output becomes v_i).
//
// The comparison decides an integer, so the score arithmetic is fixed and kept apart from
// the matrix-core kernels: acc = fma(q[t], k[t], acc) for t = 0 .. d-1 in this order in
// fp32, s = acc * scale, diff = s_i - s_{i-1}, all single IEEE operations.
//
// Mapping: a wavefront owns a query row and walks the row's keys 64 at a time, a key per
// lane; the lane's predecessor score comes from the neighbouring lane (from lane 63 of the
// previous step for lane 0).  The query row is read as fp32 from LDS (every lane the same
// address: a broadcast).  Workgroups walk the rows grid-stride and add their three counts
// to the global counters once at the end.
#include "flashd_common.h"
#include "flashd_kernels.h"

namespace flashd {

__global__ void stats_clear_kernel(unsigned long long* counts) {
    if (threadIdx.x < 3) counts[threadIdx.x] = 0ull;
}

template <typename T, int D>
__global__ __launch_bounds__(256)
void skip_stats_kernel(Problem p, float lo, float hi, unsigned long long* counts) {
    __shared__ float qs[4][D];
    __shared__ unsigned long long part[4][3];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const long rows = (long)p.B * p.Hq * p.Lq;
    const int g = p.Hq / p.Hkv;
    unsigned long long steps = 0, low = 0, high = 0;     // this wavefront's counts (uniform)

    for (long row = (long)blockIdx.x * 4 + wave; row < rows; row += (long)gridDim.x * 4) {
        const int i = (int)(row % p.Lq);
        const long bh = row / p.Lq;
        const int h = (int)(bh % p.Hq);
        const int b = (int)(bh / p.Hq);
        const size_t qoff = (size_t)row * D;
        const size_t koff = ((size_t)b * p.Hkv + h / g) * (size_t)p.Lk * D;
        // only this wavefront touches qs[wave]; the wave barriers order its own accesses
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        for (int t = lane; t < D; t += 64) qs[wave][t] = Store<T>::load(p.q, qoff + t);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        int nvis = p.Lk;
        if (p.causal) nvis = min(max(i + p.shift + 1, 0), p.Lk);
        float carry = 0.0f;                               // score of key j0 - 1
        for (int j0 = 0; j0 < nvis; j0 += 64) {
            const int j = j0 + lane;
            const bool valid = j < nvis;
            const int jr = valid ? j : nvis - 1;          // clamped: loads stay in bounds
            float acc = 0.0f;
#pragma unroll 2
            for (int t0 = 0; t0 < D; t0 += 8) {
                float kf[8];
                Store<T>::load8(p.k, koff + (size_t)jr * D + t0, kf);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(qs[wave][t0 + e], kf[e], acc);
            }
            const float s = __fmul_rn(acc, p.scale);        // never fused with the subtraction
            float prev = __shfl_up(s, 1, 64);
            if (lane == 0) prev = carry;
            const float diff = __fsub_rn(s, prev);
            const bool step = valid && j > 0;
            steps += __builtin_popcountll(__builtin_amdgcn_ballot_w64(step));
            low += __builtin_popcountll(__builtin_amdgcn_ballot_w64(step && diff <= lo));
            high += __builtin_popcountll(__builtin_amdgcn_ballot_w64(step && diff >= hi));
            carry = __shfl(s, 63, 64);
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
    const long rows = (long)p.B * p.Hq * p.Lq;
    const long want = (rows + 3) / 4;
    const unsigned grid = (unsigned)(want < 4096 ? want : 4096);
    hipLaunchKernelGGL(stats_clear_kernel, dim3(1), dim3(64), 0, st, counts);
    hipLaunchKernelGGL((skip_stats_kernel<T, D>), dim3(grid), dim3(256), 0, st, p, lo, hi, counts);
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
