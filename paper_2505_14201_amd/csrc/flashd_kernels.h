// Host-side launchers of the kernel files, called by the C-ABI layer.  Each
// checks nothing: the ABI layer has validated the problem before it gets here.
#pragma once

#include <hip/hip_runtime.h>

#include "flashd_common.h"

namespace flashd {

// Alg. 3 per key (any dtype); with p.splits > 1 also folds the partials.
hipError_t launch_perkey(const Problem& p, hipStream_t st);

// Fold p.splits partial states per query row from p.ws into p.o.
hipError_t launch_merge_splits(const Problem& p, hipStream_t st);

// How a tile of keys updates a row in the matrix-core kernels: 0 = Alg. 3 with the blend
// factor deferred (variant TILE), 1 = the Alg. 2 ablation, 2 = Alg. 3 with the blend applied
// on every tile (variant TILE_BLEND).
constexpr int kTileModeLazy = 0, kTileModeOnline = 1, kTileModeBlend = 2;
// decode kernel only: kTileModeLazy with the saturation skip of Sec. III-C on the V fetch
constexpr int kTileModeLazySkipV = 3;

// Alg. 3 on key tiles (matrix cores, f16/bf16).  With p.splits > 1 also folds the partials.
hipError_t launch_tile(const Problem& p, int mode, hipStream_t st);

// The 256-row kernel (variant TILE_256: f16/bf16, d = 128, TILE, unsplit,
// no state in or out); launch_tile hands over to it where the call asks for it and
// wide_applies() says it can serve it.
bool wide_applies(const Problem& p, int mode);
hipError_t launch_wide(const Problem& p, int mode, hipStream_t st);

// Number of workgroups launch_tile uses per split.
long tile_workgroups(int B, int Hq, int Hkv, int Lq, int d);

// Split-K decode on the matrix cores for (Hq / Hkv) * Lq <= 32 query rows per kv head
// (f16/bf16); mode as for launch_tile.  With p.splits > 1 also folds the partials.
hipError_t launch_decode(const Problem& p, int mode, hipStream_t st);
bool decode_applies(int Hq, int Hkv, int Lq);
long decode_workgroups(int B, int Hkv);

// fp8 (e4m3) K and V of `elements` elements each -> storage type `dtype` (1 f16, 2 bf16), exact.
hipError_t launch_widen_fp8(const void* k8, const void* v8, void* k, void* v, size_t elements,
                            int dtype, hipStream_t st);

// Static skip statistics of Sec. III-C: counts[0..2] = steps, steps with a score difference
// <= lo, steps with one >= hi (overwritten).  Uses p.q, p.k and the shape only.
hipError_t launch_skip_stats(const Problem& p, float lo, float hi, unsigned long long* counts,
                             hipStream_t st);

}  // namespace flashd
