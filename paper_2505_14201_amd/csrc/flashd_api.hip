// The C ABI of libflashd: argument validation, variant/split selection, the
// per-(device, stream) workspace cache, and dispatch to the kernel launchers.
#include <hip/hip_runtime.h>

#include <cstring>
#include <map>
#include <mutex>
#include <utility>
#include <vector>

#include "../../include/flashd.h"
#include "flashd_common.h"
#include "flashd_kernels.h"

namespace {

using flashd::Problem;

struct Shape { int B, Hq, Hkv, Lq, Lk, d, dtype; };

int validate_shape(const Shape& s) {
    if (s.B < 1 || s.Hq < 1 || s.Hkv < 1 || s.Lq < 1 || s.Lk < 1) return FLASHD_E_SHAPE;
    if (s.B > 65535 || s.Hq > 65535) return FLASHD_E_SHAPE;          // grid y/z limits
    // row and key indices, and their sums with the causal shift, are 32-bit in the kernels
    if (s.Lq > 1000000000 || s.Lk > 1000000000) return FLASHD_E_SHAPE;
    if (s.dtype != FLASHD_F32 && s.dtype != FLASHD_F16 && s.dtype != FLASHD_BF16)
        return FLASHD_E_DTYPE;
    if (s.d != 64 && s.d != 128) return FLASHD_E_HEADDIM;
    if (s.Hq % s.Hkv != 0) return FLASHD_E_GQA;
    // element counts must fit 2^40 so every byte offset fits size_t with room to spare
    const long double nq = (long double)s.B * s.Hq * s.Lq * s.d;
    const long double nk = (long double)s.B * s.Hkv * s.Lk * s.d;
    if (nq > 1.0e12L || nk > 1.0e12L) return FLASHD_E_SHAPE;
    return FLASHD_OK;
}

// Where the automatic choice takes the 256-row prefill kernel (measured against the 128-row
// kernel over batch sizes, head counts and lengths): it needs a workgroup per compute unit to
// be busy at all (256 of them; twice that under a causal mask, whose row tiles differ in
// length and run in pairs), and row tiles long enough to outweigh what it pays at every change
// of row tile with only one workgroup on the compute unit (about 8 us, four to five periods of
// 64 keys): 1536 keys without a mask (+ 8 % at 1536 and 2048, + 12 to 16 % from 4096 on; level
// at 1024), and under a causal mask rows that see 1536 keys on average, Lk - Lq / 2 (+ 6 % at
// 3072 x 3072, + 8 to 10 % at 4096, + 14 to 16 % from 8192 on and at 1000 x 3000; 0.90 at
// 1024).  Rows that see 1024 keys on average (2048 x 2048) are taken where the pairs of row
// tiles fill a whole number of rounds of the 256 compute units (+ 1 to 3 % then; 3 to 6 %
// behind otherwise, with compute units idle in the last round).  The kernel itself says
// which calls it can serve at all (wide_applies()).
bool prefers_256_rows(const Shape& s, bool causal) {
    if (s.d != 128 || s.dtype == FLASHD_F32) return false;
    const long wgs = (long)s.B * s.Hq * ((s.Lq + 255) / 256);
    if (!causal) return wgs >= 256 && s.Lk >= 1536;
    const long seen = (long)s.Lk - s.Lq / 2;        // keys a row sees on average
    const bool whole_rounds = s.Lq % 512 == 0 && (wgs / 2) % 256 == 0;
    return wgs >= 512 && (seen >= 1536 || (seen >= 1024 && whole_rounds));
}

int resolve_variant(const Shape& s, int variant) {
    if (variant < FLASHD_VARIANT_AUTO || variant > FLASHD_VARIANT_TILE_256) return -1;
    if (variant == FLASHD_VARIANT_AUTO)
        return s.dtype == FLASHD_F32 ? FLASHD_VARIANT_PER_KEY : FLASHD_VARIANT_TILE;
    if (s.dtype == FLASHD_F32 && variant != FLASHD_VARIANT_PER_KEY) return -1;
    return variant;
}

int ceil_div(long a, long b) { return (int)((a + b - 1) / b); }

// n partial states (o[d], s, ln w) per query row
size_t partial_bytes(const Shape& s, int n) {
    return (size_t)n * s.B * s.Hq * s.Lq * (size_t)(s.d + 2) * sizeof(float);
}

// Splits for the automatic choice: enough independent work to fill 256 compute units, but
// never key ranges shorter than 256 keys.
int auto_splits(const Shape& s, int variant) {
    long units;
    if (variant == FLASHD_VARIANT_PER_KEY) {
        const int rows_per_group = (s.d <= 64 ? 2 : 1) * 4;             // 4 wavefronts
        units = (long)s.B * s.Hq * ceil_div(s.Lq, rows_per_group);      // workgroups
    } else if (flashd::decode_applies(s.Hq, s.Hkv, s.Lq)) {
        units = flashd::decode_workgroups(s.B, s.Hkv);
    } else {
        units = flashd::tile_workgroups(s.B, s.Hq, s.Hkv, s.Lq, s.d);
    }
    // Two workgroups are resident per compute unit (512 in all), and one full round of them
    // is what the matrix-core kernels want: measured over decode, short-query and prefill
    // shapes of 64 to 512 units, the fastest split count is the one that brings the launch
    // to 256-512 workgroups; more of them only add partial states to write and merge.  The
    // per-key kernel keeps two rounds.
    const long target = variant == FLASHD_VARIANT_PER_KEY ? 1024 : 512;
    if (units < 1) units = 1;
    long sp = units >= target ? 1 : ceil_div(target, units);
    // A split costs its partial states: (d + 2) floats per query row written and read back.
    // With one row per head (decode) that is nothing and 256 keys are enough to pay for a
    // split; the tile kernel's workgroups carry 128 rows each, and measured over prefill
    // shapes a split only pays once it still holds some 2048 keys (B1 H32 L1024 causal:
    // 23 us unsplit, 39 us in two splits of 512 keys).
    // With few query rows in all (short queries that do not fit the decode kernel: 4 x 8
    // heads x 8 positions over 4096 keys runs 15 us in 16 splits, 45 us in 2) the partial
    // states are small again: splits of 256 keys are allowed as long as all the partial
    // states together stay within some 40 MB.
    const bool tile = variant != FLASHD_VARIANT_PER_KEY &&
                      !flashd::decode_applies(s.Hq, s.Hkv, s.Lq);
    long by_len = s.Lk / (tile ? 2048 : 256);
    if (tile) {
        const long double per_split = (long double)partial_bytes(s, 1) * 2.0L;   // written and read
        const long by_bytes = per_split > 0.0L ? (long)(40.0e6L / per_split) : 0;
        const long by_len_short = s.Lk / 256;
        const long few_rows = by_bytes < by_len_short ? by_bytes : by_len_short;
        if (few_rows > by_len) by_len = few_rows;
    }
    if (by_len < 1) by_len = 1;
    if (sp > by_len) sp = by_len;
    if (sp > FLASHD_MAX_SPLITS) sp = FLASHD_MAX_SPLITS;
    if (sp < 1) sp = 1;
    return (int)sp;
}

size_t ws_bytes(const Shape& s, int splits) { return splits <= 1 ? 0 : partial_bytes(s, splits); }

// ---- device check ----------------------------------------------------------

std::mutex g_mu;
std::map<int, int> g_arch_ok;      // device -> 1 ok / 0 not gfx950

int check_arch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return FLASHD_E_HIP; }
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_arch_ok.find(dev);
    if (it == g_arch_ok.end()) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) {
            (void)hipGetLastError();
            return FLASHD_E_HIP;
        }
        const int ok = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 0;
        it = g_arch_ok.emplace(dev, ok).first;
    }
    return it->second ? FLASHD_OK : FLASHD_E_ARCH;
}

// ---- workspace cache: grow-only, one buffer per (device, stream) -----------
// A buffer that is outgrown is not freed on the spot, because work enqueued earlier on the
// stream may still be reading it: it is kept in the entry's list of retired buffers until
// flashd_release_workspace() frees everything (hipFree waits for the device first).

struct CacheEntry {
    void* ptr = nullptr;
    size_t bytes = 0;
    std::vector<void*> retired;
};
std::map<std::pair<int, void*>, CacheEntry> g_cache;

int cached_workspace(void* stream, size_t bytes, void** out) {
    *out = nullptr;
    if (bytes == 0) return FLASHD_OK;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return FLASHD_E_HIP; }
    std::lock_guard<std::mutex> lk(g_mu);
    CacheEntry& e = g_cache[std::make_pair(dev, stream)];
    if (e.bytes < bytes) {
        // grow geometrically; if that much is not to be had, take exactly what is needed
        size_t want = e.bytes * 2 > bytes ? e.bytes * 2 : bytes;
        void* p = nullptr;
        if (hipMalloc(&p, want) != hipSuccess) {
            (void)hipGetLastError();
            want = bytes;
            if (hipMalloc(&p, want) != hipSuccess) { (void)hipGetLastError(); return FLASHD_E_HIP; }
        }
        if (e.ptr != nullptr) e.retired.push_back(e.ptr);
        e.ptr = p;
        e.bytes = want;
    }
    *out = e.ptr;
    return FLASHD_OK;
}

// Frees every cached buffer of the current device, live or retired.
int release_workspace() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return FLASHD_E_HIP; }
    std::lock_guard<std::mutex> lk(g_mu);
    int rc = FLASHD_OK;
    for (auto it = g_cache.begin(); it != g_cache.end();) {
        if (it->first.first != dev) { ++it; continue; }
        CacheEntry& e = it->second;
        if (e.ptr != nullptr) e.retired.push_back(e.ptr);
        for (void* q : e.retired)
            if (hipFree(q) != hipSuccess) { (void)hipGetLastError(); rc = FLASHD_E_HIP; }
        it = g_cache.erase(it);
    }
    return rc;
}

// ---- static scratch: split-K partial states for the entry point that allocates nothing ---
// One array per GPU, part of the loaded code object, held until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress: the device address is asked
// for once per device (with that device current) and kept, and only that address is ever
// handed to a kernel.
constexpr size_t kScratchBytes = FLASHD_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
std::map<int, void*> g_scratch_ptr;     // device -> address of its copy of `scratch`

int static_scratch(void** out) {
    *out = nullptr;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return FLASHD_E_HIP; }
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_scratch_ptr.find(dev);
    if (it == g_scratch_ptr.end()) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return FLASHD_E_HIP;
        }
        it = g_scratch_ptr.emplace(dev, ptr).first;
    }
    *out = it->second;
    return FLASHD_OK;
}

enum class WsMode { Caller, Cache, Static };

struct SkipArgs {
    bool on = false;                 // decode kernel with the saturation skip on the V fetch
    unsigned long long* counts = nullptr;
};

// ---- common front end --------------------------------------------------------

struct StateArgs {
    bool on = false;                 // the state entry point: o may be NULL, shift is explicit
    int shift = 0;
    const float* in = nullptr;
    float* out = nullptr;
};

struct Kv8Args {
    bool on = false;                 // k and v are fp8 (e4m3) with one scale each
    float kscale = 1.0f, vscale = 1.0f;
};

int run(const void* q, const void* k, const void* v, void* o, const Shape& s, int causal,
        float scale, void* stream, int variant, int splits, void* workspace,
        size_t workspace_bytes, WsMode mode, const StateArgs& sa = StateArgs(),
        const Kv8Args& k8 = Kv8Args(), const SkipArgs& sk = SkipArgs()) {
    const bool use_cache = mode == WsMode::Cache;
    if (!q || !k || !v) return FLASHD_E_NULL;
    if (!o && !(sa.on && sa.out)) return FLASHD_E_NULL;
    int rc = validate_shape(s);
    if (rc != FLASHD_OK) return rc;
    const uintptr_t bits = (uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o |
                           (uintptr_t)workspace | (uintptr_t)sa.in | (uintptr_t)sa.out;
    if (bits & 15u) return FLASHD_E_ALIGN;
    if ((uintptr_t)sk.counts & 7u) return FLASHD_E_ALIGN;
    const int var = resolve_variant(s, variant);
    if (var < 0) return FLASHD_E_VARIANT;
    // fp8 K/V: the split-K decode kernel reads that storage itself; for other shapes K and V
    // are first widened (exactly) into scratch memory
    if (k8.on && s.dtype == FLASHD_F32) return FLASHD_E_VARIANT;
    // the skip lives in the split-K decode kernel (f16/bf16, at most 32 query rows per kv head)
    if (sk.on && (s.dtype == FLASHD_F32 || !flashd::decode_applies(s.Hq, s.Hkv, s.Lq)))
        return FLASHD_E_VARIANT;
    const bool widen = k8.on && !flashd::decode_applies(s.Hq, s.Hkv, s.Lq);
    if (splits < 0 || splits > FLASHD_MAX_SPLITS || splits > s.Lk) return FLASHD_E_VARIANT;
    const int sp = splits == 0 ? auto_splits(s, var) : splits;
    // The state entry point always goes through partial states; a single partial may be
    // written straight into the caller's state buffer (unless that is also the input state).
    const bool direct = sa.on && sp == 1 && sa.out != nullptr && sa.out != sa.in;
    // The tile kernel can start from the state itself and write both results: no partial
    // states, no merge kernel.
    const bool in_kernel = sa.on && sp == 1 && var == FLASHD_VARIANT_TILE &&
                           !flashd::decode_applies(s.Hq, s.Hkv, s.Lq);
    const size_t need = sa.on ? ((direct || in_kernel) ? 0 : partial_bytes(s, sp)) : ws_bytes(s, sp);
    if (mode == WsMode::Caller && need > 0 && (workspace == nullptr || workspace_bytes < need))
        return FLASHD_E_WORKSPACE;
    if (mode == WsMode::Static && need > kScratchBytes) return FLASHD_E_WORKSPACE;

    rc = check_arch();
    if (rc != FLASHD_OK) return rc;
    void* ws = workspace;
    const size_t need_al = (need + 255) & ~(size_t)255;
    const size_t kv_bytes = widen ? (size_t)s.B * s.Hkv * s.Lk * s.d * 2 : 0;   // per tensor
    if (use_cache) {
        rc = cached_workspace(stream, need_al + 2 * kv_bytes, &ws);
        if (rc != FLASHD_OK) return rc;
    }
    if (mode == WsMode::Static && need > 0) {
        rc = static_scratch(&ws);
        if (rc != FLASHD_OK) return rc;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    float score_scale = scale, out_scale = 1.0f;
    bool kv8_kernel = k8.on;
    if (widen) {
        char* base = static_cast<char*>(ws) + need_al;
        if (flashd::launch_widen_fp8(k, v, base, base + kv_bytes,
                                     (size_t)s.B * s.Hkv * s.Lk * s.d, s.dtype, st) != hipSuccess)
            return FLASHD_E_HIP;
        k = base;
        v = base + kv_bytes;
        score_scale = scale * k8.kscale;       // one fp32 product, as in the decode kernel
        out_scale = k8.vscale;
        kv8_kernel = false;
    }

    Problem p;
    p.q = q; p.k = k; p.v = v; p.o = o;
    p.ws = static_cast<float*>(ws);
    p.B = s.B; p.Hq = s.Hq; p.Hkv = s.Hkv; p.Lq = s.Lq; p.Lk = s.Lk; p.d = s.d;
    p.Li = flashd::make_fast_div((uint32_t)s.Lq);
    p.dtype = s.dtype;
    p.causal = causal != 0;
    p.splits = sp;
    p.scale = score_scale;
    p.oscale = out_scale;
    // a shift of Lk or more shows every key and one below -Lq none: clamping the caller's
    // value there changes no result and keeps i + shift inside 32 bits
    const int shift_in = sa.shift > s.Lk ? s.Lk : (sa.shift < -s.Lq - 1 ? -s.Lq - 1 : sa.shift);
    p.shift = sa.on ? shift_in : s.Lk - s.Lq;
    p.partial = (sp > 1 || sa.on) ? 1 : 0;
    p.store_o = p.partial ? 0 : 1;
    p.merge = p.partial;
    p.from_state = 0;
    p.state_in = sa.in;
    p.state_out = sa.out;
    p.vskip_counts = sk.counts;
    p.wide = (var == FLASHD_VARIANT_TILE_256 ||
              (variant == FLASHD_VARIANT_AUTO && !sa.on && !k8.on && !sk.on && sp == 1 &&
               prefers_256_rows(s, causal != 0))) ? 1 : 0;
    if (in_kernel) {
        p.partial = sa.out != nullptr ? 1 : 0;     // the "partial" is the state handed out
        p.store_o = o != nullptr ? 1 : 0;
        p.merge = 0;
        p.from_state = sa.in != nullptr ? 1 : 0;
        p.ws = sa.out;
    }
    p.kv8 = kv8_kernel ? 1 : 0;
    p.kscale = k8.kscale;
    p.vscale = k8.vscale;
    if (direct && !in_kernel) p.ws = sa.out;
    hipError_t e;
    // The automatic choice takes the decode kernel with the saturation skip: on inputs where
    // nothing can be skipped it returns the bits of the unskipped kernel at the same speed.
    const bool auto_skip = variant == FLASHD_VARIANT_AUTO && !k8.on && s.dtype != FLASHD_F32 &&
                           flashd::decode_applies(s.Hq, s.Hkv, s.Lq);
    const int tmode = (sk.on || auto_skip)                 ? flashd::kTileModeLazySkipV
                      : var == FLASHD_VARIANT_ONLINE_SOFTMAX ? flashd::kTileModeOnline
                      : var == FLASHD_VARIANT_TILE_BLEND   ? flashd::kTileModeBlend
                                                           : flashd::kTileModeLazy;
    if (var == FLASHD_VARIANT_PER_KEY) e = flashd::launch_perkey(p, st);
    else if (flashd::decode_applies(s.Hq, s.Hkv, s.Lq)) e = flashd::launch_decode(p, tmode, st);
    else e = flashd::launch_tile(p, tmode, st);
    return e == hipSuccess ? FLASHD_OK : FLASHD_E_HIP;
}

}  // namespace

extern "C" {

int flashd_attn_fwd(const void* q, const void* k, const void* v, void* o, int B, int Hq, int Hkv,
                    int Lq, int Lk, int d, int causal, float scale, int dtype, void* stream) {
    const Shape s{B, Hq, Hkv, Lq, Lk, d, dtype};
    return run(q, k, v, o, s, causal, scale, stream, FLASHD_VARIANT_AUTO, 0, nullptr, 0,
               WsMode::Cache);
}

int flashd_attn_fwd_static(const void* q, const void* k, const void* v, void* o, int B, int Hq,
                           int Hkv, int Lq, int Lk, int d, int causal, float scale, int dtype,
                           void* stream) {
    const Shape s{B, Hq, Hkv, Lq, Lk, d, dtype};
    return run(q, k, v, o, s, causal, scale, stream, FLASHD_VARIANT_AUTO, 0, nullptr, 0,
               WsMode::Static);
}

int flashd_attn_fwd_ex(const void* q, const void* k, const void* v, void* o, int B, int Hq,
                       int Hkv, int Lq, int Lk, int d, int causal, float scale, int dtype,
                       void* stream, int variant, int splits, void* workspace,
                       size_t workspace_bytes) {
    const Shape s{B, Hq, Hkv, Lq, Lk, d, dtype};
    return run(q, k, v, o, s, causal, scale, stream, variant, splits, workspace, workspace_bytes,
               WsMode::Caller);
}

int flashd_attn_fwd_state(const void* q, const void* k, const void* v, void* o,
                          const float* state_in, float* state_out, int B, int Hq, int Hkv, int Lq,
                          int Lk, int d, int causal, int causal_shift, float scale, int dtype,
                          void* stream) {
    const Shape s{B, Hq, Hkv, Lq, Lk, d, dtype};
    StateArgs sa;
    sa.on = true;
    sa.shift = causal_shift;
    sa.in = state_in;
    sa.out = state_out;
    return run(q, k, v, o, s, causal, scale, stream, FLASHD_VARIANT_AUTO, 0, nullptr, 0,
               WsMode::Cache, sa);
}

int flashd_attn_fwd_kv8(const void* q, const void* k8, const void* v8, void* o, int B, int Hq,
                        int Hkv, int Lq, int Lk, int d, int causal, float scale, float kscale,
                        float vscale, int dtype, void* stream) {
    const Shape s{B, Hq, Hkv, Lq, Lk, d, dtype};
    Kv8Args a;
    a.on = true;
    a.kscale = kscale;
    a.vscale = vscale;
    return run(q, k8, v8, o, s, causal, scale, stream, FLASHD_VARIANT_AUTO, 0, nullptr, 0,
               WsMode::Cache, StateArgs(), a);
}

int flashd_attn_fwd_skipv(const void* q, const void* k, const void* v, void* o, int B, int Hq,
                          int Hkv, int Lq, int Lk, int d, int causal, float scale, int dtype,
                          void* stream, int splits, void* workspace, size_t workspace_bytes,
                          unsigned long long* counts) {
    const Shape s{B, Hq, Hkv, Lq, Lk, d, dtype};
    SkipArgs sk;
    sk.on = true;
    sk.counts = counts;
    return run(q, k, v, o, s, causal, scale, stream, FLASHD_VARIANT_TILE, splits, workspace,
               workspace_bytes, WsMode::Caller, StateArgs(), Kv8Args(), sk);
}

int flashd_skip_stats(const void* q, const void* k, int B, int Hq, int Hkv, int Lq, int Lk, int d,
                      int causal, float scale, int dtype, float lo, float hi,
                      unsigned long long* counts, void* stream) {
    if (!q || !k || !counts) return FLASHD_E_NULL;
    const Shape s{B, Hq, Hkv, Lq, Lk, d, dtype};
    int rc = validate_shape(s);
    if (rc != FLASHD_OK) return rc;
    if (((uintptr_t)q | (uintptr_t)k) & 15u) return FLASHD_E_ALIGN;
    if ((uintptr_t)counts & 7u) return FLASHD_E_ALIGN;
    rc = check_arch();
    if (rc != FLASHD_OK) return rc;
    Problem p;
    p.q = q; p.k = k; p.v = nullptr; p.o = nullptr; p.ws = nullptr;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.Lq = Lq; p.Lk = Lk; p.d = d;
    p.Li = flashd::make_fast_div((uint32_t)Lq);
    p.dtype = dtype;
    p.causal = causal != 0;
    p.splits = 1;
    p.scale = scale;
    p.shift = Lk - Lq;
    p.partial = 0;
    p.store_o = 0;
    p.merge = 0;
    p.from_state = 0;
    p.state_in = nullptr;
    p.state_out = nullptr;
    p.wide = 0;
    p.vskip_counts = nullptr;
    p.kv8 = 0;
    p.kscale = p.vscale = p.oscale = 1.0f;
    const hipError_t e =
        flashd::launch_skip_stats(p, lo, hi, counts, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FLASHD_OK : FLASHD_E_HIP;
}

int flashd_auto_splits(int B, int Hq, int Hkv, int Lq, int Lk, int d, int dtype, int variant) {
    const Shape s{B, Hq, Hkv, Lq, Lk, d, dtype};
    if (validate_shape(s) != FLASHD_OK) return 1;
    const int var = resolve_variant(s, variant);
    if (var < 0) return 1;
    return auto_splits(s, var);
}

int flashd_auto_variant(int B, int Hq, int Hkv, int Lq, int Lk, int d, int dtype, int causal) {
    const Shape s{B, Hq, Hkv, Lq, Lk, d, dtype};
    if (validate_shape(s) != FLASHD_OK) return -1;
    const int var = resolve_variant(s, FLASHD_VARIANT_AUTO);
    if (var != FLASHD_VARIANT_TILE || flashd::decode_applies(s.Hq, s.Hkv, s.Lq)) return var;
    return auto_splits(s, var) == 1 && prefers_256_rows(s, causal != 0) ? FLASHD_VARIANT_TILE_256
                                                                          : FLASHD_VARIANT_TILE;
}

size_t flashd_workspace_bytes(int B, int Hq, int Hkv, int Lq, int Lk, int d, int dtype,
                              int variant, int splits) {
    const Shape s{B, Hq, Hkv, Lq, Lk, d, dtype};
    if (validate_shape(s) != FLASHD_OK) return 0;
    const int var = resolve_variant(s, variant);
    if (var < 0 || splits < 0 || splits > FLASHD_MAX_SPLITS || splits > Lk) return 0;
    return ws_bytes(s, splits == 0 ? auto_splits(s, var) : splits);
}

int flashd_release_workspace(void) { return release_workspace(); }

const char* flashd_status_string(int status) {
    switch (status) {
    case FLASHD_OK: return "ok";
    case FLASHD_E_NULL: return "q, k, v or o is NULL";
    case FLASHD_E_SHAPE: return "a dimension is out of range";
    case FLASHD_E_DTYPE: return "unknown dtype";
    case FLASHD_E_HEADDIM: return "head dimension must be 64 or 128";
    case FLASHD_E_GQA: return "Hq must be a multiple of Hkv";
    case FLASHD_E_ALIGN: return "pointers must be 16-byte aligned";
    case FLASHD_E_WORKSPACE: return "workspace missing or too small";
    case FLASHD_E_HIP: return "a HIP call failed";
    case FLASHD_E_ARCH: return "the current device is not gfx950";
    case FLASHD_E_VARIANT: return "variant or splits not valid for this problem";
    default: return "unknown status";
    }
}

int flashd_version(void) { return 100; }

}  // extern "C"
