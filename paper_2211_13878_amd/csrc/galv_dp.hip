// Batched plan-search dynamic program for gfx950 (MI355X): kernels + C ABI.
//
// Paper section 3.3 ("Dynamic Programming Search", Eq. 1): for every layer l,
// budget column e and strategy s,
//     C[l][e][s] = c(l,s) + min_{s'} ( C[l-1][e - m(l,s)][s'] + R(s', s) ).
//
// How the recurrence is laid out here
// -----------------------------------
// The inner minimum does not depend on the memory shift, so each layer is a
// min-plus product of the (E+1) x S table with the S x S transition matrix:
//     U_l[e'][s] = c(l,s) + min_{s'} ( C[l-1][e'][s'] + R_l(s', s) )
//     C[l][e][s] = U_l[e - m(l,s)][s]                (infinity when e < m(l,s))
// The tables are stored UN-shifted (U_l, and the argmin beside it), strategy
// major and budget minor, so a wavefront covers 64 consecutive budget columns of
// one strategy: m(l,s), c(l,s) and R(s',s) are wave-uniform scalars, every
// global access is a contiguous row segment, and the shift is applied when layer
// l+1 reads column s' at offset -m(l,s').  Each lane keeps the running minima of
// its budget columns for a group of strategies in registers, so the minimum over
// s' is a serial in-lane loop: no cross-lane reduction, and the lowest-index
// tie-break falls out of the key order.
//
// Exact arithmetic paths, chosen per instance on the device
// ---------------------------------------------------------
//  * 32-bit keys (small costs and transition costs: the common case): costs are taken
//    relative to the column's smallest former cost and clamped at R_max + 1, so that
//    key = (relative cost + R) * 2^k + s' fits 32 bits; two candidates cost two
//    v_add_u32 and one v_min3_u32.  A clamped former strategy can neither win nor tie, which
//    is also what lets the sweep PRUNE: a former-layer row that is clamped in every column of
//    a tile is left out of the inner loop, and (rows being non-increasing along the budget
//    axis) two of its cells tell whether it needs to be fetched at all.  With the usual spread
//    of layer costs some 90-95 % of the candidates fall away and the sweep is bound by HBM.
//    The keys' width depends on the transition costs only; when the costs themselves outgrow
//    32-bit cells, the same body runs over 64-bit cells (up to 256 strategies).
//    Where a layer fills the chip, these instances keep a SINGLE table: the reduced key of a
//    state, (cost relative to its column's former minimum) * 2^k + argmin, is what the
//    back-pointer's 32-bit word stores, with one former minimum per budget column beside it;
//    the next layer rebuilds the cells it reads, and no cost rows are written (half the bytes).
//  * 64-bit keys: key = cost * 2^k + s' (k = ceil(log2 S)) lives in the mantissa of a double
//    whose exponent is pinned, K = 2^52 + key; one v_add_f64 + one v_min_f64 per candidate,
//    exact while K stays below 2^53.  Two storage widths: narrow (costs below 2^31 stored as
//    uint32, infinity = 2^31) and wide (the key itself stored as a double, infinity = +inf).
//  * int64: plain 64-bit integer add / compare / select with a separate index, for
//    instances whose value range does not fit a 52-bit key.
// In every packed form the minimum of keys is the minimum cost with the lowest s' among
// equals.  A preparation kernel bounds each instance's largest possible plan cost and picks
// the path; all paths produce bit-identical results.
//
// All kernels are plain VALU + LDS + global memory; there is no matrix-core work in a
// min-plus recurrence.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <type_traits>

#include "../../include/galv_dp.h"

// Workspace of galv_dp_solve_static, the entry point that allocates nothing: it lives in the
// code object, one copy per GPU for as long as the process runs.  Host code never uses this
// name as an address; it asks the runtime for the device address once per device (see
// static_scratch()).
static __device__ __align__(256) unsigned char scratch[GALV_DP_STATIC_BYTES];

namespace {

constexpr int kThreads = 256;          // workgroup = 4 wavefronts of 64
constexpr int kPrepThreads = 1024;     // prep_kernel: one workgroup per instance, whose loops are chains of
                                       // load round trips: 16 wavefronts shorten each chain
constexpr int kWave = 64;
constexpr int kEAlign = 1024;          // budget columns are padded to this
constexpr int kMaxS = 1024;
constexpr int kMaxSide = 16;          // internal streams per handle
constexpr int kMaxPp = 16;            // pipeline degrees per reduce call
#ifndef GALV_P1_BATCH
#define GALV_P1_BATCH 8
#endif
#ifndef GALV_DEPTH
#define GALV_DEPTH 2
#endif
#ifndef GALV_XCD_MAP
#define GALV_XCD_MAP 1
#endif
constexpr int kDepth = GALV_DEPTH;      // previous-layer loads kept in flight per wave
constexpr int64_t kInf = GALV_INF;
constexpr uint32_t kInf32 = 0x80000000u;             // infinity of the narrow storage
constexpr uint64_t kBias = 0x4330000000000000ull;    // bit pattern of 2^52

thread_local char g_err[512] = "";

galv_status_t fail(galv_status_t code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                  \
    do {                                                                               \
        hipError_t e_ = (expr);                                                        \
        if (e_ != hipSuccess)                                                          \
            return fail(GALV_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));  \
    } while (0)

inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Geometry of one sweep-kernel variant: TS strategies x TE budget columns of
// running minima per lane, NG strategy groups per workgroup.
struct Variant {
    int ts, te, ng, w, ux; // w: wavefronts per workgroup (w / ng budget sub-tiles); ux: see sweep_kernel
    int wpe;               // waves per SIMD the kernel is built for
    int share;             // 1: the row-sharing 32-bit-key body (one tile per workgroup, LDS for the kept rows)
};

// Everything the kernels need to find their data.  Passed by value.
struct Layout {
    int32_t B, L, S, E_max, nR;
    int32_t S_pad;        // strategies rounded up to the variant's group size
    int32_t k_bits;       // index bits in a packed key
    int32_t tile_e;       // budget columns per workgroup
    int32_t n_tiles;      // workgroups along the budget axis
    int64_t lead;         // infinity columns in front of every cost row (fast paths)
    int64_t row;          // cells per cost row: lead + padded columns (8 bytes reserved each)
    int64_t e_pad;        // padded budget columns (multiple of kEAlign)
    char *U[2];           // rolling cost rows   [B][S_pad][row] of 8-byte slots
    void *bp;             // argmin, un-shifted  [B][L-1][S][e_pad] of int32, or of uint8 (0xFF = none)
    int32_t bp_u8;        // 1: one-byte back-pointers
    int32_t peek;         // 1: the row-sharing sweep looks at two cells of a row before it fetches the row
    int32_t packed;       // 1: instances on the 32-bit-key paths keep ONE table: the back-pointer word holds the
                          //    reduced key (relative cost << k | argmin, all ones = unreachable) and the cost
                          //    rows are replaced by one former minimum per budget column (see is_packed)
    int32_t synth_l1;     // 1: the 32-bit-key sweep makes up layer 0's cells (a constant per strategy)
                          //    when it sweeps layer 1, so layer 0's row is never written nor read
    int32_t b_off, b_step; // a sweep launch covers instances b_off + z * b_step (dealt over streams)
    double *Rk;           // R * 2^k + s'        [B][nR][S][S_pad] (+inf in padded columns)
    uint64_t *ck;         // per-mode c(l,s)     [B][L][S_pad]
    uint64_t *vlist;      // usable strategies of each layer, ascending: shift << 32 | s'; the last one repeats
                          // up to the row's end  [B][L][S_pad]
    uint64_t *vcost;      // c(l, s') of the listed strategies, in the list's order (padded the same way)  [B][L][S_pad]
    int32_t *nvalid;      // how many of them    [B][L]
    uint32_t *dclamp;     // 32-bit-key path: largest R + 1, the clamp of relative costs  [B]
    int32_t *hdr;         // what a sweep workgroup needs first, in one place: status, budget, usable strategies of
                          // the former layer, clamp, transition matrix of the layer; 3 unused  [B][L][8]
    int32_t *status;      // per instance        [B]
    int32_t *last;        // best last strategy  [B]
    int32_t *lead_mode;   // whose infinity leads the rows hold (lead_kind), 0 none  [B]
    uint32_t *stats;      // 32-bit-key sweeps, per tile: rows reduced << 16 | rows listed; rows fetched  [B][L-1][n_tiles][2]
    int32_t *seen;        // pinned host word (or null): the budget tiles of all instances, as the last solve found them
    const int64_t *c;
    const int32_t *m;
    const int64_t *R;
    const int32_t *r_idx; // may be null
    const int32_t *budget;
};

__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }
// Position of the thread, without the thread-index register: the kernel reads that register
// once, at its top (wave number, a scalar), and the lane number is recomputed where it is
// needed, so no vector register stays occupied from the kernel's entry to the body it selects.
__device__ __forceinline__ int lane_id() { return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }
// Lane `lane`'s value of v, as a wave-uniform scalar.
__device__ __forceinline__ uint32_t read_lane(uint32_t v, int lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}
__device__ __forceinline__ uint64_t read_lane(uint64_t v, int lane) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), lane);
    return (uint64_t)hi << 32 | lo;
}

// Read-only view through the constant address space: data that no thread writes
// while the kernel runs (inputs, tables packed by the preparation kernel).  With a
// wave-uniform address such loads go through the scalar cache into SGPRs.
template <class T>
using ConstPtr = const T __attribute__((address_space(4))) *;
template <class T>
__device__ __forceinline__ ConstPtr<T> as_const(const T *p) {
    return (ConstPtr<T>)(uintptr_t)p;
}

// Storage of the cost rows: 32-bit cells for both packed-key paths of small costs.
__device__ __forceinline__ bool narrow_cells(int st) {
    return st == GALV_INSTANCE_OK_FAST || st == GALV_INSTANCE_OK_FAST_U32;
}
// What the infinity lead in front of a cost row must hold: 1 uint32 2^31, 2 double +inf,
// 3 uint64 2^62, 0 no lead is read.
__device__ __forceinline__ int lead_kind(int st) {
    if (narrow_cells(st)) return 1;
    if (st == GALV_INSTANCE_OK_FAST_WIDE) return 2;
    if (st == GALV_INSTANCE_OK_U32_WIDE) return 3;
    return 0;
}

// Whether instance status st keeps the single packed table (a handle-wide choice of kernels, and
// the instance must be on a 32-bit-key path; one layer has no table at all).
__device__ __forceinline__ bool is_packed(const Layout &a, int st) {
    return a.packed && a.L > 1 && (st == GALV_INSTANCE_OK_FAST_U32 || st == GALV_INSTANCE_OK_U32_WIDE);
}

// Back-pointer of un-shifted cell idx, whichever width the handle stores.
__device__ __forceinline__ int32_t load_bp(const Layout &a, int st, int64_t idx) {
    if (is_packed(a, st)) {
        const uint32_t w = static_cast<const uint32_t *>(a.bp)[idx];
        return w == 0xffffffffu ? -1 : (int32_t)(w & ((1u << a.k_bits) - 1u));
    }
    if (a.bp_u8) {
        const uint8_t v = static_cast<const uint8_t *>(a.bp)[idx];
        return v == 0xFF ? -1 : (int32_t)v;
    }
    return static_cast<const int32_t *>(a.bp)[idx];
}
__device__ __forceinline__ void store_bp(const Layout &a, int64_t idx, int32_t v) {
    if (a.bp_u8)
        static_cast<uint8_t *>(a.bp)[idx] = (uint8_t)v;      // -1 becomes 0xFF
    else
        static_cast<int32_t *>(a.bp)[idx] = v;
}

// ------------------------------------------------------------- storage policies
//
// How a cost is kept in the rolling rows, and how it becomes the biased key
// K = 2^52 + cost * 2^k that the arithmetic works on (and back).
struct Narrow {
    using Cell = uint32_t;
    static __device__ __forceinline__ double dead_key(int k) {
        return __longlong_as_double((long long)(kBias | ((uint64_t)kInf32 << k)));
    }
    // K = 2^52 + x * 2^k, built from two 32-bit operations (1 <= k <= 10): the low word is
    // x << k; the high word is one funnel shift of {bias >> k, x} by 32 - k, which puts
    // the bias back in place above the top k bits of x.
    static __device__ __forceinline__ double to_key(Cell x, int k) {
        const uint32_t lo = x << k;
        const uint32_t hi = __builtin_amdgcn_alignbit((uint32_t)(kBias >> 32) >> k, x, 32 - k);
        return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
    }
    // From the reduced key: new cell = cost + c(l,s), argmin index (-1 if unreachable).
    static __device__ __forceinline__ void finish(double key, uint64_t cs, int k, uint32_t mask,
                                                  Cell &cell, int32_t &arg) {
        const uint64_t bits = (uint64_t)__double_as_longlong(key);
        const uint32_t cost = (uint32_t)(bits >> k);          // >= 2^31 exactly when unreachable
        const uint32_t sum = cost + (uint32_t)cs;             // < 2^32 by the range check
        cell = sum < kInf32 ? sum : kInf32;
        arg = (int32_t)((uint32_t)bits & mask) | ((int32_t)cost >> 31);
    }
    static __device__ __forceinline__ Cell first_layer(uint64_t cs) { return (Cell)cs; }
    static __device__ __forceinline__ Cell infinity() { return kInf32; }
    static __device__ __forceinline__ int64_t to_int64(Cell x, int) {
        return x >= kInf32 ? kInf : (int64_t)x;
    }
};

struct Wide {
    using Cell = double;
    static __device__ __forceinline__ double dead_key(int) { return INFINITY; }
    static __device__ __forceinline__ double to_key(Cell x, int) { return x; }
    static __device__ __forceinline__ void finish(double key, uint64_t cs, int, uint32_t mask,
                                                  Cell &cell, int32_t &arg) {
        const uint64_t bits = (uint64_t)__double_as_longlong(key);
        const uint32_t hi = (uint32_t)(bits >> 32);
        // strip the index, add c * 2^k (an unbiased double): the sum keeps the bias
        cell = __longlong_as_double((long long)(bits & ~(uint64_t)mask)) +
               __longlong_as_double((long long)cs);
        // bit 29 of the high word is set for +inf (0x7ff..) and clear for 2^52 <= K < 2^53
        arg = (int32_t)((uint32_t)bits & mask) | ((int32_t)(hi << 2) >> 31);
    }
    static __device__ __forceinline__ Cell first_layer(uint64_t cs) {
        return __longlong_as_double((long long)cs) + 0x1p52;
    }
    static __device__ __forceinline__ Cell infinity() { return INFINITY; }
    static __device__ __forceinline__ int64_t to_int64(Cell x, int k) {
        if (x == INFINITY) return kInf;
        return (int64_t)((((uint64_t)__double_as_longlong(x)) & 0x000fffffffffffffull) >> k);
    }
};

// ------------------------------------------------------------------ preparation
//
// One workgroup per instance.  Checks the value preconditions, bounds the
// largest cost any plan prefix can reach, picks the arithmetic path and, for the
// fast paths, packs R and c and lists the usable strategies of every layer.
__global__ __launch_bounds__(kPrepThreads) void prep_kernel(Layout a, uint32_t flags) {
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int64_t L = a.L, S = a.S, nR = a.nR;
    const int64_t *c = a.c + (int64_t)b * L * S;
    const int32_t *m = a.m + (int64_t)b * L * S;
    const int64_t *R = a.R + (int64_t)b * nR * S * S;
    const int32_t *ridx = a.r_idx ? a.r_idx + (int64_t)b * L : nullptr;
    const unsigned long long cap = (unsigned long long)kInf;

    __shared__ int bad;
    __shared__ unsigned long long rmax[64];  // max of each transition matrix (64 at a time)
    __shared__ unsigned long long red[kPrepThreads];
    __shared__ unsigned long long bound_s;
    if (tid == 0) bad = 0;
    __syncthreads();

    const int budget = uniform(a.budget[b]);
    if (tid == 0 && (budget < 0 || budget > a.E_max)) bad = 1;

    // What the batch's sweeps really cover: the budget tiles of all instances, told to the host (a
    // word of pinned memory that the NEXT solve reads when it sizes its launches; the budgets live
    // on the device, and a solve never waits for one).
    if (a.seen && b == 0) {
        unsigned long long tiles = 0;
        for (int i = tid; i < a.B; i += kPrepThreads) {
            const int e = a.budget[i];
            if (e >= 0 && e <= a.E_max) tiles += (unsigned)(e / a.tile_e + 1);
        }
        red[tid] = tiles;
        __syncthreads();
        for (int w = kPrepThreads / 2; w > 0; w >>= 1) {
            if (tid < w) red[tid] += red[tid + w];
            __syncthreads();
        }
        if (tid == 0)
            __hip_atomic_store(a.seen, (int32_t)(red[0] < 0x7fffffffull ? red[0] : 0x7fffffffull),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        __syncthreads();
    }

    // sum over layers of max_s c(l,s), saturating at 2^62: a wave per layer, a lane per strategy
    // (one thread walking a layer's strategies is a chain of loads, and with few layers most of
    // the workgroup would idle)
    const int wave = tid >> 6, lane = tid & 63;
    unsigned long long part = 0;
    for (int64_t l = wave; l < L; l += kPrepThreads / kWave) {
        unsigned long long mx = 0;
        bool off = false;                          // (kept in a register: a store to `bad` inside the loop
                                                   // would hold the next iteration's loads back)
#pragma unroll 2
        for (int64_t s = lane; s < S; s += kWave) {
            const int64_t v = c[l * S + s];
            off |= v < 0 || v >= kInf || m[l * S + s] < 0;
            if ((unsigned long long)v > mx) mx = (unsigned long long)v;
        }
        if (off) bad = 1;
#pragma unroll
        for (int w = kWave / 2; w > 0; w >>= 1) {
            const unsigned long long o = (unsigned long long)__shfl_xor((long long)mx, w, kWave);
            if (o > mx) mx = o;
        }
        if (lane == 0) {
            if (ridx && l >= 1 && (ridx[l] < 0 || ridx[l] >= nR)) bad = 1;
            part += mx;
            if (part > cap) part = cap;
        }
    }
    red[tid] = part;
    __syncthreads();
    for (int w = kPrepThreads / 2; w > 0; w >>= 1) {
        if (tid < w) {
            const unsigned long long t = red[tid] + red[tid + w];
            red[tid] = t > cap ? cap : t;
        }
        __syncthreads();
    }
    if (tid == 0) bound_s = red[0];
    __syncthreads();

    // plus, for every layer transition, the max of the matrix it uses
    unsigned long long rsum = 0, rmax_all = 0;  // valid in thread 0 only
    for (int64_t k0 = 0; k0 < nR; k0 += 64) {
        const int64_t kn = (nR - k0 < 64) ? nR - k0 : 64;
        for (int64_t k = 0; k < kn; ++k) {
            unsigned long long mx = 0;
            const int64_t *Rm = R + (k0 + k) * S * S;
            bool off = false;
#pragma unroll 4
            for (int64_t i = tid; i < S * S; i += kPrepThreads) {
                const int64_t v = Rm[i];
                off |= v < 0 || v >= kInf;
                if ((unsigned long long)v > mx) mx = (unsigned long long)v;
            }
            if (off) bad = 1;
            red[tid] = mx;
            __syncthreads();
            for (int w = kPrepThreads / 2; w > 0; w >>= 1) {
                if (tid < w && red[tid + w] > red[tid]) red[tid] = red[tid + w];
                __syncthreads();
            }
            if (tid == 0) {
                rmax[k] = red[0];
                if (red[0] > rmax_all) rmax_all = red[0];
            }
            __syncthreads();
        }
        // (every thread adds up the layers it owns, saturating; one thread walking all layers is
        // a chain of dependent loads that takes longer than the rest of this kernel)
        unsigned long long part_r = 0;
        for (int64_t l = 1 + tid; l < L; l += kPrepThreads) {
            const int64_t k = ridx ? ridx[l] : 0;
            if (k >= k0 && k < k0 + kn) {
                part_r += rmax[k - k0];
                if (part_r > cap) part_r = cap;
            }
        }
        red[tid] = part_r;
        __syncthreads();
        for (int w = kPrepThreads / 2; w > 0; w >>= 1) {
            if (tid < w) {
                const unsigned long long t = red[tid] + red[tid + w];      // each <= 2^62: no wrap
                red[tid] = t > cap ? cap : t;
            }
            __syncthreads();
        }
        if (tid == 0) {
            rsum += red[0];
            if (rsum > cap) rsum = cap;
        }
        __syncthreads();
    }

    __shared__ int status_s;
    if (tid == 0) {
        const unsigned long long bound = bound_s + rsum;   // each <= 2^62: no wrap
        int st;
        if (bad || bound >= cap) {
            st = GALV_INSTANCE_BAD_VALUE;
        } else if (flags & GALV_DP_FORCE_INT64) {
            st = GALV_INSTANCE_OK_INT64;
        } else if (bound + rmax_all < kInf32) {
            // costs, and infinity + R, fit 32 bits.  If, besides, twice the largest R still
            // leaves room for the index in a 32-bit key, the integer path applies.
            const bool u32 = !(flags & GALV_DP_NO_U32) &&
                             ((2 * rmax_all + 2) << a.k_bits) <= (1ull << 32);
            st = u32 ? GALV_INSTANCE_OK_FAST_U32 : GALV_INSTANCE_OK_FAST;
            a.dclamp[b] = (uint32_t)(rmax_all + 1);
        } else if (a.synth_l1 && !(flags & GALV_DP_NO_U32) &&
                   ((2 * rmax_all + 2) << a.k_bits) <= (1ull << 32)) {
            // costs need 64-bit cells, but only RELATIVE costs (clamped at R_max + 1) enter the keys:
            // the 32-bit-key arithmetic and its pruning apply all the same (row-sharing variants)
            st = GALV_INSTANCE_OK_U32_WIDE;
            a.dclamp[b] = (uint32_t)(rmax_all + 1);
        } else if (bound + 1 <= (1ull << (52 - a.k_bits))) {
            st = GALV_INSTANCE_OK_FAST_WIDE;    // keys fit the 52-bit mantissa
        } else {
            st = GALV_INSTANCE_OK_INT64;
        }
        status_s = st;
        a.status[b] = st;
    }
    __syncthreads();
    const int st = status_s;
    // One record per layer with what a sweep workgroup needs before anything else, so that it
    // takes one load instead of a chain of them.  (The count of the former layer's usable
    // strategies is filled in below, by the thread that builds that layer's list.)
    for (int64_t l = tid; l < L; l += kPrepThreads) {
        int32_t *h = a.hdr + ((int64_t)b * L + l) * 8;
        h[0] = st;
        h[1] = budget;
        h[2] = 0;
        h[3] = (int32_t)a.dclamp[b];
        h[4] = (ridx && l >= 1 && st >= 0) ? ridx[l] : 0;
    }
    __syncthreads();
    if (!narrow_cells(st) && st != GALV_INSTANCE_OK_FAST_WIDE && st != GALV_INSTANCE_OK_U32_WIDE) return;

    // R key = R * 2^k + s' (s' = row = former strategy); padded columns are +inf so
    // that they never win and never read past the caller's matrix.
    const double scale = (double)(1ull << a.k_bits);
    double *Rk = a.Rk + (int64_t)b * nR * S * a.S_pad;
    // (a wave per matrix row / per layer and a lane per column: no index arithmetic per element)
    constexpr int kWaves = kPrepThreads / kWave;
    const int S_pad = a.S_pad;
    const bool keys32 = st == GALV_INSTANCE_OK_FAST_U32 || st == GALV_INSTANCE_OK_U32_WIDE;
    for (int64_t k = 0; k < nR; ++k) {
        for (int sp = wave; sp < (int)S; sp += kWaves) {
            const int64_t *src = R + (k * S + sp) * S;
            if (keys32) {
                // 32-bit keys in the first half of each matrix's slot: rows of S_pad words, one
                // matrix every S * S_pad doubles; padded columns hold the largest word.
                uint32_t *row = reinterpret_cast<uint32_t *>(Rk + k * S * S_pad) + (int64_t)sp * S_pad;
                for (int sx = lane; sx < S_pad; sx += kWave)
                    row[sx] = (sx < (int)S) ? (((uint32_t)src[sx]) << a.k_bits) | (uint32_t)sp : 0xffffffffu;
            } else {
                double *row = Rk + (k * S + sp) * S_pad;
                for (int sx = lane; sx < S_pad; sx += kWave)
                    row[sx] = (sx < (int)S) ? (double)src[sx] * scale + (double)sp : INFINITY;
            }
        }
    }
    // c(l,s) in the form the epilogue adds: the integer itself (integer cells) or the
    // double c * 2^k (cells that hold 64-bit keys).
    uint64_t *ck = a.ck + (int64_t)b * L * S_pad;
    const bool c_int = narrow_cells(st) || st == GALV_INSTANCE_OK_U32_WIDE;
    for (int64_t l = wave; l < L; l += kWaves)
        for (int sx = lane; sx < S_pad; sx += kWave) {
            const int64_t v = (sx < (int)S) ? c[l * S + sx] : 0;
            ck[l * S_pad + sx] = c_int ? (uint64_t)v : (uint64_t)__double_as_longlong((double)v * scale);
        }
    // Per layer, the strategies whose memory fits the budget at all, in ascending
    // order, with their shift: the sweep of the next layer walks this list instead
    // of all S columns (a column that never fits is infinity everywhere).
    // (a wave per layer, a lane per strategy: the usable ones find their place in the list by
    // counting the usable lanes below them)
    for (int64_t l = wave; l < L; l += kPrepThreads / kWave) {
        uint64_t *lst = a.vlist + ((int64_t)b * L + l) * a.S_pad;
        uint64_t *lc = a.vcost + ((int64_t)b * L + l) * a.S_pad;
        int n = 0;
        uint64_t last_ent = 0, last_c = 0;         // the list's last entry so far (wave-uniform)
        for (int s0 = 0; s0 < (int)S; s0 += kWave) {
            const int sx = s0 + lane;
            const bool in = sx < (int)S;
            const int sh = in ? m[l * S + sx] : 0;
            const uint64_t cv = in ? (uint64_t)c[l * S + sx] : 0;
            const bool ok = in && sh <= budget;
            const uint64_t ent = ((uint64_t)(uint32_t)sh << 32) | (uint32_t)sx;
            const uint64_t votes = __builtin_amdgcn_ballot_w64(ok);
            if (ok) {
                const int pos = n + __builtin_popcountll(votes & ((1ull << lane) - 1ull));
                lst[pos] = ent;
                lc[pos] = cv;
            }
            if (votes != 0) {                      // wave-uniform
                const int top = 63 - __builtin_clzll(votes);
                last_ent = read_lane(ent, top);
                last_c = read_lane(cv, top);
                n += __builtin_popcountll(votes);
            }
        }
        if (lane == 0) {
            a.nvalid[(int64_t)b * L + l] = n;
            if (l + 1 < L) a.hdr[((int64_t)b * L + l + 1) * 8 + 2] = n;
        }
        // Past the list's end its last entry repeats (it changes no minimum: min(x, x) = x), so
        // a sweep that walks a fixed number of entries needs no bound check; an empty list is
        // never walked.
        if (n > 0)
            for (int i = n + lane; i < a.S_pad; i += kWave) {
                lst[i] = last_ent;
                lc[i] = last_c;
            }
    }
}

// Layer 0: U_0[e'][s] = c(0,s) for every e' (the shift by m(0,s) is applied by
// whoever reads it), and the infinity lead in front of both rolling rows of the
// strategy.  Grid: (a few blocks that stride over the row, S, B).
//
// The leads never change while an instance keeps its storage mode, and no sweep
// writes into them, so only the first solve of a handle (fresh != 0) and a solve
// that finds another mode than the one recorded in lead_mode[b] write them;
// final_kernel records the mode once the solve is through.
__global__ __launch_bounds__(kThreads) void init_kernel(Layout a, int fresh) {
    const int b = blockIdx.z, s = blockIdx.y;
    const int st = uniform(a.status[b]);
    if (st < 0) return;
    const int64_t base = ((int64_t)b * a.S_pad + s) * a.row * 8;
    const int64_t x0 = (int64_t)blockIdx.x * kThreads + threadIdx.x, step = (int64_t)gridDim.x * kThreads;
    if (st == GALV_INSTANCE_OK_INT64) {
        const int64_t c0 = a.c[((int64_t)b * a.L) * a.S + s];
        for (int64_t x = a.lead + x0; x < a.row; x += step) reinterpret_cast<int64_t *>(a.U[0] + base)[x] = c0;
        return;
    }
    if (is_packed(a, st)) return;                  // no cost rows: layer 0 is made up, the sweeps test the shift
    const bool leads = fresh || a.lead_mode[b] != lead_kind(st);
    const bool u32_keys = st == GALV_INSTANCE_OK_FAST_U32 || st == GALV_INSTANCE_OK_U32_WIDE;
    const bool row0 = !(u32_keys && a.synth_l1 && a.L > 1);
    if (!leads && !row0) return;                   // the usual case after a handle's first solve
    const uint64_t cs = a.ck[((int64_t)b * a.L) * a.S_pad + s];
    if (narrow_cells(st)) {
        uint32_t *u0 = reinterpret_cast<uint32_t *>(a.U[0] + base);
        uint32_t *u1 = reinterpret_cast<uint32_t *>(a.U[1] + base);
        if (leads)
            for (int64_t x = x0; x < a.lead; x += step) {
                u0[x] = Narrow::infinity();
                u1[x] = Narrow::infinity();
            }
        if (row0)
            for (int64_t x = a.lead + x0; x < a.row; x += step) u0[x] = Narrow::first_layer(cs);
    } else if (st == GALV_INSTANCE_OK_U32_WIDE) {
        uint64_t *u0 = reinterpret_cast<uint64_t *>(a.U[0] + base);
        uint64_t *u1 = reinterpret_cast<uint64_t *>(a.U[1] + base);
        if (leads)
            for (int64_t x = x0; x < a.lead; x += step) {
                u0[x] = (uint64_t)kInf;
                u1[x] = (uint64_t)kInf;
            }
        if (row0)
            for (int64_t x = a.lead + x0; x < a.row; x += step) u0[x] = cs;
    } else {
        double *u0 = reinterpret_cast<double *>(a.U[0] + base);
        double *u1 = reinterpret_cast<double *>(a.U[1] + base);
        if (leads)
            for (int64_t x = x0; x < a.lead; x += step) {
                u0[x] = Wide::infinity();
                u1[x] = Wide::infinity();
            }
        for (int64_t x = a.lead + x0; x < a.row; x += step) u0[x] = Wide::first_layer(cs);
    }
}

// ---------------------------------------------------------------- layer sweep

// General 64-bit integer body: one budget column per thread at a time, strategy
// columns in chunks of CH running (min, argmin) pairs.
template <int CH>
__device__ __forceinline__ void sweep_int64(const Layout &a, int wave, int l, int b, int budget,
                                            int64_t tile_start) {
    const int64_t S = a.S;
    const int64_t *Uprev = reinterpret_cast<const int64_t *>(a.U[(l - 1) & 1]) +
                           (int64_t)b * a.S_pad * a.row + a.lead;
    int64_t *Unew = reinterpret_cast<int64_t *>(a.U[l & 1]) + (int64_t)b * a.S_pad * a.row + a.lead;
    const int64_t bp0 = ((int64_t)b * (a.L - 1) + (l - 1)) * S * a.e_pad;
    const int32_t *mprev = a.m + ((int64_t)b * a.L + (l - 1)) * S;
    const int64_t *cl = a.c + ((int64_t)b * a.L + l) * S;
    const int r = a.r_idx ? a.r_idx[(int64_t)b * a.L + l] : 0;
    const int64_t *R = a.R + ((int64_t)b * a.nR + r) * S * S;

    for (int64_t e = tile_start + wave * kWave + lane_id(); e < tile_start + a.tile_e; e += blockDim.x) {
        if (e > budget) continue;
        for (int64_t s0 = 0; s0 < S; s0 += CH) {
            int64_t best[CH];
            int32_t arg[CH];
#pragma unroll
            for (int q = 0; q < CH; ++q) {
                best[q] = kInf;
                arg[q] = -1;
            }
            for (int64_t sp = 0; sp < S; ++sp) {
                const int64_t shift = mprev[sp];
                if (shift > budget) continue;             // whole column is infinity
                const int64_t es = e - shift;
                const int64_t v = (es >= 0) ? Uprev[sp * a.row + es] : kInf;
                const int64_t *Rrow = R + sp * S;
#pragma unroll
                for (int q = 0; q < CH; ++q) {
                    const int64_t col = (s0 + q < S) ? s0 + q : S - 1;
                    const int64_t cand = v + Rrow[col];
                    if (cand < best[q]) {                 // strict: lowest s' keeps ties
                        best[q] = cand;
                        arg[q] = (int32_t)sp;
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < CH; ++q) {
                if (s0 + q < S) {
                    const bool dead = best[q] >= kInf;
                    Unew[(s0 + q) * a.row + e] = dead ? kInf : best[q] + cl[s0 + q];
                    store_bp(a, bp0 + (s0 + q) * a.e_pad + e, dead ? -1 : arg[q]);
                }
            }
        }
    }
}

// acc[j] = min(acc[j], v[j] + rk) on packed keys: one v_add_f64 and one v_min_f64
// per candidate, rk a wave-uniform SGPR pair.  Written as one asm block per
// strategy so that each needs only TE temporaries (left to itself the scheduler
// hoists every add of a row above the minima and spills), with the adds ahead of
// the minima so that no instruction waits on the one just issued.
typedef double double8 __attribute__((ext_vector_type(8)));

// `keep0`, `keep1` are the registers of the R group that is still being loaded while this
// statement runs: naming them as (unused) inputs keeps their next use close, so the
// register allocator has no reason to spill or move them while the load is in flight.
template <int TE, class K0, class K1>
__device__ __forceinline__ void minplus(double (&acc)[TE], const double (&v)[TE], double rk,
                                        const K0 &keep0, const K1 &keep1) {
    static_assert(TE == 1 || TE == 2 || TE == 4, "budget columns per lane");
    if constexpr (TE == 1) {
        double t0;
        asm("v_add_f64 %1, %2, %3\n\tv_min_f64 %0, %0, %1"
            : "+v"(acc[0]), "=&v"(t0)
            : "v"(v[0]), "s"(rk), "s"(keep0), "s"(keep1));
    } else if constexpr (TE == 2) {
        double t0, t1;
        asm("v_add_f64 %2, %4, %6\n\tv_add_f64 %3, %5, %6\n\t"
            "v_min_f64 %0, %0, %2\n\tv_min_f64 %1, %1, %3"
            : "+v"(acc[0]), "+v"(acc[1]), "=&v"(t0), "=&v"(t1)
            : "v"(v[0]), "v"(v[1]), "s"(rk), "s"(keep0), "s"(keep1));
    } else {
        double t0, t1, t2, t3;
        asm("v_add_f64 %4, %8, %12\n\tv_add_f64 %5, %9, %12\n\t"
            "v_add_f64 %6, %10, %12\n\tv_add_f64 %7, %11, %12\n\t"
            "v_min_f64 %0, %0, %4\n\tv_min_f64 %1, %1, %5\n\t"
            "v_min_f64 %2, %2, %6\n\tv_min_f64 %3, %3, %7"
            : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "=&v"(t0), "=&v"(t1),
              "=&v"(t2), "=&v"(t3)
            : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "s"(rk), "s"(keep0), "s"(keep1));
    }
}

// A group of R keys in SGPRs: 8 * NCH doubles fetched by NCH scalar loads of 16
// dwords.  The loads are issued by hand (the compiler would wait for each right
// where it issues it); rgroup_await makes every later use depend on the wait.
// Between request and await the compiler believes the destination registers are
// already defined; were it to spill or reuse them there (it does under heavy SGPR
// pressure, e.g. a deeper prefetch with an unsuitable tile shape), late-arriving
// data would overwrite whatever it put there.  The build refuses such code: it
// scans the produced assembly for any use of a destination register, any label or
// any branch between a request and its wait (paper_2211_13878_amd/isa_check.py).
template <int NCH>
struct RGroup {
    double8 c[NCH];
};
__device__ __forceinline__ void rgroup_request(RGroup<1> &g, ConstPtr<double> p) {
    asm volatile("s_load_dwordx16 %0, %1, 0x0" : "=&s"(g.c[0]) : "s"(p));
}
__device__ __forceinline__ void rgroup_request(RGroup<2> &g, ConstPtr<double> p) {
    asm volatile("s_load_dwordx16 %0, %2, 0x0\n\ts_load_dwordx16 %1, %2, 0x40"
                 : "=&s"(g.c[0]), "=&s"(g.c[1])
                 : "s"(p));
}
__device__ __forceinline__ void rgroup_await(RGroup<1> &g) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(g.c[0]));
}
__device__ __forceinline__ double rgroup_key(const RGroup<1> &g, int x) { return g.c[0][x]; }
__device__ __forceinline__ double rgroup_key(const RGroup<2> &g, int x) { return g.c[x / 8][x % 8]; }
__device__ __forceinline__ const double8 &rgroup_keep0(const RGroup<1> &g) { return g.c[0]; }
__device__ __forceinline__ const double8 &rgroup_keep1(const RGroup<1> &g) { return g.c[0]; }
__device__ __forceinline__ const double8 &rgroup_keep0(const RGroup<2> &g) { return g.c[0]; }
__device__ __forceinline__ const double8 &rgroup_keep1(const RGroup<2> &g) { return g.c[1]; }
// 9 to 12 keys: 8 + 4 doubles.  (Two buffers of 16 would take 64 of the ~100 scalar registers;
// the compiler then moves or spills registers that a load in flight still targets, which the
// build refuses.)
typedef double double4 __attribute__((ext_vector_type(4)));
struct RGroupMid {
    double8 lo;
    double4 hi;
};
__device__ __forceinline__ void rgroup_request(RGroupMid &g, ConstPtr<double> p) {
    asm volatile("s_load_dwordx16 %0, %2, 0x0\n\ts_load_dwordx8 %1, %2, 0x40"
                 : "=&s"(g.lo), "=&s"(g.hi)
                 : "s"(p));
}
__device__ __forceinline__ void rgroup_await(RGroupMid &g) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(g.lo), "+s"(g.hi));
}
__device__ __forceinline__ double rgroup_key(const RGroupMid &g, int x) { return x < 8 ? g.lo[x] : g.hi[x - 8]; }
__device__ __forceinline__ const double8 &rgroup_keep0(const RGroupMid &g) { return g.lo; }
__device__ __forceinline__ const double4 &rgroup_keep1(const RGroupMid &g) { return g.hi; }
__device__ __forceinline__ void rgroup_await(RGroup<2> &g) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(g.c[0]), "+s"(g.c[1]));
}

// Fast body.  Lane owns TE budget columns (64 apart) and TS strategy columns; per
// usable s' it loads its TE shifted previous-layer cells once and reuses them for
// all TS strategies, with the R keys as wave-uniform scalars.
// The wave's position is explicit: its first budget column e_wave and its first strategy s0.
template <int TS, int TE, class Store, class BP>
__device__ __forceinline__ void sweep_fast_at(const Layout &a, int l, int b, int budget,
                                              int64_t e_wave, int64_t s0) {
    using Cell = typename Store::Cell;
    constexpr int64_t kPerSlot = 8 / sizeof(Cell);     // cells per reserved 8-byte slot
    const int lane = lane_id();
    const int64_t e0 = e_wave + lane;
    if (s0 >= a.S) return;
    if (e_wave > budget) return;

    const int64_t S = a.S;
    const int k = a.k_bits;
    const int64_t pitch = a.row * kPerSlot;        // cells between rows of two strategies
    // wave-uniform base of the previous layer's rows; the lane adds only its own column, so
    // that the shifted addresses are a scalar base plus a loop-invariant lane offset
    const Cell *Up = reinterpret_cast<const Cell *>(a.U[(l - 1) & 1]) +
                     (int64_t)b * a.S_pad * pitch + a.lead + (e0 - lane);
    Cell *Un = reinterpret_cast<Cell *>(a.U[l & 1]) + ((int64_t)b * a.S_pad + s0) * pitch +
               a.lead + e0;
    BP *bp = static_cast<BP *>(a.bp) + (((int64_t)b * (a.L - 1) + (l - 1)) * S + s0) * a.e_pad + e0;
    const int r = a.r_idx ? a.r_idx[(int64_t)b * a.L + l] : 0;
    const ConstPtr<double> Rk = as_const(a.Rk + ((int64_t)b * a.nR + r) * S * a.S_pad + s0);
    const ConstPtr<uint64_t> ck = as_const(a.ck + ((int64_t)b * a.L + l) * a.S_pad + s0);

    double acc[TS][TE];
    const double dead = Store::dead_key(k);
#pragma unroll
    for (int s = 0; s < TS; ++s)
#pragma unroll
        for (int j = 0; j < TE; ++j) acc[s][j] = dead;

    // Walk the usable former-layer strategies (list built by the preparation
    // kernel; entries are wave-uniform scalars).  Two software pipelines run
    // under the arithmetic:
    //  * the shifted previous-layer cells of entry i + kDepth are requested
    //    while entry i is reduced (vector loads, kDepth - 1 entries of cover);
    //  * the R keys of a row arrive in groups of up to 16 doubles through explicit
    //    scalar loads into one of two SGPR buffers: the next group is requested
    //    before the current one is consumed and awaited after it.
    const ConstPtr<uint64_t> vl = as_const(a.vlist + ((int64_t)b * a.L + (l - 1)) * a.S_pad);
    const int n = as_const(a.nvalid)[(int64_t)b * a.L + (l - 1)];
    if (n > 0) {
        constexpr int kChunks = TS > 8 ? 2 : 1;            // scalar loads per group
        constexpr int kGroup = 8 * kChunks;                // doubles per group
        constexpr int kGroups = (TS + kGroup - 1) / kGroup;
        static_assert((kDepth * kGroups) % 2 == 0, "buffer roles must repeat every loop trip");
        Cell v[kDepth][TE];
        int sps[kDepth];
        using Group = std::conditional_t<(TS > 8 && TS <= 12), RGroupMid, RGroup<kChunks>>;
        Group buf[2];
        // Requests are never conditional (past the end they repeat the last entry,
        // which is cached) so that no wait is needed where control flow joins.
        auto request = [&](int q, int i) {
            const uint64_t ent = vl[i < n ? i : n - 1];
            sps[q] = (int)(uint32_t)ent;
            const Cell *p = Up + (int64_t)(uint32_t)ent * pitch - (int64_t)(ent >> 32);
#pragma unroll
            for (int j = 0; j < TE; ++j) v[q][j] = p[(uint32_t)lane + j * kWave];
        };
        // One entry: for each group, request the following group (of this entry or
        // of the next entry's row), reduce the current one, then await the request.
        auto reduce_entry = [&](int q) {
            double key[TE];
#pragma unroll
            for (int j = 0; j < TE; ++j) key[j] = Store::to_key(v[q][j], k);
#pragma unroll
            for (int gr = 0; gr < kGroups; ++gr) {
                const int t = q * kGroups + gr;
                const int qn = (gr + 1 < kGroups) ? q : (q + 1) % kDepth;
                const int gn = (gr + 1 < kGroups) ? gr + 1 : 0;
                rgroup_request(buf[(t + 1) & 1], Rk + (int64_t)sps[qn] * a.S_pad + gn * kGroup);
#pragma unroll
                for (int x = 0; x < kGroup; ++x)
                    if (gr * kGroup + x < TS)
                        minplus<TE>(acc[gr * kGroup + x], key, rgroup_key(buf[t & 1], x),
                                    rgroup_keep0(buf[(t + 1) & 1]), rgroup_keep1(buf[(t + 1) & 1]));
                rgroup_await(buf[(t + 1) & 1]);
            }
        };
#pragma unroll
        for (int q = 0; q < kDepth; ++q) request(q, q);
        rgroup_request(buf[0], Rk + (int64_t)sps[0] * a.S_pad);
        rgroup_await(buf[0]);
        int i = 0;
        for (; i + kDepth <= n; i += kDepth) {
#pragma unroll
            for (int q = 0; q < kDepth; ++q) {
                reduce_entry(q);
                request(q, i + q + kDepth);
            }
        }
#pragma unroll
        for (int q = 0; q < kDepth - 1; ++q)
            if (i + q < n) reduce_entry(q);
    }

    const uint32_t mask = (1u << k) - 1u;
#pragma unroll
    for (int s = 0; s < TS; ++s) {
        if (s0 + s < S) {
            const uint64_t cs = ck[s];
#pragma unroll
            for (int j = 0; j < TE; ++j) {
                Cell cell;
                int32_t arg;
                Store::finish(acc[s][j], cs, k, mask, cell, arg);
                Un[(int64_t)s * pitch + j * kWave] = cell;
                // Back-pointers are written once and read again only by the backtrack: a
                // streaming store keeps them from pushing the cost rows, which the next
                // layer reads back, out of the caches.  (-1 becomes 0xFF in one byte.)
                __builtin_nontemporal_store((BP)arg, &bp[(int64_t)s * a.e_pad + j * kWave]);
            }
        }
    }
}

// Position of a wave in a workgroup of NG strategy groups x (waves / NG) budget sub-tiles.
template <int TS, int TE, int NG, class Store, class BP>
__device__ __forceinline__ void sweep_fast(const Layout &a, int wave, int l, int b, int budget,
                                           int64_t tile_start) {
    const int g = wave % NG;                       // strategy group of this wave
    const int esub = wave / NG;                    // budget sub-tile of this wave
    sweep_fast_at<TS, TE, Store, BP>(a, l, b, budget, tile_start + (int64_t)esub * (kWave * TE),
                                     ((int64_t)blockIdx.y * NG + g) * TS);
}

// ------------------------------------------------------- 32-bit integer keys
//
// When costs fit 32 bits and twice the largest transition cost R_max still leaves
// room for the index, the inner minimum runs on 32-bit integers, two candidates per
// three instructions (two adds and one three-way minimum) instead of two per four.
// Costs are taken RELATIVE to the column's smallest former cost Cmin(e') =
// min_{s'} C[l-1][e'][s'] and clamped at D = R_max + 1:
//     key(s') = (min(C[l-1][e'][s'] - Cmin, D) + R(s', s)) * 2^k + s'   <  2^32.
// Clamping changes no result: the former strategy that attains Cmin gives a
// candidate of at most Cmin + R_max, while a clamped one costs at least
// Cmin + R_max + 1, so it neither wins nor ties.  Cmin comes from a first pass over
// the same shifted cells (they are then read again from the caches).  The new cell
// is Cmin + (key >> k) + c(l, s); a column without any reachable former cell
// (Cmin = infinity) stays infinity.
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint8v __attribute__((ext_vector_type(8)));
typedef uint32_t uint16v __attribute__((ext_vector_type(16)));
typedef uint16v uint16v_u __attribute__((aligned(8)));      // 16 words at any 8-byte boundary

// The R keys of one former strategy for TS strategy columns, in as few scalar registers as
// the loads allow (8, 8 + 4 or 16): four such rows are live at a time.
template <int TS, class = void>
struct R32Row;
template <int TS>
struct R32Row<TS, std::enable_if_t<(TS <= 8)>> {
    uint8v lo;
    uint32_t hi = 0;       // (unused; keeps the three shapes alike)
    __device__ __forceinline__ uint32_t at(int s) const { return lo[s]; }
    __device__ __forceinline__ void request(ConstPtr<uint32_t> p) {
        asm volatile("s_load_dwordx8 %0, %1, 0x0" : "=&s"(lo) : "s"(p));
    }
    __device__ __forceinline__ void tie() { asm volatile("" : "+s"(lo)); }
};
template <int TS>
struct R32Row<TS, std::enable_if_t<(TS > 8 && TS <= 12)>> {
    uint8v lo;
    uint4v hi;
    __device__ __forceinline__ uint32_t at(int s) const { return s < 8 ? lo[s] : hi[s - 8]; }
    __device__ __forceinline__ void request(ConstPtr<uint32_t> p) {
        asm volatile("s_load_dwordx8 %0, %2, 0x0\n\ts_load_dwordx4 %1, %2, 0x20"
                     : "=&s"(lo), "=&s"(hi)
                     : "s"(p));
    }
    __device__ __forceinline__ void tie() { asm volatile("" : "+s"(lo), "+s"(hi)); }
};
template <int TS>
struct R32Row<TS, std::enable_if_t<(TS > 12)>> {
    uint16v lo;
    uint32_t hi = 0;       // (unused; keeps the three shapes alike)
    __device__ __forceinline__ uint32_t at(int s) const { return lo[s]; }
    __device__ __forceinline__ void request(ConstPtr<uint32_t> p) {
        asm volatile("s_load_dwordx16 %0, %1, 0x0" : "=&s"(lo) : "s"(p));
    }
    __device__ __forceinline__ void tie() { asm volatile("" : "+s"(lo)); }
};
// Wait for every outstanding scalar load; the rows passed in become usable only after it.
template <class Row>
__device__ __forceinline__ void r32_await(Row &g0, Row &g1) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    g0.tie();
    g1.tie();
}

// acc = min(acc, va + ra, vb + rb) per budget column.  `keep...` are the registers of the
// rows still being loaded: naming them as (unused) inputs of every statement between their
// request and their wait keeps their next use close, so the register allocator has no
// reason to spill or move them while the loads are in flight.
template <int TE, class Row>
__device__ __forceinline__ void minplus_u32x2(uint32_t (&acc)[TE], const uint32_t (&va)[TE],
                                              const uint32_t (&vb)[TE], uint32_t ra, uint32_t rb,
                                              const Row &ka, const Row &kb) {
    static_assert(TE == 1 || TE == 2 || TE == 4, "budget columns per lane");
    if constexpr (TE == 1) {
        uint32_t t0, t1;
        asm("v_add_u32 %1, %5, %3\n\tv_add_u32 %2, %6, %4\n\tv_min3_u32 %0, %0, %1, %2"
            : "+v"(acc[0]), "=&v"(t0), "=&v"(t1)
            : "v"(va[0]), "v"(vb[0]), "s"(ra), "s"(rb), "s"(ka.lo), "s"(ka.hi), "s"(kb.lo), "s"(kb.hi));
    } else if constexpr (TE == 2) {
        uint32_t t0, t1, t2, t3;
        asm("v_add_u32 %2, %10, %6\n\tv_add_u32 %3, %11, %8\n\t"
            "v_add_u32 %4, %10, %7\n\tv_add_u32 %5, %11, %9\n\t"
            "v_min3_u32 %0, %0, %2, %3\n\tv_min3_u32 %1, %1, %4, %5"
            : "+v"(acc[0]), "+v"(acc[1]), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
            : "v"(va[0]), "v"(va[1]), "v"(vb[0]), "v"(vb[1]), "s"(ra), "s"(rb), "s"(ka.lo), "s"(ka.hi),
              "s"(kb.lo), "s"(kb.hi));
    } else {
        uint32_t t0, t1, t2, t3, t4, t5, t6, t7;
        asm("v_add_u32 %4, %20, %12\n\tv_add_u32 %5, %21, %16\n\t"
            "v_add_u32 %6, %20, %13\n\tv_add_u32 %7, %21, %17\n\t"
            "v_add_u32 %8, %20, %14\n\tv_add_u32 %9, %21, %18\n\t"
            "v_add_u32 %10, %20, %15\n\tv_add_u32 %11, %21, %19\n\t"
            "v_min3_u32 %0, %0, %4, %5\n\tv_min3_u32 %1, %1, %6, %7\n\t"
            "v_min3_u32 %2, %2, %8, %9\n\tv_min3_u32 %3, %3, %10, %11"
            : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "=&v"(t0), "=&v"(t1),
              "=&v"(t2), "=&v"(t3), "=&v"(t4), "=&v"(t5), "=&v"(t6), "=&v"(t7)
            : "v"(va[0]), "v"(va[1]), "v"(va[2]), "v"(va[3]), "v"(vb[0]), "v"(vb[1]), "v"(vb[2]),
              "v"(vb[3]), "s"(ra), "s"(rb), "s"(ka.lo), "s"(ka.hi), "s"(kb.lo), "s"(kb.hi));
    }
}

// Dynamic LDS of the row-sharing body below.
extern __shared__ uint32_t lds_cells[];

// Plain form: NG strategy groups x (waves / NG) budget sub-tiles per workgroup, every wave
// reads the rows it needs through the caches, twice (a first pass for the column minima, a
// second for the minimum over s'), and reduces every usable row.  It serves strategy counts
// beyond what one workgroup of the row-sharing body covers (several strategy-group blocks along
// grid.y).
template <int TS, int TE, int NG, class BP>
__device__ __forceinline__ void sweep_u32(const Layout &a, int wave, int l, int b, int budget,
                                          int64_t tile_start) {
    static_assert(TS <= 16, "one scalar load fetches the R keys of a row");
    const int lane = lane_id();
    const int g = wave % NG;
    const int esub = wave / NG;
    const int64_t e0 = tile_start + (int64_t)esub * (kWave * TE) + lane;
    const int64_t s0 = ((int64_t)blockIdx.y * NG + g) * TS;
    if (s0 >= a.S) return;
    if (tile_start + (int64_t)esub * (kWave * TE) > budget) return;      // wave-uniform

    const int64_t S = a.S;
    const int k = a.k_bits;
    const int64_t pitch = a.row * 2;               // 32-bit cells between the rows of two strategies
    const uint32_t *Up = reinterpret_cast<const uint32_t *>(a.U[(l - 1) & 1]) +
                         (int64_t)b * a.S_pad * pitch + a.lead + (e0 - lane);
    uint32_t *Un = reinterpret_cast<uint32_t *>(a.U[l & 1]) + ((int64_t)b * a.S_pad + s0) * pitch +
                   a.lead + e0;
    BP *bp = static_cast<BP *>(a.bp) + (((int64_t)b * (a.L - 1) + (l - 1)) * S + s0) * a.e_pad + e0;
    const int r = a.r_idx ? a.r_idx[(int64_t)b * a.L + l] : 0;
    const ConstPtr<uint32_t> Rk =
        as_const(reinterpret_cast<const uint32_t *>(a.Rk + ((int64_t)b * a.nR + r) * S * a.S_pad) + s0);
    const ConstPtr<uint64_t> ck = as_const(a.ck + ((int64_t)b * a.L + l) * a.S_pad + s0);
    const ConstPtr<uint64_t> vl = as_const(a.vlist + ((int64_t)b * a.L + (l - 1)) * a.S_pad);
    const int n = as_const(a.nvalid)[(int64_t)b * a.L + (l - 1)];
    const uint32_t dmax = as_const(a.dclamp)[b];

    uint32_t acc[TS][TE];
#pragma unroll
    for (int s = 0; s < TS; ++s)
#pragma unroll
        for (int j = 0; j < TE; ++j) acc[s][j] = 0xffffffffu;
    uint32_t cmin[TE];
#pragma unroll
    for (int j = 0; j < TE; ++j) cmin[j] = 0xffffffffu;

    auto cells = [&](int i) {            // shifted row of list entry i (clamped to the list)
        const uint64_t ent = vl[i < n ? i : n - 1];
        return Up + (int64_t)(uint32_t)ent * pitch - (int64_t)(ent >> 32);
    };

    if (s0 == 0 && esub == 0 && lane == 0) {       // statistics: this body reads and reduces every listed row
        uint32_t *st = a.stats + 2 * (((int64_t)b * (a.L - 1) + (l - 1)) * a.n_tiles +
                                      (uint32_t)tile_start / (uint32_t)a.tile_e);
        st[0] = (uint32_t)n << 16 | (uint32_t)n;
        st[1] = (uint32_t)n;
    }
    if (n > 0) {
        // Pass 1: the column minima of the former layer.  Pure loads: batches of kBatch list
        // entries, the next batch requested before the current one is reduced.
        constexpr int kBatch = GALV_P1_BATCH;
        uint32_t t[2][kBatch][TE];
        auto fetch = [&](int h, int i0) {
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const uint32_t *p = cells(i0 + u);
#pragma unroll
                for (int j = 0; j < TE; ++j) t[h][u][j] = p[(uint32_t)lane + j * kWave];
            }
        };
        auto fold = [&](int h) {
#pragma unroll
            for (int u = 0; u < kBatch; ++u)
#pragma unroll
                for (int j = 0; j < TE; ++j) cmin[j] = min(cmin[j], t[h][u][j]);
        };
        fetch(0, 0);
        int i = 0;
        for (; i + 2 * kBatch < n; i += 2 * kBatch) {
            fetch(1, i + kBatch);
            fold(0);
            fetch(0, i + 2 * kBatch);
            fold(1);
        }
        if (i + kBatch < n) {
            fetch(1, i + kBatch);
            fold(0);
            fold(1);
        } else {
            fold(0);
        }

        // Pass 2: pairs of list entries.  The cells of the next pair and the R rows of the
        // next pair are requested before the current pair is reduced.
        const int npair = (n + 1) / 2;             // an odd tail repeats its entry: min(x, x) = x
        uint32_t va[2][TE], vb[2][TE];
        int spa[2], spb[2];
        R32Row<TS> ra[2], rb[2];
        auto request = [&](int q, int pr) {
            const int ia = 2 * pr < n ? 2 * pr : n - 1;
            const int ib = 2 * pr + 1 < n ? 2 * pr + 1 : n - 1;
            const uint64_t ea = vl[ia], eb = vl[ib];
            spa[q] = (int)(uint32_t)ea;
            spb[q] = (int)(uint32_t)eb;
            const uint32_t *pa = Up + (int64_t)(uint32_t)ea * pitch - (int64_t)(ea >> 32);
            const uint32_t *pb = Up + (int64_t)(uint32_t)eb * pitch - (int64_t)(eb >> 32);
#pragma unroll
            for (int j = 0; j < TE; ++j) {
                va[q][j] = pa[(uint32_t)lane + j * kWave];
                vb[q][j] = pb[(uint32_t)lane + j * kWave];
            }
        };
        auto reduce_pair = [&](int q) {
            // keys of the next pair's rows, in flight under this pair's arithmetic
            ra[q ^ 1].request(Rk + (int64_t)spa[q ^ 1] * a.S_pad);
            rb[q ^ 1].request(Rk + (int64_t)spb[q ^ 1] * a.S_pad);
            uint32_t da[TE], db[TE];
#pragma unroll
            for (int j = 0; j < TE; ++j) {
                da[j] = min(va[q][j] - cmin[j], dmax) << k;
                db[j] = min(vb[q][j] - cmin[j], dmax) << k;
            }
#pragma unroll
            for (int s = 0; s < TS; ++s)
                minplus_u32x2<TE>(acc[s], da, db, ra[q].at(s), rb[q].at(s), ra[q ^ 1], rb[q ^ 1]);
            r32_await(ra[q ^ 1], rb[q ^ 1]);
        };
        request(0, 0);
        request(1, 1);
        ra[0].request(Rk + (int64_t)spa[0] * a.S_pad);
        rb[0].request(Rk + (int64_t)spb[0] * a.S_pad);
        r32_await(ra[0], rb[0]);
        int pr = 0;
        for (; pr + 2 <= npair; pr += 2) {
            reduce_pair(0);
            request(0, pr + 2);
            reduce_pair(1);
            request(1, pr + 3);
        }
        if (pr < npair) reduce_pair(0);
    }

    const uint32_t mask = (1u << k) - 1u;
#pragma unroll
    for (int s = 0; s < TS; ++s) {
        if (s0 + s < S) {
            const uint32_t cs = (uint32_t)ck[s];
#pragma unroll
            for (int j = 0; j < TE; ++j) {
                const bool alive = cmin[j] < kInf32;
                const uint32_t key = acc[s][j];
                Un[(int64_t)s * pitch + j * kWave] = alive ? cmin[j] + (key >> k) + cs : kInf32;
                // Back-pointers are written once and read again only by the backtrack: a
                // streaming store keeps them from pushing the cost rows, which the next
                // layer reads back, out of the caches.  (-1 becomes 0xFF in one byte.)
                __builtin_nontemporal_store((BP)(alive ? (int32_t)(key & mask) : -1),
                                            &bp[(int64_t)s * a.e_pad + j * kWave]);
            }
        }
    }
}

// How many surviving rows the row-sharing body below keeps in LDS for a workgroup that covers
// `cap` strategies (host and device agree through this one function).
// As many as the LDS holds without costing a resident workgroup: a CU holds wpe * 4 / ng
// workgroups by registers, each may take that share of the 160 KB (at most 128 KB); what the
// partial minima and counters leave goes to the list, in whole rows per wave and pass.  With
// 128-column tiles 8, 11, 16, 22, 32, 48, 96 and 224 rows for the eight variants below; with
// 256-column tiles 12, 16, 24, 32, 64 and 96.
constexpr int keep_rows(int ts, int ng, int wpe, int cols) {       // cols: budget columns of a tile
    const int wgs = wpe * 4 / ng > 0 ? wpe * 4 / ng : 1;
    const int share = 160 * 1024 / wgs < 128 * 1024 ? 160 * 1024 / wgs : 128 * 1024;
    const int fixed = ng * cols * 4 + ng * 8 + 16 + 256;
    int rows = (share - fixed) / (cols * 4 + 4);
    if (rows > ts * ng) rows = ts * ng;
    rows -= rows % ng;
    return rows < ng ? ng : rows;
}

// Row-sharing form of the 32-bit-key body, for S <= TS * NG (up to 256) with one budget tile of
// 64 * TE columns per workgroup of NG waves.  Wave g owns the former-layer rows g, g + NG, ...
// (TS of them, in registers) AND the strategy group g of the output.
//   1. Every wave loads its rows once (shifted, coalesced) and reduces them to partial column
//      minima; the partial minima meet in LDS (one barrier).
//   2. With the column minimum known, a wave tests each of its rows: a row whose relative cost
//      is clamped (>= dmax = R_max + 1) in every reachable column of the tile can neither win nor
//      tie any minimum of the tile (the strategy that attains the column minimum offers at most
//      Cmin + R_max) and is dropped.  The other rows are appended, as ready keys, to a short
//      list in LDS together with their strategy index (second barrier).  The order of the list
//      is whatever the appends make it: the minimum does not depend on it, and the lowest-index
//      tie-break rides in the low bits of the keys.
//   3. The inner loop runs over the surviving rows only, reading keys from LDS and R keys by
//      scalar loads.  Should more rows survive than the list holds (transition costs that dwarf
//      the spread of the layer costs), the rows go through the list in passes, a few rows of
//      every wave at a time: each wave reads its rows of the pass again, appends the live ones,
//      and every wave reduces that list.
// Only the survivors' keys live in LDS, as many rows as fit without costing a resident workgroup
// (keep_rows), which is what lets three 8-wave workgroups share a CU at S = 128.
//
// PACK: the table of back-pointers is the ONLY table.  The reduced key of a state already holds
// both results, (cost relative to the column's former minimum Cmin) << k | argmin, and
//     U_l[e'][s] = Cmin_l[e'] + (key >> k) + c(l, s),
// so the sweep stores the key where the back-pointer goes (all ones = unreachable), one Cmin
// per budget column beside it (rolling, in the space of the cost rows, which it replaces), and
// the next layer rebuilds the cells of the rows it fetches: 4 bytes written and at most 4 read
// per state instead of 8 and 4.  The backtrack masks the index out of the word.
template <int TS, int TE, int NG, class BP, class Cell, bool PACK, int KEEP>
__device__ __forceinline__ void sweep_u32_shared(const Layout &a, int g, int l, int b, int budget,
                                                 int64_t tile_start, bool add_stats, int n, uint32_t dmax,
                                                 int r_sel, uint64_t my_ent, uint64_t my_c0_64) {
    // n, dmax, r_sel: the former layer's usable strategies, the clamp and the layer's transition
    // matrix, from the header record.  my_ent, my_c0_64: lane r (and lane 32 + r) holds the list
    // entry of this wave's row g + NG * r and that strategy's c(l-1, s'), which made-up and
    // rebuilt cells add; the kernel requests them before it knows anything else (their addresses
    // depend on the workgroup's position only), so that they arrive together with the header.
    // Fetched as scalars where they are used, one row at a time, they form a chain of dependent
    // round trips (entry, then c, then the cells) that costs more than everything else a tile
    // does.  Rows that turn out to be needed get their entry broadcast from its lane.
    static_assert(!PACK || sizeof(BP) == 4, "a key needs the whole 32-bit word");
    // Cell: uint32_t (costs below 2^31, infinity = 2^31) or uint64_t (any cost up to the 2^62
    // precondition, infinity = 2^62).  Only RELATIVE costs enter the 32-bit keys, so the wide form
    // runs the same arithmetic and the same pruning; it moves 8-byte cells.
    constexpr bool kWide = sizeof(Cell) == 8;
    constexpr Cell kInfCell = kWide ? (Cell)kInf : (Cell)kInf32;
    constexpr Cell kAllOnes = ~(Cell)0;
    static_assert(TS <= 16, "one scalar load fetches the R keys of a row");
    constexpr int kCols = kWave * TE;
    constexpr int kKeep = KEEP;                    // rows the list holds (keep_rows of the variant)
    (void)budget;
    // A wave that has loads to issue goes before the waves that are in their arithmetic: the sooner a
    // tile's requests are out, the shorter its chain of round trips, and the arithmetic of the other
    // waves fills the time the requests take either way.  (Priority drops again before the inner loop.)
    __builtin_amdgcn_s_setprio(3);
    const int lane = lane_id();                    // (g: the wave = owner of rows g + NG * r = strategy group)
    const int64_t e0 = tile_start + lane;
    const int64_t s0 = (int64_t)g * TS;

    const int64_t S = a.S;
    const int k = a.k_bits;
    const int64_t pitch = a.row * (8 / (int64_t)sizeof(Cell));   // cells between the rows of two strategies
    const Cell *Up = reinterpret_cast<const Cell *>(a.U[(l - 1) & 1]) +
                     (int64_t)b * a.S_pad * pitch + a.lead + tile_start;
    // (wave-uniform: the first column of the tile in this wave's first output row)
    Cell *Un_tile = reinterpret_cast<Cell *>(a.U[l & 1]) + ((int64_t)b * a.S_pad + s0) * pitch +
                    a.lead + tile_start;
    BP *bp_tile = static_cast<BP *>(a.bp) + (((int64_t)b * (a.L - 1) + (l - 1)) * S + s0) * a.e_pad + tile_start;
    const ConstPtr<uint32_t> Rk =
        as_const(reinterpret_cast<const uint32_t *>(a.Rk + ((int64_t)b * a.nR + r_sel) * S * a.S_pad) + s0);
    const ConstPtr<uint64_t> ck = as_const(a.ck + ((int64_t)b * a.L + l) * a.S_pad + s0);
    // PACK: the former layer's words (rows of e_pad, no lead: a column below the shift is tested
    // for instead) and column minima, and this layer's column minima
    const uint32_t *Wp = static_cast<const uint32_t *>(a.bp) +
                         ((int64_t)b * (a.L - 1) + (l >= 2 ? l - 2 : 0)) * S * a.e_pad;
    const Cell *Mp = reinterpret_cast<const Cell *>(a.U[(l - 1) & 1] + (int64_t)b * a.S_pad * a.row * 8);
    Cell *Mn_tile = reinterpret_cast<Cell *>(a.U[l & 1] + (int64_t)b * a.S_pad * a.row * 8) + tile_start;
    const Cell my_c0 = (Cell)my_c0_64;

    // The shifted cells of one usable former strategy for this lane's columns.  Layer 0's table
    // is a constant per strategy, U_0[e'][s'] = c(0, s'), so when layer 1 is swept its cells are
    // made up here (infinity below the shift) instead of being read.
    const bool first = l == 1;                     // uniform
    // (cp = c(l-1, s'): what a made-up or rebuilt cell adds; unused for stored cells)
    auto load_row = [&](uint64_t ent, Cell cp, Cell (&out)[TE]) {
        const uint32_t sp = (uint32_t)ent, shift = (uint32_t)(ent >> 32);
        if (first) {
#pragma unroll
            for (int j = 0; j < TE; ++j) out[j] = e0 + j * kWave >= (int64_t)shift ? cp : kInfCell;
        } else if constexpr (PACK) {
            const uint32_t *w = Wp + (int64_t)sp * a.e_pad;
            uint32_t wv[TE];
            Cell mv[TE];
            bool ok[TE];
#pragma unroll
            for (int j = 0; j < TE; ++j) {
                const int64_t idx = e0 + j * kWave - (int64_t)shift;
                ok[j] = idx >= 0;
                const uint32_t x = ok[j] ? (uint32_t)idx : 0u;       // idx < e_pad <= 2^31 + 1024
                wv[j] = w[x];
                mv[j] = Mp[x];
            }
#pragma unroll
            for (int j = 0; j < TE; ++j) {
                // (the sum first, then a select between two values: a load used in one arm only
                // would be moved into that arm, behind the other load's round trip)
                const Cell cell = mv[j] + (Cell)(wv[j] >> k) + cp;
                out[j] = ok[j] && wv[j] != 0xffffffffu ? cell : kInfCell;
            }
        } else {
            const Cell *p = Up + (int64_t)sp * pitch - (int64_t)shift;
#pragma unroll
            for (int j = 0; j < TE; ++j) out[j] = p[(uint32_t)lane + j * kWave];
        }
    };

    Cell *part = reinterpret_cast<Cell *>(lds_cells);               // [NG][kCols] partial column minima
    Cell *wave_min = part + NG * kCols;                             // [NG] the waves' minima of the peek
    uint32_t *count = reinterpret_cast<uint32_t *>(wave_min + NG);  // [0] surviving rows, [2] rows fetched
    uint32_t *meta = count + 4;                    // [kKeep] strategy index of a kept row
    uint32_t *keys = meta + kKeep;                 // [kKeep][kCols] its keys

    uint32_t acc[TS][TE];
#pragma unroll
    for (int s = 0; s < TS; ++s)
#pragma unroll
        for (int j = 0; j < TE; ++j) acc[s][j] = 0xffffffffu;
    Cell cmin[TE];
#pragma unroll
    for (int j = 0; j < TE; ++j) cmin[j] = kAllOnes;

    if (g == 0 && lane == 0) count[0] = 0;

    // Peek.  Every stored row is non-increasing along the budget axis (more memory never costs
    // more), so a row's cells in this tile are at least its cell in the tile's last column, and
    // every column minimum of the tile is at most Cmin_before = the minimum over the rows' cells
    // in the column just BEFORE the tile.  A row whose last-column cell is at least
    // Cmin_before + dmax is therefore clamped in every column of the tile and need not be read at
    // all: two cells per row decide whether its 64 * TE cells are fetched.  (The column before the
    // tile rather than its first column: that is the last column of the neighbouring tile, whose
    // workgroup probes the same cell, so the two probes meet in the L2.)  The row that attains a
    // column's minimum always passes (its cell there is at most Cmin_before), so the minima over
    // the rows that are read are the true column minima.
    uint32_t keep = 0;                             // bit r: row g + NG * r is read (wave-uniform)
    if (n > 0 && !a.peek) {
        // (a launch that does not fill the chip is bound by latency, not by bytes: there the two
        // extra dependent steps of the peek cost more than the rows it saves)
#pragma unroll
        for (int r = 0; r < TS; ++r)
            if (g + NG * r < n) keep |= 1u << r;
        if (g == 0 && lane == 0) count[2] = (uint32_t)n;
    }
    if (n > 0 && a.peek) {
        // One gather for the whole wave: lane r (r < TS) fetches row r's cell in the column before
        // the tile (below the shift: infinity), lane 32 + r its cell in the tile's last column.
        Cell first_min = kAllOnes;
        const bool my_last = lane >= 32;
        const uint32_t my_sp = (uint32_t)my_ent, my_shift = (uint32_t)(my_ent >> 32);
        Cell mine;
        const int64_t idx = tile_start + (my_last ? kCols - 1 : -1) - (int64_t)my_shift;
        if (first) {
            mine = idx < 0 ? kInfCell : my_c0;     // this lane's column lies below the row's shift
        } else if constexpr (PACK) {
            const bool ok = idx >= 0;
            const uint32_t x = ok ? (uint32_t)idx : 0u;
            const uint32_t wv = Wp[(int64_t)my_sp * a.e_pad + x];
            const Cell mv = Mp[x];
            const Cell cell = mv + (Cell)(wv >> k) + my_c0;
            mine = ok && wv != 0xffffffffu ? cell : kInfCell;
        } else {
            mine = Up[(int64_t)my_sp * pitch + (idx - tile_start)];   // (the lead holds infinity below the shift)
        }
#pragma unroll
        for (int r = 0; r < TS; ++r) first_min = min(first_min, read_lane(mine, r));
        uint32_t *peek = count + 2;                // rows fetched by the workgroup
        if (lane == 0) wave_min[g] = first_min;
        if (g == 0 && lane == 0) peek[0] = 0;
        __syncthreads();
        Cell cmin_first = kAllOnes;
#pragma unroll
        for (int w = 0; w < NG; ++w) cmin_first = min(cmin_first, read_lane(wave_min[w], 0));
        // an unreachable column before the tile (Cmin_before = infinity) bounds nothing: read every row
        const Cell limit = cmin_first < kInfCell ? cmin_first + (Cell)dmax : kAllOnes;
        // lane 32 + r holds row r's last-column cell and votes for its row
        const bool my_keep = my_last && lane - 32 < TS && g + NG * (lane - 32) < n && mine < limit;
        keep = (uint32_t)(__builtin_amdgcn_ballot_w64(my_keep) >> 32);
        const int mine_read = __builtin_popcount(keep);
        if (lane == 0 && mine_read) atomicAdd(&peek[0], (uint32_t)mine_read);
    }

    Cell rowc[TS][TE];
    if (n > 0) {                                   // workgroup-uniform
        Cell pm[TE];
#pragma unroll
        for (int j = 0; j < TE; ++j) pm[j] = kAllOnes;
        if (PACK && !first) {
            // Rebuilt cells: the words and column minima of kChunk rows are requested before the
            // first of them is used, so the rows' round trips overlap (a row that is not read
            // counts as unreachable: it leaves every minimum alone).
            constexpr int kChunk = 4;
#pragma unroll
            for (int r0 = 0; r0 < TS; r0 += kChunk) {
                uint32_t wv[kChunk][TE];
                Cell mv[kChunk][TE];
#pragma unroll
                for (int q = 0; q < kChunk; ++q) {
                    const int r = r0 + q;
                    if (r >= TS) break;
                    if (keep >> r & 1) {
                        const uint64_t e_r = read_lane(my_ent, r);
                        const uint32_t *w = Wp + (int64_t)(uint32_t)e_r * a.e_pad;
#pragma unroll
                        for (int j = 0; j < TE; ++j) {
                            const int64_t idx = e0 + j * kWave - (int64_t)(uint32_t)(e_r >> 32);
                            const uint32_t x = idx >= 0 ? (uint32_t)idx : 0u;
                            const uint32_t v = w[x];
                            wv[q][j] = idx >= 0 ? v : 0xffffffffu;
                            mv[q][j] = Mp[x];
                        }
                    }
                }
#pragma unroll
                for (int q = 0; q < kChunk; ++q) {
                    const int r = r0 + q;
                    if (r >= TS) break;
                    if (keep >> r & 1) {           // (wave-uniform: most rows are not read at all)
                        const Cell cp = read_lane(my_c0, r);
#pragma unroll
                        for (int j = 0; j < TE; ++j) {
                            const Cell cell = mv[q][j] + (Cell)(wv[q][j] >> k) + cp;
                            rowc[r][j] = wv[q][j] != 0xffffffffu ? cell : kInfCell;
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < TE; ++j) rowc[r][j] = kAllOnes;      // leaves every minimum alone
                    }
                }
            }
        } else {
#pragma unroll
            for (int r = 0; r < TS; ++r) {
                if (keep >> r & 1) {
                    load_row(read_lane(my_ent, r), read_lane(my_c0, r), rowc[r]);
                } else {
#pragma unroll
                    for (int j = 0; j < TE; ++j) rowc[r][j] = kAllOnes;          // leaves every minimum alone
                }
            }
        }
#pragma unroll
        for (int r = 0; r < TS; ++r)
#pragma unroll
            for (int j = 0; j < TE; ++j) pm[j] = min(pm[j], rowc[r][j]);     // a repeated row changes nothing
#pragma unroll
        for (int j = 0; j < TE; ++j) part[g * kCols + j * kWave + lane] = pm[j];
    }
    __syncthreads();
    // With the column minimum known, a row's relative costs, clamped: all that its keys need.  A
    // row that is clamped in every reachable column of the tile is dropped; the others go on the
    // list (keys and strategy index), at the slot `counter` hands out.
    auto append_row = [&](int r, const Cell (&cells)[TE], uint32_t *counter) {
        uint32_t d[TE];
        bool live = false;
#pragma unroll
        for (int j = 0; j < TE; ++j) {
            const Cell rel = cells[j] - cmin[j];
            d[j] = (uint32_t)min(rel, (Cell)dmax);
            live |= rel < (Cell)dmax && cmin[j] < kInfCell;
        }
        if (__builtin_amdgcn_ballot_w64(live) != 0) {        // wave-uniform
            uint32_t slot = 0;
            if (lane == 0) slot = atomicAdd(counter, 1u);
            slot = (uint32_t)uniform((int)slot);
            if (slot < (uint32_t)kKeep) {
#pragma unroll
                for (int j = 0; j < TE; ++j) keys[slot * kCols + j * kWave + lane] = d[j] << k;
                // (broadcast with every lane active, not under the test for lane 0: a register
                // reloaded from a spill there holds lane 0's value only)
                const uint32_t sp_r = (uint32_t)read_lane(my_ent, r);
                if (lane == 0) meta[slot] = sp_r;
            }
        }
    };
    if (n > 0) {
#pragma unroll
        for (int w = 0; w < NG; ++w)
#pragma unroll
            for (int j = 0; j < TE; ++j) cmin[j] = min(cmin[j], part[w * kCols + j * kWave + lane]);
#pragma unroll
        for (int r = 0; r < TS; ++r)
            if (keep >> r & 1) append_row(r, rowc[r], count);   // listed (the padding repeats a listed row) and read
        if (g == 0 && lane == 0) count[1] = 0;     // the counter of the pass after this one
    }
    __syncthreads();

    // The list holds the rows that matter, or it has overflowed (transition costs that dwarf the
    // spread of the layer costs: few rows are clamped everywhere).  Then the rows go through the
    // list in passes, kRpw rows of every wave at a time, which always fit: each wave reads its
    // own rows of the pass again (once per workgroup, not once per wave), appends the live ones,
    // and every wave reduces that list.  Three counters take turns, so that the one a pass uses
    // was cleared while the pass before it was under way and after its last reader had gone.
    constexpr int kRpw = kKeep / NG;
    static_assert(kRpw >= 1, "one pass holds at least one row of every wave");
    __builtin_amdgcn_s_setprio(0);                 // from here on arithmetic: let the waves that fetch go first
    int cnt = n > 0 ? uniform((int)count[0]) : 0;
    int r_next = TS;                               // first row of the next pass; TS: no further pass
    if (cnt > kKeep) {
        r_next = 0;
        cnt = -1;                                  // nothing to reduce yet
    }
    uint32_t rows_reduced = 0;
    int pass = 0;
    for (;;) {
        if (cnt < 0) {                             // workgroup-uniform
            ++pass;
            uint32_t *counter = count + (pass % 3 == 2 ? 3 : pass % 3);
            if (g == 0 && lane == 0) count[(pass + 1) % 3 == 2 ? 3 : (pass + 1) % 3] = 0;
#pragma unroll
            for (int r = 0; r < TS; ++r)
                if (r >= r_next && r < r_next + kRpw && (keep >> r & 1)) {
                    Cell cells[TE];
                    load_row(read_lane(my_ent, r), read_lane(my_c0, r), cells);
                    append_row(r, cells, counter);
                }
            __syncthreads();
            cnt = uniform((int)counter[0]);        // at most NG * kRpw = kKeep
            r_next += kRpw;
        }
        rows_reduced += (uint32_t)cnt;
        if (s0 < S && cnt > 0) {                   // (an idle strategy group only contributes its rows)
            const int npair = (cnt + 1) / 2;       // an odd tail repeats its entry: min(x, x) = x
            uint32_t va[2][TE], vb[2][TE];
            int spa[2], spb[2];
            R32Row<TS> ra[2], rb[2];
            auto request = [&](int q, int pr) {
                const int ia = 2 * pr < cnt ? 2 * pr : cnt - 1;
                const int ib = 2 * pr + 1 < cnt ? 2 * pr + 1 : cnt - 1;
                spa[q] = uniform((int)meta[ia]);
                spb[q] = uniform((int)meta[ib]);
#pragma unroll
                for (int j = 0; j < TE; ++j) {
                    va[q][j] = keys[ia * kCols + j * kWave + lane];
                    vb[q][j] = keys[ib * kCols + j * kWave + lane];
                }
            };
            auto reduce_pair = [&](int q) {
                // keys of the next pair's rows, in flight under this pair's arithmetic
                ra[q ^ 1].request(Rk + (int64_t)uniform(spa[q ^ 1]) * a.S_pad);
                rb[q ^ 1].request(Rk + (int64_t)uniform(spb[q ^ 1]) * a.S_pad);
#pragma unroll
                for (int s = 0; s < TS; ++s)
                    minplus_u32x2<TE>(acc[s], va[q], vb[q], ra[q].at(s), rb[q].at(s), ra[q ^ 1], rb[q ^ 1]);
                r32_await(ra[q ^ 1], rb[q ^ 1]);
            };
            request(0, 0);
            request(1, 1);
            ra[0].request(Rk + (int64_t)uniform(spa[0]) * a.S_pad);
            rb[0].request(Rk + (int64_t)uniform(spb[0]) * a.S_pad);
            r32_await(ra[0], rb[0]);
            int pr = 0;
            for (; pr + 2 <= npair; pr += 2) {
                reduce_pair(0);
                request(0, pr + 2);
                reduce_pair(1);
                request(1, pr + 3);
            }
            if (pr < npair) reduce_pair(0);
        }
        if (r_next >= TS) break;
        __syncthreads();                           // the list is free again
        cnt = -1;
    }
    if (g == 0 && lane == 0) {                     // statistics: how much the pruning removed
        uint32_t *st = a.stats + 2 * (((int64_t)b * (a.L - 1) + (l - 1)) * a.n_tiles +
                                      (uint32_t)tile_start / (uint32_t)a.tile_e);
        const uint32_t rows = rows_reduced << 16 | (uint32_t)n;
        const uint32_t fetched = n > 0 ? count[2] : 0u;
        st[0] = add_stats ? st[0] + rows : rows;   // (a tile swept in several parts adds them up)
        st[1] = add_stats ? st[1] + fetched : fetched;
    }
    if (s0 >= S) return;                           // an idle strategy group has done its share of the rows

    const uint32_t mask = (1u << k) - 1u;
#pragma unroll
    for (int s = 0; s < TS; ++s) {
        if (s0 + s < S) {
            const Cell cs = (Cell)ck[s];
#pragma unroll
            for (int j = 0; j < TE; ++j) {
                const bool alive = cmin[j] < kInfCell;
                const uint32_t key = acc[s][j];
                // (wave-uniform row address + the lane's offset: no per-store address arithmetic)
                BP *bp_row = bp_tile + (int64_t)s * a.e_pad;
                if constexpr (PACK) {
                    // (a winning key is never all ones: the winner's relative cost is not clamped)
                    bp_row[(uint32_t)lane + j * kWave] = (BP)(alive ? key : 0xffffffffu);
                } else {
                    Cell *un_row = Un_tile + (int64_t)s * pitch;
                    un_row[(uint32_t)lane + j * kWave] = alive ? cmin[j] + (Cell)(key >> k) + cs : kInfCell;
                    __builtin_nontemporal_store((BP)(alive ? (int32_t)(key & mask) : -1),
                                                &bp_row[(uint32_t)lane + j * kWave]);
                }
            }
        }
    }
    if constexpr (PACK) {
        (void)mask;
        (void)Un_tile;
        if (g == 0) {
            // (of an unreachable column every word is all ones and this value is never used)
#pragma unroll
            for (int j = 0; j < TE; ++j) Mn_tile[(uint32_t)lane + j * kWave] = cmin[j];
        }
    }
}

// UX: the 32-bit-key body keeps half-size accumulators, so it may take UX (1 or 2) times
// the budget columns per lane; the 64-bit-key bodies then cover the same tile in UX steps.
// PACK (row-sharing variants with int32 back-pointers): the 32-bit-key instances keep the single
// packed table; the handle says so in Layout::packed and launches this instantiation.
template <int TS, int TE, int NG, int WPE, class BP, int W, int UX, int SHARE, int PACK>
__global__ __launch_bounds__(W * kWave, WPE) void sweep_kernel(Layout a, int l) {
    static_assert(!PACK || (SHARE && sizeof(BP) == 4), "the packed table needs the row-sharing body and 32-bit words");
    const int wave = uniform(threadIdx.x >> 6);    // the only use of the thread-index register (see lane_id)
    const int b = a.b_off + blockIdx.z * a.b_step;
    // The row-sharing body's list entries (see there): requested first, ahead of the header.
    uint64_t my_ent = 0, my_c0 = 0;
    if constexpr (SHARE != 0) {
        const int lane = lane_id();
        const int my_row = (lane & 31) < TS ? (lane & 31) : TS - 1;      // (idle lanes repeat the last row)
        const int64_t at = ((int64_t)b * a.L + (l - 1)) * a.S_pad + wave + NG * my_row;
        my_ent = a.vlist[at];
        my_c0 = a.vcost[at];
    }
    // One record holds what the workgroup needs to begin with.
    const ConstPtr<int32_t> hdr = as_const(a.hdr + ((int64_t)b * a.L + l) * 8);
    const int st = hdr[0];
    const int budget = hdr[1];
    const int n_prev = hdr[2];
    const uint32_t dmax = (uint32_t)hdr[3];
    const int r_sel = hdr[4];
    (void)n_prev, (void)dmax, (void)r_sel, (void)my_ent, (void)my_c0;
    if (st < 0) return;
#if GALV_XCD_MAP
    // Workgroups go round-robin to the 8 XCDs in the order of their linear index, and grid.x is
    // a multiple of 8, so blockIdx.x & 7 names the XCD.  Each XCD takes a contiguous eighth of
    // the tiles the instance needs: neighbouring tiles read overlapping cache lines of the
    // shifted former-layer rows, which then meet in one XCD's L2.
    const int nt = budget / a.tile_e + 1;
    const int per = (nt + 7) >> 3;
    if ((int)(blockIdx.x >> 3) >= per) return;
    const int64_t tile_start = (int64_t)((blockIdx.x & 7) * per + (blockIdx.x >> 3)) * a.tile_e;
#else
    const int64_t tile_start = (int64_t)blockIdx.x * a.tile_e;
#endif
    if (tile_start > budget) return;
    if (st == GALV_INSTANCE_OK_FAST_U32) {
        if constexpr (SHARE)
            sweep_u32_shared<TS, TE * UX, NG, BP, uint32_t, PACK != 0, keep_rows(TS, NG, WPE, kWave * TE * UX)>(a, wave, l, b, budget, tile_start, false, n_prev, dmax, r_sel, my_ent, my_c0);
        else
            sweep_u32<TS, TE * UX, NG, BP>(a, wave, l, b, budget, tile_start);
    } else if (st == GALV_INSTANCE_OK_U32_WIDE) {
        // 8-byte cells: half the tile's columns at a time keep the rows within the registers the narrow
        // form uses (the preparation kernel grants this path to row-sharing variants only)
        if constexpr (SHARE) {
            for (int h = 0; h < TE; ++h) {
                if (tile_start + h * (kWave * UX) > budget) break;   // workgroup-uniform
                if (h) __syncthreads();                              // the LDS of the part before is free again
                sweep_u32_shared<TS, UX, NG, BP, uint64_t, PACK != 0, keep_rows(TS, NG, WPE, kWave * TE * UX)>(a, wave, l, b, budget, tile_start + h * (kWave * UX), h > 0, n_prev, dmax, r_sel, my_ent, my_c0);
            }
        }
    } else if (st == GALV_INSTANCE_OK_FAST) {
        for (int h = 0; h < UX; ++h)
            sweep_fast<TS, TE, NG, Narrow, BP>(a, wave, l, b, budget, tile_start + h * (a.tile_e / UX));
    } else if (st == GALV_INSTANCE_OK_FAST_WIDE) {
        for (int h = 0; h < UX; ++h)
            sweep_fast<TS, TE, NG, Wide, BP>(a, wave, l, b, budget, tile_start + h * (a.tile_e / UX));
    } else {
        if (blockIdx.y == 0) sweep_int64<8>(a, wave, l, b, budget, tile_start);
    }
}

// ------------------------------------------------- final minimum and backtrack

// C[L-1][e][s] from the un-shifted last row, as an integer (GALV_INF if none).
__device__ __forceinline__ int64_t last_layer_cost(const Layout &a, int b, int st, int64_t e,
                                                   int64_t s) {
    const int64_t shift = a.m[((int64_t)b * a.L + (a.L - 1)) * a.S + s];
    if (shift > e) return kInf;
    if (is_packed(a, st)) {
        // U_{L-1}[e'][s] = Cmin[e'] + (key >> k) + c(L-1, s) with e' = e - shift
        const int64_t x = e - shift;
        const uint32_t w = static_cast<const uint32_t *>(a.bp)[(((int64_t)b * (a.L - 1) + (a.L - 2)) * a.S + s) * a.e_pad + x];
        if (w == 0xffffffffu) return kInf;
        const char *M = a.U[(a.L - 1) & 1] + (int64_t)b * a.S_pad * a.row * 8;
        const int64_t cmin = st == GALV_INSTANCE_OK_U32_WIDE ? (int64_t)reinterpret_cast<const uint64_t *>(M)[x]
                                                             : (int64_t)reinterpret_cast<const uint32_t *>(M)[x];
        return cmin + (int64_t)(w >> a.k_bits) + a.c[((int64_t)b * a.L + (a.L - 1)) * a.S + s];
    }
    const char *U = a.U[(a.L - 1) & 1] + ((int64_t)b * a.S_pad + s) * a.row * 8;
    const int64_t x = a.lead + e - shift;
    if (narrow_cells(st))
        return Narrow::to_int64(reinterpret_cast<const uint32_t *>(U)[x], a.k_bits);
    if (st == GALV_INSTANCE_OK_FAST_WIDE)
        return Wide::to_int64(reinterpret_cast<const double *>(U)[x], a.k_bits);
    if (st == GALV_INSTANCE_OK_U32_WIDE) {
        const uint64_t v = reinterpret_cast<const uint64_t *>(U)[x];
        return v >= (uint64_t)kInf ? kInf : (int64_t)v;
    }
    return reinterpret_cast<const int64_t *>(U)[x];
}

// One workgroup per instance: min over s at e = budget, lowest s first.
__global__ __launch_bounds__(kThreads) void final_kernel(Layout a, int64_t *best_cost,
                                                         int32_t *best_last) {
    const int b = blockIdx.x;
    const int st = uniform(a.status[b]);
    __shared__ int64_t val[kMaxS];
    if (st >= 0) {
        const int budget = uniform(a.budget[b]);
        for (int s = threadIdx.x; s < a.S; s += kThreads) val[s] = last_layer_cost(a, b, st, budget, s);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t opt = kInf;
        int32_t last = -1;
        if (st >= 0)
            for (int s = 0; s < a.S; ++s)
                if (val[s] < opt) {
                    opt = val[s];
                    last = s;
                }
        best_cost[b] = opt;
        best_last[b] = last;
        a.last[b] = last;
        // every block of init_kernel has long finished: safe to record what the leads hold
        // (a packed instance keeps its column minima where the first row's lead was)
        a.lead_mode[b] = st < 0 || is_packed(a, st) ? 0 : lead_kind(st);
    }
}

// Walk the un-shifted argmin table of instance b from (L-1, e, s) down to layer 0:
// L dependent loads.  Writes the plan, or all -1 when s < 0.
__device__ __forceinline__ void walk_plan(const Layout &a, int b, int64_t e, int s, int32_t *out) {
    const int st = a.status[b];
    if (s < 0) {
        for (int l = 0; l < a.L; ++l) out[l] = -1;
        return;
    }
    for (int l = a.L - 1; l >= 1; --l) {
        out[l] = s;
        e -= a.m[((int64_t)b * a.L + l) * a.S + s];
        // A reachable cell always points at a reachable cell; the guard only keeps
        // the walk inside the table if that invariant were ever broken.
        if (e < 0 || e > a.E_max) {
            for (int q = 0; q < a.L; ++q) out[q] = -1;
            return;
        }
        s = load_bp(a, st, (((int64_t)b * (a.L - 1) + (l - 1)) * a.S + s) * a.e_pad + e);
        if (s < 0 || s >= a.S) {
            for (int q = 0; q < a.L; ++q) out[q] = -1;
            return;
        }
    }
    out[0] = s;
}

// Per instance: the tiles' (rows reduced, rows listed) summed over the tiles within the budget
// and the layers; zeros for an instance that is not on the 32-bit-key path.
__global__ __launch_bounds__(kThreads) void stats_kernel(Layout a, int64_t *out) {
    const int b = blockIdx.x;
    __shared__ unsigned long long red[3][kThreads];
    unsigned long long done = 0, listed = 0, fetched = 0;
    if (a.status[b] == GALV_INSTANCE_OK_FAST_U32 || a.status[b] == GALV_INSTANCE_OK_U32_WIDE) {
        const int nt = a.budget[b] / a.tile_e + 1;
        for (int64_t i = threadIdx.x; i < (int64_t)(a.L - 1) * nt; i += kThreads) {
            const uint32_t *v = a.stats + 2 * (((int64_t)b * (a.L - 1) + i / nt) * a.n_tiles + i % nt);
            done += v[0] >> 16;
            listed += v[0] & 0xffffu;
            fetched += v[1];
        }
    }
    red[0][threadIdx.x] = done;
    red[1][threadIdx.x] = listed;
    red[2][threadIdx.x] = fetched;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w)
            for (int q = 0; q < 3; ++q) red[q][threadIdx.x] += red[q][threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0)
        for (int q = 0; q < 3; ++q) out[3 * b + q] = (int64_t)red[q][0];
}

// One wave per instance, from the full budget and the stored best last strategy.  The walk is
// a chain of dependent loads, two per layer (the memory of the chosen strategy, then the
// back-pointer it leads to); when the instance's memory table fits LDS the wave copies it there
// first, coalesced, which leaves one global load per layer in the chain.
constexpr int kWalkLds = 16384;                  // int32 words of m(l, s) kept in LDS
__global__ __launch_bounds__(kWave) void backtrack_kernel(Layout a, int32_t *plan) {
    const int b = blockIdx.x;
    __shared__ int32_t m_lds[kWalkLds];
    const int64_t n = (int64_t)a.L * a.S;
    const int32_t *m = a.m + (int64_t)b * n;
    const bool in_lds = n <= kWalkLds;
    int s = a.last[b];
    if (in_lds && s >= 0)
        for (int64_t i = threadIdx.x; i < n; i += kWave) m_lds[i] = m[i];
    __syncthreads();
    if (threadIdx.x != 0) return;
    int32_t *out = plan + (int64_t)b * a.L;
    if (!in_lds || s < 0) {
        walk_plan(a, b, a.budget[b], s, out);
        return;
    }
    int64_t e = a.budget[b];
    const int st = a.status[b];
    for (int l = a.L - 1; l >= 1; --l) {
        out[l] = s;
        e -= m_lds[(int64_t)l * a.S + s];
        if (e < 0 || e > a.E_max) {             // cannot happen for a reachable cell; keeps the walk inside the table
            for (int q = 0; q < a.L; ++q) out[q] = -1;
            return;
        }
        s = load_bp(a, st, (((int64_t)b * (a.L - 1) + (l - 1)) * a.S + s) * a.e_pad + e);
        if (s < 0 || s >= a.S) {
            for (int q = 0; q < a.L; ++q) out[q] = -1;
            return;
        }
    }
    out[0] = s;
}

// min_s C[L-1][e][s] and the lowest minimising s for one (instance, budget column).
__device__ __forceinline__ void best_at(const Layout &a, int b, int st, int64_t e, int64_t &opt,
                                        int32_t &last) {
    opt = kInf;
    last = -1;
    for (int s = 0; s < a.S; ++s) {
        const int64_t v = last_layer_cost(a, b, st, e, s);
        if (v < opt) {
            opt = v;
            last = s;
        }
    }
}

// The optimum of every budget column.  Grid: (column tiles, B).
__global__ __launch_bounds__(kThreads) void best_per_budget_kernel(Layout a, int64_t *best_cost,
                                                                   int32_t *best_last) {
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e > a.E_max) return;
    const int b = blockIdx.y;
    const int st = uniform(a.status[b]);
    int64_t opt = kInf;
    int32_t last = -1;
    if (st >= 0 && e <= a.budget[b]) best_at(a, b, st, e, opt, last);
    best_cost[(int64_t)b * (a.E_max + 1) + e] = opt;
    if (best_last) best_last[(int64_t)b * (a.E_max + 1) + e] = last;
}

// One thread per (instance, budget) query: final minimum at that column, then the walk.
__global__ __launch_bounds__(kWave) void backtrack_queries_kernel(Layout a, int n, const int32_t *inst,
                                                                  const int32_t *budgets,
                                                                  int64_t *cost, int32_t *plan) {
    const int q = blockIdx.x * kWave + threadIdx.x;
    if (q >= n) return;
    const int b = inst[q];
    const int64_t e = budgets[q];
    int64_t opt = kInf;
    int32_t last = -1;
    if (b >= 0 && b < a.B) {
        const int st = uniform(a.status[b]);
        if (st >= 0 && e >= 0 && e <= a.budget[b]) best_at(a, b, st, e, opt, last);
    }
    if (cost) cost[q] = opt;
    walk_plan(a, b < 0 || b >= a.B ? 0 : b, e, last, plan + (int64_t)q * a.L);
}

// Canonical-order tables of one instance.  Grid: (e tiles, L + 1); row L of the
// grid writes C_last, rows 0..L-1 write the back-pointers of that layer.
__global__ __launch_bounds__(kThreads) void export_kernel(Layout a, int b, int64_t *C_last,
                                                          int32_t *bp_out) {
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e > a.E_max) return;
    const int l = blockIdx.y;
    const int st = uniform(a.status[b]);
    const int budget = uniform(a.budget[b]);
    const bool live = st >= 0 && e <= budget;
    if (l == a.L) {
        for (int s = 0; s < a.S; ++s)
            C_last[e * a.S + s] = live ? last_layer_cost(a, b, st, e, s) : kInf;
        return;
    }
    if (!bp_out) return;
    int32_t *dst = bp_out + ((int64_t)l * (a.E_max + 1) + e) * a.S;
    for (int s = 0; s < a.S; ++s) {
        int32_t v = -1;
        if (live && l >= 1) {
            const int64_t shift = a.m[((int64_t)b * a.L + l) * a.S + s];
            if (shift <= e)
                v = load_bp(a, st, (((int64_t)b * (a.L - 1) + (l - 1)) * a.S + s) * a.e_pad + (e - shift));
        }
        dst[s] = v;
    }
}

// -------------------------------------------------------------------- host side

// Sweep variants, in ascending order of the strategies one workgroup covers
// (TS * NG).  The first one that covers S is used; larger S use the last one with
// several strategy groups along grid.y.  <TS, TE, NG, WPE, W, UX, SHARE>: TS * TE running
// minima per lane (2 VGPRs each with 64-bit keys, 1 with 32-bit keys) for WPE resident
// waves per SIMD (512 VGPRs / WPE each), W waves per workgroup, UX times the columns for
// the 32-bit-key body, SHARE = 1 for the row-sharing 32-bit-key body (W == NG waves, each
// owning TS rows and TS strategies of one tile of 64 * TE * UX columns; it needs
// TS * NG >= S, so the last variant, which serves any S, uses the plain body; the one before
// it covers up to 256 strategies with 16-wave workgroups).
// Measured on MI355X: with the dominated rows pruned the sweep is bound by HBM, and tiles of
// 128 columns beat 64 (longer contiguous row segments) while larger register tiles gain
// nothing; 8 waves per SIMD do not build for TS = 16 (the compiler then spills scalar
// registers that a hand-issued load still targets, which the build refuses).
#ifndef GALV_V0
#define GALV_V0 8, 2, 1, 8, 1, 1, 1
#endif
#ifndef GALV_V1
#define GALV_V1 16, 2, 1, 6, 1, 1, 1
#endif
#ifndef GALV_V2
#define GALV_V2 11, 2, 2, 8, 2, 1, 1
#endif
#ifndef GALV_V3
#define GALV_V3 16, 2, 2, 6, 2, 1, 1
#endif
#ifndef GALV_V4
#define GALV_V4 11, 2, 4, 8, 4, 1, 1
#endif
#ifndef GALV_V5
#define GALV_V5 16, 2, 4, 6, 4, 1, 1
#endif
#ifndef GALV_V6
#define GALV_V6 16, 2, 8, 6, 8, 1, 1
#endif
#ifndef GALV_V7
#define GALV_V7 16, 2, 16, 4, 16, 1, 1
#endif
#ifndef GALV_V8
#define GALV_V8 16, 2, 8, 6, 8, 1, 0
#endif
// Twins with tiles of 256 budget columns (UX = 2: four columns per lane) and fewer, fatter waves,
// for launches that fill the chip anyway: what a tile costs beside its min-plus arithmetic (its
// chain of round trips, its addresses and bookkeeping) is spread over twice the states.
// Measured against the 128-column variants: 3.5 % (44 strategies x 32768 columns x 64 instances),
// 5 % (128 x 65536 x 16), 2 % (22 x 24576 x 32), 3-6 % at 32, 64, 200 and 256 strategies; 3 %
// slower on 22 x 16384 x 8, which does not fill the chip and keeps the narrow tiles.
#ifndef GALV_V2X
#define GALV_V2X 11, 2, 2, 5, 2, 2, 1
#endif
#ifndef GALV_V3X
#define GALV_V3X 16, 2, 2, 4, 2, 2, 1
#endif
#ifndef GALV_V4X
#define GALV_V4X 11, 2, 4, 5, 4, 2, 1
#endif
#ifndef GALV_V5X
#define GALV_V5X 16, 2, 4, 4, 4, 2, 1
#endif
#ifndef GALV_V6X
#define GALV_V6X 16, 2, 8, 4, 8, 2, 1
#endif
#ifndef GALV_V7X
#define GALV_V7X 16, 2, 16, 4, 16, 2, 1
#endif

// ---------------------------------------------------------------------------------------------
// Outer loop of Algorithm 1 over a window of batch sizes: per (batch size, pipeline degree) the
// stage optima are summed, the minimum over pipeline degrees is C_opt, and the scan over batch
// sizes keeps the largest B / C_opt until the first batch size that fits under no degree.
// One workgroup: the sums in parallel, the scan by one lane (it is a dependent chain).
struct PpList {
    int n;
    int degree[kMaxPp];
};

__global__ __launch_bounds__(kThreads) void alg1_reduce_kernel(
    int n_batch, PpList pp, const int64_t *__restrict__ stage_cost,
    const int64_t *__restrict__ batch_size, int batch_index_base, int first_window,
    int64_t *__restrict__ c_p, galv_alg1_state_t *__restrict__ state) {
    for (int i = threadIdx.x; i < n_batch * pp.n; i += kThreads) {
        const int ib = i / pp.n, ip = i % pp.n;
        size_t off = 0;
        for (int j = 0; j < ip; ++j) off += (size_t)n_batch * pp.degree[j];
        const int64_t *x = stage_cost + off + (size_t)ib * pp.degree[ip];
        int64_t acc = 0;
        for (int st = 0; st < pp.degree[ip]; ++st) {
            const int64_t v = x[st];
            acc = (acc >= kInf || v < 0 || v >= kInf - acc) ? kInf : acc + v;
        }
        c_p[i] = acc;
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    galv_alg1_state_t s;
    if (first_window) {
        s.batch_size = 0; s.cost = 1; s.pp_index = -1; s.batch_index = -1;
        s.stopped = 0; s.n_explored = 0;
    } else {
        s = *state;
    }
    for (int ib = 0; ib < n_batch && !s.stopped; ++ib) {
        int64_t c_opt = kInf;
        int arg = -1;
        for (int ip = 0; ip < pp.n; ++ip) {
            const int64_t v = c_p[(size_t)ib * pp.n + ip];
            if (v < c_opt) { c_opt = v; arg = ip; }
        }
        if (arg < 0) { s.stopped = 1; break; }          // Out-Of-Memory under every degree
        ++s.n_explored;
        const int64_t bsz = batch_size[ib];
        // bsz / c_opt > s.batch_size / s.cost, compared exactly as cross products
        const unsigned __int128 lhs = (unsigned __int128)(uint64_t)bsz * (uint64_t)s.cost;
        const unsigned __int128 rhs = (unsigned __int128)(uint64_t)s.batch_size * (uint64_t)c_opt;
        if (bsz > 0 && lhs > rhs) {
            s.batch_size = bsz; s.cost = c_opt; s.pp_index = arg;
            s.batch_index = batch_index_base + ib;
        }
    }
    *state = s;
}


// ---------------------------------------------------------------------------------------------
// Coarse-grained exploration (complexity remark at the end of section 3.3): `fuse` consecutive
// layers become one layer that runs a single strategy, and memory is counted in units `gran`
// times larger.  One thread per (instance, fused layer, strategy).
__global__ __launch_bounds__(kThreads) void coarsen_kernel(
    int B, int L, int S, int nR, int fuse, int gran, int Lc, const int64_t *__restrict__ c,
    const int32_t *__restrict__ m, const int64_t *__restrict__ R, const int32_t *__restrict__ r_idx,
    const int32_t *__restrict__ budget, int64_t *__restrict__ c_out, int32_t *__restrict__ m_out,
    int32_t *__restrict__ r_idx_out, int32_t *__restrict__ budget_out) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= (int64_t)B * Lc * S) return;
    const int s = (int)(i % S);
    const int j = (int)((i / S) % Lc);
    const int b = (int)(i / ((int64_t)S * Lc));
    const int lo = j * fuse, hi = min(L, lo + fuse);
    const int E = budget[b];
    int64_t cost = 0, mem = 0;
    bool unusable = false, bad_c = false, bad_m = false;   // invalid inputs stay invalid for the solver
    for (int l = lo; l < hi; ++l) {
        const int64_t at = ((int64_t)b * L + l) * S + s;
        const int64_t cl = c[at];
        bad_c |= cl < 0 || cl >= kInf;
        cost += bad_c ? 0 : cl;
        if (l > lo) {
            const int r = r_idx ? r_idx[(int64_t)b * L + l] : 0;
            const int64_t rr = (r < 0 || r >= nR) ? -1 : R[(((int64_t)b * nR + r) * S + s) * S + s];
            bad_c |= rr < 0 || rr >= kInf;
            cost += bad_c ? 0 : rr;
        }
        bad_c |= cost >= kInf;
        const int32_t ml = m[at];
        bad_m |= ml < 0;
        unusable |= ml > E;
        mem += ml;
    }
    const int64_t units = (mem + gran - 1) / gran;       // rounded up: a coarse plan that fits, fits
    const int32_t Ec = E < 0 ? -1 : E / gran;
    const int32_t over = Ec < INT32_MAX ? Ec + 1 : INT32_MAX;
    c_out[i] = bad_c ? -1 : cost;
    m_out[i] = bad_m ? -1 : ((unusable || units > Ec) ? over : (int32_t)units);
    if (s == 0) {
        r_idx_out[(int64_t)b * Lc + j] = r_idx ? r_idx[(int64_t)b * L + lo] : 0;
        if (j == 0) budget_out[b] = Ec;
    }
}

__global__ __launch_bounds__(kThreads) void expand_plan_kernel(int B, int L, int fuse, int Lc,
                                                               const int32_t *__restrict__ coarse,
                                                               int32_t *__restrict__ plan) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= (int64_t)B * L) return;
    const int b = (int)(i / L), l = (int)(i % L);
    plan[i] = coarse[(int64_t)b * Lc + l / fuse];
}

using SweepFn = void (*)(Layout, int);
struct VariantEntry {
    Variant v;
    SweepFn fn, fn_u8;     // int32 and one-byte back-pointers
    SweepFn fn_pack;       // int32, single packed table (row-sharing variants; else null)
};
template <int TS, int TE, int NG, int WPE, int W, int UX, int SHARE>
VariantEntry variant_entry() {
    static_assert((W == 1 || W == 2 || W == 3 || W == 4 || W == 6 || W == 8 || W == 16) && W % NG == 0,
                  "strategy groups must divide the workgroup's waves");
    static_assert(!SHARE || W == NG, "the row-sharing body has one budget tile per workgroup");
    static_assert((UX == 1 || UX == 2) && TE * UX <= 4, "budget columns per lane");
    SweepFn pack = nullptr;
    if constexpr (SHARE != 0) pack = sweep_kernel<TS, TE, NG, WPE, int32_t, W, UX, SHARE, 1>;
    return {{TS, TE, NG, W, UX, WPE, SHARE},
            sweep_kernel<TS, TE, NG, WPE, int32_t, W, UX, SHARE, 0>,
            sweep_kernel<TS, TE, NG, WPE, uint8_t, W, UX, SHARE, 0>,
            pack};
}

// `wide_tiles`: the launch fills the chip; take the 256-column twin where there is one.
const VariantEntry &pick_variant(int S, bool wide_tiles) {
    static const VariantEntry table[] = {
        variant_entry<GALV_V0>(), variant_entry<GALV_V1>(), variant_entry<GALV_V2>(),
        variant_entry<GALV_V3>(), variant_entry<GALV_V4>(), variant_entry<GALV_V5>(),
        variant_entry<GALV_V6>(), variant_entry<GALV_V7>(), variant_entry<GALV_V8>()};
    static const VariantEntry twins[] = {
        variant_entry<GALV_V2X>(), variant_entry<GALV_V3X>(), variant_entry<GALV_V4X>(),
        variant_entry<GALV_V5X>(), variant_entry<GALV_V6X>(), variant_entry<GALV_V7X>()};
    constexpr int n = sizeof table / sizeof table[0];
    for (int i = 0; i < n; ++i)
        if (S <= table[i].v.ts * table[i].v.ng) {
            if (wide_tiles)
                for (const VariantEntry &t : twins)
                    if (t.v.ts == table[i].v.ts && t.v.ng == table[i].v.ng) return t;
            return table[i];
        }
    return table[n - 1];
}

}  // namespace

struct galv_dp {
    galv_dp_desc_t desc;
    Variant var;
    SweepFn sweep;
    Layout lay;        // workspace pointers filled, input pointers set per solve
    size_t ws_bytes;
    int groups_y;      // grid.y of the sweep
    unsigned lds_bytes; // dynamic LDS of a sweep workgroup (staging variants only)
    bool lds_allowed;   // the kernel has been told that it may use that much
    bool solved;
    bool fresh;         // no solve has run over this workspace yet: the infinity leads are unwritten
    int n_side;                    // side streams the handle owns (0 or >= 2); a solve uses some or all of them
    bool auto_streams;             // the solve picks how many (else: all of them, as the caller asked)
    int n_used;                    // how many the last solve used (0: none has run)
    int resident;                  // sweep workgroups the GPU holds at a time
    int32_t *seen_host;            // pinned: budget tiles of the batch as the last solve's prep_kernel found them
    hipStream_t side[kMaxSide];
    hipEvent_t fork, join[kMaxSide];
};

namespace {

struct Plan {
    Variant var;
    SweepFn sweep;
    Layout lay;
    size_t off_U[2], off_bp, off_Rk, off_ck, off_vlist, off_vcost, off_nvalid, off_hdr, off_status, off_last, off_dclamp,
        off_lead_mode, off_stats, total;
    int groups_y;
    unsigned lds_bytes;
};

galv_status_t make_plan(const galv_dp_desc_t *d, Plan *p) {
    if (!d) return fail(GALV_ERR_INVALID_ARG, "desc is NULL");
    if (d->n_instances < 1 || d->n_layers < 1 || d->n_strategies < 1 || d->max_budget < 0 ||
        d->n_transition < 1)
        return fail(GALV_ERR_INVALID_ARG,
                    "desc: need n_instances>=1, n_layers>=1, n_strategies>=1, max_budget>=0, "
                    "n_transition>=1 (got %d %d %d %d %d)",
                    d->n_instances, d->n_layers, d->n_strategies, d->max_budget, d->n_transition);
    if (d->n_strategies > kMaxS)
        return fail(GALV_ERR_INVALID_ARG, "n_strategies %d exceeds the limit %d", d->n_strategies,
                    kMaxS);
    if (d->flags & ~(GALV_DP_FORCE_INT64 | GALV_DP_BP_U8 | GALV_DP_NO_U32 | GALV_DP_NO_PEEK | GALV_DP_FORCE_PEEK |
                     GALV_DP_NO_PACK | GALV_DP_FORCE_PACK | GALV_DP_FORCE_WIDE_TILES | GALV_DP_NO_WIDE_TILES |
                     GALV_DP_STREAMS_MASK))
        return fail(GALV_ERR_INVALID_ARG, "unknown flag bits");
    if (((d->flags & GALV_DP_STREAMS_MASK) >> GALV_DP_STREAMS_SHIFT) > (uint32_t)kMaxSide)
        return fail(GALV_ERR_INVALID_ARG, "at most %d internal streams", kMaxSide);
    const bool u8 = (d->flags & GALV_DP_BP_U8) != 0;
    if (u8 && d->n_strategies > 255)
        return fail(GALV_ERR_INVALID_ARG, "one-byte back-pointers need n_strategies <= 255 (got %d)",
                    d->n_strategies);
    if (d->n_instances > 65535)
        return fail(GALV_ERR_RANGE, "n_instances %d exceeds the grid limit 65535", d->n_instances);
    if (d->max_budget > (1 << 30))
        return fail(GALV_ERR_RANGE, "max_budget %d exceeds 2^30", d->max_budget);

    memset(p, 0, sizeof *p);
    // enough workgroups per layer to fill the chip several times over (counted in 128-column tiles)?
    const bool fills_chip = ((int64_t)d->max_budget / 128 + 1) * d->n_instances >= 3072;
    const bool wide_tiles = (fills_chip || (d->flags & GALV_DP_FORCE_WIDE_TILES)) && !(d->flags & GALV_DP_NO_WIDE_TILES);
    const VariantEntry &ve = pick_variant(d->n_strategies, wide_tiles);
    const Variant v = ve.v;
    Layout &a = p->lay;
    a.B = d->n_instances;
    a.L = d->n_layers;
    a.S = d->n_strategies;
    a.E_max = d->max_budget;
    a.nR = d->n_transition;
    a.bp_u8 = u8 ? 1 : 0;
    a.synth_l1 = v.share ? 1 : 0;
    const int group = v.ts * v.ng;
    p->groups_y = (a.S + group - 1) / group;
    a.S_pad = p->groups_y * group;
    int k = 1;               // at least one index bit: the key builders shift by 32 - k
    while ((1 << k) < a.S) ++k;
    a.k_bits = k;
    a.tile_e = kWave * v.te * v.ux * (v.w / v.ng);
    // row-sharing body: partial minima [NG][columns], counters, keep_rows rows of (strategy index, keys), [NG] minima
    p->lds_bytes = 0;
    if (v.share) {
        const size_t cols = (size_t)kWave * v.te * v.ux, keep = keep_rows(v.ts, v.ng, v.wpe, (int)cols);
        const size_t narrow = ((size_t)v.ng * cols + v.ng + 4 + keep + keep * cols) * sizeof(uint32_t);
        // the 8-byte-cell form works on a part of the tile (64 x ux columns) at a time
        const size_t wcols = (size_t)kWave * v.ux;
        const size_t wide = ((size_t)v.ng * wcols + v.ng) * sizeof(uint64_t) + (4 + keep + keep * wcols) * sizeof(uint32_t);
        p->lds_bytes = (unsigned)(narrow > wide ? narrow : wide);
    }
    if (p->lds_bytes > 160u * 1024u)
        return fail(GALV_ERR_RANGE, "internal: staging variant needs %u bytes of LDS", p->lds_bytes);
    a.e_pad = (int64_t)round_up((size_t)a.E_max + 1, kEAlign);
    a.n_tiles = (int32_t)((a.E_max + a.tile_e) / a.tile_e);   // ceil((E_max+1)/tile_e)
    // measured: with ~1000 workgroups per layer (config 1) the peek costs 9 %, with ~6000 (config 2) it gains 14 %
    a.peek = fills_chip ? 1 : 0;
    if (d->flags & GALV_DP_NO_PEEK) a.peek = 0;
    if (d->flags & GALV_DP_FORCE_PEEK) a.peek = 1;
    // The single packed table halves the bytes of a state but rebuilds every cell it reads from
    // two loads: measured, it gains 15-25 % where the peek leaves few rows to read (configs 2-4)
    // and loses 15 % where every row is read and latency binds (config 1): same switch as the peek.
    bool packed = v.share && !u8 && fills_chip;
    if (d->flags & GALV_DP_NO_PACK) packed = false;
    if ((d->flags & GALV_DP_FORCE_PACK) && v.share && !u8) packed = true;
    p->sweep = packed ? ve.fn_pack : (u8 ? ve.fn_u8 : ve.fn);
    a.packed = packed ? 1 : 0;
    a.seen = nullptr;
    a.lead = (int64_t)round_up((size_t)a.E_max + 1, 64);
    a.row = a.lead + a.e_pad;
    p->var = v;

    // Sizes in long double first, to reject anything that would overflow size_t math.
    const long double approx = (long double)a.B * a.S_pad * a.row * 16 +
                               (long double)a.B * (a.L - 1) * a.S * a.e_pad * (u8 ? 1 : 4) +
                               (long double)a.B * a.nR * a.S * a.S_pad * 8;
    if (approx > 1e15L) return fail(GALV_ERR_RANGE, "tables of %.3Lg bytes cannot be indexed", approx);

    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = round_up(off + bytes, 256);
        return at;
    };
    const size_t u_bytes = (size_t)a.B * a.S_pad * a.row * 8;
    p->off_U[0] = take(u_bytes);
    p->off_U[1] = take(u_bytes);
    p->off_bp = take((size_t)a.B * (a.L - 1) * a.S * a.e_pad * (u8 ? 1 : sizeof(int32_t)));
    // + slack: a group of R keys is fetched whole even when it straddles the row end
    p->off_Rk = take((size_t)a.B * a.nR * a.S * a.S_pad * sizeof(double) + 1024);
    p->off_ck = take((size_t)a.B * a.L * a.S_pad * sizeof(uint64_t));
    p->off_vlist = take((size_t)a.B * a.L * a.S_pad * sizeof(uint64_t) + 64);   // + slack: entries are fetched eight at a time
    p->off_vcost = take((size_t)a.B * a.L * a.S_pad * sizeof(uint64_t) + 64);
    p->off_nvalid = take((size_t)a.B * a.L * sizeof(int32_t));
    p->off_status = take((size_t)a.B * sizeof(int32_t));
    p->off_last = take((size_t)a.B * sizeof(int32_t));
    p->off_dclamp = take((size_t)a.B * sizeof(uint32_t));
    p->off_hdr = take((size_t)a.B * a.L * 8 * sizeof(int32_t));
    p->off_lead_mode = take((size_t)a.B * sizeof(int32_t));
    p->off_stats = take((size_t)a.B * (a.L > 1 ? a.L - 1 : 1) * a.n_tiles * 2 * sizeof(uint32_t));
    p->total = off;
    return GALV_OK;
}

// grid.x of a sweep launch for n budget tiles.
inline unsigned kGridTiles(int n) { return GALV_XCD_MAP ? (unsigned)((n + 7) / 8 * 8) : (unsigned)n; }

// Point a layout's table pointers into a workspace laid out by make_plan.
void bind_workspace(Layout &a, const Plan &p, char *ws) {
    a.U[0] = ws + p.off_U[0];
    a.U[1] = ws + p.off_U[1];
    a.bp = ws + p.off_bp;
    a.Rk = reinterpret_cast<double *>(ws + p.off_Rk);
    a.ck = reinterpret_cast<uint64_t *>(ws + p.off_ck);
    a.vlist = reinterpret_cast<uint64_t *>(ws + p.off_vlist);
    a.vcost = reinterpret_cast<uint64_t *>(ws + p.off_vcost);
    a.nvalid = reinterpret_cast<int32_t *>(ws + p.off_nvalid);
    a.status = reinterpret_cast<int32_t *>(ws + p.off_status);
    a.last = reinterpret_cast<int32_t *>(ws + p.off_last);
    a.dclamp = reinterpret_cast<uint32_t *>(ws + p.off_dclamp);
    a.hdr = reinterpret_cast<int32_t *>(ws + p.off_hdr);
    a.lead_mode = reinterpret_cast<int32_t *>(ws + p.off_lead_mode);
    a.stats = reinterpret_cast<uint32_t *>(ws + p.off_stats);
}

// How many internal streams a solve deals its instances over, given the budget tiles (sweep
// workgroups per strategy group and layer) of the whole batch.  Measured on MI355X with 4 hardware
// queues: the sweeps run fastest when one launch holds about two thirds of the workgroups the GPU
// can keep resident, so that launches of different streams overlap in different phases (loads of
// one under the arithmetic and stores of another) -- 64 instances of 44 strategies: 5-6 streams
// for 4096 tiles, 6 for 5150, 9-10 for 8192, each 5-15 % ahead of two streams more or fewer; as
// long as a launch still takes ~12 us (shorter ones are bound by the launch rate: 32 instances of
// 22 strategies x 24576 columns take 1.16 / 1.20 / 1.70 ms with 2 / 3 / 4 streams).  A stream that
// holds two instances where others hold one sets the pace, so when most streams would hold a
// single instance every instance gets its own (16 instances of 128 strategies x 65536 columns:
// 20.3 ms with 16 streams, 21.2 with 12, 22.1 with 11).
int pick_streams(const galv_dp *h, int64_t tiles) {
    if (h->n_side <= 1) return 1;
    if (!h->auto_streams) return h->n_side;
    const Layout &a = h->lay;
    const double wgs = (double)tiles * h->groups_y;
    int n = (int)(wgs / (0.66 * h->resident) + 0.5);
    const double us = (double)tiles * a.tile_e * a.S * 8.0 / 5.5e12 * 1e6;   // a layer at 8 B per state
    if (n > (int)(us / 12.0)) n = (int)(us / 12.0);
    if (2 * n > a.B) n = a.B;
    if (n > h->n_side) n = h->n_side;
    return n < 1 ? 1 : n;
}
int64_t tiles_at_most(const galv_dp *h) { return (int64_t)h->lay.B * (h->lay.E_max / h->lay.tile_e + 1); }

// Enqueue one whole solve (preparation, layer 0, the L-1 sweeps, final minimum) of handle h on
// stream st.  Shared by every entry point that solves.
galv_status_t enqueue_solve(galv_dp *h, const int64_t *c_dev, const int32_t *m_dev,
                            const int64_t *R_dev, const int32_t *r_idx_dev,
                            const int32_t *budget_dev, int64_t *best_cost_dev,
                            int32_t *best_last_dev, hipStream_t st) {
    Layout &a = h->lay;
    a.c = c_dev;
    a.m = m_dev;
    a.R = R_dev;
    a.r_idx = r_idx_dev;
    a.budget = budget_dev;
    h->solved = false;

    if (!h->lds_allowed) {     // more than the default 64 KB of dynamic LDS: say so before any launch
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(h->sweep),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)h->lds_bytes));
        h->lds_allowed = true;
    }
    // (the budgets are on the device: what an earlier solve's preparation reported stands in for
    // them, and the largest possible count before any has; read before this solve's own
    // preparation is launched, so that the choice does not depend on how fast that one runs)
    const int32_t seen = h->seen_host ? *static_cast<volatile int32_t *>(h->seen_host) : 0;
    const int n_use = a.L < 2 ? 1 : pick_streams(h, seen > 0 ? seen : tiles_at_most(h));
    h->n_used = n_use;
    prep_kernel<<<a.B, kPrepThreads, 0, st>>>(a, h->desc.flags);
    {
        // at most 16 cells per thread: enough blocks to write a row at full rate, few enough to cost
        // nothing when, as usual after a handle's first solve, there is nothing to write
        const int64_t blocks = (a.row + 16 * kThreads - 1) / (16 * kThreads);
        init_kernel<<<dim3((unsigned)blocks, a.S, a.B), kThreads, 0, st>>>(a, h->fresh ? 1 : 0);
    }
    a.b_off = 0;
    a.b_step = 1;
    if (n_use <= 1) {
        const dim3 grid(kGridTiles(a.n_tiles), h->groups_y, a.B);
        for (int l = 1; l < a.L; ++l) h->sweep<<<grid, h->var.w * kWave, h->lds_bytes, st>>>(a, l);
    } else {
        // Instances are independent, so their layer chains need no common barrier: each
        // side stream sweeps its own share of the instances (dealt round-robin, which balances
        // unequal budgets) and the shares overlap freely.
        HIP_TRY(hipEventRecord(h->fork, st));
        // A failure after the fork must not leave side streams running behind the caller's
        // back: whatever was started is still joined into `st` before the error is returned.
        hipError_t err = hipSuccess;
        for (int g = 0; g < n_use && err == hipSuccess; ++g) {
            const int count = (a.B - g + n_use - 1) / n_use;            // instances g, g + n, g + 2n, ...
            if (count <= 0) continue;
            err = hipStreamWaitEvent(h->side[g], h->fork, 0);
            if (err != hipSuccess) break;                 // nothing enqueued on this side stream
            Layout ag = a;
            ag.b_off = g;
            ag.b_step = n_use;
            const dim3 grid(kGridTiles(a.n_tiles), h->groups_y, count);
            for (int l = 1; l < a.L; ++l) h->sweep<<<grid, h->var.w * kWave, h->lds_bytes, h->side[g]>>>(ag, l);
            err = hipEventRecord(h->join[g], h->side[g]);
            const hipError_t e2 = err == hipSuccess ? hipStreamWaitEvent(st, h->join[g], 0) : err;
            if (e2 != hipSuccess) {
                // could not order `st` after this side stream: wait for it on the host instead
                (void)hipStreamSynchronize(h->side[g]);
                err = e2;
            }
        }
        if (err != hipSuccess)
            return fail(GALV_ERR_HIP, "forking the layer sweeps over internal streams failed: %s",
                        hipGetErrorString(err));
    }
    final_kernel<<<a.B, kThreads, 0, st>>>(a, best_cost_dev, best_last_dev);
    HIP_TRY(hipGetLastError());
    h->solved = true;
    h->fresh = false;
    return GALV_OK;
}

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];       // device address of `scratch` on each GPU, once known
std::mutex g_scratch_mutex;

// Device address of the current GPU's copy of `scratch`, looked up on the first call per device.
galv_status_t static_scratch(void **out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(GALV_ERR_RANGE, "device ordinal %d is outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || reinterpret_cast<uintptr_t>(ptr) % 256 != 0)
            return fail(GALV_ERR_HIP, "the static workspace has no usable device address (%p)", ptr);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return GALV_OK;
}


}  // namespace

extern "C" {

galv_status_t galv_dp_workspace_bytes(const galv_dp_desc_t *desc, size_t *bytes) {
    if (!bytes) return fail(GALV_ERR_INVALID_ARG, "bytes is NULL");
    Plan p;
    galv_status_t st = make_plan(desc, &p);
    if (st != GALV_OK) return st;
    *bytes = p.total;
    return GALV_OK;
}

galv_status_t galv_dp_create(const galv_dp_desc_t *desc, void *workspace_dev,
                             size_t workspace_bytes, galv_dp_t **out) {
    if (!out) return fail(GALV_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    Plan p;
    galv_status_t st = make_plan(desc, &p);
    if (st != GALV_OK) return st;
    if (!workspace_dev) return fail(GALV_ERR_WORKSPACE, "workspace is NULL");
    if (reinterpret_cast<uintptr_t>(workspace_dev) % 256 != 0)
        return fail(GALV_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (workspace_bytes < p.total)
        return fail(GALV_ERR_WORKSPACE, "workspace of %zu bytes is smaller than the %zu needed",
                    workspace_bytes, p.total);

    galv_dp *h = new (std::nothrow) galv_dp;
    if (!h) return fail(GALV_ERR_INVALID_ARG, "out of host memory");
    h->desc = *desc;
    h->var = p.var;
    h->sweep = p.sweep;
    h->lay = p.lay;
    h->ws_bytes = p.total;
    h->groups_y = p.groups_y;
    h->lds_bytes = p.lds_bytes;
    h->lds_allowed = p.lds_bytes <= 64u * 1024u;
    if (!h->lds_allowed) {
        // More than the default 64 KB of dynamic LDS: the kernel is told here, once, rather than at
        // the first solve, which a caller may be capturing into a graph.  (Should this fail, the
        // solve tries again and reports it.)
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(h->sweep), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)h->lds_bytes) == hipSuccess)
            h->lds_allowed = true;
        else
            (void)hipGetLastError();
    }
    h->solved = false;
    h->fresh = true;
    h->n_side = 0;
    h->n_used = 0;
    h->seen_host = nullptr;
    h->lay.seen = nullptr;
    {
        // workgroups of the sweep that the GPU holds at a time (by registers and LDS)
        int per_cu = 0, cus = 0, dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            cus = 256;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(h->sweep),
                                                         h->var.w * kWave, h->lds_bytes) != hipSuccess || per_cu < 1)
            per_cu = h->var.wpe * 4 / h->var.w > 0 ? h->var.wpe * 4 / h->var.w : 1;
        (void)hipGetLastError();
        h->resident = per_cu * cus;
    }
    int n = (int)((desc->flags & GALV_DP_STREAMS_MASK) >> GALV_DP_STREAMS_SHIFT);
    h->auto_streams = n == 0;
    if (n == 0) {
        // Automatic: the handle owns as many streams as its largest batch could use (pick_streams
        // with every budget at the maximum), and every solve picks from the budgets the solve
        // before it met.
        h->n_side = kMaxSide;                      // (lets pick_streams answer for the cap below)
        n = pick_streams(h, tiles_at_most(h));
        h->n_side = 0;
        if (n > 1 && hipHostMalloc(reinterpret_cast<void **>(&h->seen_host), 64, hipHostMallocDefault) == hipSuccess) {
            *h->seen_host = 0;
            void *dptr = nullptr;
            if (hipHostGetDevicePointer(&dptr, h->seen_host, 0) == hipSuccess && dptr) {
                h->lay.seen = static_cast<int32_t *>(dptr);
            } else {
                (void)hipHostFree(h->seen_host);
                h->seen_host = nullptr;
            }
        }
        (void)hipGetLastError();
    }
    if (n > desc->n_instances) n = desc->n_instances;
    if (n > 1 && desc->n_layers > 1) {
        hipError_t e = hipEventCreateWithFlags(&h->fork, hipEventDisableTiming);
        const bool have_fork = e == hipSuccess;
        int made_s = 0, made_e = 0;
        for (int g = 0; g < n && e == hipSuccess; ++g) {
            e = hipStreamCreateWithFlags(&h->side[g], hipStreamNonBlocking);   // default priority
            if (e != hipSuccess) break;
            ++made_s;
            e = hipEventCreateWithFlags(&h->join[g], hipEventDisableTiming);
            if (e == hipSuccess) ++made_e;
        }
        if (e != hipSuccess) {
            for (int g = 0; g < made_s; ++g) (void)hipStreamDestroy(h->side[g]);
            for (int g = 0; g < made_e; ++g) (void)hipEventDestroy(h->join[g]);
            if (have_fork) (void)hipEventDestroy(h->fork);
            if (h->seen_host) (void)hipHostFree(h->seen_host);
            delete h;
            return fail(GALV_ERR_HIP, "creating internal streams failed: %s", hipGetErrorString(e));
        }
        h->n_side = n;
    }
    bind_workspace(h->lay, p, static_cast<char *>(workspace_dev));
    *out = h;
    return GALV_OK;
}

galv_status_t galv_dp_solve_batched(galv_dp_t *h, const int64_t *c_dev, const int32_t *m_dev,
                                    const int64_t *R_dev, const int32_t *r_idx_dev,
                                    const int32_t *budget_dev, int64_t *best_cost_dev,
                                    int32_t *best_last_dev, void *stream) {
    if (!h) return fail(GALV_ERR_INVALID_ARG, "handle is NULL");
    if (!c_dev || !m_dev || !R_dev || !budget_dev || !best_cost_dev || !best_last_dev)
        return fail(GALV_ERR_INVALID_ARG, "a required device pointer is NULL");
    return enqueue_solve(h, c_dev, m_dev, R_dev, r_idx_dev, budget_dev, best_cost_dev, best_last_dev,
                         static_cast<hipStream_t>(stream));
}

galv_status_t galv_dp_backtrack(galv_dp_t *h, int32_t *plan_dev, void *stream) {
    if (!h) return fail(GALV_ERR_INVALID_ARG, "handle is NULL");
    if (!plan_dev) return fail(GALV_ERR_INVALID_ARG, "plan_dev is NULL");
    if (!h->solved) return fail(GALV_ERR_STATE, "backtrack before a successful solve");
    const Layout &a = h->lay;
    backtrack_kernel<<<a.B, kWave, 0, static_cast<hipStream_t>(stream)>>>(a, plan_dev);
    HIP_TRY(hipGetLastError());
    return GALV_OK;
}

galv_status_t galv_dp_solve_static(const galv_dp_desc_t *desc, const int64_t *c_dev,
                                   const int32_t *m_dev, const int64_t *R_dev,
                                   const int32_t *r_idx_dev, const int32_t *budget_dev,
                                   int64_t *best_cost_dev, int32_t *best_last_dev, int32_t *plan_dev,
                                   void *stream) {
    Plan p;
    galv_status_t rc = make_plan(desc, &p);
    if (rc != GALV_OK) return rc;
    if (((desc->flags & GALV_DP_STREAMS_MASK) >> GALV_DP_STREAMS_SHIFT) > 1u)
        return fail(GALV_ERR_INVALID_ARG, "galv_dp_solve_static runs on the caller's stream only "
                                          "(GALV_DP_STREAMS must be 0 or 1)");
    if (p.total > (size_t)GALV_DP_STATIC_BYTES)
        return fail(GALV_ERR_WORKSPACE,
                    "this shape needs %zu bytes of workspace; galv_dp_solve_static holds %zu "
                    "(use galv_dp_create with a workspace of your own)",
                    p.total, (size_t)GALV_DP_STATIC_BYTES);
    if (!c_dev || !m_dev || !R_dev || !budget_dev || !best_cost_dev || !best_last_dev || !plan_dev)
        return fail(GALV_ERR_INVALID_ARG, "a required device pointer is NULL");
    void *ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != GALV_OK) return rc;

    // A handle on the stack: host memory only, no internal streams, nothing to destroy.
    galv_dp h;
    h.desc = *desc;
    h.var = p.var;
    h.sweep = p.sweep;
    h.lay = p.lay;
    h.ws_bytes = p.total;
    h.groups_y = p.groups_y;
    h.lds_bytes = p.lds_bytes;
    h.lds_allowed = p.lds_bytes <= 64u * 1024u;
    h.solved = false;
    h.fresh = true;            // the array keeps the last call's contents: write the leads anew
    h.n_side = 0;              // the caller's stream only: nothing to create, nothing to adapt
    h.auto_streams = false;
    h.n_used = 0;
    h.resident = 1;
    h.seen_host = nullptr;
    h.lay.seen = nullptr;
    bind_workspace(h.lay, p, static_cast<char *>(ws));
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = enqueue_solve(&h, c_dev, m_dev, R_dev, r_idx_dev, budget_dev, best_cost_dev, best_last_dev, st);
    if (rc != GALV_OK) return rc;
    backtrack_kernel<<<h.lay.B, kWave, 0, st>>>(h.lay, plan_dev);
    HIP_TRY(hipGetLastError());
    return GALV_OK;
}

galv_status_t galv_dp_best_per_budget(galv_dp_t *h, int64_t *best_cost_dev, int32_t *best_last_dev,
                                      void *stream) {
    if (!h) return fail(GALV_ERR_INVALID_ARG, "handle is NULL");
    if (!best_cost_dev) return fail(GALV_ERR_INVALID_ARG, "best_cost_dev is NULL");
    if (!h->solved) return fail(GALV_ERR_STATE, "best_per_budget before a successful solve");
    const Layout &a = h->lay;
    const dim3 grid((unsigned)((a.E_max + kThreads) / kThreads), a.B);
    best_per_budget_kernel<<<grid, kThreads, 0, static_cast<hipStream_t>(stream)>>>(a, best_cost_dev,
                                                                                  best_last_dev);
    HIP_TRY(hipGetLastError());
    return GALV_OK;
}

galv_status_t galv_dp_backtrack_queries(galv_dp_t *h, int32_t n_queries, const int32_t *instance_dev,
                                        const int32_t *budget_dev, int64_t *cost_dev,
                                        int32_t *plan_dev, void *stream) {
    if (!h) return fail(GALV_ERR_INVALID_ARG, "handle is NULL");
    if (n_queries < 0) return fail(GALV_ERR_INVALID_ARG, "n_queries %d is negative", n_queries);
    if (n_queries == 0) return GALV_OK;
    if (!instance_dev || !budget_dev || !plan_dev)
        return fail(GALV_ERR_INVALID_ARG, "a required device pointer is NULL");
    if (!h->solved) return fail(GALV_ERR_STATE, "backtrack_queries before a successful solve");
    backtrack_queries_kernel<<<(n_queries + kWave - 1) / kWave, kWave, 0,
                               static_cast<hipStream_t>(stream)>>>(h->lay, n_queries, instance_dev,
                                                                   budget_dev, cost_dev, plan_dev);
    HIP_TRY(hipGetLastError());
    return GALV_OK;
}

galv_status_t galv_dp_export_tables(galv_dp_t *h, int32_t instance, int64_t *C_last_dev,
                                    int32_t *bp_dev, void *stream) {
    if (!h) return fail(GALV_ERR_INVALID_ARG, "handle is NULL");
    if (!C_last_dev) return fail(GALV_ERR_INVALID_ARG, "C_last_dev is NULL");
    if (!h->solved) return fail(GALV_ERR_STATE, "export before a successful solve");
    const Layout &a = h->lay;
    if (instance < 0 || instance >= a.B)
        return fail(GALV_ERR_INVALID_ARG, "instance %d out of range [0, %d)", instance, a.B);
    if (a.L + 1 > 65535) return fail(GALV_ERR_RANGE, "too many layers to export");
    const dim3 grid((unsigned)((a.E_max + kThreads) / kThreads), a.L + 1);
    export_kernel<<<grid, kThreads, 0, static_cast<hipStream_t>(stream)>>>(a, instance, C_last_dev,
                                                                          bp_dev);
    HIP_TRY(hipGetLastError());
    return GALV_OK;
}

galv_status_t galv_dp_get_status(galv_dp_t *h, int32_t *status_dev, void *stream) {
    if (!h) return fail(GALV_ERR_INVALID_ARG, "handle is NULL");
    if (!status_dev) return fail(GALV_ERR_INVALID_ARG, "status_dev is NULL");
    if (!h->solved) return fail(GALV_ERR_STATE, "status before a successful solve");
    HIP_TRY(hipMemcpyAsync(status_dev, h->lay.status, (size_t)h->lay.B * sizeof(int32_t),
                           hipMemcpyDeviceToDevice, static_cast<hipStream_t>(stream)));
    return GALV_OK;
}

galv_status_t galv_dp_get_stats(galv_dp_t *h, int64_t *stats_dev, void *stream) {
    if (!h) return fail(GALV_ERR_INVALID_ARG, "handle is NULL");
    if (!stats_dev) return fail(GALV_ERR_INVALID_ARG, "stats_dev is NULL");
    if (!h->solved) return fail(GALV_ERR_STATE, "statistics before a successful solve");
    stats_kernel<<<h->lay.B, kThreads, 0, static_cast<hipStream_t>(stream)>>>(h->lay, stats_dev);
    HIP_TRY(hipGetLastError());
    return GALV_OK;
}

galv_status_t galv_dp_get_config(const galv_dp_t *h, int32_t *config) {
    if (!h) return fail(GALV_ERR_INVALID_ARG, "handle is NULL");
    if (!config) return fail(GALV_ERR_INVALID_ARG, "config is NULL");
    config[0] = h->lay.packed;
    config[1] = h->lay.peek && h->var.share ? 1 : 0;
    config[2] = h->n_used > 0 ? h->n_used : (h->lay.L < 2 ? 1 : pick_streams(h, tiles_at_most(h)));
    config[3] = h->lay.tile_e;
    return GALV_OK;
}

galv_status_t galv_alg1_reduce(int32_t n_batch, int32_t n_pp, const int32_t *pp_degree,
                               const int64_t *stage_cost_dev, const int64_t *batch_size_dev,
                               int32_t batch_index_base, int32_t first_window, int64_t *c_p_dev,
                               galv_alg1_state_t *state_dev, void *stream) {
    if (n_batch < 1 || n_batch > (1 << 20))
        return fail(GALV_ERR_INVALID_ARG, "n_batch %d out of range [1, 2^20]", n_batch);
    if (n_pp < 1 || n_pp > kMaxPp)
        return fail(GALV_ERR_INVALID_ARG, "n_pp %d out of range [1, %d]", n_pp, kMaxPp);
    if (!pp_degree || !stage_cost_dev || !batch_size_dev || !c_p_dev || !state_dev)
        return fail(GALV_ERR_INVALID_ARG, "a required pointer is NULL");
    PpList pp;
    pp.n = n_pp;
    for (int i = 0; i < kMaxPp; ++i) pp.degree[i] = 0;
    for (int i = 0; i < n_pp; ++i) {
        if (pp_degree[i] < 1 || pp_degree[i] > (1 << 16))
            return fail(GALV_ERR_INVALID_ARG, "pp_degree[%d] = %d out of range [1, 65536]", i,
                        pp_degree[i]);
        pp.degree[i] = pp_degree[i];
    }
    alg1_reduce_kernel<<<1, kThreads, 0, static_cast<hipStream_t>(stream)>>>(
        n_batch, pp, stage_cost_dev, batch_size_dev, batch_index_base, first_window, c_p_dev,
        state_dev);
    HIP_TRY(hipGetLastError());
    return GALV_OK;
}

galv_status_t galv_dp_coarsen(int32_t n_instances, int32_t n_layers, int32_t n_strategies,
                              int32_t n_transition, int32_t fuse, int32_t granularity,
                              const int64_t *c_dev, const int32_t *m_dev, const int64_t *R_dev,
                              const int32_t *r_idx_dev, const int32_t *budget_dev, int64_t *c_out_dev,
                              int32_t *m_out_dev, int32_t *r_idx_out_dev, int32_t *budget_out_dev,
                              void *stream) {
    if (n_instances < 1 || n_layers < 1 || n_strategies < 1 || n_transition < 1)
        return fail(GALV_ERR_INVALID_ARG, "coarsen: sizes must be >= 1");
    if (fuse < 1 || granularity < 1)
        return fail(GALV_ERR_INVALID_ARG, "coarsen: fuse %d and granularity %d must be >= 1", fuse,
                    granularity);
    if (!c_dev || !m_dev || !R_dev || !budget_dev || !c_out_dev || !m_out_dev || !r_idx_out_dev ||
        !budget_out_dev)
        return fail(GALV_ERR_INVALID_ARG, "a required device pointer is NULL");
    const int Lc = (n_layers + fuse - 1) / fuse;
    const long double cells = (long double)n_instances * Lc * n_strategies;
    if (cells > 2.0e12L) return fail(GALV_ERR_RANGE, "coarsen: %.3Lg cells cannot be indexed", cells);
    const int64_t n = (int64_t)n_instances * Lc * n_strategies;
    coarsen_kernel<<<(unsigned)((n + kThreads - 1) / kThreads), kThreads, 0,
                     static_cast<hipStream_t>(stream)>>>(
        n_instances, n_layers, n_strategies, n_transition, fuse, granularity, Lc, c_dev, m_dev, R_dev,
        r_idx_dev, budget_dev, c_out_dev, m_out_dev, r_idx_out_dev, budget_out_dev);
    HIP_TRY(hipGetLastError());
    return GALV_OK;
}

galv_status_t galv_dp_expand_plan(int32_t n_instances, int32_t n_layers, int32_t fuse,
                                  const int32_t *coarse_plan_dev, int32_t *plan_dev, void *stream) {
    if (n_instances < 1 || n_layers < 1 || fuse < 1)
        return fail(GALV_ERR_INVALID_ARG, "expand_plan: sizes must be >= 1");
    if (!coarse_plan_dev || !plan_dev) return fail(GALV_ERR_INVALID_ARG, "a required device pointer is NULL");
    const int Lc = (n_layers + fuse - 1) / fuse;
    const int64_t n = (int64_t)n_instances * n_layers;
    expand_plan_kernel<<<(unsigned)((n + kThreads - 1) / kThreads), kThreads, 0,
                         static_cast<hipStream_t>(stream)>>>(n_instances, n_layers, fuse, Lc,
                                                             coarse_plan_dev, plan_dev);
    HIP_TRY(hipGetLastError());
    return GALV_OK;
}

galv_status_t galv_dp_destroy(galv_dp_t *h) {
    if (h && h->n_side > 1) {
        for (int g = 0; g < h->n_side; ++g) {
            (void)hipStreamDestroy(h->side[g]);
            (void)hipEventDestroy(h->join[g]);
        }
        (void)hipEventDestroy(h->fork);
    }
    if (h && h->seen_host) (void)hipHostFree(h->seen_host);
    delete h;
    return GALV_OK;
}

const char *galv_dp_last_error(void) { return g_err; }

#ifndef GALV_DP_BUILD_STAMP
#define GALV_DP_BUILD_STAMP "unchecked"
#endif
const char *galv_dp_build_stamp(void) { return GALV_DP_BUILD_STAMP; }

}  // extern "C"
