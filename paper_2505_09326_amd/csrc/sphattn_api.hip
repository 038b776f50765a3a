// Host side of the C ABI declared in include/sphattn.h: argument checks, kernel
// selection by (dtype, d), launch on the caller's stream.  Allocates nothing and
// never synchronises.
#include "sphattn_device.hpp"
#include "sphattn_pipelined.hpp"
#include "sphattn_softmax32.hpp"
#include "sphattn_backward.hpp"
#include "sphattn_fp8.hpp"
#include "../../include/sphattn.h"

#include <stdint.h>

#include <atomic>

namespace {

using namespace sphattn;

constexpr int kVersion = 510;   // 0.5.1

// [a, a+an) and [b, b+bn) share a byte.  Written with differences, so that a range reaching the
// top of the address space cannot wrap the comparison.
bool overlaps(const void* a, size_t an, const void* b, size_t bn)
{
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 <= b0 ? b0 - a0 < an : a0 - b0 < bn;
}

// a buffer of `bytes` bytes at p would run past the end of the address space
bool wraps(const void* p, size_t bytes)
{
    return (uintptr_t)p + bytes < (uintptr_t)p;
}

int check_shape(int B, int H, int H_kv, int Nq, int Nk, int d, int dtype)
{
    if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || H_kv <= 0 || H % H_kv != 0) return SPHATTN_ERR_SHAPE;
    if (d != 64 && d != 128) return SPHATTN_ERR_HEAD_DIM;
    if (dtype != SPHATTN_F32 && dtype != SPHATTN_BF16 && dtype != SPHATTN_FP8QK_BF16V &&
        dtype != SPHATTN_F16)
        return SPHATTN_ERR_DTYPE;
    const unsigned __int128 nmax = Nq > Nk ? Nq : Nk;
    // B*H*N*d elements must be addressable with 64-bit offsets and B*H*tiles with int
    if ((unsigned __int128)B * H * nmax * d > ((unsigned __int128)1 << 40)) return SPHATTN_ERR_SHAPE;
    if ((unsigned __int128)B * H * ((nmax + 31) / 32) > 0x7fffffff) return SPHATTN_ERR_SHAPE;
    // one head of one tensor is addressed through a 32-bit buffer range
    if (nmax * d * 4 > 0x7fffffff) return SPHATTN_ERR_SHAPE;
    return SPHATTN_OK;
}

// `out` is what the call writes (out_bytes of it); it must not overlap anything the call reads.
int check_args(const void* Q, const void* K, const void* V, const void* out, size_t out_bytes,
               const float* mult, const float* Z,
               int B, int H, int H_kv, int Nq, int Nk, int d, int dtype)
{
    if (!Q || !K || !V || !out) return SPHATTN_ERR_NULL;
    const int rc = check_shape(B, H, H_kv, Nq, Nk, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)out) & 15) return SPHATTN_ERR_ALIGN;
    if (((uintptr_t)mult | (uintptr_t)Z) & 3) return SPHATTN_ERR_ALIGN;
    const size_t nq = (size_t)B * H * Nq * d, nkv = (size_t)B * H_kv * Nk * d;
    const size_t qk = dtype == SPHATTN_F32 ? 4 : dtype == SPHATTN_FP8QK_BF16V ? 1 : 2;
    const size_t vo = dtype == SPHATTN_F32 ? 4 : 2;
    const size_t zb = (size_t)B * H * Nq * 4;
    if (wraps(out, out_bytes) || wraps(Q, nq * qk) || wraps(K, nkv * qk) || wraps(V, nkv * vo) ||
        (Z && wraps(Z, zb)) || (mult && wraps(mult, (size_t)B * Nk * 4)))
        return SPHATTN_ERR_SHAPE;
    if (overlaps(out, out_bytes, Q, nq * qk) || overlaps(out, out_bytes, K, nkv * qk) ||
        overlaps(out, out_bytes, V, nkv * vo) ||
        (mult && overlaps(out, out_bytes, mult, (size_t)B * Nk * 4)))
        return SPHATTN_ERR_ALIAS;
    if (Z && (overlaps(Z, zb, Q, nq * qk) || overlaps(Z, zb, K, nkv * qk) || overlaps(Z, zb, V, nkv * vo) ||
              overlaps(Z, zb, out, out_bytes) || (mult && overlaps(Z, zb, mult, (size_t)B * Nk * 4))))
        return SPHATTN_ERR_ALIAS;
    return SPHATTN_OK;
}

size_t out_bytes_of(int B, int H, int N, int d, int dtype)
{
    return (size_t)B * H * N * d * (dtype == SPHATTN_F32 ? 4 : 2);
}

// Kernels that use more than 64 KB of LDS need their limit raised once per device; `done` is
// that kernel's bit mask of devices already configured (the only state the library keeps).
long long cu_count();

// How many consecutive workgroups of one XCD's range run at the same time: that XCD's share of
// the compute units times the workgroups of this kernel that fit one unit.  Feeds the kernels'
// key-stream direction (see fwd_pipelined_kernel); asked once per kernel and device.
template <typename Kern>
int stream_period(Kern kern, int lds_bytes, std::atomic<int> (&cached)[64])
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return 0;
    }
    int p = cached[dev].load(std::memory_order_relaxed);
    if (p == 0) {
        int per_cu = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)kern, kThreads, (size_t)lds_bytes) != hipSuccess ||
            per_cu <= 0) {
            (void)hipGetLastError();
            return 0;                              // 0: never reverse
        }
        p = (int)(cu_count() / kXcds) * per_cu;
        cached[dev].store(p, std::memory_order_relaxed);
    }
    return p;
}

template <typename Kern>
bool raise_lds_limit(Kern kern, int lds_bytes, std::atomic<uint64_t>& done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return false;
    }
    const uint64_t bit = 1ull << dev;
    if (done.load(std::memory_order_acquire) & bit) return true;
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                            lds_bytes) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    done.fetch_or(bit, std::memory_order_release);
    return true;
}

// A launch.  Whole problem: O is the output tensor, Z the optional row aggregates, n_splits 1.
// Partial accumulators: O is the fp32 slice-major o buffer, Z the z buffer, and the key axis
// is cut into n_splits slices of keys_per_split rows.
struct Problem {
    const void* Q; const void* K; const void* V; void* O; const float* mult; float* Z;
    int B, H, H_kv, Nq, Nk;
    hipStream_t stream;
    int n_splits = 1, keys_per_split = 0;
    int tile_rows = 0;          // query rows per workgroup: 0 = the library's choice, else 128 or 256
};

// Key slices are whole 64-key tiles.  Asking for more slices than there are tiles, or for a
// count that does not divide them evenly, yields fewer, equally sized slices (the last may be
// shorter).
struct SplitPlan { int n_splits, keys_per_split; };
SplitPlan plan_splits(int Nk, int requested)
{
    const int tiles = (int)(((long long)Nk + kBC - 1) / kBC);   // >= 1: every caller has checked Nk >= 1
    requested = requested < 1 ? 1 : requested > tiles ? tiles : requested;
    const int per = (tiles + requested - 1) / requested;   // >= 1, and no overflow: requested <= tiles
    return SplitPlan{(tiles + per - 1) / per, per * kBC};
}

// Compute units of the current device, asked once per device; 256 (MI355X) when there is no
// device to ask.
long long cu_count()
{
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return 256;
    }
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n <= 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
            (void)hipGetLastError();
            return 256;
        }
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Persistent workgroups for n_items work items when `resident` workgroups run at once (a multiple
// of the XCD count; 0 = unknown).  The items take ceil(n_items / resident) rounds; when the last
// round would be partly filled, the same number of rounds is run with fewer workgroups, all
// rounds equally full: the part is power-bound, so CUs left idle in every round give their
// share of the budget to the others as clock, while a last round of a few items runs alone at
// almost its usual duration (measured, 8 heads of d = 128, N = 41472: 162 query tiles per head on
// 32 CUs, 5.06 rounds; the 2 tiles of the sixth round cost 0.9 of a full round).
long long balanced_grid(long long n_items, long long resident)
{
    if (resident <= 0 || n_items <= resident) return n_items;
    const long long rounds = (n_items + resident - 1) / resident;
    long long grid = (n_items + rounds - 1) / rounds;
    grid = (grid + kXcds - 1) / kXcds * kXcds;
    return grid < resident ? grid : resident;
}

// Storage types for which the 128-row kernel exists (fp8 Q/K needs whole score instructions per slot).
template <QKType QKT>
constexpr bool has_narrow_kernel() { return QKT == QKType::Bf16 || QKT == QKType::F16; }

// The 128-row kernel on the remainder of a launch whose items do not fill their last round
// (launch_pipelined): items item_begin .. n_items - 1 of the 256-row numbering, one half of an
// item per workgroup.  resident_only: configure the kernel and return how many of its
// workgroups run at once (0: unknown) without launching.
template <int D, QKType QKT>
long long launch_halves(const Problem& p, int n_qtiles, int n_items, int item_begin, bool backwards, bool resident_only)
{
    constexpr int EQ = QKT == QKType::Fp8 ? 1 : 2;
    constexpr int lds_bytes = kNBuf * kBC * (D * EQ + D * 2);
    auto kern = fwd_pipelined_kernel<D, 2, QKT, Norm::Spherical, false, false>;
    static std::atomic<uint64_t> done{0};
    static std::atomic<int> period[64];
    if (!raise_lds_limit(kern, lds_bytes, done)) return 0;
    const long long resident = (long long)kXcds * stream_period(kern, lds_bytes, period);
    if (resident_only) return resident;
    const int rest = n_items - item_begin;
    const unsigned grid = 2u * kXcds * (unsigned)((rest + kXcds - 1) / kXcds);
    const float scale_log2 = 1.4426950408889634f / __builtin_sqrtf((float)D);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds_bytes, p.stream,
                       p.Q, p.K, p.V, p.O, p.mult, p.Z,
                       p.Nq, p.Nk, p.H, p.H / p.H_kv, n_qtiles, n_items, 1, 0, scale_log2,
                       item_begin, n_items, backwards ? 2 : 1);
    return hipGetLastError() == hipSuccess ? resident : -1;
}

template <int D, int NQ, QKType QKT, Norm NORM, bool MULT, bool PARTIAL = false>
int launch_pipelined(const Problem& p)
{
    constexpr int BR = kWaves * 16 * NQ;
    constexpr int EQ = QKT == QKType::Fp8 ? 1 : 2;
    constexpr int lds_bytes = kNBuf * kBC * (D * EQ + D * 2 + (MULT ? 4 : 0));
    auto kern = fwd_pipelined_kernel<D, NQ, QKT, NORM, MULT, PARTIAL>;
    static std::atomic<uint64_t> done{0};
    static std::atomic<int> period[64];
    if (!raise_lds_limit(kern, lds_bytes, done)) return SPHATTN_ERR_LAUNCH;
    const int n_qtiles = (p.Nq + BR - 1) / BR;
    const long long n_wg = (long long)p.B * p.H * n_qtiles * p.n_splits;
    if (n_wg > 0x7fffffff) return SPHATTN_ERR_SHAPE;
    const float scale_log2 = 1.4426950408889634f / __builtin_sqrtf((float)D);
    // persistent workgroups: as many as the chip runs at once (a multiple of the XCD count), or
    // one per item if that is fewer
    const long long resident = (long long)kXcds * stream_period(kern, lds_bytes, period);
    // d = 64, a remainder of at most half a round behind at least one full round: the full rounds
    // run here and the remaining tiles as two 128-row halves each in a launch of their own, which
    // fills twice as many CUs for 0.6 of the time.  In full rounds, with f = remainder / resident:
    // rounds + 0.3 + 0.6 f against 0.5 (rounds + 1) + 0.5 (rounds + f) for the balanced grid (a
    // round filled to the fraction x takes about 0.5 + 0.5 x of a full one).  Measured: 20 heads of
    // 8192 x 64 (640 tiles, 1.25 rounds) 273 against 306 us, 12 x 12345 x 64 387 against 425 us.
    // At d = 128 the 128-row kernel is too much slower per row for this (8 x 41472 x 128: 4.84
    // against 4.66 ms, 4 x 20000 x 128: 649 against 632 us), and the balanced grid stays.
    constexpr bool HAS_HALVES = D == 64 && NQ == 4 && !PARTIAL && !MULT && NORM == Norm::Spherical && has_narrow_kernel<QKT>();
    if constexpr (HAS_HALVES) {
        const long long full = resident > 0 ? n_wg / resident : 0, rem = resident > 0 ? n_wg % resident : 0;
        if (p.tile_rows == 0 && full >= 1 && rem > 0) {
            const long long narrow = launch_halves<D, QKT>(p, n_qtiles, (int)n_wg, 0, false, true);
            const double f = (double)rem / (double)resident;
            if (2 * rem <= narrow && (double)full + 0.3 + 0.6 * f < 0.97 * ((double)full + 0.5 + 0.5 * f)) {
                const int n_main = (int)(full * resident);
                hipLaunchKernelGGL(kern, dim3((unsigned)resident), dim3(kThreads), lds_bytes, p.stream,
                                   p.Q, p.K, p.V, p.O, p.mult, p.Z,
                                   p.Nq, p.Nk, p.H, p.H / p.H_kv, n_qtiles, (int)n_wg,
                                   p.n_splits, p.keys_per_split, scale_log2, 0, n_main, 0);
                if (hipGetLastError() != hipSuccess) return SPHATTN_ERR_LAUNCH;
                return launch_halves<D, QKT>(p, n_qtiles, (int)n_wg, n_main, full % 2 == 1, false) >= 0 ? SPHATTN_OK : SPHATTN_ERR_LAUNCH;
            }
        }
    }
    const long long grid = balanced_grid(n_wg, resident);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), lds_bytes, p.stream,
                       p.Q, p.K, p.V, p.O, p.mult, p.Z,
                       p.Nq, p.Nk, p.H, p.H / p.H_kv, n_qtiles, (int)n_wg,
                       p.n_splits, p.keys_per_split, scale_log2, 0, (int)n_wg, 0);
    return hipGetLastError() == hipSuccess ? SPHATTN_OK : SPHATTN_ERR_LAUNCH;
}

template <int D, bool MULT, bool PARTIAL = false>
int launch_f32(const Problem& p)
{
    constexpr int BR = 32;                         // the four waves split the key axis
    constexpr int lds_bytes = kWaves * 2 * 32 * (D + 4) * 4;
    auto kern = fwd_f32_kernel<D, MULT, PARTIAL>;
    static std::atomic<uint64_t> done{0};
    if (!raise_lds_limit(kern, lds_bytes, done)) return SPHATTN_ERR_LAUNCH;
    const int n_qtiles = (p.Nq + BR - 1) / BR;
    const long long n_wg = (long long)p.B * p.H * n_qtiles * p.n_splits;
    if (n_wg > 0x7fffffff) return SPHATTN_ERR_SHAPE;
    hipLaunchKernelGGL(kern, dim3((unsigned)n_wg), dim3(kThreads), lds_bytes, p.stream,
                       (const float*)p.Q, (const float*)p.K, (const float*)p.V, (float*)p.O, p.mult, p.Z,
                       p.Nq, p.Nk, p.H, p.H / p.H_kv, n_qtiles, (int)n_wg,
                       p.n_splits, p.keys_per_split);
    return hipGetLastError() == hipSuccess ? SPHATTN_OK : SPHATTN_ERR_LAUNCH;
}

template <int D>
int launch_softmax32(const Problem& p)
{
    constexpr int BR = 256;
    constexpr int lds_bytes = kNBuf * kBC * (D * 2 + kKPad + D * 2 + kVPad);
    auto kern = softmax32_kernel<D>;
    static std::atomic<uint64_t> done{0};
    if (!raise_lds_limit(kern, lds_bytes, done)) return SPHATTN_ERR_LAUNCH;
    const int n_qtiles = (p.Nq + BR - 1) / BR;
    const long long n_wg = (long long)p.B * p.H * n_qtiles;
    if (n_wg > 0x7fffffff) return SPHATTN_ERR_SHAPE;
    const float scale_log2 = 1.4426950408889634f / __builtin_sqrtf((float)D);
    hipLaunchKernelGGL(kern, dim3((unsigned)n_wg), dim3(kThreads), lds_bytes, p.stream,
                       p.Q, p.K, p.V, p.O, p.Nq, n_qtiles, (int)n_wg, scale_log2);
    return hipGetLastError() == hipSuccess ? SPHATTN_OK : SPHATTN_ERR_LAUNCH;
}

// Query rows per workgroup: 256 (64 per wave) is the efficient shape; 128 (32 per wave) reads
// K/V fragments twice as often per flop (measured 15-25 % slower per row) but doubles the
// number of workgroups.  It pays when the 128-row workgroups still run all at once (one per CU
// at d = 128, two at d = 64) and 256-row tiles would leave CUs without any: measured, one head
// of 32768 x 128: 0.42 against 0.51 ms; 4 heads of 8192 x 64: 65 against 84 us.  With more items
// than that the 128-row launch takes two rounds and loses (5 heads of 8192 x 128, 160 tiles:
// 182 against 151 us; 3 x 16384 x 128, 192 tiles: 368 against 290 us): a partly filled single
// round costs less than its share of idle CUs suggests, because the part is power-bound and
// idle CUs give their share of the budget to the rest.
bool narrow_tiles_pay(const Problem& p, int d)
{
    if (p.tile_rows != 0) return p.tile_rows == 128;
    const long long heads = (long long)p.B * p.H, cus = cu_count();
    return heads * ((p.Nq + 255) / 256) < cus && heads * ((p.Nq + 127) / 128) <= cus * (d == 64 ? 2 : 1);
}

template <Norm NORM, bool MULT>
int dispatch(const Problem& p, int d, int dtype)
{
    if (dtype == SPHATTN_BF16) {
        if constexpr (NORM == Norm::Spherical && !MULT) {
            if (narrow_tiles_pay(p, d)) {
                if (d == 128) return launch_pipelined<128, 2, QKType::Bf16, NORM, MULT>(p);
                return launch_pipelined<64, 2, QKType::Bf16, NORM, MULT>(p);
            }
        }
        if (d == 128) return launch_pipelined<128, 4, QKType::Bf16, NORM, MULT>(p);
        return launch_pipelined<64, 4, QKType::Bf16, NORM, MULT>(p);
    }
    if constexpr (NORM == Norm::Softmax && !MULT) {
        if (dtype == SPHATTN_FP8QK_BF16V) {
            if (d == 128) return launch_pipelined<128, 4, QKType::Fp8, NORM, MULT>(p);
            return launch_pipelined<64, 4, QKType::Fp8, NORM, MULT>(p);
        }
    }
    if constexpr (NORM == Norm::Spherical) {
        if (dtype == SPHATTN_F16) {
            if (d == 128) return launch_pipelined<128, 4, QKType::F16, NORM, MULT>(p);
            return launch_pipelined<64, 4, QKType::F16, NORM, MULT>(p);
        }
        if (dtype == SPHATTN_FP8QK_BF16V) {
            if (d == 128) return launch_pipelined<128, 4, QKType::Fp8, NORM, MULT>(p);
            return launch_pipelined<64, 4, QKType::Fp8, NORM, MULT>(p);
        }
        if (dtype == SPHATTN_F32) {
            if (d == 128) return launch_f32<128, MULT>(p);
            return launch_f32<64, MULT>(p);
        }
    }
    return SPHATTN_ERR_DTYPE;
}

// Partial accumulators over key slices: always the 256-row workgroup (the slices, not narrower
// tiles, are what fills the CUs).
template <bool MULT>
int dispatch_partial(const Problem& p, int d, int dtype)
{
    constexpr Norm S = Norm::Spherical;
    switch (dtype) {
    case SPHATTN_BF16:
        return d == 128 ? launch_pipelined<128, 4, QKType::Bf16, S, MULT, true>(p)
                        : launch_pipelined<64, 4, QKType::Bf16, S, MULT, true>(p);
    case SPHATTN_F16:
        return d == 128 ? launch_pipelined<128, 4, QKType::F16, S, MULT, true>(p)
                        : launch_pipelined<64, 4, QKType::F16, S, MULT, true>(p);
    case SPHATTN_FP8QK_BF16V:
        return d == 128 ? launch_pipelined<128, 4, QKType::Fp8, S, MULT, true>(p)
                        : launch_pipelined<64, 4, QKType::Fp8, S, MULT, true>(p);
    case SPHATTN_F32:
        return d == 128 ? launch_f32<128, MULT, true>(p) : launch_f32<64, MULT, true>(p);
    default:
        return SPHATTN_ERR_DTYPE;
    }
}

template <int D>
int launch_combine(const float* o_parts, const float* z_parts, int n_parts, void* O, float* Z,
                   size_t rows, int dtype, hipStream_t stream)
{
    const size_t threads = rows * (D / 4);
    const size_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffff) return SPHATTN_ERR_SHAPE;
    const dim3 grid((unsigned)blocks), block(256);
    if (dtype == SPHATTN_F32)
        hipLaunchKernelGGL((combine_kernel<D, 0>), grid, block, 0, stream, o_parts, z_parts, n_parts, O, Z, rows);
    else if (dtype == SPHATTN_F16)
        hipLaunchKernelGGL((combine_kernel<D, 2>), grid, block, 0, stream, o_parts, z_parts, n_parts, O, Z, rows);
    else
        hipLaunchKernelGGL((combine_kernel<D, 1>), grid, block, 0, stream, o_parts, z_parts, n_parts, O, Z, rows);
    return hipGetLastError() == hipSuccess ? SPHATTN_OK : SPHATTN_ERR_LAUNCH;
}

struct BwdProblem {
    const void* Q; const void* K; const void* V; const float* mult; const void* O; const void* dO;
    const float* Z; void* dQ; void* dK; void* dV; float* delta;
    int B, H, H_kv, N;
    hipStream_t stream;
};

template <int D, bool HALF, bool MULT, int NK>
int launch_bwd(const BwdProblem& p)
{
    constexpr int tile = kBC * D * 2;
    constexpr int lds_dq = 2 * (2 * tile + (MULT ? kBC * 4 : 0)), lds_dkv = 2 * (2 * tile + 2 * kBC * 4) + (MULT ? kWaves * NK * 16 * 4 : 0);
    auto kq = bwd_dq_kernel<D, HALF, MULT>;
    auto kkv = bwd_dkv_kernel<D, HALF, MULT, NK>;
    static std::atomic<uint64_t> done_q{0}, done_kv{0};
    if (!raise_lds_limit(kq, lds_dq, done_q) || !raise_lds_limit(kkv, lds_dkv, done_kv)) return SPHATTN_ERR_LAUNCH;
    const int n_qtiles = (p.N + 255) / 256, n_ktiles = (p.N + 64 * NK - 1) / (64 * NK);
    const long long wg_q = (long long)p.B * p.H * n_qtiles, wg_kv = (long long)p.B * p.H_kv * n_ktiles;
    if (wg_q > 0x7fffffff || wg_kv > 0x7fffffff) return SPHATTN_ERR_SHAPE;
    const int kv_group = p.H / p.H_kv;
    // the two planes of delta (delta_i r_i^2, then r_i) are written by the first kernel and read
    // by the second, in stream order
    float* rnorm = p.delta + (size_t)p.B * p.H * p.N;
    hipLaunchKernelGGL(kq, dim3((unsigned)wg_q), dim3(kThreads), lds_dq, p.stream,
                       p.Q, p.K, p.V, p.mult, p.O, p.dO, p.Z, p.dQ, p.delta, rnorm, p.N, p.H, kv_group, n_qtiles, (int)wg_q);
    if (hipGetLastError() != hipSuccess) return SPHATTN_ERR_LAUNCH;
    hipLaunchKernelGGL(kkv, dim3((unsigned)wg_kv), dim3(kThreads), lds_dkv, p.stream,
                       p.Q, p.K, p.V, p.mult, p.dO, (const float*)rnorm, (const float*)p.delta, p.dK, p.dV,
                       p.N, p.H, kv_group, n_ktiles, (int)wg_kv);
    return hipGetLastError() == hipSuccess ? SPHATTN_OK : SPHATTN_ERR_LAUNCH;
}

template <bool MULT>
int dispatch_bwd(const BwdProblem& p, int d, int dtype)
{
    if (dtype == SPHATTN_F16) return d == 128 ? launch_bwd<128, true, MULT, 2>(p) : launch_bwd<64, true, MULT, 2>(p);
    return d == 128 ? launch_bwd<128, false, MULT, 2>(p) : launch_bwd<64, false, MULT, 2>(p);
}

size_t workspace_bytes(int B, int H, int N, int d, int n_splits)
{
    const size_t rows = (size_t)B * H * N;
    return ((size_t)n_splits * rows * (d + 1) * 4 + 255) & ~(size_t)255;
}

// The two launches of the split-key forward on checked arguments: partial pairs of every slice
// into `workspace` (o parts, then z parts), then their sum and the tail.  Every partial the
// second launch reads is written by the first (every planned slice holds at least one tile),
// so the workspace needs no clearing.
int run_splitkv(const void* Q, const void* K, const void* V, const float* mult, void* O, float* Z,
                int B, int H, int H_kv, int N, int d, int dtype, SplitPlan plan, void* workspace, hipStream_t stream)
{
    if (plan.n_splits == 1) {                      // nothing to combine: the unsplit launch
        const Problem whole{Q, K, V, O, mult, Z, B, H, H_kv, N, N, stream};
        return mult ? dispatch<Norm::Spherical, true>(whole, d, dtype) : dispatch<Norm::Spherical, false>(whole, d, dtype);
    }
    const size_t rows = (size_t)B * H * N;
    float* o_parts = (float*)workspace;
    float* z_parts = o_parts + (size_t)plan.n_splits * rows * d;
    Problem p{Q, K, V, o_parts, mult, z_parts, B, H, H_kv, N, N, stream};
    p.n_splits = plan.n_splits;
    p.keys_per_split = plan.keys_per_split;
    const int r1 = mult ? dispatch_partial<true>(p, d, dtype) : dispatch_partial<false>(p, d, dtype);
    if (r1 != SPHATTN_OK) return r1;
    return d == 128 ? launch_combine<128>(o_parts, z_parts, plan.n_splits, O, Z, rows, dtype, stream)
                    : launch_combine<64>(o_parts, z_parts, plan.n_splits, O, Z, rows, dtype, stream);
}

template <int D, bool SOFTMAX, bool MULT>
int launch_fp8(const void* Q, const void* K, const unsigned char* VT, const float* kmax, const float* mult,
                      void* O, int B, int H, int H_kv, int N, int n_tiles, hipStream_t st)
{
    constexpr int lds_bytes = 4 * (2 * kFp8Tile * D + (MULT ? kFp8Tile * 4 : 0));
    static std::atomic<uint64_t> done{0};
    static std::atomic<int> period[64];
    auto kern = fwd_fp8_kernel<D, SOFTMAX, MULT>;
    if (!raise_lds_limit(kern, lds_bytes, done)) return SPHATTN_ERR_LAUNCH;
    const int n_qtiles = (N + 255) / 256;
    const long long n_wg = (long long)B * H * n_qtiles;
    hipLaunchKernelGGL(kern, dim3((unsigned)n_wg), dim3(kThreads), lds_bytes, st,
                       (const unsigned char*)Q, (const unsigned char*)K, VT, kmax, mult, (unsigned short*)O,
                       N, H, H / H_kv, n_tiles, n_qtiles, (int)n_wg, stream_period(kern, lds_bytes, period));
    return hipGetLastError() == hipSuccess ? SPHATTN_OK : SPHATTN_ERR_LAUNCH;
}

int fp8_forward(const void* Q, const void* K, const void* V, const float* mult, void* O, void* workspace,
                       size_t workspace_bytes, int B, int H, int H_kv, int N, int d, void* stream, bool softmax)
{
    if (d != 64 && d != 128) return SPHATTN_ERR_HEAD_DIM;
    if (!Q || !K || !V || !O) return SPHATTN_ERR_NULL;
    const int rc = check_shape(B, H, H_kv, N, N, d, SPHATTN_FP8QK_BF16V);
    if (rc != SPHATTN_OK) return rc;
    if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15) return SPHATTN_ERR_ALIGN;
    if ((uintptr_t)mult & 3) return SPHATTN_ERR_ALIGN;
    const size_t in_bytes = (size_t)B * H * N * d, kv_bytes = (size_t)B * H_kv * N * d, m_bytes = (size_t)B * N * 4;
    if (wraps(O, in_bytes * 2) || wraps(Q, in_bytes) || wraps(K, kv_bytes) || wraps(V, kv_bytes) ||
        (mult && wraps(mult, m_bytes)))
        return SPHATTN_ERR_SHAPE;
    if (overlaps(O, in_bytes * 2, Q, in_bytes) || overlaps(O, in_bytes * 2, K, kv_bytes) ||
        overlaps(O, in_bytes * 2, V, kv_bytes) || (mult && overlaps(O, in_bytes * 2, mult, m_bytes)))
        return SPHATTN_ERR_ALIAS;
    const size_t need = sphattn_fp8_workspace_bytes(B, H_kv, N, d);
    if (!workspace || ((uintptr_t)workspace & 15) || workspace_bytes < need || wraps(workspace, need))
        return SPHATTN_ERR_WORKSPACE;
    if (overlaps(workspace, need, Q, in_bytes) || overlaps(workspace, need, K, kv_bytes) ||
        overlaps(workspace, need, V, kv_bytes) || overlaps(workspace, need, O, in_bytes * 2) ||
        (mult && overlaps(workspace, need, mult, m_bytes)))
        return SPHATTN_ERR_ALIAS;
    const int heads = B * H_kv;                    // K/V heads: what the preparation pass covers
    const int n_tiles = (N + kFp8Tile - 1) / kFp8Tile;
    const size_t kmax_bytes = ((size_t)heads * 4 + 255) & ~(size_t)255;
    float* kmax = (float*)workspace;
    unsigned char* VT = (unsigned char*)workspace + kmax_bytes;
    hipStream_t st = (hipStream_t)stream;
    if ((long long)heads * n_tiles > 0x7fffffff) return SPHATTN_ERR_SHAPE;
    if ((long long)B * H * ((N + 255) / 256) > 0x7fffffff) return SPHATTN_ERR_SHAPE;
    if ((unsigned __int128)d * n_tiles * kFp8Tile > 0x7fffffff) return SPHATTN_ERR_SHAPE;   // one head of V^T: a 32-bit range
    // three launches; the attention kernel's attribute (the one thing that can fail without a
    // launch) is set by its launcher before it enqueues anything, so a refusal there leaves the
    // workspace written and nothing else
    hipLaunchKernelGGL(fp8_clear_kernel, dim3((heads + 255) / 256), dim3(256), 0, st, kmax, heads);
    if (hipGetLastError() != hipSuccess) return SPHATTN_ERR_LAUNCH;
    if (d == 128)
        hipLaunchKernelGGL(fp8_prepare_kernel<128>, dim3((unsigned)(heads * n_tiles)), dim3(256), 0, st,
                           (const unsigned char*)K, (const unsigned char*)V, mult, VT, kmax, N, n_tiles, H_kv);
    else
        hipLaunchKernelGGL(fp8_prepare_kernel<64>, dim3((unsigned)(heads * n_tiles)), dim3(256), 0, st,
                           (const unsigned char*)K, (const unsigned char*)V, mult, VT, kmax, N, n_tiles, H_kv);
    if (hipGetLastError() != hipSuccess) return SPHATTN_ERR_LAUNCH;
    if (d == 128) {
        if (softmax) return launch_fp8<128, true, false>(Q, K, VT, kmax, nullptr, O, B, H, H_kv, N, n_tiles, st);
        return mult ? launch_fp8<128, false, true>(Q, K, VT, kmax, mult, O, B, H, H_kv, N, n_tiles, st)
                    : launch_fp8<128, false, false>(Q, K, VT, kmax, nullptr, O, B, H, H_kv, N, n_tiles, st);
    }
    if (softmax) return launch_fp8<64, true, false>(Q, K, VT, kmax, nullptr, O, B, H, H_kv, N, n_tiles, st);
    return mult ? launch_fp8<64, false, true>(Q, K, VT, kmax, mult, O, B, H, H_kv, N, n_tiles, st)
                : launch_fp8<64, false, false>(Q, K, VT, kmax, nullptr, O, B, H, H_kv, N, n_tiles, st);
}

// Scratch memory of sphattn_splitkv_fwd_noalloc: one array per GPU, part of the library's code
// object, alive until the process ends.  Host code never uses the array's name as an address:
// its device address is asked for once per device (scratch_address) and kept.
static __device__ __align__(256) unsigned char scratch[SPHATTN_NOALLOC_SCRATCH_BYTES];

// Device address of `scratch` on the current device, or nullptr if the runtime cannot give it.
void* scratch_address()
{
    static std::atomic<void*> known[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return nullptr;
    }
    void* p = known[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        known[dev].store(p, std::memory_order_release);
    }
    return p;
}

}  // namespace

extern "C" {

int sphattn_fwd(const void* Q, const void* K, const void* V, void* O,
                int B, int H, int N, int d, int dtype, void* stream)
{
    return sphattn_fwd_z(Q, K, V, O, nullptr, B, H, N, d, dtype, stream);
}

int sphattn_fwd_z(const void* Q, const void* K, const void* V, void* O, float* Z,
                  int B, int H, int N, int d, int dtype, void* stream)
{
    return sphattn_fwd_tile_rows(Q, K, V, O, Z, B, H, N, d, dtype, 0, stream);
}

int sphattn_fwd_tile_rows(const void* Q, const void* K, const void* V, void* O, float* Z,
                          int B, int H, int N, int d, int dtype, int tile_rows, void* stream)
{
    const int rc = check_args(Q, K, V, O, out_bytes_of(B, H, N, d, dtype), nullptr, Z, B, H, H, N, N, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    if (tile_rows != 0 && tile_rows != 128 && tile_rows != 256) return SPHATTN_ERR_SHAPE;
    Problem p{Q, K, V, O, nullptr, Z, B, H, H, N, N, (hipStream_t)stream};
    p.tile_rows = tile_rows;
    return dispatch<Norm::Spherical, false>(p, d, dtype);
}

int sphattn_grn_fwd(const void* Q, const void* K, const void* V, const float* mult, void* O,
                    int B, int H, int H_kv, int N, int d, int dtype, void* stream)
{
    const int rc = check_args(Q, K, V, O, out_bytes_of(B, H, N, d, dtype), mult, nullptr, B, H, H_kv, N, N, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    const Problem p{Q, K, V, O, mult, nullptr, B, H, H_kv, N, N, (hipStream_t)stream};
    return mult ? dispatch<Norm::Spherical, true>(p, d, dtype)
                : dispatch<Norm::Spherical, false>(p, d, dtype);
}

int sphattn_cross_fwd(const void* Q, const void* K, const void* V, const float* mult, void* O, float* Z,
                      int B, int H, int H_kv, int N_q, int N_k, int d, int dtype, void* stream)
{
    const int rc = check_args(Q, K, V, O, out_bytes_of(B, H, N_q, d, dtype), mult, Z, B, H, H_kv, N_q, N_k, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    const Problem p{Q, K, V, O, mult, Z, B, H, H_kv, N_q, N_k, (hipStream_t)stream};
    return mult ? dispatch<Norm::Spherical, true>(p, d, dtype)
                : dispatch<Norm::Spherical, false>(p, d, dtype);
}

int sphattn_normalized_fwd(const void* Q, const void* K, const void* V, void* O,
                           int B, int H, int N, int d, int dtype, int normalizer, void* stream)
{
    const int rc = check_args(Q, K, V, O, out_bytes_of(B, H, N, d, dtype), nullptr, nullptr, B, H, H, N, N, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    if (normalizer < SPHATTN_NORM_L2 || normalizer > SPHATTN_NORM_SQRELU) return SPHATTN_ERR_NORMALIZER;
    if (normalizer != SPHATTN_NORM_L2 && dtype != SPHATTN_BF16 &&
        !(normalizer == SPHATTN_NORM_SOFTMAX && dtype == SPHATTN_FP8QK_BF16V))
        return SPHATTN_ERR_DTYPE;
    const Problem p{Q, K, V, O, nullptr, nullptr, B, H, H, N, N, (hipStream_t)stream};
    switch (normalizer) {
    case SPHATTN_NORM_L2: return dispatch<Norm::Spherical, false>(p, d, dtype);
    case SPHATTN_NORM_SOFTMAX: return dispatch<Norm::Softmax, false>(p, d, dtype);
    case SPHATTN_NORM_L1: return dispatch<Norm::L1, false>(p, d, dtype);
    default: return dispatch<Norm::SqRelu, false>(p, d, dtype);
    }
}

int sphattn_softmax_fwd(const void* Q, const void* K, const void* V, void* O,
                        int B, int H, int N, int d, int dtype, void* stream)
{
    const int rc = check_args(Q, K, V, O, out_bytes_of(B, H, N, d, dtype), nullptr, nullptr, B, H, H, N, N, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    if (dtype != SPHATTN_BF16) return SPHATTN_ERR_DTYPE;
    const Problem p{Q, K, V, O, nullptr, nullptr, B, H, H, N, N, (hipStream_t)stream};
    return d == 128 ? launch_softmax32<128>(p) : launch_softmax32<64>(p);
}

int sphattn_partial_fwd(const void* Q, const void* K, const void* V, const float* mult,
                        float* o_part, float* z_part,
                        int B, int H, int H_kv, int N_q, int N_k, int d, int dtype, void* stream)
{
    if (!z_part) return SPHATTN_ERR_NULL;
    const int rc = check_args(Q, K, V, o_part, (size_t)B * H * N_q * d * 4, mult, z_part,
                              B, H, H_kv, N_q, N_k, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    Problem p{Q, K, V, o_part, mult, z_part, B, H, H_kv, N_q, N_k, (hipStream_t)stream};
    p.n_splits = 1;
    p.keys_per_split = plan_splits(N_k, 1).keys_per_split;
    return mult ? dispatch_partial<true>(p, d, dtype) : dispatch_partial<false>(p, d, dtype);
}

int sphattn_combine(const float* o_parts, const float* z_parts, int n_parts, void* O, float* Z,
                    int B, int H, int N, int d, int dtype, void* stream)
{
    if (!o_parts || !z_parts || !O) return SPHATTN_ERR_NULL;
    const int rc = check_shape(B, H, H, N, N, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    if (n_parts <= 0 || n_parts > 65536) return SPHATTN_ERR_SHAPE;
    if (((uintptr_t)o_parts | (uintptr_t)O) & 15) return SPHATTN_ERR_ALIGN;
    if (((uintptr_t)z_parts | (uintptr_t)Z) & 3) return SPHATTN_ERR_ALIGN;
    const size_t rows = (size_t)B * H * N, ob = out_bytes_of(B, H, N, d, dtype);
    const size_t pob = (size_t)n_parts * rows * d * 4, pzb = (size_t)n_parts * rows * 4;
    if (overlaps(O, ob, o_parts, pob) || overlaps(O, ob, z_parts, pzb) ||
        (Z && (overlaps(Z, rows * 4, o_parts, pob) || overlaps(Z, rows * 4, z_parts, pzb) ||
               overlaps(Z, rows * 4, O, ob))))
        return SPHATTN_ERR_ALIAS;
    return d == 128 ? launch_combine<128>(o_parts, z_parts, n_parts, O, Z, rows, dtype, (hipStream_t)stream)
                    : launch_combine<64>(o_parts, z_parts, n_parts, O, Z, rows, dtype, (hipStream_t)stream);
}

size_t sphattn_splitkv_workspace_bytes(int B, int H, int N, int d, int n_splits)
{
    if (B <= 0 || H <= 0 || N <= 0 || (d != 64 && d != 128) || n_splits <= 0) return 0;
    if ((unsigned __int128)B * H * (unsigned __int128)N * (d + 1) * 4 * n_splits > ((unsigned __int128)1 << 46)) return 0;
    return workspace_bytes(B, H, N, d, n_splits);
}

int sphattn_splitkv_heuristic(int B, int H, int N, int d, int dtype)
{
    if (B <= 0 || H <= 0 || N <= 0 || (d != 64 && d != 128)) return 1;
    const long long cus = cu_count();
    const long long tiles = ((long long)N + kBC - 1) / kBC;
    const long long most = (tiles + 7) / 8;        // no slice shorter than 8 tiles
    if (dtype == SPHATTN_F32) {
        // the fp32 kernel's workgroups hold 32 query rows: enough slices to give every CU one
        const long long wg = (long long)B * H * (((long long)N + 31) / 32);
        if (wg >= cus) return 1;
        const long long want = (cus + wg - 1) / wg;
        return plan_splits(N, (int)(want < most ? want : most)).n_splits;
    }
    // 256-row workgroups, `resident` of them at once (two per CU at d = 64).  A launch of wg S
    // items takes rounds = ceil(wg S / resident) rounds, run equally full (balanced_grid); a round
    // filled to the fraction f of the chip takes about 0.5 + 0.5 f of a full round's time (the
    // part is power-bound: idle CUs give their share of the budget to the rest), and an item
    // spends about 3.5 tile times on its prologue and tail.  In units of one full round over all
    // keys: main(S) = (0.5 rounds / S + 0.5 wg / resident) (1 + 3.5 / tiles per slice); the combine
    // step adds its launch (about 3 tile times) and S passes over wg / resident of the rows, 300 / N
    // of a round each.  Unsplit, a launch of at most `resident` 128-row workgroups costs
    // 0.6 (0.5 + wg / resident) on the same scale.  Measured against these (bf16, one GPU):
    // 1 x 8192 x 128: S = 8 44 us (4: 57, unsplit 99); 2 x 8192 x 128: S = 4; 1 x 32768 x 128: S = 2;
    // 8 x 4096 x 128: unsplit; 1 x 40000 x 128 (157 tiles): S = 3 533 us (2: 645, unsplit 629);
    // 3 x 16384 x 128 (192 tiles): S = 4 291 us (2: 300, unsplit 298); 5 x 16384 x 64: S = 3 251 (unsplit 285).
    // The same holds above one round: 8 x 20000 x 128 (632 tiles, 2.47 rounds): S = 2 1080 us, unsplit 1174.
    const long long wg = (long long)B * H * (((long long)N + 255) / 256);
    const long long resident = cus * (d == 64 ? 2 : 1);
    const double share = (double)wg / (double)resident;
    const double edge = 3.5;
    const long long rounds1 = (wg + resident - 1) / resident;
    double best = (0.5 * (double)rounds1 + 0.5 * share) * (1.0 + edge / (double)tiles);
    if (d == 64 && (dtype == SPHATTN_BF16 || dtype == SPHATTN_F16) && wg > resident && wg % resident != 0 &&
        2 * (wg % resident) <= resident) {
        // the unsplit launch runs this remainder as 128-row halves (launch_pipelined)
        const double halves = ((double)(wg / resident) + 0.3 + 0.6 * (double)(wg % resident) / (double)resident) *
                              (1.0 + edge / (double)tiles);
        best = halves < best ? halves : best;
    }
    if (wg < resident && (long long)B * H * (((long long)N + 127) / 128) <= resident) {
        const double narrow = 0.6 * (0.5 + share) * (1.0 + edge / (double)tiles);
        best = narrow < best ? narrow : best;
    }
    best *= 0.97;                                  // split only for a gain of at least 3 %
    int pick = 1;
    for (long long S = 2; S <= most && S <= 32; ++S) {
        const SplitPlan plan = plan_splits(N, (int)S);
        if (plan.n_splits != S) continue;          // this count does not divide the tiles: same as a smaller one
        const long long rounds = (wg * S + resident - 1) / resident;
        const double per = (double)(plan.keys_per_split / kBC);
        const double cost = (0.5 * (double)rounds / (double)S + 0.5 * share) * (1.0 + edge / per)
                            + 3.0 / (double)tiles + (double)S * share * 300.0 / (double)N;
        // above one round the workspace is large: more slices only for more than 1 %
        if (cost < (wg >= resident ? 0.99 : 1.0) * best) {
            best = cost;
            pick = (int)S;
        }
    }
    return pick;
}

int sphattn_splitkv_fwd(const void* Q, const void* K, const void* V, const float* mult, void* O, float* Z,
                        int B, int H, int H_kv, int N, int d, int dtype, int n_splits,
                        void* workspace, size_t workspace_size, void* stream)
{
    const int rc = check_args(Q, K, V, O, out_bytes_of(B, H, N, d, dtype), mult, Z, B, H, H_kv, N, N, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    if (n_splits < 0) return SPHATTN_ERR_SHAPE;
    if (n_splits == 0) n_splits = sphattn_splitkv_heuristic(B, H, N, d, dtype);
    const SplitPlan plan = plan_splits(N, n_splits);
    const size_t need = sphattn_splitkv_workspace_bytes(B, H, N, d, plan.n_splits);
    if (!workspace || need == 0 || workspace_size < need || ((uintptr_t)workspace & 15)) return SPHATTN_ERR_WORKSPACE;
    const size_t ob = out_bytes_of(B, H, N, d, dtype);
    const size_t nq = (size_t)B * H * N * d, nkv = (size_t)B * H_kv * N * d;
    const size_t qk = dtype == SPHATTN_F32 ? 4 : dtype == SPHATTN_FP8QK_BF16V ? 1 : 2;
    const size_t vo = dtype == SPHATTN_F32 ? 4 : 2;
    if (wraps(workspace, need)) return SPHATTN_ERR_WORKSPACE;
    if (overlaps(workspace, need, Q, nq * qk) || overlaps(workspace, need, K, nkv * qk) ||
        overlaps(workspace, need, V, nkv * vo) || overlaps(workspace, need, O, ob) ||
        (mult && overlaps(workspace, need, mult, (size_t)B * N * 4)) ||
        (Z && overlaps(workspace, need, Z, (size_t)B * H * N * 4)))
        return SPHATTN_ERR_ALIAS;
    return run_splitkv(Q, K, V, mult, O, Z, B, H, H_kv, N, d, dtype, plan, workspace, (hipStream_t)stream);
}

int sphattn_splitkv_fwd_noalloc(const void* Q, const void* K, const void* V, const float* mult, void* O, float* Z,
                                int B, int H, int H_kv, int N, int d, int dtype, int n_splits, void* stream)
{
    const int rc = check_args(Q, K, V, O, out_bytes_of(B, H, N, d, dtype), mult, Z, B, H, H_kv, N, N, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    if (n_splits < 0) return SPHATTN_ERR_SHAPE;
    if (n_splits == 0) {                           // the library's choice, if the array holds it
        n_splits = sphattn_splitkv_heuristic(B, H, N, d, dtype);
        if (sphattn_splitkv_workspace_bytes(B, H, N, d, plan_splits(N, n_splits).n_splits) > (size_t)SPHATTN_NOALLOC_SCRATCH_BYTES)
            n_splits = 1;
    }
    const SplitPlan plan = plan_splits(N, n_splits);
    // one slice is the unsplit launch and needs no scratch
    if (plan.n_splits == 1) return run_splitkv(Q, K, V, mult, O, Z, B, H, H_kv, N, d, dtype, plan, nullptr, (hipStream_t)stream);
    const size_t need = sphattn_splitkv_workspace_bytes(B, H, N, d, plan.n_splits);
    if (need == 0 || need > (size_t)SPHATTN_NOALLOC_SCRATCH_BYTES) return SPHATTN_ERR_SCRATCH;
    void* ws = scratch_address();
    if (ws == nullptr) return SPHATTN_ERR_LAUNCH;
    // the caller's buffers are allocations of their own and cannot overlap the library's array
    return run_splitkv(Q, K, V, mult, O, Z, B, H, H_kv, N, d, dtype, plan, ws, (hipStream_t)stream);
}

int sphattn_grn_bwd(const void* Q, const void* K, const void* V, const float* mult,
                    const void* O, const void* dO, const float* Z,
                    void* dQ, void* dK, void* dV, float* delta,
                    int B, int H, int H_kv, int N, int d, int dtype, void* stream)
{
    if (!Q || !K || !V || !O || !dO || !Z || !dQ || !dK || !dV || !delta) return SPHATTN_ERR_NULL;
    const int rc = check_shape(B, H, H_kv, N, N, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    if (dtype != SPHATTN_BF16 && dtype != SPHATTN_F16) return SPHATTN_ERR_DTYPE;
    if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O | (uintptr_t)dO |
         (uintptr_t)dQ | (uintptr_t)dK | (uintptr_t)dV) & 15)
        return SPHATTN_ERR_ALIGN;
    if (((uintptr_t)Z | (uintptr_t)delta | (uintptr_t)mult) & 3) return SPHATTN_ERR_ALIGN;
    const size_t tq = (size_t)B * H * N * d * 2, tkv = (size_t)B * H_kv * N * d * 2, rb = (size_t)B * H * N * 4;
    const void* ins[7] = {Q, K, V, O, dO, Z, mult};
    const size_t in_bytes[7] = {tq, tkv, tkv, tq, tq, rb, mult ? (size_t)B * N * 4 : 0};
    void* outs[4] = {dQ, dK, dV, delta};
    const size_t out_bytes[4] = {tq, tkv, tkv, 2 * rb};
    for (int o = 0; o < 4; ++o) {
        for (int i = 0; i < 7; ++i)
            if (ins[i] && overlaps(outs[o], out_bytes[o], ins[i], in_bytes[i])) return SPHATTN_ERR_ALIAS;
        for (int q = o + 1; q < 4; ++q)
            if (overlaps(outs[o], out_bytes[o], outs[q], out_bytes[q])) return SPHATTN_ERR_ALIAS;
    }
    const BwdProblem p{Q, K, V, mult, O, dO, Z, dQ, dK, dV, delta, B, H, H_kv, N, (hipStream_t)stream};
    return mult ? dispatch_bwd<true>(p, d, dtype) : dispatch_bwd<false>(p, d, dtype);
}

int sphattn_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* Z,
                void* dQ, void* dK, void* dV, float* delta,
                int B, int H, int N, int d, int dtype, void* stream)
{
    return sphattn_grn_bwd(Q, K, V, nullptr, O, dO, Z, dQ, dK, dV, delta, B, H, H, N, d, dtype, stream);
}

size_t sphattn_fp8_workspace_bytes(int B, int H_kv, int N, int d)
{
    if (B <= 0 || H_kv <= 0 || N <= 0 || (d != 64 && d != 128)) return 0;
    const size_t tiles = ((size_t)N + kFp8Tile - 1) / kFp8Tile;
    return (size_t)B * H_kv * d * tiles * kFp8Tile + (((size_t)B * H_kv * 4 + 255) & ~(size_t)255);
}

int sphattn_fp8_fwd(const void* Q, const void* K, const void* V, void* O, void* workspace,
                    size_t workspace_bytes, int B, int H, int H_kv, int N, int d, void* stream)
{
    return fp8_forward(Q, K, V, nullptr, O, workspace, workspace_bytes, B, H, H_kv, N, d, stream, false);
}

int sphattn_fp8_grn_fwd(const void* Q, const void* K, const void* V, const float* mult, void* O, void* workspace,
                        size_t workspace_bytes, int B, int H, int H_kv, int N, int d, void* stream)
{
    return fp8_forward(Q, K, V, mult, O, workspace, workspace_bytes, B, H, H_kv, N, d, stream, false);
}

int sphattn_fp8_softmax_fwd(const void* Q, const void* K, const void* V, void* O, void* workspace,
                            size_t workspace_bytes, int B, int H, int H_kv, int N, int d, void* stream)
{
    return fp8_forward(Q, K, V, nullptr, O, workspace, workspace_bytes, B, H, H_kv, N, d, stream, true);
}

const char* sphattn_strerror(int code)
{
    switch (code) {
    case SPHATTN_OK: return "success";
    case SPHATTN_ERR_NULL: return "a required pointer is NULL";
    case SPHATTN_ERR_SHAPE: return "B, H, N must be positive, H_kv must divide H, and sizes must not overflow";
    case SPHATTN_ERR_HEAD_DIM: return "head dimension d must be 64 or 128";
    case SPHATTN_ERR_DTYPE: return "unsupported dtype for this entry point";
    case SPHATTN_ERR_ALIGN: return "Q, K, V and O must be 16-byte aligned";
    case SPHATTN_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    case SPHATTN_ERR_ALIAS: return "O must not overlap Q, K or V";
    case SPHATTN_ERR_NORMALIZER: return "normalizer is not a sphattn_normalizer value";
    case SPHATTN_ERR_WORKSPACE: return "workspace is NULL, misaligned or smaller than the entry point's *_workspace_bytes";
    case SPHATTN_ERR_SCRATCH: return "the problem needs more scratch than the library's own array holds (SPHATTN_NOALLOC_SCRATCH_BYTES)";
    default: return "unknown sphattn error code";
    }
}

int sphattn_version(void) { return kVersion; }


}  // extern "C"
