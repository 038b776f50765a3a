// Host side of the C ABI declared in include/sphattn.h: argument checks, kernel
// selection by (dtype, d), launch on the caller's stream.  Allocates nothing and
// never synchronises.
#include "sphattn_device.hpp"
#include "../../include/sphattn.h"

#include <stdint.h>
#include <stdlib.h>

#include <atomic>

namespace {

using namespace sphattn;

constexpr int kVersion = 200;   // 0.2.0

bool overlaps(const void* a, size_t an, const void* b, size_t bn)
{
    uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + bn && b0 < a0 + an;
}

int check_args(const void* Q, const void* K, const void* V, void* O, const float* mult,
               int B, int H, int H_kv, int N, int d, int dtype)
{
    if (!Q || !K || !V || !O) return SPHATTN_ERR_NULL;
    if (B <= 0 || H <= 0 || N <= 0 || H_kv <= 0 || H % H_kv != 0) return SPHATTN_ERR_SHAPE;
    if (d != 64 && d != 128) return SPHATTN_ERR_HEAD_DIM;
    if (dtype != SPHATTN_F32 && dtype != SPHATTN_BF16 && dtype != SPHATTN_FP8QK_BF16V &&
        dtype != SPHATTN_F16)
        return SPHATTN_ERR_DTYPE;
    // B*H*N*d elements must be addressable with 64-bit offsets and B*H*tiles with int
    unsigned __int128 elems = (unsigned __int128)B * H * (unsigned __int128)N * d;
    if (elems > ((unsigned __int128)1 << 40)) return SPHATTN_ERR_SHAPE;
    if ((unsigned __int128)B * H * (((unsigned __int128)N + 127) / 128) > 0x7fffffff)
        return SPHATTN_ERR_SHAPE;
    // one head of one tensor is addressed through a 32-bit buffer range
    if ((unsigned __int128)N * d * 4 > 0x7fffffff) return SPHATTN_ERR_SHAPE;
    if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15) return SPHATTN_ERR_ALIGN;
    if ((uintptr_t)mult & 3) return SPHATTN_ERR_ALIGN;
    const size_t n = (size_t)elems, nkv = n / H * H_kv;
    const size_t qk = dtype == SPHATTN_F32 ? 4 : dtype == SPHATTN_FP8QK_BF16V ? 1 : 2;
    const size_t vo = dtype == SPHATTN_F32 ? 4 : 2;
    if (overlaps(O, n * vo, Q, n * qk) || overlaps(O, n * vo, K, nkv * qk) ||
        overlaps(O, n * vo, V, nkv * vo) ||
        (mult && overlaps(O, n * vo, mult, (size_t)B * N * 4)))
        return SPHATTN_ERR_ALIAS;
    return SPHATTN_OK;
}

// Kernels that use more than 64 KB of LDS need their limit raised once per device; `done` is
// that kernel's bit mask of devices already configured (the only state the library keeps).
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

struct Problem {
    const void* Q; const void* K; const void* V; void* O; const float* mult;
    int B, H, H_kv, N;
    hipStream_t stream;
};

template <int D, int QB, QKType QKT, Norm NORM, bool MULT>
int launch_pipelined(const Problem& p)
{
    constexpr int BR = kWaves * 32 * QB;
    constexpr int EQ = QKT == QKType::Fp8 ? 1 : 2;
    constexpr int lds_bytes = kNBuf * kBC * (D * EQ + kKPad + D * 2 + kVPad);
    auto kern = fwd_pipelined_kernel<D, QB, QKT, NORM, MULT>;
    static std::atomic<uint64_t> done{0};
    if (!raise_lds_limit(kern, lds_bytes, done)) return SPHATTN_ERR_LAUNCH;
    const int n_qtiles = (p.N + BR - 1) / BR;
    const int n_wg = p.B * p.H * n_qtiles;
    const float scale_log2 = 1.4426950408889634f / __builtin_sqrtf((float)D);
    hipLaunchKernelGGL(kern, dim3(n_wg), dim3(kThreads), lds_bytes, p.stream,
                       p.Q, p.K, p.V, p.O, p.mult,
                       p.N, p.H, p.H / p.H_kv, n_qtiles, n_wg, scale_log2);
    return hipGetLastError() == hipSuccess ? SPHATTN_OK : SPHATTN_ERR_LAUNCH;
}

template <int D, bool MULT>
int launch_f32(const Problem& p)
{
    constexpr int BR = 32;                         // the four waves split the key axis
    constexpr int lds_bytes = kWaves * 2 * 32 * (D + 4) * 4;
    auto kern = fwd_f32_kernel<D, MULT>;
    static std::atomic<uint64_t> done{0};
    if (!raise_lds_limit(kern, lds_bytes, done)) return SPHATTN_ERR_LAUNCH;
    const int n_qtiles = (p.N + BR - 1) / BR;
    const int n_wg = p.B * p.H * n_qtiles;
    hipLaunchKernelGGL(kern, dim3(n_wg), dim3(kThreads), lds_bytes, p.stream,
                       (const float*)p.Q, (const float*)p.K, (const float*)p.V, (float*)p.O, p.mult,
                       p.N, p.H, p.H / p.H_kv, n_qtiles, n_wg);
    return hipGetLastError() == hipSuccess ? SPHATTN_OK : SPHATTN_ERR_LAUNCH;
}

// Query rows per workgroup: 256 (64 per wave) is the efficient shape; 128 (32 per wave) reads
// K/V fragments twice as often per flop (measured 15-25 % slower per row) but doubles the
// number of workgroups.  It pays when 256-row tiles would leave CUs without any workgroup
// (measured: B=H=1, N=32768, d=128: 0.46 ms against 0.57 ms); partly filled last rounds do
// not justify it, because the part is power-bound and idle CUs give their share to the rest.
bool narrow_tiles_pay(const Problem& p)
{
    if (const char* e = getenv("SPHATTN_TILE_ROWS")) {
        if (e[0] == '1' && e[1] == '2' && e[2] == '8' && !e[3]) return true;
        if (e[0] == '2' && e[1] == '5' && e[2] == '6' && !e[3]) return false;
    }
    constexpr long long kCus = 256;
    return (long long)p.B * p.H * ((p.N + 255) / 256) < kCus;
}

template <Norm NORM, bool MULT>
int dispatch(const Problem& p, int d, int dtype)
{
    if (dtype == SPHATTN_BF16) {
        if constexpr (NORM == Norm::Spherical && !MULT) {
            if (narrow_tiles_pay(p)) {
                if (d == 128) return launch_pipelined<128, 1, QKType::Bf16, NORM, MULT>(p);
                return launch_pipelined<64, 1, QKType::Bf16, NORM, MULT>(p);
            }
        }
        if (d == 128) return launch_pipelined<128, 2, QKType::Bf16, NORM, MULT>(p);
        return launch_pipelined<64, 2, QKType::Bf16, NORM, MULT>(p);
    }
    if constexpr (NORM == Norm::Spherical) {
        if (dtype == SPHATTN_F16) {
            if (d == 128) return launch_pipelined<128, 2, QKType::F16, NORM, MULT>(p);
            return launch_pipelined<64, 2, QKType::F16, NORM, MULT>(p);
        }
        if (dtype == SPHATTN_FP8QK_BF16V) {
            if (d == 128) return launch_pipelined<128, 2, QKType::Fp8, NORM, MULT>(p);
            return launch_pipelined<64, 2, QKType::Fp8, NORM, MULT>(p);
        }
        if (dtype == SPHATTN_F32) {
            if (d == 128) return launch_f32<128, MULT>(p);
            return launch_f32<64, MULT>(p);
        }
    }
    return SPHATTN_ERR_DTYPE;
}

}  // namespace

extern "C" {

int sphattn_fwd(const void* Q, const void* K, const void* V, void* O,
                int B, int H, int N, int d, int dtype, void* stream)
{
    const int rc = check_args(Q, K, V, O, nullptr, B, H, H, N, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    const Problem p{Q, K, V, O, nullptr, B, H, H, N, (hipStream_t)stream};
    return dispatch<Norm::Spherical, false>(p, d, dtype);
}

int sphattn_grn_fwd(const void* Q, const void* K, const void* V, const float* mult, void* O,
                    int B, int H, int H_kv, int N, int d, int dtype, void* stream)
{
    const int rc = check_args(Q, K, V, O, mult, B, H, H_kv, N, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    const Problem p{Q, K, V, O, mult, B, H, H_kv, N, (hipStream_t)stream};
    return mult ? dispatch<Norm::Spherical, true>(p, d, dtype)
                : dispatch<Norm::Spherical, false>(p, d, dtype);
}

int sphattn_normalized_fwd(const void* Q, const void* K, const void* V, void* O,
                           int B, int H, int N, int d, int dtype, int normalizer, void* stream)
{
    const int rc = check_args(Q, K, V, O, nullptr, B, H, H, N, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    if (normalizer < SPHATTN_NORM_L2 || normalizer > SPHATTN_NORM_SQRELU) return SPHATTN_ERR_NORMALIZER;
    if (normalizer != SPHATTN_NORM_L2 && dtype != SPHATTN_BF16) return SPHATTN_ERR_DTYPE;
    const Problem p{Q, K, V, O, nullptr, B, H, H, N, (hipStream_t)stream};
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
    const int rc = check_args(Q, K, V, O, nullptr, B, H, H, N, d, dtype);
    if (rc != SPHATTN_OK) return rc;
    if (dtype != SPHATTN_BF16) return SPHATTN_ERR_DTYPE;
    const Problem p{Q, K, V, O, nullptr, B, H, H, N, (hipStream_t)stream};
    return dispatch<Norm::Softmax, false>(p, d, dtype);
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
    default: return "unknown sphattn error code";
    }
}

int sphattn_version(void) { return kVersion; }


}  // extern "C"
