// Host side of the C ABI declared in include/sphattn.h: argument checks, kernel
// selection by (dtype, d), launch on the caller's stream.  Allocates nothing and
// never synchronises.
#include "sphattn_device.hpp"
#include "../../include/sphattn.h"

#include <stdint.h>

namespace {

using namespace sphattn;

constexpr int kVersion = 100;   // 0.1.0

bool overlaps(const void* a, size_t an, const void* b, size_t bn)
{
    uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + bn && b0 < a0 + an;
}

int check_args(const void* Q, const void* K, const void* V, void* O,
               int B, int H, int N, int d, int dtype, size_t* qk_bytes, size_t* vo_bytes)
{
    if (!Q || !K || !V || !O) return SPHATTN_ERR_NULL;
    if (B <= 0 || H <= 0 || N <= 0) return SPHATTN_ERR_SHAPE;
    if (d != 64 && d != 128) return SPHATTN_ERR_HEAD_DIM;
    if (dtype != SPHATTN_F32 && dtype != SPHATTN_BF16 && dtype != SPHATTN_FP8QK_BF16V)
        return SPHATTN_ERR_DTYPE;
    // B*H*N*d elements must be addressable with 64-bit offsets and B*H*tiles with int
    unsigned __int128 elems = (unsigned __int128)B * H * (unsigned __int128)N * d;
    if (elems > ((unsigned __int128)1 << 40)) return SPHATTN_ERR_SHAPE;
    if ((unsigned __int128)B * H * (((unsigned __int128)N + 127) / 128) > 0x7fffffff)
        return SPHATTN_ERR_SHAPE;
    // one head of one tensor is addressed through a 32-bit buffer range
    if ((unsigned __int128)N * d * 4 > 0x7fffffff) return SPHATTN_ERR_SHAPE;
    if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15) return SPHATTN_ERR_ALIGN;
    size_t n = (size_t)elems;
    size_t qk = dtype == SPHATTN_F32 ? 4 : dtype == SPHATTN_BF16 ? 2 : 1;
    size_t vo = dtype == SPHATTN_F32 ? 4 : 2;
    *qk_bytes = n * qk;
    *vo_bytes = n * vo;
    if (overlaps(O, *vo_bytes, Q, *qk_bytes) || overlaps(O, *vo_bytes, K, *qk_bytes) ||
        overlaps(O, *vo_bytes, V, *vo_bytes))
        return SPHATTN_ERR_ALIAS;
    return SPHATTN_OK;
}

template <typename Kern>
bool raise_lds_limit(Kern kern, int lds_bytes)
{
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                            lds_bytes) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return true;
}

template <int D, int QB, QKType QKT, Norm NORM>
int launch_pipelined(const void* Q, const void* K, const void* V, void* O,
                     int B, int H, int N, hipStream_t stream)
{
    constexpr int BR = kWaves * 32 * QB;
    constexpr int EQ = QKT == QKType::Fp8 ? 1 : 2;
    constexpr int lds_bytes = kNBuf * kBC * (D * EQ + kKPad + D * 2 + kVPad);
    auto kern = fwd_pipelined_kernel<D, QB, QKT, NORM>;
    static const bool configured = raise_lds_limit(kern, lds_bytes);   // once per process
    if (!configured) return SPHATTN_ERR_LAUNCH;
    const int n_qtiles = (N + BR - 1) / BR;
    const int n_wg = B * H * n_qtiles;
    const float scale_log2 = 1.4426950408889634f / __builtin_sqrtf((float)D);
    hipLaunchKernelGGL(kern, dim3(n_wg), dim3(kThreads), lds_bytes, stream,
                       Q, K, (const __bf16*)V, (__bf16*)O, N, n_qtiles, n_wg, scale_log2);
    return hipGetLastError() == hipSuccess ? SPHATTN_OK : SPHATTN_ERR_LAUNCH;
}

template <int D>
int launch_f32(const void* Q, const void* K, const void* V, void* O,
               int B, int H, int N, hipStream_t stream)
{
    constexpr int BR = kWaves * 32;
    constexpr int lds_bytes = 2 * 2 * 32 * (D + 4) * 4;
    auto kern = fwd_f32_kernel<D>;
    static const bool configured = raise_lds_limit(kern, lds_bytes);
    if (!configured) return SPHATTN_ERR_LAUNCH;
    const int n_qtiles = (N + BR - 1) / BR;
    const int n_wg = B * H * n_qtiles;
    hipLaunchKernelGGL(kern, dim3(n_wg), dim3(kThreads), lds_bytes, stream,
                       (const float*)Q, (const float*)K, (const float*)V, (float*)O,
                       N, n_qtiles, n_wg);
    return hipGetLastError() == hipSuccess ? SPHATTN_OK : SPHATTN_ERR_LAUNCH;
}

template <Norm NORM>
int dispatch(const void* Q, const void* K, const void* V, void* O,
             int B, int H, int N, int d, int dtype, hipStream_t stream)
{
    if (dtype == SPHATTN_BF16) {
        if (d == 128) return launch_pipelined<128, 2, QKType::Bf16, NORM>(Q, K, V, O, B, H, N, stream);
        return launch_pipelined<64, 2, QKType::Bf16, NORM>(Q, K, V, O, B, H, N, stream);
    }
    if constexpr (NORM == Norm::Spherical) {
        if (dtype == SPHATTN_FP8QK_BF16V) {
            if (d == 128) return launch_pipelined<128, 2, QKType::Fp8, NORM>(Q, K, V, O, B, H, N, stream);
            return launch_pipelined<64, 2, QKType::Fp8, NORM>(Q, K, V, O, B, H, N, stream);
        }
        if (dtype == SPHATTN_F32) {
            if (d == 128) return launch_f32<128>(Q, K, V, O, B, H, N, stream);
            return launch_f32<64>(Q, K, V, O, B, H, N, stream);
        }
    }
    return SPHATTN_ERR_DTYPE;
}

}  // namespace

extern "C" {

int sphattn_fwd(const void* Q, const void* K, const void* V, void* O,
                int B, int H, int N, int d, int dtype, void* stream)
{
    size_t qk, vo;
    int rc = check_args(Q, K, V, O, B, H, N, d, dtype, &qk, &vo);
    if (rc != SPHATTN_OK) return rc;
    return dispatch<Norm::Spherical>(Q, K, V, O, B, H, N, d, dtype, (hipStream_t)stream);
}

int sphattn_softmax_fwd(const void* Q, const void* K, const void* V, void* O,
                        int B, int H, int N, int d, int dtype, void* stream)
{
    size_t qk, vo;
    int rc = check_args(Q, K, V, O, B, H, N, d, dtype, &qk, &vo);
    if (rc != SPHATTN_OK) return rc;
    if (dtype != SPHATTN_BF16) return SPHATTN_ERR_DTYPE;
    return dispatch<Norm::Softmax>(Q, K, V, O, B, H, N, d, dtype, (hipStream_t)stream);
}

const char* sphattn_strerror(int code)
{
    switch (code) {
    case SPHATTN_OK: return "success";
    case SPHATTN_ERR_NULL: return "a required pointer is NULL";
    case SPHATTN_ERR_SHAPE: return "B, H and N must be positive and B*H*N*d must not overflow";
    case SPHATTN_ERR_HEAD_DIM: return "head dimension d must be 64 or 128";
    case SPHATTN_ERR_DTYPE: return "unsupported dtype for this entry point";
    case SPHATTN_ERR_ALIGN: return "Q, K, V and O must be 16-byte aligned";
    case SPHATTN_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    case SPHATTN_ERR_ALIAS: return "O must not overlap Q, K or V";
    default: return "unknown sphattn error code";
    }
}

int sphattn_version(void) { return kVersion; }


}  // extern "C"
