// Device code shared by the spherical-attention kernels for gfx950 (CDNA4, 64-wide
// wavefronts): vector types, LDS and lane-exchange helpers, the fp32 kernel for fp32 storage
// and the kernel that combines partial accumulators.  The main kernel for 16-bit and fp8
// storage is in sphattn_pipelined.hpp.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sphattn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;

#define SPH_LDS __attribute__((address_space(3)))

constexpr int kWaves = 4;          // wavefronts per workgroup, one per SIMD
constexpr int kThreads = 64 * kWaves;
constexpr int kXcds = 8;           // accelerator complex dies, each with its own L2
constexpr int kBC = 64;            // key rows per LDS tile
constexpr int kNBuf = 4;           // LDS tile buffers in rotation

// Normalizers N(x)_i = a1(x_i) / b(sum_j a2(x_j)) of Appendix A.1, Definition 2:
//   Spherical (x, x^2, sqrt)   Softmax (exp, exp, id; with running maximum)
//   L1 (x, |x|, id)            SqRelu (relu(x)^2, relu(x)^2, id)
enum class Norm { Spherical, Softmax, L1, SqRelu };
// Storage: Bf16 = Q,K,V,O bfloat16; Fp8 = Q,K OCP E4M3 with V,O bfloat16; F16 = Q,K,V,O IEEE half
// (the paper's own precision).  The 16-bit type of V and O is also the type P is rounded to.
enum class QKType { Bf16, Fp8, F16 };

// Workgroup ids are dealt round-robin to the 8 XCDs.  Remap so that each XCD
// works through a contiguous range of (head, query-tile) pairs: the query tiles
// that run together on one XCD then stream the same K/V through one L2.
__device__ __forceinline__ int xcd_contiguous_id(int wg, int n_wg)
{
    int xcd = wg % kXcds, idx = wg / kXcds;
    int base = n_wg / kXcds, rem = n_wg % kXcds;
    int start = xcd * base + (xcd < rem ? xcd : rem);
    return start + idx;
}

// Row padding of the SoftMax-specific kernel (sphattn_softmax32.hpp), whose tiles are staged
// through registers into row-major LDS rows; the spherical kernel stores unpadded fragment
// blocks instead and does not use these.
//   K rows: +16 bytes.  16 lanes reading the same column of 16 consecutive rows (the
//           matrix-core A-operand pattern, ds_read_b128) then hit 16 different 16-byte groups
//           of the 256-byte LDS line.
//   V rows: +64 bytes.  The 16 lanes of a transposing-read block touch 4 consecutive rows x
//           32 bytes; consecutive rows land in different 64-byte groups.
constexpr int kKPad = 16;
constexpr int kVPad = 64;

__device__ __forceinline__ i32x4 lds_read_b128(const SPH_LDS unsigned char* p)
{
    return *reinterpret_cast<const SPH_LDS i32x4*>(p);
}

__device__ __forceinline__ float lds_read_f32(const SPH_LDS unsigned char* p)
{
    return *reinterpret_cast<const SPH_LDS float*>(p);
}

// Keeps the workgroups that share a CU at the same place of the stream they all read.  With two
// waves per SIMD the arbiter prefers the older one, so one workgroup of a pair pulls ahead until
// the tiles it streamed have left the L2 by the time the other asks for them (measured on the
// forward at d = 64, N = 32768: 32 workgroups per XCD read K and V from HBM once, 64 read them
// 1.6 times).  Called at the top of tile j: the wave priority falls with the tile index in steps
// of 8 tiles, modulo 4, so whichever wave is behind, by up to three steps, holds the higher
// priority and catches up.  s_setprio takes an immediate, hence the switch; it sits in front of
// the tile's instruction sequence, which stays one basic block.
__device__ __forceinline__ void priority_by_tile(int j)
{
    if ((j & 7) == 0) {
        switch ((j >> 3) & 3) {
        case 0: __builtin_amdgcn_s_setprio(3); break;
        case 1: __builtin_amdgcn_s_setprio(2); break;
        case 2: __builtin_amdgcn_s_setprio(1); break;
        default: __builtin_amdgcn_s_setprio(0); break;
        }
    }
}

// Fragment blocks in LDS: 16 rows x 64 bytes = 1 KB, filled by one direct global -> LDS copy
// (lane l lands at byte 16 l: row l / 4, slot l % 4) and read as matrix operands, lane (n16, g)
// taking the 16-byte piece g of row n16.  The LDS has 64 banks of 4 bytes; a 16-byte read
// instruction is served in four passes of 16 lanes, and the lanes of a pass are not consecutive:
// in units of four lanes q = lane / 4, a pass holds the q with the same bit 3 and the same
// parity of bits 0..2 ({0-3, 12-15, 20-27}, {4-11, 16-19, 28-31}, and the same in the upper
// half); the transposing 8-byte read is served in two passes of 32 consecutive lanes (measured
// with a probe that moves one lane onto another's banks, and with SQ_LDS_BANK_CONFLICT).  With
// piece g in slot g, the lanes of a pass fall on 8 of the 16 bank groups and every fragment
// read takes 8 cycles of the LDS instead of 4.  With piece c of row r in slot c ^ ((r >> 1) & 3)
// every pass covers all 64 banks, for the row-major read and for the transposing read alike.
// The copies permute within a row's 64 bytes only, so their global accesses stay whole rows.
__device__ __forceinline__ int block_piece_offset(int row, int piece)
{
    return row * 64 + ((piece ^ (row >> 1)) & 3) * 16;
}
// the piece that copy lane `lane` has to fetch for its slot
__device__ __forceinline__ int block_piece_in_slot(int lane)
{
    return (lane ^ (lane >> 3)) & 3;
}


// ds_read_b64_tr_b16: each lane supplies the address of 4 consecutive 16-bit elements; within
// every block of 16 lanes the 16 x 4 elements are transposed, so lane i receives element (i & 3)
// of the pieces supplied by lanes (i >> 2), 4 + (i >> 2), 8 + (i >> 2), 12 + (i >> 2).
__device__ __forceinline__ i32x2 lds_read_tr64(const SPH_LDS unsigned char* p)
{
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (SPH_LDS s16x4*)const_cast<SPH_LDS unsigned char*>(p));
    return __builtin_bit_cast(i32x2, v);
}

// Two fp32 values rounded (to nearest even) and packed into one register of the 16-bit type.
template <bool HALF>
__device__ __forceinline__ int pack2(float a, float b)
{
    f32x2 v = {a, b};
    if constexpr (HALF) return __builtin_bit_cast(int, __builtin_convertvector(v, f16x2));   // v_cvt_pk_f16_f32
    else return __builtin_bit_cast(int, __builtin_convertvector(v, bf16x2));                 // v_cvt_pk_bf16_f32
}

// D = A(32 x 16) B(16 x 32) + C on 16-bit operands held as 4 raw registers each.
template <bool HALF>
__device__ __forceinline__ f32x16 mfma16(i32x4 a, i32x4 b, f32x16 c)
{
    if constexpr (HALF)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// v_permlane32_swap exchanges the upper 32 lanes of its first operand with the lower 32 lanes
// of its second.  Fed two copies of x it leaves x[lane & 31] in the first and
// x[32 + (lane & 31)] in the second register of every lane: one instruction, no LDS traffic.
// Written as inline assembly (with the wait states the instruction needs around it) because
// the compiler builtin hands back the same register for both results.
struct HalfPair { float lo, hi; };
__device__ __forceinline__ HalfPair both_halves(float x)
{
    float a = x, b = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
    return HalfPair{a, b};
}

__device__ __forceinline__ float max_across_halves(float x)
{
    const HalfPair r = both_halves(x);
    return fmaxf(r.lo, r.hi);
}

__device__ __forceinline__ float sum_across_halves(float x)
{
    const HalfPair r = both_halves(x);
    return r.lo + r.hi;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

// 8-byte store at byte `offset` of the buffer, ordinary or non-temporal (past the L2's retention).
// The policy is an immediate of the instruction; written as two buffer stores rather than as a
// pointer store with and without the non-temporal hint, which the compiler merges into one
// ordinary store when both sit in the arms of a branch.
__device__ __forceinline__ void store_b128(__amdgpu_buffer_rsrc_t rsrc, int offset, i32x4 v, bool non_temporal)
{
    if (non_temporal) __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, offset, 0, 2);   // aux 2: nt
    else __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, offset, 0, 0);
}

// A wave's finished output tile, ROWS rows of ROWB bytes that the lanes hold as 8-byte pieces
// (accumulator layout), goes through LDS so that every store instruction writes whole rows:
// 16 bytes per lane, consecutive lanes consecutive bytes.  Non-temporal stores of partial lines
// are written through piece by piece (measured: 2.3 times the bytes at the memory interface
// with 8-byte pieces); whole lines are not.  `stage` is this wave's private LDS region of
// ROWS * (ROWB + 16) bytes (rows padded by 16 bytes against bank conflicts); put_piece fills it,
// store_tile writes rows row0 .. of the buffer, those below n_rows only.
template <int ROWB>
__device__ __forceinline__ void put_piece(SPH_LDS unsigned char* stage, int row, int byte, i32x2 v)
{
    *reinterpret_cast<SPH_LDS i32x2*>(stage + row * (ROWB + 16) + byte) = v;
}

template <int ROWS, int ROWB>
__device__ __forceinline__ void store_tile(const SPH_LDS unsigned char* stage, __amdgpu_buffer_rsrc_t rsrc,
                                           int row0, int n_rows, int lane, bool non_temporal)
{
    constexpr int LPR = ROWB / 16;                 // lanes per row
#pragma unroll
    for (int i = 0; i < ROWS * LPR / 64; ++i) {
        const int r = i * (64 / LPR) + lane / LPR, c = (lane % LPR) * 16;
        const i32x4 v = *reinterpret_cast<const SPH_LDS i32x4*>(stage + r * (ROWB + 16) + c);
        if (row0 + r < n_rows) store_b128(rsrc, (row0 + r) * ROWB + c, v, non_temporal);
    }
}

// ---------------------------------------------------------------------------
// fp32 Q/K/V/O kernel on the fp32 matrix instruction v_mfma_f32_32x32x2_f32.
// Same mapping as above with k = 2 per instruction: lane l holds row/column
// (l & 31) and k index (l >> 5), so accumulator register 4g+t of S^T (key
// 8g + 4h + t) is directly the B operand of the k-step that pairs it with the
// V row of that key; V needs no transpose (one scalar per lane).
//
// fp32 problems are small and latency-bound, so the work is cut for parallelism
// rather than for reuse: a workgroup owns 32 query rows, and its four wavefronts
// split the KEY axis (wave w takes key tiles w, w+4, ...), each carrying its own
// partial (o, z).  Lemma 1's accumulator is a plain sum, so the four partials are
// simply added (through LDS) before the tail o / sqrt(z) is applied once.  Each
// wave stages its tiles in a private LDS region; there is no workgroup barrier in
// the loop.
// ---------------------------------------------------------------------------
// Nq, Nk, Zv, PARTIAL, n_splits and keys_per_split as in fwd_pipelined_kernel.
template <int D, bool MULT, bool PARTIAL = false>
__global__ __launch_bounds__(kThreads, 1)
void fwd_f32_kernel(const float* __restrict__ Q, const float* __restrict__ K,
                    const float* __restrict__ V, float* __restrict__ O,
                    const float* __restrict__ mult, float* __restrict__ Zv,
                    int Nq, int Nk, int H, int kv_group, int n_qtiles, int n_wg,
                    int n_splits, int keys_per_split)
{
    constexpr int BC = 32;                         // keys per tile
    constexpr int ROWF = D + 4;                    // padded row, in floats: conflict-free columns
    constexpr int TILE_F = BC * ROWF;
    constexpr int WAVE_F = 2 * TILE_F;             // K tile then V tile, private to a wave
    constexpr int DB = D / 32;
    constexpr int LD = BC * D / 4 / 64;            // float4 loads per lane per tensor per tile
    static_assert(kWaves * (DB * 16 + 1) * 64 <= kWaves * WAVE_F, "partials fit the staging space");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    SPH_LDS float* smem = (SPH_LDS float*)smem_raw;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int lid = xcd_contiguous_id(blockIdx.x, n_wg);
    const int qt = lid % n_qtiles;
    const int split = PARTIAL ? (lid / n_qtiles) % n_splits : 0;
    const int bh = PARTIAL ? lid / (n_qtiles * n_splits) : lid / n_qtiles;
    const size_t head_off = (size_t)bh * Nq * D;
    const int bidx = bh / H;
    const int k0 = PARTIAL ? split * keys_per_split : 0;
    const int N = PARTIAL ? min(Nk - k0, keys_per_split) : Nk;      // keys k0 .. k0 + N - 1
    const size_t kv_off = ((size_t)(bidx * (H / kv_group) + (bh % H) / kv_group) * Nk + k0) * D;
    const float* Qh = Q + head_off;
    const float* Kh = K + kv_off;
    const float* Vh = V + kv_off;
    const float* mrow = MULT ? mult + (size_t)bidx * Nk + k0 : nullptr;
    const int q0 = qt * 32;

    // Q as B operand of S^T = K Q^T: lane holds Q[q0 + l32][2kk + h]
    float qf[D / 2];
    {
        int row = q0 + l32;
        row = row < Nq ? row : Nq - 1;
#pragma unroll
        for (int kk = 0; kk < D / 2; ++kk) qf[kk] = Qh[(size_t)row * D + 2 * kk + h];
    }
    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float z = 0.f;

    SPH_LDS float* kb = smem + wave * WAVE_F;
    SPH_LDS float* vb = kb + TILE_F;
    f32x4 kreg[LD], vreg[LD];
    auto load_tile = [&](int j0) {
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int id = lane + i * 64;
            const int r = id / (D / 4), c = id % (D / 4);
            if (j0 + r < N) {
                kreg[i] = *reinterpret_cast<const f32x4*>(Kh + (size_t)(j0 + r) * D + 4 * c);
                vreg[i] = *reinterpret_cast<const f32x4*>(Vh + (size_t)(j0 + r) * D + 4 * c);
            } else {                               // zero keys add nothing to o or z
                kreg[i] = f32x4{0, 0, 0, 0};
                vreg[i] = f32x4{0, 0, 0, 0};
            }
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int id = lane + i * 64;
            const int r = id / (D / 4), c = id % (D / 4);
            *reinterpret_cast<SPH_LDS f32x4*>(kb + r * ROWF + 4 * c) = kreg[i];
            *reinterpret_cast<SPH_LDS f32x4*>(vb + r * ROWF + 4 * c) = vreg[i];
        }
    };

    const int n_tiles = (N + BC - 1) / BC;
    if (wave < n_tiles) load_tile(wave * BC);
    for (int jt = wave; jt < n_tiles; jt += kWaves) {
        // LDS executes one wave's operations in order: the reads of the previous tile are done
        // before these writes land, and the reads below see them
        store_tile();
        if (jt + kWaves < n_tiles) load_tile((jt + kWaves) * BC);
        // S^T (32 keys x 32 queries)
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < D / 2; ++kk)
            s = __builtin_amdgcn_mfma_f32_32x32x2f32(kb[l32 * ROWF + 2 * kk + h], qf[kk], s, 0, 0, 0);
        if constexpr (MULT) {                    // s_ij = m_j (q_i . k_j); keys past N are zero
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = jt * BC + 8 * (r >> 2) + 4 * h + (r & 3);
                s[r] *= key < N ? mrow[key] : 0.f;
            }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) z = __builtin_fmaf(s[r], s[r], z);
        // O^T (D x 32 queries) += V^T S^T: k-step r pairs key 8(r>>2) + 4h + (r&3) on both sides
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = 8 * (r >> 2) + 4 * h + (r & 3);
#pragma unroll
            for (int db = 0; db < DB; ++db)
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x2f32(vb[key * ROWF + db * 32 + l32], s[r], oacc[db], 0, 0, 0);
        }
    }

    // ---- add the four waves' partial (o, z): register r of block db of wave w at
    // part[w][db*16 + r][lane], z at part[w][DB*16][lane]
    __syncthreads();                               // every wave is done with its staging space
    constexpr int PART = (DB * 16 + 1) * 64;
    SPH_LDS float* part = smem;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) part[wave * PART + (db * 16 + r) * 64 + lane] = oacc[db][r];
    part[wave * PART + DB * 16 * 64 + lane] = z;
    __syncthreads();

    // wave w finishes output block db = w (32 columns of the head dimension)
    if (wave < DB) {
        float zt = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) zt += part[w * PART + DB * 16 * 64 + lane];
        zt = sum_across_halves(zt);
        const float inv = PARTIAL ? 1.f : zt > 0.f ? 1.0f / __builtin_sqrtf(zt) : 0.f;
        const int row = q0 + l32;
        // partial: the fp32 pair (o, z) of this key slice, slice-major
        const size_t rows0 = PARTIAL ? ((size_t)split * (n_wg / (n_qtiles * n_splits)) + bh) * Nq
                                     : (size_t)bh * Nq;
        if (wave == 0 && h == 0 && row < Nq && (PARTIAL || Zv != nullptr)) Zv[rows0 + row] = zt;
        float* dst = O + (rows0 + row) * D + wave * 32 + 4 * h;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            f32x4 o4;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                float acc = 0.f;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) acc += part[w * PART + (wave * 16 + 4 * g + t) * 64 + lane];
                o4[t] = acc * inv;
            }
            if (row < Nq) *reinterpret_cast<f32x4*>(dst + 8 * g) = o4;
        }
    }
}

// ---------------------------------------------------------------------------
// Adds the partial pairs (o, z) of n_parts key slices and applies the tail once
// (Lemma 1: the accumulator of a concatenation is the sum of the accumulators):
//     O[r,:] = (sum_p o_p[r,:]) / sqrt(sum_p z_p[r])        (0 if the sum of z is 0)
// rows = B*H*N query rows; part p starts rows*D floats (o) / rows floats (z) after part
// p-1.  One thread per 4 output columns; the parts are added in ascending order, so the
// result does not depend on the launch.  OUT: 0 fp32, 1 bfloat16, 2 IEEE half.
// ---------------------------------------------------------------------------
template <int D, int OUT>
__global__ __launch_bounds__(256)
void combine_kernel(const float* __restrict__ o_parts, const float* __restrict__ z_parts,
                    int n_parts, void* __restrict__ Ov, float* __restrict__ Zv, size_t rows)
{
    constexpr int C4 = D / 4;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t row = idx / C4;
    const int c4 = (int)(idx % C4);
    if (row >= rows) return;
    float z = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int p = 0; p < n_parts; ++p) {
        z += z_parts[(size_t)p * rows + row];
        acc += *reinterpret_cast<const f32x4*>(o_parts + ((size_t)p * rows + row) * D + 4 * c4);
    }
    const float inv = z > 0.f ? 1.0f / __builtin_sqrtf(z) : 0.f;
    if (Zv != nullptr && c4 == 0) Zv[row] = z;
    if constexpr (OUT == 0) {
        *reinterpret_cast<f32x4*>((float*)Ov + row * D + 4 * c4) = acc * inv;
    } else {
        const i32x2 o4 = {pack2<OUT == 2>(acc[0] * inv, acc[1] * inv), pack2<OUT == 2>(acc[2] * inv, acc[3] * inv)};
        *reinterpret_cast<i32x2*>((unsigned short*)Ov + row * D + 4 * c4) = o4;
    }
}

}  // namespace sphattn
