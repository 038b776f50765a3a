// Device code for spherical attention forward on gfx950 (CDNA4, 64-wide wavefronts).
//
// One workgroup = 4 wavefronts = one tile of BR = 4*32*QB query rows of one (b,h).
// The key axis is streamed in tiles of BC rows (Theorem 1: the query axis is
// partitioned, the key axis is streamed); the only state carried between key
// tiles is the pair (o, z) of Lemma 1, held in fp32 registers:
//
//     o_i += sum_j s_ij * v_j        z_i += sum_j s_ij^2        tail: O_i = o_i / sqrt(z_i)
//
// Matrix-core mapping.  Scores are produced TRANSPOSED, S^T = K Q^T, with
// v_mfma_f32_32x32x16_bf16 (A = 32 keys x 16, B = 16 x 32 queries).  In the
// accumulator layout of that instruction lane l owns query column (l & 31) and,
// in register 4g+t, key row 8g + 4(l>>5) + t.  Eight consecutive accumulator
// registers are therefore exactly one B operand (8 k-slots of one query column)
// of the second contraction O^T += V^T P^T, so the scores never leave their
// registers: they are squared and summed into z in place (plain fp32 FMAs),
// rounded to bf16 in place, and fed straight back to the matrix cores.  The
// A operand V^T comes from the row-major V tile in LDS through the transposing
// read ds_read_b64_tr_b16.  z is a per-lane partial sum; the two lanes that
// share a query (l and l^32) are combined once, in the tail.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sphattn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;

#define SPH_LDS __attribute__((address_space(3)))

constexpr int kWaves = 4;          // wavefronts per workgroup, one per SIMD
constexpr int kThreads = 64 * kWaves;
constexpr int kXcds = 8;           // accelerator complex dies, each with its own L2

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

// 16-byte chunk slot of chunk c in row r of a tile whose rows hold CH chunks.
// Chosen so that 16 lanes reading one chunk column of 16 consecutive rows
// (the matrix-core A-operand pattern) touch 16 different 16-byte bank groups.
template <int CH>
__device__ __forceinline__ int kswz(int r, int c)
{
    if (CH >= 16) return c ^ (r & 15);
    return c ^ ((r >> 1) & 7);        // CH == 8: two rows share one 256-byte bank line
}

// V tile swizzle for the transposing read: the 16 lanes of a read block touch
// 4 consecutive rows x 32 bytes; spread the 4 rows over different 64-byte groups.
template <int CH>
__device__ __forceinline__ int vswz(int r, int c)
{
    if (CH >= 16) return c ^ ((r & 3) << 2);
    return c ^ ((r & 1) << 2) ^ ((r >> 1) & 1) * 2;
}

__device__ __forceinline__ bf16x8 lds_read_b128(const SPH_LDS unsigned char* p)
{
    return *reinterpret_cast<const SPH_LDS bf16x8*>(p);
}

__device__ __forceinline__ bf16x4 lds_read_tr64(const SPH_LDS unsigned char* p)
{
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (SPH_LDS s16x4*)const_cast<SPH_LDS unsigned char*>(p));
    return __builtin_bit_cast(bf16x4, v);
}

__device__ __forceinline__ bf16x2 cvt2(float a, float b)
{
    f32x2 v = {a, b};
    return __builtin_convertvector(v, bf16x2);   // v_cvt_pk_bf16_f32, round to nearest even
}

enum class Norm { Spherical, Softmax };

// ---------------------------------------------------------------------------
// bf16 Q/K/V/O kernel.
//   D   head dimension (64 or 128)
//   QB  32-query blocks per wavefront (rows per workgroup = 128*QB)
//   BC  key rows per LDS tile (multiple of 32)
// LDS: 2 buffers x (K tile + V tile), each BC x D bf16, 16-byte chunks swizzled.
// ---------------------------------------------------------------------------
template <int D, int QB, int BC, Norm NORM>
__global__ __launch_bounds__(kThreads, 1)
void fwd_bf16_kernel(const __bf16* __restrict__ Q, const __bf16* __restrict__ K,
                     const __bf16* __restrict__ V, __bf16* __restrict__ O,
                     int N, int n_qtiles, int n_wg, float softmax_scale_log2)
{
    constexpr int BR = kWaves * 32 * QB;
    constexpr int CH = D * 2 / 16;                 // 16-byte chunks per row
    constexpr int TILE_BYTES = BC * D * 2;
    constexpr int CHUNKS = BC * CH;                // per tile
    constexpr int LD_PER_THREAD = CHUNKS / kThreads;
    static_assert(CHUNKS % kThreads == 0, "tile must divide over the workgroup");
    constexpr int KSTEPS = D / 16;                 // MFMA k-steps in Q K^T
    constexpr int DB = D / 32;                     // 32-wide blocks of the head dimension

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    SPH_LDS unsigned char* smem = (SPH_LDS unsigned char*)smem_raw;
    // buffer b: K at b*2*TILE_BYTES, V at b*2*TILE_BYTES + TILE_BYTES

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;

    const int lid = xcd_contiguous_id(blockIdx.x, n_wg);
    const int bh = lid / n_qtiles, qt = lid % n_qtiles;
    const size_t head_off = (size_t)bh * N * D;
    const __bf16* Qh = Q + head_off;
    const __bf16* Kh = K + head_off;
    const __bf16* Vh = V + head_off;
    __bf16* Oh = O + head_off;
    const int q0 = qt * BR + wave * 32 * QB;

    // ---- Q fragments: B operands of S^T = K Q^T, held for the whole kernel
    bf16x8 qf[QB][KSTEPS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int row = q0 + qb * 32 + l32;
        row = row < N ? row : N - 1;               // rows past the end are computed and dropped
        const __bf16* src = Qh + (size_t)row * D + 8 * h;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
            qf[qb][kk] = *reinterpret_cast<const bf16x8*>(src + kk * 16);
    }

    f32x16 oacc[DB][QB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][qb][r] = 0.f;
    float zacc[QB];      // spherical: sum of squares; softmax: running denominator
    float mrun[QB];      // softmax only: running maximum (in scaled log2 units)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { zacc[qb] = 0.f; mrun[qb] = -INFINITY; }

    // ---- global -> register -> LDS staging of one K tile and one V tile
    i32x4 kreg[LD_PER_THREAD], vreg[LD_PER_THREAD];
    auto load_tile = [&](int j0) {
#pragma unroll
        for (int i = 0; i < LD_PER_THREAD; ++i) {
            int id = tid + i * kThreads;
            int r = id / CH, c = id % CH;
            int key = j0 + r;
            if (key < N) {
                size_t off = (size_t)key * D + c * 8;
                kreg[i] = *reinterpret_cast<const i32x4*>(Kh + off);
                vreg[i] = *reinterpret_cast<const i32x4*>(Vh + off);
            } else {                               // zero keys add nothing to o or z
                kreg[i] = i32x4{0, 0, 0, 0};
                vreg[i] = i32x4{0, 0, 0, 0};
            }
        }
    };
    auto store_tile = [&](int buf) {
        SPH_LDS unsigned char* kb = smem + buf * 2 * TILE_BYTES;
        SPH_LDS unsigned char* vb = kb + TILE_BYTES;
#pragma unroll
        for (int i = 0; i < LD_PER_THREAD; ++i) {
            int id = tid + i * kThreads;
            int r = id / CH, c = id % CH;
            *reinterpret_cast<SPH_LDS i32x4*>(kb + r * (D * 2) + 16 * kswz<CH>(r, c)) = kreg[i];
            *reinterpret_cast<SPH_LDS i32x4*>(vb + r * (D * 2) + 16 * vswz<CH>(r, c)) = vreg[i];
        }
    };

    const int n_tiles = (N + BC - 1) / BC;
    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int jt = 0; jt < n_tiles; ++jt) {
        const int buf = jt & 1;
        const bool more = jt + 1 < n_tiles;
        if (more) load_tile((jt + 1) * BC);

        const SPH_LDS unsigned char* kb = smem + buf * 2 * TILE_BYTES;
        const SPH_LDS unsigned char* vb = kb + TILE_BYTES;

#pragma unroll
        for (int sub = 0; sub < BC / 32; ++sub) {
            // ---- S^T (32 keys x 32*QB queries) = K_sub Q^T
            f32x16 s[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[qb][r] = 0.f;
            const int krow = sub * 32 + l32;
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) {
                bf16x8 kf = lds_read_b128(kb + krow * (D * 2) + 16 * kswz<CH>(krow, 2 * kk + h));
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    s[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][kk], s[qb], 0, 0, 0);
            }

            // ---- normaliser on the accumulator registers, then round to bf16 in place
            bf16x8 p[QB][2];
            if (NORM == Norm::Spherical) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    float z0 = 0.f, z1 = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        z0 = __builtin_fmaf(s[qb][r], s[qb][r], z0);
                        z1 = __builtin_fmaf(s[qb][r + 1], s[qb][r + 1], z1);
                    }
                    zacc[qb] += z0 + z1;
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int e = 0; e < 8; e += 2) {
                            bf16x2 c2 = cvt2(s[qb][8 * ks + e], s[qb][8 * ks + e + 1]);
                            p[qb][ks][e] = c2[0];
                            p[qb][ks][e + 1] = c2[1];
                        }
                }
            } else {
                // SoftMax twin: running maximum, exponentials, rescale of o.
                const int key_base = jt * BC + sub * 32 + 4 * h;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    float mx = -INFINITY;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int key = key_base + 8 * (r >> 2) + (r & 3);
                        float v = s[qb][r] * softmax_scale_log2;
                        v = key < N ? v : -INFINITY;
                        s[qb][r] = v;
                        mx = fmaxf(mx, v);
                    }
                    mx = fmaxf(mx, __shfl_xor(mx, 32));
                    float mnew = fmaxf(mrun[qb], mx);
                    float alpha = __builtin_amdgcn_exp2f(mrun[qb] - mnew);
                    mrun[qb] = mnew;
                    float lsum = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        s[qb][r] = __builtin_amdgcn_exp2f(s[qb][r] - mnew);
                        lsum += s[qb][r];
                    }
                    zacc[qb] = zacc[qb] * alpha + lsum;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[db][qb][r] *= alpha;
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int e = 0; e < 8; e += 2) {
                            bf16x2 c2 = cvt2(s[qb][8 * ks + e], s[qb][8 * ks + e + 1]);
                            p[qb][ks][e] = c2[0];
                            p[qb][ks][e + 1] = c2[1];
                        }
                }
            }

            // ---- O^T (D x 32*QB queries) += V_sub^T P^T
            // k-slot (h, e) of k-step ks is key 16ks + 8(e>>2) + 4h + (e&3): two transposing
            // reads of 4 keys each.  Within a 16-lane block, lane i supplies the 8-byte piece
            // row (i>>2), columns 4(i&3)..+3 and receives column i of all 4 rows.
            const int i16 = lane & 15, blk = (lane >> 4) & 1;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const int colb = (db * 32 + 16 * blk + 4 * (i16 & 3)) * 2;   // byte column
                    const int r0 = sub * 32 + 16 * ks + 4 * h + (i16 >> 2);
                    const int r1 = r0 + 8;
                    bf16x4 lo = lds_read_tr64(vb + r0 * (D * 2) + 16 * vswz<CH>(r0, colb >> 4) + (colb & 15));
                    bf16x4 hi = lds_read_tr64(vb + r1 * (D * 2) + 16 * vswz<CH>(r1, colb >> 4) + (colb & 15));
                    bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        oacc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p[qb][ks], oacc[db][qb], 0, 0, 0);
                }
            }
        }

        if (more) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- tail: combine the two partial z of each query, O = o / b(z), store
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        float z = zacc[qb] + __shfl_xor(zacc[qb], 32);
        float inv;
        if (NORM == Norm::Spherical)
            inv = z > 0.f ? 1.0f / __builtin_sqrtf(z) : 0.f;
        else
            inv = 1.0f / z;
        const int row = q0 + qb * 32 + l32;
        if (row < N) {
            __bf16* dst = Oh + (size_t)row * D + 4 * h;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x2 a = cvt2(oacc[db][qb][4 * g] * inv, oacc[db][qb][4 * g + 1] * inv);
                    bf16x2 b = cvt2(oacc[db][qb][4 * g + 2] * inv, oacc[db][qb][4 * g + 3] * inv);
                    bf16x4 o4 = {a[0], a[1], b[0], b[1]};
                    *reinterpret_cast<bf16x4*>(dst + db * 32 + 8 * g) = o4;
                }
        }
    }
}


// ---------------------------------------------------------------------------
// Software-pipelined bf16 kernel (spherical normaliser only).
//
// The key axis advances in sub-steps of 32 keys.  Three stages of three
// consecutive sub-steps are in flight at once in every wavefront, so that the
// matrix pipe, the vector ALU and the LDS all stay busy with one wave per SIMD:
//     A(t+1)  S^T = K Q^T            matrix cores -> score registers (next)
//     B(t)    z += s^2, P = bf16(s)  plain fp32 VALU on score registers (current)
//     C(t-1)  O^T += V^T P^T         matrix cores <- P registers (previous)
// A sub-step is cut into SLOTS slots (one K fragment + one V^T fragment each);
// LDS fragment reads run PD slots ahead of their use, across sub-step and tile
// boundaries.  K/V tiles of BC = 64 keys rotate through four LDS buffers: in
// iteration j tile j and j+1 feed stage A, tiles j-1 and j feed stage C, and
// tile j+2 is written, with one workgroup barrier per tile.  Global loads go
// through buffer descriptors whose range check returns zeros past the end of the
// head: a zero key contributes nothing to o or z, so ragged N needs no masking.
// ---------------------------------------------------------------------------
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

template <int D, int QB>
__global__ __launch_bounds__(kThreads, 1)
void fwd_bf16_pipelined_kernel(const __bf16* __restrict__ Q, const __bf16* __restrict__ K,
                               const __bf16* __restrict__ V, __bf16* __restrict__ O,
                               int N, int n_qtiles, int n_wg)
{
    constexpr int BC = 64;
    constexpr int BR = kWaves * 32 * QB;
    constexpr int ROWB = D * 2;                    // bytes per tile row
    constexpr int CH = ROWB / 16;
    constexpr int TILE_BYTES = BC * ROWB;          // one K or V tile
    constexpr int BUF_BYTES = 2 * TILE_BYTES;      // K tile then V tile
    constexpr int NBUF = 4;
    constexpr int CHUNKS = BC * CH;
    constexpr int LD = CHUNKS / kThreads;          // 16-byte loads per thread per tensor per tile
    constexpr int KSTEPS = D / 16;
    constexpr int DB = D / 32;
    constexpr int SLOTS = KSTEPS;                  // slots per sub-step
    constexpr int PD = 2;                          // LDS prefetch distance in slots
    constexpr int RING = 4;                        // fragment registers in rotation
    constexpr int VALU_PER_MFMA = 3;
    static_assert(CH == 16 || CH == 8, "head dimension 128 or 64");
    static_assert(2 * DB == SLOTS, "one V^T fragment per slot");
    static_assert(2 * LD == SLOTS, "one staged chunk per slot of the second half");
    static_assert((2 * SLOTS) % RING == 0 && PD < RING, "ring indices must repeat every iteration");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    SPH_LDS unsigned char* smem = (SPH_LDS unsigned char*)smem_raw;
#ifdef SPHATTN_CLOCK_PROBE
    const long long probe_t0 = clock64(), probe_w0 = wall_clock64();
#endif

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int i16 = lane & 15, blk = (lane >> 4) & 1;

    const int lid = xcd_contiguous_id(blockIdx.x, n_wg);
    const int bh = lid / n_qtiles, qt = lid % n_qtiles;
    const size_t head_off = (size_t)bh * N * D;
    const __bf16* Qh = Q + head_off;
    __bf16* Oh = O + head_off;
    const uint32_t head_bytes = (uint32_t)N * ROWB;
    const __amdgpu_buffer_rsrc_t krs = make_rsrc(K + head_off, head_bytes);
    const __amdgpu_buffer_rsrc_t vrs = make_rsrc(V + head_off, head_bytes);
    const int q0 = qt * BR + wave * 32 * QB;

    // ---- per-lane LDS byte offsets inside a tile
    // K fragment (sub, kk): row sub*32 + l32, chunk (2kk+h) ^ swizzle(row)
    int koff[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk)
        koff[kk] = l32 * ROWB + 16 * kswz<CH>(l32, 2 * kk + h);
    // V^T fragment (sub, ks, db): rows sub*32 + 16ks + 4h + (i16>>2) [+8], 8 bytes at column
    // db*32 + 16*blk + 4*(i16&3)
    int voff[DB];
    {
        const int r = 4 * h + (i16 >> 2);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int colb = (db * 32 + 16 * blk + 4 * (i16 & 3)) * 2;
            voff[db] = r * ROWB + 16 * vswz<CH>(r, colb >> 4) + (colb & 15);
        }
    }
    // staging: chunk id = tid + i*256 -> row id/CH, chunk id%CH; chunks 0..LD-1 are K, LD..2LD-1 V
    int st_off[2 * LD], ld_off[LD];
#pragma unroll
    for (int i = 0; i < LD; ++i) {
        const int id = tid + i * kThreads;
        const int r = id / CH, c = id % CH;
        st_off[i] = r * ROWB + 16 * kswz<CH>(r, c);
        st_off[LD + i] = TILE_BYTES + r * ROWB + 16 * vswz<CH>(r, c);
        ld_off[i] = r * ROWB + c * 16;
    }

    // ---- Q fragments (B operands of S^T = K Q^T)
    bf16x8 qf[QB][KSTEPS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int row = q0 + qb * 32 + l32;
        row = row < N ? row : N - 1;
        const __bf16* src = Qh + (size_t)row * D + 8 * h;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
            qf[qb][kk] = *reinterpret_cast<const bf16x8*>(src + kk * 16);
    }

    f32x16 oacc[DB][QB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][qb][r] = 0.f;
    float zacc[QB][2];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) zacc[qb][0] = zacc[qb][1] = 0.f;

    i32x4 stage[2 * LD];
    auto gload_chunk = [&](int c, int tile) {
        const uint32_t off = (uint32_t)tile * TILE_BYTES + ld_off[c % LD];
        stage[c] = __builtin_amdgcn_raw_buffer_load_b128(c < LD ? krs : vrs, off, 0, 0);
    };
    auto lstore_chunk = [&](int c, SPH_LDS unsigned char* buf) {
        *reinterpret_cast<SPH_LDS i32x4*>(buf + st_off[c]) = stage[c];
    };

    const int n_tiles = (N + BC - 1) / BC;

    // ---- prologue: buffer 3 plays "tile -1" (zeros) for the first stage C; tiles 0 and 1 go
    // to buffers 0 and 1; tile 2 waits in registers
    {
        const i32x4 zero4 = {0, 0, 0, 0};
        for (int i = tid; i < BUF_BYTES / 16; i += kThreads)
            *reinterpret_cast<SPH_LDS i32x4*>(smem + 3 * BUF_BYTES + i * 16) = zero4;
    }
#pragma unroll
    for (int c = 0; c < 2 * LD; ++c) gload_chunk(c, 0);
#pragma unroll
    for (int c = 0; c < 2 * LD; ++c) lstore_chunk(c, smem);
#pragma unroll
    for (int c = 0; c < 2 * LD; ++c) gload_chunk(c, 1);
#pragma unroll
    for (int c = 0; c < 2 * LD; ++c) lstore_chunk(c, smem + BUF_BYTES);
#pragma unroll
    for (int c = 0; c < 2 * LD; ++c) gload_chunk(c, 2);
    __syncthreads();

    f32x16 S0[QB], S1[QB];
    bf16x8 P0[QB][2], P1[QB][2];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) { S0[qb][r] = 0.f; S1[qb][r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) { P0[qb][ks][e] = (__bf16)0.f; P1[qb][ks][e] = (__bf16)0.f; }
    }
    // S0 = scores of sub-step 0
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
        bf16x8 kfr = lds_read_b128(smem + koff[kk]);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
            S0[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr, qf[qb][kk], S0[qb], 0, 0, 0);
    }

    bf16x8 kf[RING], vf[RING];
    // Fragment reads for slot u of an iteration whose tiles j-1, j, j+1 sit at bprv, bcur, bnxt:
    //   u in [0,SLOTS)        first half : K_j sub 1,     V_{j-1} sub 1
    //   u in [SLOTS,2SLOTS)   second half: K_{j+1} sub 0, V_j sub 0
    //   u >= 2SLOTS           next iteration's first half: K_{j+1} sub 1, V_j sub 1
    auto issue_reads = [&](int u, const SPH_LDS unsigned char* bprv, const SPH_LDS unsigned char* bcur,
                           const SPH_LDS unsigned char* bnxt) {
        const int hh = u / SLOTS, i = u % SLOTS;
        const SPH_LDS unsigned char* kp = hh == 0 ? bcur + 32 * ROWB : hh == 1 ? bnxt : bnxt + 32 * ROWB;
        const SPH_LDS unsigned char* vp = (hh == 0 ? bprv + 32 * ROWB : hh == 1 ? bcur : bcur + 32 * ROWB) + TILE_BYTES;
        kf[u % RING] = lds_read_b128(kp + koff[i]);
        const int ks = i / DB, db = i % DB;
        const SPH_LDS unsigned char* a = vp + (16 * ks) * ROWB + voff[db];
        bf16x4 lo = lds_read_tr64(a);
        bf16x4 hi = lds_read_tr64(a + 8 * ROWB);
        vf[u % RING] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // buffers of tiles j-1, j, j+1, j+2
    SPH_LDS unsigned char* bprv = smem + 3 * BUF_BYTES;
    SPH_LDS unsigned char* bcur = smem;
    SPH_LDS unsigned char* bnxt = smem + BUF_BYTES;
    SPH_LDS unsigned char* bnn = smem + 2 * BUF_BYTES;
#pragma unroll
    for (int u = 0; u < PD; ++u) issue_reads(u, bprv, bcur, bnxt);

    for (int j = 0; j < n_tiles; ++j) {
#pragma unroll
        for (int s = 0; s < 2 * SLOTS; ++s) {
            const int hf = s / SLOTS, i = s % SLOTS;
            f32x16 (&Sn)[QB] = hf == 0 ? S1 : S0;
            f32x16 (&Sc)[QB] = hf == 0 ? S0 : S1;
            bf16x8 (&Pc)[QB][2] = hf == 0 ? P0 : P1;
            bf16x8 (&Pp)[QB][2] = hf == 0 ? P1 : P0;
            __builtin_amdgcn_sched_barrier(0);
            // The one barrier per tile: everything written to LDS in the previous iteration
            // (tile j+1) becomes visible before its first read, which is the prefetch below;
            // and every wave has finished the previous iteration, whose first half was the
            // last reader of the buffer that this iteration's second half overwrites.
            if (s == SLOTS - PD) {
                // LDS operations complete in issue order.  At most OUT of them have been issued
                // since this wave's last staging write of the previous iteration, so once no
                // more than OUT are outstanding that write has landed.  No full drain: the
                // fragment reads already in flight keep flying across the barrier.
                constexpr int OUT = 3 * (SLOTS - PD) < 15 ? 3 * (SLOTS - PD) : 15;
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0xC07F | (OUT << 8));
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
            issue_reads(s + PD, bprv, bcur, bnxt);
            // A: k-step i of the next sub-step's scores
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                if (i == 0) {
                    f32x16 zero = {0};
                    Sn[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s % RING], qf[qb][i], zero, 0, 0, 0);
                } else {
                    Sn[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s % RING], qf[qb][i], Sn[qb], 0, 0, 0);
                }
            }
            // C: V^T fragment i against the previous sub-step's P
            {
                const int ks = i / DB, db = i % DB;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    oacc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[s % RING], Pp[qb][ks], oacc[db][qb], 0, 0, 0);
            }
            // B: a slice of the current sub-step's scores, 16*QB/SLOTS registers per slot
            constexpr int PER = 16 * QB / SLOTS;
#pragma unroll
            for (int u = 0; u < PER; u += 2) {
                const int idx = i * PER + u;
                const int qb = idx / 16, r = idx % 16;
                const float a = Sc[qb][r], b = Sc[qb][r + 1];
                zacc[qb][0] = __builtin_fmaf(a, a, zacc[qb][0]);
                zacc[qb][1] = __builtin_fmaf(b, b, zacc[qb][1]);
                bf16x2 c2 = cvt2(a, b);
                Pc[qb][r / 8][r % 8] = c2[0];
                Pc[qb][r / 8][r % 8 + 1] = c2[1];
            }
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)     // keep the running sums where they were computed
                asm volatile("" : "+v"(zacc[qb][0]), "+v"(zacc[qb][1]));
            // staging, second half only: tile j+2 into LDS, tile j+3 out of HBM/L2
            if (hf == 1) {
                lstore_chunk(i, bnn);
                gload_chunk(i, j + 3);
            }
            // issue order inside the slot: after each matrix instruction, one LDS read and a
            // few VALU instructions, so that the matrix pipe never waits on the issue port
#pragma unroll
            for (int m = 0; m < 2 * QB; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read
                __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER_MFMA, 0);   // VALU
                if (hf == 1 && m == 2) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   // DS write
                if (hf == 1 && m == 3) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // VMEM read
            }
        }
        SPH_LDS unsigned char* t = bprv; bprv = bcur; bcur = bnxt; bnxt = bnn; bnn = t;
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- drain: stage C of the last sub-step (V of the last tile, sub 1, now at bprv)
    {
        const SPH_LDS unsigned char* vp = bprv + TILE_BYTES + 32 * ROWB;
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) {
            const int ks = i / DB, db = i % DB;
            const SPH_LDS unsigned char* a = vp + (16 * ks) * ROWB + voff[db];
            bf16x4 lo = lds_read_tr64(a);
            bf16x4 hi = lds_read_tr64(a + 8 * ROWB);
            bf16x8 vfr = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
                oacc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr, P1[qb][ks], oacc[db][qb], 0, 0, 0);
        }
    }

#ifdef SPHATTN_CLOCK_PROBE
    if (tid == 0 && blockIdx.x == 0 && bh == 0)
        printf("clock probe: %lld shader clocks, %lld x10ns, %d tiles\n", clock64() - probe_t0,
               wall_clock64() - probe_w0, n_tiles);
#endif
    // ---- tail: O = o / sqrt(z)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float zl = zacc[qb][0] + zacc[qb][1];
        const float z = zl + __shfl_xor(zl, 32);
        const float inv = z > 0.f ? 1.0f / __builtin_sqrtf(z) : 0.f;
        const int row = q0 + qb * 32 + l32;
        if (row < N) {
            __bf16* dst = Oh + (size_t)row * D + 4 * h;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x2 a = cvt2(oacc[db][qb][4 * g] * inv, oacc[db][qb][4 * g + 1] * inv);
                    bf16x2 b = cvt2(oacc[db][qb][4 * g + 2] * inv, oacc[db][qb][4 * g + 3] * inv);
                    bf16x4 o4 = {a[0], a[1], b[0], b[1]};
                    *reinterpret_cast<bf16x4*>(dst + db * 32 + 8 * g) = o4;
                }
        }
    }
}

}  // namespace sphattn
