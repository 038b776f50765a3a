// All-E4M3 forward: Q, K, V stored in OCP E4M3, BOTH contractions on the fp8 matrix
// instruction v_mfma_f32_16x16x128_f8f6f4 (k = 128), output in bf16, d = 128 or 64.
//
// The paper argues (Section 1; Section 3.1) that without the row-wise exponential the whole
// of attention can run at the matrix cores' low-precision rate.  This kernel is that case
// taken to its end: the scores, too, go back into the matrix cores as E4M3.
//
// What makes that possible for the spherical normaliser and not for SoftMax:
//   * O_i = o_i / sqrt(z_i) does not change when every score of row i is multiplied by the
//     same positive factor.  So the scores of a row can be brought into the E4M3 range by a
//     per-row factor, and nothing has to be undone afterwards: o and z are both accumulated
//     from the scaled scores and the tail is the plain one.
//   * By Cauchy-Schwarz |s_ij| <= |q_i| max_j |k_j| =: bound_i.  The factor is the power of two
//     2^-e_i with bound_i / 440 = m 2^e_i, m in [0.5, 1): every scaled score is inside +-440
//     (the E4M3 maximum is 448, and the conversion overflows to NaN rather than saturating;
//     the margin covers the fp32 rounding of the score itself), and the largest possible one
//     is above 220.  |q_i| comes from the Q fragment in registers, max_j |k_j| of the head
//     from the preparation pass.  The division by 2^e_i is part of the convert instruction
//     (v_cvt_scalef32_pk_fp8_f32), which rounds to nearest even.
//   * z_i = sum_j p_ij^2 is taken from the ROUNDED scores p_ij, on the matrix cores as well:
//     it is the diagonal of P^T P, and P's register image serves as A and as B operand alike.
//     One extra matrix instruction per query block and tile replaces 128 VALU FMAs, which
//     a single wave per SIMD cannot issue in the shadow of the matrix instructions.
//
// Matrix-core mapping.  With k = 128 both contractions have the same shape,
//     S^T block kb (16 keys x 16 queries) = K frag (A: 16 keys x 128 of d) * Q frag (B: 128 x 16 queries)
//     O^T block db (16 cols of d x 16 queries) += V^T frag (A: 16 cols x 128 keys) * P (B: 128 keys x 16)
// and lane (n16, g) of an A or B operand holds 32 of the 128 k-slots of row or column n16.
// Which 32 is free as long as A and B agree; here group g takes bytes 16g .. 16g+15 and
// 64+16g .. 64+16g+15 of the 128-byte row (every LDS read then takes one 16-byte piece from
// each row of a 1 KB block; with the pieces of a row permuted as block_piece_offset says, the
// banks serve it at full rate).  In the accumulator lane
// (n16, g) holds query n16 and, in register t, row 4g + t of the block.  The 16 rows of score
// block kb are therefore chosen to be the keys
//     key(kb, p) = 64 (kb / 4) + 16 (p / 4) + 4 (kb % 4) + (p % 4),    p = 0..15,
// of the 128-key tile: then register t of block kb in lane group g is key
// 64 (kb/4) + 16g + 4 (kb%4) + t, and the eight blocks' scores, packed four to a register, are
// exactly the k-slots that the second contraction wants from this lane.  Like the 16-bit kernels, the
// scores never leave their registers.  V is needed as V^T with keys along the contiguous axis;
// the preparation pass writes that copy once (2 N d bytes of traffic per head against
// 4 N^2 d flop), so both operand streams are read from LDS with plain 16-byte reads and there
// is no transposing read at all.
//
// d = 64 uses the same instruction with the upper half of the first contraction's k-slots
// zero on both sides (the key and query rows are 64 bytes; there is no fp8 matrix instruction
// with k = 64 in this shape), and has four V^T fragments per tile instead of eight: 52 matrix
// instructions per tile and wave for the work of 32 + 4.
//
// Gene multiplicities (paper, Section 3.1): MULT multiplies the fp32 score of key j by mult[b, j]
// before it is scaled and rounded; the row bound then uses max_j mult_j |k_j| (the preparation
// pass folds the multiplicity into the key norms).  The multipliers travel with their tile
// (512 bytes per 128 keys, copied into LDS behind K and V^T) and reach the lanes through one
// 16-byte LDS read per slot, a slot ahead of their use.
//
// Pipeline.  A slot = one score block row kb of the current tile (4 matrix instructions, one
// per query block) + one V^T fragment db of the previous tile (4 more) + the conversion of the
// block row finished in the slot before (one convert instruction and at most one LDS read
// behind every matrix instruction, in a fixed order).  P is complete one slot into the next tile,
// so the second contraction of tile T runs in slots 1..7 of tile T+1 and slot 0 of tile T+2.
// Tiles of 128 keys rotate through four 32 KB LDS buffers, filled straight from HBM/L2
// (buffer_load ... lds), with one workgroup barrier per tile.
#pragma once
#include "sphattn_pipelined.hpp"

namespace sphattn {

constexpr int kFp8Tile = 128;          // keys per tile (one k of the second contraction)

// ---- preparation: V^T copy and the largest key norm per K/V head -------------------------
//
// grid = (heads) x (tiles of 128 keys).  VT[head][c][Np] (E4M3, Np = tiles * 128, zero past
// N) receives V transposed; kmax[head] receives max_j |k_j| through an integer atomic max on
// the bits of the non-negative float (kmax must be zero before the launch).  With multiplicities
// (mult [B, N], heads_per_batch K/V heads per batch entry) the norm of key j counts mult_j times.
template <int D>
__global__ __launch_bounds__(256)
void fp8_prepare_kernel(const unsigned char* __restrict__ K, const unsigned char* __restrict__ V,
                        const float* __restrict__ mult, unsigned char* __restrict__ VT,
                        float* __restrict__ kmax, int N, int n_tiles, int heads_per_batch)
{
    // rows of D + 4 bytes: the 16 rows that one output piece gathers from then start in different
    // banks (with a 16-byte-aligned stride they would all start in the same bank)
    constexpr int T = kFp8Tile, LROW = D + 4;
    __shared__ __attribute__((aligned(16))) unsigned char tile[T * LROW];
    __shared__ float wmax[4];
    const int tid = threadIdx.x;
    const int head = blockIdx.x / n_tiles, kt = blockIdx.x % n_tiles;
    const int key0 = kt * T;
    const size_t Np = (size_t)n_tiles * T;
    const unsigned char* Vh = V + (size_t)head * N * D;
    const unsigned char* Kh = K + (size_t)head * N * D;

    for (int id = tid; id < T * (D / 16); id += 256) {
        const int row = id / (D / 16), c16 = id % (D / 16);
        i32x4 v = {0, 0, 0, 0};
        if (key0 + row < N) v = *reinterpret_cast<const i32x4*>(Vh + (size_t)(key0 + row) * D + 16 * c16);
#pragma unroll
        for (int r = 0; r < 4; ++r) *reinterpret_cast<int*>(tile + row * LROW + 16 * c16 + 4 * r) = v[r];
    }
    // |k_j|^2 of row tid/2, half tid%2 of the row
    float ss = 0.f;
    {
        const int row = tid >> 1, half = tid & 1;
        if (key0 + row < N) {
            const unsigned char* src = Kh + (size_t)(key0 + row) * D + (D / 2) * half;
#pragma unroll
            for (int c = 0; c < D / 32; ++c) {
                const i32x4 w = *reinterpret_cast<const i32x4*>(src + 16 * c);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float a = __builtin_amdgcn_cvt_f32_fp8(w[r], 0), b = __builtin_amdgcn_cvt_f32_fp8(w[r], 1);
                    const float c2 = __builtin_amdgcn_cvt_f32_fp8(w[r], 2), e = __builtin_amdgcn_cvt_f32_fp8(w[r], 3);
                    ss += a * a + b * b + c2 * c2 + e * e;
                }
            }
        }
        ss += __shfl_xor(ss, 1);
        if (mult != nullptr && key0 + row < N) {
            const float m = mult[(size_t)(head / heads_per_batch) * N + key0 + row];
            ss *= m * m;
        }
#pragma unroll
        for (int m = 2; m < 64; m <<= 1) ss = fmaxf(ss, __shfl_xor(ss, m));
        if ((tid & 63) == 0) wmax[tid >> 6] = ss;
    }
    __syncthreads();
    if (tid == 0) {
        const float m = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
        atomicMax(reinterpret_cast<int*>(kmax + head), __float_as_int(__builtin_sqrtf(m)));
    }
    // 16-byte pieces of V^T: column c of d, keys key0 + 16q .. +15
    unsigned char* VTh = VT + (size_t)head * D * Np;
    for (int id = tid; id < D * (T / 16); id += 256) {
        const int c = id / (T / 16), q = id % (T / 16);
        i32x4 out;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            unsigned w = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) w |= (unsigned)tile[(16 * q + 4 * r + e) * LROW + c] << (8 * e);
            out[r] = (int)w;
        }
        *reinterpret_cast<i32x4*>(VTh + (size_t)c * Np + key0 + 16 * q) = out;
    }
}

__global__ void fp8_clear_kernel(float* __restrict__ p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

// ---- the forward kernel ------------------------------------------------------------------
//
// One workgroup = 4 wavefronts = 256 query rows of one (b, h); a wavefront owns NQ = 4 blocks
// of 16 rows.  VT and kmax come from fp8_prepare_kernel (same stream, earlier).
//
// SOFTMAX: the comparison twin.  O = softmax(Q K^T / sqrt(d)) V on the same skeleton, made as
// cheap as a SoftMax can be here: the shift of row i is not a running maximum but the bound
// |q_i| max_j |k_j| / sqrt(d) >= max_j s_ij / sqrt(d) (any shift that is not below the maximum
// gives the same result), so there is no cross-lane maximum and no rescaling of the
// accumulators; what remains per score is one scale-and-shift and one exponential in front of
// the convert.  The weights p = exp(...) <= 1 enter the second contraction as 256 p in E4M3;
// the row sums come from the matrix cores as well (an all-ones A fragment against P).  A row
// whose largest score is more than about 12 sqrt(d) below its bound underflows to zero weights
// and gives 0: a twin for timing on inputs of moderate size, not a general SoftMax.
// d = 64: two workgroups per CU (64 KB of LDS each) where the registers allow it without
// spilling much (not with multiplicities: 624 bytes of scratch per lane)
template <int D, bool SOFTMAX, bool MULT>
__global__ __launch_bounds__(kThreads, (D == 64 && !MULT) ? 2 : 1)
void fwd_fp8_kernel(const unsigned char* __restrict__ Q, const unsigned char* __restrict__ K,
                    const unsigned char* __restrict__ VT, const float* __restrict__ kmax,
                    const float* __restrict__ mult,
                    unsigned short* __restrict__ O, int N, int H, int kv_group, int n_tiles, int n_qtiles, int n_wg,
                    int stream_period)
{
    constexpr int BC = kFp8Tile, NQ = 4;
    constexpr int BR = kWaves * 16 * NQ;
    constexpr int KH = D / 64;                     // 1 KB blocks per K block row (64-byte halves of the key rows)
    constexpr int DB = D / 16;                     // V^T fragments per tile = 16-column blocks of O
    constexpr int KTILE = BC * D;                  // K tile; the V^T tile (D rows of 128 keys) has the same size
    constexpr int MLDS = 2 * KTILE;                // the tile's 128 multiplicities (MULT only)
    constexpr int BUF_BYTES = 2 * KTILE + (MULT ? BC * 4 : 0);
    constexpr int NBUF = 4;
    constexpr int SLOTS = 8;                       // per tile: score block rows kb (and, d = 128, V^T fragments db)
    constexpr int PD = 2;                          // LDS prefetch distance in slots (measured best of 1, 2, 3)
    constexpr int RING = 4;
    constexpr int KCOPY = 2 * KH;                  // 1 KB copies per wave per tile: of K ...
    constexpr int VPW = DB / 4;                    // ... V^T fragments per wave, two copies each
    constexpr int NCOPY = KCOPY + 2 * VPW;         // 8 (d = 128) or 4 (d = 64)
    constexpr int NCOPY_ALL = NCOPY + (MULT ? 1 : 0);   // and one 512-byte copy (wave 0) of multiplicities
    static_assert(D == 64 || D == 128, "head dimension 128 or 64");
    static_assert((2 * SLOTS) % RING == 0 && PD < RING, "ring indices must repeat");
    static_assert(!(SOFTMAX && MULT), "multiplicities belong to the spherical variant");
    static_assert(2 * PD <= NCOPY, "the prologue issues whole copies of tile 1");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    SPH_LDS unsigned char* smem = (SPH_LDS unsigned char*)smem_raw;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, g = lane >> 4;

    const int lid = xcd_contiguous_id(blockIdx.x, n_wg);
    const int qt = lid % n_qtiles, bh = lid / n_qtiles;
    // kv_group query heads share one K/V head (and its V^T copy and key-norm maximum); the heads
    // of a group are adjacent in the workgroup order, so they meet in one L2
    const int kvh = (bh / H) * (H / kv_group) + (bh % H) / kv_group;
    const size_t Np = (size_t)n_tiles * BC;
    const unsigned char* Qh = Q + (size_t)bh * N * D;
    const int q0 = qt * BR + wave * 16 * NQ;

    // LDS image of a tile: K blocks (kb, h) and V^T blocks (db, h), 16 rows x 64 bytes each
    // (half h of 128-byte rows; 64-byte key rows have h = 0 only), row-major, 1 KB; K block (kb, h)
    // at (KH kb + h) KB, V^T block (db, h) behind the K tile at (2 db + h) KB.  The 32 k-slots of
    // lane group g are the bytes 16g .. 16g+15 of both halves of the row (see the key order
    // above), so each of a fragment's 16-byte reads takes one piece from every row of one block:
    // the 64 lanes cover the block's 1 KB exactly once (piece c of row r sits in slot
    // c ^ ((r >> 1) & 3), which keeps the lanes that the LDS serves together on different banks).
    const int flane = block_piece_offset(n16, g);
    constexpr int HALF1 = 1024;                    // second half of the rows: the next block
    // copies: lane l fills row l/4, slot l%4 of a block, with piece p = block_piece_in_slot(l)
    //   K   block (kb, h): tile row key(kb, l/4), bytes 64 h + 16 p of the key row;
    //                      wave w copies the block rows kb = 2w, 2w+1
    //   V^T block (db, h): row 16db + l/4 of V^T, keys 64 h + 16 p of the tile;
    //                      wave w copies the fragments db = VPW w .. VPW w + VPW - 1
    const int p = lane >> 2;
    const int kld_lane = (16 * (p >> 2) + (p & 3) + 64 * (wave >> 1) + 8 * (wave & 1)) * D + block_piece_in_slot(lane) * 16;
    const int vld_lane = (int)((16 * VPW * wave + p) * Np) + block_piece_in_slot(lane) * 16;

    // ---- Q fragments and the row factors a_i.  Q is read once and O written once by this
    // workgroup only: non-temporal, so that the L2 keeps the K/V stream instead.
    typedef __attribute__((ext_vector_type(8))) int frag_t;
    frag_t qf[NQ];
    float qdiv[NQ];                                // 2^e_i: the scores of row i are divided by it on conversion
    float qshift[NQ];
    constexpr float kSoftmaxScaleLog2 = 1.4426950408889634f * (D == 128 ? 0.08838834764831845f : 0.125f);   // log2(e) / sqrt(d)
    const float km = kmax[kvh];
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
        int row = q0 + qb * 16 + n16;
        row = row < N ? row : N - 1;               // rows past the end are computed and dropped
        const unsigned char* src = Qh + (size_t)row * D + 16 * g;
        const i32x4 lo = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(src));
        i32x4 hi = {0, 0, 0, 0};                   // d = 64: the upper k-slots stay zero
        if constexpr (KH == 2) hi = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(src + 64));
        qf[qb] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        float qq = 0.f;
#pragma unroll
        for (int r = 0; r < 4 * KH; ++r) {
            const float a = __builtin_amdgcn_cvt_f32_fp8(qf[qb][r], 0), b = __builtin_amdgcn_cvt_f32_fp8(qf[qb][r], 1);
            const float c = __builtin_amdgcn_cvt_f32_fp8(qf[qb][r], 2), e = __builtin_amdgcn_cvt_f32_fp8(qf[qb][r], 3);
            qq += a * a + b * b + c * c + e * e;
        }
        qq = sum_across_groups(qq);
        const float bound = __builtin_sqrtf(qq) * km;   // >= |s_ij| for every key (multiplicity included)
        int e = 0;
        (void)__builtin_frexpf(bound * (1.0f / 440.f), &e);   // bound / 440 = m 2^e, m in [0.5, 1)
        e = bound > 0.f ? min(max(e, -126), 127) : 0;
        qdiv[qb] = SOFTMAX ? 1.0f / 256.f : __builtin_ldexpf(1.0f, e);
        qshift[qb] = bound * kSoftmaxScaleLog2;    // SOFTMAX: exponent of 2 subtracted from every score's
    }

    f32x4 oacc[DB][NQ];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) oacc[db][qb] = f32x4{0.f, 0.f, 0.f, 0.f};

    const i32x4 krw = rsrc_words(K + (size_t)kvh * N * D, (uint32_t)N * D);
    const i32x4 vrw = rsrc_words(VT + (size_t)kvh * D * Np, (uint32_t)(D * Np));
    // multiplicities of this cell's keys; those past the last key arrive as 0 (their keys are zero anyway)
    const i32x4 mrw = rsrc_words(MULT ? mult + (size_t)(bh / H) * N : nullptr, MULT ? (uint32_t)N * 4 : 0);
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    // every other batch of workgroups of an XCD streams the keys backwards (see fwd_pipelined_kernel)
    const bool backwards = stream_period > 0 && (((int)blockIdx.x / kXcds) / stream_period) % 2 == 1;
    auto src_tile = [&](int t) { return t >= n_tiles ? n_tiles : backwards ? n_tiles - 1 - t : t; };
    // copy c of this wave's share of tile t into buffer `buf`: c < KCOPY K, then V^T, then (wave 0)
    // the multiplicities.  K rows past the end of the head are out of the descriptor's range and
    // arrive as zeros.
    auto copy_chunk = [&](int c, int t, SPH_LDS unsigned char* buf) {
        const uint32_t base = (uint32_t)(uintptr_t)buf;
        const int tile = src_tile(t);
        if (c < KCOPY) {
            const int r = c / KH, h = c % KH;      // block row 2 wave + r, half h
            copy_to_lds(krw, base + ((wave_u * 2 + r) * KH + h) * 1024, kld_lane, tile * KTILE + r * 4 * D + h * 64);
        } else if (c < NCOPY) {
            const int f = (c - KCOPY) >> 1, h = (c - KCOPY) & 1;   // fragment VPW wave + f, half h
            copy_to_lds(vrw, base + KTILE + ((wave_u * VPW + f) * 2 + h) * 1024, vld_lane,
                        tile * BC + (int)(f * 16 * Np) + h * 64);
        } else if (MULT && c == NCOPY) {
            // the tile's 128 multiplicities: two 256-byte copies, by every wave (no branch)
            copy_to_lds_b32(mrw, base + MLDS, lane * 4, tile * BC * 4);
            copy_to_lds_b32(mrw, base + MLDS + 256, lane * 4, tile * BC * 4 + 256);
        }
    };

    // ---- prologue: buffer 3 plays the tiles before the first (zeros); tile 0 goes to buffer 0
    // entirely, and of tile 1 the copies that the loop would have issued before its first slot
    {
        const i32x4 zero4 = {0, 0, 0, 0};
        for (int i = tid; i < BUF_BYTES / 16; i += kThreads)
            *reinterpret_cast<SPH_LDS i32x4*>(smem + (NBUF - 1) * BUF_BYTES + i * 16) = zero4;
    }
#pragma unroll
    for (int c = 0; c < NCOPY_ALL; ++c) copy_chunk(c, 0, smem);
#pragma unroll
    for (int c = 0; c < 2 * PD; ++c) copy_chunk(c, 1, smem + BUF_BYTES);
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): this wave's copies have landed
    __syncthreads();

    auto mfma8 = [&](frag_t a, frag_t b, f32x4 c) -> f32x4 {
        return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
    };
    auto read_frag = [&](const SPH_LDS unsigned char* blk) -> frag_t {
        const i32x4 lo = lds_read_b128(blk + flane), hi = lds_read_b128(blk + flane + HALF1);
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // stage B on one block of scores: four of them rounded to E4M3 into one register of P.
    // v_cvt_scalef32_pk_fp8_f32: two values divided by the power of two `div` and rounded to E4M3
    // (nearest even) into one half of a register.  lo starts a register (no initial value
    // needed: hi writes the other half), hi completes it.
    typedef __attribute__((ext_vector_type(2))) short s16x2;
    // `left` = how many of the lane's four keys of this block exist (keys past the end of the
    // head have zero rows, which the spherical weights turn into zeros by themselves; the
    // SoftMax twin has to leave them out explicitly).  m = the keys' multiplicities.
    auto weight = [&](float sc, float m, float shift, bool exists) -> float {
        if constexpr (SOFTMAX) return exists ? __builtin_amdgcn_exp2f(__builtin_fmaf(sc, kSoftmaxScaleLog2, -shift)) : 0.f;
        else if constexpr (MULT) return sc * m;
        else return sc;
    };
    auto stage_b_lo = [&](f32x4 sc, f32x4 m, float div, float shift, int left) -> s16x2 {
        s16x2 w;
        asm volatile("" : "=v"(w));
        return __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(w, weight(sc[0], m[0], shift, left > 0), weight(sc[1], m[1], shift, left > 1), div, false);
    };
    auto stage_b_hi = [&](s16x2 w, f32x4 sc, f32x4 m, float div, float shift, int left) -> int {
        return __builtin_bit_cast(int, __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(w, weight(sc[2], m[2], shift, left > 2), weight(sc[3], m[3], shift, left > 3), div, true));
    };
    // keys of the lane in block row kb of tile t: 128 t + 64 (kb / 4) + 16 g + 4 (kb % 4) + 0..3
    auto keys_left = [&](int t, int kb) -> int {
        if (!SOFTMAX) return 4;
        return t < 0 ? 0 : N - (128 * src_tile(t) + 64 * (kb >> 2) + 16 * g + 4 * (kb & 3));   // t = -1: before the first tile
    };
    // SOFTMAX: row sums of P as all-ones rows times P
    const frag_t ones = {0x38383838, 0x38383838, 0x38383838, 0x38383838, 0x38383838, 0x38383838, 0x38383838, 0x38383838};
    auto row_aggregate = [&](frag_t pq, f32x4 acc) -> f32x4 {
        return SOFTMAX ? mfma8(ones, pq, acc) : mfma8(pq, pq, acc);
    };
    f32x4 zz[NQ];
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) zz[qb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // score block rows: SA is written in even slots and consumed in odd ones, SB the reverse
    f32x4 SA[NQ], SB[NQ];
    frag_t P0[NQ], P1[NQ];                         // P of even and of odd tiles
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
        SA[qb] = SB[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
        P0[qb] = P1[qb] = frag_t{0, 0, 0, 0, 0, 0, 0, 0};
    }
    // multiplicities of the lane's four keys of a block row: read from LDS in the slot that
    // computes the block row's scores, used in the next slot, which converts them (by parity)
    f32x4 mreg[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};

    // Fragment registers, as the two 16-byte halves that the LDS reads deliver (d = 64: the K
    // fragments have no upper half; it stays zero).
    i32x4 kfl[RING], kfh[RING], vfl[RING], vfh[RING];
#pragma unroll
    for (int r = 0; r < RING; ++r) kfh[r] = i32x4{0, 0, 0, 0};
    auto whole = [](i32x4 lo, i32x4 hi) -> frag_t { return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7); };
    // V^T fragment that the slot u (counted from the start of a tile) uses: (u + 7) % 8, if the
    // head dimension has that many
    auto has_v = [&](int u) { return (u + 7) % 8 < DB; };
    // Read `part` (0, 1: K halves; 2, 3: V^T halves) for slot u, counted from the start of a tile
    // T whose neighbours T-2 .. T+1 sit at bpp, bprv, bcur, bnxt:
    //   K   fragment: block row u of tile T          (u >= 8: block row u-8 of tile T+1)
    //   V^T fragment: u = 0: db 7 of tile T-2;  u in 1..7: db u-1 of tile T-1;
    //                 u = 8: db 7 of tile T-1;  u > 8: db u-9 of tile T
    auto read_part = [&](int u, int part, const SPH_LDS unsigned char* bpp, const SPH_LDS unsigned char* bprv,
                         const SPH_LDS unsigned char* bcur, const SPH_LDS unsigned char* bnxt) {
        const SPH_LDS unsigned char* vp = (u == 0 ? bpp : u <= 8 ? bprv : bcur) + KTILE + ((u + 7) % 8) * 2048 + flane;
        const SPH_LDS unsigned char* kp = (u < 8 ? bcur : bnxt) + (u % 8) * KH * 1024 + flane;
        if (part == 0) kfl[u % RING] = lds_read_b128(kp);
        else if (part == 1) { if constexpr (KH == 2) kfh[u % RING] = lds_read_b128(kp + HALF1); }
        else if (!has_v(u)) return;
        else if (part == 2) vfl[u % RING] = lds_read_b128(vp);
        else vfh[u % RING] = lds_read_b128(vp + HALF1);
    };

    SPH_LDS unsigned char* bprv = smem + (NBUF - 1) * BUF_BYTES;
    SPH_LDS unsigned char* bcur = smem;
    SPH_LDS unsigned char* bnxt = smem + BUF_BYTES;
    SPH_LDS unsigned char* bnn = smem + 2 * BUF_BYTES;
#pragma unroll
    for (int u = 0; u < PD; ++u)
#pragma unroll
        for (int part = 0; part < 4; ++part) read_part(u, part, bprv, bprv, bcur, bnxt);

    // tiles are processed in pairs so that the P buffers alternate statically; a tile past the
    // end has zero keys and adds nothing
    const int n_pairs = (n_tiles + 1) / 2;
    for (int jj = 0; jj < n_pairs; ++jj) {
        if constexpr (D == 64 && !MULT) priority_by_tile(jj);   // two workgroups per CU: keep them together
#pragma unroll
        for (int s = 0; s < 2 * SLOTS; ++s) {
            const int par = s / SLOTS, i = s % SLOTS;
            const int tile = 2 * jj + par;
            f32x4 (&Sn)[NQ] = i % 2 == 0 ? SA : SB;
            f32x4 (&Sc)[NQ] = i % 2 == 0 ? SB : SA;
            // stage B of slot 0 finishes the previous tile's P; stage C of slot 0 still uses
            // the P of the tile before that, which lives in this tile's buffer
            frag_t (&Pw)[NQ] = (i == 0) == (par == 0) ? P1 : P0;
            frag_t (&Pr)[NQ] = (i == 0) == (par == 0) ? P0 : P1;
            __builtin_amdgcn_sched_barrier(0);
            // The one barrier per tile: tile T+1 becomes visible before its first read (the
            // prefetch below).  Past it every wave has also finished slot 0 of this tile, the
            // last reader of the buffer that the copies of tile T+2 overwrite.
            if (i == SLOTS - PD) {
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0x0F70);                   // vmcnt(0)
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
            // the multiplicities of block row i of this tile, for the next slot's conversion
            if constexpr (MULT)
                mreg[(s + 1) % 2] = __builtin_bit_cast(f32x4, lds_read_b128(bcur + MLDS + (64 * (i >> 2) + 16 * g + 4 * (i & 3)) * 4));
            // Eight groups, one matrix instruction each, in exactly this order (the scheduler
            // may not move anything across a group boundary): the matrix pipe never waits for
            // the VALU instructions and the one LDS read that follow it.
            //   groups 0..3  A: block row i of this tile's scores, query block m
            //   groups 4..7  C: V^T fragment (i+7)%8 of the previous tile (slot 0: of the one
            //                   before), query block m - 4; d = 64 has fragments 0..3 only
            //   every group  B: half a register of P from the block row finished in the
            //                   previous slot (query block m / 2, values 2 (m % 2), + 1)
            const frag_t kfr = whole(kfl[s % RING], kfh[s % RING]);
            const frag_t vfr = whole(vfl[s % RING], vfh[s % RING]);
            s16x2 wlo;
#pragma unroll
            for (int m = 0; m < 2 * NQ; ++m) {
                if (m < NQ) {
                    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                    Sn[m] = mfma8(kfr, qf[m], zero);
                    read_part(i + PD, m, bnn, bprv, bcur, bnxt);
                } else if (has_v(i)) {
                    oacc[(i + 7) % 8 % DB][m - NQ] = mfma8(vfr, Pr[m - NQ], oacc[(i + 7) % 8 % DB][m - NQ]);
                }
                const int qb = m / 2;
                const int left = keys_left(i == 0 ? tile - 1 : tile, (i + 7) % 8);   // the block row in Sc
                if (m % 2 == 0) wlo = stage_b_lo(Sc[qb], mreg[s % 2], qdiv[qb], qshift[qb], left);
                else Pw[qb][(i + 7) % 8] = stage_b_hi(wlo, Sc[qb], mreg[s % 2], qdiv[qb], qshift[qb], left);
                __builtin_amdgcn_sched_barrier(0);
            }
            // z of the previous tile as the diagonal of P^T P (P serves as A and as B operand:
            // lane (n16, g) holds the k-slots 32g.. of row, or column, n16 either way)
            if (i >= 1 && i <= NQ) zz[i - 1] = row_aggregate(Pr[i - 1], zz[i - 1]);
            // copies, two per slot: those of tile T+2 start behind the barrier and carry on in the
            // first slots of the next tile (where the same tile is T+1)
            if (i >= SLOTS - PD) {
                copy_chunk(2 * (i - (SLOTS - PD)), tile + 2, bnn);
                copy_chunk(2 * (i - (SLOTS - PD)) + 1, tile + 2, bnn);
            }
            if (i < (NCOPY_ALL + 1) / 2 - PD) {
                copy_chunk(2 * (i + PD), tile + 1, bnxt);
                copy_chunk(2 * (i + PD) + 1, tile + 1, bnxt);
            }
            if (i == SLOTS - 1) {
                SPH_LDS unsigned char* t = bprv; bprv = bcur; bcur = bnxt; bnxt = bnn; bnn = t;
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);            // copies past the end must not outlive the LDS

    // ---- drain.  The last tile processed is an odd one (P1); its block row 7 sits in SB
    // (written in slot 7), and V^T fragment 7 of the tile before it is still outstanding.
    {
        if constexpr (DB == 8) {
#pragma unroll
            for (int qb = 0; qb < NQ; ++qb) {
                // bcur now is the tile after the last, bprv the last, and the one before it:
                oacc[7][qb] = mfma8(whole(vfl[(2 * SLOTS) % RING], vfh[(2 * SLOTS) % RING]), P0[qb], oacc[7][qb]);
            }
        }
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb)
            P1[qb][7] = stage_b_hi(stage_b_lo(SB[qb], mreg[0], qdiv[qb], qshift[qb], keys_left(2 * n_pairs - 1, 7)), SB[qb],
                                   mreg[0], qdiv[qb], qshift[qb], keys_left(2 * n_pairs - 1, 7));
        // the last tile's Gram product (the loop adds a tile's in the next tile's slots)
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) zz[qb] = row_aggregate(P1[qb], zz[qb]);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const frag_t vfr = read_frag(bprv + KTILE + db * 2048);
#pragma unroll
            for (int qb = 0; qb < NQ; ++qb) oacc[db][qb] = mfma8(vfr, P1[qb], oacc[db][qb]);
        }
    }

    // ---- tail: O_i = o_i / sqrt(z_i); the row factor cancels.  Non-temporal stores only when
    // later batches of workgroups follow (see fwd_pipelined_kernel).
    const bool stream_out = stream_period > 0 && n_wg > kXcds * stream_period;
    const __amdgpu_buffer_rsrc_t orw = make_rsrc(O + (size_t)bh * N * D, (uint32_t)N * D * 2);
    // through a per-wave LDS stage, so that every store instruction writes whole rows (the tile
    // buffers are free once every wave has read its last tile)
    constexpr int ROWS = 16 * NQ;
    static_assert(kWaves * ROWS * (D * 2 + 16) <= NBUF * BUF_BYTES, "the output stage fits the tile buffers");
    SPH_LDS unsigned char* stage = smem + wave * ROWS * (D * 2 + 16);
    __syncthreads();
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
        // z_i: the diagonal element of query n16 (row 4g + t = n16) is held by lane group n16 / 4
        // in register n16 % 4; the other three lanes of the query get it through the sum
        const float dsel = (n16 & 3) == 0 ? zz[qb][0] : (n16 & 3) == 1 ? zz[qb][1] : (n16 & 3) == 2 ? zz[qb][2] : zz[qb][3];
        float z = sum_across_groups(g == (n16 >> 2) ? dsel : 0.f);
        // o and z were both accumulated from the scores divided by 2^e_i: the factor cancels
        float inv = z > 0.f ? 1.0f / __builtin_sqrtf(z) : 0.f;
        if constexpr (SOFTMAX) {                   // every row of the product is the row sum of query n16
            z = zz[qb][0];
            inv = z > 0.f ? 1.0f / z : 0.f;
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const i32x2 o4 = {pack2<false>(oacc[db][qb][0] * inv, oacc[db][qb][1] * inv),
                              pack2<false>(oacc[db][qb][2] * inv, oacc[db][qb][3] * inv)};
            put_piece<D * 2>(stage, qb * 16 + n16, db * 32 + 8 * g, o4);
        }
    }
    store_tile<ROWS, D * 2>(stage, orw, q0, N, lane, stream_out);
}

}  // namespace sphattn
