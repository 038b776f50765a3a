/*
 * sphattn -- spherical attention forward for AMD MI355X (gfx950), C ABI.
 *
 * Spherical attention is attention in which the SoftMax over each score row of
 * Q K^T is replaced by division by that row's L2 norm (paper, Section 3).  In the
 * paper's terms it is the normalized contraction of Appendix A.1 (Definition 2)
 * with a1(x) = x, a2(x) = x^2, b = sqrt, lifted to attention by Theorem 1:
 *
 *     s_ij       = sum_k Q[b,h,i,k] * K[b,h,j,k]
 *     z_i        = sum_j s_ij^2
 *     O[b,h,i,:] = ( sum_j s_ij * V[b,h,j,:] ) / sqrt(z_i)        (0 if z_i == 0)
 *
 * No score scale and no epsilon are applied (any positive scale cancels).  The
 * library evaluates this by streaming K/V tiles and carrying only the running
 * pair (o, z) per query row (Lemma 1), never materialising the N x N scores.
 *
 * All pointers are DEVICE pointers owned by the caller.  The library allocates
 * nothing (the one entry point that needs scratch memory, sphattn_splitkv_fwd, takes it from
 * the caller), keeps no state between calls (beyond a once-per-device kernel attribute) and is
 * re-entrant.  Work is enqueued on `stream`
 * (a hipStream_t passed as void*; NULL is the default stream) and the call
 * returns without synchronising.
 */
#ifndef SPHATTN_H
#define SPHATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Storage formats.  Arithmetic is MFMA with fp32 accumulation in every case. */
typedef enum {
    SPHATTN_F32 = 0,         /* Q,K,V,O fp32, fp32 matrix-core arithmetic */
    SPHATTN_BF16 = 1,        /* Q,K,V,O bfloat16 */
    SPHATTN_FP8QK_BF16V = 2, /* Q,K OCP E4M3 (finite-only) bytes; V,O bfloat16 */
    SPHATTN_F16 = 3          /* Q,K,V,O IEEE half (the paper's precision); scores must stay below 65504 */
} sphattn_dtype;

/* Return codes. */
enum {
    SPHATTN_OK = 0,
    SPHATTN_ERR_NULL = -1,        /* a required pointer is NULL */
    SPHATTN_ERR_SHAPE = -2,       /* B, H, N (or H_kv) not positive, H_kv not dividing H, or sizes overflow */
    SPHATTN_ERR_HEAD_DIM = -3,    /* d is not 64 or 128 */
    SPHATTN_ERR_DTYPE = -4,       /* dtype is not a sphattn_dtype value */
    SPHATTN_ERR_ALIGN = -5,       /* a pointer is not 16-byte aligned */
    SPHATTN_ERR_LAUNCH = -6,      /* the HIP runtime refused the launch */
    SPHATTN_ERR_ALIAS = -7,       /* O overlaps Q, K or V (or mult) */
    SPHATTN_ERR_NORMALIZER = -8,  /* normalizer is not a sphattn_normalizer value */
    SPHATTN_ERR_WORKSPACE = -9,   /* workspace NULL, not 16-byte aligned, or too small */
    SPHATTN_ERR_SCRATCH = -10     /* sphattn_splitkv_fwd_noalloc: needs more than SPHATTN_NOALLOC_SCRATCH_BYTES */
};

/* Normalizers N(x)_i = a1(x_i) / b(sum_j a2(x_j)) (paper, Appendix A.1, Definition 2). */
typedef enum {
    SPHATTN_NORM_L2 = 0,      /* a1 = x,          a2 = x^2,        b = sqrt : spherical attention */
    SPHATTN_NORM_SOFTMAX = 1, /* a1 = a2 = exp(x / sqrt(d)),       b = id   : standard attention  */
    SPHATTN_NORM_L1 = 2,      /* a1 = x,          a2 = |x|,        b = id                          */
    SPHATTN_NORM_SQRELU = 3   /* a1 = a2 = max(x,0)^2,             b = id                          */
} sphattn_normalizer;

/*
 * Spherical attention forward (paper, Section 3; Definition 2 and Lemma 1 of
 * Appendix A.1; Theorem 1), non-causal self-attention.
 *
 *   Q, K, V : [B,H,N,d] dense row-major, d contiguous, in the format `dtype` names.
 *   O       : [B,H,N,d] dense row-major, written in full; must not overlap Q, K, V.
 *   B, H, N : positive; N need not be a multiple of any tile size.
 *   d       : 64 or 128.
 *   dtype   : a sphattn_dtype value.
 *   stream  : hipStream_t to enqueue on.
 *
 * Returns SPHATTN_OK or a negative SPHATTN_ERR_* code; on error nothing is
 * enqueued and O is untouched.  Never throws or aborts.
 *
 * Range: scores and the row aggregates are fp32 on the device, so sum_j s_ij^2 must stay below
 * the fp32 maximum (3.4e38); beyond that a row comes out as zeros or NaN.  Inputs are expected
 * to be finite.
 *
 * 16-bit launches use workgroups of 256 query rows, or of 128 when 256-row tiles would
 * leave compute units without work (sphattn_fwd_tile_rows forces either shape).
 */
int sphattn_fwd(const void* Q, const void* K, const void* V, void* O,
                int B, int H, int N, int d, int dtype, void* stream);

/*
 * sphattn_fwd that also hands out the row aggregates of Definition 2:
 *   Z : [B,H,N] fp32 device pointer (4-byte aligned), Z[b,h,i] = z_i = sum_j s_ij^2 as the
 *       kernel accumulated it (fp32, from the fp32 scores); NULL: not written.  Must not overlap
 *       any other argument.  O_i * sqrt(z_i) recovers the unnormalised row, which is what a
 *       caller needs to merge results over key sets (Lemma 1) or to differentiate the tail.
 * Everything else as sphattn_fwd.
 */
int sphattn_fwd_z(const void* Q, const void* K, const void* V, void* O, float* Z,
                  int B, int H, int N, int d, int dtype, void* stream);

/*
 * sphattn_fwd_z with the workgroup shape of the 16-bit kernels forced, for tests and
 * measurements of both shapes on one problem (same definition as sphattn_fwd; the two shapes
 * add the same terms in different order):
 *   tile_rows : 0 = the library's choice (then this is sphattn_fwd_z), 128 or 256 query rows
 *               per workgroup; anything else returns SPHATTN_ERR_SHAPE.  Ignored where only
 *               one shape exists (fp32, fp16 and fp8-Q/K storage).
 */
int sphattn_fwd_tile_rows(const void* Q, const void* K, const void* V, void* O, float* Z,
                          int B, int H, int N, int d, int dtype, int tile_rows, void* stream);

/*
 * Gene-regulatory-network variant (paper, Section 3.1 and Appendix A.2).  Tokens are genes;
 * the key of gene j is multiplied by that gene's multiplicity in the cell before the scores
 * are formed, and K/V heads may be shared by groups of query heads (grouped-query attention):
 *
 *     s_ij = mult[b,j] * sum_k Q[b,h,i,k] * K[b,g,j,k],      g = h / (H / H_kv)
 *     O[b,h,i,:] = ( sum_j s_ij * V[b,g,j,:] ) / sqrt( sum_j s_ij^2 )
 *
 *   Q, O    : [B,H,N,d];   K, V : [B,H_kv,N,d], H_kv dividing H (H_kv == H: no sharing).
 *   mult    : [B,N] fp32 device pointer (4-byte aligned), finite values; NULL means all ones,
 *             which makes this call identical to sphattn_fwd when H_kv == H.
 * Everything else (layout, dtypes, ownership, stream, error codes) as sphattn_fwd;
 * SPHATTN_ERR_SHAPE also covers H_kv <= 0 or H % H_kv != 0.
 */
int sphattn_grn_fwd(const void* Q, const void* K, const void* V, const float* mult, void* O,
                    int B, int H, int H_kv, int N, int d, int dtype, void* stream);

/*
 * Attention with any of the normalizers above in place of the SoftMax (paper, Theorem 1: every
 * normalized contraction streams the same way; only the per-score functions and the tail
 * change).  SPHATTN_NORM_L2 is sphattn_fwd; SPHATTN_NORM_SOFTMAX computes what
 * sphattn_softmax_fwd computes, on the family's kernel (the same matrix instructions as the
 * spherical case) instead of the SoftMax-specific one.
 * A row whose aggregate sum_j a2(s_ij) is 0 gives 0.  dtype must be SPHATTN_BF16 unless the
 * normalizer is SPHATTN_NORM_L2; SPHATTN_NORM_SOFTMAX also takes SPHATTN_FP8QK_BF16V (the
 * comparison twin of the fp8-Q/K path: scores from the fp8 matrix instructions, then the same
 * exponential, running maximum and rescaling).  Other arguments, layout, ownership and errors as sphattn_fwd;
 * an unknown normalizer returns SPHATTN_ERR_NORMALIZER.
 */
int sphattn_normalized_fwd(const void* Q, const void* K, const void* V, void* O,
                           int B, int H, int N, int d, int dtype, int normalizer, void* stream);

/*
 * Comparison twin on the same tiling skeleton: standard SoftMax attention,
 * O = softmax(Q K^T / sqrt(d)) V, i.e. the same normalized contraction with
 * a1 = a2 = exp, b = id, computed with the usual running-maximum rescaling.
 * It exists to measure what the exponential costs (paper, Section 1), so it runs in the
 * form that is fastest for SoftMax (32x32x16 matrix instructions, which hide the
 * quarter-rate exponential better than the 16x16x32 ones of the spherical kernel).
 * Same arguments, layout, ownership and error behaviour as sphattn_fwd;
 * dtype must be SPHATTN_BF16.
 */
int sphattn_softmax_fwd(const void* Q, const void* K, const void* V, void* O,
                        int B, int H, int N, int d, int dtype, void* stream);

/*
 * Spherical attention between N_q query rows and N_k keys (Theorem 1 keeps the query and the
 * key axis apart; a chunk of queries against a longer key/value sequence is the case in mind):
 *
 *     O[b,h,i,:] = (sum_j s_ij V[b,g,j,:]) / sqrt(sum_j s_ij^2),   i < N_q, j < N_k,
 *
 * with s_ij as in sphattn_grn_fwd (mult NULL: all ones; H_kv == H: no sharing).
 *   Q, O : [B,H,N_q,d];   K, V : [B,H_kv,N_k,d];   mult : [B,N_k] fp32 or NULL;
 *   Z    : [B,H,N_q] fp32 or NULL, receives z_i as in sphattn_fwd_z.
 * sphattn_grn_fwd is this call with N_q == N_k and Z == NULL.  Errors as sphattn_grn_fwd
 * (SPHATTN_ERR_SHAPE also for N_q or N_k <= 0).
 */
int sphattn_cross_fwd(const void* Q, const void* K, const void* V, const float* mult, void* O, float* Z,
                      int B, int H, int H_kv, int N_q, int N_k, int d, int dtype, void* stream);

/*
 * The accumulator of Lemma 1 (Appendix A.1) over one set of keys, WITHOUT the tail: for query
 * rows Q[b,h,0..N_q) against the N_k keys/values given,
 *
 *     o_part[b,h,i,:] = sum_j s_ij * V[b,g,j,:]        z_part[b,h,i] = sum_j s_ij^2
 *
 * with s_ij as in sphattn_grn_fwd (mult NULL: all ones; H_kv == H: no sharing).  Because the
 * accumulator of a concatenation of key sets is the sum of their accumulators, the caller may
 * cut the key axis any way it likes (over calls, streams or GPUs), add the pairs, and apply
 * the tail once with sphattn_combine.
 *
 *   Q              : [B,H,N_q,d];   K, V : [B,H_kv,N_k,d] in the format `dtype` names.
 *   mult           : [B,N_k] fp32 or NULL.
 *   o_part, z_part : [B,H,N_q,d] and [B,H,N_q] fp32 (16- and 4-byte aligned), written in full;
 *                    must not overlap each other or the inputs.
 * Errors as sphattn_fwd (SPHATTN_ERR_SHAPE also for N_q or N_k <= 0).
 */
int sphattn_partial_fwd(const void* Q, const void* K, const void* V, const float* mult,
                        float* o_part, float* z_part,
                        int B, int H, int H_kv, int N_q, int N_k, int d, int dtype, void* stream);

/*
 * Sum of n_parts accumulator pairs followed by the tail of Lemma 1:
 *
 *     z_i = sum_p z_parts[p][b,h,i]      O[b,h,i,:] = (sum_p o_parts[p][b,h,i,:]) / sqrt(z_i)
 *
 * (0 if z_i == 0).  The parts are added in ascending p, in fp32.
 *   o_parts : [n_parts][B,H,N,d] fp32, contiguous;   z_parts : [n_parts][B,H,N] fp32.
 *   O       : [B,H,N,d] in the OUTPUT type of `dtype` (fp32 for SPHATTN_F32, IEEE half for
 *             SPHATTN_F16, bfloat16 otherwise);   Z : [B,H,N] fp32 or NULL, receives z_i.
 *   n_parts : 1 .. 65536.
 * Outputs must not overlap the parts.  Errors as sphattn_fwd.
 */
int sphattn_combine(const float* o_parts, const float* z_parts, int n_parts, void* O, float* Z,
                    int B, int H, int N, int d, int dtype, void* stream);

/*
 * sphattn_grn_fwd with the key axis cut into n_splits slices that run as separate workgroups
 * (sphattn_partial_fwd per slice, then sphattn_combine, in two launches; with one slice it is
 * sphattn_grn_fwd itself and the workspace is not touched).  It pays when B * H * N / 256 is
 * below the number of workgroups the device runs at once, i.e. few heads of moderate length.
 *
 *   n_splits       : slices asked for; 0 lets sphattn_splitkv_heuristic choose.  Slices are
 *                    whole 64-key tiles of equal size, so fewer than asked may be used (any
 *                    count above the number of tiles means one tile per slice).
 *   workspace      : device scratch, 16-byte aligned, at least
 *                    sphattn_splitkv_workspace_bytes(B,H,N,d,n_splits) bytes (n_splits as passed
 *                    here, or the heuristic's value when 0); contents undefined afterwards.
 *                    Must not overlap any other argument; calls that overlap in time need
 *                    workspaces of their own.
 *   Z              : [B,H,N] fp32 or NULL, as in sphattn_fwd_z.
 * Other arguments and errors as sphattn_grn_fwd; a bad workspace returns SPHATTN_ERR_WORKSPACE,
 * n_splits < 0 returns SPHATTN_ERR_SHAPE.
 */
int sphattn_splitkv_fwd(const void* Q, const void* K, const void* V, const float* mult, void* O, float* Z,
                        int B, int H, int H_kv, int N, int d, int dtype, int n_splits,
                        void* workspace, size_t workspace_size, void* stream);

/*
 * sphattn_splitkv_fwd for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (without the workspace), same kernels, same result bit for bit; the partial pairs
 * live in an array of SPHATTN_NOALLOC_SCRATCH_BYTES bytes that is part of the library itself
 * (one per GPU the library runs on, held until the process ends).  The call allocates and
 * frees nothing.
 *   - A problem whose slices need more, sphattn_splitkv_workspace_bytes(B,H,N,d,n_splits) >
 *     SPHATTN_NOALLOC_SCRATCH_BYTES (n_splits as used: the heuristic's value when 0 is passed,
 *     never more than the number of 64-key tiles), returns SPHATTN_ERR_SCRATCH; nothing is enqueued.
 *     One slice is the unsplit launch, uses no scratch and has no such limit; when 0 is passed
 *     and the heuristic's slices would not fit, one slice is used instead of an error.
 *   - Every call on a GPU uses that GPU's one array: calls that may overlap in time on one GPU
 *     (different streams, different threads) race on it and must be ordered by the caller.
 *     Nothing in the array has to start at zero: each call writes every partial it reads.
 * Other arguments and errors as sphattn_splitkv_fwd.
 */
#define SPHATTN_NOALLOC_SCRATCH_BYTES (64u << 20)
int sphattn_splitkv_fwd_noalloc(const void* Q, const void* K, const void* V, const float* mult, void* O, float* Z,
                                int B, int H, int H_kv, int N, int d, int dtype, int n_splits, void* stream);

/* Bytes of workspace sphattn_splitkv_fwd needs for n_splits >= 1 slices: n_splits * B*H*N * (d+1)
 * fp32 values, rounded up to 256.  Returns 0 for arguments sphattn_splitkv_fwd would reject. */
size_t sphattn_splitkv_workspace_bytes(int B, int H, int N, int d, int n_splits);

/* Number of slices sphattn_splitkv_fwd uses when asked for 0: 1 when whole-key-axis workgroups
 * fill their rounds on the compute units of the current device (256 when no device can be
 * asked) or when cutting is not expected to gain at least 3 %; otherwise the count, in slices of at least
 * 8 tiles, with the lowest estimated run time: rounds of workgroups, how full they are, the
 * slices' prologues and the combine step are priced from measurements on one MI355X.
 * Launches nothing. */
int sphattn_splitkv_heuristic(int B, int H, int N, int d, int dtype);

/*
 * Backward of sphattn_fwd.  The paper states no backward pass; this is the chain rule on its
 * definition.  With r_i = 1/sqrt(z_i) and delta_i = dO[b,h,i,:] . O[b,h,i,:]:
 *
 *     dV[b,h,j,:] = sum_i r_i s_ij dO[b,h,i,:]
 *     ds_ij       = r_i (dO[b,h,i,:] . V[b,h,j,:]) - delta_i r_i^2 s_ij
 *     dQ[b,h,i,:] = sum_j ds_ij K[b,h,j,:]          dK[b,h,j,:] = sum_i ds_ij Q[b,h,i,:]
 *
 * (rows with z_i == 0 contribute nothing).  The scores are recomputed tile by tile; nothing
 * N x N is stored and no atomics are used, so results do not depend on the launch.
 *
 *   Q, K, V, O, dO : [B,H,N,d] in the 16-bit format of `dtype` (SPHATTN_BF16 or SPHATTN_F16;
 *                    anything else returns SPHATTN_ERR_DTYPE); O and Z as sphattn_fwd_z wrote them.
 *   Z              : [B,H,N] fp32, the row aggregates z_i.
 *   dQ, dK, dV     : [B,H,N,d] in the same 16-bit format, written in full.
 *   delta          : [2,B,H,N] fp32 scratch from the caller; the first launch leaves delta_i r_i^2 (first
 *                    plane) and r_i (second plane) there for the second.
 * Outputs and scratch must not overlap each other or the inputs.  Two launches on `stream`.
 * Other arguments and errors as sphattn_fwd.
 */
int sphattn_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* Z,
                void* dQ, void* dK, void* dV, float* delta,
                int B, int H, int N, int d, int dtype, void* stream);

/*
 * Backward of sphattn_grn_fwd: with s_ij = mult[b,j] (q_i . k_j) and K/V heads shared by groups
 * of H / H_kv query heads,
 *
 *     dQ[b,h,i,:] = sum_j ds_ij mult[b,j] K[b,g,j,:]
 *     dK[b,g,j,:] = mult[b,j] sum_{h in group g} sum_i ds_ij Q[b,h,i,:]
 *     dV[b,g,j,:] = sum_{h in group g} sum_i r_i s_ij dO[b,h,i,:]
 *
 * with ds_ij, r_i, delta_i as in sphattn_bwd.  The multiplicities are data: no gradient.
 *   Q, O, dO, dQ : [B,H,N,d];  K, V, dK, dV : [B,H_kv,N,d];  Z : [B,H,N] fp32;  delta : [2,B,H,N] fp32;
 *   mult : [B,N] fp32 or NULL (all ones).
 * Everything else as sphattn_bwd, which is this call with mult == NULL and H_kv == H.
 */
int sphattn_grn_bwd(const void* Q, const void* K, const void* V, const float* mult,
                    const void* O, const void* dO, const float* Z,
                    void* dQ, void* dK, void* dV, float* delta,
                    int B, int H, int H_kv, int N, int d, int dtype, void* stream);

/*
 * Spherical attention with Q, K AND V stored in OCP E4M3 and both contractions on the fp8
 * matrix instructions (paper, Section 1 and Section 3.1: without the row-wise exponential the
 * whole operator can run at the matrix cores' low-precision rate).  Same function as
 * sphattn_fwd on the stored values, O_i = (sum_j s_ij v_j) / sqrt(sum_j s_ij^2) with
 * s_ij = q_i . k_j, except that the scores are rounded to E4M3 before they are used: row i is
 * divided by the power of two 2^e_i with |q_i| max_j |k_j| / 440 = m 2^e_i, m in [0.5, 1), rounded
 * to nearest even, and both sums are taken over the rounded values (the row factor cancels in
 * the quotient).  The result carries the relative error of a 3-bit mantissa on every term
 * of the sum: about 2.7 % of rms(O) in the root mean square and up to about 15 % of rms(O) on
 * single elements, not the 2^-9 of the 16-bit paths.
 *   Q        : device, [B,H,N,d] contiguous, one byte per element (E4M3, finite values),
 *              16-byte aligned.  d is 64 or 128 (anything else: SPHATTN_ERR_HEAD_DIM); d = 64 runs
 *              the first contraction on the same k = 128 instruction with half of its slots zero.
 *   K, V     : the same with H_kv heads, [B,H_kv,N,d]; H_kv divides H, and query head h reads
 *              K/V head h / (H / H_kv) (Appendix A.2); H_kv == H: no sharing.
 *   O        : device, [B,H,N,d] bfloat16, written by the call, must not overlap the inputs.
 *   workspace: device scratch owned by the caller, 16-byte aligned, at least
 *              sphattn_fp8_workspace_bytes(B, H_kv, N, d) bytes (a transposed copy of V padded
 *              to whole 128-key tiles, and the largest key norm of every K/V head); overwritten by the
 *              call, must not overlap Q, K, V or O.  A NULL, misaligned or short workspace
 *              returns SPHATTN_ERR_WORKSPACE.  Calls that share a workspace must be ordered.
 * Three launches on `stream` (clear, prepare, attention); no allocation, no synchronisation.
 * Other errors as sphattn_fwd.  sphattn_fp8_workspace_bytes returns 0 for an invalid shape.
 */
size_t sphattn_fp8_workspace_bytes(int B, int H_kv, int N, int d);
int sphattn_fp8_fwd(const void* Q, const void* K, const void* V, void* O,
                    void* workspace, size_t workspace_bytes,
                    int B, int H, int H_kv, int N, int d, void* stream);

/*
 * sphattn_fp8_fwd with the gene multiplicities of sphattn_grn_fwd (paper, Section 3.1):
 * s_ij = mult[b,j] (q_i . k_j), multiplied in fp32 before the score is scaled and rounded to
 * E4M3; the row factor 2^e_i then comes from |q_i| max_j |mult[b,j]| |k_j|.
 *   mult : [B,N] fp32 device pointer (4-byte aligned), finite values; NULL means all ones
 *          (then this is sphattn_fp8_fwd).  Must not overlap O or the workspace.
 * Everything else as sphattn_fp8_fwd.
 */
int sphattn_fp8_grn_fwd(const void* Q, const void* K, const void* V, const float* mult, void* O,
                        void* workspace, size_t workspace_bytes,
                        int B, int H, int H_kv, int N, int d, void* stream);

/*
 * Comparison twin of sphattn_fp8_fwd: O = softmax(Q K^T / sqrt(d)) V with the same storage, the
 * same kernel skeleton and the weights entering the second contraction as E4M3, made as cheap
 * as a SoftMax can be there: row i is shifted by the bound |q_i| max_j |k_j| / sqrt(d) instead
 * of its running maximum (mathematically the same function), so that only a scale-and-shift and
 * an exponential per score are added to the spherical kernel's work.  For timing the cost of the
 * exponential at the fp8 matrix rate (paper, Section 1) on inputs of moderate size: a row whose
 * largest score lies more than about 12 sqrt(d) below that bound underflows to all-zero
 * weights and gives 0.  Arguments, workspace and errors as sphattn_fp8_fwd.
 */
int sphattn_fp8_softmax_fwd(const void* Q, const void* K, const void* V, void* O,
                            void* workspace, size_t workspace_bytes,
                            int B, int H, int H_kv, int N, int d, void* stream);

/* Human-readable text for a return code (static storage, never NULL). */
const char* sphattn_strerror(int code);

/* Library version as major*10000 + minor*100 + patch. */
int sphattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPHATTN_H */
