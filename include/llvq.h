/*
 * llvq.h -- C ABI of the MI355X (gfx950) library for Leech Lattice Vector Quantization inference.
 *
 * The library decodes 48-bit indices into points of the ball cut Lambda_24(m_max) of the Leech
 * lattice (union of shells 2..m_max, paper Sec. 2.2), applies the shape-gain scale (paper App. E,
 * "Shape-gain": w = g * s, s = x/||x||), and multiplies activations by the dequantised weight
 * matrix without materialising it (paper App. C).  Every step runs in HIP kernels on the device;
 * there is no CPU fallback: a call made without a usable GPU returns LLVQ_EHIP.
 *
 * Conventions
 *   - All pointers named d_* are DEVICE pointers owned by the caller.  The library allocates device
 *     memory only inside llvq_create (constant tables) and frees it in llvq_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work on
 *     it and return without synchronising, except llvq_validate.
 *   - Return value: 0 on success, a negative LLVQ_E* code otherwise.  Nothing throws or aborts.
 *   - Index (paper Sec. 3.2, App. A): 0-based, I in [0, N(m_max)); shells by increasing radius,
 *     classes contiguous inside a shell, inside a class the Golay refinement r is the least
 *     significant digit, then the sign pattern s, then the permutation rank I''.
 *   - Decoded coordinates are those of L_int = sqrt(8) * Lambda_24 (paper Sec. 2.3): integers with
 *     sum x_i^2 = 16 m on shell m.
 *   - An index >= N(m_max) (the paper does not define it) decodes to the all-zero block.
 *   - n_blocks == 0 is a valid no-op; the data pointers are then not examined.
 *   - A weight matrix W_hat[N][K], K = 24*KB, is stored block-wise: one index and one fp16 gain per
 *     (row n, block b), blocks partitioning the input channels of each row (paper App. B, Alg. 1).
 *     Activations are supplied zero-padded to K (paper App. C uses 4096 -> 4104).
 */
#ifndef LLVQ_H
#define LLVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct llvq_ctx llvq_ctx;

enum {
    LLVQ_OK = 0,
    LLVQ_EINVAL = -1,    /* null pointer, non-positive size, unsupported dtype/format, m_max out of range */
    LLVQ_EALIGN = -2,    /* a pointer is not aligned as its format requires                              */
    LLVQ_EHIP = -3,      /* a HIP call failed (no device, allocation, launch); see llvq_last_hip_error   */
    LLVQ_ENOTIMPL = -4   /* valid request that this build does not implement                             */
};

/* index storage formats */
enum {
    LLVQ_IDX_U48 = 0,    /* 6 bytes per index, little endian, densely packed; 2-byte aligned base        */
    LLVQ_IDX_U64 = 1,    /* one uint64 per index (upper 16 bits ignored; upper 8 bits in contexts with
                            m_max > 13); 8-byte aligned base                                             */
    LLVQ_IDX_U24 = 2     /* 3 bytes per word, little endian, densely packed; no alignment requirement: the
                            1 bit/weight layout of a single small shell (paper App. C, "single shell")      */
};

/* metrics of llvq_quantize */
enum {
    LLVQ_ANGULAR = 0,    /* maximise <w, x> / ||x||  (shape-gain: the code is the set of directions)             */
    LLVQ_EUCLIDEAN = 1   /* minimise ||w - x||^2     (spherical shaping: the code is the ball cut itself)        */
};

/* element types */
enum {
    LLVQ_F16 = 0,
    LLVQ_BF16 = 1,
    LLVQ_F32 = 2
};

/* Create a context for the code Lambda_24(m_max), 2 <= m_max <= 19, on HIP device `device`.
 * m_max <= 13 (indices below 2^48; 13 is the paper's 2 bits per weight) gets the full library.  14 <= m_max <= 19 (paper
 * Table 1, row m = 19: 23,546,209,100,646,960 points, 55-bit indices) gets the dequantiser only: llvq_decode_i8,
 * llvq_decode, llvq_matmul with M <= 16 (LLVQ_ENOTIMPL above), llvq_matmul_ws (same as llvq_matmul), llvq_validate,
 * llvq_validate_static, llvq_num_points, llvq_num_classes and llvq_shell_offset, through a slower decoder that keeps
 * its tables in global memory; every other call returns LLVQ_ENOTIMPL.  In these contexts a LLVQ_IDX_U64 word carries
 * the index in its low 56 bits (upper 8 bits ignored), and llvq_matmul combines partial sums with fp32 atomic adds.
 * Builds the constant tables (Golay words, class records, ranking tables) on the host and copies
 * them to the device.  The tables are immutable afterwards; llvq_decode*, llvq_matmul, llvq_matmul_multi, llvq_matmul_coded, llvq_encode,
 * llvq_repack, llvq_quantize and llvq_shell_offset may be called on one context from several threads.  llvq_matmul_ws,
 * llvq_gptq_quantize (they share the context's BLAS handle) and llvq_validate (its counter) may not.   */
int llvq_create(llvq_ctx** out, int m_max, int device);
void llvq_destroy(llvq_ctx* ctx);

const char* llvq_strerror(int rc);
/* Text of the last failure seen by this context ("" if none).  The text is written under a lock, so calls that fail
 * on several threads at once do not corrupt it, but it is one buffer per context: read it before another call on the
 * same context can fail.                                                                                   */
const char* llvq_last_hip_error(const llvq_ctx* ctx);

/* N(m_max) = |Lambda_24(m_max)| (paper Table 1): 280,974,212,784,720 for m_max = 13, 23,546,209,100,646,960 for 19. */
uint64_t llvq_num_points(const llvq_ctx* ctx);
/* number of classes over all shells (383 for m_max = 13, 1,457 for m_max = 19) */
int llvq_num_classes(const llvq_ctx* ctx);

/* Index of the first point of shell m, i.e. N(m-1) of paper Table 1 (0 for m <= 2, N(m_max) for m > m_max):
 * the base_index that makes a coded word address shell m alone.                                     */
uint64_t llvq_shell_offset(const llvq_ctx* ctx, int m);

/* Dequantiser of paper App. A: d_out[k][0..23] = integer coordinates of index k, int8.
 * d_idx: n_blocks indices in format `fmt`.  d_out must be 8-byte aligned (LLVQ_EALIGN otherwise).  */
int llvq_decode_i8(llvq_ctx* ctx, const void* d_idx, int fmt, size_t n_blocks,
                   int8_t* d_out, void* stream);

/* Shape-gain reconstruction (paper App. E): d_out[k][i] = g_k * x_i / sqrt(16 m_k), computed in
 * fp32 and rounded to out_dtype (LLVQ_F16, LLVQ_BF16 or LLVQ_F32).  d_gain: n_blocks fp16 gains
 * (2-byte aligned).  d_out must be 16-byte aligned (LLVQ_EALIGN otherwise).                       */
int llvq_decode(llvq_ctx* ctx, const void* d_idx, int fmt, const void* d_gain, size_t n_blocks,
                void* d_out, int out_dtype, void* stream);

/* Fused dequantise + multiply (paper App. C): d_y[m][n] = sum_k d_x[m][k] * W_hat[n][k], fp32.
 *   d_x   : [M][24*KB] row-major, x_dtype LLVQ_F16 or LLVQ_BF16, zero-padded by the caller; 16-byte aligned
 *   d_idx : [N][KB] indices in format `fmt`;  d_gain: [N][KB] fp16
 *   d_y   : [M][N] row-major fp32, overwritten
 * 1 <= M <= 1024.  M = 1 is the decode (matrix-vector) case the paper times.
 * M <= 2: products activation * integer coordinate are exact in fp32, accumulated in fp32 and scaled by
 *   gain / sqrt(16 m) per block (v_dot2 kernel); the partial sums of a row are combined with fp32 atomic adds in
 *   LDS, so the last bits of y can differ between calls (about 1e-7 relative).
 * M >= 3 (batched decode, prefill): the weights gain * x / sqrt(16 m) are formed in fp32, brought to the activation
 *   type (fp16: one value, relative rounding error 2^-11; bf16: two values, the rounding and the rounding of what it
 *   leaves, together 2^-17) and contracted on the matrix cores with fp32 accumulation.
 *   3 <= M <= 32: a tile of 16 rows is reduced over K inside one workgroup in a fixed order: no clearing, no atomic
 *   adds, the same bits from call to call.  33 <= M <= 64: partial sums of different K ranges are combined with fp32
 *   atomic adds after y was cleared, so the last bits of y can differ between calls.  M > 64: strips of 256 rows x
 *   256 tokens, from M = 384 on panels of 128 rows x 512 tokens; when they number more than half the compute units
 *   K is not split and y is reproducible, otherwise as for 33 <= M <= 64.
 *   Requires N*KB < 2^32, KB < 2^24 and M*N < 2^32 (LLVQ_EINVAL otherwise).                            */
int llvq_matmul(llvq_ctx* ctx, const void* d_x, int x_dtype, int M,
                const void* d_idx, int fmt, const void* d_gain, int N, int KB,
                float* d_y, void* stream);

/* The products y_i = W_i x of n_items (1..4) matrices that share the activations x, K (KB blocks per row) and the word
 * format: the q/k/v or the gate/up matrices of a transformer block (the fused product of paper App. C, several
 * weight matrices per launch).  d_idx, d_gain, N and d_y are HOST arrays of n_items entries (device pointers and row
 * counts, read during the call); every matrix and every output is laid out as for llvq_matmul (y_i is [M][N_i]).  For
 * M <= 64 all products run in ONE launch (for 33 <= M <= 64 after one launch that clears all outputs), which pays the
 * per-launch start-up once.  For M >= 384 the 128-row strips of all matrices share one launch of the prefill kernel
 * when at least one matrix alone would leave more than half of the compute units idle (k and v next to q; gate and up
 * below 1024 tokens); otherwise, and for 64 < M < 384, the call is the same as n_items calls of llvq_matmul.  Requires
 * (N_0 + .. + N_last)*KB < 2^32; arguments and errors otherwise as for llvq_matmul (LLVQ_EINVAL also for n_items
 * outside 1..4).                                                                                              */
int llvq_matmul_multi(llvq_ctx* ctx, const void* d_x, int x_dtype, int M, int n_items,
                      const void* const* d_idx, int fmt, const void* const* d_gain, const int* N, int KB,
                      float* const* d_y, void* stream);

/* llvq_matmul with a caller-provided device workspace of ws_bytes >= N*KB*48 bytes (16-byte aligned).  For
 * M >= 96 the weights are then dequantised ONCE into the workspace in the activation type (the kernel of
 * llvq_decode) and multiplied by a plain dense library GEMM (rocBLAS, matrix cores, fp32 accumulation): the
 * prefill path for large M, where re-decoding per token tile would dominate.  With a smaller workspace, a NULL
 * one or a smaller M it behaves exactly like llvq_matmul.  The workspace content is overwritten; nothing is
 * kept in it between calls.                                                                              */
int llvq_matmul_ws(llvq_ctx* ctx, const void* d_x, int x_dtype, int M,
                   const void* d_idx, int fmt, const void* d_gain, int N, int KB,
                   float* d_y, void* d_ws, size_t ws_bytes, void* stream);

/* Coded words (paper App. E "Shape-gain": one integer carries the shape index and the gain index; paper
 * Sec. 4 tables, "1 bit / 2 bit gain"; paper App. C, single-shell variant).  A stored word v of 48 bits
 * (LLVQ_IDX_U48, LLVQ_IDX_U64) or 24 bits (LLVQ_IDX_U24) is split as
 *     lattice index I = (v mod 2^shape_bits) + base_index,      gain code c = v >> shape_bits,
 * 1 <= shape_bits <= word bits, base_index < 2^48.  With d_gain_lut != NULL the gain of the block is
 * d_gain_lut[c] (DEVICE, fp16, 2^(word bits - shape_bits) <= 4096 entries: the levels of the scalar gain
 * quantiser) and d_gain is ignored (may be NULL); with d_gain_lut == NULL the bits above shape_bits are
 * ignored and d_gain holds one fp16 per block as in the plain calls.  base_index = llvq_shell_offset(ctx, m)
 * with shape_bits = ceil(log2 n(m)) addresses shell m alone.  I >= N(m_max) decodes to the zero block.
 * Everything else (layouts, M ranges, rounding) is as in llvq_decode_i8 / llvq_decode / llvq_matmul.  */
int llvq_decode_i8_coded(llvq_ctx* ctx, const void* d_idx, int fmt, int shape_bits, uint64_t base_index,
                         size_t n_blocks, int8_t* d_out, void* stream);
int llvq_decode_coded(llvq_ctx* ctx, const void* d_idx, int fmt, int shape_bits, uint64_t base_index,
                      const void* d_gain_lut, const void* d_gain, size_t n_blocks,
                      void* d_out, int out_dtype, void* stream);
int llvq_matmul_coded(llvq_ctx* ctx, const void* d_x, int x_dtype, int M,
                      const void* d_idx, int fmt, int shape_bits, uint64_t base_index,
                      const void* d_gain_lut, const void* d_gain, int N, int KB,
                      float* d_y, void* stream);

/* One aligned 64-bit word per block (8 bytes per block as with separate arrays: paper App. E, one integer carries
 * shape and gain): d_packed[k] = index k (bits 0..47) | the fp16 bits of gain k (bits 48..63).
 *   d_idx : n_blocks indices, LLVQ_IDX_U48 or LLVQ_IDX_U64;  d_gain: n_blocks fp16;  d_packed: n_blocks uint64, 8-byte aligned
 * The packed array is read by llvq_decode_coded and llvq_matmul_coded called with fmt = LLVQ_IDX_U64, shape_bits = 48,
 * d_gain_lut = NULL and d_gain = NULL: with no gain table and no gain array the gain of a block is taken from
 * the top 16 bits of its word.  (llvq_decode_i8_coded ignores those bits anyway.)                            */
int llvq_repack(llvq_ctx* ctx, const void* d_idx, int fmt, const void* d_gain, size_t n_blocks,
                uint64_t* d_packed, void* stream);

/* Encoder side of the index map (paper Sec. 3.2, "bijective indexing"; the inverse of the dequantiser of
 * App. A): d_idx[k] = the index I with llvq_decode_i8(I) = d_x[k][0..23].
 *   d_x   : [n_blocks][24] int8 coordinates of L_int (sum x^2 = 16 m), 8-byte aligned
 *   d_idx : n_blocks indices in format `fmt` (LLVQ_IDX_U48 or LLVQ_IDX_U64), written
 * A vector that is not a point of Lambda_24(m_max) -- mixed parity, (x - parity)/2 mod 2 not a Golay word, wrong
 * sum modulo 8 (paper Sec. 2.3, conditions (i)-(iii)), or a norm outside shells 2..m_max -- gets the all-ones
 * code (48 or 64 one bits), which every decoding call treats as out of range.                            */
int llvq_encode(llvq_ctx* ctx, const int8_t* d_x, size_t n_blocks, void* d_idx, int fmt, void* stream);

/* Quantiser (paper Sec. 3 and 3.1: search over leaders, Golay placements and parity-constrained signs, extended
 * to the union of shells with angular or Euclidean scoring): for every block of 24 reals the point x of
 * Lambda_24(m_max) that maximises <w, x> / ||x|| (LLVQ_ANGULAR) or minimises ||w - x|| (LLVQ_EUCLIDEAN), both in
 * the coordinates of L_int (||x||^2 = 16 m; scale w accordingly for the Euclidean metric).
 *   d_w      : [n_blocks][24] fp32, finite
 *   d_points : [n_blocks][24] int8, written: the chosen points (8-byte aligned)
 *   d_idx    : n_blocks indices in format `fmt`, written through llvq_encode; NULL: not wanted
 *   d_score  : n_blocks fp32, written: <w, x> / ||x|| (angular; this is also the least-squares gain of the block,
 *              paper App. E "optimal scales") or <w, x> - ||x||^2 / 2 (Euclidean); NULL: not wanted
 * Scores are accumulated in fp32: among candidates whose scores differ by less than rounding (about 2e-6
 * relative) either may be returned; the returned point is always a point of the ball cut.                  */
int llvq_quantize(llvq_ctx* ctx, const float* d_w, size_t n_blocks, int metric, int8_t* d_points,
                  void* d_idx, int fmt, float* d_score, void* stream);

/* Block-wise quantisation of a layer with Hessian corrections (paper App. B, Alg. 1; Sec. 3.3 "Spherical
 * GPTQ"; App. F "Hessian-based corrections"): input-channel blocks of 24 are processed left to right; for every
 * row the current block v is replaced by g * x / ||x||, x the nearest direction of Lambda_24(m_max) (the search of
 * llvq_quantize) and g = ||v|| rounded to fp16 (gain reset onto the sphere of radius ||v||); the error
 * E = v - g x/||x|| is propagated into the not yet processed columns R: W[:, R] -= (E U_QQ^-1) U_QR.
 *   d_W   : [N][ldw] fp32 row-major, ldw >= 24*KB; in: the layer's weights, out: the quantised layer
 *           (exactly what llvq_decode reconstructs from d_idx and d_gain, up to fp32 rounding)
 *   d_U   : [K][K] fp32 row-major, K = 24*KB: the upper-triangular factor U with H^-1 = U^T U of the layer's
 *           input second-moment matrix H (the caller's, e.g. damped); only the upper triangle is read
 *   d_idx : [N][KB] indices in format `fmt` (LLVQ_IDX_U48 or LLVQ_IDX_U64), written;  d_gain: [N][KB] fp16, written
 *   d_ws  : device workspace of at least llvq_gptq_workspace_bytes(N) bytes, 16-byte aligned
 * The dense steps (a 24 x 24 triangular solve and an N x 24 x |R| product per block) are library BLAS calls.
 * K not a multiple of 24: pad W with zero columns and U with an identity block.                         */
size_t llvq_gptq_workspace_bytes(int N);
int llvq_gptq_quantize(llvq_ctx* ctx, float* d_W, int N, int KB, size_t ldw, const float* d_U,
                       void* d_idx, int fmt, void* d_gain, void* d_ws, size_t ws_bytes, void* stream);

/* llvq_gptq_quantize with the optional scalar gain quantiser of paper App. B, Alg. 1 (the line "optionally: Q_gain"):
 * the gain of a block is the nearest of the n_levels reconstruction levels d_gain_levels (DEVICE, fp16, ascending,
 * 1 <= n_levels <= 4096; ties go to the lower level) instead of the rounded norm, and the error that is propagated
 * includes that choice.  d_gain receives the chosen level of every block.  d_gain_levels == NULL: exactly
 * llvq_gptq_quantize.  Everything else as for llvq_gptq_quantize.                                            */
int llvq_gptq_quantize_levels(llvq_ctx* ctx, float* d_W, int N, int KB, size_t ldw, const float* d_U,
                              void* d_idx, int fmt, void* d_gain, const void* d_gain_levels, int n_levels,
                              void* d_ws, size_t ws_bytes, void* stream);

/* Closed-form group scales after the block loop (paper App. J, algorithm "Spherically projected GPTQ with group
 * scales", final per-row block-scale refinement in the Hessian metric): with the directions fixed, every row i gets the
 * gains s_i = (M_i + lambda I)^-1 r_i, M_i[p][q] = Wq_{i,p} H_{pq} Wq_{i,q}^T, r_i[p] = Wq_{i,p} H_{p,:} W0_i^T, i.e. the
 * minimiser of (W0_i - sum_p s_p Wq_{i,p}) H (...)^T + lambda |s|^2.
 *   d_Wq  : [N][ldw] fp32, in: the quantised layer (as written by llvq_gptq_quantize), out: the refined layer
 *   d_W0  : [N][ldw] fp32, the original weights;  d_H: [K][K] fp32, symmetric positive definite, K = 24*KB <= 24576
 *   d_gain: [N][KB] fp16, in: the gains of the quantised layer, out: gain * s rounded to fp16; every block of d_Wq is
 *           rescaled by exactly the ratio of the two fp16 gains, so that it stays what llvq_decode reconstructs
 *   d_s   : [N][KB] fp32, written: the scales (NULL: not wanted);  lambda >= 0
 *   d_ws  : workspace of at least llvq_gptq_group_scales_workspace_bytes(N, KB) bytes, 16-byte aligned
 * Arithmetic in fp32 (dense products by library BLAS calls, one Cholesky factorisation per row in a kernel of this
 * library); a row whose system is not positive definite in fp32 is left unchanged (s = 1).                      */
size_t llvq_gptq_group_scales_workspace_bytes(int N, int KB);
int llvq_gptq_group_scales(llvq_ctx* ctx, float* d_Wq, const float* d_W0, int N, int KB, size_t ldw,
                           const float* d_H, float lambda, void* d_gain, float* d_s,
                           void* d_ws, size_t ws_bytes, void* stream);

/* Count indices that are not below N(m_max).  Synchronises the stream; *h_bad is a HOST pointer.  */
int llvq_validate(llvq_ctx* ctx, const void* d_idx, int fmt, size_t n_blocks,
                  uint64_t* h_bad, void* stream);

/* llvq_validate for callers that cannot allocate or synchronise: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The count goes to DEVICE memory, nothing synchronises, and the call
 * allocates nothing: the per-workgroup partial counts live in a 4 KB device array that is part of the library
 * (every GPU the library runs on holds its copy until the process ends).
 *   d_bad : DEVICE pointer, 8-byte aligned: receives the number of indices >= N(m_max) once the stream gets there
 * n_blocks > LLVQ_VALIDATE_STATIC_MAX_BLOCKS is refused with LLVQ_EINVAL (llvq_last_hip_error names the limit):
 * a workgroup's partial count has 32 bits.  n_blocks == 0 writes 0.  Every call on one GPU uses that GPU's one
 * array, whatever the context: calls that overlap in time on one GPU (different streams, different threads)
 * race and may report wrong counts; calls ordered on one stream are safe (each overwrites the partial counts
 * it then adds, nothing needs clearing in between).                                                      */
#define LLVQ_VALIDATE_STATIC_MAX_BLOCKS ((size_t)1 << 32)
int llvq_validate_static(llvq_ctx* ctx, const void* d_idx, int fmt, size_t n_blocks,
                         uint64_t* d_bad, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LLVQ_H */
