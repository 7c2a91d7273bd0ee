/*
 * halo.h -- C ABI of the MI355X (gfx950) HALO low-precision linear layer.
 *
 * HALO (Hadamard-Assisted Lower-Precision Optimization) runs the three matrix products of a
 * linear layer in INT8:
 *      F:  Y   = X  W^T      (Section 2, Eq. 1a)        X [b x m], W [n x m], Y [b x n]
 *      G:  G   = E^T X       (Section 2, Eq. 1b)        E = E_Y [b x n], G [n x m]
 *      E:  E_X = E  W        (Section 2, Eq. 1c)        E_X [b x m]
 * with Walsh-Hadamard rotations placed according to the HALO level (Appendix, Table "HALO
 * levels"; Section 3.3).  Every operand is quantised with a symmetric absmax scale per row of
 * the GEMM operand, round-to-nearest-even, codes in [-127, 127].
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers (HIP device memory of the current device).  The
 *     caller owns every buffer; the library never allocates, frees or synchronises.  All work
 *     is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - Matrices are row-major.  A leading dimension `ld*` is in ELEMENTS of that matrix and the
 *     buffer must span rows*ld elements.  Data pointers must be 16-byte aligned and
 *     ld*sizeof(element) must be a multiple of 16, else HALO_EALIGN.
 *   - Arguments are checked on the host before anything is launched; a failed check returns an
 *     error code and enqueues nothing.  HIP launch failures return HALO_EHIP.
 *   - Same inputs give bit-identical outputs (no result depends on atomic ordering).
 *   - A Hadamard block size is 0 (no rotation) or a power of two in [2, 4096] (right-hand, along
 *     the contiguous axis) / [2, 65536] (left-hand, along the strided axis) that divides the axis
 *     length; the rotation is block-diagonal, I (x) H_block, when the block is shorter than the
 *     axis.  H_block is the normalised Walsh-Hadamard matrix of the recursion H_d = H_2 (x) H_{d/2}
 *     (Section 2, "Hadamard Transformations"); its butterflies run in ascending stride order
 *     in fp32 and the 1/sqrt(block) factor is applied once at the end.
 *   - A right-hand block may also be 28 * 2^n with 64 <= 2^n <= 512 (1792, 3584, 7168, 14336), dividing a row of at
 *     most 14336 elements: the Kronecker construction H_block = H_{2^n} (x) H_28 of the same section for dimensions
 *     that are not powers of two (14336 = 512 * 28).  Element i * 28 + j of a block has index i into the Walsh-Hadamard
 *     factor and j into H_28, the symmetric Hadamard matrix of order 28 of Paley's second construction from the
 *     quadratic character chi modulo 13: with C = [[0, 1^T], [1, (chi(i - j))]] of order 14, every 0 of C becomes
 *     [[1, -1], [-1, -1]] and every entry +-1 becomes +-[[1, 1], [1, -1]].  Arithmetic, all fp32: each run of 28
 *     consecutive elements x becomes x H_28 (every output a running sum over the 28 terms in ascending index order),
 *     then the butterflies over i in ascending stride order, then one multiply by 1/sqrt(block).  Other sizes, the
 *     left-hand axis and halo_mx6_quant take power-of-two blocks only (HALO_ESHAPE / HALO_EUNSUPPORTED).
 */
#ifndef HALO_H
#define HALO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HALO_OK = 0,
    HALO_EINVAL = 1,        /* null pointer, negative size, unknown enum value            */
    HALO_ESHAPE = 2,        /* sizes that do not fit together (block does not divide, ld) */
    HALO_EALIGN = 3,        /* pointer or leading dimension not 16-byte aligned           */
    HALO_EWORKSPACE = 4,    /* workspace missing or smaller than *_workspace_bytes()      */
    HALO_EUNSUPPORTED = 5,  /* valid request this build has no kernel for                 */
    HALO_EHIP = 6           /* a HIP call failed                                          */
} halo_status;

typedef enum { HALO_BF16 = 0, HALO_F32 = 1 } halo_dtype;
typedef enum { HALO_LEVEL0 = 0, HALO_LEVEL1 = 1, HALO_LEVEL2 = 2 } halo_level;
/* Granularity of the symmetric absmax scales: one per row of the GEMM operand (this library's default), or one per
 * tensor, the quantiser the paper itself uses (Section 4 setup; Appendix "HALO Levels for FFT"). */
typedef enum { HALO_SCALE_PER_ROW = 0, HALO_SCALE_PER_TENSOR = 1 } halo_scale_mode;

typedef enum {
    HALO_QUANT_ROWS = 0,    /* one scale per row of `in`; codes keep the layout of `in`            */
    HALO_QUANT_COLS_T = 1   /* one scale per column of `in`; codes are written TRANSPOSED [cols x rows] */
} halo_axis;

const char* halo_status_string(halo_status s);
int halo_version(void);

/* ---------------------------------------------------------------------------------------------
 * halo_hadamard_quant: rotate -> fold -> absmax -> INT8.       (Section 2: h(A) = A H, h'(A) = H^T A;
 * Section 4 setup: symmetric round-to-nearest quantiser; Table "HALO levels": (XH)_Q, (WH)_Q, (E_Y)_Q,
 * (H E_Y)_Q, (E_Y^T)_Q.)
 *
 *   in            [rows x cols], bf16 or fp32, leading dimension ld_in.
 *   had_block     right-hand rotation along each row (0 = none).
 *   had_block_left left-hand rotation down each column (0 = none).  Needs workspace.
 *   fold          optional fp32 vector multiplied into the rotated values before the absmax; it is
 *                 indexed along the axis the scales do NOT run over (length cols for
 *                 HALO_QUANT_ROWS, length rows for HALO_QUANT_COLS_T).  This is how the saved per-row
 *                 scales of (WH)_Q / (XH)_Q enter the backward GEMMs.  NULL = none.
 *   HALO_QUANT_ROWS:   v = rotate(in) * fold[k];  amax_r = max_k |v[r,k]|;
 *                      out_q[r*ld_q + k] = rint(v * (127/amax_r)), out_scale[r] = amax_r/127
 *                      (amax_r == 0: codes 0, scale 1).
 *   HALO_QUANT_COLS_T: v = in * fold[r];  amax_k = max_r |v[r,k]|;
 *                      out_q[k*ld_q + r] = rint(v * (127/amax_k)), out_scale[k] = amax_k/127.
 *                      Rotations are not available on this axis (HALO_EUNSUPPORTED).
 *   out_q         int8, leading dimension ld_q (>= cols, resp. >= rows).
 *   out_scale     fp32, one per row (resp. per column).
 *   workspace     device scratch of at least halo_hadamard_quant_workspace_bytes(...) bytes
 *                 (may be NULL when that is 0).
 * rows == 0 or cols == 0 is a no-op returning HALO_OK.
 */
size_t halo_hadamard_quant_workspace_bytes(int64_t rows, int64_t cols, halo_axis axis,
                                           int32_t had_block_left);

halo_status halo_hadamard_quant(const void* in, halo_dtype in_dt, int64_t rows, int64_t cols,
                                int64_t ld_in, halo_axis axis, int32_t had_block,
                                int32_t had_block_left, const float* fold, int8_t* out_q,
                                int64_t ld_q, float* out_scale, void* workspace,
                                size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * halo_hadamard_quant_tensor: rotate -> absmax of the WHOLE tensor -> INT8, the paper's quantiser (Section 4 setup:
 * "tensor-wise symmetric quantization"; Table "HALO levels").  Arguments as in halo_hadamard_quant, without a fold
 * (a scalar scale factors out of the integer sums, so nothing has to be folded in):
 *      amax = max |rotate(in)|;   codes = rint(rotate(in) * (127/amax));   scale = amax/127  (amax == 0: codes 0, scale 1)
 * out_scale receives that one scale in EVERY entry (rows entries for HALO_QUANT_ROWS, cols for HALO_QUANT_COLS_T), so
 * that every consumer of per-row scales works unchanged.  Two passes over the input (absmax, then quantise):
 * 2 + 2 bytes read and 1 byte written per element.  Workspace: halo_hadamard_quant_tensor_workspace_bytes(...).
 */
size_t halo_hadamard_quant_tensor_workspace_bytes(int64_t rows, int64_t cols, halo_axis axis, int32_t had_block_left);

halo_status halo_hadamard_quant_tensor(const void* in, halo_dtype in_dt, int64_t rows, int64_t cols, int64_t ld_in,
                                       halo_axis axis, int32_t had_block, int32_t had_block_left, int8_t* out_q,
                                       int64_t ld_q, float* out_scale, void* workspace, size_t workspace_bytes,
                                       void* stream);

/* ---------------------------------------------------------------------------------------------
 * halo_quant_dual: both quantisations of the output gradient E that levels 0 and 1 need, from one tiling of E.
 * (Table "HALO levels": (E_Y)_Q for the E product and (E_Y^T)_Q for the G product.)
 *
 *   out_q  [rows x cols] = codes of  Q_row( in[r,k] * fold_cols[k] ),  row_scale[rows]
 *   out_qT [cols x rows] = codes of  Q_row( (in[r,k] * fold_rows[r])^T ),  col_scale[cols]
 * i.e. exactly what halo_hadamard_quant(HALO_QUANT_ROWS, fold = fold_cols) and
 * halo_hadamard_quant(HALO_QUANT_COLS_T, fold = fold_rows) produce, bit for bit, with E read twice instead of
 * three times and three kernels instead of five.  in is bf16; fold vectors are fp32 and may be NULL.
 * workspace: halo_quant_dual_workspace_bytes(rows, cols) bytes (partial maxima per 32 x 256 tile).
 */
size_t halo_quant_dual_workspace_bytes(int64_t rows, int64_t cols);

halo_status halo_quant_dual(const void* in, int64_t rows, int64_t cols, int64_t ld_in, const float* fold_cols,
                            const float* fold_rows, int8_t* out_q, int64_t ld_q, float* row_scale,
                            int8_t* out_qT, int64_t ld_qT, float* col_scale, void* workspace,
                            size_t workspace_bytes, void* stream);

/* halo_quant_dual for callers that cannot allocate or bring a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments (minus the workspace), same kernels and bit-identical
 * results; the partial maxima live in an array built into the library
 * (halo_quant_dual_static_max_workspace_bytes() bytes, 8 MiB, one copy per GPU, held until the process ends).  The
 * call allocates nothing and frees nothing.  Sizes whose halo_quant_dual_workspace_bytes(rows, cols) exceeds that
 * array are refused with HALO_EWORKSPACE.  All calls on one GPU share the array: calls that may overlap in time on one
 * GPU (different streams, different host threads) race and must be serialised by the caller; halo_quant_dual with
 * separate workspaces has no such restriction. */
size_t halo_quant_dual_static_max_workspace_bytes(void);

halo_status halo_quant_dual_static(const void* in, int64_t rows, int64_t cols, int64_t ld_in, const float* fold_cols,
                                   const float* fold_rows, int8_t* out_q, int64_t ld_q, float* row_scale,
                                   int8_t* out_qT, int64_t ld_qT, float* col_scale, void* stream);

/* ---------------------------------------------------------------------------------------------
 * halo_gemm_i8: INT8 GEMM with int32 accumulation and a scaling epilogue.   (Section 2, Eqs. 1a-1c on
 * quantised operands; Table "HALO levels".)
 *
 *   acc[i,j] = sum_k A[i,k] * opB[k,j]          exact in int32 (caller keeps 127*127*K < 2^31)
 *   C[i,j]   = (float(acc[i,j]) * row_scale[i]) * col_scale[j]      rounded to c_dt
 *
 *   A        int8 [M x K], leading dimension lda (K contiguous).
 *   B        transB != 0: int8 [N x K], ldb  (K contiguous; C = A B^T, the forward product)
 *            transB == 0: int8 [K x N], ldb  (K strided;    C = A B,   both backward products)
 *   K        must be a multiple of 16 (HALO_ESHAPE otherwise); M, N arbitrary.
 *   row_scale [M], col_scale [N]   fp32, each may be NULL (= 1).
 *   C        bf16 or fp32 [M x N], ldc; may be NULL if only acc_out is wanted.
 *   acc_out  optional int32 [M x N], ld_acc: the raw accumulators.
 * At least one of C / acc_out must be non-NULL.  M, N or K == 0: no-op (K == 0 writes zeros).
 */
halo_status halo_gemm_i8(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb, int transB,
                         int64_t M, int64_t N, int64_t K, const float* row_scale,
                         const float* col_scale, void* C, halo_dtype c_dt, int64_t ldc,
                         int32_t* acc_out, int64_t ld_acc, void* stream);

/* Tile configurations of the INT8 GEMM: macro tile M x N x K-step (bytes), wavefronts per workgroup.  They differ in
 * speed only, the results are identical.  HALO_GEMM_AUTO lets the library choose by shape.  A configuration whose
 * K step does not divide K is refused with HALO_ESHAPE (the staged one takes any K that is a multiple of 16). */
typedef enum {
    HALO_GEMM_AUTO = -1,
    HALO_GEMM_256x256x64 = 0,        /* 8 wavefronts, four-stage global->LDS ring                  */
    HALO_GEMM_256x256x128 = 1,       /* 8 wavefronts, two-stage ring                               */
    HALO_GEMM_256x128x128 = 2,       /* 8 wavefronts, three-stage ring                             */
    HALO_GEMM_128x128x64 = 3,        /* 4 wavefronts, four-stage ring                              */
    HALO_GEMM_STAGED_128x128x64 = 4  /* 4 wavefronts, register-staged, zero-fills a ragged K       */
} halo_gemm_config;

/* One product described by a struct: every field means what the argument of the same name means in halo_gemm_i8;
 * `config` is a halo_gemm_config. */
typedef struct halo_gemm_desc {
    const int8_t* A; int64_t lda;
    const int8_t* B; int64_t ldb;
    int32_t transB;
    int64_t M, N, K;
    const float* row_scale; const float* col_scale;
    void* C; int32_t c_dt /* halo_dtype */; int64_t ldc;
    int32_t* acc_out; int64_t ld_acc;
    int32_t config /* halo_gemm_config */;
} halo_gemm_desc;

/* halo_gemm_i8 with the tile configuration under the caller's control (measurements, tests of every configuration). */
halo_status halo_gemm_i8_desc(const halo_gemm_desc* g, void* stream);

/* Two independent products in one launch: same semantics and bit-identical results as two halo_gemm_i8_desc calls (in
 * either order).  halo_linear_bwd uses it for E_X = E W and G = E^T X, where the tail and the epilogue of one product
 * overlap the main loop of the other and the smaller one cannot leave compute units idle.  Products with a
 * K-contiguous B, a K that is not a multiple of 64, different configurations, a configuration other than AUTO,
 * 256x256x64 or 128x128x64, or an empty shape are simply run one after the other. */
halo_status halo_gemm_i8_pair(const halo_gemm_desc* g1, const halo_gemm_desc* g2, void* stream);

/* Measurement aid: the INT8 MFMA rate this machine sustains on given operand bytes.  256 workgroups of 8 wavefronts
 * each issue iters x 16 v_mfma_i32_32x32x32_i8 on the 4096 operand bytes at `operands` (device, 16-byte aligned) with
 * nothing else in the loop: 256 * 8 * iters * 16 * 65536 integer operations.  The rate depends on the operand data
 * (the clock drops as more multiplier bits toggle), which is why the throughput of halo_gemm_i8 is reported against
 * this figure next to the published peak (Section 4, "Speedup Analysis", measures against an ideal layer likewise).
 * `sink` is an optional int32 the kernel may write (it keeps the loop from being optimised away). */
halo_status halo_mfma_i8_probe(const int8_t* operands, int32_t iters, int32_t* sink, void* stream);

/* ---------------------------------------------------------------------------------------------
 * MXFP6 variant of the forward product (Section 4 "Setup": FP6 E3M2 elements; Appendix "MXFP6": microscaling; the
 * paper names the formats only, the arithmetic below is the public OCP Microscaling Formats specification's).
 *
 * halo_mx6_quant: rotate -> per-block scale -> FP6.   in bf16 [rows x cols] (ld_in elements), cols a multiple of 32.
 *   v = in (I (x) H_had_block) as in halo_hadamard_quant.  Every block of 32 consecutive elements of a row shares the
 *   scale 2^(floor(log2(max |v|)) - 4), stored as an E8M0 byte (exponent + 127; an all-zero block: 127) in
 *   out_scales[r * ld_scales + k/32].  Elements are v / scale rounded to the nearest E3M2 value (1 sign, 3 exponent
 *   bits with bias 3, 2 mantissa bits; ties to the even mantissa, saturating at +-28, zero stored as +0) and packed
 *   least-significant element first, 24 bytes per block, in out_codes[r * ld_codes + (k/32) * 24 ...] (ld_codes in
 *   bytes, a multiple of 8).
 * halo_gemm_mx6: C[M x N] = A[M x K] B[N x K]^T on such operands (both K-contiguous, K a multiple of 128, leading
 *   dimensions of the code matrices multiples of 16 bytes, of the scale matrices multiples of 4), fp32
 *   accumulation in the matrix cores (v_mfma_scale_f32_16x16x128_f8f6f4), C bf16 or fp32 with leading dimension ldc
 *   (elements).  The accumulation order is the hardware's: results agree with an exact evaluation to fp32 rounding
 *   of the partial sums, not bit for bit.
 */
halo_status halo_mx6_quant(const void* in, int64_t rows, int64_t cols, int64_t ld_in, int32_t had_block,
                           uint8_t* out_codes, int64_t ld_codes, uint8_t* out_scales, int64_t ld_scales, void* stream);

halo_status halo_gemm_mx6(const uint8_t* A, int64_t lda, const uint8_t* scales_a, int64_t ld_scales_a, const uint8_t* B,
                          int64_t ldb, const uint8_t* scales_b, int64_t ld_scales_b, int64_t M, int64_t N, int64_t K,
                          void* C, halo_dtype c_dt, int64_t ldc, void* stream);

/* ---------------------------------------------------------------------------------------------
 * halo_dequant_unrotate: the tail of both backward products.   (Table "HALO levels": the trailing H^T
 * of  (E_Y)_Q (WH)_Q H^T  and  (E_Y^T)_Q (XH)_Q H^T,  and the leading H^T of level 2.)
 *
 *   T[r,k] = (float(acc[r,k]) * row_scale[r]) * tensor_scale[0];
 *   T <- (I (x) H_had_block_left)^T T          (left-hand, if had_block_left: the table does not bracket the two
 *                                               un-rotations; the left-hand one is taken first);
 *   T <- T (I (x) H_had_block)                 (right-hand, if had_block);   out = T rounded to out_dt.
 *
 *   acc int32 [rows x cols] ld_acc; row_scale fp32 [rows] or NULL; tensor_scale: device pointer to ONE fp32 or NULL
 *   (the saved operand's scale in the one-scale-per-tensor mode); out bf16/fp32 [rows x cols] ld_out.
 *   workspace: halo_dequant_unrotate_workspace_bytes(rows, cols, had_block_left) bytes.
 */
size_t halo_dequant_unrotate_workspace_bytes(int64_t rows, int64_t cols, int32_t had_block_left);

halo_status halo_dequant_unrotate(const int32_t* acc, int64_t ld_acc, int64_t rows, int64_t cols,
                                  const float* row_scale, const float* tensor_scale, int32_t had_block,
                                  int32_t had_block_left, void* out, halo_dtype out_dt, int64_t ld_out, void* workspace,
                                  size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * The layer.  (Table "HALO levels"; Section 3.2 Steps 1-3; Section 3.3.)
 *
 *   level 0:  F = X_Q W_Q^T          E = (E_Y)_Q W_Q                     G = (E_Y^T)_Q X_Q
 *   level 1:  F = (XH)_Q (WH)_Q^T    E = (E_Y)_Q (WH)_Q H^T              G = (E_Y^T)_Q (XH)_Q H^T
 *   level 2:  F = (XH)_Q (WH)_Q^T    E = H^T (H E_Y)_Q (WH)_Q H^T        G = (E_Y^T)_Q (XH)_Q H^T
 *
 *   b, m, n        tokens, in-features, out-features.  m and n multiples of 16, b a multiple of 16.
 *   had_block_m    right-hand block over m; 0 = largest power of two dividing m, capped at 4096 (a Kronecker block
 *                  28 * 2^n has to be asked for by its size).
 *   had_block_b    left-hand block over b (level 2 only); 0 = largest power of two dividing b.
 *   out_dt         type of Y, E_X and G.
 *   scale_mode     HALO_SCALE_PER_ROW: one scale per row of every GEMM operand; the saved scale vectors are folded
 *                  into E before E is quantised for the backward products.  HALO_SCALE_PER_TENSOR: the paper's
 *                  quantiser, one scale per tensor; s_x / s_w hold that scale in every entry; E is quantised as it is
 *                  (left-rotated at level 2) and the two scales multiply the accumulators afterwards:
 *                  E_X = ((acc * s_e) * s_w) ...,  G = ((acc * s_g) * s_x) ...   Needs the workspace in the forward
 *                  pass too.
 */
typedef struct halo_linear_desc {
    int64_t b, m, n;
    int32_t level;          /* halo_level */
    int32_t had_block_m;
    int32_t had_block_b;
    int32_t out_dt;         /* halo_dtype */
    int32_t scale_mode;     /* halo_scale_mode */
} halo_linear_desc;

/* Bytes of device scratch halo_linear_bwd needs (and halo_linear_fwd in the per-tensor mode). */
size_t halo_linear_workspace_bytes(const halo_linear_desc* desc);

/* Forward.  X bf16 [b x m] (ld m), W bf16 [n x m] (ld m), Y [b x n] (ld n).
 * Xq int8 [b x m], s_x fp32 [b], Wq int8 [n x m], s_w fp32 [n] are the saved-for-backward tensors
 * (Section 3.2 Step 2), always caller-allocated.  If X is NULL, Xq/s_x are taken as already holding
 * (XH)_Q (e.g. q/k/v share one activation); likewise W NULL -> Wq/s_w are inputs. */
halo_status halo_linear_fwd(const halo_linear_desc* desc, const void* X, const void* W, void* Y,
                            int8_t* Xq, float* s_x, int8_t* Wq, float* s_w, void* workspace,
                            size_t workspace_bytes, void* stream);

/* Backward.  E bf16 [b x n] (ld n); EX [b x m] and G [n x m] in desc->out_dt; either may be NULL to
 * skip that product (not both). */
halo_status halo_linear_bwd(const halo_linear_desc* desc, const void* E, const int8_t* Xq,
                            const float* s_x, const int8_t* Wq, const float* s_w, void* EX, void* G,
                            void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * HALO-PEFT: a LoRA-style module on a frozen, quantised weight.  (Section 3.3 "Parameter Efficient Fine Tuning";
 * Appendix "LoRA-style Linear Module and HALO for PEFT".)
 *
 *   Y   = (XH)_Q (WH)_Q^T  +  (X U^T) V^T
 *   E_X = H^T (H E_Y)_Q (WH)_Q H^T  +  (E_Y V) U            (the forms of desc->level; the paper uses level 2)
 *   G_V = E_Y^T (X U^T)        G_U = (V^T E_Y^T) X           (adapter gradients; there is no G for the frozen W)
 *
 * The frozen weight is rotated and quantised ONCE, before fine-tuning, with
 * halo_hadamard_quant(W, HALO_BF16, n, m, m, HALO_QUANT_ROWS, had_block_m, 0, NULL, Wq, m, s_w, ...); Wq int8 [n x m] and
 * s_w fp32 [n] are inputs here.  U bf16 [rank x m] (ld m) and V bf16 [n x rank] (ld rank) are the adapters; any LoRA
 * scaling factor is folded into V by the caller.  The low-rank products are the "high precision" part: bf16 inputs,
 * fp32 accumulation, the intermediates T = X U^T and S = E_Y V kept in fp32, and the low-rank term is added to the fp32
 * value of the quantised branch before the single rounding to desc->out_dt.  (For E_X it is added in the rotated
 * domain, as (H S)(U H), and un-rotated together with the product: equal to S U up to fp32 rounding.)
 *
 *   rank          a multiple of 8, at most 64.
 *   desc          as for halo_linear_*; scale_mode must be HALO_SCALE_PER_ROW; m and n multiples of 64.
 *   T             fp32 [b x rank] (dense): written by the forward pass, read by the backward pass (for G_V).
 *   G_U, G_V      fp32 [rank x m] and [n x rank], dense.
 *   workspace     halo_peft_workspace_bytes(desc, rank) bytes of device memory, 16-byte aligned; nothing in it is
 *                 carried from the forward to the backward call.
 * All pointers are device pointers, 16-byte aligned.  Errors as elsewhere: HALO_EINVAL (null / bad enum), HALO_ESHAPE,
 * HALO_EALIGN, HALO_EWORKSPACE, HALO_EUNSUPPORTED (per-tensor scales, rank > 64), HALO_EHIP.
 */
size_t halo_peft_workspace_bytes(const halo_linear_desc* desc, int32_t rank);

halo_status halo_peft_fwd(const halo_linear_desc* desc, int32_t rank, const void* X, const int8_t* Wq, const float* s_w,
                          const void* U, const void* V, void* Y, float* T, void* workspace, size_t workspace_bytes,
                          void* stream);

/* EX [b x m] in desc->out_dt; any of EX, GU, GV may be NULL to skip it (not all three).  X is read for G_U only, T for
 * G_V only, Wq / s_w / U for E_X only. */
halo_status halo_peft_bwd(const halo_linear_desc* desc, int32_t rank, const void* E, const void* X, const float* T,
                          const int8_t* Wq, const float* s_w, const void* U, const void* V, void* EX, float* GU, float* GV,
                          void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HALO_H */
