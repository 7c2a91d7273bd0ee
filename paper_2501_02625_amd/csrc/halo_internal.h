// Internal declarations shared by the HIP translation units of libhalo (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "halo.h"

namespace halo {

enum InKind { IN_BF16 = 0, IN_F32 = 1, IN_I32 = 2 };
enum OutKind { OUT_Q8 = 0, OUT_BF16 = 1, OUT_F32 = 2, OUT_MX6 = 3 };

// ---- row transform: [pre-scale] -> right-hand FWHT -> [fold] -> {absmax+INT8 | bf16 | fp32} ----
struct RowArgs {
    const void* in;
    int64_t ld_in;
    int64_t rows, cols;
    const float* pre_scale;  // IN_I32 only: per-row multiplier, may be null
    const float* fold;       // per-column multiplier, may be null
    void* out;
    int64_t ld_out;
    float* out_scale;        // OUT_Q8 only
    int log_block;           // log2 of the Hadamard block, 0 = no rotation
    int kron_m;              // 0, or 28: the block is 28 * 2^log_block elements, rotated by H_{2^log_block} (x) H_28
    float in_mul;            // IN_F32 only: every element is multiplied by this once when it is loaded; 0 = no multiply
    int left_top;            // launch_row_left_top only: number of top strides of the left-hand rotation still to run (1..5)
    // One scale per tensor (OUT_Q8 only): amax_only writes each row's absmax to out_scale and no codes; given_amax
    // (device scalar) replaces the row's own absmax.  post_scale (IN_I32 only, device scalar) is multiplied in after
    // pre_scale.  All three apply to both matrices of a batched launch.
    int amax_only;
    const float* given_amax;
    const float* post_scale;
    // OUT_MX6 only (bf16 input, cols a multiple of 32): `out` receives the packed FP6 E3M2 codes (24 bytes per block of
    // 32 elements, ld_out in BYTES per row), mx_scales the E8M0 scale bytes [rows x cols/32] with ld_mx_scales bytes per row.
    uint8_t* mx_scales;
    int64_t ld_mx_scales;
    // Optional second matrix handled by the same launch (same cols, leading dimensions, fold and block; its own
    // row count and buffers): rows2 == 0 means none.  Saves one launch ramp/tail when two independent tensors get
    // the same treatment (X and W in the forward pass, the two accumulators of the backward pass).
    int64_t rows2;
    const void* in2;
    const float* pre_scale2;
    void* out2;
    float* out_scale2;
    const float* given_amax2;    // the second matrix's own given_amax / post_scale; null: those of the first
    const float* post_scale2;
};
// Largest row length the row kernels accept.
constexpr int64_t kMaxRowCols = 32768;
hipError_t launch_row_transform(const RowArgs& a, InKind in, OutKind out, hipStream_t s);
// Kronecker blocks (kron_m == 28): true if a row of `cols` elements can be rotated in blocks of `block` = 28 * 2^n
// elements (64 <= 2^n <= 512, block divides cols, cols <= 14336).  launch_row_transform forwards such launches.
// The end of a left+right un-rotation in one kernel.  `in` is fp32 [rows x cols] on which all strides of a left-hand
// rotation of block 256 << left_top have run except the top left_top ones; the kernel runs those (the 2^left_top rows
// they mix sit in the wavefronts of one workgroup and meet in LDS), multiplies by in_mul, un-rotates each row in blocks
// of 2^log_block and stores bf16 / fp32.  row_left_top_ok: the shapes it takes (log_block 9..12 dividing cols,
// left_top 1..4, or 5 with log_block <= 11, rows a multiple of the left block).
bool row_left_top_ok(int64_t rows, int64_t cols, int log_block, int left_top);
hipError_t launch_row_left_top(const RowArgs& a, OutKind out, hipStream_t s);
bool row_kron_shape_ok(int64_t cols, int64_t block);
hipError_t launch_row_kron(const RowArgs& a, InKind in, OutKind out, hipStream_t s);

// ---- left-hand (strided axis) FWHT: all stages of block 2^log_block, ascending, possibly several passes ----
// in/out may alias when in_kind == out_kind == fp32.  tmp (fp32 [rows x ld_tmp]) is used when more than one
// pass is needed and in/out cannot carry fp32 intermediates.
struct ColFwhtArgs {
    const void* in;
    InKind in_kind;          // IN_BF16 or IN_F32
    int64_t ld_in;
    void* out;
    OutKind out_kind;        // OUT_F32 or OUT_BF16
    int64_t ld_out;
    float* tmp;
    int64_t ld_tmp;
    int64_t rows, cols;
    int log_block;
    // IN_I32 input (accumulators of a product): element (r, k) enters as (float(in[r,k]) * row_scale[r]) * post_scale[0]
    // (either pointer may be null).  first_stage: the strides below 2^first_stage have been applied already.  skip_norm:
    // leave the 1/sqrt(block) multiply to the caller.
    const float* row_scale;
    const float* post_scale;
    int first_stage;
    int skip_norm;
    // side_amax != null (bf16 input, log_block >= 6, first_stage 0): the first pass also accumulates, per column, the
    // absolute maximum of in[r, k] * side_fold[r] (side_fold may be null) over all rows into side_amax[cols], as bit
    // patterns of non-negative floats; the caller zeroes it beforehand (launch_zero_u32).
    const float* side_fold;
    uint32_t* side_amax;
};
hipError_t launch_col_fwht(const ColFwhtArgs& a, hipStream_t s);
hipError_t launch_zero_u32(uint32_t* p, int64_t n, hipStream_t s);

// ---- column-wise absmax quantiser with transposed output (E^T)_Q ----
struct ColQuantArgs {
    const void* in;          // bf16 [rows x cols]
    int64_t ld_in;
    int64_t rows, cols;
    const float* fold;       // per-row multiplier, may be null
    int8_t* out_q;           // [cols x rows]
    int64_t ld_q;
    float* out_scale;        // [cols]
    float* amax_ws;          // [cols] scratch: column absmax accumulated as bit patterns
};
hipError_t launch_col_quant_t(const ColQuantArgs& a, hipStream_t s);
// The same with the columns' absolute maxima already in a.amax_ws (bit patterns, from the side output of launch_col_fwht).
hipError_t launch_col_quant_t_ready(const ColQuantArgs& a, hipStream_t s);
// The same with one given absmax (device scalar) for every column instead of the columns' own: the tensor-wide scale.
hipError_t launch_col_quant_t_given(const ColQuantArgs& a, const float* given_amax, hipStream_t s);
// out[0] = max(in[0..n-1]) (n >= 1, non-negative values).  With in2: out2[0] = max(in2[0..n2-1]) in the same launch.
hipError_t launch_reduce_max(const float* in, int64_t n, float* out, hipStream_t s, const float* in2 = nullptr,
                             int64_t n2 = 0, float* out2 = nullptr);

// ---- both quantisations of E for the backward pass from one tiling (rows for E_X, transposed columns for G) ----
struct DualQuantArgs {
    const void* in;          // bf16 [rows x cols]
    int64_t ld_in;
    int64_t rows, cols;
    const float* fold_c;     // per-column multiplier of the row-wise quantisation (saved weight scales), may be null
    const float* fold_r;     // per-row multiplier of the column-wise quantisation (saved activation scales), may be null
    int8_t* out_q;           // [rows x cols]
    int64_t ld_q;
    float* row_scale;        // [rows]
    int8_t* out_qt;          // [cols x rows]
    int64_t ld_qt;
    float* col_scale;        // [cols]
    float* amax_ws;          // dual_quant_workspace_floats(rows, cols) floats of scratch
};
size_t dual_quant_workspace_floats(int64_t rows, int64_t cols);
hipError_t launch_dual_quant(const DualQuantArgs& a, hipStream_t s);
// The same with the partial maxima in a file-scope device array instead of a.amax_ws (which is ignored): no allocation,
// no workspace argument.  Sizes whose partial maxima exceed kStaticScratchBytes are refused by the caller.
constexpr size_t kStaticScratchBytes = size_t(8) << 20;
hipError_t launch_dual_quant_static(DualQuantArgs a, hipStream_t s);

// ---- INT8 GEMM ----
struct GemmArgs {
    const int8_t* A;
    int64_t lda;
    const int8_t* B;
    int64_t ldb;
    int transB;
    int64_t M, N, K;
    const float* row_scale;
    const float* col_scale;
    void* C;
    int c_is_f32;
    int64_t ldc;
    int32_t* acc_out;
    int64_t ld_acc;
    int config;              // halo_gemm_config: -1 = chosen by shape
    // left_stages == 8 (256-row tiles only, C fp32, M a multiple of 256): the epilogue scales the accumulators,
    // (float(acc) * row_scale[row]) * post_scale[0], and then runs the eight lowest strides (1 .. 128 rows) of a left-hand
    // Walsh-Hadamard rotation down each column of the tile, unnormalised, before it stores C.
    int left_stages;
    const float* post_scale;
    // lr_rank > 0 (C required, no acc_out; K-step configurations only): the epilogue adds a low-rank product to the
    // scaled accumulators before anything else happens to them,
    //   value(row, col) = ((float(acc) * row_scale[row]) * col_scale[col]) * post_scale + sum_k lr_a[row, k] * lr_b[k, col]
    // with lr_a fp32 [M x lr_rank] and lr_b [N x lr_rank] (fp32, or bf16 with lr_b_bf16), both dense, 16-byte aligned,
    // lr_rank a multiple of 8; the sum is accumulated in fp32.
    int lr_rank;
    const float* lr_a;
    const void* lr_b;
    int lr_b_bf16;
};
constexpr int kMaxLowRank = 64;
hipError_t launch_gemm_i8(const GemmArgs& a, hipStream_t s);
hipError_t launch_gemm_i8_pair(const GemmArgs& a1, const GemmArgs& a2, hipStream_t s);
// True if `cfg` names a tile configuration that can run a product with reduction length K.
bool gemm_config_valid(int cfg, int64_t K);
// 256 workgroups x 8 wavefronts x iters x 16 MFMAs on the 4 KB of operand bytes at `operands`.
hipError_t launch_mfma_i8_probe(const int8_t* operands, int iters, int32_t* sink, hipStream_t s);

// ---- low-rank side branch (LoRA adapters next to the quantised products) ----
// out fp32 [rows x rank] = in bf16 [rows x K] times the thin bf16 operand: [rank x K] (its transpose is applied), or
// [K x rank] with k_major.  K a multiple of 64.
hipError_t launch_lr_down(const void* in, int64_t ld_in, const void* thin, int k_major, int64_t ld_b, float* out, int64_t rows,
                          int64_t K, int rank, hipStream_t s);
// out = big^T small: big bf16 [rows x wide], small fp32 [rows x rank] dense; out fp32 [wide x rank], or its transpose
// [rank x wide] with transpose_out.  part: lr_grad_workspace_floats(rows, wide, rank) floats of scratch.
struct LrGradArgs {
    const void* big;
    int64_t ld_big;
    const float* small;
    float* out;
    int transpose_out;
    float* part;
    int64_t wide;
};
size_t lr_grad_workspace_floats(int64_t rows, int64_t wide, int rank);
// The rotated forms of the thin operands of the E_X epilogue:  u_rot fp32 [m x rank] = the TRANSPOSE of u bf16
// [rank x m] with every row rotated in blocks of block_m (2^n, or 28 * 2^n; <= 1: only widened), and sm_rot fp32
// [b x rank] = sm fp32 [b x rank] with every column rotated in blocks of block_b (a power of two).  Either pair may be null.
struct LrRotArgs {
    const void* u;
    float* u_rot;
    int64_t m, block_m;
    const float* sm;
    float* sm_rot;
    int64_t b, block_b;
};
bool lr_row_fwht_shape_ok(int64_t cols, int64_t block);
bool lr_col_fwht_shape_ok(int64_t rows, int64_t block);
// Everything small of the backward pass of the low-rank branch in two launches: the gradient products a and b (either or
// both may be null), then the sums over their token ranges together with the rotations `rot` (may be null).
hipError_t launch_lr_backward_small(const LrGradArgs* a, const LrGradArgs* b, int64_t rows, int rank, const LrRotArgs* rot,
                                    hipStream_t s);

// ---- MXFP6 GEMM: C[M x N] = A[M x K] B[N x K]^T on packed E3M2 codes with one E8M0 scale per 32 elements along K ----
struct Mx6GemmArgs {
    const uint8_t* A; int64_t lda;          // packed codes, bytes per row
    const uint8_t* SA; int64_t ldsa;        // scale bytes, bytes per row
    const uint8_t* B; int64_t ldb;
    const uint8_t* SB; int64_t ldsb;
    int64_t M, N, K;                        // K a multiple of 128
    void* C; int c_is_f32; int64_t ldc;     // elements
};
hipError_t launch_gemm_mx6(const Mx6GemmArgs& a, hipStream_t s);

// fp32 -> bf16, round to nearest even, on the hardware conversion (v_cvt_pk_bf16_f32: two values per instruction).
typedef __bf16 halo_bf16x2 __attribute__((ext_vector_type(2)));
typedef float halo_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const halo_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, halo_bf16x2));
}
__device__ __forceinline__ uint16_t bf16_bits(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

inline int ilog2_exact(int64_t v) {
    int l = 0;
    while ((int64_t(1) << l) < v) ++l;
    return l;
}
inline bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }

}  // namespace halo
