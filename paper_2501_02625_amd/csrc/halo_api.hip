// C ABI of libhalo: argument checking on the host, then kernel launches on the caller's stream.
#include <cmath>
#include <cstdint>

#include "halo_internal.h"

using namespace halo;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t v) { return (v + 255) & ~size_t(255); }
inline halo_status from_hip(hipError_t e) { return e == hipSuccess ? HALO_OK : HALO_EHIP; }

// Hadamard block check: 0, or a power of two in [2, cap] dividing `len`.
inline halo_status check_block(int32_t block, int64_t len, int64_t cap) {
    if (block < 0) return HALO_EINVAL;
    if (block == 0) return HALO_OK;
    if (block == 1 || !is_pow2(block)) return HALO_ESHAPE;
    if (block > cap) return HALO_EUNSUPPORTED;
    if (len % block != 0) return HALO_ESHAPE;
    return HALO_OK;
}

constexpr int64_t kMaxRightBlock = 4096;
constexpr int64_t kMaxLeftBlock = 65536;

// Right-hand Hadamard block: what check_block accepts up to 4096, or 28 * 2^n with 64 <= 2^n <= 512 dividing `len`,
// len <= 14336 (the Kronecker construction H_{2^n} (x) H_28).
inline halo_status check_right_block(int32_t block, int64_t len) {
    if (block > 0 && block % 28 == 0 && is_pow2(block / 28)) {
        if (len % block != 0) return HALO_ESHAPE;
        return row_kron_shape_ok(len, block) ? HALO_OK : HALO_EUNSUPPORTED;
    }
    return check_block(block, len, kMaxRightBlock);
}

inline void set_right_block(RowArgs& r, int32_t block) {
    if (block > 0 && !is_pow2(block)) {
        r.kron_m = 28;
        r.log_block = ilog2_exact(block / 28);
    } else {
        r.kron_m = 0;
        r.log_block = block ? ilog2_exact(block) : 0;
    }
}
constexpr int64_t kMaxDim = int64_t(1) << 22;   // rows / columns of any matrix argument

struct BwdWorkspace {
    size_t eq, s_e, eqt, s_g, amax, acc, acc_g, f32, tq, total;
};

inline bool acc_fits_int32(int64_t k) { return 127ll * 127ll * k < (1ll << 31); }

inline int32_t default_block(int64_t len, int64_t cap) {
    int64_t b = len & -len;
    if (b > cap) b = cap;
    return b >= 2 ? (int32_t)b : 0;
}

halo_status resolve_desc(const halo_linear_desc* d, int32_t* hm, int32_t* hb) {
    if (!d) return HALO_EINVAL;
    if (d->b < 0 || d->m < 0 || d->n < 0) return HALO_EINVAL;
    if (d->level < 0 || d->level > 2) return HALO_EINVAL;
    if (d->out_dt != HALO_BF16 && d->out_dt != HALO_F32) return HALO_EINVAL;
    if (d->scale_mode != HALO_SCALE_PER_ROW && d->scale_mode != HALO_SCALE_PER_TENSOR) return HALO_EINVAL;
    if (d->b > kMaxDim || d->m > kMaxDim || d->n > kMaxDim) return HALO_EUNSUPPORTED;
    if (d->b % 16 || d->m % 16 || d->n % 16) return HALO_ESHAPE;
    if (d->m > kMaxRowCols || d->n > kMaxRowCols) return HALO_EUNSUPPORTED;
    // every one of b, m, n is the reduction length of one of the three products: the largest possible sum of
    // products of codes, 127*127*K, must fit the int32 accumulator
    if (!acc_fits_int32(d->b) || !acc_fits_int32(d->m) || !acc_fits_int32(d->n)) return HALO_ESHAPE;
    *hm = 0;
    *hb = 0;
    if (d->level >= 1) {
        *hm = d->had_block_m ? d->had_block_m : default_block(d->m, kMaxRightBlock);
        halo_status st = check_right_block(*hm, d->m);
        if (st != HALO_OK) return st;
    }
    if (d->level >= 2) {
        *hb = d->had_block_b ? d->had_block_b : default_block(d->b, kMaxLeftBlock);
        halo_status st = check_block(*hb, d->b, kMaxLeftBlock);
        if (st != HALO_OK) return st;
    }
    return HALO_OK;
}

BwdWorkspace bwd_layout(const halo_linear_desc* d) {
    BwdWorkspace w{};
    size_t off = 0;
    const size_t b = (size_t)d->b, m = (size_t)d->m, n = (size_t)d->n;
    w.eq = off;   off += round256(b * n);
    w.s_e = off;  off += round256(b * 4);
    w.eqt = off;  off += round256(n * b);
    w.s_g = off;  off += round256(n * 4);
    w.amax = off; off += round256(dual_quant_workspace_floats(d->b, d->n) * 4);
    w.acc = off;  off += round256(b * m * 4);       // accumulators of the E product
    w.acc_g = off; off += round256(n * m * 4);      // accumulators of the G product
    w.f32 = off;
    if (d->level >= 2) off += round256(b * (m > n ? m : n) * 4);
    w.tq = off;                                     // scratch of the one-scale-per-tensor quantiser (without its left part)
    if (d->scale_mode == HALO_SCALE_PER_TENSOR) {
        const size_t longest = b > n ? b : n;
        off += round256((longest + 64) * 4) + round256(n * 4) + 1024;       // + a second vector's maximum (forward: X and W)
    }
    w.total = off;
    return w;
}

// Level 2: the low eight strides of the left-hand un-rotation of E_X can run in the epilogue of the E product when the
// left block covers whole 256-row tiles and the product can take the 256 x 256 configuration (K = n in 64-byte steps).
inline bool left_in_epilogue(int64_t b, int64_t n, int32_t hb) { return hb >= 256 && b % 256 == 0 && n % 64 == 0; }

// The rest of that un-rotation: t [b x m] fp32 holds the product after the eight low left-hand strides.  Either one
// kernel (top strides across the wavefronts of a workgroup, then each row's right-hand un-rotation), or the remaining
// strides in place and then the row kernel (1/sqrt(left block), right-hand un-rotation, conversion).
// first_stage: the left-hand strides below 2^first_stage have run already (8 after the GEMM epilogue that runs them, 0
// after a plain epilogue).
hipError_t finish_left_unrotation(float* t, int64_t b, int64_t m, int32_t hb, int32_t hm, void* out, halo_dtype odt,
                                  hipStream_t s, int first_stage = 8) {
    RowArgs r{};
    r.in = t; r.ld_in = m; r.rows = b; r.cols = m; r.out = out; r.ld_out = m;
    r.in_mul = (float)(1.0 / sqrt((double)hb));
    set_right_block(r, hm);
    const OutKind ok = odt == HALO_BF16 ? OUT_BF16 : OUT_F32;
    // up to four top strides left and a right-hand block of 512 .. 4096: one kernel does the rest
    const int top = ilog2_exact(hb) - 8;
    if (first_stage == 8 && r.kron_m == 0 && row_left_top_ok(b, m, r.log_block, top)) {
        r.left_top = top;
        return launch_row_left_top(r, ok, s);
    }
    ColFwhtArgs c{t, IN_F32, m, t, OUT_F32, m, t, m, b, m, ilog2_exact(hb)};
    c.first_stage = first_stage; c.skip_norm = 1;
    hipError_t e = launch_col_fwht(c, s);
    if (e != hipSuccess) return e;
    return launch_row_transform(r, IN_F32, ok, s);
}

// Scratch of the HALO-PEFT entry points (one layout for both directions).
struct PeftWorkspace {
    size_t xq, s_x, eq, s_e, c32, f32, s, sp, up, part, part_u, total;
};

PeftWorkspace peft_layout(const halo_linear_desc* d, int32_t rank) {
    PeftWorkspace w{};
    size_t off = 0;
    const size_t b = (size_t)d->b, m = (size_t)d->m, n = (size_t)d->n, r = (size_t)rank;
    w.xq = off;   off += round256(b * m);
    w.s_x = off;  off += round256(b * 4);
    w.eq = off;   off += round256(b * n);
    w.s_e = off;  off += round256(b * 4);
    w.c32 = off;  off += round256(b * m * 4);       // the E product in fp32, before its un-rotation
    w.f32 = off;
    if (d->level >= 2) off += round256(b * (m > n ? m : n) * 4);
    w.s = off;    off += round256(b * r * 4);
    w.sp = off;   off += round256(b * r * 4);
    w.up = off;   off += round256(r * m * 4);
    const size_t pn = lr_grad_workspace_floats(d->b, d->n, rank), pm = lr_grad_workspace_floats(d->b, d->m, rank);
    w.part = off; off += round256(pn * 4);          // partial sums of G_V
    w.part_u = off; off += round256(pm * 4);        // partial sums of G_U
    w.total = off;
    return w;
}

halo_status resolve_peft(const halo_linear_desc* d, int32_t rank, int32_t* hm, int32_t* hb) {
    halo_status st = resolve_desc(d, hm, hb);
    if (st != HALO_OK) return st;
    if (d->scale_mode != HALO_SCALE_PER_ROW) return HALO_EUNSUPPORTED;
    if (rank <= 0) return HALO_EINVAL;
    if (rank % 8) return HALO_ESHAPE;
    if (rank > kMaxLowRank) return HALO_EUNSUPPORTED;
    if (d->m % 64 || d->n % 64) return HALO_ESHAPE;       // both are reduction lengths of a K-step GEMM
    if (!lr_row_fwht_shape_ok(d->m, *hm)) return HALO_EUNSUPPORTED;
    return HALO_OK;
}

}  // namespace

extern "C" {

const char* halo_status_string(halo_status s) {
    switch (s) {
        case HALO_OK: return "ok";
        case HALO_EINVAL: return "invalid argument";
        case HALO_ESHAPE: return "sizes do not fit together";
        case HALO_EALIGN: return "pointer or leading dimension not 16-byte aligned";
        case HALO_EWORKSPACE: return "workspace missing or too small";
        case HALO_EUNSUPPORTED: return "not supported by this build";
        case HALO_EHIP: return "HIP call failed";
    }
    return "unknown status";
}

int halo_version(void) { return 2; }

// ------------------------------------------------------------------------------------------------
size_t halo_hadamard_quant_workspace_bytes(int64_t rows, int64_t cols, halo_axis axis, int32_t had_block_left) {
    if (rows <= 0 || cols <= 0) return 0;
    if (axis == HALO_QUANT_COLS_T) return round256((size_t)cols * 4);
    if (had_block_left > 0) return round256((size_t)rows * (size_t)cols * 4);
    return 0;
}

halo_status halo_hadamard_quant(const void* in, halo_dtype in_dt, int64_t rows, int64_t cols, int64_t ld_in,
                                halo_axis axis, int32_t had_block, int32_t had_block_left, const float* fold,
                                int8_t* out_q, int64_t ld_q, float* out_scale, void* workspace,
                                size_t workspace_bytes, void* stream) {
    if (rows < 0 || cols < 0) return HALO_EINVAL;
    if (in_dt != HALO_BF16 && in_dt != HALO_F32) return HALO_EINVAL;
    if (axis != HALO_QUANT_ROWS && axis != HALO_QUANT_COLS_T) return HALO_EINVAL;
    if (rows == 0 || cols == 0) return HALO_OK;
    if (!in || !out_q || !out_scale) return HALO_EINVAL;
    if (rows > kMaxDim || cols > kMaxDim) return HALO_EUNSUPPORTED;
    const int64_t esz = in_dt == HALO_BF16 ? 2 : 4;
    if (ld_in < cols) return HALO_ESHAPE;
    if (ld_q < (axis == HALO_QUANT_ROWS ? cols : rows)) return HALO_ESHAPE;
    if (!aligned16(in) || !aligned16(out_q) || (ld_in * esz) % 16 || ld_q % 16) return HALO_EALIGN;
    if (fold && !aligned16(fold)) return HALO_EALIGN;
    halo_status st = check_right_block(had_block, cols);
    if (st != HALO_OK) return st;
    st = check_block(had_block_left, rows, kMaxLeftBlock);
    if (st != HALO_OK) return st;
    const size_t need = halo_hadamard_quant_workspace_bytes(rows, cols, axis, had_block_left);
    if (need > 0 && (!workspace || workspace_bytes < need)) return HALO_EWORKSPACE;
    if (need > 0 && !aligned16(workspace)) return HALO_EALIGN;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);

    if (axis == HALO_QUANT_COLS_T) {
        if (had_block || had_block_left) return HALO_EUNSUPPORTED;
        if (in_dt != HALO_BF16) return HALO_EUNSUPPORTED;
        ColQuantArgs a{in, ld_in, rows, cols, fold, out_q, ld_q, out_scale, reinterpret_cast<float*>(workspace)};
        return from_hip(launch_col_quant_t(a, s));
    }
    if (cols > kMaxRowCols) return HALO_EUNSUPPORTED;
    RowArgs r{};
    r.rows = rows; r.cols = cols; r.fold = fold; r.out = out_q; r.ld_out = ld_q; r.out_scale = out_scale;
    set_right_block(r, had_block);
    if (had_block_left == 0) {
        r.in = in; r.ld_in = ld_in;
        return from_hip(launch_row_transform(r, in_dt == HALO_BF16 ? IN_BF16 : IN_F32, OUT_Q8, s));
    }
    // left-hand rotation first (strided passes into fp32 scratch), then the row kernel on the scratch
    if ((cols * 4) % 16) return HALO_EALIGN;   // scratch rows must stay 16-byte aligned
    float* tmp = reinterpret_cast<float*>(workspace);
    ColFwhtArgs c{in, in_dt == HALO_BF16 ? IN_BF16 : IN_F32, ld_in, tmp, OUT_F32, cols, tmp, cols, rows, cols,
                  ilog2_exact(had_block_left)};
    hipError_t e = launch_col_fwht(c, s);
    if (e != hipSuccess) return HALO_EHIP;
    r.in = tmp; r.ld_in = cols;
    return from_hip(launch_row_transform(r, IN_F32, OUT_Q8, s));
}

// ------------------------------------------------------------------------------------------------
// Workspace of the tensor-wide quantiser: [left-rotation scratch fp32 rows x cols] [row maxima: rows floats]
// [tensor maximum: 64 floats] [column quantiser: cols floats].
size_t halo_hadamard_quant_tensor_workspace_bytes(int64_t rows, int64_t cols, halo_axis axis, int32_t had_block_left) {
    if (rows <= 0 || cols <= 0) return 0;
    size_t need = round256(((size_t)rows + 64) * 4);
    if (axis == HALO_QUANT_COLS_T) need += round256((size_t)cols * 4);
    if (had_block_left > 0) need += round256((size_t)rows * (size_t)cols * 4);
    return need;
}

halo_status halo_hadamard_quant_tensor(const void* in, halo_dtype in_dt, int64_t rows, int64_t cols, int64_t ld_in,
                                       halo_axis axis, int32_t had_block, int32_t had_block_left, int8_t* out_q,
                                       int64_t ld_q, float* out_scale, void* workspace, size_t workspace_bytes,
                                       void* stream) {
    if (rows < 0 || cols < 0) return HALO_EINVAL;
    if (in_dt != HALO_BF16 && in_dt != HALO_F32) return HALO_EINVAL;
    if (axis != HALO_QUANT_ROWS && axis != HALO_QUANT_COLS_T) return HALO_EINVAL;
    if (rows == 0 || cols == 0) return HALO_OK;
    if (!in || !out_q || !out_scale) return HALO_EINVAL;
    if (rows > kMaxDim || cols > kMaxDim) return HALO_EUNSUPPORTED;
    if (cols > kMaxRowCols) return HALO_EUNSUPPORTED;
    const int64_t esz = in_dt == HALO_BF16 ? 2 : 4;
    if (ld_in < cols) return HALO_ESHAPE;
    if (ld_q < (axis == HALO_QUANT_ROWS ? cols : rows)) return HALO_ESHAPE;
    if (!aligned16(in) || !aligned16(out_q) || (ld_in * esz) % 16 || ld_q % 16) return HALO_EALIGN;
    halo_status st = check_right_block(had_block, cols);
    if (st != HALO_OK) return st;
    st = check_block(had_block_left, rows, kMaxLeftBlock);
    if (st != HALO_OK) return st;
    if (axis == HALO_QUANT_COLS_T && (had_block || had_block_left || in_dt != HALO_BF16)) return HALO_EUNSUPPORTED;
    const size_t need = halo_hadamard_quant_tensor_workspace_bytes(rows, cols, axis, had_block_left);
    if (!workspace || workspace_bytes < need) return HALO_EWORKSPACE;
    if (!aligned16(workspace)) return HALO_EALIGN;
    if (had_block_left > 0 && (cols * 4) % 16) return HALO_EALIGN;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
    float* row_max = reinterpret_cast<float*>(ws);
    float* tensor_max = row_max + rows;                        // 64 floats reserved, one used
    unsigned char* next = ws + round256(((size_t)rows + 64) * 4);
    float* col_ws = reinterpret_cast<float*>(next);
    if (axis == HALO_QUANT_COLS_T) next += round256((size_t)cols * 4);
    float* tmp = reinterpret_cast<float*>(next);

    // what the row kernel reads: the input itself, or its left-rotated fp32 copy
    const void* src = in;
    int64_t ld_src = ld_in;
    InKind src_kind = in_dt == HALO_BF16 ? IN_BF16 : IN_F32;
    if (had_block_left > 0) {
        ColFwhtArgs c{in, src_kind, ld_in, tmp, OUT_F32, cols, tmp, cols, rows, cols, ilog2_exact(had_block_left)};
        if (launch_col_fwht(c, s) != hipSuccess) return HALO_EHIP;
        src = tmp; ld_src = cols; src_kind = IN_F32;
    }
    // phase 1: rotate, absmax of every row; then the maximum of those
    RowArgs r{};
    r.in = src; r.ld_in = ld_src; r.rows = rows; r.cols = cols;
    set_right_block(r, had_block);
    r.out = out_q; r.ld_out = ld_q; r.out_scale = row_max; r.amax_only = 1;
    if (launch_row_transform(r, src_kind, OUT_Q8, s) != hipSuccess) return HALO_EHIP;
    if (launch_reduce_max(row_max, rows, tensor_max, s) != hipSuccess) return HALO_EHIP;
    // phase 2: rotate again and quantise with the tensor's absmax
    if (axis == HALO_QUANT_COLS_T) {
        ColQuantArgs a{in, ld_in, rows, cols, nullptr, out_q, ld_q, out_scale, col_ws};
        return from_hip(launch_col_quant_t_given(a, tensor_max, s));
    }
    r.amax_only = 0; r.given_amax = tensor_max; r.out_scale = out_scale;
    return from_hip(launch_row_transform(r, src_kind, OUT_Q8, s));
}

// ------------------------------------------------------------------------------------------------
size_t halo_quant_dual_workspace_bytes(int64_t rows, int64_t cols) {
    if (rows <= 0 || cols <= 0) return 0;
    return round256(dual_quant_workspace_floats(rows, cols) * 4);
}

halo_status halo_quant_dual(const void* in, int64_t rows, int64_t cols, int64_t ld_in, const float* fold_cols,
                            const float* fold_rows, int8_t* out_q, int64_t ld_q, float* row_scale, int8_t* out_qT,
                            int64_t ld_qT, float* col_scale, void* workspace, size_t workspace_bytes, void* stream) {
    if (rows < 0 || cols < 0) return HALO_EINVAL;
    if (rows == 0 || cols == 0) return HALO_OK;
    if (!in || !out_q || !row_scale || !out_qT || !col_scale) return HALO_EINVAL;
    if (rows > kMaxDim || cols > kMaxDim) return HALO_EUNSUPPORTED;
    if (ld_in < cols || ld_q < cols || ld_qT < rows) return HALO_ESHAPE;
    if (!aligned16(in) || !aligned16(out_q) || !aligned16(out_qT) || (ld_in * 2) % 16 || ld_q % 16 || ld_qT % 16)
        return HALO_EALIGN;
    const size_t need = halo_quant_dual_workspace_bytes(rows, cols);
    if (!workspace || workspace_bytes < need) return HALO_EWORKSPACE;
    if (!aligned16(workspace)) return HALO_EALIGN;
    DualQuantArgs dq{in, ld_in, rows, cols, fold_cols, fold_rows, out_q, ld_q, row_scale, out_qT, ld_qT, col_scale,
                     reinterpret_cast<float*>(workspace)};
    return from_hip(launch_dual_quant(dq, reinterpret_cast<hipStream_t>(stream)));
}

size_t halo_quant_dual_static_max_workspace_bytes(void) { return kStaticScratchBytes; }

halo_status halo_quant_dual_static(const void* in, int64_t rows, int64_t cols, int64_t ld_in, const float* fold_cols,
                                   const float* fold_rows, int8_t* out_q, int64_t ld_q, float* row_scale,
                                   int8_t* out_qT, int64_t ld_qT, float* col_scale, void* stream) {
    if (rows < 0 || cols < 0) return HALO_EINVAL;
    if (rows == 0 || cols == 0) return HALO_OK;
    if (!in || !out_q || !row_scale || !out_qT || !col_scale) return HALO_EINVAL;
    if (rows > kMaxDim || cols > kMaxDim) return HALO_EUNSUPPORTED;
    if (ld_in < cols || ld_q < cols || ld_qT < rows) return HALO_ESHAPE;
    if (!aligned16(in) || !aligned16(out_q) || !aligned16(out_qT) || (ld_in * 2) % 16 || ld_q % 16 || ld_qT % 16)
        return HALO_EALIGN;
    // the partial maxima of this size must fit the built-in scratch array
    if (halo_quant_dual_workspace_bytes(rows, cols) > kStaticScratchBytes) return HALO_EWORKSPACE;
    DualQuantArgs dq{in, ld_in, rows, cols, fold_cols, fold_rows, out_q, ld_q, row_scale, out_qT, ld_qT, col_scale, nullptr};
    return from_hip(launch_dual_quant_static(dq, reinterpret_cast<hipStream_t>(stream)));
}

// ------------------------------------------------------------------------------------------------
// Argument check shared by halo_gemm_i8 and halo_gemm_i8_pair.  *skip is set when the product is empty (a no-op).
static halo_status check_gemm(const halo_gemm_desc* d, GemmArgs* out, bool* skip) {
    *skip = false;
    if (d->M < 0 || d->N < 0 || d->K < 0) return HALO_EINVAL;
    if (d->c_dt != HALO_BF16 && d->c_dt != HALO_F32) return HALO_EINVAL;
    if (d->M == 0 || d->N == 0) { *skip = true; return HALO_OK; }
    if (!d->C && !d->acc_out) return HALO_EINVAL;
    if (d->K > 0 && (!d->A || !d->B)) return HALO_EINVAL;
    if (d->M > kMaxDim || d->N > kMaxDim || d->K > kMaxDim) return HALO_EUNSUPPORTED;
    if (d->K % 16) return HALO_ESHAPE;
    if (!acc_fits_int32(d->K)) return HALO_ESHAPE;
    if (d->K > 0) {
        if (d->lda < d->K || d->ldb < (d->transB ? d->K : d->N)) return HALO_ESHAPE;
        if (!aligned16(d->A) || !aligned16(d->B) || d->lda % 16 || d->ldb % 16) return HALO_EALIGN;
    }
    if (d->C) {
        if (d->ldc < d->N) return HALO_ESHAPE;
        if (!aligned16(d->C) || (d->ldc * (d->c_dt == HALO_BF16 ? 2 : 4)) % 16) return HALO_EALIGN;
    }
    if (d->acc_out) {
        if (d->ld_acc < d->N) return HALO_ESHAPE;
        if (!aligned16(d->acc_out) || (d->ld_acc * 4) % 16) return HALO_EALIGN;
    }
    if (d->config < HALO_GEMM_AUTO || d->config > HALO_GEMM_STAGED_128x128x64) return HALO_EINVAL;
    if (!gemm_config_valid(d->config, d->K)) return HALO_ESHAPE;
    *out = GemmArgs{d->A, d->lda, d->B, d->ldb, d->transB ? 1 : 0, d->M, d->N, d->K, d->row_scale, d->col_scale, d->C,
                    d->c_dt == HALO_F32 ? 1 : 0, d->ldc, d->acc_out, d->ld_acc, d->config};
    return HALO_OK;
}

halo_status halo_gemm_i8(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb, int transB, int64_t M,
                         int64_t N, int64_t K, const float* row_scale, const float* col_scale, void* C,
                         halo_dtype c_dt, int64_t ldc, int32_t* acc_out, int64_t ld_acc, void* stream) {
    const halo_gemm_desc d{A, lda, B, ldb, transB, M, N, K, row_scale, col_scale, C, (int32_t)c_dt, ldc, acc_out, ld_acc,
                           HALO_GEMM_AUTO};
    return halo_gemm_i8_desc(&d, stream);
}

halo_status halo_gemm_i8_desc(const halo_gemm_desc* g, void* stream) {
    if (!g) return HALO_EINVAL;
    GemmArgs a;
    bool skip;
    const halo_status st = check_gemm(g, &a, &skip);
    if (st != HALO_OK || skip) return st;
    return from_hip(launch_gemm_i8(a, reinterpret_cast<hipStream_t>(stream)));
}

halo_status halo_mfma_i8_probe(const int8_t* operands, int32_t iters, int32_t* sink, void* stream) {
    if (!operands || iters < 0) return HALO_EINVAL;
    if (!aligned16(operands)) return HALO_EALIGN;
    if (iters == 0) return HALO_OK;
    return from_hip(launch_mfma_i8_probe(operands, iters, sink, reinterpret_cast<hipStream_t>(stream)));
}

halo_status halo_gemm_i8_pair(const halo_gemm_desc* g1, const halo_gemm_desc* g2, void* stream) {
    if (!g1 || !g2) return HALO_EINVAL;
    GemmArgs a1, a2;
    bool skip1, skip2;
    halo_status st = check_gemm(g1, &a1, &skip1);
    if (st != HALO_OK) return st;
    st = check_gemm(g2, &a2, &skip2);
    if (st != HALO_OK) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (skip1 && skip2) return HALO_OK;
    if (skip1) return from_hip(launch_gemm_i8(a2, s));
    if (skip2) return from_hip(launch_gemm_i8(a1, s));
    return from_hip(launch_gemm_i8_pair(a1, a2, s));
}

// ------------------------------------------------------------------------------------------------
halo_status halo_mx6_quant(const void* in, int64_t rows, int64_t cols, int64_t ld_in, int32_t had_block,
                           uint8_t* out_codes, int64_t ld_codes, uint8_t* out_scales, int64_t ld_scales, void* stream) {
    if (rows < 0 || cols < 0) return HALO_EINVAL;
    if (rows == 0 || cols == 0) return HALO_OK;
    if (!in || !out_codes || !out_scales) return HALO_EINVAL;
    if (rows > kMaxDim || cols > kMaxRowCols) return HALO_EUNSUPPORTED;
    if (cols % 32) return HALO_ESHAPE;
    if (ld_in < cols || ld_codes < cols / 32 * 24 || ld_scales < cols / 32) return HALO_ESHAPE;
    if (!aligned16(in) || !aligned16(out_codes) || (ld_in * 2) % 16 || ld_codes % 8) return HALO_EALIGN;
    const halo_status st = check_block(had_block, cols, kMaxRightBlock);
    if (st != HALO_OK) return st;
    RowArgs r{};
    r.in = in; r.ld_in = ld_in; r.rows = rows; r.cols = cols; r.out = out_codes; r.ld_out = ld_codes;
    r.mx_scales = out_scales; r.ld_mx_scales = ld_scales;
    r.log_block = had_block ? ilog2_exact(had_block) : 0;
    return from_hip(launch_row_transform(r, IN_BF16, OUT_MX6, reinterpret_cast<hipStream_t>(stream)));
}

halo_status halo_gemm_mx6(const uint8_t* A, int64_t lda, const uint8_t* scales_a, int64_t ld_scales_a, const uint8_t* B,
                          int64_t ldb, const uint8_t* scales_b, int64_t ld_scales_b, int64_t M, int64_t N, int64_t K,
                          void* C, halo_dtype c_dt, int64_t ldc, void* stream) {
    if (M < 0 || N < 0 || K < 0) return HALO_EINVAL;
    if (c_dt != HALO_BF16 && c_dt != HALO_F32) return HALO_EINVAL;
    if (M == 0 || N == 0) return HALO_OK;
    if (!C) return HALO_EINVAL;
    if (K > 0 && (!A || !B || !scales_a || !scales_b)) return HALO_EINVAL;
    if (M > kMaxDim || N > kMaxDim || K > kMaxDim) return HALO_EUNSUPPORTED;
    if (K % 128) return HALO_ESHAPE;
    if (ldc < N) return HALO_ESHAPE;
    if (K > 0) {
        if (lda < K / 32 * 24 || ldb < K / 32 * 24 || ld_scales_a < K / 32 || ld_scales_b < K / 32) return HALO_ESHAPE;
        if (!aligned16(A) || !aligned16(B) || lda % 16 || ldb % 16) return HALO_EALIGN;
        if ((reinterpret_cast<uintptr_t>(scales_a) & 3u) || (reinterpret_cast<uintptr_t>(scales_b) & 3u) ||
            ld_scales_a % 4 || ld_scales_b % 4)
            return HALO_EALIGN;
    }
    if (!aligned16(C)) return HALO_EALIGN;
    Mx6GemmArgs g{A, lda, scales_a, ld_scales_a, B, ldb, scales_b, ld_scales_b, M, N, K, C, c_dt == HALO_F32 ? 1 : 0, ldc};
    return from_hip(launch_gemm_mx6(g, reinterpret_cast<hipStream_t>(stream)));
}

// ------------------------------------------------------------------------------------------------
size_t halo_dequant_unrotate_workspace_bytes(int64_t rows, int64_t cols, int32_t had_block_left) {
    if (rows <= 0 || cols <= 0 || had_block_left <= 0) return 0;
    return round256((size_t)rows * (size_t)cols * 4);
}

halo_status halo_dequant_unrotate(const int32_t* acc, int64_t ld_acc, int64_t rows, int64_t cols,
                                  const float* row_scale, const float* tensor_scale, int32_t had_block,
                                  int32_t had_block_left, void* out, halo_dtype out_dt, int64_t ld_out, void* workspace,
                                  size_t workspace_bytes, void* stream) {
    if (rows < 0 || cols < 0) return HALO_EINVAL;
    if (out_dt != HALO_BF16 && out_dt != HALO_F32) return HALO_EINVAL;
    if (rows == 0 || cols == 0) return HALO_OK;
    if (!acc || !out) return HALO_EINVAL;
    if (rows > kMaxDim || cols > kMaxRowCols) return HALO_EUNSUPPORTED;
    if (ld_acc < cols || ld_out < cols) return HALO_ESHAPE;
    if (!aligned16(acc) || !aligned16(out) || (ld_acc * 4) % 16 || (ld_out * (out_dt == HALO_BF16 ? 2 : 4)) % 16)
        return HALO_EALIGN;
    halo_status st = check_right_block(had_block, cols);
    if (st != HALO_OK) return st;
    st = check_block(had_block_left, rows, kMaxLeftBlock);
    if (st != HALO_OK) return st;
    const size_t need = halo_dequant_unrotate_workspace_bytes(rows, cols, had_block_left);
    if (need > 0 && (!workspace || workspace_bytes < need)) return HALO_EWORKSPACE;
    if (need > 0 && (!aligned16(workspace) || (cols * 4) % 16)) return HALO_EALIGN;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);

    RowArgs r{};
    r.in = acc; r.ld_in = ld_acc; r.rows = rows; r.cols = cols; r.pre_scale = row_scale; r.post_scale = tensor_scale;
    set_right_block(r, had_block);
    if (had_block_left == 0) {
        r.out = out; r.ld_out = ld_out;
        return from_hip(launch_row_transform(r, IN_I32, out_dt == HALO_BF16 ? OUT_BF16 : OUT_F32, s));
    }
    // Left-hand un-rotation first: strided passes from the accumulators into the fp32 scratch (butterflies only), then
    // the row kernel multiplies by 1/sqrt(left block), un-rotates along the rows and converts.
    float* tmp = reinterpret_cast<float*>(workspace);
    ColFwhtArgs c{acc, IN_I32, ld_acc, tmp, OUT_F32, cols, tmp, cols, rows, cols, ilog2_exact(had_block_left)};
    c.row_scale = row_scale; c.post_scale = tensor_scale; c.skip_norm = 1;
    if (launch_col_fwht(c, s) != hipSuccess) return HALO_EHIP;
    r.in = tmp; r.ld_in = cols; r.pre_scale = nullptr; r.post_scale = nullptr;
    r.in_mul = (float)(1.0 / sqrt((double)had_block_left));
    r.out = out; r.ld_out = ld_out;
    return from_hip(launch_row_transform(r, IN_F32, out_dt == HALO_BF16 ? OUT_BF16 : OUT_F32, s));
}

// ------------------------------------------------------------------------------------------------
size_t halo_linear_workspace_bytes(const halo_linear_desc* desc) {
    int32_t hm, hb;
    if (resolve_desc(desc, &hm, &hb) != HALO_OK) return 0;
    return bwd_layout(desc).total;
}

halo_status halo_linear_fwd(const halo_linear_desc* desc, const void* X, const void* W, void* Y, int8_t* Xq,
                            float* s_x, int8_t* Wq, float* s_w, void* workspace, size_t workspace_bytes,
                            void* stream) {
    int32_t hm, hb;
    halo_status st = resolve_desc(desc, &hm, &hb);
    if (st != HALO_OK) return st;
    if (!Y || !Xq || !s_x || !Wq || !s_w) return HALO_EINVAL;
    const int64_t b = desc->b, m = desc->m, n = desc->n;
    if (b == 0 || n == 0) return HALO_OK;
    if ((X && !aligned16(X)) || (W && !aligned16(W)) || !aligned16(Y) || !aligned16(Xq) || !aligned16(Wq))
        return HALO_EALIGN;
    const halo_dtype odt = (halo_dtype)desc->out_dt;
    const bool tensor = desc->scale_mode == HALO_SCALE_PER_TENSOR;
    if (tensor && (X || W)) {
        // one scale per tensor (the paper's quantiser): two passes per operand, scratch from the workspace
        const BwdWorkspace L = bwd_layout(desc);
        if (!workspace || workspace_bytes < L.total) return HALO_EWORKSPACE;
        if (!aligned16(workspace)) return HALO_EALIGN;
        unsigned char* tq = reinterpret_cast<unsigned char*>(workspace) + L.tq;
        const size_t tq_bytes = L.total - L.tq;
        if (X && W) {
            // X and W get the same treatment: one launch for the row maxima of both, one for the two tensor maxima, one
            // that rotates again and quantises both
            hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
            float* row_max_x = reinterpret_cast<float*>(tq);
            float* row_max_w = row_max_x + b;
            float* tmax = row_max_w + n;                       // two maxima, 64 floats apart
            if (tq_bytes < (size_t)(b + n + 128) * 4) return HALO_EWORKSPACE;
            RowArgs r{};
            r.in = X; r.ld_in = m; r.rows = b; r.cols = m; r.out = Xq; r.ld_out = m; r.out_scale = row_max_x;
            set_right_block(r, hm);
            r.rows2 = n; r.in2 = W; r.out2 = Wq; r.out_scale2 = row_max_w;
            r.amax_only = 1;
            if (launch_row_transform(r, IN_BF16, OUT_Q8, hs) != hipSuccess) return HALO_EHIP;
            if (launch_reduce_max(row_max_x, b, tmax, hs, row_max_w, n, tmax + 64) != hipSuccess) return HALO_EHIP;
            r.amax_only = 0; r.given_amax = tmax; r.given_amax2 = tmax + 64; r.out_scale = s_x; r.out_scale2 = s_w;
            if (launch_row_transform(r, IN_BF16, OUT_Q8, hs) != hipSuccess) return HALO_EHIP;
            return halo_gemm_i8(Xq, m, Wq, m, 1, b, n, m, s_x, s_w, Y, odt, n, nullptr, 0, stream);
        }
        if (X) {
            st = halo_hadamard_quant_tensor(X, HALO_BF16, b, m, m, HALO_QUANT_ROWS, hm, 0, Xq, m, s_x, tq, tq_bytes, stream);
            if (st != HALO_OK) return st;
        }
        if (W) {
            st = halo_hadamard_quant_tensor(W, HALO_BF16, n, m, m, HALO_QUANT_ROWS, hm, 0, Wq, m, s_w, tq, tq_bytes, stream);
            if (st != HALO_OK) return st;
        }
        return halo_gemm_i8(Xq, m, Wq, m, 1, b, n, m, s_x, s_w, Y, odt, n, nullptr, 0, stream);
    }
    if (X && W && !tensor) {
        // X and W get the same treatment: one launch rotates and quantises both
        RowArgs r{};
        r.in = X; r.ld_in = m; r.rows = b; r.cols = m; r.out = Xq; r.ld_out = m; r.out_scale = s_x;
        set_right_block(r, hm);
        r.rows2 = n; r.in2 = W; r.out2 = Wq; r.out_scale2 = s_w;
        if (launch_row_transform(r, IN_BF16, OUT_Q8, reinterpret_cast<hipStream_t>(stream)) != hipSuccess) return HALO_EHIP;
        return halo_gemm_i8(Xq, m, Wq, m, 1, b, n, m, s_x, s_w, Y, odt, n, nullptr, 0, stream);
    }
    if (X) {
        st = halo_hadamard_quant(X, HALO_BF16, b, m, m, HALO_QUANT_ROWS, hm, 0, nullptr, Xq, m, s_x, nullptr, 0, stream);
        if (st != HALO_OK) return st;
    }
    if (W) {
        st = halo_hadamard_quant(W, HALO_BF16, n, m, m, HALO_QUANT_ROWS, hm, 0, nullptr, Wq, m, s_w, nullptr, 0, stream);
        if (st != HALO_OK) return st;
    }
    return halo_gemm_i8(Xq, m, Wq, m, 1, b, n, m, s_x, s_w, Y, odt, n, nullptr, 0, stream);
}

halo_status halo_linear_bwd(const halo_linear_desc* desc, const void* E, const int8_t* Xq, const float* s_x,
                            const int8_t* Wq, const float* s_w, void* EX, void* G, void* workspace,
                            size_t workspace_bytes, void* stream) {
    int32_t hm, hb;
    halo_status st = resolve_desc(desc, &hm, &hb);
    if (st != HALO_OK) return st;
    if (!E || (!EX && !G)) return HALO_EINVAL;
    if (EX && (!Wq || !s_w)) return HALO_EINVAL;
    if (G && (!Xq || !s_x)) return HALO_EINVAL;
    const int64_t b = desc->b, m = desc->m, n = desc->n;
    if (b == 0 || m == 0 || n == 0) return HALO_OK;
    const BwdWorkspace L = bwd_layout(desc);
    if (!workspace || workspace_bytes < L.total) return HALO_EWORKSPACE;
    if (!aligned16(workspace) || !aligned16(E) || (EX && !aligned16(EX)) || (G && !aligned16(G))) return HALO_EALIGN;
    const halo_dtype odt = (halo_dtype)desc->out_dt;
    const int level = desc->level;
    unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
    int8_t* Eq = reinterpret_cast<int8_t*>(ws + L.eq);
    float* s_e = reinterpret_cast<float*>(ws + L.s_e);
    int8_t* EqT = reinterpret_cast<int8_t*>(ws + L.eqt);
    float* s_g = reinterpret_cast<float*>(ws + L.s_g);
    float* amax = reinterpret_cast<float*>(ws + L.amax);
    int32_t* acc = reinterpret_cast<int32_t*>(ws + L.acc);
    int32_t* acc_g = reinterpret_cast<int32_t*>(ws + L.acc_g);
    float* f32 = reinterpret_cast<float*>(ws + L.f32);

    hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
    const bool both = EX && G;
    const bool tensor = desc->scale_mode == HALO_SCALE_PER_TENSOR;

    if (tensor) {
        // The paper's scalar scales factor out of the integer sums: E is quantised as it is (left-rotated at level
        // 2), and E's scale and the saved tensor's scale multiply the accumulators afterwards, in that order.
        unsigned char* tq = ws + L.tq;
        const size_t tq_bytes = L.total - L.tq;
        if (both && level <= 1) {
            // No left-hand rotation: both quantisations of E share the tensor's maximum.  One absmax pass and one reduction,
            // then the row and the (transposed) column quantiser with that maximum, both products in one launch, both
            // un-rotations in one launch.
            if (tq_bytes < round256(((size_t)b + 64) * 4) + round256((size_t)n * 4)) return HALO_EWORKSPACE;
            float* row_max = reinterpret_cast<float*>(tq);
            float* tmax = row_max + b;
            float* col_ws = reinterpret_cast<float*>(tq + round256(((size_t)b + 64) * 4));
            RowArgs r{};
            r.in = E; r.ld_in = n; r.rows = b; r.cols = n; r.out = Eq; r.ld_out = n; r.out_scale = row_max; r.amax_only = 1;
            if (launch_row_transform(r, IN_BF16, OUT_Q8, hs) != hipSuccess) return HALO_EHIP;
            if (launch_reduce_max(row_max, b, tmax, hs) != hipSuccess) return HALO_EHIP;
            r.amax_only = 0; r.given_amax = tmax; r.out_scale = s_e;
            if (launch_row_transform(r, IN_BF16, OUT_Q8, hs) != hipSuccess) return HALO_EHIP;
            ColQuantArgs q{E, n, b, n, nullptr, EqT, b, s_g, col_ws};
            if (launch_col_quant_t_given(q, tmax, hs) != hipSuccess) return HALO_EHIP;
            GemmArgs gx{Eq, n, Wq, m, 0, b, m, n, nullptr, nullptr, nullptr, 0, m, acc, m, HALO_GEMM_AUTO};
            GemmArgs gg{EqT, b, Xq, m, 0, n, m, b, nullptr, nullptr, nullptr, 0, m, acc_g, m, HALO_GEMM_AUTO};
            if (launch_gemm_i8_pair(gx, gg, hs) != hipSuccess) return HALO_EHIP;
            RowArgs u{};
            u.in = acc; u.ld_in = m; u.rows = b; u.cols = m; u.pre_scale = s_e; u.post_scale = s_w; u.out = EX; u.ld_out = m;
            set_right_block(u, level >= 1 ? hm : 0);
            u.rows2 = n; u.in2 = acc_g; u.pre_scale2 = s_g; u.post_scale2 = s_x; u.out2 = G;
            return from_hip(launch_row_transform(u, IN_I32, odt == HALO_BF16 ? OUT_BF16 : OUT_F32, hs));
        }
        // The left-rotated copy of E is made here, in the layer's fp32 scratch, and handed to the quantiser as fp32
        // input (the un-rotation reuses that scratch afterwards).
        if (EX) {
            const void* src = E;
            halo_dtype src_dt = HALO_BF16;
            if (level >= 2) {
                ColFwhtArgs c{E, IN_BF16, n, f32, OUT_F32, n, f32, n, b, n, ilog2_exact(hb)};
                if (launch_col_fwht(c, hs) != hipSuccess) return HALO_EHIP;
                src = f32; src_dt = HALO_F32;
            }
            st = halo_hadamard_quant_tensor(src, src_dt, b, n, n, HALO_QUANT_ROWS, 0, 0, Eq, n, s_e, tq, tq_bytes, stream);
            if (st != HALO_OK) return st;
            if (level >= 2 && left_in_epilogue(b, n, hb)) {
                GemmArgs gx{Eq, n, Wq, m, 0, b, m, n, s_e, nullptr, acc, 1, m, nullptr, 0, HALO_GEMM_256x256x64};
                gx.left_stages = 8; gx.post_scale = s_w;
                if (launch_gemm_i8(gx, hs) != hipSuccess) return HALO_EHIP;
                if (finish_left_unrotation(reinterpret_cast<float*>(acc), b, m, hb, hm, EX, odt, hs) != hipSuccess)
                    return HALO_EHIP;
            } else {
                GemmArgs gx{Eq, n, Wq, m, 0, b, m, n, nullptr, nullptr, nullptr, 0, m, acc, m, HALO_GEMM_AUTO};
                if (launch_gemm_i8(gx, hs) != hipSuccess) return HALO_EHIP;
                st = halo_dequant_unrotate(acc, m, b, m, s_e, s_w, level >= 1 ? hm : 0, level >= 2 ? hb : 0, EX, odt, m, f32,
                                           level >= 2 ? round256((size_t)b * m * 4) : 0, stream);
                if (st != HALO_OK) return st;
            }
        }
        if (G) {
            st = halo_hadamard_quant_tensor(E, HALO_BF16, b, n, n, HALO_QUANT_COLS_T, 0, 0, EqT, b, s_g, tq, tq_bytes, stream);
            if (st != HALO_OK) return st;
            GemmArgs gg{EqT, b, Xq, m, 0, n, m, b, nullptr, nullptr, nullptr, 0, m, acc_g, m, HALO_GEMM_AUTO};
            if (launch_gemm_i8(gg, hs) != hipSuccess) return HALO_EHIP;
            st = halo_dequant_unrotate(acc_g, m, n, m, s_g, s_x, level >= 1 ? hm : 0, 0, G, odt, m, nullptr, 0, stream);
            if (st != HALO_OK) return st;
        }
        return HALO_OK;
    }

    // ---- quantise E: per row for the E product (left-rotated first at level 2), per column (transposed) for G.
    // Levels 0 and 1 want both from the same E: one tiling of E does both.
    if (both && level <= 1) {
        st = halo_quant_dual(E, b, n, n, s_w, s_x, Eq, n, s_e, EqT, b, s_g, amax, halo_quant_dual_workspace_bytes(b, n), stream);
        if (st != HALO_OK) return st;
    } else {
        // Level 2, both products: the first strided pass of E's left-hand rotation reads all of E anyway and also
        // takes the column maxima of E (x) s_x that the column quantiser needs (left blocks of at least 64 tokens).
        const bool side = both && level >= 2 && hb >= 64;
        if (side) {
            uint32_t* amax_bits = reinterpret_cast<uint32_t*>(amax);
            if (launch_zero_u32(amax_bits, n, hs) != hipSuccess) return HALO_EHIP;
            ColFwhtArgs c{E, IN_BF16, n, f32, OUT_F32, n, f32, n, b, n, ilog2_exact(hb)};
            c.side_fold = s_x; c.side_amax = amax_bits;
            if (launch_col_fwht(c, hs) != hipSuccess) return HALO_EHIP;
            RowArgs r{};
            r.in = f32; r.ld_in = n; r.rows = b; r.cols = n; r.fold = s_w; r.out = Eq; r.ld_out = n; r.out_scale = s_e;
            if (launch_row_transform(r, IN_F32, OUT_Q8, hs) != hipSuccess) return HALO_EHIP;
            ColQuantArgs q{E, n, b, n, s_x, EqT, b, s_g, amax};
            if (launch_col_quant_t_ready(q, hs) != hipSuccess) return HALO_EHIP;
        } else {
            if (EX) {
                st = halo_hadamard_quant(E, HALO_BF16, b, n, n, HALO_QUANT_ROWS, 0, level >= 2 ? hb : 0, s_w, Eq, n, s_e, f32,
                                         level >= 2 ? round256((size_t)b * n * 4) : 0, stream);
                if (st != HALO_OK) return st;
            }
            if (G) {
                st = halo_hadamard_quant(E, HALO_BF16, b, n, n, HALO_QUANT_COLS_T, 0, 0, s_x, EqT, b, s_g, amax,
                                         round256((size_t)n * 4), stream);
                if (st != HALO_OK) return st;
            }
        }
    }

    // ---- the two products on the saved codes.  Level 0 scales and stores the result in the epilogue; levels 1, 2
    // leave int32 accumulators for the un-rotation.  When both are wanted they share one launch.
    GemmArgs gx{Eq, n, Wq, m, 0, b, m, n, level == 0 ? s_e : nullptr, nullptr, level == 0 ? EX : nullptr,
                odt == HALO_F32 ? 1 : 0, m, level == 0 ? nullptr : acc, m, HALO_GEMM_AUTO};
    GemmArgs gg{EqT, b, Xq, m, 0, n, m, b, level == 0 ? s_g : nullptr, nullptr, level == 0 ? G : nullptr,
                odt == HALO_F32 ? 1 : 0, m, level == 0 ? nullptr : acc_g, m, HALO_GEMM_AUTO};
    // Level 2: the E product scales its accumulators and runs the low strides of the left-hand un-rotation in its
    // epilogue, and leaves fp32 where the int32 accumulators would go (same size).
    const bool left_fused = EX && level >= 2 && left_in_epilogue(b, n, hb);
    if (left_fused) {
        gx.row_scale = s_e; gx.C = acc; gx.c_is_f32 = 1; gx.ldc = m; gx.acc_out = nullptr; gx.left_stages = 8;
        gx.config = HALO_GEMM_256x256x64;
        gg.config = HALO_GEMM_256x256x64;
    }
    hipError_t he = hipSuccess;
    if (both) he = launch_gemm_i8_pair(gx, gg, hs);
    else if (EX) he = launch_gemm_i8(gx, hs);
    else he = launch_gemm_i8(gg, hs);
    if (he != hipSuccess) return HALO_EHIP;
    if (level == 0) return HALO_OK;

    // ---- dequantise and un-rotate
    if (both && level == 1 && !tensor) {
        RowArgs r{};
        r.in = acc; r.ld_in = m; r.rows = b; r.cols = m; r.pre_scale = s_e; r.out = EX; r.ld_out = m;
        set_right_block(r, hm);
        r.rows2 = n; r.in2 = acc_g; r.pre_scale2 = s_g; r.out2 = G;
        if (launch_row_transform(r, IN_I32, odt == HALO_BF16 ? OUT_BF16 : OUT_F32, hs) != hipSuccess) return HALO_EHIP;
        return HALO_OK;
    }
    if (left_fused) {
        if (finish_left_unrotation(reinterpret_cast<float*>(acc), b, m, hb, hm, EX, odt, hs) != hipSuccess) return HALO_EHIP;
    } else if (EX) {
        st = halo_dequant_unrotate(acc, m, b, m, s_e, nullptr, hm, level >= 2 ? hb : 0, EX, odt, m, f32,
                                   level >= 2 ? round256((size_t)b * m * 4) : 0, stream);
        if (st != HALO_OK) return st;
    }
    if (G) {
        st = halo_dequant_unrotate(acc_g, m, n, m, s_g, nullptr, hm, 0, G, odt, m, nullptr, 0, stream);
        if (st != HALO_OK) return st;
    }
    return HALO_OK;
}

// ------------------------------------------------------------------------------------------------
size_t halo_peft_workspace_bytes(const halo_linear_desc* desc, int32_t rank) {
    int32_t hm, hb;
    if (resolve_peft(desc, rank, &hm, &hb) != HALO_OK) return 0;
    return peft_layout(desc, rank).total;
}

halo_status halo_peft_fwd(const halo_linear_desc* desc, int32_t rank, const void* X, const int8_t* Wq, const float* s_w,
                          const void* U, const void* V, void* Y, float* T, void* workspace, size_t workspace_bytes,
                          void* stream) {
    int32_t hm, hb;
    halo_status st = resolve_peft(desc, rank, &hm, &hb);
    if (st != HALO_OK) return st;
    if (!X || !Wq || !s_w || !U || !V || !Y || !T) return HALO_EINVAL;
    const int64_t b = desc->b, m = desc->m, n = desc->n;
    if (b == 0 || m == 0 || n == 0) return HALO_OK;
    const PeftWorkspace L = peft_layout(desc, rank);
    if (!workspace || workspace_bytes < L.total) return HALO_EWORKSPACE;
    if (!aligned16(workspace) || !aligned16(X) || !aligned16(Wq) || !aligned16(U) || !aligned16(V) || !aligned16(Y) ||
        !aligned16(T))
        return HALO_EALIGN;
    unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
    int8_t* Xq = reinterpret_cast<int8_t*>(ws + L.xq);
    float* s_x = reinterpret_cast<float*>(ws + L.s_x);
    hipStream_t hs = reinterpret_cast<hipStream_t>(stream);

    st = halo_hadamard_quant(X, HALO_BF16, b, m, m, HALO_QUANT_ROWS, hm, 0, nullptr, Xq, m, s_x, nullptr, 0, stream);
    if (st != HALO_OK) return st;
    if (launch_lr_down(X, m, U, 0, m, T, b, m, rank, hs) != hipSuccess) return HALO_EHIP;
    GemmArgs g{Xq, m, Wq, m, 1, b, n, m, s_x, s_w, Y, desc->out_dt == HALO_F32 ? 1 : 0, n, nullptr, 0, HALO_GEMM_AUTO};
    g.lr_rank = rank; g.lr_a = T; g.lr_b = V; g.lr_b_bf16 = 1;      // V as it is, [n x rank]
    return from_hip(launch_gemm_i8(g, hs));
}

halo_status halo_peft_bwd(const halo_linear_desc* desc, int32_t rank, const void* E, const void* X, const float* T,
                          const int8_t* Wq, const float* s_w, const void* U, const void* V, void* EX, float* GU, float* GV,
                          void* workspace, size_t workspace_bytes, void* stream) {
    int32_t hm, hb;
    halo_status st = resolve_peft(desc, rank, &hm, &hb);
    if (st != HALO_OK) return st;
    if (!E || (!EX && !GU && !GV)) return HALO_EINVAL;
    if ((EX || GU) && !V) return HALO_EINVAL;
    if (EX && (!Wq || !s_w || !U)) return HALO_EINVAL;
    if (GU && !X) return HALO_EINVAL;
    if (GV && !T) return HALO_EINVAL;
    const int64_t b = desc->b, m = desc->m, n = desc->n;
    if (b == 0 || m == 0 || n == 0) return HALO_OK;
    const PeftWorkspace L = peft_layout(desc, rank);
    if (!workspace || workspace_bytes < L.total) return HALO_EWORKSPACE;
    if (!aligned16(workspace) || !aligned16(E) || (X && !aligned16(X)) || (T && !aligned16(T)) || (Wq && !aligned16(Wq)) ||
        (U && !aligned16(U)) || (V && !aligned16(V)) || (EX && !aligned16(EX)) || (GU && !aligned16(GU)) ||
        (GV && !aligned16(GV)))
        return HALO_EALIGN;
    const halo_dtype odt = (halo_dtype)desc->out_dt;
    const int level = desc->level;
    unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
    int8_t* Eq = reinterpret_cast<int8_t*>(ws + L.eq);
    float* s_e = reinterpret_cast<float*>(ws + L.s_e);
    float* c32 = reinterpret_cast<float*>(ws + L.c32);
    float* f32 = reinterpret_cast<float*>(ws + L.f32);
    float* S = reinterpret_cast<float*>(ws + L.s);
    float* Sp = reinterpret_cast<float*>(ws + L.sp);
    float* Up = reinterpret_cast<float*>(ws + L.up);
    float* part = reinterpret_cast<float*>(ws + L.part);
    float* part_u = reinterpret_cast<float*>(ws + L.part_u);
    hipStream_t hs = reinterpret_cast<hipStream_t>(stream);

    // ---- the thin products: S = E V, G_V = E^T T, G_U = S^T X
    if ((EX || GU) && launch_lr_down(E, n, V, 1, rank, S, b, n, rank, hs) != hipSuccess) return HALO_EHIP;
    // E_X = S U + [un-rotation of the quantised product].  The low-rank term joins the product before the un-rotation,
    // in the rotated domain: (H_left S) (U H_right), added to the scaled accumulators in the GEMM epilogue; the un-rotation
    // of the sum then returns S U next to the quantised term (the rotations are orthogonal).
    const float* lr_a = S;
    const bool rotate_s = EX && level >= 2;
    const bool s_small = rotate_s && lr_col_fwht_shape_ok(b, hb);
    if (rotate_s) lr_a = Sp;
    {
        const LrGradArgs gv{E, n, T, GV, 0, part, n}, gu{X, m, S, GU, 1, part_u, m};
        const LrRotArgs rot{U, Up, m, level >= 1 ? hm : 0, s_small ? S : nullptr, Sp, b, hb};
        if (launch_lr_backward_small(GV ? &gv : nullptr, GU ? &gu : nullptr, b, rank, EX ? &rot : nullptr, hs) != hipSuccess)
            return HALO_EHIP;
    }
    if (!EX) return HALO_OK;
    if (rotate_s && !s_small) {            // left blocks too long for one workgroup's LDS: the strided passes
        ColFwhtArgs c{S, IN_F32, rank, Sp, OUT_F32, rank, Sp, rank, b, rank, ilog2_exact(hb)};
        if (launch_col_fwht(c, hs) != hipSuccess) return HALO_EHIP;
    }
    st = halo_hadamard_quant(E, HALO_BF16, b, n, n, HALO_QUANT_ROWS, 0, level >= 2 ? hb : 0, s_w, Eq, n, s_e, f32,
                             level >= 2 ? round256((size_t)b * n * 4) : 0, stream);
    if (st != HALO_OK) return st;
    const bool left_fused = level >= 2 && left_in_epilogue(b, n, hb);
    GemmArgs gx{Eq, n, Wq, m, 0, b, m, n, s_e, nullptr, level == 0 ? EX : (void*)c32,
                (level > 0 || odt == HALO_F32) ? 1 : 0, m, nullptr, 0, HALO_GEMM_AUTO};
    gx.lr_rank = rank; gx.lr_a = lr_a; gx.lr_b = Up;                 // (U H)^T, [m x rank]
    if (left_fused) { gx.left_stages = 8; gx.config = HALO_GEMM_256x256x64; }
    if (launch_gemm_i8(gx, hs) != hipSuccess) return HALO_EHIP;
    if (level == 0) return HALO_OK;
    if (level >= 2) return from_hip(finish_left_unrotation(c32, b, m, hb, hm, EX, odt, hs, left_fused ? 8 : 0));
    RowArgs r{};
    r.in = c32; r.ld_in = m; r.rows = b; r.cols = m; r.out = EX; r.ld_out = m;
    set_right_block(r, hm);
    return from_hip(launch_row_transform(r, IN_F32, odt == HALO_BF16 ? OUT_BF16 : OUT_F32, hs));
}

}  // extern "C"
