// The high-precision low-rank side branch of a LoRA-style linear module next to the quantised products (Section 3.3
// "Parameter Efficient Fine Tuning"; Appendix "LoRA-style Linear Module and HALO for PEFT"):
//   T = X U^T,  S = E_Y V            (tall input times a thin matrix: lr_down_kernel, bf16 matrix instructions)
//   G_V = E_Y^T T,  G_U = S^T X      (thin result, reduction over the tokens: lr_grad_kernel + lr_reduce_kernel)
// and the small helpers that bring V and U into the form the GEMM epilogue wants (fp32, rank-major).  The additions
// T V^T and S U themselves happen in the epilogue of the INT8 GEMM.  All inputs are bf16, every product accumulates in
// fp32 and the intermediates T and S stay fp32.  Every kernel here is bound by one read of its tall operand from HBM.
#pragma clang fp contract(off)

#include "halo_internal.h"

namespace halo {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// ------------------------------------------------------------------------------------------------ down-projection
// out[row, c] = sum_k in[row, k] * bt[c, k]:  in bf16 [rows x K] (pitch ld_in), bt [rank x K] (pitch ld_b) either bf16 or
// fp32 holding bf16-representable values, out fp32 [rows x rank] dense.  K a multiple of 32, rank <= 64.
// A workgroup owns 16 rows; its eight wavefronts take the 32-element K chunks round robin (v_mfma_f32_16x16x32_bf16:
// lane l supplies row l % 16, elements 8 (l / 16) .. + 8 of the chunk, for both operands; result lane l holds column
// l % 16, rows 4 (l / 16) .. + 4) and their partial sums meet in LDS, added in wavefront order.
constexpr int kDownWaves = 8;

template <bool B_F32>
__global__ void __launch_bounds__(64 * kDownWaves)
lr_down_kernel(const uint16_t* __restrict__ in, int64_t ld_in, const void* __restrict__ bt, int64_t ld_b,
               float* __restrict__ out, int64_t rows, int64_t K, int rank) {
    __shared__ float s_part[kDownWaves][4][4][64];      // [wavefront][rank tile][register][lane]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lr = lane & 15, kg = lane >> 4;
    const int64_t row0 = (int64_t)blockIdx.x * 16;
    int64_t row = row0 + lr;
    if (row > rows - 1) row = rows - 1;                 // clamped rows are computed and never stored
    const uint16_t* ap = in + row * ld_in + kg * 8;
    const int ntile = (rank + 15) >> 4;
    v4f acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = v4f{0.0f, 0.0f, 0.0f, 0.0f};


    for (int64_t k0 = (int64_t)wave * 32; k0 < K; k0 += kDownWaves * 32) {
        const v8bf a = *reinterpret_cast<const v8bf*>(ap + k0);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (t >= ntile) break;                      // uniform
            const int c = t * 16 + lr;
            v8bf b;
            if (c < rank) {
                if constexpr (B_F32) {
                    const float* bp = reinterpret_cast<const float*>(bt) + (int64_t)c * ld_b + k0 + kg * 8;
                    const float4 lo = *reinterpret_cast<const float4*>(bp);
                    const float4 hi = *reinterpret_cast<const float4*>(bp + 4);
                    // the values are bf16-representable: the conversion is exact
                    b = v8bf{(__bf16)lo.x, (__bf16)lo.y, (__bf16)lo.z, (__bf16)lo.w,
                             (__bf16)hi.x, (__bf16)hi.y, (__bf16)hi.z, (__bf16)hi.w};
                } else {
                    b = *reinterpret_cast<const v8bf*>(reinterpret_cast<const uint16_t*>(bt) + (int64_t)c * ld_b + k0 + kg * 8);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) b[e] = (__bf16)0.0f;
            }
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[t], 0, 0, 0);
        }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) s_part[wave][t][v][lane] = acc[t][v];
    __syncthreads();
    // 4 tiles x 4 registers x 64 lanes = 1024 sums, two per thread
    for (int idx = threadIdx.x; idx < ntile * 256; idx += 64 * kDownWaves) {
        const int t = idx >> 8, v = (idx >> 6) & 3, l = idx & 63;
        float sum = s_part[0][t][v][l];
#pragma unroll
        for (int w = 1; w < kDownWaves; ++w) sum += s_part[w][t][v][l];
        const int64_t r = row0 + 4 * (l >> 4) + v;
        const int c = t * 16 + (l & 15);
        if (r < rows && c < rank) out[r * rank + c] = sum;
    }
}

// ------------------------------------------------------------------------------------------------ adapter gradients
// part[split][col][c] = sum over the tokens t of the split of big[t, col] * small[t, c]:  big bf16 [rows x wide] (pitch
// ld_big), small fp32 [rows x rank] dense.  A workgroup owns 128 columns of `big` and one range of tokens; its four
// wavefronts take groups of four tokens round robin.  v_mfma_f32_16x16x4_f32 (lane l supplies A[i = l % 16][k = l / 16]
// and B[k = l / 16][j = l % 16]; result lane l holds j = l % 16, i = 4 (l / 16) .. + 4) with k = token, j = rank index
// and i = one of sixteen columns: a lane loads 8 consecutive columns of one token (16 bytes), and the v-th of them feeds
// the v-th of eight instructions, so instruction v covers columns c0 + 8 i + v.  NTILE = rank tiles of 16.
constexpr int kGradWaves = 4;

template <int NTILE>
__global__ void __launch_bounds__(64 * kGradWaves)
lr_grad_kernel(const uint16_t* __restrict__ big, int64_t ld_big, const float* __restrict__ small, float* __restrict__ part,
               int64_t rows, int64_t wide, int rank, int64_t rows_per_split) {
    __shared__ float s_sum[NTILE * 8 * 4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i16 = lane & 15, kq = lane >> 4;
    const int64_t c0 = (int64_t)blockIdx.x * 128;
    const int64_t col = c0 + 8 * i16;
    const bool col_ok = col < wide;                      // wide is a multiple of 8
    const int64_t t_begin = (int64_t)blockIdx.y * rows_per_split;
    int64_t t_end = t_begin + rows_per_split;
    if (t_end > rows) t_end = rows;

    v4f acc[NTILE][8];
#pragma unroll
    for (int t = 0; t < NTILE; ++t)
#pragma unroll
        for (int v = 0; v < 8; ++v) acc[t][v] = v4f{0.0f, 0.0f, 0.0f, 0.0f};


    for (int64_t t0 = t_begin + wave * 4; t0 < t_end; t0 += kGradWaves * 4) {
        const int64_t tr = t0 + kq;
        const bool ok = tr < t_end;
        uint4 raw = make_uint4(0u, 0u, 0u, 0u);
        if (ok && col_ok) raw = *reinterpret_cast<const uint4*>(big + tr * ld_big + col);
        float sv[NTILE];
#pragma unroll
        for (int t = 0; t < NTILE; ++t) {
            const int c = t * 16 + i16;
            sv[t] = (ok && c < rank) ? small[tr * rank + c] : 0.0f;
        }
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const float a = (v & 1) ? __uint_as_float(w[v >> 1] & 0xFFFF0000u) : __uint_as_float(w[v >> 1] << 16);
#pragma unroll
            for (int t = 0; t < NTILE; ++t) acc[t][v] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, sv[t], acc[t][v], 0, 0, 0);
        }
    }
    // the four wavefronts add their sums in LDS one after the other (a fixed order)
    for (int w = 0; w < kGradWaves; ++w) {
        if (wave == w) {
#pragma unroll
            for (int t = 0; t < NTILE; ++t)
#pragma unroll
                for (int v = 0; v < 8; ++v)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float* p = &s_sum[(t * 8 + v) * 4 + e][lane];
                        *p = (w == 0) ? acc[t][v][e] : *p + acc[t][v][e];
                    }
        }
        __syncthreads();
    }
    if (wave == 0) {
#pragma unroll
        for (int t = 0; t < NTILE; ++t)
#pragma unroll
            for (int v = 0; v < 8; ++v)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int64_t oc = c0 + 8 * (4 * kq + e) + v;
                    const int c = t * 16 + i16;
                    if (oc < wide && c < rank)
                        part[((int64_t)blockIdx.y * wide + oc) * rank + c] = s_sum[(t * 8 + v) * 4 + e][lane];
                }
    }
}

// out = sum over the splits, in order.  transpose_out: out[c * wide + col] (a [rank x wide] result), else
// out[col * rank + c].
__global__ void __launch_bounds__(256)
lr_reduce_kernel(const float* __restrict__ part, float* __restrict__ out, int64_t wide, int rank, int splits,
                 int transpose_out) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = wide * rank;
    if (idx >= total) return;
    float sum = part[idx];
    for (int s = 1; s < splits; ++s) sum += part[(int64_t)s * total + idx];
    if (transpose_out) {
        const int64_t colw = idx / rank;
        const int c = (int)(idx % rank);
        out[(int64_t)c * wide + colw] = sum;
    } else {
        out[idx] = sum;
    }
}

// ------------------------------------------------------------------------------------------------ small helpers
// out[k * n + j] = float(in[j * rank + k]):  V bf16 [n x rank]  ->  V^T fp32 [rank x n].
__global__ void __launch_bounds__(256)
lr_transpose_kernel(const uint16_t* __restrict__ in, float* __restrict__ out, int64_t n, int rank) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * rank) return;
    const int64_t j = idx / rank;
    const int k = (int)(idx % rank);
    out[(int64_t)k * n + j] = bf16_to_f32(in[idx]);
}

// Sign rows of the order-28 Hadamard matrix (bit c of row r set: entry +1), built like the row kernel's: Paley's second
// construction from the quadratic character modulo 13.  The matrix is symmetric.
constexpr int lr_chi13(int a) {
    a %= 13;
    if (a < 0) a += 13;
    if (a == 0) return 0;
    for (int t = 1; t < 13; ++t)
        if ((t * t) % 13 == a) return 1;
    return -1;
}
constexpr bool lr_h28_plus(int r, int c) {
    const int i = r >> 1, j = c >> 1;
    const int conf = (i == 0 && j == 0) ? 0 : ((i == 0 || j == 0) ? 1 : lr_chi13(i - j));
    const int u = r & 1, w = c & 1;
    if (conf == 0) return u == 0 && w == 0;
    return (conf > 0) != (u == 1 && w == 1);
}
struct H28Rows { uint32_t row[28]; };
constexpr H28Rows make_h28_rows() {
    H28Rows m{};
    for (int r = 0; r < 28; ++r)
        for (int c = 0; c < 28; ++c)
            if (lr_h28_plus(r, c)) m.row[r] |= 1u << c;
    return m;
}
__device__ const H28Rows kH28Rows = make_h28_rows();

// out[row, :] = in[row, :] rotated in blocks of `block` elements (block = 2^n, or 28 * 2^n: H_{2^n} (x) H_28 with element
// i * 28 + j indexed by i in the Walsh-Hadamard factor), normalised; block <= 1: a plain conversion.  bf16 in, fp32 out,
// a handful of rows (the adapter U): one workgroup per (row, block), the block in LDS.  The order of the additions is
// not that of the row kernels; nothing here needs to be reproducible to the bit against a reference.
constexpr int kSmallFwhtMax = 14336;

__global__ void __launch_bounds__(256)
lr_row_fwht_kernel(const uint16_t* __restrict__ in, int64_t ld_in, float* __restrict__ out, int64_t ld_out, int block,
                   int unit, float c_norm) {
    __shared__ float s_x[kSmallFwhtMax];
    const int64_t row = blockIdx.y;
    const int64_t base = (int64_t)blockIdx.x * block;
    const uint16_t* src = in + row * ld_in + base;
    for (int i = threadIdx.x; i < block; i += 256) s_x[i] = bf16_to_f32(src[i]);
    __syncthreads();
    const int p = block / unit;                          // length of the Walsh-Hadamard factor
    if (unit == 28) {
        for (int run = threadIdx.x; run < p; run += 256) {
            float x[28], y[28];
#pragma unroll
            for (int j = 0; j < 28; ++j) x[j] = s_x[run * 28 + j];
#pragma unroll
            for (int c = 0; c < 28; ++c) {
                const uint32_t m = kH28Rows.row[c];
                float acc = 0.0f;
#pragma unroll
                for (int j = 0; j < 28; ++j) acc += ((m >> j) & 1u) ? x[j] : -x[j];
                y[c] = acc;
            }
#pragma unroll
            for (int j = 0; j < 28; ++j) s_x[run * 28 + j] = y[j];
        }
        __syncthreads();
    }
    for (int h = 1; h < p; h <<= 1) {
        for (int q = threadIdx.x; q < block / 2; q += 256) {
            const int j = q % unit, ii = q / unit;
            const int i = ((ii / h) * 2 * h) + (ii % h);
            const float a = s_x[i * unit + j], b = s_x[(i + h) * unit + j];
            s_x[i * unit + j] = a + b;
            s_x[(i + h) * unit + j] = a - b;
        }
        __syncthreads();
    }
    float* dst = out + row * ld_out + base;
    for (int i = threadIdx.x; i < block; i += 256) dst[i] = s_x[i] * c_norm;
}

__global__ void __launch_bounds__(256)
lr_widen_kernel(const uint16_t* __restrict__ in, int64_t ld_in, float* __restrict__ out, int64_t ld_out, int64_t cols) {
    const int64_t row = blockIdx.y;
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c < cols) out[row * ld_out + c] = bf16_to_f32(in[row * ld_in + c]);
}

}  // namespace

// ------------------------------------------------------------------------------------------------ launchers
hipError_t launch_lr_down(const void* in, int64_t ld_in, const void* bt, int bt_is_f32, int64_t ld_b, float* out,
                          int64_t rows, int64_t K, int rank, hipStream_t s) {
    if (rows <= 0 || rank <= 0) return hipSuccess;
    if (rank > kMaxLowRank || K % 32 != 0 || K <= 0 || ld_in < K || ld_b < K || ld_in % 8 != 0 ||
        ld_b % (bt_is_f32 ? 4 : 8) != 0)
        return hipErrorInvalidValue;
    const int64_t blocks = (rows + 15) / 16;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    if (bt_is_f32)
        hipLaunchKernelGGL(lr_down_kernel<true>, dim3((unsigned)blocks), dim3(64 * kDownWaves), 0, s,
                           reinterpret_cast<const uint16_t*>(in), ld_in, bt, ld_b, out, rows, K, rank);
    else
        hipLaunchKernelGGL(lr_down_kernel<false>, dim3((unsigned)blocks), dim3(64 * kDownWaves), 0, s,
                           reinterpret_cast<const uint16_t*>(in), ld_in, bt, ld_b, out, rows, K, rank);
    return hipGetLastError();
}

// Token ranges of the gradient kernel: enough workgroups to fill the chip, ranges a multiple of 16 tokens, at most 16.
int lr_grad_splits(int64_t rows, int64_t wide) {
    const int64_t col_tiles = (wide + 127) / 128;
    int64_t splits = (768 + col_tiles - 1) / col_tiles;
    if (splits > 16) splits = 16;
    const int64_t max_splits = (rows + 63) / 64;         // at least 64 tokens per range
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    return (int)splits;
}

size_t lr_grad_workspace_floats(int64_t rows, int64_t wide, int rank) {
    return (size_t)lr_grad_splits(rows, wide) * (size_t)wide * (size_t)rank;
}

hipError_t launch_lr_grad(const void* big, int64_t ld_big, const float* small, float* out, int transpose_out, float* part,
                          int64_t rows, int64_t wide, int rank, hipStream_t s) {
    if (wide <= 0 || rank <= 0) return hipSuccess;
    if (rank > kMaxLowRank || wide % 8 != 0 || ld_big < wide || ld_big % 8 != 0 || rows <= 0) return hipErrorInvalidValue;
    const int splits = lr_grad_splits(rows, wide);
    int64_t per = (rows + splits - 1) / splits;
    per = (per + 15) / 16 * 16;
    const dim3 grid((unsigned)((wide + 127) / 128), (unsigned)splits);
    const uint16_t* b16 = reinterpret_cast<const uint16_t*>(big);
    if (rank <= 16)
        hipLaunchKernelGGL(lr_grad_kernel<1>, grid, dim3(64 * kGradWaves), 0, s, b16, ld_big, small, part, rows, wide, rank, per);
    else if (rank <= 32)
        hipLaunchKernelGGL(lr_grad_kernel<2>, grid, dim3(64 * kGradWaves), 0, s, b16, ld_big, small, part, rows, wide, rank, per);
    else
        hipLaunchKernelGGL(lr_grad_kernel<4>, grid, dim3(64 * kGradWaves), 0, s, b16, ld_big, small, part, rows, wide, rank, per);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t total = wide * rank;
    hipLaunchKernelGGL(lr_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, part, out, wide, rank, splits,
                       transpose_out);
    return hipGetLastError();
}

hipError_t launch_lr_transpose(const void* in, float* out, int64_t n, int rank, hipStream_t s) {
    if (n <= 0 || rank <= 0) return hipSuccess;
    const int64_t total = n * rank;
    hipLaunchKernelGGL(lr_transpose_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                       reinterpret_cast<const uint16_t*>(in), out, n, rank);
    return hipGetLastError();
}

bool lr_row_fwht_shape_ok(int64_t cols, int64_t block) {
    if (block <= 1) return true;
    if (block > kSmallFwhtMax || cols % block != 0) return false;
    if ((block & (block - 1)) == 0) return true;
    if (block % 28 != 0) return false;
    const int64_t p = block / 28;
    return (p & (p - 1)) == 0;
}

hipError_t launch_lr_row_fwht(const void* in, int64_t ld_in, float* out, int64_t ld_out, int64_t rows, int64_t cols,
                              int64_t block, hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    if (!lr_row_fwht_shape_ok(cols, block) || rows > 65535) return hipErrorInvalidValue;
    const uint16_t* src = reinterpret_cast<const uint16_t*>(in);
    if (block <= 1) {
        hipLaunchKernelGGL(lr_widen_kernel, dim3((unsigned)((cols + 255) / 256), (unsigned)rows), dim3(256), 0, s, src, ld_in,
                           out, ld_out, cols);
        return hipGetLastError();
    }
    const int unit = (block & (block - 1)) == 0 ? 1 : 28;
    const float c_norm = (float)(1.0 / sqrt((double)block));
    hipLaunchKernelGGL(lr_row_fwht_kernel, dim3((unsigned)(cols / block), (unsigned)rows), dim3(256), 0, s, src, ld_in, out,
                       ld_out, (int)block, unit, c_norm);
    return hipGetLastError();
}

}  // namespace halo
