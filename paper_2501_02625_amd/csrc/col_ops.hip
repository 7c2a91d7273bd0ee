// Kernels that work down the strided (row-index) axis of a row-major matrix:
//   * left-hand Walsh-Hadamard rotation  h'(A) = H^T A  over blocks of rows, done directly on strided data
//     (no transposes): each lane keeps 2^LOGR rows of one or two columns in registers, so all butterflies of
//     a pass are register-to-register and the memory accesses stay coalesced along the rows;
//   * the column-wise absmax INT8 quantiser with transposed output, (E^T)_Q.
#pragma clang fp contract(off)

#include "halo_internal.h"

namespace halo {
namespace {

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// ------------------------------------------------------------------------------------------------
// One pass of the left-hand FWHT: stages with row strides 2^p .. 2^(p+LOGR-1), ascending.
// A wavefront owns 64*CPL consecutive columns and the 2^LOGR rows  base + t*2^p.
template <int LOGR, int CPL, int IN, int OUT>
__global__ void __launch_bounds__(256)
col_fwht_kernel(const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows, int64_t cols,
                int p, float c_final, int64_t col_tiles) {
    constexpr int R = 1 << LOGR;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t ct = (int64_t)blockIdx.x % col_tiles;
    const int64_t grp = (int64_t)blockIdx.x / col_tiles;
    const int64_t col = (ct * 4 + wave) * 64 * CPL + (int64_t)lane * CPL;
    const int64_t lo = grp & ((int64_t(1) << p) - 1);
    const int64_t hi = grp >> p;
    const int64_t base = (hi << (p + LOGR)) + lo;
    const int64_t stride = int64_t(1) << p;
    if (col >= cols) return;
    const bool pair_ok = (CPL == 1) || (col + 1 < cols);

    float v[R][CPL];
#pragma unroll
    for (int t = 0; t < R; ++t) {
        const int64_t r = base + t * stride;
        if constexpr (IN == IN_BF16) {
            const uint16_t* src = reinterpret_cast<const uint16_t*>(in) + r * ld_in + col;
            if constexpr (CPL == 2) {
                if (pair_ok) {
                    const uint32_t w = *reinterpret_cast<const uint32_t*>(src);
                    v[t][0] = __uint_as_float(w << 16);
                    v[t][1] = __uint_as_float(w & 0xFFFF0000u);
                } else {
                    v[t][0] = __uint_as_float((uint32_t)src[0] << 16);
                    v[t][1] = 0.0f;
                }
            } else {
                v[t][0] = __uint_as_float((uint32_t)src[0] << 16);
            }
        } else {
            const float* src = reinterpret_cast<const float*>(in) + r * ld_in + col;
            if constexpr (CPL == 2) {
                if (pair_ok) {
                    const float2 w = *reinterpret_cast<const float2*>(src);
                    v[t][0] = w.x; v[t][1] = w.y;
                } else {
                    v[t][0] = src[0]; v[t][1] = 0.0f;
                }
            } else {
                v[t][0] = src[0];
            }
        }
    }

#pragma unroll
    for (int b = 0; b < LOGR; ++b) {
        const int h = 1 << b;
#pragma unroll
        for (int t = 0; t < R; ++t) {
            if ((t & h) == 0) {
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    const float x = v[t][c], y = v[t | h][c];
                    v[t][c] = x + y;
                    v[t | h][c] = x - y;
                }
            }
        }
    }

    if (c_final != 1.0f) {
#pragma unroll
        for (int t = 0; t < R; ++t)
#pragma unroll
            for (int c = 0; c < CPL; ++c) v[t][c] *= c_final;
    }

#pragma unroll
    for (int t = 0; t < R; ++t) {
        const int64_t r = base + t * stride;
        if constexpr (OUT == OUT_F32) {
            float* dst = reinterpret_cast<float*>(out) + r * ld_out + col;
            if constexpr (CPL == 2) {
                if (pair_ok) *reinterpret_cast<float2*>(dst) = make_float2(v[t][0], v[t][1]);
                else dst[0] = v[t][0];
            } else {
                dst[0] = v[t][0];
            }
        } else {
            uint16_t* dst = reinterpret_cast<uint16_t*>(out) + r * ld_out + col;
            if constexpr (CPL == 2) {
                if (pair_ok) *reinterpret_cast<uint32_t*>(dst) = f32_to_bf16_rne(v[t][0]) | (f32_to_bf16_rne(v[t][1]) << 16);
                else dst[0] = (uint16_t)f32_to_bf16_rne(v[t][0]);
            } else {
                dst[0] = (uint16_t)f32_to_bf16_rne(v[t][0]);
            }
        }
    }
}

template <int LOGR, int CPL, int IN, int OUT>
hipError_t launch_pass(const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows, int64_t cols,
                       int p, float c_final, hipStream_t s) {
    const int64_t col_tiles = (cols + 256 * CPL - 1) / (256 * CPL);
    const int64_t groups = rows >> LOGR;
    const int64_t blocks = col_tiles * groups;
    if (blocks <= 0 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL((col_fwht_kernel<LOGR, CPL, IN, OUT>), dim3((unsigned)blocks), dim3(256), 0, s, in, ld_in,
                       out, ld_out, rows, cols, p, c_final, col_tiles);
    return hipGetLastError();
}

template <int IN, int OUT>
hipError_t launch_pass_by_logr(int logr, const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows,
                               int64_t cols, int p, float c_final, hipStream_t s) {
    switch (logr) {
        case 1: return launch_pass<1, 2, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s);
        case 2: return launch_pass<2, 2, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s);
        case 3: return launch_pass<3, 2, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s);
        case 4: return launch_pass<4, 2, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s);
        case 5: return launch_pass<5, 2, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s);
        case 6: return launch_pass<6, 2, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s);
        case 7:
            if constexpr (IN == IN_F32) return launch_pass<7, 1, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s);
            return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

// ------------------------------------------------------------------------------------------------
// Column absmax of  in[r,k] * fold[r]  (non-negative floats compare like their bit patterns, so an integer
// atomic max accumulates them exactly and in any order).
__global__ void __launch_bounds__(256) fill_u32_kernel(uint32_t* p, int64_t n, uint32_t value) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = value;
}

constexpr int kAmaxRows = 64;   // rows per workgroup in the absmax pass
__global__ void __launch_bounds__(256)
col_amax_kernel(const uint16_t* in, int64_t ld_in, int64_t rows, int64_t cols, const float* fold, uint32_t* amax_bits) {
    __shared__ float s_part[4][256];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t col = ((int64_t)blockIdx.x * 64 + lane) * 4;
    const int64_t r0 = (int64_t)blockIdx.y * kAmaxRows;
    float m[4] = {0.f, 0.f, 0.f, 0.f};
    if (col < cols) {
        const bool full = col + 4 <= cols;
        for (int t = wave; t < kAmaxRows; t += 4) {
            const int64_t r = r0 + t;
            if (r >= rows) break;
            const float f = fold ? fold[r] : 1.0f;
            const uint16_t* src = in + r * ld_in + col;
            float x[4] = {0.f, 0.f, 0.f, 0.f};
            if (full) {
                const uint2 w = *reinterpret_cast<const uint2*>(src);
                x[0] = __uint_as_float(w.x << 16); x[1] = __uint_as_float(w.x & 0xFFFF0000u);
                x[2] = __uint_as_float(w.y << 16); x[3] = __uint_as_float(w.y & 0xFFFF0000u);
            } else {
                for (int e = 0; e < 4; ++e)
                    if (col + e < cols) x[e] = __uint_as_float((uint32_t)src[e] << 16);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) m[e] = fmaxf(m[e], fabsf(x[e] * f));
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) s_part[wave][lane * 4 + e] = m[e];
    __syncthreads();
    if (wave == 0 && col < cols) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float t = fmaxf(fmaxf(s_part[0][lane * 4 + e], s_part[1][lane * 4 + e]),
                                  fmaxf(s_part[2][lane * 4 + e], s_part[3][lane * 4 + e]));
            if (col + e < cols && t > 0.0f) atomicMax(amax_bits + col + e, __float_as_uint(t));
        }
    }
}

// Quantise a 128(rows) x 128(cols) tile and write it transposed.  Codes of four consecutive rows are packed
// into one dword per column, staged in LDS as [col][row/4] with a pitch of 33 dwords, and read back as
// 16 consecutive rows per lane so that every output row is written in full 128-byte lines.
constexpr int kTI = 128, kTJ = 128, kPitch = kTI / 4 + 1;
__global__ void __launch_bounds__(256)
col_quant_t_kernel(const uint16_t* in, int64_t ld_in, int64_t rows, int64_t cols, const float* fold,
                   const uint32_t* amax_bits, int8_t* out_q, int64_t ld_q, float* out_scale) {
    __shared__ uint32_t s_tile[kTJ * kPitch];
    const int tid = threadIdx.x;
    const int64_t j0 = (int64_t)blockIdx.x * kTJ;
    const int64_t i0 = (int64_t)blockIdx.y * kTI;

    // phase 1: load, scale, round, pack along rows
    {
        const int jl = tid & 31;           // 4 columns each
        const int64_t col = j0 + 4 * jl;
        float inv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float am = 0.0f;
            if (col + e < cols) am = __uint_as_float(amax_bits[col + e]);
            inv[e] = am > 0.0f ? 127.0f / am : 0.0f;
            if (blockIdx.y == 0 && tid < 32 && col + e < cols) out_scale[col + e] = am > 0.0f ? am / 127.0f : 1.0f;
        }
        const bool full = col + 4 <= cols;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int iq = (tid >> 5) + 8 * s;           // row quad inside the tile
            uint32_t b[4][4];                             // [row in quad][col]
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t row = i0 + 4 * iq + r;
                float x[4] = {0.f, 0.f, 0.f, 0.f};
                float f = 1.0f;
                if (row < rows && col < cols) {
                    if (fold) f = fold[row];
                    const uint16_t* src = in + row * ld_in + col;
                    if (full) {
                        const uint2 w = *reinterpret_cast<const uint2*>(src);
                        x[0] = __uint_as_float(w.x << 16); x[1] = __uint_as_float(w.x & 0xFFFF0000u);
                        x[2] = __uint_as_float(w.y << 16); x[3] = __uint_as_float(w.y & 0xFFFF0000u);
                    } else {
                        for (int e = 0; e < 4; ++e)
                            if (col + e < cols) x[e] = __uint_as_float((uint32_t)src[e] << 16);
                    }
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float t = (x[e] * f) * inv[e];
                    b[r][e] = __float_as_uint(t + 12582912.0f);
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t lo = __builtin_amdgcn_perm(b[1][e], b[0][e], 0x0c0c0400u);
                const uint32_t hi = __builtin_amdgcn_perm(b[3][e], b[2][e], 0x0c0c0400u);
                s_tile[(4 * jl + e) * kPitch + iq] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
            }
        }
    }
    __syncthreads();
    // phase 2: each lane writes 16 consecutive rows (16 bytes) of one output row
    {
        const int seg = tid & 7;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int jj = (tid >> 3) + 32 * s;
            const int64_t col = j0 + jj;
            if (col >= cols) continue;
            uint32_t w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) w[q] = s_tile[jj * kPitch + 4 * seg + q];
            const int64_t i = i0 + 16 * seg;
            int8_t* dst = out_q + col * ld_q + i;
            if (i + 16 <= rows) {
                *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
            } else {
                for (int e = 0; e < 16; ++e)
                    if (i + e < rows) dst[e] = (int8_t)((w[e >> 2] >> (8 * (e & 3))) & 0xFF);
            }
        }
    }
}

}  // namespace

hipError_t launch_col_fwht(const ColFwhtArgs& a, hipStream_t s) {
    if (a.rows == 0 || a.cols == 0 || a.log_block == 0) return hipSuccess;
    // split the log_block stages into passes of at most 6 (a final 7 is allowed for fp32 input)
    int sizes[8], np = 0, left = a.log_block;
    while (left > 0) {
        int q = left <= 6 ? left : (left == 7 && np > 0 ? 7 : 6);
        sizes[np++] = q;
        left -= q;
        if (np >= 8) return hipErrorInvalidValue;
    }
    const float c = (float)(1.0 / sqrt((double)(int64_t(1) << a.log_block)));
    int p = 0;
    for (int i = 0; i < np; ++i) {
        const bool first = i == 0, last = i == np - 1;
        const void* src = first ? a.in : (const void*)a.tmp;
        const int64_t ld_src = first ? a.ld_in : a.ld_tmp;
        const InKind ik = first ? a.in_kind : IN_F32;
        void* dst = last ? a.out : (void*)a.tmp;
        const int64_t ld_dst = last ? a.ld_out : a.ld_tmp;
        const OutKind ok = last ? a.out_kind : OUT_F32;
        const float cf = last ? c : 1.0f;
        hipError_t e;
        if (ik == IN_BF16 && ok == OUT_F32)
            e = launch_pass_by_logr<IN_BF16, OUT_F32>(sizes[i], src, ld_src, dst, ld_dst, a.rows, a.cols, p, cf, s);
        else if (ik == IN_F32 && ok == OUT_F32)
            e = launch_pass_by_logr<IN_F32, OUT_F32>(sizes[i], src, ld_src, dst, ld_dst, a.rows, a.cols, p, cf, s);
        else if (ik == IN_F32 && ok == OUT_BF16)
            e = launch_pass_by_logr<IN_F32, OUT_BF16>(sizes[i], src, ld_src, dst, ld_dst, a.rows, a.cols, p, cf, s);
        else
            e = hipErrorInvalidValue;
        if (e != hipSuccess) return e;
        p += sizes[i];
    }
    return hipSuccess;
}

hipError_t launch_col_quant_t(const ColQuantArgs& a, hipStream_t s) {
    if (a.rows == 0 || a.cols == 0) return hipSuccess;
    uint32_t* amax_bits = reinterpret_cast<uint32_t*>(a.amax_ws);
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((a.cols + 255) / 256)), dim3(256), 0, s, amax_bits, a.cols, 0u);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 g1((unsigned)((a.cols + 255) / 256), (unsigned)((a.rows + kAmaxRows - 1) / kAmaxRows));
    hipLaunchKernelGGL(col_amax_kernel, g1, dim3(256), 0, s, reinterpret_cast<const uint16_t*>(a.in), a.ld_in,
                       a.rows, a.cols, a.fold, amax_bits);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 g2((unsigned)((a.cols + kTJ - 1) / kTJ), (unsigned)((a.rows + kTI - 1) / kTI));
    hipLaunchKernelGGL(col_quant_t_kernel, g2, dim3(256), 0, s, reinterpret_cast<const uint16_t*>(a.in), a.ld_in,
                       a.rows, a.cols, a.fold, amax_bits, a.out_q, a.ld_q, a.out_scale);
    return hipGetLastError();
}

}  // namespace halo
