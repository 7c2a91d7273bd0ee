// Kernels that work down the strided (row-index) axis of a row-major matrix:
//   * left-hand Walsh-Hadamard rotation  h'(A) = H^T A  over blocks of rows, done directly on strided data
//     (no transposes): each lane keeps 2^LOGR rows of one or two columns in registers, so all butterflies of
//     a pass are register-to-register and the memory accesses stay coalesced along the rows;
//   * the column-wise absmax INT8 quantiser with transposed output, (E^T)_Q;
//   * the dual quantiser: row-wise codes (E_Y)_Q and transposed column-wise codes (E_Y^T)_Q from one tiling of E.
#pragma clang fp contract(off)

#include <mutex>

#include "halo_internal.h"

namespace halo {
namespace {

// Scratch of the allocation-free dual quantiser (halo_quant_dual_static): partial maxima of pass 1.  One copy per GPU
// the library runs on, held until the process ends.  Host code never uses this name as an address: it asks the runtime
// for the device address once per device (static_scratch_address) and passes that to the kernels.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// ------------------------------------------------------------------------------------------------
// One pass of the left-hand FWHT: stages with row strides 2^p .. 2^(p+LOGR-1), ascending.
// A wavefront owns 64*CPL consecutive columns and the 2^LOGR rows  base + t*2^p.
// SIDE (bf16 input, first pass only): the pass also accumulates, per column, the absolute maximum of in[r, k] * side_fold[r]
// over all rows into side_amax (bit patterns of non-negative floats, atomic integer max; zeroed by the caller): what the
// column quantiser of the same matrix needs, taken from the one read of it.
template <int LOGR, int CPL, int IN, int OUT, bool SIDE = false>
__global__ void __launch_bounds__(256)
col_fwht_kernel(const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows, int64_t cols,
                int p, float c_final, int64_t col_tiles, const float* row_scale, const float* post_scale,
                const float* side_fold = nullptr, uint32_t* side_amax = nullptr) {
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
    // IN_I32: the scales of the wavefront's 2^LOGR rows, one per lane (lane t: row base + t * stride), handed out below
    // with v_readlane (the row is the same for every lane, a vector load per row would repeat one address 64 times).
    // Loaded before any lane leaves, so that every lane that is read from holds its value.
    float my_scale = 1.0f;
    if constexpr (IN == IN_I32) {
        if (row_scale && lane < R) my_scale = row_scale[base + (int64_t)lane * stride];
    }
    if constexpr (SIDE) {
        if (side_fold && lane < R) my_scale = side_fold[base + (int64_t)lane * stride];
    }
    if (col >= cols) return;
    const bool pair_ok = (CPL == 1) || (col + 1 < cols);
    float v[R][CPL];
    // Every load is issued before the first use, with one branch around the whole set and none inside it (a branch per row
    // makes the compiler wait for each load before it issues the next).
    if constexpr (IN == IN_BF16) {
        const uint16_t* src0 = reinterpret_cast<const uint16_t*>(in) + base * ld_in + col;
        if (CPL == 2 && pair_ok) {
            uint32_t w[R];
#pragma unroll
            for (int t = 0; t < R; ++t) w[t] = *reinterpret_cast<const uint32_t*>(src0 + (int64_t)t * stride * ld_in);
#pragma unroll
            for (int t = 0; t < R; ++t) {
                v[t][0] = __uint_as_float(w[t] << 16);
                v[t][CPL - 1] = __uint_as_float(w[t] & 0xFFFF0000u);
            }
        } else {
            uint16_t w[R];
#pragma unroll
            for (int t = 0; t < R; ++t) w[t] = src0[(int64_t)t * stride * ld_in];
#pragma unroll
            for (int t = 0; t < R; ++t) {
                if (CPL == 2) v[t][CPL - 1] = 0.0f;
                v[t][0] = __uint_as_float((uint32_t)w[t] << 16);
            }
        }
    } else if constexpr (IN == IN_F32) {
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const float* src = reinterpret_cast<const float*>(in) + (base + t * stride) * ld_in + col;
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

    if constexpr (SIDE) {
        float mx[CPL];
#pragma unroll
        for (int c = 0; c < CPL; ++c) mx[c] = 0.0f;
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const float f = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_scale), t));
#pragma unroll
            for (int c = 0; c < CPL; ++c) mx[c] = fmaxf(mx[c], fabsf(v[t][c] * f));
        }
#pragma unroll
        for (int c = 0; c < CPL; ++c)
            if (col + c < cols && mx[c] > 0.0f) atomicMax(side_amax + col + c, __float_as_uint(mx[c]));
    }

    if constexpr (IN == IN_I32) {
        // accumulators of a product: (float(acc) * scale of the row) * tensor-wide scale, as the row kernel does.  Every
        // load is issued before the first conversion (one branch around the whole set, none inside it).
        int raw[R][CPL];
        const int32_t* src0 = reinterpret_cast<const int32_t*>(in) + base * ld_in + col;
        if (CPL == 2 && pair_ok) {
#pragma unroll
            for (int t = 0; t < R; ++t) {
                const int2 w = *reinterpret_cast<const int2*>(src0 + (int64_t)t * stride * ld_in);
                raw[t][0] = w.x; raw[t][CPL - 1] = w.y;
            }
        } else {
#pragma unroll
            for (int t = 0; t < R; ++t) {
                raw[t][0] = src0[(int64_t)t * stride * ld_in];
                if (CPL == 2) raw[t][CPL - 1] = 0;
            }
        }
        const float post = post_scale ? *post_scale : 1.0f;         // x * 1.0f is x
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const float rs = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_scale), t));
#pragma unroll
            for (int c = 0; c < CPL; ++c) v[t][c] = ((float)raw[t][c] * rs) * post;
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

    if constexpr (OUT == OUT_F32) {
        float* dst0 = reinterpret_cast<float*>(out) + base * ld_out + col;
        if (CPL == 2 && pair_ok) {
#pragma unroll
            for (int t = 0; t < R; ++t)
                *reinterpret_cast<float2*>(dst0 + (int64_t)t * stride * ld_out) = make_float2(v[t][0], v[t][CPL - 1]);
        } else {
#pragma unroll
            for (int t = 0; t < R; ++t) dst0[(int64_t)t * stride * ld_out] = v[t][0];
        }
    } else {
        uint16_t* dst0 = reinterpret_cast<uint16_t*>(out) + base * ld_out + col;
        if (CPL == 2 && pair_ok) {
#pragma unroll
            for (int t = 0; t < R; ++t)
                *reinterpret_cast<uint32_t*>(dst0 + (int64_t)t * stride * ld_out) = pack_bf16x2(v[t][0], v[t][CPL - 1]);
        } else {
#pragma unroll
            for (int t = 0; t < R; ++t) dst0[(int64_t)t * stride * ld_out] = bf16_bits(v[t][0]);
        }
    }
}

template <int LOGR, int CPL, int IN, int OUT>
hipError_t launch_pass(const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows, int64_t cols,
                       int p, float c_final, hipStream_t s, const float* row_scale, const float* post_scale) {
    const int64_t col_tiles = (cols + 256 * CPL - 1) / (256 * CPL);
    const int64_t groups = rows >> LOGR;
    const int64_t blocks = col_tiles * groups;
    if (blocks <= 0 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL((col_fwht_kernel<LOGR, CPL, IN, OUT>), dim3((unsigned)blocks), dim3(256), 0, s, in, ld_in,
                       out, ld_out, rows, cols, p, c_final, col_tiles, row_scale, post_scale);
    return hipGetLastError();
}

// First pass with the side absmax: bf16 in, six stages, fp32 out.
hipError_t launch_pass_side(const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows, int64_t cols, float c_final,
                            hipStream_t s, const float* side_fold, uint32_t* side_amax) {
    const int64_t col_tiles = (cols + 511) / 512;
    const int64_t blocks = col_tiles * (rows >> 6);
    if (blocks <= 0 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL((col_fwht_kernel<6, 2, IN_BF16, OUT_F32, true>), dim3((unsigned)blocks), dim3(256), 0, s, in, ld_in, out,
                       ld_out, rows, cols, 0, c_final, col_tiles, nullptr, nullptr, side_fold, side_amax);
    return hipGetLastError();
}

template <int IN, int OUT>
hipError_t launch_pass_by_logr(int logr, const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows,
                               int64_t cols, int p, float c_final, hipStream_t s, const float* row_scale = nullptr,
                               const float* post_scale = nullptr) {
    switch (logr) {
        case 1: return launch_pass<1, 2, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s, row_scale, post_scale);
        case 2: return launch_pass<2, 2, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s, row_scale, post_scale);
        case 3: return launch_pass<3, 2, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s, row_scale, post_scale);
        case 4: return launch_pass<4, 2, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s, row_scale, post_scale);
        case 5: return launch_pass<5, 2, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s, row_scale, post_scale);
        case 6: return launch_pass<6, 2, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s, row_scale, post_scale);
        case 7:
            if constexpr (IN == IN_F32) return launch_pass<7, 1, IN, OUT>(in, ld_in, out, ld_out, rows, cols, p, c_final, s, row_scale, post_scale);
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

// out[0] = max over in[0..n-1]: one workgroup (the vectors reduced here are per-row maxima, a few thousand entries).
__global__ void __launch_bounds__(1024) reduce_max_kernel(const float* in, int64_t n, float* out, const float* in2, int64_t n2,
                                                          float* out2) {
    __shared__ float s_part[16];
    if (blockIdx.x == 1) { in = in2; n = n2; out = out2; }     // the second vector of a paired launch
    float m = 0.0f;
    for (int64_t i = threadIdx.x; i < n; i += 1024) m = fmaxf(m, in[i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = s_part[0];
        for (int i = 1; i < 16; ++i) t = fmaxf(t, s_part[i]);
        out[0] = t;
    }
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
                   const uint32_t* amax_bits, int8_t* out_q, int64_t ld_q, float* out_scale, const float* given_amax = nullptr) {
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
            if (col + e < cols) am = given_amax ? *given_amax : __uint_as_float(amax_bits[col + e]);   // one maximum for all columns
            inv[e] = am > 0.0f ? 127.0f / am : 0.0f;
            if (blockIdx.y == 0 && tid < 32 && col + e < cols) out_scale[col + e] = am > 0.0f ? am / 127.0f : 1.0f;
        }
        // The 16 rows of this thread (4 quads of 4): all loads first.  A tile inside the matrix takes them with no branch in
        // between (a branch per row makes the compiler wait for each load before it issues the next); a tile on the edge
        // goes element by element.
        uint2 w[4][4];
        float f[4][4];
        const bool interior = i0 + kTI <= rows && j0 + kTJ <= cols;
        if (interior) {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int64_t row = i0 + 4 * ((tid >> 5) + 8 * s) + r;
                    w[s][r] = *reinterpret_cast<const uint2*>(in + row * ld_in + col);
                }
            if (fold) {
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int r = 0; r < 4; ++r) f[s][r] = fold[i0 + 4 * ((tid >> 5) + 8 * s) + r];
            } else {
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int r = 0; r < 4; ++r) f[s][r] = 1.0f;
            }
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int64_t row = i0 + 4 * ((tid >> 5) + 8 * s) + r;
                    uint32_t h[4] = {0u, 0u, 0u, 0u};
                    f[s][r] = 1.0f;
                    if (row < rows) {
                        if (fold) f[s][r] = fold[row];
                        for (int e = 0; e < 4; ++e)
                            if (col + e < cols) h[e] = in[row * ld_in + col + e];
                    }
                    w[s][r] = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                }
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int iq = (tid >> 5) + 8 * s;           // row quad inside the tile
            uint32_t b[4][4];                             // [row in quad][col]
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float x[4] = {__uint_as_float(w[s][r].x << 16), __uint_as_float(w[s][r].x & 0xFFFF0000u),
                                    __uint_as_float(w[s][r].y << 16), __uint_as_float(w[s][r].y & 0xFFFF0000u)};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float t = (x[e] * f[s][r]) * inv[e];
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


// ------------------------------------------------------------------------------------------------
// Both quantisations of E that the backward pass needs, from one tiling of E:
//   rows:  Eq [b x n]  = Q_row( E[i,j] * fold_c[j] )   (the saved weight scales folded in; feeds E_X = E W)
//   cols:  EqT [n x b] = Q_row( (E[i,j] * fold_r[i])^T ) (the saved activation scales folded in; feeds G = E^T X)
// Pass 1 writes the partial maxima of both absmax vectors per tile (no atomics); pass 2 reduces the partials it needs,
// re-reads E (cache-hot), emits the row-wise codes directly and the column-wise codes through an LDS transpose.
constexpr int kAC = 256;                                         // absmax pass: tile columns (tile rows: 32 per round)
constexpr int kDR = 128, kDC = 128, kDPitch = kDR / 4 + 1;     // quantising pass: tile rows, columns, LDS dwords per column

__device__ __forceinline__ float max_across_32(float x) {
    // max over the 32 lanes that share (lane >> 5)
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0xB1, 0xF, 0xF, true)));
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0x4E, 0xF, 0xF, true)));
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), 0x101F)));
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0x128, 0xF, 0xF, true)));
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), 0x401F)));
    return x;
}

// The 8 bf16 of E at (row, col .. col+7) as four dwords; out-of-range elements are zero.
__device__ __forceinline__ uint4 load_row8(const uint16_t* __restrict__ in, int64_t ld_in, int64_t rows, int64_t cols,
                                           int64_t row, int64_t col) {
    uint4 w = make_uint4(0u, 0u, 0u, 0u);
    if (row < rows && col < cols) {
        const uint16_t* src = in + row * ld_in + col;
        if (col + 8 <= cols) {
            w = *reinterpret_cast<const uint4*>(src);
        } else {
            uint32_t h[8];
            for (int e = 0; e < 8; ++e) h[e] = col + e < cols ? (uint32_t)src[e] : 0u;
            w = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
        }
    }
    return w;
}

__device__ __forceinline__ void widen_row8(const uint4& w, float (&x)[8]) {
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[2 * i] = __uint_as_float(ww[i] << 16);
        x[2 * i + 1] = __uint_as_float(ww[i] & 0xFFFF0000u);
    }
}

// Pass 1: every workgroup writes the partial maxima of its (32 * ROUNDS) x 256 tile (no atomics: device-scope atomics
// are resolved beyond the per-XCD L2 and cost more than the whole pass): row_part[row][column tile],
// col_part[row tile][col].  A thread owns 8 columns of 4 * ROUNDS rows and issues all its loads before the first use;
// taller tiles leave pass 2 fewer partial maxima to reduce, shorter ones fill the chip when E is small.
template <int ROUNDS>
__global__ void __launch_bounds__(256)
dual_amax_kernel(const uint16_t* __restrict__ in, int64_t ld_in, int64_t rows, int64_t cols,
                 const float* __restrict__ fold_c, const float* __restrict__ fold_r, float* __restrict__ row_part,
                 float* __restrict__ col_part) {
    __shared__ float s_col[8][kAC];
    const int tid = threadIdx.x, lane = tid & 63;
    const int jl = tid & 31, rq = tid >> 5;             // 32 column groups of 8, 8 row quads per round of 32 rows
    const int64_t col = (int64_t)blockIdx.x * kAC + 8 * jl;
    const int64_t row_base = (int64_t)blockIdx.y * (32 * ROUNDS) + 4 * rq;
    uint4 raw[ROUNDS][4];
    float frow[ROUNDS][4];
    // a tile inside the matrix takes its loads with no branch in between (a branch per load makes the compiler wait for
    // each before it issues the next)
    const bool interior = (int64_t)(blockIdx.y + 1) * (32 * ROUNDS) <= rows && (int64_t)(blockIdx.x + 1) * kAC <= cols;
    if (interior) {
#pragma unroll
        for (int s = 0; s < ROUNDS; ++s)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                raw[s][r] = *reinterpret_cast<const uint4*>(in + (row_base + 32 * s + r) * ld_in + col);
        if (fold_r) {
#pragma unroll
            for (int s = 0; s < ROUNDS; ++s)
#pragma unroll
                for (int r = 0; r < 4; ++r) frow[s][r] = fold_r[row_base + 32 * s + r];
        } else {
#pragma unroll
            for (int s = 0; s < ROUNDS; ++s)
#pragma unroll
                for (int r = 0; r < 4; ++r) frow[s][r] = 1.0f;
        }
    } else {
#pragma unroll
        for (int s = 0; s < ROUNDS; ++s)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t row = row_base + 32 * s + r;
                raw[s][r] = load_row8(in, ld_in, rows, cols, row, col);
                frow[s][r] = (fold_r && row < rows) ? fold_r[row] : 1.0f;
            }
    }
    float fc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) fc[e] = (fold_c && col + e < cols) ? fold_c[col + e] : 1.0f;
    float cmax[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < ROUNDS; ++s) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t row = row_base + 32 * s + r;
            const float fr = frow[s][r];
            float x[8];
            widen_row8(raw[s][r], x);
            float rmax = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                rmax = fmaxf(rmax, fabsf(x[e] * fc[e]));
                cmax[e] = fmaxf(cmax[e], fabsf(x[e] * fr));
            }
            rmax = max_across_32(rmax);
            if ((lane & 31) == 0 && row < rows) row_part[row * gridDim.x + blockIdx.x] = rmax;
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) s_col[rq][8 * jl + e] = cmax[e];
    __syncthreads();
    {
        float t = s_col[0][tid];
#pragma unroll
        for (int q = 1; q < 8; ++q) t = fmaxf(t, s_col[q][tid]);
        const int64_t c = (int64_t)blockIdx.x * kAC + tid;
        if (c < cols) col_part[(int64_t)blockIdx.y * cols + c] = t;
    }
}

__global__ void __launch_bounds__(256)
dual_quant_kernel(const uint16_t* __restrict__ in, int64_t ld_in, int64_t rows, int64_t cols,
                  const float* __restrict__ fold_c, const float* __restrict__ fold_r, const float* __restrict__ row_part,
                  const float* __restrict__ col_part, int col_tiles, int row_tiles, int8_t* __restrict__ out_q, int64_t ld_q,
                  float* __restrict__ row_scale, int8_t* __restrict__ out_qt, int64_t ld_qt, float* __restrict__ col_scale) {
    __shared__ uint32_t s_tile[kDC * kDPitch];
    __shared__ float s_red[2][2][128];     // [row/col][half][index]
    __shared__ float s_amax_c[kDC], s_amax_r[kDR];
    const int tid = threadIdx.x;
    const int jl = tid & 15, rq = tid >> 4;             // 16 column groups of 8, 16 row quads (two rounds)
    const int64_t j0 = (int64_t)blockIdx.x * kDC, i0 = (int64_t)blockIdx.y * kDR;
    const int64_t col = j0 + 8 * jl;
    // E first (cache-hot after pass 1): all eight loads of the thread are in flight while the maxima are reduced.
    uint4 raw[2][4];
    float frow[2][4];
    const bool interior = i0 + kDR <= rows && j0 + kDC <= cols;
    if (interior) {                        // no branch between the loads
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                raw[s][r] = *reinterpret_cast<const uint4*>(in + (i0 + 4 * (rq + 16 * s) + r) * ld_in + col);
        if (fold_r) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int r = 0; r < 4; ++r) frow[s][r] = fold_r[i0 + 4 * (rq + 16 * s) + r];
        } else {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int r = 0; r < 4; ++r) frow[s][r] = 1.0f;
        }
    } else {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t row = i0 + 4 * (rq + 16 * s) + r;
                raw[s][r] = load_row8(in, ld_in, rows, cols, row, col);
                frow[s][r] = (fold_r && row < rows) ? fold_r[row] : 1.0f;
            }
    }
    // Absmax of this tile's 128 columns and 128 rows from the partial maxima of pass 1 (every workgroup redoes the
    // reduction it needs: a few KB of L2 hits instead of one more kernel between the passes).
    {
        const int o = tid & 127, h = tid >> 7;
        float tc = 0.0f, tr = 0.0f;
        if (j0 + o < cols) {
#pragma unroll 16
            for (int q = h; q < row_tiles; q += 2) tc = fmaxf(tc, col_part[(int64_t)q * cols + j0 + o]);
        }
        if (i0 + o < rows) {
#pragma unroll 8
            for (int q = h; q < col_tiles; q += 2) tr = fmaxf(tr, row_part[(i0 + o) * col_tiles + q]);
        }
        s_red[0][h][o] = tc;
        s_red[1][h][o] = tr;
        __syncthreads();
        if (tid < 128) {
            const float am = fmaxf(s_red[0][0][tid], s_red[0][1][tid]);
            s_amax_c[tid] = am;
            if (blockIdx.y == 0 && j0 + tid < cols) col_scale[j0 + tid] = am > 0.0f ? am / 127.0f : 1.0f;
        } else {
            const int r = tid - 128;
            const float am = fmaxf(s_red[1][0][r], s_red[1][1][r]);
            s_amax_r[r] = am;
            if (blockIdx.x == 0 && i0 + r < rows) row_scale[i0 + r] = am > 0.0f ? am / 127.0f : 1.0f;
        }
        __syncthreads();
    }
    float fc[8], inv_c[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const bool ok = col + e < cols;
        fc[e] = (fold_c && ok) ? fold_c[col + e] : 1.0f;
        const float am = s_amax_c[8 * jl + e];
        inv_c[e] = am > 0.0f ? 127.0f / am : 0.0f;
    }
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int iq = rq + 16 * s;
        const int64_t row0 = i0 + 4 * iq;
        float x[4][8];
#pragma unroll
        for (int r = 0; r < 4; ++r) widen_row8(raw[s][r], x[r]);
        uint32_t bc[4][8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t row = row0 + r;
            const bool rok = row < rows;
            const float fr = frow[s][r];
            const float am = s_amax_r[4 * iq + r];
            const float inv_r = am > 0.0f ? 127.0f / am : 0.0f;
            uint32_t br[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                br[e] = __float_as_uint((x[r][e] * fc[e]) * inv_r + 12582912.0f);
                bc[r][e] = __float_as_uint((x[r][e] * fr) * inv_c[e] + 12582912.0f);
            }
            if (rok && col < cols) {
                const uint32_t p0 = __builtin_amdgcn_perm(__builtin_amdgcn_perm(br[3], br[2], 0x0c0c0400u),
                                                          __builtin_amdgcn_perm(br[1], br[0], 0x0c0c0400u), 0x05040100u);
                const uint32_t p1 = __builtin_amdgcn_perm(__builtin_amdgcn_perm(br[7], br[6], 0x0c0c0400u),
                                                          __builtin_amdgcn_perm(br[5], br[4], 0x0c0c0400u), 0x05040100u);
                int8_t* dst = out_q + row * ld_q + col;
                if (col + 8 <= cols) {
                    *reinterpret_cast<uint2*>(dst) = make_uint2(p0, p1);
                } else {
                    for (int e = 0; e < 8; ++e)
                        if (col + e < cols) dst[e] = (int8_t)(((e < 4 ? p0 : p1) >> (8 * (e & 3))) & 0xFF);
                }
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t lo = __builtin_amdgcn_perm(bc[1][e], bc[0][e], 0x0c0c0400u);
            const uint32_t hi = __builtin_amdgcn_perm(bc[3][e], bc[2][e], 0x0c0c0400u);
            s_tile[(8 * jl + e) * kDPitch + iq] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
    }
    __syncthreads();
    {
        const int seg = tid & 7;
#pragma unroll
        for (int s = 0; s < kDC / 32; ++s) {
            const int jj = (tid >> 3) + 32 * s;
            const int64_t c = j0 + jj;
            if (c >= cols) continue;
            uint32_t w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) w[q] = s_tile[jj * kDPitch + 4 * seg + q];
            const int64_t i = i0 + 16 * seg;
            int8_t* dst = out_qt + c * ld_qt + i;
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
    if (a.first_stage < 0 || a.first_stage > a.log_block) return hipErrorInvalidValue;
    // split the remaining stages into passes of at most 6 (a final 7 is allowed for fp32 input)
    int sizes[8], np = 0, left = a.log_block - a.first_stage;
    if (left == 0) return (a.in == a.out && a.skip_norm) ? hipSuccess : hipErrorInvalidValue;   // nothing left to do in place
    while (left > 0) {
        int q = left <= 6 ? left : (left == 7 && np > 0 ? 7 : 6);
        sizes[np++] = q;
        left -= q;
        if (np >= 8) return hipErrorInvalidValue;
    }
    const float c = a.skip_norm ? 1.0f : (float)(1.0 / sqrt((double)(int64_t(1) << a.log_block)));
    int p = a.first_stage;
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
        if (first && a.side_amax) {
            // only the shape the layer uses: bf16 in, a first pass of six stages from stage 0
            if (ik != IN_BF16 || ok != OUT_F32 || sizes[i] != 6 || p != 0) return hipErrorInvalidValue;
            e = launch_pass_side(src, ld_src, dst, ld_dst, a.rows, a.cols, cf, s, a.side_fold, a.side_amax);
        } else if (ik == IN_BF16 && ok == OUT_F32)
            e = launch_pass_by_logr<IN_BF16, OUT_F32>(sizes[i], src, ld_src, dst, ld_dst, a.rows, a.cols, p, cf, s);
        else if (ik == IN_F32 && ok == OUT_F32)
            e = launch_pass_by_logr<IN_F32, OUT_F32>(sizes[i], src, ld_src, dst, ld_dst, a.rows, a.cols, p, cf, s);
        else if (ik == IN_F32 && ok == OUT_BF16)
            e = launch_pass_by_logr<IN_F32, OUT_BF16>(sizes[i], src, ld_src, dst, ld_dst, a.rows, a.cols, p, cf, s);
        else if (ik == IN_I32 && ok == OUT_F32)
            e = launch_pass_by_logr<IN_I32, OUT_F32>(sizes[i], src, ld_src, dst, ld_dst, a.rows, a.cols, p, cf, s, a.row_scale,
                                                     a.post_scale);
        else
            e = hipErrorInvalidValue;
        if (e != hipSuccess) return e;
        p += sizes[i];
    }
    return hipSuccess;
}

// Rounds of 32 rows per workgroup of the absmax pass: the tallest tile that still gives the chip two workgroups per
// compute unit.
static int dual_amax_rounds(int64_t rows, int64_t cols) {
    const int64_t col_tiles = (cols + kAC - 1) / kAC;
    for (int r = 4; r > 1; r >>= 1)
        if (col_tiles * ((rows + 32 * r - 1) / (32 * r)) >= 512) return r;
    return 1;
}

size_t dual_quant_workspace_floats(int64_t rows, int64_t cols) {
    const int64_t col_tiles = (cols + kAC - 1) / kAC, row_tiles = (rows + 31) / 32;     // sized for one-round tiles
    return (size_t)(rows * col_tiles + row_tiles * cols);
}

hipError_t launch_dual_quant(const DualQuantArgs& a, hipStream_t s) {
    if (a.rows == 0 || a.cols == 0) return hipSuccess;
    const int rounds = dual_amax_rounds(a.rows, a.cols);
    const int64_t col_tiles = (a.cols + kAC - 1) / kAC, row_tiles = (a.rows + 32 * rounds - 1) / (32 * rounds);
    float* row_part = a.amax_ws;                                           // [rows][col_tiles]
    float* col_part = row_part + a.rows * col_tiles;                       // [row_tiles][cols]
    const dim3 grid_a((unsigned)col_tiles, (unsigned)row_tiles);
    const dim3 grid((unsigned)((a.cols + kDC - 1) / kDC), (unsigned)((a.rows + kDR - 1) / kDR));
    const uint16_t* in = reinterpret_cast<const uint16_t*>(a.in);
    auto* amax = rounds == 4 ? dual_amax_kernel<4> : rounds == 2 ? dual_amax_kernel<2> : dual_amax_kernel<1>;
    hipLaunchKernelGGL(amax, grid_a, dim3(256), 0, s, in, a.ld_in, a.rows, a.cols, a.fold_c, a.fold_r, row_part, col_part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(dual_quant_kernel, grid, dim3(256), 0, s, in, a.ld_in, a.rows, a.cols, a.fold_c, a.fold_r, row_part,
                       col_part, (int)col_tiles, (int)row_tiles, a.out_q, a.ld_q, a.row_scale, a.out_qt, a.ld_qt, a.col_scale);
    return hipGetLastError();
}

// Device address of `scratch` on the current device, looked up on the first call for that device and kept.
hipError_t static_scratch_address(void** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* address[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!address[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        address[dev] = p;
    }
    *out = address[dev];
    return hipSuccess;
}

hipError_t launch_dual_quant_static(DualQuantArgs a, hipStream_t s) {
    if (a.rows == 0 || a.cols == 0) return hipSuccess;
    if (dual_quant_workspace_floats(a.rows, a.cols) * sizeof(float) > kStaticScratchBytes) return hipErrorInvalidValue;
    void* p = nullptr;
    hipError_t e = static_scratch_address(&p);
    if (e != hipSuccess) return e;
    a.amax_ws = reinterpret_cast<float*>(p);     // every entry pass 2 reads is written by pass 1 first: nothing to clear
    return launch_dual_quant(a, s);
}

hipError_t launch_reduce_max(const float* in, int64_t n, float* out, hipStream_t s, const float* in2, int64_t n2, float* out2) {
    if (n <= 0 || (in2 && n2 <= 0)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(reduce_max_kernel, dim3(in2 ? 2 : 1), dim3(1024), 0, s, in, n, out, in2, n2, out2);
    return hipGetLastError();
}

hipError_t launch_col_quant_t_given(const ColQuantArgs& a, const float* given_amax, hipStream_t s) {
    if (a.rows == 0 || a.cols == 0) return hipSuccess;
    const dim3 g2((unsigned)((a.cols + kTJ - 1) / kTJ), (unsigned)((a.rows + kTI - 1) / kTI));
    hipLaunchKernelGGL(col_quant_t_kernel, g2, dim3(256), 0, s, reinterpret_cast<const uint16_t*>(a.in), a.ld_in,
                       a.rows, a.cols, a.fold, static_cast<const uint32_t*>(nullptr), a.out_q, a.ld_q, a.out_scale, given_amax);
    return hipGetLastError();
}

hipError_t launch_zero_u32(uint32_t* p, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n, 0u);
    return hipGetLastError();
}

hipError_t launch_col_quant_t_ready(const ColQuantArgs& a, hipStream_t s) {
    if (a.rows == 0 || a.cols == 0) return hipSuccess;
    const dim3 g2((unsigned)((a.cols + kTJ - 1) / kTJ), (unsigned)((a.rows + kTI - 1) / kTI));
    hipLaunchKernelGGL(col_quant_t_kernel, g2, dim3(256), 0, s, reinterpret_cast<const uint16_t*>(a.in), a.ld_in,
                       a.rows, a.cols, a.fold, reinterpret_cast<const uint32_t*>(a.amax_ws), a.out_q, a.ld_q, a.out_scale);
    return hipGetLastError();
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
