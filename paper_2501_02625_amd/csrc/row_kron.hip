// Row transform with the Kronecker rotation H_{2^n} (x) H_28 (Section 2, "Hadamard Transformations": a dimension
// d = 2^n * m with a known Hadamard matrix of order m; 14336 = 512 * 28), fused with the same quantiser / un-rotation
// stores as the power-of-two row kernel.
//
// Element k = i * 28 + j of a Hadamard block has index i into the Walsh-Hadamard factor and j into H_28.  One thread owns
// the 28 consecutive elements of one i; a workgroup owns one row (cols / 28 threads, at most 512).  The order of the
// arithmetic, every add and subtract a separately rounded fp32 operation:
//   1. y_c = +-x_0 +- x_1 ... +- x_27 for each of the 28 columns c of H_28, a running sum in ascending index order, all in
//      the thread's registers (the signs are compile-time constants, so this is straight-line add/sub code);
//   2. the butterflies of H_{2^n} over i in ascending stride order: six stages across the lanes of a wavefront
//      (i's low six bits are the lane), then n - 6 stages across the wavefronts of the workgroup through LDS;
//   3. one multiply by 1/sqrt(28 * 2^n), then the optional per-column fold vector.
// H_28 is built at compile time by Paley's second construction from the quadratic character modulo 13: with
// Q[i][j] = chi(i - j) and the conference matrix C = [[0, 1^T], [1, Q]], every 0 of C becomes [[1, -1], [-1, -1]] and
// every +-1 becomes +-[[1, 1], [1, -1]].  It is symmetric, so rotating and un-rotating are the same transform.
//
// The lane stages use x <- x + s * partner(x) with s = -1 in the lane holding the upper element: that lane then
// carries the exact negation of the wanted difference, later stages pair elements with equal accumulated sign, and the
// sign (parity of the lane number) is folded into the normalisation multiply.
#pragma clang fp contract(off)

#include <utility>

#include "halo_internal.h"

namespace halo {
namespace {

constexpr int kM = 28;
constexpr float kRoundMagic = 12582912.0f;  // 1.5 * 2^23: adding it rounds |x| < 2^22 to an integer, ties to even

constexpr int chi13(int a) {
    a %= 13;
    if (a < 0) a += 13;
    if (a == 0) return 0;
    for (int t = 1; t < 13; ++t)
        if ((t * t) % 13 == a) return 1;
    return -1;
}

// Entry (r, c) of the order-28 Hadamard matrix.
constexpr int h28_entry(int r, int c) {
    const int i = r >> 1, j = c >> 1;
    const int conf = (i == 0 && j == 0) ? 0 : ((i == 0 || j == 0) ? 1 : chi13(i - j));
    const int u = r & 1, w = c & 1;
    if (conf == 0) return (u == 0 && w == 0) ? 1 : -1;        // [[1, -1], [-1, -1]]
    return conf * ((u == 1 && w == 1) ? -1 : 1);              // +-[[1, 1], [1, -1]]
}

template <int R, int C>
constexpr bool kPlus = h28_entry(R, C) > 0;

template <int C, int... J>
__device__ __forceinline__ float h28_column(const float (&x)[kM], std::integer_sequence<int, J...>) {
    float acc = kPlus<0, C> ? x[0] : -x[0];
    ((acc = kPlus<J + 1, C> ? acc + x[J + 1] : acc - x[J + 1]), ...);
    return acc;
}

template <int... C>
__device__ __forceinline__ void h28_mix(const float (&x)[kM], float (&y)[kM], std::integer_sequence<int, C...>) {
    ((y[C] = h28_column<C>(x, std::make_integer_sequence<int, kM - 1>{})), ...);
}

template <int J>
__device__ __forceinline__ float lane_xor(float x, int bperm_addr) {
    const int xi = __float_as_int(x);
    int r;
    if constexpr (J == 0) {
        r = __builtin_amdgcn_mov_dpp(xi, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
    } else if constexpr (J == 1) {
        r = __builtin_amdgcn_mov_dpp(xi, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
    } else if constexpr (J == 2) {
        r = __builtin_amdgcn_ds_swizzle(xi, 0x101F);              // bit mode: xor 4
    } else if constexpr (J == 3) {
        r = __builtin_amdgcn_mov_dpp(xi, 0x128, 0xF, 0xF, true);  // row_ror:8 == xor 8 inside a row of 16
    } else if constexpr (J == 4) {
        r = __builtin_amdgcn_ds_swizzle(xi, 0x401F);              // bit mode: xor 16
    } else {
        r = __builtin_amdgcn_ds_bpermute(bperm_addr, xi);         // lane ^ 32
    }
    return __int_as_float(r);
}

template <int J>
__device__ __forceinline__ void stage_across_lanes(float (&v)[kM], int lane, int bperm_addr) {
    const float s = ((lane >> J) & 1) ? -1.0f : 1.0f;
#pragma unroll
    for (int r = 0; r < kM; ++r) {
        const float p = lane_xor<J>(v[r], bperm_addr);
        v[r] = __builtin_fmaf(p, s, v[r]);      // the product is exact, so this is one rounded add or subtract
    }
}

// LOGP: log2 of the Walsh-Hadamard factor (6 .. 9); a Hadamard block is 28 * 2^LOGP elements = 2^(LOGP-6) wavefronts.
template <int IN, int OUT, int LOGP>
__global__ void __launch_bounds__(512)
row_kron28_kernel(RowArgs a, float c_norm, unsigned blocks1) {
    __shared__ float s_amax[8];
    extern __shared__ float s_xbuf[];        // [wavefronts][28][64]: exchange buffer of the stages across wavefronts

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bperm_addr = (lane ^ 32) << 2;
    unsigned block = blockIdx.x;
    if (block >= blocks1) {                  // the second matrix of a batched launch
        block -= blocks1;
        a.in = a.in2; a.pre_scale = a.pre_scale2; a.out = a.out2; a.out_scale = a.out_scale2; a.rows = a.rows2;
        if (a.given_amax2) a.given_amax = a.given_amax2;
        if (a.post_scale2) a.post_scale = a.post_scale2;
    }
    const int64_t row = block;               // the grid holds exactly one workgroup per row
    const int64_t k0 = (int64_t)tid * kM;

    float x[kM];
    if constexpr (IN == IN_BF16) {
        const uint2* src = reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(a.in) + row * a.ld_in + k0);
#pragma unroll
        for (int q = 0; q < kM / 4; ++q) {
            const uint2 w = src[q];
            x[4 * q + 0] = __uint_as_float(w.x << 16);
            x[4 * q + 1] = __uint_as_float(w.x & 0xFFFF0000u);
            x[4 * q + 2] = __uint_as_float(w.y << 16);
            x[4 * q + 3] = __uint_as_float(w.y & 0xFFFF0000u);
        }
    } else if constexpr (IN == IN_F32) {
        const float4* src = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(a.in) + row * a.ld_in + k0);
#pragma unroll
        for (int q = 0; q < kM / 4; ++q) {
            const float4 w = src[q];
            x[4 * q + 0] = w.x; x[4 * q + 1] = w.y; x[4 * q + 2] = w.z; x[4 * q + 3] = w.w;
        }
        if (a.in_mul != 0.0f) {
#pragma unroll
            for (int j = 0; j < kM; ++j) x[j] *= a.in_mul;
        }
    } else {
        const float pre = a.pre_scale ? a.pre_scale[row] : 1.0f;
        const int4* src = reinterpret_cast<const int4*>(reinterpret_cast<const int32_t*>(a.in) + row * a.ld_in + k0);
#pragma unroll
        for (int q = 0; q < kM / 4; ++q) {
            const int4 w = src[q];
            x[4 * q + 0] = (float)w.x * pre; x[4 * q + 1] = (float)w.y * pre;
            x[4 * q + 2] = (float)w.z * pre; x[4 * q + 3] = (float)w.w * pre;
        }
        if (a.post_scale) {                  // one more (tensor-wide) scale, applied after the per-row one
            const float post = *a.post_scale;
#pragma unroll
            for (int j = 0; j < kM; ++j) x[j] *= post;
        }
    }

    float v[kM];
    h28_mix(x, v, std::make_integer_sequence<int, kM>{});

    stage_across_lanes<0>(v, lane, bperm_addr);
    stage_across_lanes<1>(v, lane, bperm_addr);
    stage_across_lanes<2>(v, lane, bperm_addr);
    stage_across_lanes<3>(v, lane, bperm_addr);
    stage_across_lanes<4>(v, lane, bperm_addr);
    stage_across_lanes<5>(v, lane, bperm_addr);
#pragma unroll
    for (int xs = 0; xs < LOGP - 6; ++xs) {
        // stride 2^(6+xs) of i pairs this wavefront with wavefront ^ 2^xs (same Hadamard block: blocks are aligned
        // groups of 2^(LOGP-6) wavefronts); the lane signs carried so far are the same in both
        if (xs > 0) __syncthreads();         // everyone has read the previous round
#pragma unroll
        for (int j = 0; j < kM; ++j) s_xbuf[(wave * kM + j) * 64 + lane] = v[j];
        __syncthreads();
        const bool upper = (wave >> xs) & 1;
        const int pw = wave ^ (1 << xs);
#pragma unroll
        for (int j = 0; j < kM; ++j) {
            const float p = s_xbuf[(pw * kM + j) * 64 + lane];
            v[j] = upper ? p - v[j] : v[j] + p;
        }
    }
    const float c_l = (__builtin_popcount(lane) & 1) ? -c_norm : c_norm;
#pragma unroll
    for (int j = 0; j < kM; ++j) v[j] *= c_l;

    if (a.fold) {
        const float4* f = reinterpret_cast<const float4*>(a.fold + k0);
#pragma unroll
        for (int q = 0; q < kM / 4; ++q) {
            const float4 w = f[q];
            v[4 * q + 0] *= w.x; v[4 * q + 1] *= w.y; v[4 * q + 2] *= w.z; v[4 * q + 3] *= w.w;
        }
    }

    if constexpr (OUT == OUT_Q8) {
        float amax = 0.0f;
#pragma unroll
        for (int j = 0; j < kM; j += 2) asm("v_max3_f32 %0, %0, |%1|, |%2|" : "+v"(amax) : "v"(v[j]), "v"(v[j + 1]));
        amax = __builtin_fmaxf(amax, lane_xor<0>(amax, bperm_addr));
        amax = __builtin_fmaxf(amax, lane_xor<1>(amax, bperm_addr));
        amax = __builtin_fmaxf(amax, lane_xor<2>(amax, bperm_addr));
        amax = __builtin_fmaxf(amax, lane_xor<3>(amax, bperm_addr));
        amax = __builtin_fmaxf(amax, lane_xor<4>(amax, bperm_addr));
        amax = __builtin_fmaxf(amax, lane_xor<5>(amax, bperm_addr));
        const int waves = blockDim.x >> 6;
        if (waves > 1) {
            if (lane == 0) s_amax[wave] = amax;
            __syncthreads();
            float t = s_amax[0];
            for (int i = 1; i < waves; ++i) t = fmaxf(t, s_amax[i]);
            amax = t;
        }
        if (a.amax_only) {
            if (tid == 0) a.out_scale[row] = amax;
            return;
        }
        if (a.given_amax) amax = *a.given_amax;
        const bool nz = amax > 0.0f;
        const float inv = nz ? 127.0f / amax : 0.0f;
        if (tid == 0) a.out_scale[row] = nz ? amax / 127.0f : 1.0f;
        uint32_t* dst = reinterpret_cast<uint32_t*>(reinterpret_cast<int8_t*>(a.out) + row * a.ld_out + k0);
#pragma unroll
        for (int q = 0; q < kM / 4; ++q) {
            uint32_t b[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) b[e] = __float_as_uint(v[4 * q + e] * inv + kRoundMagic);
            const uint32_t lo = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u);
            const uint32_t hi = __builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u);
            dst[q] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
    } else if constexpr (OUT == OUT_BF16) {
        uint2* dst = reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + row * a.ld_out + k0);
#pragma unroll
        for (int q = 0; q < kM / 4; ++q)
            dst[q] = make_uint2(pack_bf16x2(v[4 * q], v[4 * q + 1]),
                                pack_bf16x2(v[4 * q + 2], v[4 * q + 3]));
    } else {
        float4* dst = reinterpret_cast<float4*>(reinterpret_cast<float*>(a.out) + row * a.ld_out + k0);
#pragma unroll
        for (int q = 0; q < kM / 4; ++q) dst[q] = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    }
}

template <int IN, int OUT, int LOGP>
hipError_t launch_logp(const RowArgs& a, hipStream_t s) {
    const int threads = (int)(a.cols / kM);
    const int64_t blocks = a.rows + a.rows2;
    const float c_norm = (float)(1.0 / sqrt((double)(kM << LOGP)));
    const size_t lds = LOGP > 6 ? (size_t)(threads / 64) * kM * 64 * sizeof(float) : 0;
    hipLaunchKernelGGL((row_kron28_kernel<IN, OUT, LOGP>), dim3((unsigned)blocks), dim3(threads), lds, s, a, c_norm,
                       (unsigned)a.rows);
    return hipGetLastError();
}

template <int IN, int OUT>
hipError_t launch_kind(const RowArgs& a, hipStream_t s) {
    switch (a.log_block) {
        case 6: return launch_logp<IN, OUT, 6>(a, s);
        case 7: return launch_logp<IN, OUT, 7>(a, s);
        case 8: return launch_logp<IN, OUT, 8>(a, s);
        case 9: return launch_logp<IN, OUT, 9>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool row_kron_shape_ok(int64_t cols, int64_t block) {
    if (block <= 0 || block % kM != 0) return false;
    const int64_t p = block / kM;
    if (!is_pow2(p) || p < 64 || p > 512) return false;
    return cols > 0 && cols % block == 0 && cols / kM <= 512;
}

hipError_t launch_row_kron(const RowArgs& a, InKind in, OutKind out, hipStream_t s) {
    if ((a.rows == 0 && a.rows2 == 0) || a.cols == 0) return hipSuccess;
    if (a.kron_m != kM || !row_kron_shape_ok(a.cols, (int64_t)kM << a.log_block)) return hipErrorInvalidValue;
    if (a.rows + a.rows2 > 0x7fffffffll) return hipErrorInvalidValue;
    if (in == IN_BF16 && out == OUT_Q8) return launch_kind<IN_BF16, OUT_Q8>(a, s);
    if (in == IN_F32 && out == OUT_Q8) return launch_kind<IN_F32, OUT_Q8>(a, s);
    if (in == IN_I32 && out == OUT_BF16) return launch_kind<IN_I32, OUT_BF16>(a, s);
    if (in == IN_I32 && out == OUT_F32) return launch_kind<IN_I32, OUT_F32>(a, s);
    if (in == IN_F32 && out == OUT_BF16) return launch_kind<IN_F32, OUT_BF16>(a, s);
    if (in == IN_F32 && out == OUT_F32) return launch_kind<IN_F32, OUT_F32>(a, s);
    return hipErrorInvalidValue;
}

}  // namespace halo
