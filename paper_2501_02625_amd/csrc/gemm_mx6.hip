// MXFP6 GEMM on the CDNA4 scaled matrix instruction v_mfma_scale_f32_16x16x128_f8f6f4 with both operands in FP6 E3M2
// (format selector 3) and one E8M0 scale per block of 32 elements along K:  C = A B^T, fp32 accumulation.
//
// Operand layout of the instruction (established with a one-tile numeric probe against an exact reference): lane l
// supplies the 32 consecutive K-elements of row (l % 16) that start at K offset 32 * (l / 16), i.e. exactly one
// scaling block, as 192 bits packed least-significant element first in six registers, plus that block's E8M0 byte in
// byte 0 of the scale register.  Accumulator: lane l holds column (l % 16), rows 4 * (l / 16) + r, r = 0..3.
// So the packed codes in memory ([row][block][24 bytes]) are the register image: a lane loads its block with three
// 8-byte loads straight from global memory, no LDS stage, no shuffle.
//
// Workgroup = 4 wavefronts (2 x 2), macro tile 128 x 128, each wavefront 64 x 64 = 4 x 4 instruction tiles; K step 128.
// The operands of K step t+1 are requested before the sixteen instructions of step t are issued.
#include "halo_internal.h"

namespace halo {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kFmtE3M2 = 3;     // "bf6" in the instruction's format field (0 E4M3, 1 E5M2, 2 E2M3, 3 E3M2, 4 E2M1)

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

struct Mx6Frag {
    uint2 d[3];        // the 24 bytes of one block
    uint32_t scales;   // the four scale bytes of the row's K step; byte (lane / 16) is this lane's
};

__device__ __forceinline__ void load_frag(const uint8_t* codes, const uint8_t* scales, int kt, Mx6Frag& f) {
    const uint2* p = reinterpret_cast<const uint2*>(codes + (int64_t)kt * 96);
    f.d[0] = p[0]; f.d[1] = p[1]; f.d[2] = p[2];
    f.scales = *reinterpret_cast<const uint32_t*>(scales + (int64_t)kt * 4);
}

__device__ __forceinline__ v8i operand(const Mx6Frag& f) {
    return v8i{(int)f.d[0].x, (int)f.d[0].y, (int)f.d[1].x, (int)f.d[1].y, (int)f.d[2].x, (int)f.d[2].y, 0, 0};
}

__global__ void __launch_bounds__(256) gemm_mx6_kernel(Mx6GemmArgs a, int tiles_n) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int r16 = lane & 15, g = lane >> 4;
    const int64_t m0 = (int64_t)(blockIdx.x / tiles_n) * 128 + wave_m * 64;
    const int64_t n0 = (int64_t)(blockIdx.x % tiles_n) * 128 + wave_n * 64;
    const int nk = (int)(a.K / 128);

    const uint8_t* pa[4]; const uint8_t* psa[4];
    const uint8_t* pb[4]; const uint8_t* psb[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        int64_t row = m0 + t * 16 + r16;
        row = row < a.M ? row : a.M - 1;                 // clamped rows are computed and never stored
        pa[t] = a.A + row * a.lda + g * 24;
        psa[t] = a.SA + row * a.ldsa;
        int64_t col = n0 + t * 16 + r16;
        col = col < a.N ? col : a.N - 1;
        pb[t] = a.B + col * a.ldb + g * 24;
        psb[t] = a.SB + col * a.ldsb;
    }

    v4f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    Mx6Frag fa[2][4], fb[2][4];
    if (nk > 0) {
#pragma unroll
        for (int t = 0; t < 4; ++t) { load_frag(pa[t], psa[t], 0, fa[0][t]); load_frag(pb[t], psb[t], 0, fb[0][t]); }
    }
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                load_frag(pa[t], psa[t], kt + 1, fa[cur ^ 1][t]);
                load_frag(pb[t], psb[t], kt + 1, fb[cur ^ 1][t]);
            }
        }
        v8i va[4], vb[4];
        int sa[4], sb[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            va[t] = operand(fa[cur][t]); vb[t] = operand(fb[cur][t]);
            sa[t] = (int)((fa[cur][t].scales >> (8 * g)) & 0xFFu);
            sb[t] = (int)((fb[cur][t].scales >> (8 * g)) & 0xFFu);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(va[i], vb[j], acc[i][j], kFmtE3M2, kFmtE3M2,
                                                                             0, sa[i], 0, sb[j]);
    }

#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t col = n0 + j * 16 + r16;
            if (col >= a.N) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t row = m0 + i * 16 + 4 * g + r;
                if (row >= a.M) continue;
                if (a.c_is_f32) reinterpret_cast<float*>(a.C)[row * a.ldc + col] = acc[i][j][r];
                else reinterpret_cast<uint16_t*>(a.C)[row * a.ldc + col] = (uint16_t)f32_to_bf16_rne(acc[i][j][r]);
            }
        }
}

}  // namespace

hipError_t launch_gemm_mx6(const Mx6GemmArgs& a, hipStream_t s) {
    if (a.M == 0 || a.N == 0) return hipSuccess;
    if (a.K % 128 != 0) return hipErrorInvalidValue;
    const int64_t tiles_m = (a.M + 127) / 128, tiles_n = (a.N + 127) / 128;
    if (tiles_m * tiles_n > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gemm_mx6_kernel, dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 0, s, a, (int)tiles_n);
    return hipGetLastError();
}

}  // namespace halo
