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
// Workgroup = 4 wavefronts (2 x 2), macro tile 128 x 128, each wavefront 64 x 64 = 4 x 4 instruction tiles; K step 128
// elements = 96 code bytes + 4 scale bytes per row.  Two LDS stages: the 256 rows of a K step (128 of A, 128 of B) lie
// at a pitch of 112 bytes (28 dwords: the sixteen rows one quarter-wavefront reads fall on sixteen different groups of
// four banks), the scale dwords behind them.  The next K step travels global -> registers (six 16-byte loads and one
// scale dword per thread) while the current one is multiplied, then registers -> LDS, one barrier per K step.  A lane
// reads its block as three 8-byte LDS loads: the code bytes in memory are the register image, nothing is unpacked.
#include "halo_internal.h"

namespace halo {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kFmtE3M2 = 3;     // "bf6" in the instruction's format field (0 E4M3, 1 E5M2, 2 E2M3, 3 E3M2, 4 E2M1)
constexpr int kPitch = 112;                         // LDS bytes per row and K step
constexpr int kCodeBytes = 256 * kPitch;            // 128 rows of A, then 128 rows of B
constexpr int kStageBytes = kCodeBytes + 256 * 4;   // + one dword of four scale bytes per row

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__global__ void __launch_bounds__(256, 2) gemm_mx6_kernel(Mx6GemmArgs a, int tiles_n) {
    __shared__ __align__(16) unsigned char smem[2 * kStageBytes];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int r16 = lane & 15, g = lane >> 4;
    const int64_t m0 = (int64_t)(blockIdx.x / tiles_n) * 128;
    const int64_t n0 = (int64_t)(blockIdx.x % tiles_n) * 128;
    const int nk = (int)(a.K / 128);

    // ---- what this thread moves per K step: six 16-byte chunks of the 256 x 96 code bytes, one scale dword
    const uint8_t* src[6];
    int dst[6];
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        const int q = tid + i * 256;                 // chunk number: row = q / 6, chunk of the row = q % 6
        const int row = q / 6, c = q % 6;
        int64_t gr;
        const uint8_t* base;
        int64_t ld;
        if (row < 128) { gr = m0 + row; gr = gr < a.M ? gr : a.M - 1; base = a.A; ld = a.lda; }
        else { gr = n0 + row - 128; gr = gr < a.N ? gr : a.N - 1; base = a.B; ld = a.ldb; }
        src[i] = base + gr * ld + c * 16;            // rows beyond the matrix are clamped; their results are never stored
        dst[i] = row * kPitch + c * 16;
    }
    const uint8_t* ssrc;
    {
        int64_t gr;
        if (tid < 128) { gr = m0 + tid; gr = gr < a.M ? gr : a.M - 1; ssrc = a.SA + gr * a.ldsa; }
        else { gr = n0 + tid - 128; gr = gr < a.N ? gr : a.N - 1; ssrc = a.SB + gr * a.ldsb; }
    }
    // two register sets: the loads of K step t+2 are in flight while step t is multiplied and step t+1 waits in the
    // other set for its turn to be written to LDS
    v4i reg0[6], reg1[6];
    uint32_t sreg0 = 0, sreg1 = 0;

    // ---- fragment addresses inside a stage (row tile t of A: rows wave_m*64 + 16t + r16; of B: 128 + wave_n*64 + ...)
    int fa_off[4], fb_off[4], sa_off[4], sb_off[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int ra = wave_m * 64 + t * 16 + r16, rb = 128 + wave_n * 64 + t * 16 + r16;
        fa_off[t] = ra * kPitch + g * 24; fb_off[t] = rb * kPitch + g * 24;
        sa_off[t] = kCodeBytes + ra * 4; sb_off[t] = kCodeBytes + rb * 4;
    }

    v4f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    // One K step: request step kt+2 into `far` (free: its previous content went to LDS one step ago), multiply the
    // LDS stage of step kt, then hand step kt+1 (waiting in `near`) to the other LDS stage.
    // One K step (FAR = register set that receives step kt+2; the other one holds step kt+1): request step kt+2,
    // multiply the LDS stage of step kt, then hand step kt+1 to the other LDS stage.  Loads and LDS writes are
    // unconditional (beyond the last step they repeat the last one into a stage nobody reads any more).
#define HALO_MX6_K_STEP(KT, FAR, FAR_S, NEAR, NEAR_S)                                                                       \
    {                                                                                                                       \
        const int kt_ = (KT);                                                                                               \
        const int64_t koff = (int64_t)(kt_ + 2 < nk ? kt_ + 2 : nk - 1);                                                    \
        _Pragma("unroll") for (int i = 0; i < 6; ++i) FAR[i] = *reinterpret_cast<const v4i*>(src[i] + koff * 96);           \
        FAR_S = *reinterpret_cast<const uint32_t*>(ssrc + koff * 4);                                                        \
        const unsigned char* s = smem + (kt_ & 1) * kStageBytes;                                                            \
        v8i va[4], vb[4];                                                                                                   \
        int sa[4], sb[4];                                                                                                   \
        _Pragma("unroll") for (int t = 0; t < 4; ++t) {                                                                     \
            const uint2* pa = reinterpret_cast<const uint2*>(s + fa_off[t]);                                                \
            const uint2* pb = reinterpret_cast<const uint2*>(s + fb_off[t]);                                                \
            const uint2 a0 = pa[0], a1 = pa[1], a2 = pa[2], b0 = pb[0], b1 = pb[1], b2 = pb[2];                             \
            va[t] = v8i{(int)a0.x, (int)a0.y, (int)a1.x, (int)a1.y, (int)a2.x, (int)a2.y, 0, 0};                            \
            vb[t] = v8i{(int)b0.x, (int)b0.y, (int)b1.x, (int)b1.y, (int)b2.x, (int)b2.y, 0, 0};                            \
            sa[t] = (int)((*reinterpret_cast<const uint32_t*>(s + sa_off[t]) >> (8 * g)) & 0xFFu);                          \
            sb[t] = (int)((*reinterpret_cast<const uint32_t*>(s + sb_off[t]) >> (8 * g)) & 0xFFu);                          \
        }                                                                                                                   \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                                       \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                                   \
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(va[i], vb[j], acc[i][j], kFmtE3M2, kFmtE3M2,  \
                                                                             0, sa[i], 0, sb[j]);                           \
        __builtin_amdgcn_sched_barrier(0); /* the LDS writes (which wait for global data) stay behind the MFMAs */        \
        unsigned char* w = smem + ((kt_ + 1) & 1) * kStageBytes;                                                            \
        _Pragma("unroll") for (int i = 0; i < 6; ++i) *reinterpret_cast<v4i*>(w + dst[i]) = NEAR[i];                        \
        reinterpret_cast<uint32_t*>(w + kCodeBytes)[tid] = NEAR_S;                                                          \
        __syncthreads();                                                                                                    \
    }

    if (nk > 0) {
        const int64_t k1 = nk > 1 ? 1 : 0;
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            reg0[i] = *reinterpret_cast<const v4i*>(src[i]);
            reg1[i] = *reinterpret_cast<const v4i*>(src[i] + k1 * 96);
        }
        sreg0 = *reinterpret_cast<const uint32_t*>(ssrc);
        sreg1 = *reinterpret_cast<const uint32_t*>(ssrc + k1 * 4);
#pragma unroll
        for (int i = 0; i < 6; ++i) *reinterpret_cast<v4i*>(smem + dst[i]) = reg0[i];
        reinterpret_cast<uint32_t*>(smem + kCodeBytes)[tid] = sreg0;
        __syncthreads();
        int kt = 0;
        for (; kt + 1 < nk; kt += 2) {
            HALO_MX6_K_STEP(kt, reg0, sreg0, reg1, sreg1)          // even step: step kt+1 waits in set 1, kt+2 goes to set 0
            HALO_MX6_K_STEP(kt + 1, reg1, sreg1, reg0, sreg0)
        }
        if (kt < nk) HALO_MX6_K_STEP(kt, reg0, sreg0, reg1, sreg1)
    }
#undef HALO_MX6_K_STEP

#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t col = n0 + wave_n * 64 + j * 16 + r16;
            if (col >= a.N) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t row = m0 + wave_m * 64 + i * 16 + 4 * g + r;
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
