// INT8 GEMM on the CDNA4 matrix cores (v_mfma_i32_32x32x32_i8) with int32 accumulation and a fused
// dequantisation epilogue:  C = diag(row_scale) * (A * op(B)) * diag(col_scale).
//
//   A  [M x K]  K contiguous.
//   B  transB:  [N x K], K contiguous  -> both operands stream 16-byte K-chunks straight into LDS.
//      !transB: [K x N], K strided     -> 4(k) x 4(n) byte blocks are transposed in registers with v_perm_b32
//               on their way to LDS, so the saved (WH)_Q / (XH)_Q codes are reused by the backward
//               products without a transposed copy in HBM.
//
// Workgroup = WAVES_M x WAVES_N wavefronts, macro tile BM x BN, K step BK bytes, two LDS stages with the next
// K step prefetched into registers while the current one is multiplied.  Each wavefront owns a
// (BM/WAVES_M) x (BN/WAVES_N) sub-tile as a grid of 32x32 MFMA tiles.
//
// MFMA operand layout (32x32x32 i8): lane l supplies 16 consecutive K-bytes of row (l % 32), taken from K
// offset 16*(l / 32) of the 32-byte K step, for A and for B alike; since both operands use the same
// assignment of K positions to (lane group, byte), the dot products are exact whatever order the hardware
// sums them in.  Accumulator layout: lane l holds column (l % 32) and rows 8*(r/4) + 4*(l/32) + (r%4),
// r = 0..15.
//
// LDS layouts.  K-contiguous operands: [row][BK bytes], the 16-byte chunk index XOR-swizzled with the row
// so that the 16 rows read by one quarter-wave ds_read_b128 fall in 16 different bank groups.
// K-strided B: dwords of four consecutive k, laid out [k/4][n] with a row pitch of BN+8 dwords; the
// transposing writes are contiguous 16-byte stores and the operand reads are conflict-free ds_read_b32.
#include "halo_internal.h"

namespace halo {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool TRANSB>
struct GemmCfg {
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int CH = BK / 16;        // 16-byte chunks per K-contiguous row
    static constexpr int RPS = 256 / BK;      // rows per 256-byte sweep of the LDS banks
    static constexpr int KSTEPS = BK / 32;
    static constexpr int LDB_NN = BN + 8;     // dword pitch of the K-strided layout
    static constexpr int A_BYTES = BM * BK;
    static constexpr int B_BYTES = TRANSB ? BN * BK : (BK / 4) * LDB_NN * 4;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static constexpr int SLOTS_A = BM * CH / NT;
    static constexpr int SLOTS_B = BN * CH / NT;                 // transB
    static constexpr int BLKS_B = (BK / 4) * (BN / 4) / NT;      // !transB
    static_assert(BM * CH % NT == 0 && BN * CH % NT == 0, "tile/threads mismatch");
    static_assert(((BK / 4) * (BN / 4)) % NT == 0, "tile/threads mismatch");
};

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool TRANSB>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N)
gemm_i8_kernel(GemmArgs a, int tiles_m, int tiles_n) {
    using Cfg = GemmCfg<BM, BN, BK, WAVES_M, WAVES_N, TRANSB>;
    constexpr int NT = Cfg::NT, CH = Cfg::CH, RPS = Cfg::RPS, TM = Cfg::TM, TN = Cfg::TN;
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_m = wave / WAVES_N;
    const int wave_n = wave % WAVES_N;

    // ---- tile assignment: consecutive workgroup ids go to different XCDs (8 per chip), so give every XCD a
    // contiguous range of tile numbers, and walk tiles in groups of 8 tile-rows so that one XCD's resident
    // tiles share A and B panels in its L2.
    const int ntiles = tiles_m * tiles_n;
    int pid;
    {
        const int bid = blockIdx.x;
        const int xcd = bid & 7, q = bid >> 3;
        const int base = ntiles >> 3, rem = ntiles & 7;
        pid = xcd * base + (xcd < rem ? xcd : rem) + q;
    }
    int tile_m, tile_n;
    {
        constexpr int GROUP = 8;
        const int per_group = GROUP * tiles_n;
        const int group = pid / per_group;
        const int first_m = group * GROUP;
        const int gsize = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
        const int in_group = pid % per_group;
        tile_m = first_m + in_group % gsize;
        tile_n = in_group / gsize;
    }
    const int64_t m0 = (int64_t)tile_m * BM;
    const int64_t n0 = (int64_t)tile_n * BN;

    // ---- per-thread global -> LDS assignments (fixed over the K loop)
    const int8_t* a_src[Cfg::SLOTS_A];
    int a_koff[Cfg::SLOTS_A];
#pragma unroll
    for (int i = 0; i < Cfg::SLOTS_A; ++i) {
        const int p = tid + i * NT;
        const int row = p / CH, pc = p % CH;
        const int g = pc ^ ((row / RPS) % CH);
        int64_t gr = m0 + row;
        if (gr > a.M - 1) gr = a.M - 1;
        a_src[i] = a.A + gr * a.lda + 16 * g;
        a_koff[i] = 16 * g;
    }
    const int8_t* b_src[TRANSB ? Cfg::SLOTS_B : Cfg::BLKS_B];
    int b_koff[TRANSB ? Cfg::SLOTS_B : Cfg::BLKS_B];
    bool b_ok[TRANSB ? Cfg::SLOTS_B : Cfg::BLKS_B];
    if constexpr (TRANSB) {
#pragma unroll
        for (int i = 0; i < Cfg::SLOTS_B; ++i) {
            const int p = tid + i * NT;
            const int row = p / CH, pc = p % CH;
            const int g = pc ^ ((row / RPS) % CH);
            int64_t gr = n0 + row;
            if (gr > a.N - 1) gr = a.N - 1;
            b_src[i] = a.B + gr * a.ldb + 16 * g;
            b_koff[i] = 16 * g;
            b_ok[i] = true;
        }
    } else {
#pragma unroll
        for (int i = 0; i < Cfg::BLKS_B; ++i) {
            const int q = tid + i * NT;
            const int nb = q % (BN / 4), kb = q / (BN / 4);
            b_ok[i] = (n0 + 4 * nb) < a.N;
            b_src[i] = a.B + (int64_t)(4 * kb) * a.ldb + (b_ok[i] ? n0 + 4 * nb : 0);
            b_koff[i] = 4 * kb;
        }
    }

    uint4 a_reg[Cfg::SLOTS_A];
    uint4 b_reg[TRANSB ? Cfg::SLOTS_B : Cfg::BLKS_B];

    auto load_global = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < Cfg::SLOTS_A; ++i) {
            a_reg[i] = (k0 + a_koff[i] < a.K) ? *reinterpret_cast<const uint4*>(a_src[i] + k0)
                                               : make_uint4(0, 0, 0, 0);
        }
        if constexpr (TRANSB) {
#pragma unroll
            for (int i = 0; i < Cfg::SLOTS_B; ++i) {
                b_reg[i] = (k0 + b_koff[i] < a.K) ? *reinterpret_cast<const uint4*>(b_src[i] + k0)
                                                   : make_uint4(0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < Cfg::BLKS_B; ++i) {
                uint32_t r[4];
                const int8_t* p = b_src[i] + k0 * a.ldb;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    r[j] = (b_ok[i] && (k0 + b_koff[i] + j < a.K))
                               ? *reinterpret_cast<const uint32_t*>(p + (int64_t)j * a.ldb) : 0u;
                }
                // 4x4 byte transpose: t[e] = (r0.byte[e], r1.byte[e], r2.byte[e], r3.byte[e])
                const uint32_t u0 = __builtin_amdgcn_perm(r[1], r[0], 0x05010400u);
                const uint32_t u1 = __builtin_amdgcn_perm(r[1], r[0], 0x07030602u);
                const uint32_t v0 = __builtin_amdgcn_perm(r[3], r[2], 0x05010400u);
                const uint32_t v1 = __builtin_amdgcn_perm(r[3], r[2], 0x07030602u);
                b_reg[i].x = __builtin_amdgcn_perm(v0, u0, 0x05040100u);
                b_reg[i].y = __builtin_amdgcn_perm(v0, u0, 0x07060302u);
                b_reg[i].z = __builtin_amdgcn_perm(v1, u1, 0x05040100u);
                b_reg[i].w = __builtin_amdgcn_perm(v1, u1, 0x07060302u);
            }
        }
    };

    auto store_lds = [&](int stage) {
        unsigned char* sa = smem + stage * Cfg::STAGE_BYTES;
        unsigned char* sb = sa + Cfg::A_BYTES;
#pragma unroll
        for (int i = 0; i < Cfg::SLOTS_A; ++i)
            *reinterpret_cast<uint4*>(sa + (tid + i * NT) * 16) = a_reg[i];
        if constexpr (TRANSB) {
#pragma unroll
            for (int i = 0; i < Cfg::SLOTS_B; ++i)
                *reinterpret_cast<uint4*>(sb + (tid + i * NT) * 16) = b_reg[i];
        } else {
#pragma unroll
            for (int i = 0; i < Cfg::BLKS_B; ++i) {
                const int q = tid + i * NT;
                const int nb = q % (BN / 4), kb = q / (BN / 4);
                *reinterpret_cast<uint4*>(sb + (kb * Cfg::LDB_NN + 4 * nb) * 4) = b_reg[i];
            }
        }
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int lrow = lane & 31, half = lane >> 5;

    auto compute = [&](int stage) {
        const unsigned char* sa = smem + stage * Cfg::STAGE_BYTES;
        const unsigned char* sb = sa + Cfg::A_BYTES;
#pragma unroll
        for (int kk = 0; kk < Cfg::KSTEPS; ++kk) {
            v4i af[TM], bf[TN];
            const int g = 2 * kk + half;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = wave_m * Cfg::WM + i * 32 + lrow;
                const int pc = g ^ ((row / RPS) % CH);
                af[i] = *reinterpret_cast<const v4i*>(sa + row * BK + 16 * pc);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = wave_n * Cfg::WN + j * 32 + lrow;
                if constexpr (TRANSB) {
                    const int pc = g ^ ((col / RPS) % CH);
                    bf[j] = *reinterpret_cast<const v4i*>(sb + col * BK + 16 * pc);
                } else {
                    const uint32_t* sbw = reinterpret_cast<const uint32_t*>(sb);
#pragma unroll
                    for (int w = 0; w < 4; ++w) bf[j][w] = (int)sbw[(4 * g + w) * Cfg::LDB_NN + col];
                }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
    };

    const int nk = (int)((a.K + BK - 1) / BK);
    if (nk > 0) {
        load_global(0);
        store_lds(0);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const bool more = kt + 1 < nk;
            if (more) load_global((int64_t)(kt + 1) * BK);
            compute(kt & 1);
            if (more) store_lds((kt + 1) & 1);
            __syncthreads();
        }
    }

    // ---- epilogue
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t col = n0 + wave_n * Cfg::WN + j * 32 + lrow;
            if (col >= a.N) continue;
            const float cs = a.col_scale ? a.col_scale[col] : 1.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wave_m * Cfg::WM + i * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                if (row >= a.M) continue;
                const int v = acc[i][j][r];
                if (a.acc_out) a.acc_out[row * a.ld_acc + col] = v;
                if (a.C) {
                    const float rs = a.row_scale ? a.row_scale[row] : 1.0f;
                    const float f = ((float)v * rs) * cs;
                    if (a.c_is_f32) {
                        reinterpret_cast<float*>(a.C)[row * a.ldc + col] = f;
                    } else {
                        reinterpret_cast<uint16_t*>(a.C)[row * a.ldc + col] = (uint16_t)f32_to_bf16_rne(f);
                    }
                }
            }
        }
    }
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool TRANSB>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t s) {
    using Cfg = GemmCfg<BM, BN, BK, WAVES_M, WAVES_N, TRANSB>;
    auto kern = gemm_i8_kernel<BM, BN, BK, WAVES_M, WAVES_N, TRANSB>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(Cfg::NT), Cfg::LDS_BYTES, s, a,
                       tiles_m, tiles_n);
    return hipGetLastError();
}

template <bool TRANSB>
hipError_t launch_by_shape(const GemmArgs& a, hipStream_t s) {
    auto tiles = [&](int bm, int bn) { return ((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn); };
    if (tiles(256, 256) >= 200) return launch_cfg<256, 256, 64, 2, 4, TRANSB>(a, s);
    if (tiles(256, 128) >= 200) return launch_cfg<256, 128, 64, 2, 2, TRANSB>(a, s);
    return launch_cfg<128, 128, 64, 2, 2, TRANSB>(a, s);
}

}  // namespace

hipError_t launch_gemm_i8(const GemmArgs& a, hipStream_t s) {
    if (a.M == 0 || a.N == 0) return hipSuccess;
    return a.transB ? launch_by_shape<true>(a, s) : launch_by_shape<false>(a, s);
}

}  // namespace halo
