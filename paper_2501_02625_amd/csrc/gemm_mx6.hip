// MXFP6 GEMM on the CDNA4 scaled matrix instruction v_mfma_scale_f32_16x16x128_f8f6f4 with both operands in FP6 E3M2
// (format selector 3) and one E8M0 scale per block of 32 elements along K:  C = A B^T, fp32 accumulation.
//
// Operand layout of the instruction (established with a one-tile numeric probe against an exact reference): lane l
// supplies the 32 consecutive K-elements of row (l % 16) that start at K offset 32 * (l / 16), i.e. exactly one
// scaling block, as 192 bits packed least-significant element first in six registers, plus that block's E8M0 byte in
// byte 0 of the scale register.  Accumulator: lane l holds column (l % 16), rows 4 * (l / 16) + r, r = 0..3.
// So the packed codes in memory ([row][block][24 bytes]) are the register image: nothing is unpacked or shuffled.
// Two kernels: the one below for small products, a 256 x 256-tile one with DMA-fed LDS further down for large ones.
//
// Small products: workgroup = 4 wavefronts (2 x 2), macro tile 128 x 128, each wavefront 64 x 64 = 4 x 4 instruction tiles; K step 128
// elements = 96 code bytes + 4 scale bytes per row.  Two LDS stages: the 256 rows of a K step (128 of A, 128 of B) lie
// at a pitch of 112 bytes (28 dwords: the sixteen rows one quarter-wavefront reads fall on sixteen different groups of
// four banks), the scale dwords behind them.  The next K step travels global -> registers (six 16-byte loads and one
// scale dword per thread) while the current one is multiplied, then registers -> LDS, one barrier per K step.  A lane
// reads its block as three 8-byte LDS loads: the code bytes in memory are the register image, nothing is unpacked.
#include <mutex>
#include <type_traits>

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
                else reinterpret_cast<uint16_t*>(a.C)[row * a.ldc + col] = bf16_bits(acc[i][j][r]);
            }
        }
}


// ------------------------------------------------------------------------------------------------ large products
// 256 x 256 macro tile, 8 wavefronts (2 x 4), each 128 x 64 = 4 x 2 tiles of v_mfma_scale_f32_32x32x64_f8f6f4: twice
// the arithmetic per operand register of the 16x16x128 form.  Lane l of that instruction supplies the 32 consecutive
// K-elements (one scaling block, 24 bytes) of row l % 32 that start at K offset 32 * (l / 32); the accumulator has the
// usual 32 x 32 layout (lane l: column l % 32, rows 8 * (r / 4) + 4 * (l / 32) + r % 4 for r = 0..15).
//
// K step = 128 elements = 96 code bytes + 4 scale bytes per row.  Codes and scales travel global -> LDS by DMA
// (global_load_lds, 16 and 4 bytes per lane) through a ring of three stages, two K steps in flight.  A stage holds,
// per operand, sixteen blocks of 16 rows; a block is six planes of [16 rows][16 bytes], plane c holding bytes
// 16c .. 16c+15 of the rows' 96 (one DMA instruction then fetches 64 or 32 contiguous bytes of 16 or 32 rows; with
// planes of 32 rows it was 32 bytes of 32 rows each time, and the kernel 10 % slower: the transfers are bound by the
// number of cache lines an instruction touches).  A lane reads its 24 bytes as three 8-byte pieces: the two halves of
// the wavefront (K blocks 2s and 2s+1 of sub-step s) always sit on complementary halves of the 16-byte chunks, so every
// such read covers all 64 banks evenly.
constexpr int kBigOpBytes = 256 * 96;                       // one operand's codes per stage
constexpr int kBigScaleOff = 2 * kBigOpBytes;               // 512 scale dwords (A rows, then B rows)
constexpr int kBigStage = kBigScaleOff + 512 * 4;
constexpr int kBigNS = 3;
constexpr int kBigLoads = 7;                                // DMA instructions per thread per K step
constexpr int kBigEpiPitch = 64 + 8;
constexpr int kBigLds = kBigNS * kBigStage;
static_assert(kBigLds <= 160 * 1024 && 8 * 32 * kBigEpiPitch * 4 <= kBigLds, "LDS budget");
// WIDE form (K a multiple of 512, 16-byte aligned scale rows): the stages hold codes only, and the scale bytes of FOUR K
// steps travel as one 16-byte chunk per row into one of two buffers behind the stages - a quarter of the scale requests,
// each of which touches 64 different cache lines.
constexpr int kWideStage = 2 * kBigOpBytes;
constexpr int kWideScaleOff = kBigNS * kWideStage;
constexpr int kWideLds = kWideScaleOff + 2 * 512 * 16;
static_assert(kWideLds <= 160 * 1024, "LDS budget");

#define HALO_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define HALO_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

typedef float v16f __attribute__((ext_vector_type(16)));

typedef int v2i __attribute__((ext_vector_type(2)));

// The three 8-byte pieces of each of the six fragments (four of A, two of B) of one K sub-step.
struct BigFrags {
    v2i a[4][3], b[2][3];
};

// Requests the fragments of K sub-step KS (64 elements) of one stage.  addr_a / addr_b: LDS byte address of this
// lane's piece j of K block 2 * KS + half in the wavefront's first 32 rows; 32 rows are 3072 bytes apart.
// Issued as inline assembly: seen as LDS reads, the compiler would make them wait for every outstanding global->LDS
// transfer (s_waitcnt vmcnt(0)), which empties the ring at every K step.  big_wait_frags() waits for the data.
template <int KS>
__device__ __forceinline__ void big_load_frags(const uint32_t (&addr_a)[2][3], const uint32_t (&addr_b)[2][3], BigFrags& f) {
#pragma unroll
    for (int j = 0; j < 3; ++j)
        asm volatile("ds_read_b64 %0, %4\n\tds_read_b64 %1, %4 offset:3072\n\t"
                     "ds_read_b64 %2, %4 offset:6144\n\tds_read_b64 %3, %4 offset:9216"
                     : "=&v"(f.a[0][j]), "=&v"(f.a[1][j]), "=&v"(f.a[2][j]), "=&v"(f.a[3][j])
                     : "v"(addr_a[KS][j]));
#pragma unroll
    for (int j = 0; j < 3; ++j)
        asm volatile("ds_read_b64 %0, %2\n\tds_read_b64 %1, %2 offset:3072"
                     : "=&v"(f.b[0][j]), "=&v"(f.b[1][j])
                     : "v"(addr_b[KS][j]));
}

// Waits for every outstanding LDS read.  The registers are operands of the wait, so nothing that uses them can move
// above it.
__device__ __forceinline__ void big_wait_frags(BigFrags& f) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f.a[0][0]), "+v"(f.a[0][1]), "+v"(f.a[0][2]), "+v"(f.a[1][0]), "+v"(f.a[1][1]), "+v"(f.a[1][2]),
                   "+v"(f.a[2][0]), "+v"(f.a[2][1]), "+v"(f.a[2][2]), "+v"(f.a[3][0]), "+v"(f.a[3][1]), "+v"(f.a[3][2]),
                   "+v"(f.b[0][0]), "+v"(f.b[0][1]), "+v"(f.b[0][2]), "+v"(f.b[1][0]), "+v"(f.b[1][1]), "+v"(f.b[1][2]));
}

__device__ __forceinline__ v8i big_operand(const v2i (&p)[3]) {
    return v8i{p[0][0], p[0][1], p[1][0], p[1][1], p[2][0], p[2][1], 0, 0};
}

template <int KS>
__device__ __forceinline__ void big_mma(const BigFrags& f, const int (&sca)[4], const int (&scb)[2], v16f (&acc)[4][2]) {
    v8i va[4], vb[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) va[i] = big_operand(f.a[i]);
#pragma unroll
    for (int j = 0; j < 2; ++j) vb[j] = big_operand(f.b[j]);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va[i], vb[j], acc[i][j], kFmtE3M2, kFmtE3M2,
                                                                        2 * KS, sca[i], 2 * KS, scb[j]);
}

template <bool WIDE>
__global__ void __launch_bounds__(512) gemm_mx6_big_kernel(Mx6GemmArgs a, int tiles_m, int tiles_n) {
    constexpr int kStage = WIDE ? kWideStage : kBigStage;
    extern __shared__ __align__(16) unsigned char smem_big[];
    unsigned char* smem = smem_big;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 2, wave_n = wave & 3;
    const int lrow = lane & 31, half = lane >> 5;

    // consecutive workgroups go to different XCDs: give each XCD a contiguous range of tiles, walked four tile-rows
    // at a time so that its resident tiles share operand panels in its L2
    int tile_m, tile_n;
    {
        const int bid = blockIdx.x;
        const int ntiles = tiles_m * tiles_n;
        const int xcd = bid & 7, q = bid >> 3;
        const int base = ntiles >> 3, rem = ntiles & 7;
        const int pid = xcd * base + (xcd < rem ? xcd : rem) + q;
        const int per_group = 4 * tiles_n;
        const int group = pid / per_group, first_m = group * 4;
        const int gsize = (tiles_m - first_m) < 4 ? (tiles_m - first_m) : 4;
        const int in_group = pid % per_group;
        tile_m = first_m + in_group % gsize;
        tile_n = in_group / gsize;
    }
    const int64_t m0 = (int64_t)tile_m * 256, n0 = (int64_t)tile_n * 256;
    const int nk = (int)(a.K / 128);

    // ---- per-thread DMA sources (fixed over the K loop): three 16-byte chunks of each operand, one scale dword.  Slot s
    // of an operand = block s / 96 (16 rows), plane (s % 96) / 16, row-in-block s % 16.  Rows beyond the matrix are clamped; their
    // results are never stored.
    const uint8_t* a_src[3];
    const uint8_t* b_src[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int slot = tid + i * 512;
        const int row = (slot / 96) * 16 + slot % 16, c = (slot % 96) / 16;
        int64_t gr = m0 + row;
        gr = gr < a.M ? gr : a.M - 1;
        a_src[i] = a.A + gr * a.lda + c * 16;
        gr = n0 + row;
        gr = gr < a.N ? gr : a.N - 1;
        b_src[i] = a.B + gr * a.ldb + c * 16;
    }
    const uint8_t* s_src;
    {
        int64_t gr;
        if (tid < 256) { gr = m0 + tid; gr = gr < a.M ? gr : a.M - 1; s_src = a.SA + gr * a.ldsa; }
        else { gr = n0 + tid - 256; gr = gr < a.N ? gr : a.N - 1; s_src = a.SB + gr * a.ldsb; }
    }
    // K step t (codes of step `src`) into ring slot t % NS.  with_scales: in the WIDE form, also the scale chunk of the
    // group of four K steps that starts at t (t a multiple of 4) into scale buffer (t / 4) % 2.
    auto issue_dma = [&](int t, int src, bool with_scales) {
        unsigned char* st = smem + (t % kBigNS) * kStage;
#pragma unroll
        for (int i = 0; i < 3; ++i)
            __builtin_amdgcn_global_load_lds(HALO_GLOBAL_PTR(a_src[i] + (int64_t)src * 96),
                                             HALO_LDS_PTR(st + (wave * 64 + i * 512) * 16), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < 3; ++i)
            __builtin_amdgcn_global_load_lds(HALO_GLOBAL_PTR(b_src[i] + (int64_t)src * 96),
                                             HALO_LDS_PTR(st + kBigOpBytes + (wave * 64 + i * 512) * 16), 16, 0, 0);
        if constexpr (!WIDE) {
            __builtin_amdgcn_global_load_lds(HALO_GLOBAL_PTR(s_src + (int64_t)src * 4),
                                             HALO_LDS_PTR(st + kBigScaleOff + wave * 64 * 4), 4, 0, 0);
        } else if (with_scales) {
            const int g = src / 4;
            __builtin_amdgcn_global_load_lds(HALO_GLOBAL_PTR(s_src + (int64_t)g * 16),
                                             HALO_LDS_PTR(smem + kWideScaleOff + ((t / 4) & 1) * 8192 + wave * 64 * 16), 16, 0, 0);
        }
    };

    // ---- this lane's three 8-byte pieces of K block 2 * ks + half, as byte offsets inside a stage
    uint32_t off_a[2][3], off_b[2][3], off_sa, off_sb;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const int o = (2 * ks + half) * 24 + 8 * j;
            const uint32_t in_block = (uint32_t)((lrow / 16) * 1536 + ((o / 16) * 16 + lrow % 16) * 16 + o % 16);
            off_a[ks][j] = (uint32_t)(wave_m * 4 * 3072) + in_block;
            off_b[ks][j] = (uint32_t)(kBigOpBytes + wave_n * 2 * 3072) + in_block;
        }
    off_sa = WIDE ? (uint32_t)(kWideScaleOff + (wave_m * 128 + lrow) * 16) : (uint32_t)(kBigScaleOff + (wave_m * 128 + lrow) * 4);
    off_sb = WIDE ? (uint32_t)(kWideScaleOff + (256 + wave_n * 64 + lrow) * 16)
                  : (uint32_t)(kBigScaleOff + (256 + wave_n * 64 + lrow) * 4);
    const uint32_t lds0 = (uint32_t)(uintptr_t)HALO_LDS_PTR(smem);

    v16f acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    if (nk > 0) {
        constexpr int D = kBigNS - 1;
        // One K step.  PH: kt % 4 in the WIDE form (it fixes which steps carry a scale chunk, hence the wait count and the
        // byte of the chunk to use), -1 otherwise.
        auto k_step = [&](auto ph, int kt) {
            constexpr int PH = decltype(ph)::value;
            // outstanding afterwards: the loads of step kt + 1 only (6 code chunks, plus its scale request)
            constexpr int kAllowed = WIDE ? (PH == 3 ? 7 : 6) : (D - 1) * kBigLoads;
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(kAllowed) : "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            // ring slot (kt - 1) % NS: everyone is past reading it
            issue_dma(kt + D, kt + D < nk ? kt + D : nk - 1, PH == 2);
            const uint32_t st = lds0 + (uint32_t)((kt % kBigNS) * kStage);
            uint32_t addr_a[2][3], addr_b[2][3];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int j = 0; j < 3; ++j) { addr_a[ks][j] = st + off_a[ks][j]; addr_b[ks][j] = st + off_b[ks][j]; }
            // the four scale bytes of each of this lane's six rows (same inline-assembly reasoning as the fragments)
            int sca[4], scb[2];
            if constexpr (WIDE) {
                const uint32_t sbase = lds0 + (uint32_t)(((kt / 4) & 1) * 8192 + PH * 4);
                asm volatile("ds_read_b32 %0, %6\n\tds_read_b32 %1, %6 offset:512\n\tds_read_b32 %2, %6 offset:1024\n\t"
                             "ds_read_b32 %3, %6 offset:1536\n\tds_read_b32 %4, %7\n\tds_read_b32 %5, %7 offset:512"
                             : "=&v"(sca[0]), "=&v"(sca[1]), "=&v"(sca[2]), "=&v"(sca[3]), "=&v"(scb[0]), "=&v"(scb[1])
                             : "v"(sbase + off_sa), "v"(sbase + off_sb));
            } else {
                asm volatile("ds_read_b32 %0, %6\n\tds_read_b32 %1, %6 offset:128\n\tds_read_b32 %2, %6 offset:256\n\t"
                             "ds_read_b32 %3, %6 offset:384\n\tds_read_b32 %4, %7\n\tds_read_b32 %5, %7 offset:128"
                             : "=&v"(sca[0]), "=&v"(sca[1]), "=&v"(sca[2]), "=&v"(sca[3]), "=&v"(scb[0]), "=&v"(scb[1])
                             : "v"(st + off_sa), "v"(st + off_sb));
            }
            BigFrags f0, f1;
            big_load_frags<0>(addr_a, addr_b, f0);
            big_wait_frags(f0);              // the hardware counts at most 15 outstanding LDS reads: no partial wait here
            asm volatile("" : "+v"(sca[0]), "+v"(sca[1]), "+v"(sca[2]), "+v"(sca[3]), "+v"(scb[0]), "+v"(scb[1]));
            big_load_frags<1>(addr_a, addr_b, f1);       // in flight while sub-step 0 is multiplied
#pragma unroll
            for (int i = 0; i < 4; ++i) sca[i] = (int)((uint32_t)sca[i] >> (8 * half));
#pragma unroll
            for (int j = 0; j < 2; ++j) scb[j] = (int)((uint32_t)scb[j] >> (8 * half));
            big_mma<0>(f0, sca, scb, acc);
            big_wait_frags(f1);
            big_mma<1>(f1, sca, scb, acc);
        };
        if constexpr (WIDE) {
            // nk is a multiple of 4 here.  Step 0 carries the first scale chunk; step 1 none.
            issue_dma(0, 0, true);
            issue_dma(1, 1, false);
            for (int kt = 0; kt < nk; kt += 4) {
                k_step(std::integral_constant<int, 0>{}, kt);
                k_step(std::integral_constant<int, 1>{}, kt + 1);
                k_step(std::integral_constant<int, 2>{}, kt + 2);
                k_step(std::integral_constant<int, 3>{}, kt + 3);
            }
        } else {
            for (int t = 0; t < D; ++t) issue_dma(t, t < nk ? t : nk - 1, false);
            for (int kt = 0; kt < nk; ++kt) k_step(std::integral_constant<int, -1>{}, kt);
        }
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    }

    // ---- epilogue: each wavefront drops a 32-row slab of its sub-tile into a private LDS region and reads it back four
    // consecutive columns per lane, so the global stores are 16-byte (fp32) or 8-byte (bf16) pieces of covered rows
    __syncthreads();
    float* region = reinterpret_cast<float*>(smem) + wave * 32 * kBigEpiPitch;
    const int cc = (lane % 16) * 4;
    const int64_t col = n0 + wave_n * 64 + cc;
    const bool col_any = col < a.N, col_all = col + 4 <= a.N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) region[(8 * (r / 4) + 4 * half + (r % 4)) * kBigEpiPitch + j * 32 + lrow] = acc[i][j][r];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int rr = p * 4 + lane / 16;
            const float4 v = *reinterpret_cast<const float4*>(region + rr * kBigEpiPitch + cc);
            const int64_t row = m0 + wave_m * 128 + i * 32 + rr;
            if (row >= a.M || !col_any) continue;
            const float f[4] = {v.x, v.y, v.z, v.w};
            if (a.c_is_f32) {
                float* dst = reinterpret_cast<float*>(a.C) + row * a.ldc + col;
                if (col_all) {
                    *reinterpret_cast<float4*>(dst) = v;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e < a.N) dst[e] = f[e];
                }
            } else {
                uint16_t* dst = reinterpret_cast<uint16_t*>(a.C) + row * a.ldc + col;
                if (col_all) {
                    *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf16x2(f[0], f[1]),
                                                                 pack_bf16x2(f[2], f[3]));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e < a.N) dst[e] = bf16_bits(f[e]);
                }
            }
        }
    }
}

}  // namespace

hipError_t launch_gemm_mx6(const Mx6GemmArgs& a, hipStream_t s) {
    if (a.M == 0 || a.N == 0) return hipSuccess;
    if (a.K % 128 != 0) return hipErrorInvalidValue;
    // Enough 256 x 256 tiles to give most compute units one: the DMA kernel.  Its 16-byte stores need aligned rows of C.
    const int64_t big_m = (a.M + 255) / 256, big_n = (a.N + 255) / 256;
    const int64_t c_bytes = a.c_is_f32 ? 4 : 2;
    if (big_m * big_n >= 192 && big_m * big_n <= 0x7FFFFFFF && (a.ldc * c_bytes) % 16 == 0 &&
        (reinterpret_cast<uintptr_t>(a.C) & 15u) == 0) {
        static std::once_flag once;
        static hipError_t attr_result = hipSuccess;
        std::call_once(once, [&] {
            attr_result = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_mx6_big_kernel<false>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, kBigLds);
            if (attr_result == hipSuccess)
                attr_result = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_mx6_big_kernel<true>),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, kWideLds);
        });
        if (attr_result != hipSuccess) return attr_result;
        const bool wide = a.K % 512 == 0 && a.ldsa % 16 == 0 && a.ldsb % 16 == 0 &&
                          (reinterpret_cast<uintptr_t>(a.SA) & 15u) == 0 && (reinterpret_cast<uintptr_t>(a.SB) & 15u) == 0;
        if (wide)
            hipLaunchKernelGGL(gemm_mx6_big_kernel<true>, dim3((unsigned)(big_m * big_n)), dim3(512), kWideLds, s, a, (int)big_m,
                               (int)big_n);
        else
            hipLaunchKernelGGL(gemm_mx6_big_kernel<false>, dim3((unsigned)(big_m * big_n)), dim3(512), kBigLds, s, a, (int)big_m,
                               (int)big_n);
        return hipGetLastError();
    }
    const int64_t tiles_m = (a.M + 127) / 128, tiles_n = (a.N + 127) / 128;
    if (tiles_m * tiles_n > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gemm_mx6_kernel, dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 0, s, a, (int)tiles_n);
    return hipGetLastError();
}

}  // namespace halo
