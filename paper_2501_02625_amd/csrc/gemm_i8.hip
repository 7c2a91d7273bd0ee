// INT8 GEMM on the CDNA4 matrix cores (v_mfma_i32_32x32x32_i8) with int32 accumulation and a fused
// dequantisation epilogue:  C = diag(row_scale) * (A * op(B)) * diag(col_scale).
//
//   A  [M x K]  K contiguous.
//   B  transB:  [N x K], K contiguous.
//      !transB: [K x N], K strided: the saved (WH)_Q / (XH)_Q codes are reused by the backward products as they are,
//               without a transposed copy in HBM.
//
// Workgroup = WAVES_M x WAVES_N wavefronts, macro tile BM x BN, K step BK bytes.  Each wavefront owns a
// (BM/WAVES_M) x (BN/WAVES_N) sub-tile as a grid of 32x32 MFMA tiles.
//
// Main loops:
//   * "dma" (every K that is a multiple of the K step): an NS-deep ring of LDS stages filled by
//     global_load_lds_dwordx4 (global memory -> LDS without passing through registers).  Exactly one K step is issued
//     per iteration, sliced between the MFMA sub-steps, so the s_waitcnt vmcnt(n) that waits for the oldest stage only
//     is a constant; one s_barrier per K step.  A K-contiguous operand is stored [row][BK bytes]; a K-strided B is
//     stored as it lies in memory (K-major rows of BN bytes) and transposed by the LDS read itself,
//     ds_read_b64_tr_b8: a group of 16 lanes reads an 8(k) x 16(n) byte block, lane i supplying the address of row
//     i/2, half i%2, and receiving column i.
//   * "staged" (ragged K): two LDS stages of a 128 x 128 tile, the next K step prefetched in registers and zero-filled
//     beyond K; a K-strided B is transposed in registers (4x4 byte blocks through v_perm_b32).
// A launch may carry two independent products (halo_gemm_i8_pair): workgroups past the first product's tile count
// take the second argument block.
//
// MFMA operand layout (32x32x32 i8): lane l supplies 16 consecutive K-bytes of row (l % 32), taken from K
// offset 16*(l / 32) of the 32-byte K step, for A and for B alike; since both operands use the same
// assignment of K positions to (lane group, byte), the dot products are exact whatever order the hardware
// sums them in.  Accumulator layout: lane l holds column (l % 32) and rows 8*(r/4) + 4*(l/32) + (r%4),
// r = 0..15.
//
// LDS layouts.  K-contiguous operands: the 16-byte chunk index is XOR-swizzled with the row so that the 16 rows read
// by one quarter-wave ds_read_b128 fall in 16 different bank groups (measured: zero LDS bank conflicts); a DMA lane
// writes LDS slot (wave slot base + lane), so the swizzle is applied to the global address it fetches.  K-major B:
// chunks XOR-swizzled by 2*(row % 8) (BN = 256) so that the two lane groups of one transposing read stay on even and
// odd chunks.  Register-transposed B (staged loop): dwords of four consecutive k, laid out [k/4][n] with a row pitch
// of BN+8 dwords.
//
// What bounds it.  A loop of nothing but these MFMAs sustains 4.9 POP/s on constant operands but only about 3.5 POP/s
// on random int8 operands (the chip lowers its clock as the multiplier arrays toggle), and about 2.9 POP/s once the
// LDS fragment reads and the global->LDS stream of a 256 x 256 tile run beside them: the published 5.0 POP/s is not
// reachable on real data (halo_mfma_i8_probe measures these ceilings on the machine at hand).  That is also why
// deeper rings, longer K steps, four instead of eight wavefronts, accumulators in AGPRs or a strict
// memory-phase/MFMA-phase alternation of the two wavefronts of a SIMD all land on the same throughput.
#include <mutex>

#include "halo_internal.h"

namespace halo {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v2i __attribute__((ext_vector_type(2)));

#define HALO_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define HALO_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

// TR: the K-strided B operand goes to LDS untransposed (K-major rows of BN bytes, by DMA like A) and is transposed
// by the LDS read itself (ds_read_b64_tr_b8).  !TRANSB && !TR: B is transposed in registers (staged loop only).
template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool TRANSB, int NS, bool TR = false>
struct GemmCfg {
    static constexpr bool IS_TR = TR;
    static constexpr int BM_ = BM, BN_ = BN;
    static constexpr int WAVES_M_ = WAVES_M, WAVES_N_ = WAVES_N;
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    // tile-rows per group of the workgroup->tile map (4 measured best of 2/4/8/16 on the Llama-shaped products)
    static constexpr int GROUP_M = 4;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int CH = BK / 16;        // 16-byte chunks per K-contiguous row
    static constexpr int RPS = 256 / BK;      // rows per 256-byte sweep of the LDS banks
    static constexpr int KSTEPS = BK / 32;
    static constexpr int LDB_NN = BN + 8;     // dword pitch of the register-transposed layout
    static constexpr int A_BYTES = BM * BK;
    static constexpr int CHB = BN / 16;       // 16-byte chunks per K-major row of B (TR)
    static constexpr int RPSB = 256 / BN;     // K-major rows per 256-byte sweep of the LDS banks (TR)
    static constexpr int B_BYTES = (TRANSB || TR) ? BN * BK : (BK / 4) * LDB_NN * 4;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int EPI_PITCH = WN + 8;                     // dwords per row of the epilogue staging region
    static constexpr int EPI_BYTES = WAVES_M * WAVES_N * 32 * EPI_PITCH * 4;
    static constexpr int LDS_BYTES = NS * STAGE_BYTES > EPI_BYTES ? NS * STAGE_BYTES : EPI_BYTES;
    static constexpr int SLOTS_A = BM * CH / NT;
    static constexpr int SLOTS_B = BN * CH / NT;                 // transB, and TR (BK rows of BN/16 chunks)
    static constexpr int BLKS_B = (BK / 4) * (BN / 4) / NT;      // register-transposed B
    static constexpr int NB = (TRANSB || TR) ? SLOTS_B : BLKS_B;
    static_assert(!TR || (!TRANSB && (BN == 128 || BN == 256)), "TR is for the K-strided B operand");
    static_assert(BM * CH % NT == 0 && BN * CH % NT == 0, "tile/threads mismatch");
    static_assert(((BK / 4) * (BN / 4)) % NT == 0, "tile/threads mismatch");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

// Consecutive workgroup ids go to different XCDs (8 per chip): give every XCD a contiguous range of tile
// numbers, and walk tiles in groups of GROUP tile-rows so that one XCD's resident tiles share A and B panels in
// its L2 (measured on an 8192^3 product: 22 % L2 misses with this map, 51 % without the XCD step).  `bid` counts
// from the first workgroup of the product: for the second product of a paired launch that rotates the XCD numbers by
// (first product's workgroups) % 8, which still hands every hardware XCD one contiguous range of tile numbers.
template <int GROUP>
__device__ __forceinline__ void tile_of_block(int bid, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
    const int ntiles = tiles_m * tiles_n;
    const int xcd = bid & 7, q = bid >> 3;
    const int base = ntiles >> 3, rem = ntiles & 7;
    const int pid = xcd * base + (xcd < rem ? xcd : rem) + q;
    const int per_group = GROUP * tiles_n;
    const int group = pid / per_group;
    const int first_m = group * GROUP;
    const int gsize = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
    const int in_group = pid % per_group;
    tile_m = first_m + in_group % gsize;
    tile_n = in_group / gsize;
}

// 4x4 byte transpose: r[j] holds bytes (n..n+3) of k-row j; returns t with t[e] = (r0.b[e], r1.b[e], r2.b[e], r3.b[e]).
__device__ __forceinline__ uint4 transpose4x4(const uint32_t (&r)[4]) {
    const uint32_t u0 = __builtin_amdgcn_perm(r[1], r[0], 0x05010400u);
    const uint32_t u1 = __builtin_amdgcn_perm(r[1], r[0], 0x07030602u);
    const uint32_t v0 = __builtin_amdgcn_perm(r[3], r[2], 0x05010400u);
    const uint32_t v1 = __builtin_amdgcn_perm(r[3], r[2], 0x07030602u);
    uint4 t;
    t.x = __builtin_amdgcn_perm(v0, u0, 0x05040100u);
    t.y = __builtin_amdgcn_perm(v0, u0, 0x07060302u);
    t.z = __builtin_amdgcn_perm(v1, u1, 0x05040100u);
    t.w = __builtin_amdgcn_perm(v1, u1, 0x07060302u);
    return t;
}

// Operand fragments of one wavefront for one K sub-step (32 bytes of K).  bt holds the halves of the B fragments as
// the transposing reads deliver them, until wait_frags() has assembled them into b.
template <class Cfg>
struct Frags {
    v4i a[Cfg::TM], b[Cfg::TN];
    v2i bt[Cfg::TN][2];
};

// Requests the fragments of K sub-step KK of one LDS stage.
template <class Cfg, bool TRANSB, int BK, int KK>
__device__ __forceinline__ void load_frags(const unsigned char* sa, const unsigned char* sb, int wave_m, int wave_n,
                                           int lrow, int half, Frags<Cfg>& f) {
    constexpr int CH = Cfg::CH, RPS = Cfg::RPS;
    const int g = 2 * KK + half;
#pragma unroll
    for (int i = 0; i < Cfg::TM; ++i) {
        const int row = wave_m * Cfg::WM + i * 32 + lrow;
        const int pc = g ^ ((row / RPS) % CH);
        f.a[i] = *reinterpret_cast<const v4i*>(sa + row * BK + 16 * pc);
    }
#pragma unroll
    for (int j = 0; j < Cfg::TN; ++j) {
        const int col = wave_n * Cfg::WN + j * 32 + lrow;
        if constexpr (TRANSB) {
            const int pc = g ^ ((col / RPS) % CH);
            f.b[j] = *reinterpret_cast<const v4i*>(sb + col * BK + 16 * pc);
        } else if constexpr (Cfg::IS_TR) {
            // A group of 16 lanes reads an 8(k) x 16(n) byte block: lane i supplies the address of 8 bytes of
            // K-major row k0 + i/2 at column offset 8*(i%2) and receives the 8 k-values of column i of the block.
            // Rows are XOR-swizzled by 2*((row / RPSB) % (CHB/2)) chunks, which keeps the two lane groups of one
            // read on even and odd chunks respectively (no bank conflicts) and is undone by the DMA addresses.  The
            // swizzle term depends on the lane only, so one address per column block serves every K sub-step through
            // the instruction's immediate offset.
            const int lane16 = (lrow & 15), gsel = lrow >> 4;
            const int chunk = (wave_n * Cfg::WN + j * 32) / 16 + gsel;
            const int s8 = lane16 >> 1;
            const int pc = chunk ^ (2 * ((s8 / Cfg::RPSB) % (Cfg::CHB / 2)));
            const uint32_t addr =
                (uint32_t)(uintptr_t)HALO_LDS_PTR(sb + (16 * half + s8) * Cfg::BN_ + 16 * pc + 8 * (lane16 & 1));
            // Issued as inline assembly: seen as an LDS read, the compiler would order it after every outstanding
            // global->LDS transfer (s_waitcnt vmcnt(0)), which empties the ring at every K step.  wait_frags() waits
            // for the data before the MFMAs that use it.
            asm volatile("ds_read_b64_tr_b8 %0, %2 offset:%3\n\tds_read_b64_tr_b8 %1, %2 offset:%4"
                         : "=&v"(f.bt[j][0]), "=&v"(f.bt[j][1])
                         : "v"(addr), "n"(32 * KK * Cfg::BN_), "n"((32 * KK + 8) * Cfg::BN_));
        } else {
            const uint32_t* sbw = reinterpret_cast<const uint32_t*>(sb);
#pragma unroll
            for (int w = 0; w < 4; ++w) f.b[j][w] = (int)sbw[(4 * g + w) * Cfg::LDB_NN + col];
        }
    }
}

// Waits for the transposing LDS reads issued by load_frags (the compiler does not track them) and assembles the B
// fragments.  The registers are operands of the wait, so nothing that uses them can move above it.
template <class Cfg>
__device__ __forceinline__ void wait_frags(Frags<Cfg>& f) {
    auto& bt = f.bt;
    if constexpr (Cfg::TN == 1) {
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bt[0][0]), "+v"(bt[0][1]));
    } else if constexpr (Cfg::TN == 2) {
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bt[0][0]), "+v"(bt[0][1]), "+v"(bt[1][0]), "+v"(bt[1][1]));
    } else {
        static_assert(Cfg::TN == 4, "B fragments per wavefront");
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(bt[0][0]), "+v"(bt[0][1]), "+v"(bt[1][0]), "+v"(bt[1][1]), "+v"(bt[2][0]), "+v"(bt[2][1]),
                       "+v"(bt[3][0]), "+v"(bt[3][1]));
    }
#pragma unroll
    for (int j = 0; j < Cfg::TN; ++j) {
        f.b[j][0] = bt[j][0][0]; f.b[j][1] = bt[j][0][1]; f.b[j][2] = bt[j][1][0]; f.b[j][3] = bt[j][1][1];
    }
}

// Scheduling recipe for one LDS stage, written as sched_group_barrier groups in pipeline order:
//   READS LDS reads (fragments of sub-step 0);
//   for every sub-step but the last: MFMAS times { 1 MFMA, up to PER LDS reads (fragments of the next sub-step) },
//                                    then the VM global->LDS DMA instructions the caller placed there;
//   the MFMAs of the last sub-step.
// Reads behind MFMAs keep the matrix pipe from draining while a wave waits for LDS; slicing the DMA instructions of
// a K step over the sub-steps keeps the vector-memory queue from filling up in one burst.
template <int IDX, int TOTAL, int MFMAS, int READS, int VM>
struct StageSched {
    static __device__ __forceinline__ void run() {
        constexpr int Q = IDX % MFMAS;                       // MFMA number inside its sub-step
        constexpr int PER = (READS + MFMAS - 1) / MFMAS;
        constexpr int LEFT = READS - Q * PER;
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if constexpr (LEFT > 0) __builtin_amdgcn_sched_group_barrier(0x100, LEFT < PER ? LEFT : PER, 0);
        if constexpr (VM > 0 && Q == MFMAS - 1) __builtin_amdgcn_sched_group_barrier(0x020, VM, 0);
        StageSched<IDX + 1, TOTAL, MFMAS, READS, VM>::run();
    }
};
template <int TOTAL, int MFMAS, int READS, int VM>
struct StageSched<TOTAL, TOTAL, MFMAS, READS, VM> {
    static __device__ __forceinline__ void run() { __builtin_amdgcn_sched_group_barrier(0x008, MFMAS, 0); }
};

struct NoBetween {
    __device__ __forceinline__ void operator()(int) const {}
};

// Sub-step KK of one LDS stage: the fragments of sub-step KK+1 are requested while the MFMAs of sub-step KK run.
template <class Cfg, bool TRANSB, int BK, int KK, class Between>
__device__ __forceinline__ void mma_substep(const unsigned char* sa, const unsigned char* sb, int wave_m, int wave_n,
                                            int lrow, int half, v16i (&acc)[Cfg::TM][Cfg::TN], const Between& between,
                                            Frags<Cfg>& cur) {
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    if constexpr (Cfg::IS_TR) wait_frags<Cfg>(cur);
    Frags<Cfg> nxt;
    if constexpr (KK + 1 < Cfg::KSTEPS) load_frags<Cfg, TRANSB, BK, KK + 1>(sa, sb, wave_m, wave_n, lrow, half, nxt);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur.a[i], cur.b[j], acc[i][j], 0, 0, 0);
    if constexpr (KK + 1 < Cfg::KSTEPS) {
        between(KK);
        mma_substep<Cfg, TRANSB, BK, KK + 1, Between>(sa, sb, wave_m, wave_n, lrow, half, acc, between, nxt);
    }
}

// All MFMAs of one LDS stage.  between(kk) is called after the MFMAs of sub-step kk (all but the last): the DMA kernel
// issues a slice of the next K step's global->LDS loads there; VM = number of such instructions per call (for the
// scheduling recipe).
template <class Cfg, bool TRANSB, int BK, int VM = 0, class Between = NoBetween>
__device__ __forceinline__ void mma_stage(const unsigned char* sa, const unsigned char* sb, int wave_m, int wave_n,
                                          int lrow, int half, v16i (&acc)[Cfg::TM][Cfg::TN],
                                          const Between& between = Between()) {
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    // LDS read instructions per sub-step that the scheduler sees (the transposing reads are inline assembly)
    constexpr int READS = TM + (TRANSB ? TN : (Cfg::IS_TR ? 0 : 4 * TN));
    constexpr int MFMAS = TM * TN;
    Frags<Cfg> first;
    load_frags<Cfg, TRANSB, BK, 0>(sa, sb, wave_m, wave_n, lrow, half, first);
    mma_substep<Cfg, TRANSB, BK, 0, Between>(sa, sb, wave_m, wave_n, lrow, half, acc, between, first);
    __builtin_amdgcn_sched_group_barrier(0x100, READS, 0);
    StageSched<0, (Cfg::KSTEPS - 1) * MFMAS, MFMAS, READS, VM>::run();
}

// Epilogue.  The accumulator layout (a lane owns one column of a 32x32 tile) would give 2- or 4-byte stores
// scattered over 32 rows, so each wavefront first drops a 32-row slab of its sub-tile into a private LDS region
// (one dword per element, row pitch WN+8 dwords: conflict-free writes) and reads it back four consecutive
// columns per lane, which turns the global stores into 16-byte (int32/fp32) or 8-byte (bf16) pieces of fully
// covered rows.  Only the owning wavefront touches its region, so after the first barrier the wavefront only has to
// order its own LDS writes and reads (the lanes of a wavefront run in lockstep; the wavefront-scope fences keep the
// compiler from moving the accesses across the slab boundaries).
// PRE: the accumulator registers already hold the fp32 values to store, as bit patterns (lowrank_prepare).
template <class Cfg, bool PRE = false>
__device__ __forceinline__ void epilogue(const GemmArgs& a, int64_t m0, int64_t n0, int wave, int wave_m, int wave_n,
                                         int lane, const v16i (&acc)[Cfg::TM][Cfg::TN], unsigned char* smem) {
    constexpr int WN = Cfg::WN, PITCH = Cfg::EPI_PITCH;
    constexpr int LPR = WN / 4;            // lanes per row when reading back
    constexpr int RPP = 64 / LPR;          // rows per read-back pass
    const int lrow = lane & 31, half = lane >> 5;
    uint32_t* region = reinterpret_cast<uint32_t*>(smem) + wave * 32 * PITCH;
    __syncthreads();                       // every wavefront is done with the operand stages

    const int cc = (lane % LPR) * 4;
    const int64_t col = n0 + wave_n * WN + cc;
    const bool col_any = col < a.N, col_all = col + 4 <= a.N;
    float cs[4] = {1.0f, 1.0f, 1.0f, 1.0f};
    if (!PRE && a.C && a.col_scale) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < a.N) cs[e] = a.col_scale[col + e];
    }
#pragma unroll
    for (int i = 0; i < Cfg::TM; ++i) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the read-back of the previous slab is complete
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                region[(8 * (r / 4) + 4 * half + (r % 4)) * PITCH + j * 32 + lrow] = (uint32_t)acc[i][j][r];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the slab is written before other lanes read it
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int p = 0; p < 32 / RPP; ++p) {
            const int rr = p * RPP + lane / LPR;
            const int4 v = *reinterpret_cast<const int4*>(region + rr * PITCH + cc);
            const int64_t row = m0 + wave_m * Cfg::WM + i * 32 + rr;
            if (row >= a.M || !col_any) continue;
            const int vv[4] = {v.x, v.y, v.z, v.w};
            if (!PRE && a.acc_out) {
                int32_t* dst = a.acc_out + row * a.ld_acc + col;
                if (col_all) {
                    *reinterpret_cast<int4*>(dst) = v;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e < a.N) dst[e] = vv[e];
                }
            }
            if (a.C) {
                float f[4];
                if constexpr (PRE) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) f[e] = __int_as_float(vv[e]);
                } else {
                    const float rs = a.row_scale ? a.row_scale[row] : 1.0f;
#pragma unroll
                    for (int e = 0; e < 4; ++e) f[e] = ((float)vv[e] * rs) * cs[e];
                }
                if (a.c_is_f32) {
                    float* dst = reinterpret_cast<float*>(a.C) + row * a.ldc + col;
                    if (col_all) {
                        *reinterpret_cast<float4*>(dst) = make_float4(f[0], f[1], f[2], f[3]);
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
}

// Epilogue of a product whose output is then un-rotated on the left (level 2, E_X = H^T ( ... )): the accumulators are
// scaled, (float(acc) * row_scale[row]) * post_scale, and the eight lowest strides of the left-hand Walsh-Hadamard
// rotation run on the 256 rows of the tile before anything is stored, in ascending order and with every add and
// subtract a separately rounded fp32 operation, exactly as a pass over memory would do them.  Row index inside the
// tile = [wave_m | tile i (2 bits) | r >> 2 (2 bits) | lane half | r & 3 (2 bits)], so strides 1, 2 pair registers,
// stride 4 pairs the two halves of the wavefront, strides 8 .. 64 pair registers again, and stride 128 pairs this
// wavefront with the one holding the other 128 rows of the same columns: that last stage is folded into the slab
// staging of the store (each wavefront reads its own slab and its partner's).  The columns are independent, so one
// 32-column tile of the wavefront is taken through all of this at a time (64 live values per lane).  No normalisation:
// the 1/sqrt(block) of the rotation is applied after its last stride, by whoever runs it.
template <class Cfg, bool PRE = false>
__device__ __forceinline__ void epilogue_left8(const GemmArgs& a, int64_t m0, int64_t n0, int wave, int wave_m, int wave_n,
                                               int lane, const v16i (&acc)[Cfg::TM][Cfg::TN], unsigned char* smem) {
    static_assert(Cfg::TM == 4 && Cfg::WAVES_M_ == 2, "256-row tiles, two wavefronts down the rows");
    constexpr int WN = Cfg::WN, TM = Cfg::TM, TN = Cfg::TN;
    constexpr int PITCH = 32 + 8;          // dwords per row of a staged 32 x 32 slab: conflict-free writes, 16-byte rows
    constexpr int SLAB = 32 * PITCH;       // one slab; a wavefront's region holds two (64 rows of one column tile)
    static_assert(1024 + 8 * 2 * SLAB * 4 <= Cfg::LDS_BYTES, "row scales and staging regions fit the operand stages' LDS");
    const int lrow = lane & 31, half = lane >> 5;
    float* s_scale = reinterpret_cast<float*>(smem);
    float* region = reinterpret_cast<float*>(smem + 1024) + wave * 2 * SLAB;
    const float* partner = reinterpret_cast<const float*>(smem + 1024) + (wave ^ Cfg::WAVES_N_) * 2 * SLAB;
    __syncthreads();                       // every wavefront is done with the operand stages
    const int tid = wave * 64 + lane;
    if constexpr (!PRE) {
        if (tid < 256) s_scale[tid] = a.row_scale ? a.row_scale[m0 + tid] : 1.0f;  // M is a multiple of 256
        __syncthreads();
    }
    const float post = a.post_scale ? *a.post_scale : 1.0f;                          // x * 1.0f is x
    const float sgn = half ? -1.0f : 1.0f;                   // lower half: a + b;  upper half: a - b = partner - own
    const float sgn_w = wave_m ? -1.0f : 1.0f;               // the same for the two wavefronts of stride 128
    const int addr = (lane ^ 32) << 2;
    const int cc = (lane & 7) * 4;                           // read-back: 8 lanes per 32-column row, 8 rows per pass

#pragma unroll
    for (int j = 0; j < TN; ++j) {
        float f[TM][16];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if constexpr (PRE) {
                    f[i][r] = __int_as_float(acc[i][j][r]);
                } else {
                    const float rs = s_scale[wave_m * 128 + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3)];
                    f[i][r] = ((float)acc[i][j][r] * rs) * post;
                }
            }
        // strides 1, 2, (4), 8, 16: bits 0, 1, 2, 3 of r; stride 4 across the lane halves in between
#pragma unroll
        for (int bit = 0; bit < 4; ++bit) {
            if (bit == 2) {
#pragma unroll
                for (int i = 0; i < TM; ++i) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float p = __int_as_float(__builtin_amdgcn_ds_bpermute(addr, __float_as_int(f[i][r])));
                        f[i][r] = __builtin_fmaf(f[i][r], sgn, p);             // the product is exact: one rounded add/sub
                    }
                    __builtin_amdgcn_sched_barrier(0);       // sixteen exchanges in flight at a time, not sixty-four
                }
            }
            const int h = 1 << bit;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if ((r & h) == 0) {
                        const float x = f[i][r], y = f[i][r | h];
                        f[i][r] = x + y;
                        f[i][r | h] = x - y;
                    }
        }
        // strides 32, 64: the four 32-row tiles of the wavefront
#pragma unroll
        for (int bit = 0; bit < 2; ++bit) {
            const int h = 1 << bit;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                if ((i & h) == 0) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float x = f[i][r], y = f[i | h][r];
                        f[i][r] = x + y;
                        f[i | h][r] = x - y;
                    }
                }
        }
        // stride 128 and the store, 64 rows (two slabs) at a time: the slabs go to the wavefront's region, then every
        // lane combines four consecutive columns of its own and its partner's slabs
        const int64_t col = n0 + wave_n * WN + j * 32 + cc;
        const bool col_any = col < a.N, col_all = col + 4 <= a.N;
#pragma unroll
        for (int hs = 0; hs < TM / 2; ++hs) {
            if (j > 0 || hs > 0) __syncthreads();      // the previous slabs have been read by both wavefronts
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    region[i * SLAB + (8 * (r / 4) + 4 * half + (r % 4)) * PITCH + lrow] = f[2 * hs + i][r];
            __syncthreads();                           // the partner's slabs are written too
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int rr = p * 8 + (lane >> 3);            // row inside these 64
                const int off = (rr >> 5) * SLAB + (rr & 31) * PITCH + cc;
                const float4 own = *reinterpret_cast<const float4*>(region + off);
                const float4 oth = *reinterpret_cast<const float4*>(partner + off);
                // wave_m == 0: own + other;  wave_m == 1: other - own (the product own * -1 is exact)
                const float v[4] = {__builtin_fmaf(own.x, sgn_w, oth.x), __builtin_fmaf(own.y, sgn_w, oth.y),
                                    __builtin_fmaf(own.z, sgn_w, oth.z), __builtin_fmaf(own.w, sgn_w, oth.w)};
                if (!col_any) continue;
                const int64_t row = m0 + wave_m * Cfg::WM + hs * 64 + rr;
                float* dst = reinterpret_cast<float*>(a.C) + row * a.ldc + col;
                if (col_all) {
                    *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e < a.N) dst[e] = v[e];
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);     // finish this column tile before the next one starts
    }
}

// Low-rank side product (a LoRA branch next to the quantised product): turns the int32 accumulators, in place, into the
// fp32 values
//   ((float(acc) * row_scale[row]) * col_scale[col]) * post_scale  +  sum_k lr_a[row, k] * lr_b[k, col],
// the first part rounded exactly as the plain epilogues round it, the sum added by matrix instructions with the scaled
// accumulator as their addend.  The registers then hold float bit patterns and the PRE variants of the epilogues take
// over.
template <class Cfg>
__device__ __forceinline__ void lowrank_prepare(const GemmArgs& a, int64_t m0, int64_t n0, int wave, int wave_m, int wave_n,
                                                int lane, v16i (&acc)[Cfg::TM][Cfg::TN], unsigned char* smem) {
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    static_assert(Cfg::BM_ * 4 <= 1024, "row scales fit below the staging regions of the left-hand epilogue");
    typedef float v16f __attribute__((ext_vector_type(16)));
    const int lrow = lane & 31, half = lane >> 5;
    float* s_scale = reinterpret_cast<float*>(smem);
    __syncthreads();                       // every wavefront is done with the operand stages
    for (int t = wave * 64 + lane; t < Cfg::BM_; t += Cfg::NT) {
        const int64_t row = m0 + t;
        s_scale[t] = (a.row_scale && row < a.M) ? a.row_scale[row] : 1.0f;
    }
    __syncthreads();
    const float post = a.post_scale ? *a.post_scale : 1.0f;                          // x * 1.0f is x
    float cs[TN];
    int64_t colj[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        colj[j] = n0 + wave_n * Cfg::WN + j * 32 + lrow;
        cs[j] = (a.col_scale && colj[j] < a.N) ? a.col_scale[colj[j]] : 1.0f;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float rs = s_scale[wave_m * Cfg::WM + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3)];
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j][r] = __float_as_int((((float)acc[i][j][r] * rs) * cs[j]) * post);
        }
    // The low-rank sum, sixteen ranks at a time, by bf16 matrix instructions (v_mfma_f32_32x32x16_bf16: lane l supplies
    // row / column l % 32, ranks 8 (l / 32) .. + 8; the result layout is that of the int8 instruction).  fp32 operands
    // are split exactly into three bf16 pieces (8 + 8 + 8 mantissa bits, x = hi + mid + lo); every product of two pieces
    // is exact and is accumulated in fp32.  The products kept are those down to 2^-16 of the full one (all of them when
    // one operand is bf16 already): what is dropped is below 2^-23 of |a b|, an fp32 rounding.  Smallest terms first.
    // Every address is clamped into its matrix, so that all loads are unconditional and in flight together; what lies
    // outside is zeroed afterwards.
    typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    auto hi16 = [](uint32_t x, uint32_t y) { return __builtin_amdgcn_perm(y, x, 0x07060302u); };
    auto split8 = [&](const float (&x)[8], v8bf& h, v8bf& m, v8bf& l) {
        uint32_t ph[8], pm[8], pl[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            ph[e] = __float_as_uint(x[e]) & 0xFFFF0000u;
            const float r1 = x[e] - __uint_as_float(ph[e]);
            pm[e] = __float_as_uint(r1) & 0xFFFF0000u;
            pl[e] = __float_as_uint(r1 - __uint_as_float(pm[e]));
        }
        h = __builtin_bit_cast(v8bf, (v4u){hi16(ph[0], ph[1]), hi16(ph[2], ph[3]), hi16(ph[4], ph[5]), hi16(ph[6], ph[7])});
        m = __builtin_bit_cast(v8bf, (v4u){hi16(pm[0], pm[1]), hi16(pm[2], pm[3]), hi16(pm[4], pm[5]), hi16(pm[6], pm[7])});
        l = __builtin_bit_cast(v8bf, (v4u){hi16(pl[0], pl[1]), hi16(pl[2], pl[3]), hi16(pl[4], pl[5]), hi16(pl[6], pl[7])});
    };
    int64_t rowc[TM], colc[TN];
    bool row_ok[TM], col_ok[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int64_t row = m0 + wave_m * Cfg::WM + i * 32 + lrow;
        row_ok[i] = row < a.M;
        rowc[i] = row_ok[i] ? row : a.M - 1;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        col_ok[j] = colj[j] < a.N;
        colc[j] = col_ok[j] ? colj[j] : a.N - 1;
    }
    for (int c0 = 0; c0 < a.lr_rank; c0 += 16) {
        const bool k_ok = c0 + 8 * half < a.lr_rank;            // the rank is a multiple of 8
        const int kb = k_ok ? c0 + 8 * half : 0;
        float4 araw[TM][2];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const float4* p = reinterpret_cast<const float4*>(a.lr_a + rowc[i] * a.lr_rank + kb);
            araw[i][0] = p[0];
            araw[i][1] = p[1];
        }
        v8bf bh[TN], bm[TN], bl[TN];
        if (a.lr_b_bf16) {                 // uniform
            uint4 braw[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j)
                braw[j] = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(a.lr_b) + colc[j] * a.lr_rank + kb);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (!(k_ok && col_ok[j])) braw[j] = make_uint4(0u, 0u, 0u, 0u);
                bh[j] = __builtin_bit_cast(v8bf, braw[j]);
            }
        } else {
            float4 braw[TN][2];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(a.lr_b) + colc[j] * a.lr_rank + kb);
                braw[j][0] = p[0];
                braw[j][1] = p[1];
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const bool in = k_ok && col_ok[j];
                const float x[8] = {in ? braw[j][0].x : 0.0f, in ? braw[j][0].y : 0.0f, in ? braw[j][0].z : 0.0f,
                                    in ? braw[j][0].w : 0.0f, in ? braw[j][1].x : 0.0f, in ? braw[j][1].y : 0.0f,
                                    in ? braw[j][1].z : 0.0f, in ? braw[j][1].w : 0.0f};
                split8(x, bh[j], bm[j], bl[j]);
            }
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const bool in = k_ok && row_ok[i];
            const float x[8] = {in ? araw[i][0].x : 0.0f, in ? araw[i][0].y : 0.0f, in ? araw[i][0].z : 0.0f,
                                in ? araw[i][0].w : 0.0f, in ? araw[i][1].x : 0.0f, in ? araw[i][1].y : 0.0f,
                                in ? araw[i][1].z : 0.0f, in ? araw[i][1].w : 0.0f};
            v8bf ah, am, al;
            split8(x, ah, am, al);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                v16f f = __builtin_bit_cast(v16f, acc[i][j]);
                if (a.lr_b_bf16) {
                    f = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh[j], f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bh[j], f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh[j], f, 0, 0, 0);
                } else {
                    f = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh[j], f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl[j], f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bm[j], f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bh[j], f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bm[j], f, 0, 0, 0);
                    f = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh[j], f, 0, 0, 0);
                }
                acc[i][j] = __builtin_bit_cast(v16i, f);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------ dma main loop
// Both operands go through the DMA ring.  K must be a multiple of BK (the DMA cannot zero-fill a K tail).
// LEFT: this instance also carries the epilogue that runs the low strides of a left-hand rotation (its own instance, so
// that the register spills of that epilogue stay out of the kernels that never take it).
// LR: this instance also carries the low-rank side product (lowrank_prepare), again its own instance.
template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool TRANSB, int NS, bool LEFT = false, bool LR = false>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N)
gemm_i8_dma_kernel(GemmArgs a, int tiles_m, int tiles_n, GemmArgs a2, int tiles_m2, int tiles_n2, unsigned blocks1) {
    using Cfg = GemmCfg<BM, BN, BK, WAVES_M, WAVES_N, TRANSB, NS, !TRANSB>;
    // A second, independent product may ride in the same launch (workgroups from blocks1 on): the tail and the
    // epilogue of one then overlap the main loop of the other.
    int bid = blockIdx.x;
    if (blockIdx.x >= blocks1) {
        bid -= blocks1;
        a = a2;
        tiles_m = tiles_m2;
        tiles_n = tiles_n2;
    }
    constexpr int NT = Cfg::NT, CH = Cfg::CH, RPS = Cfg::RPS, TM = Cfg::TM, TN = Cfg::TN;
    constexpr int D = NS - 1;                                     // K steps in flight
    constexpr int LOADS = Cfg::SLOTS_A + Cfg::SLOTS_B;            // DMA loads per thread per K step
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_m = wave / WAVES_N;
    const int wave_n = wave % WAVES_N;
    const int lrow = lane & 31, half = lane >> 5;

    int tile_m, tile_n;
    tile_of_block<Cfg::GROUP_M>(bid, tiles_m, tiles_n, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * BM;
    const int64_t n0 = (int64_t)tile_n * BN;
    const int nk = (int)(a.K / BK);

    // ---- per-thread source addresses (fixed over the K loop); rows beyond the matrix are clamped, their results
    // are never stored
    const int8_t* a_src[Cfg::SLOTS_A];
#pragma unroll
    for (int i = 0; i < Cfg::SLOTS_A; ++i) {
        const int p = tid + i * NT;
        const int row = p / CH, pc = p % CH;
        const int g = pc ^ ((row / RPS) % CH);
        int64_t gr = m0 + row;
        if (gr > a.M - 1) gr = a.M - 1;
        a_src[i] = a.A + gr * a.lda + 16 * g;
    }
    const int8_t* b_src[Cfg::SLOTS_B];
#pragma unroll
    for (int i = 0; i < Cfg::SLOTS_B; ++i) {
        const int p = tid + i * NT;
        if constexpr (TRANSB) {
            const int row = p / CH, pc = p % CH;
            const int g = pc ^ ((row / RPS) % CH);
            int64_t gr = n0 + row;
            if (gr > a.N - 1) gr = a.N - 1;
            b_src[i] = a.B + gr * a.ldb + 16 * g;
        } else {
            // K-major rows of BN bytes; LDS slot (row, pc) holds chunk pc ^ swizzle(row) of that row.  A chunk whose
            // columns start beyond the row pitch is replaced by chunk 0 (those columns are never stored).
            const int row = p / Cfg::CHB, pc = p % Cfg::CHB;
            const int c = pc ^ (2 * ((row / Cfg::RPSB) % (Cfg::CHB / 2)));
            int64_t colb = n0 + 16 * c;
            if (colb >= a.ldb) colb = 0;
            b_src[i] = a.B + (int64_t)row * a.ldb + colb;
        }
    }
    const int64_t b_step = TRANSB ? (int64_t)BK : (int64_t)BK * a.ldb;

    // DMA of K step src into ring slot t % NS.  lo..hi select a sub-range of the step's DMA instructions (A slots
    // first, then B slots), so that the caller can thread them between the MFMAs instead of issuing one burst.
    auto issue_dma = [&](int t, int src, int lo = 0, int hi = 1 << 20) {
        unsigned char* sa = smem + (t % NS) * Cfg::STAGE_BYTES;
        unsigned char* sb = sa + Cfg::A_BYTES;
#pragma unroll
        for (int i = 0; i < Cfg::SLOTS_A; ++i) {
            if (i < lo || i >= hi) continue;
            __builtin_amdgcn_global_load_lds(HALO_GLOBAL_PTR(a_src[i] + (int64_t)src * BK),
                                             HALO_LDS_PTR(sa + (wave * 64 + i * NT) * 16), 16, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < Cfg::SLOTS_B; ++i) {
            if (Cfg::SLOTS_A + i < lo || Cfg::SLOTS_A + i >= hi) continue;
            __builtin_amdgcn_global_load_lds(HALO_GLOBAL_PTR(b_src[i] + (int64_t)src * b_step),
                                             HALO_LDS_PTR(sb + (wave * 64 + i * NT) * 16), 16, 0, 0);
        }
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    if (nk > 0) {
        // Every iteration issues exactly one K step (beyond the end: the last step again, into a ring slot nobody
        // reads), so the loop body is one straight block with a constant wait count.
        for (int t = 0; t < D; ++t) issue_dma(t, t < nk ? t : nk - 1);
        for (int kt = 0; kt < nk; ++kt) {
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((D - 1) * LOADS) : "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            // ring slot (kt-1) % NS: everyone is past reading it
            const int src = kt + D < nk ? kt + D : nk - 1;
            const unsigned char* sa = smem + (kt % NS) * Cfg::STAGE_BYTES;
            if constexpr (Cfg::KSTEPS > 1 && LOADS % (Cfg::KSTEPS - 1) == 0) {
                constexpr int PER = LOADS / (Cfg::KSTEPS - 1);
                auto between = [&](int kk) { issue_dma(kt + D, src, kk * PER, (kk + 1) * PER); };
                mma_stage<Cfg, TRANSB, BK, PER>(sa, sa + Cfg::A_BYTES, wave_m, wave_n, lrow, half, acc, between);
            } else {
                issue_dma(kt + D, src);
                mma_stage<Cfg, TRANSB, BK>(sa, sa + Cfg::A_BYTES, wave_m, wave_n, lrow, half, acc);
            }
        }
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    }
    if constexpr (LR) {
        if (a.lr_rank > 0) {               // uniform over the workgroup
            lowrank_prepare<Cfg>(a, m0, n0, wave, wave_m, wave_n, lane, acc, smem);
            if constexpr (LEFT) {
                if (a.left_stages != 0) {
                    epilogue_left8<Cfg, true>(a, m0, n0, wave, wave_m, wave_n, lane, acc, smem);
                    return;
                }
            }
            epilogue<Cfg, true>(a, m0, n0, wave, wave_m, wave_n, lane, acc, smem);
            return;
        }
    }
    if constexpr (LEFT) {
        if (a.left_stages != 0) {          // uniform over the workgroup
            epilogue_left8<Cfg>(a, m0, n0, wave, wave_m, wave_n, lane, acc, smem);
            return;
        }
    }
    epilogue<Cfg>(a, m0, n0, wave, wave_m, wave_n, lane, acc, smem);
}

// ------------------------------------------------------------------------------------------------ staged main loop
template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool TRANSB>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N)
gemm_i8_staged_kernel(GemmArgs a, int tiles_m, int tiles_n) {
    using Cfg = GemmCfg<BM, BN, BK, WAVES_M, WAVES_N, TRANSB, 2>;
    constexpr int NT = Cfg::NT, CH = Cfg::CH, RPS = Cfg::RPS, TM = Cfg::TM, TN = Cfg::TN;
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_m = wave / WAVES_N;
    const int wave_n = wave % WAVES_N;
    const int lrow = lane & 31, half = lane >> 5;

    int tile_m, tile_n;
    tile_of_block<Cfg::GROUP_M>((int)blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * BM;
    const int64_t n0 = (int64_t)tile_n * BN;

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
    const int8_t* b_src[Cfg::NB];
    int b_koff[Cfg::NB];
    bool b_ok[Cfg::NB];
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
    uint4 b_reg[Cfg::NB];

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
                b_reg[i] = transpose4x4(r);
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

    const int nk = (int)((a.K + BK - 1) / BK);
    if (nk > 0) {
        load_global(0);
        store_lds(0);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const bool more = kt + 1 < nk;
            if (more) load_global((int64_t)(kt + 1) * BK);
            const unsigned char* sa = smem + (kt & 1) * Cfg::STAGE_BYTES;
            mma_stage<Cfg, TRANSB, BK>(sa, sa + Cfg::A_BYTES, wave_m, wave_n, lrow, half, acc);
            if (more) store_lds((kt + 1) & 1);
            __syncthreads();
        }
    }
    epilogue<Cfg>(a, m0, n0, wave, wave_m, wave_n, lane, acc, smem);
}

// ------------------------------------------------------------------------------------------------ ceiling probe
// iters x 16 MFMAs per wavefront on operands read once from `operands` (4 KB: 16 bytes per lane and fragment, four
// fragments), nothing else in the loop: the rate the matrix pipes sustain on this machine for this operand data.
__global__ void __launch_bounds__(512) mfma_i8_probe_kernel(const int8_t* operands, int iters, int32_t* sink) {
    const int lane = threadIdx.x & 63;
    v4i f[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = *reinterpret_cast<const v4i*>(operands + (i * 64 + lane) * 16);
    v16i acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < 16; ++m)
            acc[m % 8] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f[m % 2], f[2 + (m / 2) % 2], acc[m % 8], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (sink && s == 0x7fffffff) sink[0] = s;      // keeps the loop alive; practically never taken
}

// ------------------------------------------------------------------------------------------------ launch
// The dynamic-LDS limit of a kernel is raised once per kernel (and per process); call_once makes that safe when
// several host threads launch the same kernel for the first time.
template <class Kern>
hipError_t raise_lds_limit(Kern kern, int lds_bytes, std::once_flag* once, hipError_t* result) {
    std::call_once(*once, [&] {
        *result = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      lds_bytes);
    });
    return *result;
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool TRANSB, int NS, bool LEFT = false, bool LR = false>
hipError_t launch_dma(const GemmArgs& a, hipStream_t s, const GemmArgs* a2 = nullptr) {
    using Cfg = GemmCfg<BM, BN, BK, WAVES_M, WAVES_N, TRANSB, NS, !TRANSB>;
    const bool wants_left = a.left_stages != 0 || (a2 && a2->left_stages != 0);
    const bool wants_lr = a.lr_rank != 0 || (a2 && a2->lr_rank != 0);
    // The low-rank instances exist for the configurations the layer uses: K-contiguous B with 128-byte K steps or the
    // small tile, K-strided B with 256x256 (which then also carries the left-hand epilogue) or the small tile.
    constexpr bool kLeftShape = BM == 256 && WAVES_M == 2 && !TRANSB;
    constexpr bool kLrShape = TRANSB ? (BK == 128 || BM == 128) : (BK == 64);
    if constexpr (!LR && kLrShape) {
        if (wants_lr) return launch_dma<BM, BN, BK, WAVES_M, WAVES_N, TRANSB, NS, kLeftShape, true>(a, s, a2);
    }
    if (wants_lr && !LR) return hipErrorInvalidValue;
    if constexpr (!LEFT && !LR && kLeftShape) {
        if (wants_left) return launch_dma<BM, BN, BK, WAVES_M, WAVES_N, TRANSB, NS, true>(a, s, a2);
    }
    if (wants_left && !LEFT) return hipErrorInvalidValue;
    auto lr_ok = [](const GemmArgs& g) {
        if (g.lr_rank == 0) return true;
        return g.lr_rank > 0 && g.lr_rank <= kMaxLowRank && g.lr_rank % 8 == 0 && g.lr_a && g.lr_b && g.C && !g.acc_out;
    };
    if (!lr_ok(a) || (a2 && !lr_ok(*a2))) return hipErrorInvalidValue;
    static std::once_flag once;
    static hipError_t attr_result = hipSuccess;
    auto kern = gemm_i8_dma_kernel<BM, BN, BK, WAVES_M, WAVES_N, TRANSB, NS, LEFT, LR>;
    hipError_t e = raise_lds_limit(kern, Cfg::LDS_BYTES, &once, &attr_result);
    if (e != hipSuccess) return e;
    if (a.K % BK != 0 || (a2 && a2->K % BK != 0)) return hipErrorInvalidValue;
    // the epilogue that runs the low strides of a left-hand rotation: 256-row tiles that lie inside the matrix, fp32 out
    auto left_ok = [](const GemmArgs& g) {
        if (g.left_stages == 0) return true;
        return g.left_stages == 8 && g.M % 256 == 0 && g.C && g.c_is_f32 && !g.acc_out && (!g.col_scale || g.lr_rank) &&
               g.K > 0;
    };
    if (!left_ok(a) || (a2 && !left_ok(*a2))) return hipErrorInvalidValue;
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    const unsigned blocks1 = (unsigned)(tiles_m * tiles_n);
    int tiles_m2 = 0, tiles_n2 = 0;
    if (a2) {
        tiles_m2 = (int)((a2->M + BM - 1) / BM);
        tiles_n2 = (int)((a2->N + BN - 1) / BN);
    }
    hipLaunchKernelGGL(kern, dim3(blocks1 + (unsigned)(tiles_m2 * tiles_n2)), dim3(Cfg::NT), Cfg::LDS_BYTES, s, a, tiles_m,
                       tiles_n, a2 ? *a2 : a, tiles_m2, tiles_n2, blocks1);
    return hipGetLastError();
}

template <bool TRANSB>
hipError_t launch_staged(const GemmArgs& a, hipStream_t s) {
    using Cfg = GemmCfg<128, 128, 64, 2, 2, TRANSB, 2>;
    static std::once_flag once;
    static hipError_t attr_result = hipSuccess;
    if (a.left_stages != 0 || a.lr_rank != 0) return hipErrorInvalidValue;
    auto kern = gemm_i8_staged_kernel<128, 128, 64, 2, 2, TRANSB>;
    hipError_t e = raise_lds_limit(kern, Cfg::LDS_BYTES, &once, &attr_result);
    if (e != hipSuccess) return e;
    const int tiles_m = (int)((a.M + 127) / 128), tiles_n = (int)((a.N + 127) / 128);
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(Cfg::NT), Cfg::LDS_BYTES, s, a, tiles_m, tiles_n);
    return hipGetLastError();
}

// K step (bytes) of the DMA configurations 0..3.
constexpr int kStepOfConfig[4] = {64, 128, 128, 64};

// Tile configurations (halo_gemm_config in halo.h): macro tile M x N x K-step bytes, wavefronts, ring depth.
//   0: 256x256x64  8 (2x4) NS4      1: 256x256x128 8 (2x4) NS2      2: 256x128x128 8 (4x2) NS3
//   3: 128x128x64  4 (2x2) NS4      4: staged 128x128x64 (any K)
template <bool TRANSB>
hipError_t launch_by_shape(const GemmArgs& a, hipStream_t s) {
    auto tiles = [&](int bm, int bn) { return ((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn); };
    int cfg = a.config;
    if (cfg < 0) {
        // Enough 256x256 tiles to fill the 256 CUs: largest tile (128-byte K steps when both operands are
        // K-contiguous).  Otherwise halve the tile in N; small problems take 128x128 tiles.  The DMA loops need whole
        // K steps; a ragged K takes the staged loop.
        if (TRANSB) cfg = tiles(256, 256) >= 200 ? 1 : (tiles(256, 128) >= 200 ? 2 : 3);
        else cfg = tiles(256, 256) >= 200 ? 0 : 3;
        if (a.K % kStepOfConfig[cfg] != 0) cfg = (a.K % 64 == 0) ? 3 : 4;
    }
    switch (cfg) {
        case 0: return launch_dma<256, 256, 64, 2, 4, TRANSB, 4>(a, s);
        case 1: return launch_dma<256, 256, 128, 2, 4, TRANSB, 2>(a, s);
        case 2: return launch_dma<256, 128, 128, 4, 2, TRANSB, 3>(a, s);
        case 3: return launch_dma<128, 128, 64, 2, 2, TRANSB, 4>(a, s);
        case 4: return launch_staged<TRANSB>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool gemm_config_valid(int cfg, int64_t K) {
    if (cfg == -1 || cfg == 4) return true;
    return cfg >= 0 && cfg <= 3 && K % kStepOfConfig[cfg] == 0;
}

// Two K-strided-B products in one launch (the two backward products of the layer).  Falls back to two launches when
// the shapes do not allow the shared configuration.
hipError_t launch_gemm_i8_pair(const GemmArgs& a1, const GemmArgs& a2, hipStream_t s) {
    const bool ok = !a1.transB && !a2.transB && a1.M > 0 && a1.N > 0 && a2.M > 0 && a2.N > 0 && a1.K > 0 && a2.K > 0 &&
                    a1.K % 64 == 0 && a2.K % 64 == 0 && a1.config == a2.config &&
                    (a1.config == -1 || a1.config == 0 || a1.config == 3);
    if (!ok) {
        hipError_t e = launch_gemm_i8(a1, s);
        return e != hipSuccess ? e : launch_gemm_i8(a2, s);
    }
    // 256x256 tiles: the E product alone would leave half the CUs idle at 2048 tokens, the pair fills them
    // (measured on config c2: 183-190 us per step against 197 with 128x128 tiles and 204 with two launches).
    if (a1.config == 3) return launch_dma<128, 128, 64, 2, 2, false, 4>(a1, s, &a2);
    return launch_dma<256, 256, 64, 2, 4, false, 4>(a1, s, &a2);
}

hipError_t launch_gemm_i8(const GemmArgs& a, hipStream_t s) {
    if (a.M == 0 || a.N == 0) return hipSuccess;
    return a.transB ? launch_by_shape<true>(a, s) : launch_by_shape<false>(a, s);
}

hipError_t launch_mfma_i8_probe(const int8_t* operands, int iters, int32_t* sink, hipStream_t s) {
    hipLaunchKernelGGL(mfma_i8_probe_kernel, dim3(256), dim3(512), 0, s, operands, iters, sink);
    return hipGetLastError();
}

}  // namespace halo
