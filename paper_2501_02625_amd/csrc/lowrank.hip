// The high-precision low-rank side branch of a LoRA-style linear module next to the quantised products (Section 3.3
// "Parameter Efficient Fine Tuning"; Appendix "LoRA-style Linear Module and HALO for PEFT"):
//   T = X U^T,  S = E_Y V            (tall input times a thin matrix: lr_down_kernel, bf16 matrix instructions)
//   G_V = E_Y^T T,  G_U = S^T X      (thin result, reduction over the tokens: lr_grad_kernel, summed up in lr_tail_kernel)
// and the rotations H S and (U H)^T of the thin operands that the epilogue of the E_X product wants (lr_tail_kernel).  The
// additions T V^T and S U themselves happen in the epilogue of the INT8 GEMM.  All inputs are bf16, every product accumulates in
// fp32 and the intermediates T and S stay fp32.  Every kernel here is bound by one read of its tall operand from HBM.
#pragma clang fp contract(off)

#include "halo_internal.h"

namespace halo {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

typedef uint32_t v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// (high half of y) << 16 | (high half of x), and the same for the low halves: two bf16 values side by side.
__device__ __forceinline__ uint32_t pack_hi(uint32_t x, uint32_t y) { return __builtin_amdgcn_perm(y, x, 0x07060302u); }
__device__ __forceinline__ uint32_t pack_lo(uint32_t x, uint32_t y) { return __builtin_amdgcn_perm(y, x, 0x05040100u); }

// x = hi + mid + lo exactly, each piece an fp32 value whose low 16 bits are zero (a bf16): truncating the 24-bit mantissa
// to its top 8 bits, subtracting (exact), and again; what is left has at most 8 significant bits.
__device__ __forceinline__ void split3(float x, uint32_t& hi, uint32_t& mid, uint32_t& lo) {
    hi = __float_as_uint(x) & 0xFFFF0000u;
    const float r1 = x - __uint_as_float(hi);
    mid = __float_as_uint(r1) & 0xFFFF0000u;
    lo = __float_as_uint(r1 - __uint_as_float(mid));
}

// ------------------------------------------------------------------------------------------------ down-projection
// out[row, c] = sum_k in[row, k] * B[k, c]:  in bf16 [rows x K] (pitch ld_in), out fp32 [rows x rank] dense.  The thin
// operand is bf16 in either orientation: [rank x K] (K-contiguous rows, pitch ld_b: the adapter U for T = X U^T) or,
// with KMAJOR, [K x rank] (pitch ld_b: the adapter V for S = E V).  K a multiple of 64, rank <= 64 (NTILE rank tiles of 16).
// A workgroup owns 16 rows; its sixteen wavefronts take pairs of 32-element K chunks round robin (a pair is one
// 128-byte line of every row).  v_mfma_f32_16x16x32_bf16: lane l supplies row l % 16, elements 8 (l / 16) .. + 8 of the
// chunk, for both operands; result lane l holds column l % 16, rows 4 (l / 16) .. + 4.  The partial sums meet in LDS and
// are added in wavefront order.
constexpr int kDownWaves = 16;

template <bool KMAJOR>
__device__ __forceinline__ v8bf lr_load_b(const uint16_t* __restrict__ bt, int64_t ld_b, int c, int64_t k) {
    if constexpr (KMAJOR) {
        // eight rows of the [K x rank] matrix, one element each
        uint32_t e[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) e[u] = bt[(k + u) * ld_b + c];
        const v4u packed = {pack_lo(e[0], e[1]), pack_lo(e[2], e[3]), pack_lo(e[4], e[5]), pack_lo(e[6], e[7])};
        return __builtin_bit_cast(v8bf, packed);
    } else {
        return *reinterpret_cast<const v8bf*>(bt + (int64_t)c * ld_b + k);
    }
}

template <int NTILE, bool KMAJOR>
__global__ void __launch_bounds__(64 * kDownWaves)
lr_down_kernel(const uint16_t* __restrict__ in, int64_t ld_in, const uint16_t* __restrict__ bt, int64_t ld_b,
               float* __restrict__ out, int64_t rows, int64_t K, int rank) {
    __shared__ float s_part[kDownWaves][NTILE][4][64];      // [wavefront][rank tile][register][lane]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lr = lane & 15, kg = lane >> 4;
    const int64_t row0 = (int64_t)blockIdx.x * 16;
    int64_t row = row0 + lr;
    if (row > rows - 1) row = rows - 1;                 // clamped rows are computed and never stored
    const uint16_t* ap = in + row * ld_in + kg * 8;
    // columns beyond the rank are replaced by column 0; their results are never stored
    int cb[NTILE];
#pragma unroll
    for (int t = 0; t < NTILE; ++t) cb[t] = (t * 16 + lr) < rank ? (t * 16 + lr) : 0;
    v4f acc[NTILE];
#pragma unroll
    for (int t = 0; t < NTILE; ++t) acc[t] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

    constexpr int64_t STEP = kDownWaves * 64;
    constexpr int UNR = NTILE <= 2 ? 4 : 2;              // chunk pairs per trip, all loads issued before the first product
    int64_t k0 = (int64_t)wave * 64;
    for (; k0 + (UNR - 1) * STEP < K; k0 += UNR * STEP) {
        v8bf a[UNR][2], b[UNR][2][NTILE];
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int64_t k = k0 + u * STEP + h * 32;
                a[u][h] = *reinterpret_cast<const v8bf*>(ap + k);
#pragma unroll
                for (int t = 0; t < NTILE; ++t) b[u][h][t] = lr_load_b<KMAJOR>(bt, ld_b, cb[t], k + kg * 8);
            }
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int t = 0; t < NTILE; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][h], b[u][h][t], acc[t], 0, 0, 0);
    }
    for (; k0 < K; k0 += STEP) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int64_t k = k0 + h * 32;
            const v8bf a = *reinterpret_cast<const v8bf*>(ap + k);
#pragma unroll
            for (int t = 0; t < NTILE; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, lr_load_b<KMAJOR>(bt, ld_b, cb[t], k + kg * 8), acc[t], 0, 0, 0);
        }
    }
#pragma unroll
    for (int t = 0; t < NTILE; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) s_part[wave][t][v][lane] = acc[t][v];
    __syncthreads();
    for (int idx = threadIdx.x; idx < NTILE * 256; idx += 64 * kDownWaves) {
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
// part[split] = sum over the tokens t of the split of big[t, col] * small[t, c]:  big bf16 [rows x wide] (pitch
// ld_big), small fp32 [rows x rank] dense.  A workgroup owns 128 columns of `big` and one range of tokens; its four
// wavefronts take groups of 32 tokens round robin.  v_mfma_f32_16x16x32_bf16 with k = token: lane l supplies, for row
// (A) / column (B) l % 16, the eight tokens 8 (l / 16) .. + 8 of the group.  `big` is read row-wise, 8 consecutive columns
// of one token per load (16 bytes), one load for each of the lane's eight tokens; the v-th column of the eight loads,
// packed with byte permutes, is the A operand of the v-th instruction, which therefore covers columns c0 + 8 i + v.
// `small` is fp32: every value is split exactly into three bf16 pieces (8 + 8 + 8 mantissa bits; x = hi + mid + lo), each
// piece multiplied by the bf16 `big` exactly and accumulated in fp32, so the result is that of an fp32 product sum.
// NTILE = rank tiles of 16.  The partial result is laid out like the final one: [wide x rank], or [rank x wide] with
// `transpose`.  Two independent products ride in one launch (blockIdx.z): G_V = E^T T and G_U = S^T X.
constexpr int kGradWaves = 4;

struct GradJob {
    const uint16_t* big;
    int64_t ld_big;
    const float* small;
    float* part;             // [splits][wide * rank], or the result itself when splits == 1
    int64_t rows, wide;
    int64_t rows_per_split;
    int splits;
    int transpose;
};

template <int NTILE>
__global__ void __launch_bounds__(64 * kGradWaves)
lr_grad_kernel(GradJob j0, GradJob j1, int rank) {
    __shared__ float s_sum[kGradWaves][32][64];          // one rank tile of every wavefront: [v * 4 + e][lane]
    const GradJob& g = blockIdx.z == 0 ? j0 : j1;
    const int64_t wide = g.wide;
    const int64_t c0 = (int64_t)blockIdx.x * 128;
    if (c0 >= wide || (int)blockIdx.y >= g.splits) return;           // uniform over the workgroup
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i16 = lane & 15, kq = lane >> 4;
    const int64_t col = c0 + 8 * i16;
    const bool col_ok = col < wide;                      // wide is a multiple of 8
    const int64_t t_begin = (int64_t)blockIdx.y * g.rows_per_split;
    int64_t t_end = t_begin + g.rows_per_split;
    if (t_end > g.rows) t_end = g.rows;
    const uint16_t* __restrict__ big = g.big;
    const float* __restrict__ small = g.small;
    const int64_t ld_big = g.ld_big;

    v4f acc[NTILE][8];
#pragma unroll
    for (int t = 0; t < NTILE; ++t)
#pragma unroll
        for (int v = 0; v < 8; ++v) acc[t][v] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

    // rows beyond the range and columns beyond the matrix: the address is clamped, the loaded value zeroed
    const int64_t colc = col_ok ? col : 0;
    constexpr int64_t STEP = kGradWaves * 32;
    for (int64_t t0 = t_begin + wave * 32; t0 < t_end; t0 += STEP) {
        uint4 raw[8];
        float sv[NTILE][8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t tr = t0 + 8 * kq + u;
            const bool ok = tr < t_end;
            const int64_t trc = ok ? tr : t_end - 1;
            raw[u] = *reinterpret_cast<const uint4*>(big + trc * ld_big + colc);
            if (!(ok && col_ok)) raw[u] = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int t = 0; t < NTILE; ++t) {
                const int c = t * 16 + i16;
                const float x = small[trc * rank + (c < rank ? c : 0)];
                sv[t][u] = (ok && c < rank) ? x : 0.0f;
            }
        }
        // B operands: the three bf16 pieces of the eight tokens' values, packed two to a register
        v8bf bp[NTILE][3];
#pragma unroll
        for (int t = 0; t < NTILE; ++t) {
            uint32_t piece[3][8];
#pragma unroll
            for (int u = 0; u < 8; ++u) split3(sv[t][u], piece[0][u], piece[1][u], piece[2][u]);
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const v4u packed = {pack_hi(piece[q][0], piece[q][1]), pack_hi(piece[q][2], piece[q][3]),
                                    pack_hi(piece[q][4], piece[q][5]), pack_hi(piece[q][6], piece[q][7])};
                bp[t][q] = __builtin_bit_cast(v8bf, packed);
            }
        }
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            // column v of the eight tokens: the low or the high half of dword v / 2 of every load
            uint32_t w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) w[u] = (v >> 1) == 0 ? raw[u].x : (v >> 1) == 1 ? raw[u].y : (v >> 1) == 2 ? raw[u].z : raw[u].w;
            v4u packed;
            if (v & 1) packed = v4u{pack_hi(w[0], w[1]), pack_hi(w[2], w[3]), pack_hi(w[4], w[5]), pack_hi(w[6], w[7])};
            else packed = v4u{pack_lo(w[0], w[1]), pack_lo(w[2], w[3]), pack_lo(w[4], w[5]), pack_lo(w[6], w[7])};
            const v8bf a = __builtin_bit_cast(v8bf, packed);
#pragma unroll
            for (int t = 0; t < NTILE; ++t)
#pragma unroll
                for (int q = 0; q < 3; ++q) acc[t][v] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bp[t][q], acc[t][v], 0, 0, 0);
        }
    }
    // The wavefronts' sums meet in LDS, one rank tile at a time, and are added in wavefront order; wavefront w then
    // stores the columns v = 2 w, 2 w + 1 of every group of eight.
    float* dst = g.part + (int64_t)blockIdx.y * wide * rank;
#pragma unroll
    for (int t = 0; t < NTILE; ++t) {
        if (t > 0) __syncthreads();
#pragma unroll
        for (int v = 0; v < 8; ++v)
#pragma unroll
            for (int e = 0; e < 4; ++e) s_sum[wave][v * 4 + e][lane] = acc[t][v][e];
        __syncthreads();
        const int c = t * 16 + i16;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float o[2];
#pragma unroll
            for (int d = 0; d < 2; ++d) {
                const int q = (2 * wave + d) * 4 + e;
                float sum = s_sum[0][q][lane];
#pragma unroll
                for (int w = 1; w < kGradWaves; ++w) sum += s_sum[w][q][lane];
                o[d] = sum;
            }
            const int64_t oc = c0 + 8 * (4 * kq + e) + 2 * wave;     // columns oc, oc + 1
            if (oc >= wide || c >= rank) continue;
            if (g.transpose) {
                *reinterpret_cast<float2*>(dst + (int64_t)c * wide + oc) = make_float2(o[0], o[1]);
            } else {
                dst[oc * rank + c] = o[0];
                dst[(oc + 1) * rank + c] = o[1];
            }
        }
    }
}

// out[i] = sum over the splits of part[s][i], in order; four consecutive elements per thread (total a multiple of 4).
// All partial sums are fetched before the first addition (absent ones count as zero).
struct ReduceJob {
    const float* part;
    float* out;
    int64_t total;
    int splits;
};
constexpr int kMaxGradSplits = 16;

constexpr int kTailThreads = 1024;

__device__ __forceinline__ void lr_reduce_body(const ReduceJob& r, int blk) {
    const int64_t idx = ((int64_t)blk * kTailThreads + threadIdx.x) * 4;
    if (idx >= r.total || r.splits <= 1) return;
    float4 p[kMaxGradSplits];
#pragma unroll
    for (int s = 0; s < kMaxGradSplits; ++s) {
        const int sc = s < r.splits ? s : 0;
        p[s] = *reinterpret_cast<const float4*>(r.part + (int64_t)sc * r.total + idx);
    }
    float4 sum = p[0];
#pragma unroll
    for (int s = 1; s < kMaxGradSplits; ++s) {
        if (s < r.splits) { sum.x += p[s].x; sum.y += p[s].y; sum.z += p[s].z; sum.w += p[s].w; }
    }
    *reinterpret_cast<float4*>(r.out + idx) = sum;
}

// ------------------------------------------------------------------------------------------------ small helpers
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

// Rotations of thin matrices, each vector in LDS: a job is a set of vectors of `block` elements (block = 2^n, or
// 28 * 2^n: H_{2^n} (x) H_28 with element i * 28 + j indexed by i in the Walsh-Hadamard factor; block 64 with
// log_p = -1: no rotation, only the conversion), element e of vector (a, b) at  a * stride_a + b * stride_b + e * stride_e
// in the source and at the same expression with the dst_ strides in the destination.  bf16 or fp32 in, fp32 out, normalised.  One workgroup per vector; the first
// job's vectors come first in the grid.  The order of the additions is not that of the row kernels; nothing here needs to
// be reproducible to the bit against a reference.  Used for U H (rows of the adapter U) and H S (columns of S = E V).
constexpr int kSmallFwhtMax = 16384;
constexpr int kSmallFwhtThreads = kTailThreads;

struct FwhtJob {
    const void* src;
    float* dst;
    int src_bf16;
    int64_t stride_a, stride_b, stride_e;
    int64_t dst_a, dst_b, dst_e;     // the same three strides in the destination
    int count_b;             // vectors per a
    int vectors;             // count_a * count_b
    int block, unit, log_p;  // unit 1 or 28; log_p = log2(block / unit), or -1
    float c_norm;
};

// The small work at the end of the thin backward products, one launch: the first nb0 + nb1 workgroups add up the token
// ranges of the two adapter gradients (lr_reduce_body), the others each rotate one vector.
__global__ void __launch_bounds__(kTailThreads)
lr_tail_kernel(ReduceJob r0, ReduceJob r1, int nb0, int nb1, FwhtJob j0, FwhtJob j1) {
    __shared__ float s_x[kSmallFwhtMax];
    int blk = blockIdx.x;
    if (blk < nb0 + nb1) {                 // uniform over the workgroup
        if (blk < nb0) lr_reduce_body(r0, blk);
        else lr_reduce_body(r1, blk - nb0);
        return;
    }
    blk -= nb0 + nb1;
    const bool first = blk < j0.vectors;
    const FwhtJob& g = first ? j0 : j1;
    const int vec = first ? blk : blk - j0.vectors;
    const int64_t va = vec / g.count_b, vb = vec % g.count_b;
    const int64_t base = va * g.stride_a + vb * g.stride_b;
    const int block = g.block, unit = g.unit;
    if (g.src_bf16) {
        const uint16_t* src = reinterpret_cast<const uint16_t*>(g.src) + base;
        for (int i = threadIdx.x; i < block; i += kSmallFwhtThreads) s_x[i] = bf16_to_f32(src[i * g.stride_e]);
    } else {
        const float* src = reinterpret_cast<const float*>(g.src) + base;
        for (int i = threadIdx.x; i < block; i += kSmallFwhtThreads) s_x[i] = src[i * g.stride_e];
    }
    __syncthreads();
    const int p = g.log_p >= 0 ? 1 << g.log_p : 0;       // length of the Walsh-Hadamard factor
    if (unit == 28) {
        for (int run = threadIdx.x; run < p; run += kSmallFwhtThreads) {
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
    for (int lh = 0; lh < g.log_p; ++lh) {
        const int h = 1 << lh;
        if (unit == 1) {
            for (int ii = threadIdx.x; ii < (p >> 1); ii += kSmallFwhtThreads) {
                const int i = ((ii >> lh) << (lh + 1)) | (ii & (h - 1));
                const float a = s_x[i], b = s_x[i + h];
                s_x[i] = a + b;
                s_x[i + h] = a - b;
            }
        } else {
            // pairs (ii, j): 28 consecutive threads share one ii
            for (int q = threadIdx.x; q < (p >> 1) * 28; q += kSmallFwhtThreads) {
                const int ii = q / 28, j = q - ii * 28;
                const int i = ((ii >> lh) << (lh + 1)) | (ii & (h - 1));
                const float a = s_x[i * 28 + j], b = s_x[(i + h) * 28 + j];
                s_x[i * 28 + j] = a + b;
                s_x[(i + h) * 28 + j] = a - b;
            }
        }
        __syncthreads();
    }
    float* dst = g.dst + va * g.dst_a + vb * g.dst_b;
    for (int i = threadIdx.x; i < block; i += kSmallFwhtThreads) dst[i * g.dst_e] = s_x[i] * g.c_norm;
}

template <bool KMAJOR>
hipError_t launch_down_by_rank(const uint16_t* in, int64_t ld_in, const uint16_t* bt, int64_t ld_b, float* out, int64_t rows,
                               int64_t K, int rank, unsigned blocks, hipStream_t s) {
    const dim3 grid(blocks), block(64 * kDownWaves);
    if (rank <= 16)
        hipLaunchKernelGGL((lr_down_kernel<1, KMAJOR>), grid, block, 0, s, in, ld_in, bt, ld_b, out, rows, K, rank);
    else if (rank <= 32)
        hipLaunchKernelGGL((lr_down_kernel<2, KMAJOR>), grid, block, 0, s, in, ld_in, bt, ld_b, out, rows, K, rank);
    else
        hipLaunchKernelGGL((lr_down_kernel<4, KMAJOR>), grid, block, 0, s, in, ld_in, bt, ld_b, out, rows, K, rank);
    return hipGetLastError();
}

// Token ranges of the gradient kernel: enough workgroups to fill the chip, at least 64 tokens each, at most 16.
int lr_grad_splits(int64_t rows, int64_t wide) {
    const int64_t col_tiles = (wide + 127) / 128;
    int64_t splits = (512 + col_tiles - 1) / col_tiles;
    if (splits > kMaxGradSplits) splits = kMaxGradSplits;
    const int64_t max_splits = (rows + 63) / 64;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    return (int)splits;
}

bool fill_fwht_job(FwhtJob* j, const void* src, int src_bf16, float* dst, int64_t stride_a, int64_t stride_b, int64_t stride_e,
                   int64_t count_a, int64_t count_b, int64_t block) {
    j->src = src; j->dst = dst; j->src_bf16 = src_bf16;
    j->stride_a = stride_a; j->stride_b = stride_b; j->stride_e = stride_e;
    j->dst_a = stride_a; j->dst_b = stride_b; j->dst_e = stride_e;
    if (count_a * count_b > (int64_t(1) << 24) || block > kSmallFwhtMax || block < 1) return false;
    j->count_b = (int)count_b;
    j->vectors = (int)(count_a * count_b);
    j->block = (int)block;
    const bool pow2 = (block & (block - 1)) == 0;
    if (!pow2 && block % 28 != 0) return false;
    j->unit = pow2 ? 1 : 28;
    const int64_t p = block / j->unit;
    if ((p & (p - 1)) != 0) return false;
    j->log_p = 0;
    while ((int64_t(1) << j->log_p) < p) ++j->log_p;
    j->c_norm = (float)(1.0 / sqrt((double)block));
    return true;
}

}  // namespace

// ------------------------------------------------------------------------------------------------ launchers
hipError_t launch_lr_down(const void* in, int64_t ld_in, const void* thin, int k_major, int64_t ld_b, float* out, int64_t rows,
                          int64_t K, int rank, hipStream_t s) {
    if (rows <= 0 || rank <= 0) return hipSuccess;
    if (rank > kMaxLowRank || K % 64 != 0 || K <= 0 || ld_in < K || ld_in % 8 != 0) return hipErrorInvalidValue;
    if (k_major ? ld_b < rank : (ld_b < K || ld_b % 8 != 0)) return hipErrorInvalidValue;
    const int64_t blocks = (rows + 15) / 16;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    const uint16_t* a = reinterpret_cast<const uint16_t*>(in);
    const uint16_t* b = reinterpret_cast<const uint16_t*>(thin);
    return k_major ? launch_down_by_rank<true>(a, ld_in, b, ld_b, out, rows, K, rank, (unsigned)blocks, s)
                   : launch_down_by_rank<false>(a, ld_in, b, ld_b, out, rows, K, rank, (unsigned)blocks, s);
}

size_t lr_grad_workspace_floats(int64_t rows, int64_t wide, int rank) {
    return (size_t)lr_grad_splits(rows, wide) * (size_t)wide * (size_t)rank;
}

bool lr_row_fwht_shape_ok(int64_t cols, int64_t block) {
    if (block <= 1) return cols % 64 == 0;
    if (block > kSmallFwhtMax || cols % block != 0) return false;
    if ((block & (block - 1)) == 0) return true;
    if (block % 28 != 0) return false;
    const int64_t p = block / 28;
    return (p & (p - 1)) == 0;
}

bool lr_col_fwht_shape_ok(int64_t rows, int64_t block) {
    return block >= 2 && block <= kSmallFwhtMax && (block & (block - 1)) == 0 && rows % block == 0;
}

hipError_t launch_lr_backward_small(const LrGradArgs* a, const LrGradArgs* b, int64_t rows, int rank, const LrRotArgs* rot,
                                    hipStream_t s) {
    if (rank <= 0 || rank > kMaxLowRank || rank % 4 != 0 || rows <= 0) return hipErrorInvalidValue;
    if (!a) { a = b; b = nullptr; }
    // ---- the gradient products, one launch
    GradJob gj[2] = {};
    ReduceJob rj[2] = {};
    int nb[2] = {0, 0};
    if (a) {
        unsigned gx = 0, gy = 0;
        const LrGradArgs* src[2] = {a, b};
        const int njobs = b ? 2 : 1;
        for (int i = 0; i < njobs; ++i) {
            const LrGradArgs& q = *src[i];
            if (q.wide <= 0 || q.wide % 8 != 0 || q.ld_big < q.wide || q.ld_big % 8 != 0 || !q.big || !q.small || !q.out ||
                !q.part)
                return hipErrorInvalidValue;
            const int splits = lr_grad_splits(rows, q.wide);
            int64_t per = (rows + splits - 1) / splits;
            per = (per + 15) / 16 * 16;
            gj[i] = GradJob{reinterpret_cast<const uint16_t*>(q.big), q.ld_big, q.small, splits == 1 ? q.out : q.part, rows,
                            q.wide, per, splits, q.transpose_out};
            if (splits > 1) {              // a single range writes the result itself
                rj[i] = ReduceJob{q.part, q.out, q.wide * rank, splits};
                nb[i] = (int)((q.wide * rank / 4 + kTailThreads - 1) / kTailThreads);
            }
            const unsigned tiles = (unsigned)((q.wide + 127) / 128);
            if (tiles > gx) gx = tiles;
            if ((unsigned)splits > gy) gy = (unsigned)splits;
        }
        const dim3 grid(gx, gy, (unsigned)njobs), block(64 * kGradWaves);
        if (rank <= 16) hipLaunchKernelGGL(lr_grad_kernel<1>, grid, block, 0, s, gj[0], gj[1], rank);
        else if (rank <= 32) hipLaunchKernelGGL(lr_grad_kernel<2>, grid, block, 0, s, gj[0], gj[1], rank);
        else hipLaunchKernelGGL(lr_grad_kernel<4>, grid, block, 0, s, gj[0], gj[1], rank);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // ---- the sums over the token ranges and the rotations of the thin operands, one launch
    FwhtJob fj[2] = {};
    if (rot) {
        int n = 0;
        if (rot->u) {
            if (!lr_row_fwht_shape_ok(rot->m, rot->block_m)) return hipErrorInvalidValue;
            // rows of U [rank x m]: vector (row, block of the row); no rotation: blocks of 64, conversion only
            const int64_t blk = rot->block_m <= 1 ? 64 : rot->block_m;
            if (!fill_fwht_job(&fj[n], rot->u, 1, rot->u_rot, rot->m, blk, 1, rank, rot->m / blk, blk)) return hipErrorInvalidValue;
            if (rot->block_m <= 1) { fj[n].log_p = -1; fj[n].c_norm = 1.0f; }
            fj[n].dst_a = 1; fj[n].dst_b = blk * rank; fj[n].dst_e = rank;       // transposed: element (col, r) at col * rank + r
            ++n;
        }
        if (rot->sm) {
            if (!lr_col_fwht_shape_ok(rot->b, rot->block_b)) return hipErrorInvalidValue;
            // columns of S [b x rank]: vector (left block, column)
            if (!fill_fwht_job(&fj[n], rot->sm, 0, rot->sm_rot, rot->block_b * rank, 1, rank, rot->b / rot->block_b, rank,
                               rot->block_b))
                return hipErrorInvalidValue;
            ++n;
        }
    }
    const int64_t blocks = (int64_t)nb[0] + nb[1] + fj[0].vectors + fj[1].vectors;
    if (blocks == 0) return hipSuccess;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(lr_tail_kernel, dim3((unsigned)blocks), dim3(kTailThreads), 0, s, rj[0], rj[1], nb[0], nb[1], fj[0], fj[1]);
    return hipGetLastError();
}

}  // namespace halo
