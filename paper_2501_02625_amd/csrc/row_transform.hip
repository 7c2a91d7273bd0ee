// Row transform kernels: right-hand Walsh-Hadamard rotation along the contiguous axis fused with the
// symmetric absmax INT8 quantiser (or with a plain bf16/fp32 store for the un-rotation of GEMM outputs).
//
// One wavefront owns one SEGMENT of 2^LOGSEG consecutive elements of a row and keeps it in registers:
// element index inside the segment = [chunk | lane (6 bits) | e], with the low LOGE bits (e) in
// consecutive registers (one 16-byte load per chunk), the next six bits across the 64 lanes, and the
// remaining high bits across chunks.  The butterflies therefore run
//      strides 1 .. EPL/2      in registers,
//      the next six strides    across lanes (DPP / ds_swizzle / ds_bpermute),
//      the highest strides     in registers again,
// i.e. in ascending stride order, every add/sub a separately rounded fp32 operation.
//
// Cross-lane stages use r = fma(partner, s, own) with s = +1 in the lane holding the lower element and
// s = -1 in the other one.  The lower lane gets a+b exactly; the upper lane gets b-a = -(a-b), the exact
// negation of the wanted difference (fp32 add/sub/fma with an exact product are sign-symmetric under
// round-to-nearest-even).  Two elements that meet in a later butterfly always differ in one index bit
// only, so they carry the same accumulated sign and every later stage is again exact up to that common
// sign.  The sign of a lane, parity of (lane & mask-of-cross-lane-stages-run), is folded into the
// 1/sqrt(d) factor at the end, which costs nothing.
#pragma clang fp contract(off)

#include <mutex>

#include "halo_internal.h"

namespace halo {
namespace {

constexpr float kRoundMagic = 12582912.0f;  // 1.5 * 2^23: adding it rounds |x| < 2^22 to an integer, ties to even

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

__device__ __forceinline__ float wave_max(float x, int bperm_addr) {
    x = fmaxf(x, lane_xor<0>(x, bperm_addr));
    x = fmaxf(x, lane_xor<1>(x, bperm_addr));
    x = fmaxf(x, lane_xor<2>(x, bperm_addr));
    x = fmaxf(x, lane_xor<3>(x, bperm_addr));
    x = fmaxf(x, lane_xor<4>(x, bperm_addr));
    x = fmaxf(x, lane_xor<5>(x, bperm_addr));
    return x;
}

template <int VPL, int RB>
__device__ __forceinline__ void stage_in_regs(float (&v)[VPL]) {
    constexpr int H = 1 << RB;
#pragma unroll
    for (int r = 0; r < VPL; ++r) {
        if ((r & H) == 0) {
            const float a = v[r], b = v[r | H];
            v[r] = a + b;
            v[r | H] = a - b;
        }
    }
}

// Eight  x <- x + s * partner(x)  steps in one asm block: v_fmac_f32 with the partner read through DPP.  The
// leading s_nop supplies the two wait states a DPP read needs after a VALU write of the same register, whatever
// the compiler placed before the block; inside the block every register is read and written by one instruction.
#define HALO_FMAC_DPP8(CTRL)                                                                                   \
    asm volatile("s_nop 1\n\t"                                                                                 \
                 "v_fmac_f32_dpp %0, %0, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
                 "v_fmac_f32_dpp %1, %1, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
                 "v_fmac_f32_dpp %2, %2, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
                 "v_fmac_f32_dpp %3, %3, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
                 "v_fmac_f32_dpp %4, %4, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
                 "v_fmac_f32_dpp %5, %5, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
                 "v_fmac_f32_dpp %6, %6, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
                 "v_fmac_f32_dpp %7, %7, %8 " CTRL " row_mask:0xf bank_mask:0xf"                                 \
                 : "+v"(v[r]), "+v"(v[r + 1]), "+v"(v[r + 2]), "+v"(v[r + 3]), "+v"(v[r + 4]), "+v"(v[r + 5]),   \
                   "+v"(v[r + 6]), "+v"(v[r + 7])                                                               \
                 : "v"(s))

template <int VPL, int J>
__device__ __forceinline__ void stage_across_lanes(float (&v)[VPL], int lane, int bperm_addr) {
    static_assert(VPL % 8 == 0, "values per lane come in chunks of eight");
    const float s = ((lane >> J) & 1) ? -1.0f : 1.0f;
    if constexpr (J == 0) {
#pragma unroll
        for (int r = 0; r < VPL; r += 8) HALO_FMAC_DPP8("quad_perm:[1,0,3,2]");
    } else if constexpr (J == 1) {
#pragma unroll
        for (int r = 0; r < VPL; r += 8) HALO_FMAC_DPP8("quad_perm:[2,3,0,1]");
    } else if constexpr (J == 3) {
#pragma unroll
        for (int r = 0; r < VPL; r += 8) HALO_FMAC_DPP8("row_ror:8");
    } else {
#pragma unroll
        for (int r = 0; r < VPL; ++r) {
            const float p = lane_xor<J>(v[r], bperm_addr);
            v[r] = __builtin_fmaf(p, s, v[r]);
        }
    }
}

// Run stage number BIT (stride 2^BIT) of the segment-local FWHT if it is below log_block.
template <int VPL, int LOGE, int BIT>
__device__ __forceinline__ void fwht_stage(float (&v)[VPL], int log_block, int lane, int bperm_addr) {
    if (BIT < log_block) {
        if constexpr (BIT < LOGE) {
            stage_in_regs<VPL, BIT>(v);
        } else if constexpr (BIT < LOGE + 6) {
            stage_across_lanes<VPL, BIT - LOGE>(v, lane, bperm_addr);
        } else {
            stage_in_regs<VPL, BIT - 6>(v);
        }
    }
}

template <int VPL, int LOGE, int BIT, int LOGSEG>
struct FwhtStages {
    static __device__ __forceinline__ void run(float (&v)[VPL], int log_block, int lane, int bperm_addr) {
        fwht_stage<VPL, LOGE, BIT>(v, log_block, lane, bperm_addr);
        FwhtStages<VPL, LOGE, BIT + 1, LOGSEG>::run(v, log_block, lane, bperm_addr);
    }
};
template <int VPL, int LOGE, int LOGSEG>
struct FwhtStages<VPL, LOGE, LOGSEG, LOGSEG> {
    static __device__ __forceinline__ void run(float (&)[VPL], int, int, int) {}
};

// Per-wave geometry shared by the phases of the kernel.
struct RowCtx {
    int lane, bperm_addr;
    int wave, seg;          // wavefront in the workgroup; segment of the row it owns
    float* xbuf;            // LDS exchange buffer [waves][values per lane][64] (only with cross-wave stages)
    int64_t row, kbase;     // kbase: first element of this lane's chunk 0
    bool row_ok;
};

// Load one segment into registers, rotate it, apply the fold vector; returns the local absmax (quantising kernels).
// FAST: the row exists and the whole segment lies inside it, so nothing is bounds-checked.
template <int LOGSEG, int IN, int OUT, bool FAST, int LB, int XS>
__device__ __forceinline__ float row_phase1(const RowArgs& a, const RowCtx& x, float c_norm,
                                            float (&v)[1 << (LOGSEG - 6)]) {
    constexpr int LOGE = (IN == IN_BF16) ? 3 : 2;
    constexpr int EPL = 1 << LOGE;
    constexpr int VPL = 1 << (LOGSEG - 6);
    constexpr int NCH = VPL / EPL;

    float pre = 1.0f;
    if constexpr (IN == IN_I32) {
        if (x.row_ok && a.pre_scale) pre = a.pre_scale[x.row];
    }
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int64_t k0 = x.kbase + (int64_t)c * 64 * EPL;
        if (FAST || (x.row_ok && k0 + EPL <= a.cols)) {
            if constexpr (IN == IN_BF16) {
                const uint4 q = *reinterpret_cast<const uint4*>(
                    reinterpret_cast<const uint16_t*>(a.in) + x.row * a.ld_in + k0);
                const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    v[c * EPL + 2 * i] = __uint_as_float(w[i] << 16);
                    v[c * EPL + 2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
                }
            } else if constexpr (IN == IN_F32) {
                const float4 q = *reinterpret_cast<const float4*>(
                    reinterpret_cast<const float*>(a.in) + x.row * a.ld_in + k0);
                v[c * EPL + 0] = q.x; v[c * EPL + 1] = q.y; v[c * EPL + 2] = q.z; v[c * EPL + 3] = q.w;
            } else {
                const int4 q = *reinterpret_cast<const int4*>(
                    reinterpret_cast<const int32_t*>(a.in) + x.row * a.ld_in + k0);
                v[c * EPL + 0] = (float)q.x * pre; v[c * EPL + 1] = (float)q.y * pre;
                v[c * EPL + 2] = (float)q.z * pre; v[c * EPL + 3] = (float)q.w * pre;
            }
        } else {
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                float t = 0.0f;
                if (x.row_ok && k0 + e < a.cols) {
                    if constexpr (IN == IN_BF16) {
                        t = __uint_as_float((uint32_t)(reinterpret_cast<const uint16_t*>(a.in)[x.row * a.ld_in + k0 + e]) << 16);
                    } else if constexpr (IN == IN_F32) {
                        t = reinterpret_cast<const float*>(a.in)[x.row * a.ld_in + k0 + e];
                    } else {
                        t = (float)reinterpret_cast<const int32_t*>(a.in)[x.row * a.ld_in + k0 + e] * pre;
                    }
                }
                v[c * EPL + e] = t;
            }
        }
    }

    if constexpr (IN == IN_F32) {
        if (a.in_mul != 0.0f) {      // e.g. the 1/sqrt(block) of a left-hand rotation whose butterflies ran before
#pragma unroll
            for (int r = 0; r < VPL; ++r) v[r] *= a.in_mul;
        }
    }
    if constexpr (IN == IN_I32) {
        if (a.post_scale) {          // one more (tensor-wide) scale, applied after the per-row one
            const float post = *a.post_scale;
#pragma unroll
            for (int r = 0; r < VPL; ++r) v[r] *= post;
        }
    }

    // ---- rotate (LB >= 0: block size known at compile time, so the stage sequence is straight-line code)
    const int log_block = LB >= 0 ? LB : a.log_block;
    if (log_block > 0) {
        FwhtStages<VPL, LOGE, 0, LOGSEG>::run(v, log_block, x.lane, x.bperm_addr);
        if constexpr (XS > 0) {
            // Strides 2^LOGSEG .. 2^(LOGSEG+XS-1) pair up whole segments, i.e. wavefronts of this workgroup: each
            // wavefront publishes its registers in LDS and combines them with its partner's, the lower segment
            // taking a+b and the upper one a-b (the lane signs carried so far are the same in both).
#pragma unroll
            for (int xs = 0; xs < XS; ++xs) {
                if (xs > 0) __syncthreads();        // everyone has read the previous round
#pragma unroll
                for (int r = 0; r < VPL; ++r) x.xbuf[(x.wave * VPL + r) * 64 + x.lane] = v[r];
                __syncthreads();
                const bool upper = (x.seg >> xs) & 1;
                const int pw = x.wave ^ (1 << xs);
#pragma unroll
                for (int r = 0; r < VPL; ++r) {
                    const float p = x.xbuf[(pw * VPL + r) * 64 + x.lane];
                    v[r] = upper ? p - v[r] : v[r] + p;
                }
            }
        }
        // lanes whose (lane & mask) has odd parity hold negated values: the sign rides on the 1/sqrt(d) multiply
        int nlane_stages = log_block - LOGE;
        nlane_stages = nlane_stages < 0 ? 0 : (nlane_stages > 6 ? 6 : nlane_stages);
        const int mask = (1 << nlane_stages) - 1;
        const float sign_l = (__builtin_popcount(x.lane & mask) & 1) ? -1.0f : 1.0f;
        const float c_l = sign_l * c_norm;
#pragma unroll
        for (int r = 0; r < VPL; ++r) v[r] *= c_l;
    }

    // ---- fold
    if (a.fold) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int64_t k0 = x.kbase + (int64_t)c * 64 * EPL;
            if (FAST || k0 + EPL <= a.cols) {
#pragma unroll
                for (int i = 0; i < EPL / 4; ++i) {
                    const float4 f = *reinterpret_cast<const float4*>(a.fold + k0 + 4 * i);
                    v[c * EPL + 4 * i + 0] *= f.x; v[c * EPL + 4 * i + 1] *= f.y;
                    v[c * EPL + 4 * i + 2] *= f.z; v[c * EPL + 4 * i + 3] *= f.w;
                }
            } else {
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    if (k0 + e < a.cols) v[c * EPL + e] *= a.fold[k0 + e];
            }
        }
    }

    float amax = 0.0f;
    if constexpr (OUT == OUT_Q8) {
        // one v_max3_f32 with |.| source modifiers per pair of values (written out: the compiler's fmaxf chain takes
        // four instructions per pair), in two chains
        float amax2 = 0.0f;
#pragma unroll
        for (int r = 0; r < VPL; r += 4) {
            asm("v_max3_f32 %0, %0, |%1|, |%2|" : "+v"(amax) : "v"(v[r]), "v"(v[r + 1]));
            asm("v_max3_f32 %0, %0, |%1|, |%2|" : "+v"(amax2) : "v"(v[r + 2]), "v"(v[r + 3]));
        }
        amax = __builtin_fmaxf(amax, amax2);
        amax = wave_max(amax, x.bperm_addr);
    }
    return amax;
}

// Quantise (inv_l = per-lane signed 127/absmax) or convert, and store the segment.
template <int LOGSEG, int IN, int OUT, bool FAST>
__device__ __forceinline__ void row_phase2(const RowArgs& a, const RowCtx& x, const float (&v)[1 << (LOGSEG - 6)],
                                           float inv_l) {
    constexpr int LOGE = (IN == IN_BF16) ? 3 : 2;
    constexpr int EPL = 1 << LOGE;
    constexpr int VPL = 1 << (LOGSEG - 6);
    constexpr int NCH = VPL / EPL;
    if constexpr (OUT == OUT_Q8) {
        int8_t* orow = reinterpret_cast<int8_t*>(a.out) + x.row * a.ld_out;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int64_t k0 = x.kbase + (int64_t)c * 64 * EPL;
            uint32_t packed[EPL / 4];
#pragma unroll
            for (int i = 0; i < EPL / 4; ++i) {
                uint32_t b[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float t = v[c * EPL + 4 * i + e] * inv_l;
                    b[e] = __float_as_uint(t + kRoundMagic);
                }
                const uint32_t lo = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u);
                const uint32_t hi = __builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u);
                packed[i] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
            }
            if (FAST || (x.row_ok && k0 + EPL <= a.cols)) {
                if constexpr (EPL == 8) {
                    *reinterpret_cast<uint2*>(orow + k0) = make_uint2(packed[0], packed[1]);
                } else {
                    *reinterpret_cast<uint32_t*>(orow + k0) = packed[0];
                }
            } else if (x.row_ok) {
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    if (k0 + e < a.cols) orow[k0 + e] = (int8_t)((packed[e / 4] >> (8 * (e & 3))) & 0xFF);
            }
        }
    } else if constexpr (OUT == OUT_MX6) {
        // Microscaling FP6: the four lanes of a quad hold one block of 32 consecutive elements.  Shared scale
        // 2^(floor(log2(block absmax)) - 4) (E8M0), elements rounded to E3M2 (ties to even mantissa, saturating at 28),
        // eight 6-bit codes per lane packed least-significant first; the quad's 24 bytes leave as 8 + 4 + 8 + 4.
        static_assert(EPL == 8, "MXFP6 output takes bf16 input");
        unsigned char* orow = reinterpret_cast<unsigned char*>(a.out) + x.row * a.ld_out;
        const int j = x.lane & 3;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int64_t k0 = x.kbase + (int64_t)c * 64 * EPL;
            float bm = 0.0f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) bm = __builtin_fmaxf(bm, fabsf(v[c * EPL + e]));
            bm = __builtin_fmaxf(bm, lane_xor<0>(bm, x.bperm_addr));
            bm = __builtin_fmaxf(bm, lane_xor<1>(bm, x.bperm_addr));
            int shared = (int)(__float_as_uint(bm) >> 23) - 127 - 4;
            shared = shared < -127 ? -127 : shared;               // the upper clamp cannot bind: exponent <= 127 - 4
            if (!(bm > 0.0f)) shared = 0;
            uint32_t code[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const float xs = __builtin_ldexpf(v[c * EPL + e], -shared);
                const float ax = fabsf(xs);
                uint32_t bits = __float_as_uint(ax);
                bits += 0x000FFFFFu + ((bits >> 21) & 1u);          // round to two mantissa bits, ties to even
                uint32_t q = (bits >> 21) - (124u << 2);            // [exponent + 3 | mantissa]
                q = q > 31u ? 31u : q;
                const uint32_t sub = (uint32_t)__builtin_rintf(ax * 16.0f);     // below the smallest normal: steps of 2^-4
                q = ax < 0.25f ? sub : q;
                code[e] = q | ((q != 0u && xs < 0.0f) ? 32u : 0u);
            }
            const uint32_t w0 = code[0] | (code[1] << 6) | (code[2] << 12) | (code[3] << 18) | (code[4] << 24) | (code[5] << 30);
            const uint32_t w1 = (code[5] >> 2) | (code[6] << 4) | (code[7] << 10);
            const uint32_t nb_w0 = (uint32_t)__builtin_amdgcn_mov_dpp((int)w0, 0xF9, 0xF, 0xF, true);   // quad_perm [1,2,3,3]
            if (FAST || (x.row_ok && k0 + EPL <= a.cols)) {
                unsigned char* blk = orow + (k0 >> 5) * 24;          // k0 >> 5 is the same for the four lanes of the quad
                if ((j & 1) == 0) {
                    uint32_t* dst = reinterpret_cast<uint32_t*>(blk + 12 * (j >> 1));
                    dst[0] = w0;
                    dst[1] = w1 | (nb_w0 << 16);
                } else {
                    *reinterpret_cast<uint32_t*>(blk + 8 + 12 * (j >> 1)) = (w0 >> 16) | (w1 << 16);
                }
                if (j == 0) a.mx_scales[x.row * a.ld_mx_scales + (k0 >> 5)] = (uint8_t)(shared + 127);
            }
        }
    } else if constexpr (OUT == OUT_BF16) {
        uint16_t* orow = reinterpret_cast<uint16_t*>(a.out) + x.row * a.ld_out;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int64_t k0 = x.kbase + (int64_t)c * 64 * EPL;
            uint32_t packed[EPL / 2];
#pragma unroll
            for (int i = 0; i < EPL / 2; ++i)
                packed[i] = pack_bf16x2(v[c * EPL + 2 * i], v[c * EPL + 2 * i + 1]);
            if (FAST || (x.row_ok && k0 + EPL <= a.cols)) {
                if constexpr (EPL == 8) {
                    *reinterpret_cast<uint4*>(orow + k0) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
                } else {
                    *reinterpret_cast<uint2*>(orow + k0) = make_uint2(packed[0], packed[1]);
                }
            } else if (x.row_ok) {
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    if (k0 + e < a.cols) orow[k0 + e] = (uint16_t)(packed[e / 2] >> (16 * (e & 1)));
            }
        }
    } else {
        float* orow = reinterpret_cast<float*>(a.out) + x.row * a.ld_out;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int64_t k0 = x.kbase + (int64_t)c * 64 * EPL;
            if (FAST || (x.row_ok && k0 + EPL <= a.cols)) {
#pragma unroll
                for (int i = 0; i < EPL / 4; ++i)
                    *reinterpret_cast<float4*>(orow + k0 + 4 * i) =
                        make_float4(v[c * EPL + 4 * i], v[c * EPL + 4 * i + 1], v[c * EPL + 4 * i + 2], v[c * EPL + 4 * i + 3]);
            } else if (x.row_ok) {
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    if (k0 + e < a.cols) orow[k0 + e] = v[c * EPL + e];
            }
        }
    }
}

// LB: log2 of the Hadamard block when it is 0 (no rotation) or LOGSEG (block = segment); -1 = read it at run time.
// XS: number of butterfly stages that span wavefronts (Hadamard block = 2^(LOGSEG+XS) elements = 2^XS segments).
template <int LOGSEG, int IN, int OUT, int LB, int XS = 0>
__global__ void __launch_bounds__(LOGSEG >= 11 ? 512 : 1024)
row_transform_kernel(RowArgs a, int segs, int rows_per_wg, float c_norm, unsigned blocks1) {
    constexpr int LOGE = (IN == IN_BF16) ? 3 : 2;
    constexpr int EPL = 1 << LOGE;            // consecutive elements per lane per chunk
    constexpr int VPL = 1 << (LOGSEG - 6);    // values per lane
    constexpr int SEG = 1 << LOGSEG;

    __shared__ float s_amax[16];
    extern __shared__ float s_xbuf[];

    const int wave = threadIdx.x >> 6;
    const int seg = wave % segs;
    const int row_local = wave / segs;
    RowCtx x;
    x.wave = wave;
    x.seg = seg;
    x.xbuf = s_xbuf;
    x.lane = threadIdx.x & 63;
    x.bperm_addr = (x.lane ^ 32) << 2;
    unsigned block = blockIdx.x;
    if (block >= blocks1) {          // the second matrix of a batched launch
        block -= blocks1;
        a.in = a.in2; a.pre_scale = a.pre_scale2; a.out = a.out2; a.out_scale = a.out_scale2; a.rows = a.rows2;
        if (a.given_amax2) a.given_amax = a.given_amax2;
        if (a.post_scale2) a.post_scale = a.post_scale2;
    }
    x.row = (int64_t)block * rows_per_wg + row_local;
    x.row_ok = x.row < a.rows;
    x.kbase = (int64_t)seg * SEG + (int64_t)x.lane * EPL;
    const bool fast = x.row_ok && ((int64_t)(seg + 1) * SEG <= a.cols);   // uniform over the wavefront

    float v[VPL];
    float amax = fast ? row_phase1<LOGSEG, IN, OUT, true, LB, XS>(a, x, c_norm, v)
                      : row_phase1<LOGSEG, IN, OUT, false, LB, XS>(a, x, c_norm, v);

    float inv_l = 0.0f;
    if constexpr (OUT == OUT_Q8) {
        if (segs > 1) {
            if (x.lane == 0) s_amax[wave] = amax;
            __syncthreads();
            const int w0 = row_local * segs;
            float t = s_amax[w0];
            for (int i = 1; i < segs; ++i) t = fmaxf(t, s_amax[w0 + i]);
            amax = t;
        }
        if (a.amax_only) {
            // first phase of the one-scale-per-tensor quantiser: the row's absmax, nothing else
            if (x.row_ok && seg == 0 && x.lane == 0) a.out_scale[x.row] = amax;
            return;
        }
        if (a.given_amax) amax = *a.given_amax;          // second phase: the tensor's absmax for every row
        const bool nz = amax > 0.0f;
        inv_l = nz ? 127.0f / amax : 0.0f;
        if (x.row_ok && seg == 0 && x.lane == 0) a.out_scale[x.row] = nz ? amax / 127.0f : 1.0f;
    }
    if (fast) row_phase2<LOGSEG, IN, OUT, true>(a, x, v, inv_l);
    else row_phase2<LOGSEG, IN, OUT, false>(a, x, v, inv_l);
}

// Hadamard block of 2^(10+XS) elements handled by 2^XS wavefronts of 1024 elements each: four times the
// wavefronts of the one-wavefront-per-block layout and a quarter of the registers, at the price of XS round trips
// through LDS.  It pays when there are too few rows to fill the machine otherwise.
template <int IN, int OUT, int XS>
hipError_t launch_split(const RowArgs& a, hipStream_t s) {
    constexpr int LOGSEG = 10;
    const int segs = (int)(a.cols >> LOGSEG);
    const int rows_per_wg = segs >= 4 ? 1 : 4 / segs;
    const int threads = 64 * segs * rows_per_wg;
    const int64_t blocks1 = (a.rows + rows_per_wg - 1) / rows_per_wg;
    const int64_t blocks = blocks1 + (a.rows2 + rows_per_wg - 1) / rows_per_wg;
    const float c_norm = (float)(1.0 / sqrt((double)(int64_t(1) << a.log_block)));
    const size_t lds = (size_t)(threads / 64) * (1 << (LOGSEG - 6)) * 64 * sizeof(float);
    hipLaunchKernelGGL((row_transform_kernel<LOGSEG, IN, OUT, LOGSEG + XS, XS>), dim3((unsigned)blocks), dim3(threads), lds,
                       s, a, segs, rows_per_wg, c_norm, (unsigned)blocks1);
    return hipGetLastError();
}

template <int LOGSEG, int IN, int OUT>
hipError_t launch_one(const RowArgs& a, int segs, hipStream_t s) {
    const int rows_per_wg = segs >= 4 ? 1 : 4 / segs;
    const int threads = 64 * segs * rows_per_wg;
    const int64_t blocks1 = (a.rows + rows_per_wg - 1) / rows_per_wg;
    const int64_t blocks = blocks1 + (a.rows2 + rows_per_wg - 1) / rows_per_wg;
    const float c_norm = a.log_block > 0 ? (float)(1.0 / sqrt((double)(int64_t(1) << a.log_block))) : 1.0f;
    if (a.log_block == 0)
        hipLaunchKernelGGL((row_transform_kernel<LOGSEG, IN, OUT, 0>), dim3((unsigned)blocks), dim3(threads), 0, s,
                           a, segs, rows_per_wg, c_norm, (unsigned)blocks1);
    else if (a.log_block == LOGSEG)
        hipLaunchKernelGGL((row_transform_kernel<LOGSEG, IN, OUT, LOGSEG>), dim3((unsigned)blocks), dim3(threads), 0, s,
                           a, segs, rows_per_wg, c_norm, (unsigned)blocks1);
    else
        hipLaunchKernelGGL((row_transform_kernel<LOGSEG, IN, OUT, -1>), dim3((unsigned)blocks), dim3(threads), 0, s,
                           a, segs, rows_per_wg, c_norm, (unsigned)blocks1);
    return hipGetLastError();
}

template <int IN, int OUT>
hipError_t launch_by_seg(const RowArgs& a, hipStream_t s) {
    // Split blocks of 2048 / 4096 over 2 / 4 wavefronts (measured): the 32-bit-input un-rotation gains at every size
    // for 4096-blocks (5.7 vs 5.2 TB/s at 32768 rows, 12.7 vs 16.0 us at 2048 rows); the quantiser only when whole
    // rows would leave the 1024 SIMDs with fewer than four wavefronts each.
    if ((a.log_block == 11 || a.log_block == 12) && a.cols % 1024 == 0 && a.cols <= 16384) {
        const int64_t wavefronts_unsplit = (a.rows + a.rows2) * (a.cols >> a.log_block);
        const bool want = IN == IN_I32 ? a.log_block == 12 : wavefronts_unsplit < 4096;
        if (want) return a.log_block == 11 ? launch_split<IN, OUT, 1>(a, s) : launch_split<IN, OUT, 2>(a, s);
    }
    // Segment = max(Hadamard block, 512), grown until the row fits the workgroup (16 waves, 8 from 2048 up).
    int logseg = a.log_block < 9 ? 9 : a.log_block;
    if (a.log_block == 0) {
        // no rotation: any segmentation is valid; 1024-element segments keep register use low
        logseg = a.cols <= 512 ? 9 : 10;
    }
    for (;; ++logseg) {
        if (logseg > 12) return hipErrorInvalidValue;
        const int64_t segs = (a.cols + (int64_t(1) << logseg) - 1) >> logseg;
        if (segs <= (logseg >= 11 ? 8 : 16)) break;
    }
    const int segs = (int)((a.cols + (int64_t(1) << logseg) - 1) >> logseg);
    switch (logseg) {
        case 9: return launch_one<9, IN, OUT>(a, segs, s);
        case 10: return launch_one<10, IN, OUT>(a, segs, s);
        case 11: return launch_one<11, IN, OUT>(a, segs, s);
        default: return launch_one<12, IN, OUT>(a, segs, s);
    }
}

// The end of a left+right un-rotation (see halo_internal.h).  Workgroup = 2^TOP wavefronts; wavefront t owns row
// blk * hb + t * 256 + q of one right-hand block of 2^LOGSEG columns, hb = 256 << TOP: exactly the rows that the top TOP
// strides of the left-hand rotation (256, 512, ...) combine.  Stage st pairs wavefront t with t ^ 2^st through LDS (the
// lower row takes a + b, the upper one a - b), ascending; then the wavefront has its row of the left-rotated matrix in
// registers, in the layout of the row kernel, and goes on as that kernel does.
// TOP == 5 (segments up to 2048 columns): the 32 rows sit two to a wavefront, rows t * 256 + q and (t + 16) * 256 + q of the
// block of 8192; the first four of the five strides go through LDS as before, for both rows, and the last one (4096 rows)
// pairs the wavefront's own two rows in registers.
template <int LOGSEG, int OUT, int TOP>
__global__ void __launch_bounds__(TOP >= 5 ? 1024 : (64 << TOP), (LOGSEG >= 12 || TOP >= 5) ? 4 : 8)
row_left_top_kernel(RowArgs a, int segs, float c_norm) {
    constexpr int LOGE = 2, EPL = 4;
    constexpr int VPL = 1 << (LOGSEG - 6);
    constexpr int NCH = VPL / EPL;
    constexpr int SEG = 1 << LOGSEG;
    constexpr int NR = TOP >= 5 ? 2 : 1;                    // rows per wavefront
    constexpr int XT = TOP >= 5 ? 4 : TOP;                  // strides that go through LDS
    static_assert(TOP <= 5 && (TOP < 5 || LOGSEG <= 11), "32 rows of 4096 columns do not fit a compute unit");
    extern __shared__ __align__(16) float s_exch[];        // exchange buffer of the stages across wavefronts

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t g = (int64_t)blockIdx.x / segs;                 // group of 2^TOP rows: g = blk * 256 + q
    const int seg = (int)((int64_t)blockIdx.x % segs);
    const int64_t row0 = ((g >> 8) << (8 + TOP)) + ((int64_t)wave << 8) + (g & 255);
    const int64_t kbase = (int64_t)seg * SEG + (int64_t)lane * EPL;

    float v[NR][VPL];
#pragma unroll
    for (int n = 0; n < NR; ++n) {
        const float* src = reinterpret_cast<const float*>(a.in) + (row0 + (int64_t)n * 4096) * a.ld_in + kbase;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const float4 q = *reinterpret_cast<const float4*>(src + c * 64 * EPL);
            v[n][c * EPL + 0] = q.x; v[n][c * EPL + 1] = q.y; v[n][c * EPL + 2] = q.z; v[n][c * EPL + 3] = q.w;
        }
    }
    // Exchange buffer: [wavefront][value / 4][lane][4] (16-byte LDS accesses), HALF values per wavefront at a time so that
    // two workgroups fit one compute unit's LDS and one of them can load while the other exchanges.
    constexpr int HALF = VPL > 16 ? VPL / 2 : VPL;
    float4* xb = reinterpret_cast<float4*>(s_exch);
    bool first_round = true;
#pragma unroll
    for (int st = 0; st < XT; ++st) {
        const bool upper = (wave >> st) & 1;
        const int pw = wave ^ (1 << st);
#pragma unroll
        for (int n = 0; n < NR; ++n) {
#pragma unroll
            for (int h0 = 0; h0 < VPL; h0 += HALF) {
                if (!first_round) __syncthreads();   // everyone has read the previous round
                first_round = false;
#pragma unroll
                for (int r = 0; r < HALF; r += 4)
                    xb[(wave * (HALF / 4) + r / 4) * 64 + lane] =
                        make_float4(v[n][h0 + r], v[n][h0 + r + 1], v[n][h0 + r + 2], v[n][h0 + r + 3]);
                __syncthreads();
#pragma unroll
                for (int r = 0; r < HALF; r += 4) {
                    const float4 p = xb[(pw * (HALF / 4) + r / 4) * 64 + lane];
                    v[n][h0 + r + 0] = upper ? p.x - v[n][h0 + r + 0] : v[n][h0 + r + 0] + p.x;
                    v[n][h0 + r + 1] = upper ? p.y - v[n][h0 + r + 1] : v[n][h0 + r + 1] + p.y;
                    v[n][h0 + r + 2] = upper ? p.z - v[n][h0 + r + 2] : v[n][h0 + r + 2] + p.z;
                    v[n][h0 + r + 3] = upper ? p.w - v[n][h0 + r + 3] : v[n][h0 + r + 3] + p.w;
                }
            }
        }
    }
    if constexpr (NR == 2) {               // the last stride: the wavefront's own two rows
#pragma unroll
        for (int r = 0; r < VPL; ++r) {
            const float x = v[0][r], y = v[NR - 1][r];
            v[0][r] = x + y;
            v[NR - 1][r] = x - y;
        }
    }
    const int bperm_addr = (lane ^ 32) << 2;
    const float c_l = (__builtin_popcount(lane) & 1) ? -c_norm : c_norm;     // the sign the lane stages leave behind
#pragma unroll
    for (int n = 0; n < NR; ++n) {
        if (a.in_mul != 0.0f) {
#pragma unroll
            for (int r = 0; r < VPL; ++r) v[n][r] *= a.in_mul;
        }
        // right-hand un-rotation of the row (block = segment), as in row_phase1
        FwhtStages<VPL, LOGE, 0, LOGSEG>::run(v[n], LOGSEG, lane, bperm_addr);
#pragma unroll
        for (int r = 0; r < VPL; ++r) v[n][r] *= c_l;

        RowCtx x;
        x.lane = lane; x.bperm_addr = bperm_addr; x.wave = wave; x.seg = seg; x.xbuf = s_exch;
        x.row = row0 + (int64_t)n * 4096; x.kbase = kbase; x.row_ok = true;
        row_phase2<LOGSEG, IN_F32, OUT, true>(a, x, v[n], 0.0f);
    }
}

template <int LOGSEG, int OUT, int TOP>
hipError_t launch_left_top(const RowArgs& a, hipStream_t s) {
    constexpr int VPL = 1 << (LOGSEG - 6);
    constexpr int kWaves = TOP >= 5 ? 16 : (1 << TOP);
    constexpr int kLds = kWaves * (VPL > 16 ? VPL / 2 : VPL) * 64 * (int)sizeof(float);
    static std::once_flag once;
    static hipError_t attr_result = hipSuccess;
    auto kern = row_left_top_kernel<LOGSEG, OUT, TOP>;
    std::call_once(once, [&] {
        if (kLds > 64 * 1024)
            attr_result = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    });
    if (attr_result != hipSuccess) return attr_result;
    const int segs = (int)(a.cols >> LOGSEG);
    const int64_t blocks = (a.rows >> TOP) * segs;
    if (blocks <= 0 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    const float c_norm = (float)(1.0 / sqrt((double)(int64_t(1) << LOGSEG)));
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * kWaves), kLds, s, a, segs, c_norm);
    return hipGetLastError();
}

template <int LOGSEG, int OUT>
hipError_t launch_left_top_by_top(const RowArgs& a, hipStream_t s) {
    switch (a.left_top) {
        case 1: return launch_left_top<LOGSEG, OUT, 1>(a, s);
        case 2: return launch_left_top<LOGSEG, OUT, 2>(a, s);
        case 3: return launch_left_top<LOGSEG, OUT, 3>(a, s);
        case 4: return launch_left_top<LOGSEG, OUT, 4>(a, s);
        case 5:
            if constexpr (LOGSEG <= 11) return launch_left_top<LOGSEG, OUT, 5>(a, s);
            return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

template <int OUT>
hipError_t launch_left_top_by_seg(const RowArgs& a, hipStream_t s) {
    switch (a.log_block) {
        case 9: return launch_left_top_by_top<9, OUT>(a, s);
        case 10: return launch_left_top_by_top<10, OUT>(a, s);
        case 11: return launch_left_top_by_top<11, OUT>(a, s);
        case 12: return launch_left_top_by_top<12, OUT>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool row_left_top_ok(int64_t rows, int64_t cols, int log_block, int left_top) {
    if (log_block < 9 || log_block > 12 || left_top < 1 || left_top > 5) return false;
    if (left_top == 5 && log_block > 11) return false;      // 32 rows of 4096 columns do not fit a compute unit
    if (rows <= 0 || cols <= 0 || cols % (int64_t(1) << log_block) != 0) return false;
    return rows % (int64_t(256) << left_top) == 0;
}

hipError_t launch_row_left_top(const RowArgs& a, OutKind out, hipStream_t s) {
    if (a.kron_m != 0 || a.fold || a.rows2 != 0 || !row_left_top_ok(a.rows, a.cols, a.log_block, a.left_top))
        return hipErrorInvalidValue;
    if (out == OUT_BF16) return launch_left_top_by_seg<OUT_BF16>(a, s);
    if (out == OUT_F32) return launch_left_top_by_seg<OUT_F32>(a, s);
    return hipErrorInvalidValue;
}

hipError_t launch_row_transform(const RowArgs& a, InKind in, OutKind out, hipStream_t s) {
    if ((a.rows == 0 && a.rows2 == 0) || a.cols == 0) return hipSuccess;
    if (a.kron_m != 0) return out == OUT_MX6 ? hipErrorInvalidValue : launch_row_kron(a, in, out, s);
    if (a.cols > kMaxRowCols || a.log_block > 12) return hipErrorInvalidValue;
    if (in == IN_BF16 && out == OUT_Q8) return launch_by_seg<IN_BF16, OUT_Q8>(a, s);
    if (in == IN_F32 && out == OUT_Q8) return launch_by_seg<IN_F32, OUT_Q8>(a, s);
    if (in == IN_I32 && out == OUT_BF16) return launch_by_seg<IN_I32, OUT_BF16>(a, s);
    if (in == IN_I32 && out == OUT_F32) return launch_by_seg<IN_I32, OUT_F32>(a, s);
    if (in == IN_F32 && out == OUT_BF16) return launch_by_seg<IN_F32, OUT_BF16>(a, s);
    if (in == IN_F32 && out == OUT_F32) return launch_by_seg<IN_F32, OUT_F32>(a, s);
    if (in == IN_BF16 && out == OUT_MX6) return a.cols % 32 == 0 ? launch_by_seg<IN_BF16, OUT_MX6>(a, s) : hipErrorInvalidValue;
    return hipErrorInvalidValue;
}

}  // namespace halo
