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

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
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

template <int VPL, int J>
__device__ __forceinline__ void stage_across_lanes(float (&v)[VPL], int lane, int bperm_addr) {
    const float s = ((lane >> J) & 1) ? -1.0f : 1.0f;
#pragma unroll
    for (int r = 0; r < VPL; ++r) {
        const float p = lane_xor<J>(v[r], bperm_addr);
        v[r] = __builtin_fmaf(p, s, v[r]);
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

template <int LOGSEG, int IN, int OUT>
__global__ void __launch_bounds__(LOGSEG >= 12 ? 512 : 1024)
row_transform_kernel(RowArgs a, int segs, int rows_per_wg, float c_norm) {
    constexpr int LOGE = (IN == IN_BF16) ? 3 : 2;
    constexpr int EPL = 1 << LOGE;            // consecutive elements per lane per chunk
    constexpr int VPL = 1 << (LOGSEG - 6);    // values per lane
    constexpr int NCH = VPL / EPL;            // chunks per lane
    constexpr int SEG = 1 << LOGSEG;

    __shared__ float s_amax[16];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int seg = wave % segs;
    const int row_local = wave / segs;
    const int64_t row = (int64_t)blockIdx.x * rows_per_wg + row_local;
    const bool row_ok = row < a.rows;
    const int bperm_addr = (lane ^ 32) << 2;
    const int64_t kbase = (int64_t)seg * SEG + (int64_t)lane * EPL;

    float v[VPL];

    // ------------------------------------------------------------------ load
    float pre = 1.0f;
    if constexpr (IN == IN_I32) {
        if (row_ok && a.pre_scale) pre = a.pre_scale[row];
    }
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int64_t k0 = kbase + (int64_t)c * 64 * EPL;
        if (row_ok && k0 + EPL <= a.cols) {
            if constexpr (IN == IN_BF16) {
                const uint4 q = *reinterpret_cast<const uint4*>(
                    reinterpret_cast<const uint16_t*>(a.in) + row * a.ld_in + k0);
                const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    v[c * EPL + 2 * i] = __uint_as_float(w[i] << 16);
                    v[c * EPL + 2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
                }
            } else if constexpr (IN == IN_F32) {
                const float4 q = *reinterpret_cast<const float4*>(
                    reinterpret_cast<const float*>(a.in) + row * a.ld_in + k0);
                v[c * EPL + 0] = q.x; v[c * EPL + 1] = q.y; v[c * EPL + 2] = q.z; v[c * EPL + 3] = q.w;
            } else {
                const int4 q = *reinterpret_cast<const int4*>(
                    reinterpret_cast<const int32_t*>(a.in) + row * a.ld_in + k0);
                v[c * EPL + 0] = (float)q.x * pre; v[c * EPL + 1] = (float)q.y * pre;
                v[c * EPL + 2] = (float)q.z * pre; v[c * EPL + 3] = (float)q.w * pre;
            }
        } else {
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                float t = 0.0f;
                if (row_ok && k0 + e < a.cols) {
                    if constexpr (IN == IN_BF16) {
                        t = __uint_as_float((uint32_t)(reinterpret_cast<const uint16_t*>(a.in)[row * a.ld_in + k0 + e]) << 16);
                    } else if constexpr (IN == IN_F32) {
                        t = reinterpret_cast<const float*>(a.in)[row * a.ld_in + k0 + e];
                    } else {
                        t = (float)reinterpret_cast<const int32_t*>(a.in)[row * a.ld_in + k0 + e] * pre;
                    }
                }
                v[c * EPL + e] = t;
            }
        }
    }

    // ------------------------------------------------------------------ rotate
    const int log_block = a.log_block;
    if (log_block > 0) {
        FwhtStages<VPL, LOGE, 0, LOGSEG>::run(v, log_block, lane, bperm_addr);
        // lanes whose (lane & mask) has odd parity hold negated values; fold that into the normalisation
        int nlane_stages = log_block - LOGE;
        nlane_stages = nlane_stages < 0 ? 0 : (nlane_stages > 6 ? 6 : nlane_stages);
        const int mask = (1 << nlane_stages) - 1;
        const float c_l = (__builtin_popcount(lane & mask) & 1) ? -c_norm : c_norm;
#pragma unroll
        for (int r = 0; r < VPL; ++r) v[r] *= c_l;
    }

    // ------------------------------------------------------------------ fold
    if (a.fold) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int64_t k0 = kbase + (int64_t)c * 64 * EPL;
            if (k0 + EPL <= a.cols) {
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

    // ------------------------------------------------------------------ store
    if constexpr (OUT == OUT_Q8) {
        float amax = 0.0f;
#pragma unroll
        for (int r = 0; r < VPL; ++r) amax = fmaxf(amax, fabsf(v[r]));
        amax = wave_max(amax, bperm_addr);
        if (segs > 1) {
            if (lane == 0) s_amax[wave] = amax;
            __syncthreads();
            const int w0 = row_local * segs;
            float t = s_amax[w0];
            for (int i = 1; i < segs; ++i) t = fmaxf(t, s_amax[w0 + i]);
            amax = t;
        }
        const bool nz = amax > 0.0f;
        const float inv = nz ? 127.0f / amax : 0.0f;
        if (row_ok && seg == 0 && lane == 0) a.out_scale[row] = nz ? amax / 127.0f : 1.0f;
        int8_t* orow = reinterpret_cast<int8_t*>(a.out) + row * a.ld_out;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int64_t k0 = kbase + (int64_t)c * 64 * EPL;
            uint32_t packed[EPL / 4];
#pragma unroll
            for (int i = 0; i < EPL / 4; ++i) {
                uint32_t b[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float t = v[c * EPL + 4 * i + e] * inv;
                    b[e] = __float_as_uint(t + kRoundMagic);
                }
                const uint32_t lo = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u);
                const uint32_t hi = __builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u);
                packed[i] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
            }
            if (row_ok && k0 + EPL <= a.cols) {
                if constexpr (EPL == 8) {
                    *reinterpret_cast<uint2*>(orow + k0) = make_uint2(packed[0], packed[1]);
                } else {
                    *reinterpret_cast<uint32_t*>(orow + k0) = packed[0];
                }
            } else if (row_ok) {
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    if (k0 + e < a.cols) orow[k0 + e] = (int8_t)((packed[e / 4] >> (8 * (e & 3))) & 0xFF);
            }
        }
    } else if constexpr (OUT == OUT_BF16) {
        uint16_t* orow = reinterpret_cast<uint16_t*>(a.out) + row * a.ld_out;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int64_t k0 = kbase + (int64_t)c * 64 * EPL;
            uint32_t packed[EPL / 2];
#pragma unroll
            for (int i = 0; i < EPL / 2; ++i)
                packed[i] = f32_to_bf16_rne(v[c * EPL + 2 * i]) | (f32_to_bf16_rne(v[c * EPL + 2 * i + 1]) << 16);
            if (row_ok && k0 + EPL <= a.cols) {
                if constexpr (EPL == 8) {
                    *reinterpret_cast<uint4*>(orow + k0) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
                } else {
                    *reinterpret_cast<uint2*>(orow + k0) = make_uint2(packed[0], packed[1]);
                }
            } else if (row_ok) {
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    if (k0 + e < a.cols) orow[k0 + e] = (uint16_t)(packed[e / 2] >> (16 * (e & 1)));
            }
        }
    } else {
        float* orow = reinterpret_cast<float*>(a.out) + row * a.ld_out;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int64_t k0 = kbase + (int64_t)c * 64 * EPL;
            if (row_ok && k0 + EPL <= a.cols) {
#pragma unroll
                for (int i = 0; i < EPL / 4; ++i)
                    *reinterpret_cast<float4*>(orow + k0 + 4 * i) =
                        make_float4(v[c * EPL + 4 * i], v[c * EPL + 4 * i + 1], v[c * EPL + 4 * i + 2], v[c * EPL + 4 * i + 3]);
            } else if (row_ok) {
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    if (k0 + e < a.cols) orow[k0 + e] = v[c * EPL + e];
            }
        }
    }
}

template <int LOGSEG, int IN, int OUT>
hipError_t launch_one(const RowArgs& a, int segs, hipStream_t s) {
    const int rows_per_wg = segs >= 4 ? 1 : 4 / segs;
    const int threads = 64 * segs * rows_per_wg;
    const int64_t blocks = (a.rows + rows_per_wg - 1) / rows_per_wg;
    const float c_norm = a.log_block > 0 ? (float)(1.0 / sqrt((double)(int64_t(1) << a.log_block))) : 1.0f;
    hipLaunchKernelGGL((row_transform_kernel<LOGSEG, IN, OUT>), dim3((unsigned)blocks), dim3(threads), 0, s,
                       a, segs, rows_per_wg, c_norm);
    return hipGetLastError();
}

template <int IN, int OUT>
hipError_t launch_by_seg(const RowArgs& a, hipStream_t s) {
    // Segment = max(Hadamard block, 512), grown until the row fits the workgroup (16 waves, 8 at 4096).
    int logseg = a.log_block < 9 ? 9 : a.log_block;
    if (a.log_block == 0) {
        // no rotation: any segmentation is valid; 1024-element segments keep register use low
        logseg = a.cols <= 512 ? 9 : 10;
    }
    for (;; ++logseg) {
        if (logseg > 12) return hipErrorInvalidValue;
        const int64_t segs = (a.cols + (int64_t(1) << logseg) - 1) >> logseg;
        if (segs <= (logseg == 12 ? 8 : 16)) break;
    }
    const int segs = (int)((a.cols + (int64_t(1) << logseg) - 1) >> logseg);
    switch (logseg) {
        case 9: return launch_one<9, IN, OUT>(a, segs, s);
        case 10: return launch_one<10, IN, OUT>(a, segs, s);
        case 11: return launch_one<11, IN, OUT>(a, segs, s);
        default: return launch_one<12, IN, OUT>(a, segs, s);
    }
}

}  // namespace

hipError_t launch_row_transform(const RowArgs& a, InKind in, OutKind out, hipStream_t s) {
    if (a.rows == 0 || a.cols == 0) return hipSuccess;
    if (a.cols > kMaxRowCols || a.log_block > 12) return hipErrorInvalidValue;
    if (in == IN_BF16 && out == OUT_Q8) return launch_by_seg<IN_BF16, OUT_Q8>(a, s);
    if (in == IN_F32 && out == OUT_Q8) return launch_by_seg<IN_F32, OUT_Q8>(a, s);
    if (in == IN_I32 && out == OUT_BF16) return launch_by_seg<IN_I32, OUT_BF16>(a, s);
    if (in == IN_I32 && out == OUT_F32) return launch_by_seg<IN_I32, OUT_F32>(a, s);
    return hipErrorInvalidValue;
}

}  // namespace halo
