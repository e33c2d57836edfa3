// Stage 2 of the SageAttention2++ 8+8 forward on gfx950: the fused attention
// kernel (paper Sec. 2.1 for the tiling / online softmax and the scales,
// Sec. 3.1 for the bounded FP8 range P_r of P~).
//
// Mapping to CDNA4.  A workgroup of 4 wavefronts owns BM = 64*NQ query rows of
// one (batch, head); a wavefront owns NQ tiles of 16 query rows.  Per step of
// 128 keys the K^ tile [128][D] int8 and the V^ tile [D][128] fp8 are staged in
// LDS (16-byte chunks XOR-swizzled against bank conflicts).
//   S^T = K^ Q^T   with v_mfma_i32_16x16x64_i8 (keys are MFMA rows, queries are
//                  MFMA columns).  A lane then holds, for ONE query (lane&15),
//                  the scores of keys 16t + 4(lane>>4) + i, t<8, i<4: the row
//                  maximum and sum are in-lane work plus two cross-lane steps.
//   softmax        base 2, FP32; the de-quantisation constant
//                  delta_Q*delta_K*sm_scale*log2(e) is one FMA operand, the
//                  maximum is taken on the integer scores per 64-key K block.
//   P^             v_cvt_pk_fp8_f32 in registers: the 32 bytes a lane produces
//                  are exactly its B operand of v_mfma_f32_16x16x128_f8f6f4.
//   O^T += V^T P^T with that instruction (FP8 E4M3 both sides, FP32 accumulate);
//                  V^ is stored transposed and key-permuted by the quantiser so
//                  that the A operand is 32 contiguous bytes of LDS.
// The accumulator is rescaled only in steps where some row maximum moved
// (multiplying by alpha == 1 is the identity, so skipping is exact).
#include "sage_internal.h"

#include <limits.h>
#include <math.h>

namespace sage {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

// LDS byte offset of 16-byte chunk `c16` of row `row` of the K^ tile (row = key, D bytes per row).
template <int D>
__device__ __forceinline__ int k_off(int row, int c16) {
    if constexpr (D == 128) {
        return row * 128 + ((c16 ^ (row & 7)) << 4);
    } else {
        return row * 64 + ((c16 ^ ((row >> 1) & 3)) << 4);
    }
}
// Same for the V^ tile (row = channel, 128 bytes = 8 chunks per row).
__device__ __forceinline__ int v_off(int row, int c16) { return row * 128 + ((c16 ^ (row & 7)) << 4); }

__device__ __forceinline__ int imax3(int a, int b, int c) { return max(max(a, b), c); }

template <bool BF16>
__device__ __forceinline__ uint32_t pack2(float a, float b) {
    if constexpr (BF16) {
        uint32_t ua = __builtin_bit_cast(uint32_t, a), ub = __builtin_bit_cast(uint32_t, b);
        ua = (ua + 0x7fffu + ((ua >> 16) & 1u)) >> 16;
        ub = (ub + 0x7fffu + ((ub >> 16) & 1u)) >> 16;
        return ua | (ub << 16);
    } else {
        const uint32_t ua = __builtin_bit_cast(uint16_t, (_Float16)a);
        const uint32_t ub = __builtin_bit_cast(uint16_t, (_Float16)b);
        return ua | (ub << 16);
    }
}

template <int D, int NQ, bool CAUSAL, bool BF16>
__global__ __launch_bounds__(256, 2) void attn_kernel(
    const int8_t *__restrict__ Qc, const int8_t *__restrict__ Kc, const uint8_t *__restrict__ Vt,
    const float *__restrict__ dq, const float *__restrict__ dk, const float *__restrict__ dv,
    uint16_t *__restrict__ out, int N, int nT, int nQblk, int nKblk, float sm_scale, float log2_pr) {
    constexpr int BM = 64 * NQ;  // query rows per workgroup
    constexpr int KC = D / 64;   // 64-wide contraction chunks of Q.K^T
    constexpr int CT = D / 16;   // 16-channel tiles of the output
    __shared__ __attribute__((aligned(16))) uint8_t Ks[128 * D];
    __shared__ __attribute__((aligned(16))) uint8_t Vs[D * 128];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 15, g = lane >> 4;
    const int bh = blockIdx.y;
    // causal: heaviest (last) query tiles are launched first
    const int qtile = CAUSAL ? (int)(gridDim.x - 1 - blockIdx.x) : (int)blockIdx.x;
    const int wg_row0 = qtile * BM;
    const int row0 = wg_row0 + wave * (16 * NQ);

    const int8_t *Qh = Qc + (size_t)bh * N * D;
    const int8_t *Kh = Kc + (size_t)bh * N * D;
    const uint8_t *Vh = Vt + (size_t)bh * nT * D * 128;

    v4i qreg[NQ][KC];
    double cq[NQ];
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        const int r = row0 + qt * 16 + lq;
#pragma unroll
        for (int ch = 0; ch < KC; ++ch) {
            v4i z = {0, 0, 0, 0};
            qreg[qt][ch] = r < N ? *reinterpret_cast<const v4i *>(Qh + (size_t)r * D + ch * 64 + g * 16) : z;
        }
        const int blk = min(row0 + qt * 16, N - 1) / kBQ;
        cq[qt] = (double)dq[(size_t)bh * nQblk + blk] * (double)sm_scale * 1.4426950408889634;
    }

    float m[NQ], l[NQ];
    v4f o[CT][NQ];
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        m[qt] = -INFINITY;
        l[qt] = 0.0f;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) o[ct][qt] = v4f{0.f, 0.f, 0.f, 0.f};
    }

    int nsteps = nT;
    if constexpr (CAUSAL) nsteps = min(N - 1, wg_row0 + BM - 1) / kW + 1;

    for (int j = 0; j < nsteps; ++j) {
        const int key0 = j * kW;
        __syncthreads();  // every wave is done reading the previous tiles
#pragma unroll
        for (int k = 0; k < D / 32; ++k) {
            const int e = tid + 256 * k;
            const int row = e / (D / 16), c16 = e % (D / 16);
            const int gr = key0 + row;
            v4i val = {0, 0, 0, 0};
            if (gr < N) val = *reinterpret_cast<const v4i *>(Kh + (size_t)gr * D + c16 * 16);
            *reinterpret_cast<v4i *>(Ks + k_off<D>(row, c16)) = val;
        }
#pragma unroll
        for (int k = 0; k < D / 32; ++k) {
            const int e = tid + 256 * k;
            const int row = e >> 3, c16 = e & 7;
            const v4i val = *reinterpret_cast<const v4i *>(Vh + ((size_t)j * D + row) * 128 + c16 * 16);
            *reinterpret_cast<v4i *>(Vs + v_off(row, c16)) = val;
        }
        __syncthreads();

        // causal tile skipping at wavefront granularity: every key of this step lies
        // above every query row of this wavefront
        if (CAUSAL && key0 > row0 + 16 * NQ - 1) continue;

        // ---- S^T = K^ Q^T (INT8, INT32 accumulation) ----
        v4i s[8][NQ];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
#pragma unroll
            for (int qt = 0; qt < NQ; ++qt) s[t][qt] = v4i{0, 0, 0, 0};
#pragma unroll
            for (int ch = 0; ch < KC; ++ch) {
                const v4i a = *reinterpret_cast<const v4i *>(Ks + k_off<D>(16 * t + lq, 4 * ch + g));
#pragma unroll
                for (int qt = 0; qt < NQ; ++qt)
                    s[t][qt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, qreg[qt][ch], s[t][qt], 0, 0, 0);
            }
        }

        const bool masked_step = (key0 + kW > N) || (CAUSAL && key0 + kW - 1 > row0);
        const int kb0 = min(2 * j, nKblk - 1), kb1 = min(2 * j + 1, nKblk - 1);
        const double dk0 = (double)dk[(size_t)bh * nKblk + kb0], dk1 = (double)dk[(size_t)bh * nKblk + kb1];

        v8i pb[NQ];
        float alpha[NQ];
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
            const float c0 = (float)(cq[qt] * dk0), c1 = (float)(cq[qt] * dk1);
            if (masked_step) {
                const int r = row0 + qt * 16 + lq;
                int lim = N - 1;  // last visible key of this query row
                if constexpr (CAUSAL) lim = min(lim, r);
#pragma unroll
                for (int t = 0; t < 8; ++t)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (key0 + 16 * t + 4 * g + i > lim) s[t][qt][i] = INT_MIN;
            }
            // step maximum, taken on the integers of each 64-key K block (its scale is positive)
            int im0 = INT_MIN, im1 = INT_MIN;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                im0 = imax3(im0, s[t][qt][0], s[t][qt][1]);
                im0 = imax3(im0, s[t][qt][2], s[t][qt][3]);
                im1 = imax3(im1, s[t + 4][qt][0], s[t + 4][qt][1]);
                im1 = imax3(im1, s[t + 4][qt][2], s[t + 4][qt][3]);
            }
            float mc0 = (float)im0 * c0, mc1 = (float)im1 * c1;
            if (masked_step) {
                mc0 = im0 == INT_MIN ? -INFINITY : mc0;
                mc1 = im1 == INT_MIN ? -INFINITY : mc1;
            }
            float mc = fmaxf(mc0, mc1);
            mc = fmaxf(mc, __shfl_xor(mc, 16));
            mc = fmaxf(mc, __shfl_xor(mc, 32));
            const float m_new = fmaxf(m[qt], mc);
            alpha[qt] = __builtin_amdgcn_exp2f(m[qt] - m_new);
            const float mo = log2_pr - m_new;  // P~ * P_r = 2^(x - m' + log2 P_r)
            float lsum = 0.0f;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const float cb = t < 4 ? c0 : c1;
                float p[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    p[i] = __builtin_amdgcn_exp2f(__builtin_fmaf((float)s[t][qt][i], cb, mo));
                    if (masked_step) p[i] = s[t][qt][i] == INT_MIN ? 0.0f : p[i];
                }
                lsum += (p[0] + p[1]) + (p[2] + p[3]);
                int w = 0;
                w = __builtin_amdgcn_cvt_pk_fp8_f32(p[0], p[1], w, false);
                w = __builtin_amdgcn_cvt_pk_fp8_f32(p[2], p[3], w, true);
                pb[qt][t] = w;
            }
            l[qt] = l[qt] * alpha[qt] + lsum;
            m[qt] = m_new;
        }

        // ---- rescale O only when some running maximum moved ----
        bool moved = false;
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) moved |= alpha[qt] != 1.0f;
        if (__builtin_amdgcn_ballot_w64(moved) != 0) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int qt = 0; qt < NQ; ++qt) o[ct][qt] *= alpha[qt];
        }

        // ---- O^T += V^T P^T (FP8 E4M3 x E4M3, FP32 accumulation) ----
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const int row = 16 * ct + lq;
            const v4i lo = *reinterpret_cast<const v4i *>(Vs + v_off(row, 2 * g));
            const v4i hi = *reinterpret_cast<const v4i *>(Vs + v_off(row, 2 * g + 1));
            const v8i a = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
#pragma unroll
            for (int qt = 0; qt < NQ; ++qt)
                o[ct][qt] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, pb[qt], o[ct][qt], 0, 0, 0, 0, 0, 0);
        }
    }

    // ---- epilogue: O = acc * delta_V / (P_r * l); l already carries the factor P_r ----
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        float lt = l[qt];
        lt += __shfl_xor(lt, 16);
        lt += __shfl_xor(lt, 32);
        const float inv = 1.0f / lt;
        const int r = row0 + qt * 16 + lq;
        if (r < N) {
            uint16_t *orow = out + ((size_t)bh * N + r) * D;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const int c = 16 * ct + 4 * g;
                const float4 sc = *reinterpret_cast<const float4 *>(dv + (size_t)bh * D + c);
                const float y0 = o[ct][qt][0] * (sc.x * inv), y1 = o[ct][qt][1] * (sc.y * inv);
                const float y2 = o[ct][qt][2] * (sc.z * inv), y3 = o[ct][qt][3] * (sc.w * inv);
                *reinterpret_cast<uint2 *>(orow + c) = make_uint2(pack2<BF16>(y0, y1), pack2<BF16>(y2, y3));
            }
        }
    }
}

template <int D, int NQ>
hipError_t launch_d(const int8_t *q_i8, const int8_t *k_i8, const uint8_t *v_fp8, const float *q_scale,
                    const float *k_scale, const float *v_scale, void *out, int BH, int N, bool causal,
                    float sm_scale, float log2_pr, bool bf16_out, hipStream_t stream) {
    constexpr int BM = 64 * NQ;
    const dim3 grid(cdiv(N, BM), BH);
    const int nT = cdiv(N, kW), nQ = cdiv(N, kBQ), nK = cdiv(N, kBK);
    uint16_t *o16 = static_cast<uint16_t *>(out);
#define SAGE_LAUNCH(C, BF)                                                                             \
    attn_kernel<D, NQ, C, BF><<<grid, 256, 0, stream>>>(q_i8, k_i8, v_fp8, q_scale, k_scale, v_scale, \
                                                        o16, N, nT, nQ, nK, sm_scale, log2_pr)
    if (causal) {
        if (bf16_out) SAGE_LAUNCH(true, true); else SAGE_LAUNCH(true, false);
    } else {
        if (bf16_out) SAGE_LAUNCH(false, true); else SAGE_LAUNCH(false, false);
    }
#undef SAGE_LAUNCH
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn(const int8_t *q_i8, const int8_t *k_i8, const uint8_t *v_fp8, const float *q_scale,
                       const float *k_scale, const float *v_scale, void *out, int B, int H, int N, int d,
                       bool causal, float sm_scale, float p_r, bool bf16_out, hipStream_t stream) {
    const float log2_pr = (float)log2((double)p_r);
    if (d == 128)
        return launch_d<128, 2>(q_i8, k_i8, v_fp8, q_scale, k_scale, v_scale, out, B * H, N, causal, sm_scale,
                                log2_pr, bf16_out, stream);
    return launch_d<64, 2>(q_i8, k_i8, v_fp8, q_scale, k_scale, v_scale, out, B * H, N, causal, sm_scale,
                           log2_pr, bf16_out, stream);
}

}  // namespace sage
