// Device-side building blocks shared by the attention kernels of libsage (gfx950): vector types, the lane
// exchanges over the four 16-lane rows of a wavefront, 16-bit conversions, and the online-softmax step of the
// 8+8 path (paper Sec. 2.1 for the online softmax and the scales, Sec. 3.1 for the bounded FP8 range of P~).
// Included by sage_attn.hip (prefill) and sage_decode.hip (decode-shaped calls); every function is inlined.
#pragma once
#include <hip/hip_runtime.h>
#include <limits.h>
#include <math.h>
#include <stdint.h>

namespace sage {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;

// 16-byte-chunk swizzles.  K^ tile: row = key, D bytes per row.  V^ tile: row = channel, 128 bytes per row.
template <int D>
__device__ __forceinline__ int k_swz(int row) {
    return D == 128 ? (row & 7) : ((row >> 1) & 3);
}
template <int D>
__device__ __forceinline__ int k_off(int row, int c16) {
    return row * D + ((c16 ^ k_swz<D>(row)) << 4);
}
__device__ __forceinline__ int v_off(int row, int c16) { return row * 128 + ((c16 ^ (row & 7)) << 4); }

__device__ __forceinline__ int imax3(int a, int b, int c) { return max(max(a, b), c); }

// Cross-lane exchange over the four 16-lane rows of a wavefront (lanes l, l^16, l^32, l^48).
// v_permlane16_swap exchanges the odd rows of its first register with the even rows of its second,
// v_permlane32_swap the upper half of the first with the lower half of the second: starting from
// two copies of x, the pair (a, b) then holds both partners' values in every lane.  The two copies
// must live in distinct registers.
// (Written as asm so that the two registers stay distinct; the s_nop around each swap cover the
// wait states between vector ALU writes and a lane-permuting read/write of the same registers.)
__device__ __forceinline__ void swap16(float &a, float &b) {
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void swap32(float &a, float &b) {
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
// max of two numbers that are known not to be NaN: one v_max_f32 (fmaxf would first canonicalise
// both operands, which come out of an asm statement, with two more instructions)
__device__ __forceinline__ float max_no_nan(float a, float b) {
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float rowgroup_max(float x) {
    float a = x, b = x;
    swap16(a, b);
    a = b = max_no_nan(a, b);
    swap32(a, b);
    return fmaxf(a, b);
}
__device__ __forceinline__ float rowgroup_sum(float x) {
    float a = x, b = x;
    swap16(a, b);
    a = b = a + b;
    swap32(a, b);
    return a + b;
}

// 16-bit input value (bits in the low half of u) -> binary32, exact
template <bool BF16>
__device__ __forceinline__ float to_f32(uint32_t u) {
    if constexpr (BF16) return __builtin_bit_cast(float, u << 16);
    return (float)__builtin_bit_cast(_Float16, (uint16_t)u);
}

template <bool BF16>
__device__ __forceinline__ uint32_t pack2(float a, float b) {
    if constexpr (BF16) {
        // one v_cvt_pk_bf16_f32 (round to nearest even)
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        const f32x2 v = {a, b};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    } else {
        const uint32_t ua = __builtin_bit_cast(uint16_t, (_Float16)a);
        const uint32_t ub = __builtin_bit_cast(uint16_t, (_Float16)b);
        return ua | (ub << 16);
    }
}

// The INT8 MFMA accumulates onto kMagic = 0x4B400000 instead of 0: the INT32 result MAGIC + S,
// read as binary32, IS the number K + S with K = 1.5*2^23 (exact for |S| < 2^22; |S| <= 127*127*128
// here), so no int->float conversion instruction is needed.  -K*c is split exactly into two
// binary32 numbers kh + kl; then fma(bits, c, kh) = fl(c*S - kl) and adding (kl + offset) restores c*S.
constexpr int kMagic = 0x4B400000;
constexpr float kMagicF = 12582912.0f;

// One online-softmax step for one 16-query tile: biased scores s[t] (t<8: 16-key tiles of the
// 128-key step) -> P^ packed as the FP8 MFMA operand; updates m, l; returns alpha.
// c0/c1: de-quantisation constants of the two 64-key K blocks of the step; kh/kl: the exact split of -K*c.
// MASKED (causal diagonal or ragged tail): keys beyond `lim` are excluded.  The wavefront-uniform
// bounds t_lo <= t_hi say which 16-key tiles need no mask (t < t_lo), an element-wise mask
// (t_lo <= t < t_hi) or are invisible to every lane (t >= t_hi: no arithmetic at all, P^ = 0).
template <bool MASKED>
__device__ __forceinline__ float softmax_step(v4i (&s)[8], float c0, float c1, float kh0, float kh1, float kl0, float kl1, float log2_pr,
                                              float &m, float &l, v8i &pb, int key_base, int lim, int t_lo, int t_hi) {
    // step maximum on the integers of each 64-key K block (its scale is positive; the bias keeps order)
    int im0 = INT_MIN, im1 = INT_MIN;
    if constexpr (MASKED) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (t >= t_hi) continue;
            if (t >= t_lo) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (key_base + 16 * t + i > lim) s[t][i] = INT_MIN;
            }
            int &im = t < 4 ? im0 : im1;
            im = imax3(im, s[t][0], s[t][1]);
            im = imax3(im, s[t][2], s[t][3]);
        }
    } else {
        im0 = imax3(s[0][0], s[0][1], s[0][2]);
        im1 = imax3(s[4][0], s[4][1], s[4][2]);
        im0 = max(im0, s[0][3]);
        im1 = max(im1, s[4][3]);
#pragma unroll
        for (int t = 1; t < 4; ++t) {
            im0 = imax3(im0, s[t][0], s[t][1]);
            im0 = imax3(im0, s[t][2], s[t][3]);
            im1 = imax3(im1, s[t + 4][0], s[t + 4][1]);
            im1 = imax3(im1, s[t + 4][2], s[t + 4][3]);
        }
    }
    float mc0 = __builtin_fmaf(__builtin_bit_cast(float, im0), c0, kh0) + kl0;
    float mc1 = __builtin_fmaf(__builtin_bit_cast(float, im1), c1, kh1) + kl1;
    if constexpr (MASKED) {
        mc0 = im0 == INT_MIN ? -INFINITY : mc0;
        mc1 = im1 == INT_MIN ? -INFINITY : mc1;
    }
    const float mc = rowgroup_max(fmaxf(mc0, mc1));
    const float m_new = fmaxf(m, mc);
    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
    const float mo = log2_pr - m_new;  // P~ * P_r = 2^(x - m' + log2 P_r)
    const float mo0 = mo + kl0, mo1 = mo + kl1;
    float lsum0 = -0.0f, lsum1 = -0.0f;  // x + (-0) is x for every x: the first addition folds away
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        if constexpr (MASKED) {
            if (t >= t_hi) {
                pb[t] = 0;
                continue;
            }
        }
        const float cb = t < 4 ? c0 : c1, khb = t < 4 ? kh0 : kh1, mob = t < 4 ? mo0 : mo1;
        float p[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int sbits = s[t][i];  // (bit_cast needs a scalar object, not a vector element)
            p[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(__builtin_bit_cast(float, sbits), cb, khb) + mob);
        }
        if constexpr (MASKED) {
            if (t >= t_lo) {
#pragma unroll
                for (int i = 0; i < 4; ++i) p[i] = s[t][i] == INT_MIN ? 0.0f : p[i];
            }
        }
        lsum0 += p[0] + p[1];
        lsum1 += p[2] + p[3];
        int w;  // both halves are overwritten below: an opaque undefined seed saves the v_mov of a zero
        asm volatile("" : "=v"(w));
        w = __builtin_amdgcn_cvt_pk_fp8_f32(p[0], p[1], w, false);
        w = __builtin_amdgcn_cvt_pk_fp8_f32(p[2], p[3], w, true);
        pb[t] = w;
    }
    l = l * alpha + (lsum0 + lsum1);
    m = m_new;
    return alpha;
}

}  // namespace
}  // namespace sage
