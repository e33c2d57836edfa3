// Stage 1 of the SageAttention2++ 8+8 forward on gfx950: K smoothing, per-block
// INT8 quantisation of Q and K, per-channel FP8 (E4M3) quantisation of V.
//
// All kernels here are bandwidth bound (read 2 bytes, write 1 byte per element
// and tensor): every global access is a 16-byte load or a 8/16-byte store whose
// lanes cover whole rows, statistics are reduced in registers -> LDS -> a small
// partial buffer in a fixed order (no atomics), so results do not depend on
// scheduling.
//
// This translation unit must be compiled with -ffp-contract=off: each quantiser
// step (x - mean, a / range, range / a, x * r) is one correctly rounded binary32
// operation, which is what makes codes and scales reproducible bit for bit
// (paper Sec. 2.1 for the scales, Sec. 3 for the smoothing).
#include "sage_internal.h"

#include <algorithm>
#include <atomic>

namespace sage {
namespace {

template <bool BF16>
__device__ __forceinline__ float to_f32(uint32_t h16) {
    if constexpr (BF16) {
        return __builtin_bit_cast(float, h16 << 16);
    } else {
        return (float)__builtin_bit_cast(_Float16, (uint16_t)h16);
    }
}

template <bool BF16>
__device__ __forceinline__ void unpack8(const uint4 &u, float (&f)[8]) {
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = to_f32<BF16>(w[i] & 0xffffu);
        f[2 * i + 1] = to_f32<BF16>(w[i] >> 16);
    }
}

// ---------------------------------------------------------------------------
// Partial column statistics over chunks of kStatRows tokens.
//   IS_V = false: sum_n K[n][c] in double (smoothing mean, Sec. 3)
//   IS_V = true : max_n |V[n][c]|        (per-channel FP8 scale, Sec. 2.1)
// One workgroup of 256 threads per (chunk, batch*head); a thread owns 8 adjacent channels.
// Launched per tensor (grid (chunks, B*H)) or for K and V together (grid (chunks, B*H, 2)).
// ---------------------------------------------------------------------------
template <int D>
constexpr int colstats_smem_bytes() {
    return (256 / (D / 8)) * D * (int)sizeof(double);
}

template <bool BF16, int D, bool IS_V>
__device__ __forceinline__ void colstats_body(const uint16_t *__restrict__ X, Strides st, int H, int N, int chunks,
                                              double *__restrict__ sum_part, float *__restrict__ max_part,
                                              void *smem, int bh, int chunk) {
    constexpr int LPR = D / 8;     // lanes per row
    constexpr int RP = 256 / LPR;  // rows per pass
    using acc_t = typename std::conditional<IS_V, float, double>::type;
    acc_t(*sm)[D] = reinterpret_cast<acc_t(*)[D]>(smem);

    const int co = threadIdx.x % LPR, rr = threadIdx.x / LPR;
    const uint16_t *Xh = X + (bh / H) * st.b + (bh % H) * st.h;
    const int r0 = chunk * kStatRows;
    const int r1 = min(r0 + kStatRows, N);

    acc_t acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0;
    // four independent 16-byte loads in flight per thread (one per trip leaves the kernel bound by
    // memory latency); rows past the end contribute zeros, which change neither a sum nor a max of |.|
#ifndef SAGE_STAT_UNROLL
#define SAGE_STAT_UNROLL 4
#endif
    constexpr int UNROLL = SAGE_STAT_UNROLL;
    for (int rb = r0 + rr; rb < r1; rb += RP * UNROLL) {
        uint4 u[UNROLL];
#pragma unroll
        for (int k = 0; k < UNROLL; ++k) {
            const int r = rb + k * RP;
            u[k] = r < r1 ? *reinterpret_cast<const uint4 *>(Xh + r * st.n + co * 8) : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int k = 0; k < UNROLL; ++k) {
            float f[8];
            unpack8<BF16>(u[k], f);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if constexpr (IS_V) {
                    acc[j] = fmaxf(acc[j], fabsf(f[j]));
                } else {
                    acc[j] += (double)f[j];
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) sm[rr][co * 8 + j] = acc[j];
    __syncthreads();
    if (threadIdx.x < D) {
        acc_t a = sm[0][threadIdx.x];
        for (int i = 1; i < RP; ++i) {
            if constexpr (IS_V) {
                a = fmaxf(a, sm[i][threadIdx.x]);
            } else {
                a += sm[i][threadIdx.x];
            }
        }
        const size_t o = ((size_t)bh * chunks + chunk) * D + threadIdx.x;
        if constexpr (IS_V) {
            max_part[o] = a;
        } else {
            sum_part[o] = a;
        }
    }
}

template <bool BF16, int D, bool IS_V>
__global__ __launch_bounds__(256) void colstats_kernel(const uint16_t *__restrict__ X, Strides st, int H, int N,
                                                       int chunks, double *__restrict__ sum_part,
                                                       float *__restrict__ max_part) {
    __shared__ __attribute__((aligned(16))) unsigned char smem[colstats_smem_bytes<D>()];
    colstats_body<BF16, D, IS_V>(X, st, H, N, chunks, sum_part, max_part, smem, blockIdx.y, blockIdx.x);
}

// K sums (blockIdx.z == 0) and V maxima (blockIdx.z == 1) in one launch
template <bool BF16, int D>
__global__ __launch_bounds__(256) void colstats_kv_kernel(const uint16_t *__restrict__ K, Strides k_st,
                                                          const uint16_t *__restrict__ V, Strides v_st, int H, int N,
                                                          int chunks, double *__restrict__ sum_part,
                                                          float *__restrict__ max_part) {
    __shared__ __attribute__((aligned(16))) unsigned char smem[colstats_smem_bytes<D>()];
    if (blockIdx.z == 0)
        colstats_body<BF16, D, false>(K, k_st, H, N, chunks, sum_part, nullptr, smem, blockIdx.y, blockIdx.x);
    else
        colstats_body<BF16, D, true>(V, v_st, H, N, chunks, nullptr, max_part, smem, blockIdx.y, blockIdx.x);
}

// mean[c] = float(sum / N).  1024 threads: 1024/D threads share a channel, each adds every
// (1024/D)-th partial sum in chunk order, the shares are added in a fixed order through LDS
// (the loads of one thread are independent, so the loop is not a chain of memory latencies).
__device__ __forceinline__ void finalize_mean_body(const double *__restrict__ sum_part, int chunks, int N, int D,
                                                   float *__restrict__ mean, double *sm, int bh) {
    const int c = threadIdx.x % D, part = threadIdx.x / D, parts = 1024 / D;
    double s = 0.0;
    for (int i = part; i < chunks; i += parts) s += sum_part[((size_t)bh * chunks + i) * D + c];
    sm[threadIdx.x] = s;
    __syncthreads();
    if (part == 0) {
        for (int k = 1; k < parts; ++k) s += sm[k * D + c];
        mean[(size_t)bh * D + c] = (float)(s / (double)N);
    }
}

// delta_V[c] = a_c / V_r and the multiplier V_r / a_c (0 for an all-zero channel); same thread layout.
__device__ __forceinline__ void finalize_vscale_body(const float *__restrict__ max_part, int chunks, int D, float v_r,
                                                     float *__restrict__ v_scale, float *__restrict__ v_rcp,
                                                     float *sm, int bh) {
    const int c = threadIdx.x % D, part = threadIdx.x / D, parts = 1024 / D;
    float a = 0.0f;
    for (int i = part; i < chunks; i += parts) a = fmaxf(a, max_part[((size_t)bh * chunks + i) * D + c]);
    sm[threadIdx.x] = a;
    __syncthreads();
    if (part == 0) {
        for (int k = 1; k < parts; ++k) a = fmaxf(a, sm[k * D + c]);
        v_scale[(size_t)bh * D + c] = a / v_r;
        v_rcp[(size_t)bh * D + c] = a > 0.0f ? v_r / a : 0.0f;
    }
}

__global__ __launch_bounds__(1024) void finalize_mean_kernel(const double *__restrict__ sum_part, int chunks, int N,
                                                             int D, float *__restrict__ mean) {
    __shared__ double sm[1024];
    finalize_mean_body(sum_part, chunks, N, D, mean, sm, blockIdx.x);
}

__global__ __launch_bounds__(1024) void finalize_vscale_kernel(const float *__restrict__ max_part, int chunks, int D,
                                                               float v_r, float *__restrict__ v_scale,
                                                               float *__restrict__ v_rcp) {
    __shared__ float sm[1024];
    finalize_vscale_body(max_part, chunks, D, v_r, v_scale, v_rcp, sm, blockIdx.x);
}

// the K mean (blockIdx.y == 0) and the V scales (blockIdx.y == 1) in one launch
__global__ __launch_bounds__(1024) void finalize_kv_kernel(const double *__restrict__ sum_part,
                                                           const float *__restrict__ max_part, int chunks, int N, int D,
                                                           float v_r, float *__restrict__ mean,
                                                           float *__restrict__ v_scale, float *__restrict__ v_rcp) {
    __shared__ double sm[1024];
    if (blockIdx.y == 0)
        finalize_mean_body(sum_part, chunks, N, D, mean, sm, blockIdx.x);
    else
        finalize_vscale_body(max_part, chunks, D, v_r, v_scale, v_rcp, reinterpret_cast<float *>(sm), blockIdx.x);
}

// ---------------------------------------------------------------------------
// Per-block integer quantisation (Sec. 2.1): one workgroup per block of BLOCK
// tokens, the block lives in registers between the max pass and the code pass.
// QMAX = 127: INT8 codes; QMAX = 7: the INT4 codes of the 4+8 variant (one per
// byte).  SMOOTH = 0: no mean is subtracted; 1: `mean` holds one vector per
// head (K smoothing, Sec. 3); 2: one vector per head and block (Q smoothing of
// the 4+8 variant).  256 threads; wmax: four floats of LDS.
// ---------------------------------------------------------------------------
template <bool BF16, int D, int BLOCK, int SMOOTH, int QMAX>
__device__ __forceinline__ void quant_int8_body(const uint16_t *__restrict__ X, Strides st, int H,
                                                const float *__restrict__ mean, int8_t *__restrict__ codes,
                                                float *__restrict__ scale, int N, int nblk, float *wmax, int bh,
                                                int blk) {
    constexpr int LPR = D / 8;
    constexpr int RP = 256 / LPR;
    constexpr int ITER = BLOCK / RP;
    constexpr float kRange = (float)QMAX;
    static_assert(BLOCK % RP == 0, "block must be a multiple of the rows covered per pass");

    const int co = threadIdx.x % LPR, rr = threadIdx.x / LPR;
    const uint16_t *Xh = X + (bh / H) * st.b + (bh % H) * st.h;

    float mu[8];
    const size_t mrow = SMOOTH == 2 ? (size_t)bh * nblk + blk : (size_t)bh;
#pragma unroll
    for (int j = 0; j < 8; ++j) mu[j] = SMOOTH ? mean[mrow * D + co * 8 + j] : 0.0f;

    float x[ITER][8];
    float amax = 0.0f;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int r = blk * BLOCK + it * RP + rr;
        if (r < N) {
            const uint4 u = *reinterpret_cast<const uint4 *>(Xh + r * st.n + co * 8);
            unpack8<BF16>(u, x[it]);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if constexpr (SMOOTH != 0) x[it][j] = x[it][j] - mu[j];
                amax = fmaxf(amax, fabsf(x[it][j]));
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) x[it][j] = 0.0f;
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = amax;
    __syncthreads();
    const float a = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    const float rcp = a > 0.0f ? kRange / a : 0.0f;
    if (threadIdx.x == 0) scale[(size_t)bh * nblk + blk] = a / kRange;

#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int r = blk * BLOCK + it * RP + rr;
        if (r < N) {
            uint32_t w[2] = {0u, 0u};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = (int)__builtin_rintf(x[it][j] * rcp);
                w[j >> 2] |= ((uint32_t)c & 0xffu) << (8 * (j & 3));
            }
            *reinterpret_cast<uint2 *>(codes + ((size_t)bh * N + r) * D + co * 8) = make_uint2(w[0], w[1]);
        }
    }
}

// ---------------------------------------------------------------------------
// 4+8 variant: what smoothing of Q subtracts (Sec. 3 names the step; reading: the mean of each Q block,
// per channel, over the block's valid tokens).  mean[bh][blk][c] = float(sum_r Q[r][c] / rows), the sum in
// double (exact for 16-bit inputs, so the order of the additions does not matter).  One workgroup of 256
// threads per Q block; sm: RP x D doubles.
// ---------------------------------------------------------------------------
template <bool BF16, int D>
__global__ __launch_bounds__(256) void block_mean_kernel(const uint16_t *__restrict__ Q, Strides st, int H, int N,
                                                         int nblk, float *__restrict__ mean) {
    constexpr int LPR = D / 8;
    constexpr int RP = 256 / LPR;
    __shared__ double sm[RP][D];
    const int bh = blockIdx.y, blk = blockIdx.x;
    const int co = threadIdx.x % LPR, rr = threadIdx.x / LPR;
    const uint16_t *Qh = Q + (bh / H) * st.b + (bh % H) * st.h;
    const int r0 = blk * kBQ, r1 = min(r0 + kBQ, N);
    double acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.0;
    for (int r = r0 + rr; r < r1; r += RP) {
        float f[8];
        unpack8<BF16>(*reinterpret_cast<const uint4 *>(Qh + r * st.n + co * 8), f);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += (double)f[j];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) sm[rr][co * 8 + j] = acc[j];
    __syncthreads();
    if (threadIdx.x < D) {
        double a = sm[0][threadIdx.x];
        for (int i = 1; i < RP; ++i) a += sm[i][threadIdx.x];
        mean[((size_t)bh * nblk + blk) * D + threadIdx.x] = (float)(a / (double)(r1 - r0));
    }
}

// ---------------------------------------------------------------------------
// 4+8 variant: the score correction.  With Q' = Q - qbar_i on Q block i, Q K'^T = Q' K'^T + qbar_i K'^T; the
// second term, dS[i][n] = sum_c qbar[i][c] * K'[n][c] with the smoothed UNquantised keys K' = K - mu_K, is
// computed here in FP32 and stored in the units of the softmax exponent (times sm_scale * log2 e), in the key
// order in which a lane of the attention kernel holds its scores: [B*Hq][nQ][nT][128] floats, position
// 32*g + 4*t + i of a tile = key 16*t + 4*g + i (t < 8, g < 4, i < 4).  Keys >= Nk hold 0.
// One workgroup of 128 threads per 128-key tile and K/V head; a thread owns one key and keeps its K' row in
// registers; the block means of 16 Q blocks at a time are staged in LDS and read as broadcasts.
// Causal launches skip the Q blocks that see no key of the tile.
// ---------------------------------------------------------------------------
template <bool BF16, int D>
__global__ __launch_bounds__(128) void delta_s_kernel(const uint16_t *__restrict__ K, Strides k_st, int Hkv,
                                                      const float *__restrict__ k_mean,
                                                      const float *__restrict__ q_mean, float *__restrict__ dsx,
                                                      int Hq, int Nq, int Nk, int nQ, int nT, float sm_log2e,
                                                      int causal) {
    constexpr int QB = 32;  // Q blocks per LDS stage
    __shared__ __attribute__((aligned(16))) float qm[QB][D];
    const int T = blockIdx.x, bhk = blockIdx.y;
    const int group = Hq / Hkv;
    const int n = T * 128 + threadIdx.x;
    float kp[D];
    {
        const uint16_t *Kh = K + (bhk / Hkv) * k_st.b + (bhk % Hkv) * k_st.h;
#pragma unroll
        for (int c8 = 0; c8 < D / 8; ++c8) {
            float f[8];
            if (n < Nk) {
                unpack8<BF16>(*reinterpret_cast<const uint4 *>(Kh + n * k_st.n + c8 * 8), f);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) f[j] = 0.0f;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) kp[c8 * 8 + j] = n < Nk ? f[j] - k_mean[(size_t)bhk * D + c8 * 8 + j] : 0.0f;
        }
    }
    // position of this key inside its tile in the attention kernel's lane order
    const int kt = threadIdx.x;
    const int pos = 32 * ((kt >> 2) & 3) + 4 * (kt >> 4) + (kt & 3);
    // causal (mask aligned to the end of both sequences): Q block i sees key n iff n <= i*kBQ + kBQ-1 + Nk - Nq
    int i_first = 0;
    if (causal) i_first = max(0, (T * 128 - (Nk - Nq)) / kBQ);
    for (int hq = 0; hq < group; ++hq) {
        const int bhq = (bhk / Hkv) * Hq + (bhk % Hkv) * group + hq;
        for (int i0 = i_first - i_first % QB; i0 < nQ; i0 += QB) {
            __syncthreads();
            for (int e = threadIdx.x; e < QB * D / 4; e += 128) {
                const int i = i0 + e / (D / 4);
                const float4 v = i < nQ ? *reinterpret_cast<const float4 *>(q_mean + ((size_t)bhq * nQ + i) * D + 4 * (e % (D / 4)))
                                        : make_float4(0.f, 0.f, 0.f, 0.f);
                *reinterpret_cast<float4 *>(&qm[e / (D / 4)][4 * (e % (D / 4))]) = v;
            }
            __syncthreads();
            // one Q block at a time (a rolled loop: the key's row stays in registers, the block's means are
            // broadcast reads at constant offsets), four partial sums
#pragma unroll 1
            for (int i = 0; i < QB; ++i) {
                if (i0 + i >= nQ) break;
                float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
#pragma unroll
                for (int c4 = 0; c4 < D / 4; ++c4) {
                    const float4 m = *reinterpret_cast<const float4 *>(&qm[i][4 * c4]);
                    a0 = __builtin_fmaf(m.x, kp[4 * c4], a0);
                    a1 = __builtin_fmaf(m.y, kp[4 * c4 + 1], a1);
                    a2 = __builtin_fmaf(m.z, kp[4 * c4 + 2], a2);
                    a3 = __builtin_fmaf(m.w, kp[4 * c4 + 3], a3);
                }
                dsx[(((size_t)bhq * nQ + i0 + i) * nT + T) * 128 + pos] = ((a0 + a1) + (a2 + a3)) * sm_log2e;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Per-channel FP8 quantisation of V into the transposed, key-permuted tile
// layout the attention kernel consumes: [B*H][tile][D][128] bytes, byte
// 64*(t>>2) + 16*g + 4*(t&3) + i of a row = key 16*t + 4*g + i of the tile.  A thread converts
// 4 consecutive keys x 8 channels, so the four keys of one channel pack into
// one dword; the tile is transposed through LDS and leaves as one contiguous
// D*128-byte burst.  256 threads; tile: D*32 dwords of LDS.
// ---------------------------------------------------------------------------
template <bool BF16, int D>
__device__ __forceinline__ void quant_v_body(const uint16_t *__restrict__ V, Strides st, int H,
                                             const float *__restrict__ v_rcp, uint8_t *__restrict__ Vt, int N, int nT,
                                             uint32_t *tile, int bh, int T) {
    constexpr int LPR = D / 8;
    constexpr int UPT = 32 * LPR / 256;  // (key quad, channel octet) units per thread

    const uint16_t *Vh = V + (bh / H) * st.b + (bh % H) * st.h;
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
        const int u = threadIdx.x + 256 * k;
        const int co = u % LPR, kq = u / LPR;
        const int t = kq >> 2, g = kq & 3;
        float rc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) rc[j] = v_rcp[(size_t)bh * D + co * 8 + j];
        float y[4][8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = T * 128 + kq * 4 + i;
            if (r < N) {
                const uint4 raw = *reinterpret_cast<const uint4 *>(Vh + r * st.n + co * 8);
                unpack8<BF16>(raw, y[i]);
#pragma unroll
                for (int j = 0; j < 8; ++j) y[i][j] = y[i][j] * rc[j];
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) y[i][j] = 0.0f;
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            int w = 0;
            w = __builtin_amdgcn_cvt_pk_fp8_f32(y[0][j], y[1][j], w, false);
            w = __builtin_amdgcn_cvt_pk_fp8_f32(y[2][j], y[3][j], w, true);
            tile[(co * 8 + j) * 32 + (t >> 2) * 16 + g * 4 + (t & 3)] = (uint32_t)w;
        }
    }
    __syncthreads();
    uint4 *dst = reinterpret_cast<uint4 *>(Vt + ((size_t)bh * nT + T) * D * 128);
    const uint4 *src = reinterpret_cast<const uint4 *>(tile);
#pragma unroll
    for (int k = 0; k < D / 32; ++k) dst[threadIdx.x + 256 * k] = src[threadIdx.x + 256 * k];
}

// grid (blocks, B*H)
template <bool BF16, int D, int BLOCK, int SMOOTH, int QMAX>
__global__ __launch_bounds__(256) void quant_int8_kernel(const uint16_t *__restrict__ X, Strides st, int H,
                                                         const float *__restrict__ mean, int8_t *__restrict__ codes,
                                                         float *__restrict__ scale, int N, int nblk) {
    __shared__ float wmax[4];
    quant_int8_body<BF16, D, BLOCK, SMOOTH, QMAX>(X, st, H, mean, codes, scale, N, nblk, wmax, blockIdx.y, blockIdx.x);
}

// grid (tiles, B*H)
template <bool BF16, int D>
__global__ __launch_bounds__(256) void quant_v_kernel(const uint16_t *__restrict__ V, Strides st, int H,
                                                      const float *__restrict__ v_rcp, uint8_t *__restrict__ Vt, int N,
                                                      int nT) {
    __shared__ uint32_t tile[D * 32];
    quant_v_body<BF16, D>(V, st, H, v_rcp, Vt, N, nT, tile, blockIdx.y, blockIdx.x);
}

// K blocks (blockIdx.x < nK) and V tiles (the rest) in one launch: grid (nK + nT, B*H)
template <bool BF16, int D, int QMAX>
__global__ __launch_bounds__(256) void quant_kv_kernel(const uint16_t *__restrict__ K, Strides k_st,
                                                       const float *__restrict__ mean, int8_t *__restrict__ k_codes,
                                                       float *__restrict__ k_scale, int nK,
                                                       const uint16_t *__restrict__ V, Strides v_st,
                                                       const float *__restrict__ v_rcp, uint8_t *__restrict__ Vt, int nT,
                                                       int H, int N) {
    __shared__ uint32_t tile[D * 32];
    const int x = blockIdx.x;  // (workgroup-uniform branch)
    if (x < nK)
        quant_int8_body<BF16, D, kBK, 1, QMAX>(K, k_st, H, mean, k_codes, k_scale, N, nK,
                                               reinterpret_cast<float *>(tile), blockIdx.y, x);
    else
        quant_v_body<BF16, D>(V, v_st, H, v_rcp, Vt, N, nT, tile, blockIdx.y, x - nK);
}

// ---------------------------------------------------------------------------
// K and V quantised with ONE read of each tensor (smoothing of Sec. 3, scales of Sec. 2.1; the same binary32
// steps and the same outputs as the three launches above).  The codes of a token need a statistic of its whole
// head (the K mean, the V maxima), so a token must wait somewhere between the statistics and the codes: here it
// waits in registers.  A workgroup of 256 threads loads kResidentBytes of one (head, tensor) — 256 tokens at
// d = 128, 512 at d = 64 — keeps them as 16 packed uint4 per thread, publishes its partial column statistic,
// and then waits for the partials of all G = ceil(N / tokens) workgroups of the (head, tensor).  A partial is
// its own "there" flag: the partial buffers are zero at launch (the host enqueues zero_words_kernel in front)
// and a value is stored with a bit pattern that is never all zero (+0.0 goes out as -0.0, which adds and
// compares like it), each with one write-through store that is atomic for its 4 or 8 bytes.  Thread t first
// polls element 0 of partial t, sleeping between polls, for at most `wait_ticks` ticks of the constant 100 MHz
// clock; once those are there every workgroup loads all G x d values (again until none is zero) and adds them
// itself, in index order, so all workgroups of a head see the same statistic (workgroup 0 of the group also
// writes it out: mean, or delta_V).  No workgroup waits for another one to do work on its behalf: the only chain
// is "partial stored -> partial seen".  A workgroup whose wait runs out (its partners not resident: another
// kernel holds the CUs, or a dispatch order other than by index) computes the head's statistic itself from
// global memory and goes on, so every wavefront leaves the kernel whatever the others do.  (The two questions of
// a poll -- is a partial missing, has my time run out -- are two workgroup-wide reductions: __syncthreads_or only
// tells whether any thread's value is non-zero.)
// Workgroup ids are group-major, and the hardware dispatches them in id order, so the G partners are resident
// together as long as G does not exceed the workgroups the chip holds; since every workgroup reads G partials the
// host takes this path only up to kResidentMaxGroup.  Grid: B*H*2*G; group 2*bh is K of head bh, 2*bh + 1 is V.
// ---------------------------------------------------------------------------
constexpr int kResidentBytes = 65536;
constexpr int kResidentMaxGroup = 128;       // largest group the shape-based choice takes (every workgroup reads G partials:
                                             // measured faster than the three launches up to here, 17-26 % slower at 192-256)
constexpr int kResidentHardMaxGroup = 256;   // largest group a forced choice may take (thread t polls partner t)
constexpr long long kResidentWaitTicks = 50000;  // 0.5 ms
inline int resident_group_size(int N, int d) { return cdiv(N, kResidentBytes / (2 * d)); }

__global__ __launch_bounds__(256) void zero_words_kernel(uint4 *w, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) w[i] = make_uint4(0u, 0u, 0u, 0u);
}


// The packed rows stay packed between the passes over them: without this the compiler keeps the unpacked
// floats of one pass alive for the next (twice the registers of the packed rows).
__device__ __forceinline__ void keep_packed(uint4 (&raw)[16]) {
#pragma unroll
    for (int it = 0; it < 16; ++it) asm volatile("" : "+v"(raw[it].x), "+v"(raw[it].y), "+v"(raw[it].z), "+v"(raw[it].w));
}

// What the workgroups of a group tell each other goes through device-scope relaxed atomic accesses: stores
// that write through to memory and loads that do not take a line another XCD's L2 may hold stale.  No cache is
// written back or invalidated as a whole (a device-scope release fence does that, per wavefront, and with a
// few thousand workgroups writing codes at the same time it costs ten times the kernel's own work).
template <class T>
__device__ __forceinline__ void put_shared(T *p, T v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <class T>
__device__ __forceinline__ T get_shared(const T *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The bit pattern a partial is stored with (never all zero) and read back from.
__device__ __forceinline__ unsigned long long tag_bits(double a) {
    const unsigned long long b = __builtin_bit_cast(unsigned long long, a);
    return b ? b : 0x8000000000000000ull;
}
__device__ __forceinline__ unsigned tag_bits(float a) {
    const unsigned b = __builtin_bit_cast(unsigned, a);
    return b ? b : 0x80000000u;
}

// Wait until element 0 of each of the G partials (rows of d words) is there.  True when they are, false when
// the wait ran out (workgroup-uniform).  Contains a barrier in every case.
template <class W>
__device__ __forceinline__ bool resident_wait(const W *rows, int d, int G, long long wait_ticks, long long t0) {
    if (wait_ticks < 0) {
        __syncthreads();
        return false;
    }
    for (;;) {
        const bool missing = (int)threadIdx.x < G && get_shared(&rows[(size_t)threadIdx.x * d]) == 0;  // partner t
        const bool late = wall_clock64() - t0 >= wait_ticks;                                          // my time is up
        // (__syncthreads_or tells WHETHER any thread's value is non-zero, not which bits: one call per question)
        if (!__syncthreads_or(missing)) return true;
        if (__syncthreads_or(late)) return false;
        __builtin_amdgcn_s_sleep(8);
    }
}

template <bool BF16, int D, int QMAX>
__global__ __launch_bounds__(256, 4) void quant_kv_resident_kernel(
    const uint16_t *__restrict__ K, Strides k_st, const uint16_t *__restrict__ V, Strides v_st, int H, int N, int G,
    double *k_sum_part, float *v_max_part, float *k_mean, float *v_scale, float v_r,
    int8_t *__restrict__ k_codes, float *__restrict__ k_scale, int nK, uint8_t *__restrict__ Vt, int nT,
    long long wait_ticks) {
    constexpr int C = kResidentBytes / (2 * D);  // tokens of a workgroup
    constexpr int LPR = D / 8;                   // lanes per row
    constexpr int RP = 256 / LPR;                // rows per pass of the workgroup
    constexpr int NU = 16;                       // uint4 per thread
    static_assert(C * LPR == NU * 256, "a workgroup's chunk is 16 uint4 per thread");
    __shared__ __attribute__((aligned(16))) unsigned char smem[16384];
    __shared__ float stat[D];      // the head's mean (K) or V_r / max (V)
    __shared__ float wmax[4][8];   // per wavefront and K block: max |K'|

    const int grp = blockIdx.x / G, part = blockIdx.x % G;
    const int bh = grp >> 1;
    const bool is_v = grp & 1;  // (workgroup-uniform)
    const int tid = threadIdx.x;
    const int co = tid % LPR, rr = tid / LPR;
    const int row0 = part * C;
    unsigned long long *k_bits = reinterpret_cast<unsigned long long *>(k_sum_part);
    unsigned *v_bits = reinterpret_cast<unsigned *>(v_max_part);
    uint4 raw[NU];

    if (!is_v) {
        // ---- K: thread owns channels co*8.. of rows row0 + it*RP + rr ----
        const uint16_t *Kh = K + (bh / H) * k_st.b + (bh % H) * k_st.h;
        // (all sixteen loads are issued before the first is waited for: rows past the end are loaded from the
        // head's last row and zeroed afterwards — a branch around a load would make each load wait for itself)
        const int nrow = min(max((N - row0 - rr + RP - 1) / RP, 0), NU);  // this thread's rows that exist
        {
            const uint16_t *last = Kh + (int64_t)(N - 1) * k_st.n + co * 8;
            const uint16_t *p = Kh + (int64_t)(row0 + rr) * k_st.n + co * 8;
            const int64_t step = (int64_t)RP * k_st.n;
#pragma unroll
            for (int it = 0; it < NU; ++it) raw[it] = *reinterpret_cast<const uint4 *>(it < nrow ? p + it * step : last);
        }
#pragma unroll
        for (int it = 0; it < NU; ++it)
            if (it >= nrow) raw[it] = make_uint4(0u, 0u, 0u, 0u);
        double(*smd)[D] = reinterpret_cast<double(*)[D]>(smem);
        {
            double acc[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = 0.0;
#pragma unroll
            for (int it = 0; it < NU; ++it) {
                float f[8];
                unpack8<BF16>(raw[it], f);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] += (double)f[j];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) smd[rr][co * 8 + j] = acc[j];
        }
        __syncthreads();
        if (tid < D) {
            double a = smd[0][tid];
            for (int i = 1; i < RP; ++i) a += smd[i][tid];
            put_shared(&k_bits[((size_t)bh * G + part) * D + tid], tag_bits(a));
        }
        const long long t0 = wall_clock64();
        bool there = resident_wait(k_bits + (size_t)bh * G * D, D, G, wait_ticks, t0);
        if (there) {
            // the G partial sums in index order, 256 / D threads per channel (eight loads in flight: each is a
            // round trip to memory); repeated in the rare case that a word of a partial lags behind its element 0
            const int c = tid % D, share = tid / D;
            constexpr int SHARES = 256 / D;
            double s;
            for (;;) {
                s = 0.0;
                int v = 0;
                for (int i0 = share; i0 < G; i0 += 8 * SHARES) {
                    unsigned long long t[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        t[u] = get_shared(&k_bits[((size_t)bh * G + min(i0 + u * SHARES, G - 1)) * D + c]);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        if (t[u] == 0) v = 1;
                        if (i0 + u * SHARES < G) s += __builtin_bit_cast(double, t[u]);
                    }
                }
                const bool late = wall_clock64() - t0 >= wait_ticks;
                if (!__syncthreads_or(v)) break;
                if (__syncthreads_or(late)) {
                    there = false;
                    break;
                }
                __builtin_amdgcn_s_sleep(8);
            }
            if (there) {
                double *sd = reinterpret_cast<double *>(smem);
                sd[tid] = s;
                __syncthreads();
                if (share == 0) {
                    for (int k = 1; k < SHARES; ++k) s += sd[k * D + c];
                    const float mu = (float)(s / (double)N);
                    if (part == 0) k_mean[(size_t)bh * D + c] = mu;
                    stat[c] = mu;
                }
            }
        }
        if (!there) {
            // alone: the column sums of the whole head, from global memory
            double acc[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = 0.0;
#pragma unroll 1
            for (int r = rr; r < N; r += RP) {
                float f[8];
                unpack8<BF16>(*reinterpret_cast<const uint4 *>(Kh + r * k_st.n + co * 8), f);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] += (double)f[j];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) smd[rr][co * 8 + j] = acc[j];
            __syncthreads();
            if (tid < D) {
                double a = smd[0][tid];
                for (int i = 1; i < RP; ++i) a += smd[i][tid];
                const float mu = (float)(a / (double)N);
                if (part == 0) k_mean[(size_t)bh * D + tid] = mu;
                stat[tid] = mu;
            }
        }
        __syncthreads();

        // ---- codes: the quantiser of quant_int8_body on the resident rows, one K block after the other; the
        // smoothed values of a block stay in registers between its maximum and its codes ----
        constexpr int NB = C / kBK;    // K blocks of the chunk
        constexpr int IPB = kBK / RP;  // passes per block
        constexpr float kRange = (float)QMAX;
        float mu[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) mu[j] = stat[co * 8 + j];
        keep_packed(raw);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int blk = part * NB + b;  // (workgroup-uniform)
            if (blk >= nK) break;
            float x[IPB][8];
            float a = 0.0f;
#pragma unroll
            for (int i = 0; i < IPB; ++i) {
                float f[8];
                unpack8<BF16>(raw[b * IPB + i], f);
#pragma unroll
                for (int j = 0; j < 8; ++j) x[i][j] = f[j] - mu[j];
                if (b * IPB + i < nrow) {  // rows past the end do not count
#pragma unroll
                    for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(x[i][j]));
                }
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) a = fmaxf(a, __shfl_xor(a, off));
            if ((tid & 63) == 0) wmax[tid >> 6][b] = a;
            __syncthreads();  // (every block has its own column of wmax: one barrier per block)
            a = fmaxf(fmaxf(wmax[0][b], wmax[1][b]), fmaxf(wmax[2][b], wmax[3][b]));
            const float rcp = a > 0.0f ? kRange / a : 0.0f;
            if (tid == 0) k_scale[(size_t)bh * nK + blk] = a / kRange;
#pragma unroll
            for (int i = 0; i < IPB; ++i) {
                const int it = b * IPB + i;
                const int r = row0 + it * RP + rr;
                if (it < nrow) {
                    // rint(y) for |y| <= 127 as the low byte of fl(y + 1.5 * 2^23): the addition rounds y to the
                    // nearest integer, ties to even, and the sum's bit pattern is 0x4B400000 + that integer
                    uint32_t cb[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) cb[j] = __builtin_bit_cast(uint32_t, x[i][j] * rcp + 12582912.0f);
                    uint32_t w[2];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const uint32_t lo = __builtin_amdgcn_perm(cb[4 * h + 1], cb[4 * h], 0x0c0c0400u);
                        const uint32_t hi = __builtin_amdgcn_perm(cb[4 * h + 3], cb[4 * h + 2], 0x0c0c0400u);
                        w[h] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                    }
                    *reinterpret_cast<uint2 *>(k_codes + ((size_t)bh * N + r) * D + co * 8) = make_uint2(w[0], w[1]);
                }
            }
        }
    } else {
        // ---- V: per 128-key tile a thread owns UPT units of 4 consecutive keys x 8 channels (quant_v_body) ----
        constexpr int UPT = 32 * LPR / 256;
        constexpr int TILES = C / kW;
        static_assert(TILES * UPT * 4 == NU, "a workgroup's chunk is 16 uint4 per thread");
        const uint16_t *Vh = V + (bh / H) * v_st.b + (bh % H) * v_st.h;
        // this thread's rows are row0 + (tid / LPR) * 4 + (kW / UPT) * (q >> 2) + (q & 3), q = 0 .. 15
        uint32_t exists = 0u;
        {
            const uint16_t *last = Vh + (int64_t)(N - 1) * v_st.n + co * 8;
            const int rbase = row0 + rr * 4;
            const uint16_t *p = Vh + (int64_t)rbase * v_st.n + co * 8;
#pragma unroll
            for (int q = 0; q < NU; ++q) {
                const int dr = (kW / UPT) * (q >> 2) + (q & 3);
                const bool ok = rbase + dr < N;
                exists |= (ok ? 1u : 0u) << q;
                raw[q] = *reinterpret_cast<const uint4 *>(ok ? p + dr * v_st.n : last);
            }
        }
#pragma unroll
        for (int q = 0; q < NU; ++q)
            if (!((exists >> q) & 1u)) raw[q] = make_uint4(0u, 0u, 0u, 0u);
        float(*smf)[D] = reinterpret_cast<float(*)[D]>(smem);
        {
            float acc[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
#pragma unroll
            for (int it = 0; it < NU; ++it) {
                float f[8];
                unpack8<BF16>(raw[it], f);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = fmaxf(acc[j], fabsf(f[j]));
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) smf[rr][co * 8 + j] = acc[j];
        }
        __syncthreads();
        if (tid < D) {
            float a = smf[0][tid];
            for (int i = 1; i < RP; ++i) a = fmaxf(a, smf[i][tid]);
            put_shared(&v_bits[((size_t)bh * G + part) * D + tid], tag_bits(a));
        }
        const long long t0 = wall_clock64();
        bool there = resident_wait(v_bits + (size_t)bh * G * D, D, G, wait_ticks, t0);
        if (there) {
            const int c = tid % D, share = tid / D;
            constexpr int SHARES = 256 / D;
            float a;
            for (;;) {
                a = 0.0f;
                int v = 0;
                for (int i0 = share; i0 < G; i0 += 16 * SHARES) {
                    unsigned t[16];
#pragma unroll
                    for (int u = 0; u < 16; ++u)
                        t[u] = get_shared(&v_bits[((size_t)bh * G + min(i0 + u * SHARES, G - 1)) * D + c]);
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        if (t[u] == 0u) v = 1;
                        a = fmaxf(a, fabsf(__builtin_bit_cast(float, t[u])));  // (a partial taken twice does not change a maximum)
                    }
                }
                const bool late = wall_clock64() - t0 >= wait_ticks;
                if (!__syncthreads_or(v)) break;
                if (__syncthreads_or(late)) {
                    there = false;
                    break;
                }
                __builtin_amdgcn_s_sleep(8);
            }
            if (there) {
                float *sf = reinterpret_cast<float *>(smem);
                sf[tid] = a;
                __syncthreads();
                if (share == 0) {
                    for (int k = 1; k < SHARES; ++k) a = fmaxf(a, sf[k * D + c]);
                    if (part == 0) v_scale[(size_t)bh * D + c] = a / v_r;
                    stat[c] = a > 0.0f ? v_r / a : 0.0f;
                }
            }
        }
        if (!there) {
            float acc[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
#pragma unroll 1
            for (int r = rr; r < N; r += RP) {
                float f[8];
                unpack8<BF16>(*reinterpret_cast<const uint4 *>(Vh + r * v_st.n + co * 8), f);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = fmaxf(acc[j], fabsf(f[j]));
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) smf[rr][co * 8 + j] = acc[j];
            __syncthreads();
            if (tid < D) {
                float a = smf[0][tid];
                for (int i = 1; i < RP; ++i) a = fmaxf(a, smf[i][tid]);
                if (part == 0) v_scale[(size_t)bh * D + tid] = a / v_r;
                stat[tid] = a > 0.0f ? v_r / a : 0.0f;
            }
        }
        __syncthreads();

        float rc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) rc[j] = stat[co * 8 + j];
        keep_packed(raw);
        uint32_t *tile = reinterpret_cast<uint32_t *>(smem);  // D * 32 dwords
#pragma unroll
        for (int tl = 0; tl < TILES; ++tl) {
            const int T = part * TILES + tl;  // (workgroup-uniform)
            if (T >= nT) break;
#pragma unroll
            for (int k = 0; k < UPT; ++k) {
                const int kq = (tid + 256 * k) / LPR;
                const int t = kq >> 2, g = kq & 3;
                // two channels (one packed dword of each of the four keys) at a time; rows >= N hold zeros
#pragma unroll
                for (int j2 = 0; j2 < 4; ++j2) {
                    float y[4][2];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint4 &u = raw[(tl * UPT + k) * 4 + i];
                        const uint32_t w16 = j2 == 0 ? u.x : j2 == 1 ? u.y : j2 == 2 ? u.z : u.w;
                        y[i][0] = to_f32<BF16>(w16 & 0xffffu) * rc[2 * j2];
                        y[i][1] = to_f32<BF16>(w16 >> 16) * rc[2 * j2 + 1];
                    }
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int j = 2 * j2 + e;
                        int w = 0;
                        w = __builtin_amdgcn_cvt_pk_fp8_f32(y[0][e], y[1][e], w, false);
                        w = __builtin_amdgcn_cvt_pk_fp8_f32(y[2][e], y[3][e], w, true);
                        tile[(co * 8 + j) * 32 + (t >> 2) * 16 + g * 4 + (t & 3)] = (uint32_t)w;
                    }
                }
            }
            __syncthreads();
            uint4 *dst = reinterpret_cast<uint4 *>(Vt + ((size_t)bh * nT + T) * D * 128);
            const uint4 *src = reinterpret_cast<const uint4 *>(tile);
#pragma unroll
            for (int k = 0; k < D / 32; ++k) dst[tid + 256 * k] = src[tid + 256 * k];
            __syncthreads();
        }
    }
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

template <bool BF16, int D>
hipError_t quant_q_impl(const uint16_t *q, Strides st, int8_t *q_i8, float *q_scale, int BH, int H, int N,
                        hipStream_t stream) {
    const int nQ = cdiv(N, kBQ);
    quant_int8_kernel<BF16, D, kBQ, 0, 127><<<dim3(nQ, BH), 256, 0, stream>>>(q, st, H, nullptr, q_i8, q_scale, N, nQ);
    return hipGetLastError();
}

template <bool BF16, int D>
hipError_t quant_k_impl(const uint16_t *k, Strides st, int8_t *k_i8, float *k_scale, float *k_mean, int BH, int H,
                        int N, hipStream_t stream, const QuantScratch &ws) {
    const int chunks = cdiv(N, kStatRows);
    const int nK = cdiv(N, kBK);
    colstats_kernel<BF16, D, false><<<dim3(chunks, BH), 256, 0, stream>>>(k, st, H, N, chunks, ws.k_sum_part, nullptr);
    finalize_mean_kernel<<<BH, 1024, 0, stream>>>(ws.k_sum_part, chunks, N, D, k_mean);
    // K right after its statistics pass: its second read can still be served by the last-level cache
    quant_int8_kernel<BF16, D, kBK, 1, 127><<<dim3(nK, BH), 256, 0, stream>>>(k, st, H, k_mean, k_i8, k_scale, N, nK);
    return hipGetLastError();
}

template <bool BF16, int D>
hipError_t quant_v_impl(const uint16_t *v, Strides st, uint8_t *v_fp8, float *v_scale, float v_r, int BH, int H,
                        int N, hipStream_t stream, const QuantScratch &ws) {
    const int chunks = cdiv(N, kStatRows);
    const int nT = cdiv(N, kW);
    colstats_kernel<BF16, D, true><<<dim3(chunks, BH), 256, 0, stream>>>(v, st, H, N, chunks, nullptr, ws.v_max_part);
    finalize_vscale_kernel<<<BH, 1024, 0, stream>>>(ws.v_max_part, chunks, D, v_r, v_scale, ws.v_rcp);
    quant_v_kernel<BF16, D><<<dim3(nT, BH), 256, 0, stream>>>(v, st, H, ws.v_rcp, v_fp8, N, nT);
    return hipGetLastError();
}

// K and V of one shape in three launches instead of six (same kernels' bodies, same results)
template <bool BF16, int D, int QMAX>
hipError_t quant_kv_impl(const uint16_t *k, Strides k_st, const uint16_t *v, Strides v_st, int8_t *k_i8, float *k_scale,
                         float *k_mean, uint8_t *v_fp8, float *v_scale, float v_r, int BH, int H, int N,
                         hipStream_t stream, const QuantScratch &ws) {
    const int chunks = cdiv(N, kStatRows);
    const int nK = cdiv(N, kBK), nT = cdiv(N, kW);
    colstats_kv_kernel<BF16, D><<<dim3(chunks, BH, 2), 256, 0, stream>>>(k, k_st, v, v_st, H, N, chunks, ws.k_sum_part,
                                                                         ws.v_max_part);
    finalize_kv_kernel<<<dim3(BH, 2), 1024, 0, stream>>>(ws.k_sum_part, ws.v_max_part, chunks, N, D, v_r, k_mean,
                                                         v_scale, ws.v_rcp);
    quant_kv_kernel<BF16, D, QMAX><<<dim3(nK + nT, BH), 256, 0, stream>>>(k, k_st, k_mean, k_i8, k_scale, nK, v, v_st,
                                                                          ws.v_rcp, v_fp8, nT, H, N);
    return hipGetLastError();
}

// The same outputs from one read of K and V (quant_kv_resident_kernel); the caller has checked that the
// group size fits.
template <bool BF16, int D, int QMAX>
hipError_t quant_kv_resident_impl(const uint16_t *k, Strides k_st, const uint16_t *v, Strides v_st, int8_t *k_i8,
                                  float *k_scale, float *k_mean, uint8_t *v_fp8, float *v_scale, float v_r, int BH,
                                  int H, int N, hipStream_t stream, const QuantScratch &ws, long long wait_ticks) {
    const int G = resident_group_size(N, D);
    const int nK = cdiv(N, kBK), nT = cdiv(N, kW);
    // both partial buffers, which lie back to back (each a multiple of 256 bytes)
    const size_t span = reinterpret_cast<char *>(ws.v_rcp) - reinterpret_cast<char *>(ws.k_sum_part);
    const int words = (int)(span / 16);
    zero_words_kernel<<<cdiv(words, 256), 256, 0, stream>>>(reinterpret_cast<uint4 *>(ws.k_sum_part), words);
    quant_kv_resident_kernel<BF16, D, QMAX><<<BH * 2 * G, 256, 0, stream>>>(
        k, k_st, v, v_st, H, N, G, ws.k_sum_part, ws.v_max_part, k_mean, v_scale, v_r, k_i8, k_scale,
        nK, v_fp8, nT, wait_ticks);
    return hipGetLastError();
}

// 4+8 variant, Q side: block means, and (stand-alone) the INT4 codes of Q minus its block means
template <bool BF16, int D>
hipError_t q4_impl(const uint16_t *q, Strides st, float *q_mean, int8_t *q_i4, float *q_scale, int BH, int H, int N,
                   hipStream_t stream) {
    const int nQ = cdiv(N, kBQ);
    block_mean_kernel<BF16, D><<<dim3(nQ, BH), 256, 0, stream>>>(q, st, H, N, nQ, q_mean);
    if (q_i4)
        quant_int8_kernel<BF16, D, kBQ, 2, 7><<<dim3(nQ, BH), 256, 0, stream>>>(q, st, H, q_mean, q_i4, q_scale, N, nQ);
    return hipGetLastError();
}

}  // namespace

// which path launch_quant_kv takes (0: by shape) and how long a workgroup of the single-read kernel waits for its
// partners (ticks of the 100 MHz clock; negative: not at all)
std::atomic<int> g_kv_path{0};
std::atomic<long long> g_kv_wait_ticks{kResidentWaitTicks};

void set_quant_kv_path(int path, long long wait_ticks) {
    g_kv_path.store(path);
    g_kv_wait_ticks.store(wait_ticks);
}

QuantScratch quant_scratch_layout(void *base, int B, int H, int N, int d) {
    const size_t BH = (size_t)B * H;
    // partial statistics: one per kStatRows tokens (three-launch path) or per resident chunk (single-read path)
    const size_t chunks = (size_t)std::max(cdiv(N, kStatRows), resident_group_size(N, d));
    char *p = static_cast<char *>(base);
    QuantScratch ws;
    size_t off = 0;
    ws.k_sum_part = reinterpret_cast<double *>(p + off);
    off += align256(BH * chunks * d * sizeof(double));
    ws.v_max_part = reinterpret_cast<float *>(p + off);
    off += align256(BH * chunks * d * sizeof(float));
    ws.v_rcp = reinterpret_cast<float *>(p + off);
    off += align256(BH * d * sizeof(float));
    ws.bytes = off;
    return ws;
}

hipError_t launch_quant_q(const void *q, Strides st, int8_t *q_i8, float *q_scale, int B, int H, int N, int d,
                          bool bf16, hipStream_t stream) {
    const uint16_t *q16 = static_cast<const uint16_t *>(q);
    const int BH = B * H;
    if (d == 128)
        return bf16 ? quant_q_impl<true, 128>(q16, st, q_i8, q_scale, BH, H, N, stream)
                    : quant_q_impl<false, 128>(q16, st, q_i8, q_scale, BH, H, N, stream);
    return bf16 ? quant_q_impl<true, 64>(q16, st, q_i8, q_scale, BH, H, N, stream)
                : quant_q_impl<false, 64>(q16, st, q_i8, q_scale, BH, H, N, stream);
}

hipError_t launch_quant_k(const void *k, Strides st, int8_t *k_i8, float *k_scale, float *k_mean, int B, int H,
                          int N, int d, bool bf16, hipStream_t stream, const QuantScratch &ws) {
    const uint16_t *k16 = static_cast<const uint16_t *>(k);
    const int BH = B * H;
    if (d == 128)
        return bf16 ? quant_k_impl<true, 128>(k16, st, k_i8, k_scale, k_mean, BH, H, N, stream, ws)
                    : quant_k_impl<false, 128>(k16, st, k_i8, k_scale, k_mean, BH, H, N, stream, ws);
    return bf16 ? quant_k_impl<true, 64>(k16, st, k_i8, k_scale, k_mean, BH, H, N, stream, ws)
                : quant_k_impl<false, 64>(k16, st, k_i8, k_scale, k_mean, BH, H, N, stream, ws);
}

hipError_t launch_quant_v(const void *v, Strides st, uint8_t *v_fp8, float *v_scale, float v_r, int B, int H, int N,
                          int d, bool bf16, hipStream_t stream, const QuantScratch &ws) {
    const uint16_t *v16 = static_cast<const uint16_t *>(v);
    const int BH = B * H;
    if (d == 128) {
        return bf16 ? quant_v_impl<true, 128>(v16, st, v_fp8, v_scale, v_r, BH, H, N, stream, ws)
                    : quant_v_impl<false, 128>(v16, st, v_fp8, v_scale, v_r, BH, H, N, stream, ws);
    }
    return bf16 ? quant_v_impl<true, 64>(v16, st, v_fp8, v_scale, v_r, BH, H, N, stream, ws)
                : quant_v_impl<false, 64>(v16, st, v_fp8, v_scale, v_r, BH, H, N, stream, ws);
}

hipError_t launch_quant_kv(const void *k, Strides k_st, const void *v, Strides v_st, int8_t *k_i8, float *k_scale,
                           float *k_mean, uint8_t *v_fp8, float *v_scale, float v_r, int B, int H, int N, int d,
                           bool bf16, hipStream_t stream, const QuantScratch &ws, bool int4) {
    const uint16_t *k16 = static_cast<const uint16_t *>(k), *v16 = static_cast<const uint16_t *>(v);
    const int BH = B * H;
    const int path = g_kv_path.load();
    const bool resident = path == 2 || (path == 0 && resident_group_size(N, d) <= kResidentMaxGroup);
    if (resident && resident_group_size(N, d) > kResidentHardMaxGroup) return hipErrorInvalidValue;
    const long long wait_ticks = g_kv_wait_ticks.load();
#define SAGE_KV(BF, DD, QM)                                                                                           \
    (resident ? quant_kv_resident_impl<BF, DD, QM>(k16, k_st, v16, v_st, k_i8, k_scale, k_mean, v_fp8, v_scale, v_r, \
                                                   BH, H, N, stream, ws, wait_ticks)                                 \
              : quant_kv_impl<BF, DD, QM>(k16, k_st, v16, v_st, k_i8, k_scale, k_mean, v_fp8, v_scale, v_r, BH, H, N, \
                                          stream, ws))
    if (int4) {
        if (d == 128) return bf16 ? SAGE_KV(true, 128, 7) : SAGE_KV(false, 128, 7);
        return bf16 ? SAGE_KV(true, 64, 7) : SAGE_KV(false, 64, 7);
    }
    if (d == 128) return bf16 ? SAGE_KV(true, 128, 127) : SAGE_KV(false, 128, 127);
    return bf16 ? SAGE_KV(true, 64, 127) : SAGE_KV(false, 64, 127);
#undef SAGE_KV
}

hipError_t launch_quant_q4(const void *q, Strides st, float *q_mean, int8_t *q_i4, float *q_scale, int B, int H, int N,
                           int d, bool bf16, hipStream_t stream) {
    const uint16_t *q16 = static_cast<const uint16_t *>(q);
    const int BH = B * H;
    if (d == 128)
        return bf16 ? q4_impl<true, 128>(q16, st, q_mean, q_i4, q_scale, BH, H, N, stream)
                    : q4_impl<false, 128>(q16, st, q_mean, q_i4, q_scale, BH, H, N, stream);
    return bf16 ? q4_impl<true, 64>(q16, st, q_mean, q_i4, q_scale, BH, H, N, stream)
                : q4_impl<false, 64>(q16, st, q_mean, q_i4, q_scale, BH, H, N, stream);
}

hipError_t launch_delta_s(const void *k, Strides k_st, const float *k_mean, const float *q_mean, float *dsx, int B,
                          int Hq, int Hkv, int Nq, int Nk, int d, bool causal, float sm_scale, bool bf16,
                          hipStream_t stream) {
    const uint16_t *k16 = static_cast<const uint16_t *>(k);
    const dim3 grid(cdiv(Nk, kW), B * Hkv);
    const int nQ = cdiv(Nq, kBQ), nT = cdiv(Nk, kW);
    const float sm_log2e = (float)((double)sm_scale * 1.4426950408889634);
#define SAGE_DS(BF, DD) \
    delta_s_kernel<BF, DD><<<grid, 128, 0, stream>>>(k16, k_st, Hkv, k_mean, q_mean, dsx, Hq, Nq, Nk, nQ, nT, sm_log2e, \
                                                     causal ? 1 : 0)
    if (d == 128) {
        if (bf16) SAGE_DS(true, 128); else SAGE_DS(false, 128);
    } else {
        if (bf16) SAGE_DS(true, 64); else SAGE_DS(false, 64);
    }
#undef SAGE_DS
    return hipGetLastError();
}

}  // namespace sage
