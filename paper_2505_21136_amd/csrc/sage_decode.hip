// Decode-shaped attention on gfx950: a few query rows per head over a long key sequence (not treated in the
// paper; the arithmetic of a key step is the 8+8 path's, Sec. 2.1 / Sec. 3.1, through the same softmax_step).
//
// The prefill kernel gives a workgroup 128 query rows of one head and shares every K^/V^ tile among its eight
// wavefronts through LDS.  Here a head has at most a handful of rows, so that shape leaves 7 of 8 wavefronts
// and 15 of 16 MFMA columns idle and B*Hq workgroups cannot fill 256 CUs.  Instead:
//   * the R = (Hq/Hkv) * Nq <= 64 query rows of all query heads that share one K/V head are packed into the 16
//     columns of T = ceil(R/16) <= 4 MFMA tiles (exact: every row keeps its own scale, running maximum and sum), so
//     K^ and V^ of a head leave HBM once for all of them (the T wavefronts of a range sit in one workgroup and
//     read the same tiles at the same time: all but the first hit L2);
//   * the keys are cut into ranges of `steps_per_split` key steps and ONE WAVEFRONT owns one (batch, K/V head,
//     range, row tile): it runs the step recurrence on its range from m = -inf, l = 0, acc = 0 and writes (m, l, acc) per
//     row; merge_kernel then combines the ranges as partial softmax sums (m = max m_s, weights 2^(m_s - m));
//   * a wavefront uses each tile exactly once, so the operands go global -> registers directly (16 bytes per
//     lane and load, in the lane order the MFMA wants), K^ of step j+1 and V^ of step j in flight under the
//     arithmetic of step j; no LDS, no barrier.
// The stage is bound by HBM: K^ + V^ are read once, (2 * Nk * d bytes per K/V head).
#include "sage_attn_device.h"
#include "sage_internal.h"

#include <algorithm>

namespace sage {
namespace {

// D: head dimension; CAUSAL: end-aligned mask (key n visible to row r iff n <= r + Nk - Nq); BF16: type of Q / O.
// Grid: ceil(B*Hkv*S*T / 4) workgroups of 4 wavefronts; wavefront w = ((b*Hkv + kvh)*S + split)*T + row tile.
// NT: row tiles per wavefront (1: up to 16 rows per K/V head, 2 wavefronts per SIMD; 2: up to 32 rows per
// wavefront -- the operands of a key step are fetched once for both tiles --, 1 wavefront per SIMD).
template <int D, bool CAUSAL, bool BF16, int NT>
__global__ __launch_bounds__(256, NT == 1 ? 2 : 1) void decode_kernel(const uint16_t *__restrict__ Q, const int8_t *__restrict__ Kc,
                                                        const uint8_t *__restrict__ Vt, const float *__restrict__ dk,
                                                        float *__restrict__ part_acc, float *__restrict__ part_ml,
                                                        int n_waves, int Hq, int Hkv, int group, int Nq, int Nk, int nT,
                                                        int nKblk, int S, int T, int steps_per_split, float sm_scale,
                                                        float log2_pr) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int KC = D / 64;  // 64-wide contraction chunks of Q.K^T
    constexpr int CT = D / 16;  // 16-channel tiles of the output
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane((int)blockIdx.x * 4 + (int)(threadIdx.x >> 6));
    if (w >= n_waves) return;  // (whole wavefronts leave; the kernel has no barrier)
    const int lq = lane & 15, g = lane >> 4;
    // T row tiles in groups of NT per wavefront: TW = ceil(T / NT) wavefronts per (K/V head, range)
    const int TW = (T + NT - 1) / NT;
    const int rt0 = (w % TW) * NT, split = (w / TW) % S, bhk = w / (TW * S);
    const int b = bhk / Hkv, kvh = bhk % Hkv;
    const int R = group * Nq;  // rows in use (<= 16 * T)
    const int shift = Nk - Nq;

    const int8_t *Kh = Kc + (size_t)bhk * Nk * D;
    const uint8_t *Vh = Vt + (size_t)bhk * nT * D * 128;
    const int j0 = split * steps_per_split, j1 = min(nT, j0 + steps_per_split);

    // per row tile: row 16*(rt0 + qt) + lq of the K/V head = query row r of query head hq (rows past R repeat row 0
    // of head 0 and are never stored)
    bool row_ok[NT];
    int lim[NT];
    v4i qreg[NT][KC];
    double cq[NT];
#pragma unroll
    for (int qt = 0; qt < NT; ++qt) {
        const int ri = 16 * (rt0 + qt) + lq;
        row_ok[qt] = ri < R;
        const int hq = kvh * group + (row_ok[qt] ? ri / Nq : 0);
        const int r = row_ok[qt] ? ri % Nq : 0;
        lim[qt] = CAUSAL ? min(Nk - 1, r + shift) : Nk - 1;  // last visible key of this lane's row
        // ---- Q: load 16-bit, quantise per head over its Nq rows (the stand-alone quantiser's binary32 steps on
        // one block of Nq <= 64 rows: a head's rows are one Q quantisation block), straight into the B operand
        // layout of the INT8 MFMA ----
        const uint16_t *Qr = Q + (((size_t)b * Hq + hq) * Nq + r) * D;
        uint4 qraw[KC][2];
        float amax = 0.0f;
#pragma unroll
        for (int ch = 0; ch < KC; ++ch)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                qraw[ch][h] = *reinterpret_cast<const uint4 *>(Qr + ch * 64 + g * 16 + h * 8);
                const uint32_t u[4] = {qraw[ch][h].x, qraw[ch][h].y, qraw[ch][h].z, qraw[ch][h].w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    amax = fmaxf(amax, fmaxf(fabsf(to_f32<BF16>(u[i] & 0xffffu)), fabsf(to_f32<BF16>(u[i] >> 16))));
            }
        // the head's maximum: this lane's channels of all Nq rows of its head (they may sit in another row tile),
        // then over the four lanes that share the row
        const uint16_t *Qhd = Q + ((size_t)b * Hq + hq) * Nq * D;
        for (int rr = 0; rr < Nq; ++rr) {
            if (rr == r) continue;
#pragma unroll
            for (int ch = 0; ch < KC; ++ch)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint4 x = *reinterpret_cast<const uint4 *>(Qhd + (size_t)rr * D + ch * 64 + g * 16 + h * 8);
                    const uint32_t u[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        amax = fmaxf(amax, fmaxf(fabsf(to_f32<BF16>(u[i] & 0xffffu)), fabsf(to_f32<BF16>(u[i] >> 16))));
                }
        }
        float a = rowgroup_max(amax);
        if (!row_ok[qt]) a = 0.0f;
        const float rcp = a > 0.0f ? 127.0f / a : 0.0f;
        cq[qt] = (double)(a / 127.0f) * (double)sm_scale * 1.4426950408889634;
#pragma unroll
        for (int ch = 0; ch < KC; ++ch)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t u[4] = {qraw[ch][h].x, qraw[ch][h].y, qraw[ch][h].z, qraw[ch][h].w};
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    uint32_t cb[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t v = u[2 * hh + (i >> 1)];
                        float y = to_f32<BF16>((i & 1) ? (v >> 16) : (v & 0xffffu)) * rcp;
                        asm volatile("" : "+v"(y));  // keeps the product a rounded binary32 value (no FMA)
                        cb[i] = __builtin_bit_cast(uint32_t, y + kMagicF);  // low byte = rne(y), two's complement
                    }
                    const uint32_t lo2 = __builtin_amdgcn_perm(cb[1], cb[0], 0x0c0c0400u);
                    const uint32_t hi2 = __builtin_amdgcn_perm(cb[3], cb[2], 0x0c0c0400u);
                    qreg[qt][ch][2 * h + hh] = (int)__builtin_amdgcn_perm(hi2, lo2, 0x05040100u);
                }
            }
    }
    const v4i cinit = {kMagic, kMagic, kMagic, kMagic};

    // last visible key of the first / last row in use
    const int lim_min = CAUSAL ? min(Nk - 1, shift) : Nk - 1;
    const int lim_max = Nk - 1;

    float m[NT], l[NT];
    v4f o[NT][CT];
#pragma unroll
    for (int qt = 0; qt < NT; ++qt) {
        m[qt] = -INFINITY;
        l[qt] = 0.0f;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) o[qt][ct] = v4f{0.f, 0.f, 0.f, 0.f};
    }

    // K^ operand of step j: rows 16t + lq, 16-byte chunk 4ch + g (rows past the end are read from the last row
    // and masked)
    v4i ka[KC][8];
    auto load_k = [&](int j) {
#pragma unroll
        for (int ch = 0; ch < KC; ++ch)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int row = min(j * kW + 16 * t + lq, Nk - 1);
                ka[ch][t] = *reinterpret_cast<const v4i *>(Kh + (size_t)row * D + (4 * ch + g) * 16);
            }
    };
    if (j0 < j1) load_k(j0);

    for (int j = j0; j < j1; ++j) {
        const int key0 = j * kW;
        // V^ operand of this step: channel rows 16ct + lq of tile j, chunks g and 4 + g (consumed after the softmax)
        v4i va[CT][2];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const uint8_t *vr = Vh + ((size_t)j * D + 16 * ct + lq) * 128;
            va[ct][0] = *reinterpret_cast<const v4i *>(vr + g * 16);
            va[ct][1] = *reinterpret_cast<const v4i *>(vr + (4 + g) * 16);
        }
        const float dk0 = dk[(size_t)bhk * nKblk + min(2 * j, nKblk - 1)];
        const float dk1 = dk[(size_t)bhk * nKblk + min(2 * j + 1, nKblk - 1)];
        const bool masked_step = (key0 + kW > Nk) || (CAUSAL && key0 + kW - 1 > lim_min);
        const int t_lo = min(8, max(0, (lim_min - key0 + 1) >> 4));
        const int t_hi = min(8, max(0, ((lim_max - key0) >> 4) + 1));
#pragma unroll
        for (int qt = 0; qt < NT; ++qt) {
            // ---- S^T = K^ Q^T ----
            v4i s[8];
#pragma unroll
            for (int ch = 0; ch < KC; ++ch)
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    s[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ka[ch][t], qreg[qt][ch], ch == 0 ? cinit : s[t], 0, 0, 0);
            if (qt == NT - 1 && j + 1 < j1) load_k(j + 1);

            // ---- softmax step: every lane has the constants of its own row (its head's delta_Q) ----
            const float c0 = (float)(cq[qt] * (double)dk0), c1 = (float)(cq[qt] * (double)dk1);
            const float kh0 = -kMagicF * c0, kh1 = -kMagicF * c1;
            const float kl0 = __builtin_fmaf(-kMagicF, c0, -kh0), kl1 = __builtin_fmaf(-kMagicF, c1, -kh1);
            v8i pb;
            float alpha;
            if (masked_step) {
                const float l_old = l[qt];
                alpha = softmax_step<true>(s, c0, c1, kh0, kh1, kl0, kl1, log2_pr, m[qt], l[qt], pb, key0 + 4 * g, lim[qt],
                                           t_lo, t_hi);
                // a row that has seen no key yet and sees none in this step keeps its empty state (the step's
                // arithmetic on (-inf) - (-inf) is undefined; its P^ is zero either way)
                if (lim[qt] < key0 && m[qt] == -INFINITY) {
                    alpha = 1.0f;
                    l[qt] = l_old;
                }
            } else {
                alpha = softmax_step<false>(s, c0, c1, kh0, kh1, kl0, kl1, log2_pr, m[qt], l[qt], pb, 0, 0, 8, 8);
            }

            // ---- O^T = alpha O^T + V^T P^T ----
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) o[qt][ct] *= alpha;
            }
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const v8i a = {va[ct][0][0], va[ct][0][1], va[ct][0][2], va[ct][0][3],
                               va[ct][1][0], va[ct][1][1], va[ct][1][2], va[ct][1][3]};
                o[qt][ct] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, pb, o[qt][ct], 0, 0, 0, 0, 0, 0);
            }
        }
    }

    // ---- this range's (m, l, acc) of every row in use; l is the sum over the row's four lanes.  Partial rows are
    // indexed (((b*Hkv + kvh)*S + split)*T + row tile)*16 + lq ----
#pragma unroll
    for (int qt = 0; qt < NT; ++qt) {
        const float lsum = rowgroup_sum(l[qt]);
        if (row_ok[qt]) {
            const size_t prow = (((size_t)bhk * S + split) * T + rt0 + qt) * 16 + lq;
            if (g == 0) *reinterpret_cast<float2 *>(part_ml + prow * 2) = make_float2(m[qt], lsum);
            float *pa = part_acc + prow * D;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
                *reinterpret_cast<float4 *>(pa + 16 * ct + 4 * g) =
                    make_float4(o[qt][ct][0], o[qt][ct][1], o[qt][ct][2], o[qt][ct][3]);
        }
    }
#endif  // __HIP_DEVICE_COMPILE__
}

// Combine the S ranges of one row: m = max_s m_s, l = sum_s 2^(m_s - m) l_s, acc likewise, then the epilogue of the
// prefill kernel, O = acc * (delta_V / l) (l carries the factor P_r), rounded to the output type.
// T > 0: the partial results come from decode_kernel (T row tiles); T = 0: from attn_kernel<..., SPLIT> (query tiles
// of 128 rows).  One workgroup of 256 threads per row (grid B*Hq*Nq): thread t owns channels 4*(t % (D/4)) .. +3 and the ranges
// t / (D/4), + 256/(D/4), ...; the shares are added in a fixed order through LDS, so the result does not depend on
// timing.  (A row's ranges are read by many threads at once: with one thread walking them the launch is a chain
// of S memory latencies.)
template <int D, bool BF16>
__global__ __launch_bounds__(256) void merge_kernel(const float *__restrict__ part_acc, const float *__restrict__ part_ml,
                                                    const float *__restrict__ dv, uint16_t *__restrict__ out, int Hq,
                                                    int Hkv, int group, int Nq, int S, int T) {
    constexpr int Q4 = D / 4;      // channel quads
    constexpr int SL = 256 / Q4;   // range lanes
    __shared__ float red[256];
    __shared__ float4 acc_s[SL][Q4];
    __shared__ float l_s[SL];
    const int row = blockIdx.x;  // (b*Hq + hq)*Nq + r
    const int r = row % Nq, bh = row / Nq, hq = bh % Hq, b = bh / Hq;
    const int kvh = hq / group;
    // where range s of this row lies: partial row index p0 + s * ps
    size_t p0, ps;
    if (T > 0) {
        // decode_kernel: row ri of the K/V head sits in row tile ri / 16, column ri % 16 of wavefront
        // ((b*Hkv + kvh)*S + s)*T + tile
        const int ri = (hq % group) * Nq + r;
        p0 = (((size_t)b * Hkv + kvh) * S * T + ri / 16) * 16 + ri % 16;
        ps = (size_t)T * 16;
    } else {
        // attn_kernel<..., SPLIT>: row r of the head sits in query tile r / 128, row r % 128 of workgroup
        // ((b*Hq + hq)*tiles + tile)*S + s
        const int tiles = (Nq + kBQ - 1) / kBQ;
        p0 = (((size_t)bh * tiles + r / kBQ) * S) * kBQ + r % kBQ;
        ps = kBQ;
    }
    const int tid = threadIdx.x, cq = tid % Q4, sl = tid / Q4;
    // the row's maximum over all ranges
    float mx = -INFINITY;
    for (int s = tid; s < S; s += 256) mx = fmaxf(mx, part_ml[(p0 + s * ps) * 2]);
    red[tid] = mx;
    __syncthreads();
    for (int k = 128; k >= 1; k >>= 1) {
        if (tid < k) red[tid] = fmaxf(red[tid], red[tid + k]);
        __syncthreads();
    }
    mx = red[0];
    float l = 0.0f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int s = sl; s < S; s += SL) {
        const float2 ml = *reinterpret_cast<const float2 *>(part_ml + (p0 + s * ps) * 2);
        const float4 a = *reinterpret_cast<const float4 *>(part_acc + (p0 + s * ps) * D + 4 * cq);
        // a range in which the row saw no key has m = -inf, l = 0, acc = 0: its weight 2^(-inf) = 0 is exact
        const float wgt = __builtin_amdgcn_exp2f(ml.x - mx);
        l = __builtin_fmaf(wgt, ml.y, l);
        acc.x = __builtin_fmaf(wgt, a.x, acc.x);
        acc.y = __builtin_fmaf(wgt, a.y, acc.y);
        acc.z = __builtin_fmaf(wgt, a.z, acc.z);
        acc.w = __builtin_fmaf(wgt, a.w, acc.w);
    }
    acc_s[sl][cq] = acc;
    if (cq == 0) l_s[sl] = l;
    __syncthreads();
    if (sl == 0) {
        for (int k = 1; k < SL; ++k) {
            const float4 a = acc_s[k][cq];
            acc.x += a.x, acc.y += a.y, acc.z += a.z, acc.w += a.w;
            l += l_s[k];
        }
        const float inv = 1.0f / l;
        const float4 sc = *reinterpret_cast<const float4 *>(dv + ((size_t)b * Hkv + kvh) * D + 4 * cq);
        const float y0 = acc.x * (sc.x * inv), y1 = acc.y * (sc.y * inv);
        const float y2 = acc.z * (sc.z * inv), y3 = acc.w * (sc.w * inv);
        *reinterpret_cast<uint2 *>(out + (size_t)row * D + 4 * cq) = make_uint2(pack2<BF16>(y0, y1), pack2<BF16>(y2, y3));
    }
}

}  // namespace

int decode_auto_steps_per_split(int B, int Hkv, int Nk) {
    // about four wavefronts per CU over the whole launch (measured: 1024 wavefronts stream a 0.3-0.5 GB cache 4-8 %
    // faster than 2048 -- fewer partial results to write and combine -- and much faster than 512), at least two key
    // steps per wavefront
    const int nT = cdiv(Nk, kW);
    const long heads = (long)B * Hkv;
    const int want = (int)std::max<long>(1, std::min<long>(nT, (1024 + heads - 1) / heads));
    return std::max(std::min(nT, 2), cdiv(nT, want));
}

DecodeScratch decode_scratch_layout(void *base, int B, int Hkv, int Nk, int d, int steps_per_split, int row_tiles) {
    const int S = cdiv(cdiv(Nk, kW), steps_per_split);
    const size_t waves = (size_t)B * Hkv * S * row_tiles;
    char *p = static_cast<char *>(base);
    DecodeScratch ws;
    ws.n_splits = S;
    ws.part_acc = reinterpret_cast<float *>(p);
    size_t off = (waves * 16 * d * sizeof(float) + 255) & ~(size_t)255;
    ws.part_ml = reinterpret_cast<float *>(p + off);
    off += (waves * 16 * 2 * sizeof(float) + 255) & ~(size_t)255;
    ws.bytes = off;
    return ws;
}

hipError_t launch_decode(const void *q, const int8_t *k_i8, const uint8_t *v_fp8, const float *k_scale,
                         const float *v_scale, void *out, int B, int Hq, int Hkv, int Nq, int Nk, int d, bool causal,
                         float sm_scale, float p_r, int steps_per_split, bool bf16, hipStream_t stream,
                         const DecodeScratch &ws) {
    const int group = Hq / Hkv;
    const int nT = cdiv(Nk, kW), nK = cdiv(Nk, kBK);
    const int S = ws.n_splits;
    const int T = cdiv(group * Nq, 16);
    const int nt = T >= 2 ? 2 : 1;  // row tiles per wavefront (measured: 0.16 against 0.25 ms at 64 rows per K/V head, B 8, 32768 keys)
    const int n_waves = B * Hkv * S * cdiv(T, nt);
    const float log2_pr = (float)log2((double)p_r);
    const uint16_t *q16 = static_cast<const uint16_t *>(q);
    uint16_t *o16 = static_cast<uint16_t *>(out);
#define SAGE_DEC(DD, C, BF)                                                                                       \
    do {                                                                                                          \
        if (nt == 1)                                                                                              \
            decode_kernel<DD, C, BF, 1><<<cdiv(n_waves, 4), 256, 0, stream>>>(                                     \
                q16, k_i8, v_fp8, k_scale, ws.part_acc, ws.part_ml, n_waves, Hq, Hkv, group, Nq, Nk, nT, nK, S, T, \
                steps_per_split, sm_scale, log2_pr);                                                              \
        else                                                                                                      \
            decode_kernel<DD, C, BF, 2><<<cdiv(n_waves, 4), 256, 0, stream>>>(                                     \
                q16, k_i8, v_fp8, k_scale, ws.part_acc, ws.part_ml, n_waves, Hq, Hkv, group, Nq, Nk, nT, nK, S, T, \
                steps_per_split, sm_scale, log2_pr);                                                              \
    } while (0)
    if (d == 128) {
        if (causal) { if (bf16) SAGE_DEC(128, true, true); else SAGE_DEC(128, true, false); }
        else        { if (bf16) SAGE_DEC(128, false, true); else SAGE_DEC(128, false, false); }
    } else {
        if (causal) { if (bf16) SAGE_DEC(64, true, true); else SAGE_DEC(64, true, false); }
        else        { if (bf16) SAGE_DEC(64, false, true); else SAGE_DEC(64, false, false); }
    }
#undef SAGE_DEC
    const int n_rows = B * Hq * Nq;
#define SAGE_MERGE(DD, BF) \
    merge_kernel<DD, BF><<<n_rows, 256, 0, stream>>>(ws.part_acc, ws.part_ml, v_scale, o16, Hq, Hkv, group, Nq, S, T)
    if (d == 128) {
        if (bf16) SAGE_MERGE(128, true); else SAGE_MERGE(128, false);
    } else {
        if (bf16) SAGE_MERGE(64, true); else SAGE_MERGE(64, false);
    }
#undef SAGE_MERGE
    return hipGetLastError();
}


// Few workgroups, many keys (more than 64 query rows per K/V head): the prefill kernel with the key steps cut into
// ranges on separate workgroups, then the same combination launch.
hipError_t launch_attn_ranges(const void *q, const int8_t *k_i8, const uint8_t *v_fp8, const float *k_scale,
                              const float *v_scale, void *out, int B, int Hq, int Hkv, int Nq, int Nk, int d, bool causal,
                              float sm_scale, float p_r, int steps_per_split, bool bf16, hipStream_t stream,
                              const DecodeScratch &ws) {
    const int S = ws.n_splits;
    if (S == 1) {
        // one range is the uncut kernel, which writes the output itself
        const Strides st = contiguous_bhnd(Hq, Nq, d);
        return launch_attn(q, true, st, k_i8, v_fp8, nullptr, k_scale, v_scale, out, st, B, Hq, Hkv, Nq, Nk, d, causal,
                           sm_scale, p_r, bf16, stream);
    }
    hipError_t e = launch_attn_split(q, k_i8, v_fp8, k_scale, v_scale, B, Hq, Hkv, Nq, Nk, d, causal, sm_scale, p_r, bf16,
                                     S, steps_per_split, ws.part_acc, ws.part_ml, stream);
    if (e != hipSuccess) return e;
    uint16_t *o16 = static_cast<uint16_t *>(out);
    const int n_rows = B * Hq * Nq, group = Hq / Hkv;
#define SAGE_MERGE(DD, BF) \
    merge_kernel<DD, BF><<<n_rows, 256, 0, stream>>>(ws.part_acc, ws.part_ml, v_scale, o16, Hq, Hkv, group, Nq, S, 0)
    if (d == 128) {
        if (bf16) SAGE_MERGE(128, true); else SAGE_MERGE(128, false);
    } else {
        if (bf16) SAGE_MERGE(64, true); else SAGE_MERGE(64, false);
    }
#undef SAGE_MERGE
    return hipGetLastError();
}

int ranges_auto_steps_per_split(int B, int Hq, int Nq, int Nk) {
    // Measured (B*Hq*tiles = 16 .. 512 workgroups before the cut, 4096 .. 65536 keys): the cut pays up to 128
    // workgroups, and best with about 512 workgroups after it (one for each of the chip's slots); from 256 workgroups
    // on the uncut kernel is faster (every range writes 128 x (d + 2) floats per workgroup that the combination
    // reads back).  At least four key steps per range.
    const int nT = cdiv(Nk, kW);
    const long items = (long)B * Hq * cdiv(Nq, kBQ);
    if (items > 128) return nT;
    const int want = (int)std::max<long>(1, std::min<long>(nT, 512 / items));
    return std::max(std::min(nT, 4), cdiv(nT, want));
}

DecodeScratch ranges_scratch_layout(void *base, int B, int Hq, int Nq, int Nk, int d, int steps_per_split) {
    const int S = cdiv(cdiv(Nk, kW), steps_per_split);
    const size_t rows = (size_t)B * Hq * cdiv(Nq, kBQ) * S * kBQ;
    char *p = static_cast<char *>(base);
    DecodeScratch ws;
    ws.n_splits = S;
    ws.part_acc = reinterpret_cast<float *>(p);
    size_t off = (rows * d * sizeof(float) + 255) & ~(size_t)255;
    ws.part_ml = reinterpret_cast<float *>(p + off);
    off += (rows * 2 * sizeof(float) + 255) & ~(size_t)255;
    ws.bytes = off;
    return ws;
}

}  // namespace sage
