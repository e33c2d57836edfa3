// Stage 2 of the SageAttention2++ 8+8 forward on gfx950: the fused attention
// kernel (paper Sec. 2.1 for the tiling / online softmax and the scales,
// Sec. 3.1 for the bounded FP8 range P_r of P~).
//
// Mapping to CDNA4.  A workgroup of NWAVE wavefronts owns BM = 16*NQ*NWAVE query
// rows of one (batch, head); a wavefront owns NQ tiles of 16 query rows.  Per
// step of 128 keys the K^ tile [128][D] int8 and the V^ tile [D][128] fp8 are
// copied global -> LDS by buffer loads that write LDS directly (no register
// staging; chunks beyond the end of a head's K^ are not fetched and read as zero), double buffered so that the copy of
// step j+1 runs under the arithmetic of step j (two barriers per step, see "Schedule").
// 16-byte LDS chunks are XOR-swizzled against bank conflicts.
//   S^T = K^ Q^T   with v_mfma_i32_16x16x64_i8 (keys are MFMA rows, queries are
//                  MFMA columns).  A lane then holds, for ONE query (lane&15),
//                  the scores of keys 16t + 4(lane>>4) + i, t<8, i<4: the row
//                  maximum and sum are in-lane work plus two cross-lane steps.
//   softmax        base 2, FP32; the de-quantisation constant
//                  delta_Q*delta_K*sm_scale*log2(e) is one FMA operand (kept in
//                  a VGPR: FMAs with a scalar operand issue at half rate), the
//                  maximum is taken on the integer scores per 64-key K block;
//                  the INT32 accumulator starts at the bit pattern of 1.5*2^23,
//                  which makes its bits a valid binary32 number (no conversion).
//   P^             v_cvt_pk_fp8_f32 in registers: the 32 bytes a lane produces
//                  are exactly its B operand of v_mfma_f32_16x16x128_f8f6f4.
//   O^T += V^T P^T with that instruction (FP8 E4M3 both sides, FP32 accumulate;
//                  the older 16x16x32 fp8 MFMA runs at half its rate);
//                  V^ is stored transposed and key-permuted by the quantiser so
//                  that the A operand is two 16-byte LDS chunks read in the same
//                  conflict-free pattern as the K^ operand.
// The accumulator is rescaled only in steps where some row maximum moved
// (multiplying by alpha == 1 is the identity, so skipping is exact).
#include "sage_attn_device.h"
#include "sage_internal.h"

#include <limits.h>
#include <math.h>

namespace sage {
namespace {

// The same step for the 4+8 variant (INT4 codes, Q smoothed by its block means): the de-quantised score of a
// key gets the correction term ds = (qbar . K'[n]) * sm_scale * log2(e) added, which differs from key to key,
// so the step maximum is taken on the finished exponents x = c * S + ds (FP32) instead of on the integers:
// per score one conversion, one FMA, half a max3, one addition, one exp2, one addition, half an FP8 pack.
// s holds plain INT32 scores.  ds: this lane's 32 correction terms of the step (LDS), 8 x float4 in the order
// of its scores.
template <bool MASKED>
__device__ __forceinline__ float softmax_step_q4(const v4i (&s)[8], float c0, float c1, float log2_pr, float &m, float &l,
                                                 v8i &pb, int key_base, int lim, int t_lo, int t_hi,
                                                 const float4 *__restrict__ ds) {
    float mx0 = -INFINITY, mx1 = -INFINITY;
    float xf[8][4];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        bool live = true;
        if constexpr (MASKED) live = t < t_hi;
        if (live) {
            const float4 d4 = ds[t];
            const float dd[4] = {d4.x, d4.y, d4.z, d4.w};
            const float cb = t < 4 ? c0 : c1;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int sv = s[t][i];
                float x = __builtin_fmaf((float)sv, cb, dd[i]);
                if constexpr (MASKED) {
                    if (t >= t_lo && key_base + 16 * t + i > lim) x = -INFINITY;
                }
                xf[t][i] = x;
                if (i < 2) mx0 = fmaxf(mx0, x); else mx1 = fmaxf(mx1, x);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) xf[t][i] = -INFINITY;
        }
        // (keeps the compiler from fetching all 32 correction terms up front)
        if (t == 3) __builtin_amdgcn_sched_barrier(0);
    }
    const float mc = rowgroup_max(fmaxf(mx0, mx1));
    const float m_new = fmaxf(m, mc);
    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
    const float mo = log2_pr - m_new;  // P~ * P_r = 2^(x - m' + log2 P_r)
    float lsum0 = -0.0f, lsum1 = -0.0f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        if constexpr (MASKED) {
            if (t >= t_hi) {
                pb[t] = 0;
                continue;
            }
        }
        float p[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) p[i] = __builtin_amdgcn_exp2f(xf[t][i] + mo);  // a masked key: 2^(-inf) = 0
        lsum0 += p[0] + p[1];
        lsum1 += p[2] + p[3];
        int w;  // both halves are overwritten below
        asm volatile("" : "=v"(w));
        w = __builtin_amdgcn_cvt_pk_fp8_f32(p[0], p[1], w, false);
        w = __builtin_amdgcn_cvt_pk_fp8_f32(p[2], p[3], w, true);
        pb[t] = w;
    }
    l = l * alpha + (lsum0 + lsum1);
    m = m_new;
    return alpha;
}

#if defined(__HIP_DEVICE_COMPILE__)
// Enqueue piece k of the global -> LDS copy of one [128 x D]-byte tile (K^ or V^) of key step j.  A tile is
// copied by the NW wavefronts of one group, CPG pieces each; a piece (one buffer load) moves 16 bytes per
// lane straight into LDS at dst + 1024*(k*NW + w) + 16*lane; the per-lane source offset carries the
// swizzle.  Every piece gets a buffer descriptor of its own whose base is the piece's first byte and whose
// size is what is left of the head's buffer from there (scalar arithmetic only): the hardware bounds check
// covers the per-lane offset but not a scalar offset, and this way a 16-byte chunk beyond the last byte of
// the buffer (rows >= Nk of the last K^ tile) is never fetched and reads as zero.
template <int D, int NW>
__device__ __forceinline__ void issue_tile_piece(uint8_t *dst, const uint8_t *head, int head_bytes, int voff, int w,
                                                 int k, int j) {
    constexpr int TILE = 128 * D;
    // (piece k of a wavefront lies NW KB after piece 0 on both sides: the swizzles repeat every 8 rows)
    const int first = j * TILE + k * NW * 1024;
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)(head + first), 0, max(head_bytes - first, 0), 0x00020000);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)(dst + (k * NW + w) * 1024), 16, voff, 0, 0, 0);
}
#endif  // __HIP_DEVICE_COMPILE__

// Schedule.  The wavefronts of a workgroup form two groups (first and second half) that run the
// same per-step sequence  M(j) = [PV(j-1), QK(j)]  ->  S(j) = softmax(j)  one slot apart: while
// one group is in its matrix slot (MFMA + LDS reads) the other is in its softmax slot (vector
// ALU), so the two pipes of every SIMD are busy at the same time instead of colliding.  A slot
// ends with a workgroup barrier.  The copy of K^(j+1) is issued by the first group at the start of
// slot 2j, the copy of V^(j) by the second group at the start of slot 2j+1 (each in its own matrix
// slot); both are needed from slot 2j+2 on.
//
// QRAW: Q arrives unquantised (16-bit, the output's type) and the workgroup, whose 128 rows are
// exactly one Q quantisation block, quantises it in its prologue (paper Sec. 2.1: per-block INT8,
// delta = max|Q| / 127) with the same binary32 operations as the stand-alone quantiser, so codes
// and scale are the same bits; Q^ and delta_Q then never touch memory.
//
// Q4 (with QRAW): the 4+8 variant.  K^ holds INT4 codes (one per byte, same INT8 MFMA), Q is smoothed by the
// block means `q_mean` before its INT4 quantisation (delta = max|Q - qbar| / 7), and the score correction
// `dsx` (see softmax_step_q4) is added in the softmax part; everything else is shared with the 8+8 kernel.
// (Its softmax part keeps the 32 exponents of a step in registers next to the scores they come from; at d = 128
// that does not fit the 128 registers of four wavefronts per SIMD, so this one variant is built for two: one
// workgroup per CU instead of two.)
//
// SPLIT (with QRAW, without Q4): the key steps are cut into `n_splits` ranges of `steps_per_split` steps and the
// grid holds one workgroup per (head, query tile, range).  A workgroup runs the recurrence on its range alone, from
// m = -inf, l = 0, acc = 0, and instead of O writes the range's (m, l, acc) of every row to `part_ml` / `part_acc`
// ([item][range][128 rows][2] and [...][D] floats, item = head * tiles + tile); merge_kernel (sage_decode.hip)
// combines the ranges.  For calls whose (head, tile) pairs alone cannot fill the GPU: few query rows over many keys.
template <int D, int NQ, int NWAVE, int WPS, bool CAUSAL, bool BF16, bool QRAW, bool Q4, bool SPLIT = false>
__global__ __launch_bounds__(NWAVE * 64, (Q4 && D == 128) ? 2 : WPS) void attn_kernel(
    const void *__restrict__ Qsrc, const int8_t *__restrict__ Kc, const uint8_t *__restrict__ Vt,
    const float *__restrict__ dq, const float *__restrict__ dk, const float *__restrict__ dv,
    uint16_t *__restrict__ out, Strides q_st, Strides o_st, int Nq, int Nk, int nT, int nQblk, int nKblk, int Hq,
    int group, float sm_scale, float log2_pr, int nQtiles, const float *__restrict__ q_mean,
    const float *__restrict__ dsx, int n_splits, int steps_per_split, float *__restrict__ part_acc,
    float *__restrict__ part_ml) {
    static_assert(!Q4 || QRAW, "the 4+8 variant quantises Q in the kernel");
    static_assert(!SPLIT || (QRAW && !Q4 && NQ == 1), "key ranges: unquantised Q, 8+8, one row tile per wavefront");
#if defined(__HIP_DEVICE_COMPILE__)  // the body uses device-only types; the host pass only needs the stub
    constexpr int BM = 16 * NQ * NWAVE;  // query rows per workgroup
    constexpr int KC = D / 64;           // 64-wide contraction chunks of Q.K^T
    constexpr int CT = D / 16;           // 16-channel tiles of the output
    constexpr int TILE = 128 * D;        // bytes of one K^ (or V^) tile
    constexpr int NTHR = NWAVE * 64;
    constexpr int NWG = NWAVE / 2;                 // wavefronts per group
    constexpr int CPG = TILE / 16 / (NTHR / 2);    // 16-byte chunks a thread copies per tile (one group copies a tile)
    static_assert(TILE / 16 % (NTHR / 2) == 0, "tile chunks must divide over the threads of a group");
    __shared__ __attribute__((aligned(1024))) uint8_t ldsK[2][TILE];
    __shared__ __attribute__((aligned(1024))) uint8_t ldsV[2][TILE];
    __shared__ float q_wave_max[NWAVE];
    // per wavefront: the de-quantisation constants (c, kh, kl, -) of 64 consecutive K blocks (32 key steps)
    __shared__ __attribute__((aligned(16))) float4 cst_lds[NWAVE][64];
    // 4+8 variant: the score-correction terms of three consecutive key steps (128 floats each, lane order)
    __shared__ __attribute__((aligned(16))) float ds_lds[Q4 ? 3 : 1][128];
    __shared__ __attribute__((aligned(16))) float dv_lds[D];  // delta_V of this head, for the epilogue

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >= NWAVE / 2 ? 1 : 0;  // second group runs one slot behind
    const int lq = lane & 15, g = lane >> 4;
    // Workgroup -> (head, query tile); the grid is one-dimensional.  The hardware deals consecutive
    // workgroup ids round-robin to the 8 XCDs, each with an L2 of its own: workgroup id is the `slot`-th
    // of XCD `xcd`.  Co-resident workgroups of an XCD should stream through the same K^/V^ tiles (its L2
    // then serves every fetch after the first), and a causal launch must also end on its short tiles.
    const int n_items = (int)gridDim.x / (SPLIT ? n_splits : 1), n_qt = nQtiles, n_bh = n_items / n_qt;
    const int xcd = (int)blockIdx.x % 8, slot = (int)blockIdx.x / 8;
    int bh, qtile;  // (batch, query head), query tile
    int split = 0;  // SPLIT: this workgroup's key range (the ranges of an item are adjacent workgroup ids)
    if constexpr (SPLIT) {
        split = (int)blockIdx.x % n_splits;
        bh = ((int)blockIdx.x / n_splits) / n_qt;
        qtile = ((int)blockIdx.x / n_splits) % n_qt;
    } else if (!CAUSAL && n_qt >= 128) {
        // a head has 16 or more tiles per XCD anyway: ids in order (query tile fastest), every XCD works
        // on the same one or two heads, and a tile missed by one L2 is likely still in the last-level cache
        bh = (int)blockIdx.x / n_qt;
        qtile = (int)blockIdx.x % n_qt;
    } else if (!CAUSAL) {
        // shorter sequences: head-major items cut into 8 contiguous ranges, one per XCD, walked in order
        // (otherwise an XCD would hold only n_qt/8 tiles of each of many heads at a time)
        const int pos = xcd * (n_items / 8) + min(xcd, n_items % 8) + slot;
        bh = pos / n_qt;
        qtile = pos % n_qt;
    } else if (n_bh % 8 == 0) {
        // an XCD owns n_bh/8 adjacent heads and takes them in windows of G heads -- enough tiles to fill
        // its 64 workgroup slots twice --, inside a window the longest tiles of all heads first
        const int hp = n_bh / 8;
        const int G = max(1, min(hp, (127 + n_qt) / n_qt));
        const int w = slot / (G * n_qt), r = slot - w * G * n_qt;
        const int hw = min(G, hp - w * G);  // heads in this window (the last one may be short)
        bh = xcd * hp + w * G + r % hw;
        qtile = n_qt - 1 - r / hw;
    } else {
        // any other head count: longest tiles first over all heads
        bh = (int)blockIdx.x % n_bh;
        qtile = n_qt - 1 - (int)blockIdx.x / n_bh;
    }
    const int wg_row0 = qtile * BM;
    const int row0 = wg_row0 + wave * (16 * NQ);
    // grouped-query attention: `group` consecutive query heads share one K/V head
    const int bhk = (bh / Hq) * (Hq / group) + (bh % Hq) / group;
    // causal mask aligned to the end of both sequences: key n visible to query r iff n <= r + shift
    const int shift = Nk - Nq;

    // this head's K^ [Nk][D] and V^ [nT][D][128] and their sizes in bytes (the tile copies are bounded to them)
    const uint8_t *Kh = reinterpret_cast<const uint8_t *>(Kc) + (size_t)bhk * Nk * D;
    const uint8_t *Vh = Vt + (size_t)bhk * nT * D * 128;
    const int k_bytes = Nk * D, v_bytes = nT * D * 128;

    // Tile copies.  The first group copies the K^ tiles, the second the V^ tiles, each at the start of its own
    // matrix slot: the texture path accepts one 1 KB piece per 16 cycles per CU, and a wavefront that cannot
    // issue its piece cannot issue anything else either -- harmless in the matrix slot (it has slack), costly
    // in front of the softmax arithmetic (which is the critical path).
    // Per-lane source offset of this wavefront's piece 0 (the LDS side is linear in the lane index):
    const int wig = wave % NWG;  // wavefront within its group
    int c_voff;
    {
        static_assert(NWG * 64 % (8 * (D / 16)) == 0 && NWG * 8 % 8 == 0, "pieces must be whole swizzle periods apart");
        const int slot = wig * 64 + lane;
        if (grp == 0) {
            constexpr int CPR = D / 16;  // chunks per K row
            const int row = slot / CPR, pc = slot % CPR;
            c_voff = row * D + ((pc ^ k_swz<D>(row)) << 4);
        } else {
            const int row = slot >> 3, pc = slot & 7;
            c_voff = row * 128 + ((pc ^ (row & 7)) << 4);
        }
    }

    // key steps [jb, nsteps) of this workgroup (jb = 0 unless SPLIT)
    int nsteps = nT;
    if constexpr (CAUSAL) nsteps = min(Nk - 1, wg_row0 + BM - 1 + shift) / kW + 1;
    const int jb = SPLIT ? split * steps_per_split : 0;
    if constexpr (SPLIT) nsteps = max(jb, min(nsteps, jb + steps_per_split));  // (empty when the range lies above the rows)
    // steps this wavefront takes part in (causal: tiles entirely above its rows are skipped)
    int my_steps = nsteps;
    if constexpr (CAUSAL) my_steps = min(nsteps, (row0 + 16 * NQ - 1 + shift) / kW + 1);
    if (row0 >= Nq) my_steps = jb;  // a wavefront without a valid row only takes part in the copies and barriers
    // 4+8 variant: the correction terms of this Q block, [nT][128] floats; the first wavefront copies those of
    // key step j into ds_lds[j % 3] with the K^ tile of that step (two 256-byte pieces, global -> LDS direct)
    auto copy_ds = [&](int j) {
        if constexpr (Q4) {
            if (wave == 0 && j < nsteps) {
                const float *src = dsx + (((size_t)bh * nQblk + qtile) * nT + j) * 128;
                const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)src, 0, 512, 0x00020000);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)&ds_lds[j % 3][0], 4, lane * 4, 0, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)&ds_lds[j % 3][64], 4, 256 + lane * 4, 0, 0, 0);
            }
        }
    };
    if (grp == 0) {
#pragma unroll
        for (int k = 0; k < CPG; ++k) issue_tile_piece<D, NWG>(ldsK[jb & 1], Kh, k_bytes, c_voff, wig, k, jb);
    }
    copy_ds(jb);

    // the lane's B operand of S^T = K^ Q^T: 16 consecutive channels (64*ch + 16*g ..) of query row lq
    v4i qreg[NQ][KC];
    uint4 qraw[NQ][KC][2];  // QRAW: the same 16 channels as 16-bit values
    if constexpr (QRAW) {
        static_assert(BM == kBQ, "a workgroup must own exactly one Q quantisation block");
        const uint16_t *Qh = static_cast<const uint16_t *>(Qsrc) + (bh / Hq) * q_st.b + (bh % Hq) * q_st.h;
        float amax = 0.0f;
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
            const int r = row0 + qt * 16 + lq;
#pragma unroll
            for (int ch = 0; ch < KC; ++ch)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    qraw[qt][ch][h] = r < Nq ? *reinterpret_cast<const uint4 *>(Qh + r * q_st.n + ch * 64 + g * 16 + h * 8)
                                             : make_uint4(0u, 0u, 0u, 0u);
                    const uint32_t w[4] = {qraw[qt][ch][h].x, qraw[qt][ch][h].y, qraw[qt][ch][h].z, qraw[qt][ch][h].w};
                    if constexpr (Q4) {
                        // max |Q - qbar| over the valid rows (a missing row would contribute |qbar|)
                        const float *qm = q_mean + ((size_t)bh * nQblk + qtile) * D + ch * 64 + g * 16 + h * 8;
                        const float4 ma = *reinterpret_cast<const float4 *>(qm), mb = *reinterpret_cast<const float4 *>(qm + 4);
                        const float mu[8] = {ma.x, ma.y, ma.z, ma.w, mb.x, mb.y, mb.z, mb.w};
                        if (r < Nq) {
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                amax = fmaxf(amax, fmaxf(fabsf(to_f32<BF16>(w[i] & 0xffffu) - mu[2 * i]),
                                                         fabsf(to_f32<BF16>(w[i] >> 16) - mu[2 * i + 1])));
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            amax = fmaxf(amax, fmaxf(fabsf(to_f32<BF16>(w[i] & 0xffffu)), fabsf(to_f32<BF16>(w[i] >> 16))));
                    }
                }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
        if (lane == 0) q_wave_max[wave] = amax;
    } else {
        const int8_t *Qh = static_cast<const int8_t *>(Qsrc) + (bh / Hq) * q_st.b + (bh % Hq) * q_st.h;
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
            const int r = row0 + qt * 16 + lq;
#pragma unroll
            for (int ch = 0; ch < KC; ++ch) {
                v4i z = {0, 0, 0, 0};
                qreg[qt][ch] = r < Nq ? *reinterpret_cast<const v4i *>(Qh + r * q_st.n + ch * 64 + g * 16) : z;
            }
        }
    }
    // (the 4+8 variant converts its scores explicitly: plain INT32 accumulators)
    constexpr int kInit = Q4 ? 0 : kMagic;
    const v4i cinit = {kInit, kInit, kInit, kInit};

    // the output scales are fetched now and parked in LDS: the epilogue then waits for no global load
    if (tid < D / 4)
        *reinterpret_cast<float4 *>(dv_lds + 4 * tid) = *reinterpret_cast<const float4 *>(dv + (size_t)bhk * D + 4 * tid);
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): K^(0) has landed
    __syncthreads();

    // de-quantisation constant of this wave's query block (its 16*NQ rows lie inside one Q block)
    float delta_q;
    if constexpr (QRAW) {
        float a = 0.0f;
#pragma unroll
        for (int w = 0; w < NWAVE; ++w) a = fmaxf(a, q_wave_max[w]);
        constexpr float kRange = Q4 ? 7.0f : 127.0f;
        const float rcp = a > 0.0f ? kRange / a : 0.0f;
        delta_q = a / kRange;
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt)
#pragma unroll
            for (int ch = 0; ch < KC; ++ch)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint32_t w[4] = {qraw[qt][ch][h].x, qraw[qt][ch][h].y, qraw[qt][ch][h].z, qraw[qt][ch][h].w};
                    float mu[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    if constexpr (Q4) {
                        const float *qm = q_mean + ((size_t)bh * nQblk + qtile) * D + ch * 64 + g * 16 + h * 8;
                        const float4 ma = *reinterpret_cast<const float4 *>(qm), mb = *reinterpret_cast<const float4 *>(qm + 4);
                        mu[0] = ma.x, mu[1] = ma.y, mu[2] = ma.z, mu[3] = ma.w;
                        mu[4] = mb.x, mu[5] = mb.y, mu[6] = mb.z, mu[7] = mb.w;
                    }
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        // code = rne(fl(x * rcp)): adding 1.5*2^23 to the (separately rounded) product rounds
                        // it to the nearest integer, ties to even, and leaves the code's two's-complement
                        // byte in the low byte of the sum's bit pattern; three byte permutes pack four codes
                        uint32_t b[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const uint32_t u = w[2 * hh + (i >> 1)];
                            float x = to_f32<BF16>((i & 1) ? (u >> 16) : (u & 0xffffu));
                            if constexpr (Q4) x = x - mu[4 * hh + i];  // one binary32 subtraction, as the quantiser does
                            float y = x * rcp;
                            asm volatile("" : "+v"(y));  // keeps the product a rounded binary32 value (no FMA)
                            b[i] = __builtin_bit_cast(uint32_t, y + kMagicF);
                        }
                        const uint32_t lo2 = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u);
                        const uint32_t hi2 = __builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u);
                        qreg[qt][ch][2 * h + hh] = (int)__builtin_amdgcn_perm(hi2, lo2, 0x05040100u);
                    }
                }
    } else {
        delta_q = dq[(size_t)bh * nQblk + min(row0, Nq - 1) / kBQ];
    }
    const double cq = (double)delta_q * (double)sm_scale * 1.4426950408889634;

    // (the accumulators start their life here, after the prologue, whose Q registers they reuse)
    float m[NQ], l[NQ], alpha[NQ];
    v4f o[CT][NQ];
    v4i s[NQ][8];
    v8i pb[NQ];
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        m[qt] = -INFINITY;
        l[qt] = 0.0f;
        alpha[qt] = 1.0f;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) o[ct][qt] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 8; ++t) s[qt][t] = cinit;
        pb[qt] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
    }


    // piece k of the copy this group makes during its matrix slot M(j): K^(j+1) (first group), V^(j) (second)
    auto copy_k = [&](int j) {
        if (j + 1 < nsteps) {
#pragma unroll
            for (int k = 0; k < CPG; ++k) issue_tile_piece<D, NWG>(ldsK[(j + 1) & 1], Kh, k_bytes, c_voff, wig, k, j + 1);
        }
        copy_ds(j + 1);
    };
    auto copy_v = [&](int j) {
        if (j < nsteps) {
#pragma unroll
            for (int k = 0; k < CPG; ++k) issue_tile_piece<D, NWG>(ldsV[j & 1], Vh, v_bytes, c_voff, wig, k, j);
        }
    };
    // matrix slot M(j): PV(j-1), then QK(j)
    auto matrix_slot = [&](int j) {
        if (j > jb && j <= my_steps) {
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
            const uint8_t *Vs = ldsV[(j - 1) & 1];
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const int row = 16 * ct + lq;
                const v4i lo = *reinterpret_cast<const v4i *>(Vs + v_off(row, g));
                const v4i hi = *reinterpret_cast<const v4i *>(Vs + v_off(row, 4 + g));
                const v8i a = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
#pragma unroll
                for (int qt = 0; qt < NQ; ++qt)
                    o[ct][qt] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, pb[qt], o[ct][qt], 0, 0, 0, 0, 0, 0);
            }
        }
        if (j < my_steps) {
            // ---- S^T = K^ Q^T (INT8, INT32 accumulation onto the float-view bias) ----
            // contraction chunk outermost: consecutive MFMAs never depend on each other
            const uint8_t *Ks = ldsK[j & 1];
#pragma unroll
            for (int ch = 0; ch < KC; ++ch) {
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const v4i a = *reinterpret_cast<const v4i *>(Ks + k_off<D>(16 * t + lq, 4 * ch + g));
#pragma unroll
                    for (int qt = 0; qt < NQ; ++qt)
                        s[qt][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, qreg[qt][ch], ch == 0 ? cinit : s[qt][t], 0, 0, 0);
                }
            }
        }
    };
    // softmax slot S(j)
    auto softmax_slot = [&](int j) {
        if (j >= my_steps) return;
        // the softmax part is the critical path of a slot (the matrix part has slack): its wavefront goes
        // first when both want the vector issue port
        __builtin_amdgcn_s_setprio(1);
        const int key0 = j * kW;
        // de-quantisation constants of the two K blocks of this step: every 32 steps each lane computes the
        // constants of one K block (c, and the exact split -K*c = kh + kl) and parks them in this wavefront's own
        // strip of LDS; a step then fetches its two blocks with two broadcast reads and no vector arithmetic
        if ((j & 31) == 0 || (SPLIT && j == jb)) {
            const int blk = min(64 * (j >> 5) + lane, nKblk - 1);
            const float c = (float)(cq * (double)dk[(size_t)bhk * nKblk + blk]);
            const float kh = -kMagicF * c;
            cst_lds[wave][lane] = make_float4(c, kh, __builtin_fmaf(-kMagicF, c, -kh), 0.0f);
        }
        const float4 k0 = cst_lds[wave][(2 * j) & 63], k1 = cst_lds[wave][(2 * j + 1) & 63];
        float c0 = k0.x, c1 = k1.x, kh0 = k0.y, kh1 = k1.y, kl0 = k0.z, kl1 = k1.z;
        const bool masked_step = (key0 + kW > Nk) || (CAUSAL && key0 + kW - 1 > row0 + shift);
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
            if (masked_step) {
                int lim = Nk - 1;  // last visible key of this lane's query row
                if constexpr (CAUSAL) lim = min(lim, row0 + qt * 16 + lq + shift);
                // last visible key of the tile's first / last row: tiles wholly at or below the former
                // need no mask, tiles wholly above the latter are invisible
                const int lim_min = CAUSAL ? min(Nk - 1, row0 + qt * 16 + shift) : Nk - 1;
                const int lim_max = CAUSAL ? min(Nk - 1, row0 + qt * 16 + 15 + shift) : Nk - 1;
                const int t_lo = min(8, max(0, (lim_min - key0 + 1) >> 4));
                const int t_hi = min(8, max(0, ((lim_max - key0) >> 4) + 1));
                if constexpr (Q4)
                    alpha[qt] = softmax_step_q4<true>(s[qt], c0, c1, log2_pr, m[qt], l[qt], pb[qt], key0 + 4 * g, lim, t_lo,
                                                      t_hi, reinterpret_cast<const float4 *>(&ds_lds[j % 3][32 * g]));
                else {
                    const float l_old = l[qt];
                    alpha[qt] = softmax_step<true>(s[qt], c0, c1, kh0, kh1, kl0, kl1, log2_pr, m[qt], l[qt], pb[qt],
                                                   key0 + 4 * g, lim, t_lo, t_hi);
                    if constexpr (SPLIT) {
                        // a row that has seen no key of this range yet and sees none in this step keeps its empty
                        // state (the step's arithmetic on (-inf) - (-inf) is undefined; its P^ is zero either way);
                        // without ranges every row sees key 0 in its first step
                        if (lim < key0 && m[qt] == -INFINITY) {
                            alpha[qt] = 1.0f;
                            l[qt] = l_old;
                        }
                    }
                }
            } else {
                if constexpr (Q4)
                    alpha[qt] = softmax_step_q4<false>(s[qt], c0, c1, log2_pr, m[qt], l[qt], pb[qt], 0, 0, 8, 8,
                                                       reinterpret_cast<const float4 *>(&ds_lds[j % 3][32 * g]));
                else
                    alpha[qt] = softmax_step<false>(s[qt], c0, c1, kh0, kh1, kl0, kl1, log2_pr, m[qt], l[qt], pb[qt], 0, 0,
                                                    8, 8);
            }
        }
        __builtin_amdgcn_s_setprio(0);
    };

    // 2*nsteps + 2 slots, one barrier each.  K^(j+1) is copied during slot 2j (the first group's M(j)) and
    // V^(j) during slot 2j+1 (the second group's M(j)); both are first read in slot 2j+2 and both target
    // buffers whose last readers finished in slot 2j-1.  Every wavefront waits for its own pieces before the
    // barrier that ends slot 2j+1.
    if (grp == 0) {
        for (int j = jb; j <= nsteps; ++j) {
            copy_k(j);  // slot 2j
            matrix_slot(j);
            __syncthreads();
            softmax_slot(j);  // slot 2j+1
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
            __syncthreads();
        }
    } else {
        __syncthreads();  // slot 0: this group idles
        for (int j = jb; j <= nsteps; ++j) {
            copy_v(j);  // slot 2j+1
            matrix_slot(j);
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
            __syncthreads();
            if (j < nsteps) {
                softmax_slot(j);  // slot 2j+2
                __syncthreads();
            }
        }
    }

    if constexpr (SPLIT) {
        // ---- the range's (m, l, acc) of every valid row; l is the sum over the row's four lanes ----
        const float lsum = rowgroup_sum(l[0]);
        const int r = row0 + lq;
        if (r < Nq) {
            const size_t prow = (((size_t)bh * n_qt + qtile) * n_splits + split) * BM + (r - wg_row0);
            if (g == 0) *reinterpret_cast<float2 *>(part_ml + prow * 2) = make_float2(m[0], lsum);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
                *reinterpret_cast<float4 *>(part_acc + prow * D + 16 * ct + 4 * g) =
                    make_float4(o[ct][0][0], o[ct][0][1], o[ct][0][2], o[ct][0][3]);
        }
        return;
    }
    // ---- epilogue: O = acc * delta_V / (P_r * l); l already carries the factor P_r ----
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        const float inv = 1.0f / rowgroup_sum(l[qt]);
        const int r = row0 + qt * 16 + lq;
        if (r < Nq) {
            uint16_t *orow = out + (bh / Hq) * o_st.b + (bh % Hq) * o_st.h + r * o_st.n;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const int c = 16 * ct + 4 * g;
                const float4 sc = *reinterpret_cast<const float4 *>(dv_lds + c);
                const float y0 = o[ct][qt][0] * (sc.x * inv), y1 = o[ct][qt][1] * (sc.y * inv);
                const float y2 = o[ct][qt][2] * (sc.z * inv), y3 = o[ct][qt][3] * (sc.w * inv);
                *reinterpret_cast<uint2 *>(orow + c) = make_uint2(pack2<BF16>(y0, y1), pack2<BF16>(y2, y3));
            }
        }
    }
#endif  // __HIP_DEVICE_COMPILE__
}

template <int D, int NQ, int NWAVE, int WPS>
hipError_t launch_d(const void *q, bool q_raw, Strides q_st, const int8_t *k_i8, const uint8_t *v_fp8, const float *q_scale,
                    const float *k_scale, const float *v_scale, void *out, Strides o_st, int B, int Hq, int Hkv, int Nq,
                    int Nk, bool causal, float sm_scale, float log2_pr, bool bf16_out, hipStream_t stream,
                    const float *q_mean, const float *dsx) {
    constexpr int BM = 16 * NQ * NWAVE;
    const int BH = B * Hq;
    const dim3 grid(BH * cdiv(Nq, BM));  // (at most 65535 * 32768 < 2^31 workgroups)
    const int nT = cdiv(Nk, kW), nQ = cdiv(Nq, kBQ), nK = cdiv(Nk, kBK);
    uint16_t *o16 = static_cast<uint16_t *>(out);
    const bool q4 = dsx != nullptr;  // the 4+8 variant (always with unquantised Q)
#define SAGE_LAUNCH(C, BF, QR, F4)                                                                               \
    attn_kernel<D, NQ, NWAVE, WPS, C, BF, QR, F4><<<grid, NWAVE * 64, 0, stream>>>(                                \
        q, k_i8, v_fp8, q_scale, k_scale, v_scale, o16, q_st, o_st, Nq, Nk, nT, nQ, nK, Hq, Hq / Hkv, sm_scale, \
        log2_pr, cdiv(Nq, BM), q_mean, dsx, 1, 0, nullptr, nullptr)
#define SAGE_LAUNCH_Q(C, BF)                                   \
    if (q4) SAGE_LAUNCH(C, BF, true, true);                    \
    else if (q_raw) SAGE_LAUNCH(C, BF, true, false);           \
    else SAGE_LAUNCH(C, BF, false, false)
    if (causal) {
        if (bf16_out) { SAGE_LAUNCH_Q(true, true); } else { SAGE_LAUNCH_Q(true, false); }
    } else {
        if (bf16_out) { SAGE_LAUNCH_Q(false, true); } else { SAGE_LAUNCH_Q(false, false); }
    }
#undef SAGE_LAUNCH_Q
#undef SAGE_LAUNCH
    return hipGetLastError();
}

// Key ranges on separate workgroups (SPLIT): grid B*Hq*tiles*S, partial results into ws (see attn_kernel).
template <int D>
hipError_t launch_split_d(const void *q, Strides q_st, const int8_t *k_i8, const uint8_t *v_fp8, const float *k_scale,
                          const float *v_scale, int B, int Hq, int Hkv, int Nq, int Nk, bool causal, float sm_scale,
                          float log2_pr, bool bf16, int n_splits, int steps_per_split, float *part_acc, float *part_ml,
                          hipStream_t stream) {
    const int nQt = cdiv(Nq, kBQ);
    const dim3 grid(B * Hq * nQt * n_splits);
    const int nT = cdiv(Nk, kW), nQ = cdiv(Nq, kBQ), nK = cdiv(Nk, kBK);
#define SAGE_SPLIT(C, BF)                                                                                          \
    attn_kernel<D, 1, 8, 4, C, BF, true, false, true><<<grid, 512, 0, stream>>>(                                    \
        q, k_i8, v_fp8, nullptr, k_scale, v_scale, nullptr, q_st, q_st, Nq, Nk, nT, nQ, nK, Hq, Hq / Hkv, sm_scale, \
        log2_pr, nQt, nullptr, nullptr, n_splits, steps_per_split, part_acc, part_ml)
    if (causal) {
        if (bf16) SAGE_SPLIT(true, true); else SAGE_SPLIT(true, false);
    } else {
        if (bf16) SAGE_SPLIT(false, true); else SAGE_SPLIT(false, false);
    }
#undef SAGE_SPLIT
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_split(const void *q, const int8_t *k_i8, const uint8_t *v_fp8, const float *k_scale,
                             const float *v_scale, int B, int Hq, int Hkv, int Nq, int Nk, int d, bool causal,
                             float sm_scale, float p_r, bool bf16, int n_splits, int steps_per_split, float *part_acc,
                             float *part_ml, hipStream_t stream) {
    const float log2_pr = (float)log2((double)p_r);
    const Strides st = contiguous_bhnd(Hq, Nq, d);
    if (d == 128)
        return launch_split_d<128>(q, st, k_i8, v_fp8, k_scale, v_scale, B, Hq, Hkv, Nq, Nk, causal, sm_scale, log2_pr,
                                   bf16, n_splits, steps_per_split, part_acc, part_ml, stream);
    return launch_split_d<64>(q, st, k_i8, v_fp8, k_scale, v_scale, B, Hq, Hkv, Nq, Nk, causal, sm_scale, log2_pr, bf16,
                              n_splits, steps_per_split, part_acc, part_ml, stream);
}

hipError_t launch_attn(const void *q, bool q_raw, Strides q_st, const int8_t *k_i8, const uint8_t *v_fp8,
                       const float *q_scale, const float *k_scale, const float *v_scale, void *out, Strides o_st, int B,
                       int Hq, int Hkv, int Nq, int Nk, int d, bool causal, float sm_scale, float p_r, bool bf16_out,
                       hipStream_t stream, const float *q_mean, const float *dsx) {
    const float log2_pr = (float)log2((double)p_r);
    // 16 query rows per wavefront, 8 wavefronts (128 rows) per workgroup, 4 wavefronts per SIMD:
    // the fastest of the measured shapes for both head dimensions (the kernel is bound by vector
    // ALU issue, and more resident wavefronts overlap MFMA and VALU work better than wider tiles)
    if (d == 128)
        return launch_d<128, 1, 8, 4>(q, q_raw, q_st, k_i8, v_fp8, q_scale, k_scale, v_scale, out, o_st, B, Hq, Hkv, Nq, Nk,
                                      causal, sm_scale, log2_pr, bf16_out, stream, q_mean, dsx);
    return launch_d<64, 1, 8, 4>(q, q_raw, q_st, k_i8, v_fp8, q_scale, k_scale, v_scale, out, o_st, B, Hq, Hkv, Nq, Nk, causal,
                                 sm_scale, log2_pr, bf16_out, stream, q_mean, dsx);
}

}  // namespace sage
