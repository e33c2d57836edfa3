// Internal launch interface between the C-ABI translation unit and the kernel
// translation units of libsage (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace sage {

constexpr int kBQ = 128;        // tokens per Q quantisation block
constexpr int kBK = 64;         // tokens per K quantisation block
constexpr int kW = 128;         // keys per online-softmax step (= V tile)
#ifndef SAGE_STAT_ROWS
#define SAGE_STAT_ROWS 1024
#endif
constexpr int kStatRows = SAGE_STAT_ROWS;  // tokens per partial column statistic

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// Element strides (batch, head, token) of a 4-D tensor whose channels are contiguous.
struct Strides {
    int64_t b, h, n;
};
inline Strides contiguous_bhnd(int H, int N, int d) { return Strides{(int64_t)H * N * d, (int64_t)N * d, (int64_t)d}; }

// Scratch of the quantisation stage (all offsets 256-byte aligned).
struct QuantScratch {
    double *k_sum_part;  // [B*H][chunks][d]  partial column sums of K
    float *v_max_part;   // [B*H][chunks][d]  partial column max|V|
    float *v_rcp;        // [B*H][d]          V_r / max|V|
    size_t bytes;
};
QuantScratch quant_scratch_layout(void *base, int B, int H, int N, int d);

// stage 1 launches (sage_quant.hip)
// (the inputs are read through their strides; every output is contiguous [B,H,...])
hipError_t launch_quant_q(const void *q, Strides q_st, int8_t *q_i8, float *q_scale, int B, int H, int N, int d,
                          bool bf16, hipStream_t stream);
hipError_t launch_quant_k(const void *k, Strides k_st, int8_t *k_i8, float *k_scale, float *k_mean, int B, int H,
                          int N, int d, bool bf16, hipStream_t stream, const QuantScratch &ws);
hipError_t launch_quant_v(const void *v, Strides v_st, uint8_t *v_fp8, float *v_scale, float v_r, int B, int H, int N,
                          int d, bool bf16, hipStream_t stream, const QuantScratch &ws);

// K and V of the same shape together: three launches instead of six, identical results
// (int4: the K codes of the 4+8 variant, range [-7, 7], one per byte)
hipError_t launch_quant_kv(const void *k, Strides k_st, const void *v, Strides v_st, int8_t *k_i8, float *k_scale,
                           float *k_mean, uint8_t *v_fp8, float *v_scale, float v_r, int B, int H, int N, int d,
                           bool bf16, hipStream_t stream, const QuantScratch &ws, bool int4 = false);

// Which kernels launch_quant_kv uses: 0 = by shape (the single-read kernel up to 128 workgroups per head),
// 1 = always the three launches (statistics, finalize, codes), 2 = always the single-read kernel (error above 256
// workgroups per head).  wait_ticks: how long a workgroup of the single-read kernel waits for its partners before
// it computes the head's statistic alone (100 MHz ticks; negative: no wait).  Process-wide.
void set_quant_kv_path(int path, long long wait_ticks);

// 4+8 variant.  Block means of Q ([B,H,ceil(N/kBQ),d]); with q_i4 != NULL also the stand-alone INT4 codes and
// scales of Q minus its block means.
hipError_t launch_quant_q4(const void *q, Strides q_st, float *q_mean, int8_t *q_i4, float *q_scale, int B, int H, int N,
                           int d, bool bf16, hipStream_t stream);
// The score correction qbar K'^T in exponent units, [B*Hq][ceil(Nq/kBQ)][ceil(Nk/kW)][128] floats in the attention
// kernel's lane order (see delta_s_kernel).
hipError_t launch_delta_s(const void *k, Strides k_st, const float *k_mean, const float *q_mean, float *dsx, int B,
                          int Hq, int Hkv, int Nq, int Nk, int d, bool causal, float sm_scale, bool bf16,
                          hipStream_t stream);

// stage 2 launch (sage_attn.hip): Hq query heads over Hkv K/V heads, Nq query rows over Nk keys.
// q_raw = false: q is Q^ (int8) with scales q_scale; q_raw = true: q is the unquantised 16-bit Q
// (type of the output), quantised inside the kernel, q_scale unused.  q and out are addressed
// through their strides; K^, V^ and the scales are contiguous.
// dsx != NULL selects the 4+8 variant: q is the unquantised Q, k_i8 holds INT4 codes, q_mean the block means of Q
// (launch_quant_q4) and dsx the score correction (launch_delta_s).
hipError_t launch_attn(const void *q, bool q_raw, Strides q_st, const int8_t *k_i8, const uint8_t *v_fp8, const float *q_scale,
                       const float *k_scale, const float *v_scale, void *out, Strides o_st, int B, int Hq, int Hkv,
                       int Nq, int Nk, int d, bool causal, float sm_scale, float p_r, bool bf16_out,
                       hipStream_t stream, const float *q_mean = nullptr, const float *dsx = nullptr);

// Decode-shaped attention (sage_decode.hip): (Hq/Hkv)*Nq <= 64 query rows per K/V head in T = ceil(rows/16) row
// tiles, the keys cut into ranges of `steps_per_split` key steps; one wavefront per (batch, K/V head, range, row
// tile) writes its (m, l, acc) per row into the scratch, a second launch combines the ranges.  q and out are
// contiguous [B,Hq,Nq,d].
struct DecodeScratch {
    float *part_acc;  // [B*Hkv][S][T][16][d]  un-normalised outputs of every range
    float *part_ml;   // [B*Hkv][S][T][16][2]  running maximum and sum of every range
    int n_splits;     // S = ceil(ceil(Nk/128) / steps_per_split)
    size_t bytes;
};
int decode_auto_steps_per_split(int B, int Hkv, int Nk);
DecodeScratch decode_scratch_layout(void *base, int B, int Hkv, int Nk, int d, int steps_per_split, int row_tiles);
hipError_t launch_decode(const void *q, const int8_t *k_i8, const uint8_t *v_fp8, const float *k_scale,
                         const float *v_scale, void *out, int B, int Hq, int Hkv, int Nq, int Nk, int d, bool causal,
                         float sm_scale, float p_r, int steps_per_split, bool bf16, hipStream_t stream,
                         const DecodeScratch &ws);

// The same idea for calls with more than 64 query rows per K/V head but too few (head, query tile) pairs to fill
// the GPU: attn_kernel with its key steps cut into ranges on separate workgroups (sage_attn.hip), then the
// combination launch of sage_decode.hip.  Partial results: [B*Hq*tiles][S][128 rows][d] and [...][2] floats.
hipError_t launch_attn_split(const void *q, const int8_t *k_i8, const uint8_t *v_fp8, const float *k_scale,
                             const float *v_scale, int B, int Hq, int Hkv, int Nq, int Nk, int d, bool causal,
                             float sm_scale, float p_r, bool bf16, int n_splits, int steps_per_split, float *part_acc,
                             float *part_ml, hipStream_t stream);
int ranges_auto_steps_per_split(int B, int Hq, int Nq, int Nk);
DecodeScratch ranges_scratch_layout(void *base, int B, int Hq, int Nq, int Nk, int d, int steps_per_split);
hipError_t launch_attn_ranges(const void *q, const int8_t *k_i8, const uint8_t *v_fp8, const float *k_scale,
                              const float *v_scale, void *out, int B, int Hq, int Hkv, int Nq, int Nk, int d, bool causal,
                              float sm_scale, float p_r, int steps_per_split, bool bf16, hipStream_t stream,
                              const DecodeScratch &ws);

}  // namespace sage
