/*
 * libsage -- SageAttention2++ "8+8" quantised attention forward for AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer named "device" is a device (HBM) pointer owned by the
 * caller; the library allocates nothing, never synchronises and enqueues all
 * its work on `stream` (a hipStream_t passed as void*; NULL = the default
 * stream).  Inputs are never modified.  The only state it keeps is, per
 * calling thread, the HIP error code behind the last SAGE_EHIP (read by
 * sage_strerror); a call that enqueues kernels discards a HIP error left
 * pending on the thread by earlier, unrelated HIP calls.
 *
 * Tensors.  Q, K, V and the output are contiguous [B, H, N, d] arrays of a
 * 16-bit floating type (`sage_dtype`), d in {64, 128}, 1 <= N <= 2^22 arbitrary
 * (not a multiple of anything), B*H <= 65535; larger sizes return SAGE_EINVAL.  The
 * plain entry points take N_q = N_k = N and H_q = H_kv = H; the *_gqa entry
 * points take Q/out as [B, Hq, Nq, d] and K/V as [B, Hkv, Nk, d], Hq a multiple
 * of Hkv (query head h uses K/V head h / (Hq/Hkv)).
 *
 * The method (paper sections in brackets):
 *   stage 1  K is smoothed by subtracting its per-(b,h,channel) mean over the
 *            N tokens [Sec. 3]; Q and the smoothed K are quantised to INT8 per
 *            block of SAGE_BQ / SAGE_BK consecutive tokens with scale
 *            delta = max|X| / 127 [Sec. 2.1]; V is quantised to FP8 E4M3 per
 *            channel with scale delta_V = max_n|V| / V_r [Sec. 2.1, Eq. 2].
 *   stage 2  per query block, key steps of SAGE_W keys in ascending order:
 *            S = Q^ K^T in INT8 with INT32 accumulation, de-quantised by
 *            delta_Q delta_K, base-2 online softmax, P~ quantised to FP8 E4M3
 *            as P^ = rne(P~ * P_r), O += P^ V^ in FP8 with FP32 accumulation;
 *            finally O * delta_V / (P_r * l) [Sec. 2.1, Sec. 3.1].
 * Rounding is round-to-nearest-even everywhere; each quantiser step is one
 * IEEE binary32 operation (x - mean, a / range, range / a, x * r), which is
 * what makes codes and scales reproducible bit for bit.
 *
 * Return value of every call: SAGE_OK (0) or a negative error code; nothing
 * is enqueued when an argument check fails.  No exceptions, no aborts.
 */
#ifndef SAGE_H
#define SAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SAGE_BQ 128      /* tokens per Q quantisation block  [Sec. 2.1 "per-block"] */
#define SAGE_BK 64       /* tokens per K quantisation block  */
#define SAGE_W 128       /* keys consumed per online-softmax step */
#define SAGE_VTILE 128   /* keys per tile of the transposed FP8 V layout */
#define SAGE_STATIC_SCRATCH_BYTES (8u << 20) /* scratch built into the library for sage_quant_kv_static */

typedef enum { SAGE_F16 = 0, SAGE_BF16 = 1 } sage_dtype;

enum {
    SAGE_OK = 0,
    SAGE_EINVAL = -1,     /* NULL pointer, d not in {64,128}, size out of range, pointer not 16-byte aligned */
    SAGE_EWORKSPACE = -2, /* workspace missing or smaller than the matching *_workspace_bytes() */
    SAGE_EHIP = -3,       /* a kernel launch failed; text from sage_strerror() */
    SAGE_ESCRATCH = -4    /* sage_quant_kv_static: the problem needs more than SAGE_STATIC_SCRATCH_BYTES */
};

typedef struct {
    int bq, bk, w, v_tile; /* SAGE_BQ, SAGE_BK, SAGE_W, SAGE_VTILE */
    float p_r, v_r;        /* default FP8 ranges, 224 and 4.5 [Sec. 3.2] */
} sage_params;

/* Report the fixed blocking and the default ranges.  Host call. */
int sage_get_params(sage_params *out);

/* Human-readable text for a return code (static storage, never NULL). */
const char *sage_strerror(int code);

/* ---- sizes (host calls, no GPU work) ----------------------------------- */

/* Bytes of the transposed FP8 V buffer: B*H*ceil(N/128)*d*128. */
size_t sage_v_fp8_bytes(int B, int H, int N, int d);
/* Scratch needed by sage_quant_qk / sage_quant_v (partial column statistics). */
size_t sage_quant_workspace_bytes(int B, int H, int N, int d);
/* Scratch needed by sage_attn_fwd (quantised operands + scales + the above). */
size_t sage_workspace_bytes(int B, int H, int N, int d);
/* Same for sage_attn_fwd_gqa. */
size_t sage_workspace_bytes_gqa(int B, int Hq, int Hkv, int Nq, int Nk, int d);

/* ---- stage 1 ----------------------------------------------------------- */

/*
 * K smoothing + per-block INT8 quantisation of Q and K  [Sec. 3; Sec. 2.1].
 *   q, k      device, [B,H,N,d] of `dt`                                  (in)
 *   q_i8,k_i8 device, [B,H,N,d] int8 codes in [-127,127]                 (out)
 *   q_scale   device, [B,H,ceil(N/SAGE_BQ)] float, delta_Q               (out)
 *   k_scale   device, [B,H,ceil(N/SAGE_BK)] float, delta_K               (out)
 *   k_mean    device, [B,H,d] float, the subtracted mean                 (out)
 *   workspace device, >= sage_quant_workspace_bytes(), 256-byte aligned (scratch)
 * mean = float(sum_n K / N) with the sum in double; K' = K - mean;
 * a = max|K'| over the valid rows of a block; delta = a / 127;
 * code = rne(K' * (127 / a)); a == 0 gives delta 0 and codes 0.
 */
int sage_quant_qk(const void *q, const void *k, int8_t *q_i8, int8_t *k_i8,
                  float *q_scale, float *k_scale, float *k_mean,
                  int B, int H, int N, int d, sage_dtype dt, void *stream,
                  void *workspace, size_t workspace_bytes);

/*
 * The two halves of sage_quant_qk as separate calls, for inputs whose Q and K
 * differ in head count or length (grouped-query attention, cross-attention,
 * the models of Sec. 4.1 with fewer K/V heads than query heads).  Arguments,
 * arithmetic and error behaviour as above; sage_quant_q needs no workspace.
 */
int sage_quant_q(const void *q, int8_t *q_i8, float *q_scale,
                 int B, int H, int N, int d, sage_dtype dt, void *stream);
int sage_quant_k(const void *k, int8_t *k_i8, float *k_scale, float *k_mean,
                 int B, int H, int N, int d, sage_dtype dt, void *stream,
                 void *workspace, size_t workspace_bytes);

/*
 * Per-channel FP8 E4M3 quantisation of V  [Sec. 2.1; Sec. 3.1 Eq. 2].
 *   v        device, [B,H,N,d] of `dt`                                   (in)
 *   v_fp8    device, sage_v_fp8_bytes() bytes                            (out)
 *   v_scale  device, [B,H,d] float, delta_V = max_n|V| / v_r             (out)
 * code = e4m3_rne(V * (v_r / a_c)); a_c == 0 gives delta 0 and codes 0.
 *
 * Layout of v_fp8 (private to this library but documented, because the codes
 * are part of the parity contract): [B*H][T = ceil(N/128)][d][128] bytes; the
 * 128 bytes of (tile T, channel c) hold the 128 keys of the tile permuted so
 * that byte 64*(t>>2) + 16*g + 4*(t&3) + i is key 128*T + 16*t + 4*g + i
 * (t<8, g<4, i<4); keys >= N hold code 0.
 */
int sage_quant_v(const void *v, uint8_t *v_fp8, float *v_scale, float v_r,
                 int B, int H, int N, int d, sage_dtype dt, void *stream,
                 void *workspace, size_t workspace_bytes);

/*
 * sage_quant_k and sage_quant_v for K and V of one shape in one call  [same passages]:
 * the two tensors share their launches (three kernels instead of six); every output
 * is bit-identical to the separate calls.  Arguments as for those two calls.
 */
int sage_quant_kv(const void *k, const void *v, int8_t *k_i8, float *k_scale, float *k_mean,
                  uint8_t *v_fp8, float *v_scale, float v_r,
                  int B, int H, int N, int d, sage_dtype dt, void *stream,
                  void *workspace, size_t workspace_bytes);

/*
 * sage_quant_kv for callers that cannot allocate and have no workspace to hand over: code recorded
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same
 * outputs bit for bit; the scratch (partial column statistics, 12 bytes per channel and per 256 tokens
 * (d = 128) or 512 tokens (d = 64) of every head) lives in a static device array inside the library, SAGE_STATIC_SCRATCH_BYTES (8 MiB)
 * per GPU, which each GPU the library runs on holds until the process ends.  The call allocates nothing
 * and frees nothing; on its first use on a device it looks up that device's copy of the array (the
 * device must be current, as for every call).  Arguments as for sage_quant_kv, without the workspace.
 *   returns SAGE_ESCRATCH when sage_quant_workspace_bytes(B,H,N,d) > SAGE_STATIC_SCRATCH_BYTES
 *           (nothing is enqueued; use sage_quant_kv), otherwise as sage_quant_kv.
 * All calls on one GPU share that GPU's array: the scratch keeps the last call's contents (what has to
 * start at zero is cleared by a fill kernel of the same call, everything else is written before it is read), and two calls that
 * overlap on one GPU -- different streams, or different threads -- race on it.  Calls on one stream,
 * and calls on different GPUs, are safe.
 */
int sage_quant_kv_static(const void *k, const void *v, int8_t *k_i8, float *k_scale, float *k_mean,
                         uint8_t *v_fp8, float *v_scale, float v_r,
                         int B, int H, int N, int d, sage_dtype dt, void *stream);

/* ---- stage 2 ----------------------------------------------------------- */

/*
 * Fused attention on already quantised operands  [Sec. 2.1; Sec. 3.1].
 * Arguments as produced by sage_quant_qk / sage_quant_v (same layouts);
 *   out      device, [B,H,N,d] of `out_dt`; every element is written     (out)
 *   causal   0: all keys visible; 1: key n visible to query r iff n <= r;
 *            key tiles entirely above the diagonal are skipped
 *   sm_scale softmax scale; anything but a positive finite number (0, negative,
 *            NaN, infinity) selects 1/sqrt(d)
 *   p_r      FP8 range of P~ (224 by default), must lie in (0, 448]
 * The running maximum is updated once per SAGE_W keys to the exact step
 * maximum; l accumulates the unquantised P~.
 */
int sage_attn_fwd_quantized(const int8_t *q_i8, const int8_t *k_i8, const uint8_t *v_fp8,
                            const float *q_scale, const float *k_scale, const float *v_scale,
                            void *out, int B, int H, int N, int d, int causal, float sm_scale,
                            float p_r, sage_dtype out_dt, void *stream);

/*
 * Generalisation of sage_attn_fwd_quantized  [same passages]: Hq query heads over
 * Hkv K/V heads (Hq % Hkv == 0), Nq query rows over Nk keys.
 *   q_i8, q_scale, out   [B,Hq,Nq,d], [B,Hq,ceil(Nq/SAGE_BQ)], [B,Hq,Nq,d]
 *   k_i8, k_scale        [B,Hkv,Nk,d], [B,Hkv,ceil(Nk/SAGE_BK)]
 *   v_fp8, v_scale       sage_v_fp8_bytes(B,Hkv,Nk,d) bytes, [B,Hkv,d]
 *   causal   the mask is aligned to the END of both sequences: key n is visible
 *            to query r iff n <= r + (Nk - Nq); requires Nk >= Nq (SAGE_EINVAL otherwise)
 */
int sage_attn_fwd_quantized_gqa(const int8_t *q_i8, const int8_t *k_i8, const uint8_t *v_fp8,
                                const float *q_scale, const float *k_scale, const float *v_scale,
                                void *out, int B, int Hq, int Hkv, int Nq, int Nk, int d, int causal,
                                float sm_scale, float p_r, sage_dtype out_dt, void *stream);

/*
 * Fused attention on quantised K^, V^ and UNQUANTISED Q  [Sec. 2.1; Sec. 3.1]: the
 * per-block INT8 quantisation of Q (blocks of SAGE_BQ rows, delta = max|Q|/127,
 * round to nearest even) runs in the prologue of the attention kernel, whose
 * workgroups own exactly one Q block each; Q^ and delta_Q are the same bits
 * sage_quant_q would produce, but are never written to memory.  Output and every
 * other argument as for sage_attn_fwd_quantized_gqa;
 *   q        device, [B,Hq,Nq,d] of `dt`, 16-byte aligned                 (in)
 *   out      device, [B,Hq,Nq,d] of `dt`                                  (out)
 * Returns SAGE_EINVAL / SAGE_EHIP like the other stage-2 calls.
 */
int sage_attn_fwd_kvquantized_gqa(const void *q, const int8_t *k_i8, const uint8_t *v_fp8,
                                  const float *k_scale, const float *v_scale, void *out,
                                  int B, int Hq, int Hkv, int Nq, int Nk, int d, int causal,
                                  float sm_scale, float p_r, sage_dtype dt, void *stream);

/*
 * The whole forward pass: sage_quant_kv + sage_attn_fwd_kvquantized_gqa
 * with the default ranges (P_r = 224, V_r = 4.5), intermediates in `workspace`
 * (device, >= sage_workspace_bytes(), 256-byte aligned).  The result is bit-identical
 * to sage_quant_qk + sage_quant_v + sage_attn_fwd_quantized.
 *   q, k, v  device, [B,H,N,d] of `dt`                                   (in)
 *   out      device, [B,H,N,d] of `dt`                                   (out)
 */
int sage_attn_fwd(const void *q, const void *k, const void *v, void *out,
                  int B, int H, int N, int d, int causal, float sm_scale, void *stream,
                  sage_dtype dt, void *workspace, size_t workspace_bytes);

/*
 * The whole forward pass for grouped-query / cross attention: sage_quant_kv +
 * sage_attn_fwd_kvquantized_gqa, default ranges,
 * workspace >= sage_workspace_bytes_gqa().
 */
int sage_attn_fwd_gqa(const void *q, const void *k, const void *v, void *out,
                      int B, int Hq, int Hkv, int Nq, int Nk, int d, int causal, float sm_scale,
                      void *stream, sage_dtype dt, void *workspace, size_t workspace_bytes);

/*
 * The whole forward pass on strided tensors  [same passages as sage_attn_fwd]: the
 * four tensors may be any views whose channel dimension is contiguous, e.g. the
 * token-major [B,N,H,d] layout or slices of a packed QKV projection; nothing is
 * copied, the kernels read and write through the strides.
 *   *_strides  host pointers to three ELEMENT strides {batch, head, token}; NULL means
 *              contiguous [B,H,N,d].  Inputs: every stride >= 0, <= 2^40 and a multiple of 8
 *              (16-byte aligned rows; 0 broadcasts that dimension).  Output: the same,
 *              and no two rows may overlap.  SAGE_EINVAL otherwise.
 * All other arguments, the workspace and the result (bit-identical to sage_attn_fwd_gqa
 * on contiguous copies) as for sage_attn_fwd_gqa.  The stride arrays are read before the
 * call returns.
 */
int sage_attn_fwd_strided(const void *q, const void *k, const void *v, void *out,
                          int B, int Hq, int Hkv, int Nq, int Nk, int d,
                          const int64_t *q_strides, const int64_t *k_strides,
                          const int64_t *v_strides, const int64_t *out_strides,
                          int causal, float sm_scale, void *stream, sage_dtype dt,
                          void *workspace, size_t workspace_bytes);

/* ---- the 4+8 variant: INT4 Q K^T with smoothing of Q and K, FP8 P V ------------------------------------
 *
 * [Sec. 2.1 "INT4/INT8 with per-block granularity"; Sec. 3 "smoothing of Q and K"; Sec. 4.1 "SageAttn2++(4+8)".]
 * The paper names the ingredients and prints no formula for them; this library takes:
 *   INT4 codes   integers in [-7, 7], delta = max|X| / 7, same blocks and binary32 steps as the INT8 quantiser,
 *                stored one code per byte (gfx950 has no INT4 matrix instruction: the codes run through the
 *                INT8 one, so the variant buys no speed here and exists for completeness and accuracy studies);
 *   K smoothing  as in 8+8 (per-head channel mean over all tokens);
 *   Q smoothing  the mean of each block of SAGE_BQ query rows, per channel, over the block's valid rows
 *                (double sum, one rounding to binary32), subtracted with one binary32 operation;
 *   correction   what the Q smoothing removed is put back on the scores in full precision:
 *                S = delta_Q delta_K Q^ K^^T + qbar_i . K'[n],  K' = K - mean_K (unquantised, FP32 here);
 *   everything after the scores (online softmax, P~ to FP8, P^ V^, epilogue) as in 8+8.
 * All calls take the grouped-query shapes of sage_attn_fwd_gqa (Hq = Hkv, Nq = Nk for plain self-attention).
 */

/* Bytes of the score-correction buffer: B*Hq*ceil(Nq/SAGE_BQ)*ceil(Nk/128)*128 floats (0: invalid sizes). */
size_t sage_delta_s_bytes(int B, int Hq, int Nq, int Nk);
/* Scratch needed by sage_attn_fwd_4bit. */
size_t sage_workspace_bytes_4bit(int B, int Hq, int Hkv, int Nq, int Nk, int d);

/*
 * Block means of Q and, optionally, the stand-alone INT4 codes of Q minus its block means.
 *   q       device, [B,H,N,d] of `dt`                                              (in)
 *   q_mean  device, [B,H,ceil(N/SAGE_BQ),d] float                                  (out)
 *   q_i4    device, [B,H,N,d] int8 codes in [-7,7], or NULL                        (out)
 *   q_scale device, [B,H,ceil(N/SAGE_BQ)] float, NULL exactly when q_i4 is NULL    (out)
 * (The attention call quantises Q itself from q and q_mean; the stand-alone codes exist so that they can be
 * compared bit for bit.)
 */
int sage_quant_q4(const void *q, float *q_mean, int8_t *q_i4, float *q_scale,
                  int B, int H, int N, int d, sage_dtype dt, void *stream);

/* sage_quant_kv with INT4 codes for K (range [-7,7], one per byte); V as in 8+8.  Arguments as sage_quant_kv. */
int sage_quant_kv4(const void *k, const void *v, int8_t *k_i4, float *k_scale, float *k_mean,
                   uint8_t *v_fp8, float *v_scale, float v_r,
                   int B, int H, int N, int d, sage_dtype dt, void *stream,
                   void *workspace, size_t workspace_bytes);

/*
 * The score correction in the units of the softmax exponent:
 *   dsx[b,hq,i,T,pos] = (sum_c q_mean[b,hq,i,c] * (K[b,hkv,n,c] - k_mean[b,hkv,c])) * sm_scale * log2(e)
 * for Q block i and key n = 128*T + 16*t + 4*g + j stored at pos = 32*g + 4*t + j (the order in which a lane
 * of the attention kernel holds its scores); keys >= Nk hold 0.  FP32 arithmetic.
 *   k       device, [B,Hkv,Nk,d] of `dt` (the unquantised keys)       (in)
 *   k_mean  device, [B,Hkv,d] float, from sage_quant_kv4              (in)
 *   q_mean  device, [B,Hq,ceil(Nq/SAGE_BQ),d] float                   (in)
 *   dsx     device, sage_delta_s_bytes() bytes                        (out)
 *   causal  1: (Q block, key tile) pairs the end-aligned mask hides completely may be left unwritten
 *   sm_scale as for the attention calls (the same value must be passed there)
 */
int sage_delta_s(const void *k, const float *k_mean, const float *q_mean, float *dsx,
                 int B, int Hq, int Hkv, int Nq, int Nk, int d, int causal, float sm_scale,
                 sage_dtype dt, void *stream);

/*
 * Fused attention of the 4+8 variant on unquantised Q (smoothed and quantised to INT4 in the kernel's prologue
 * with the block means given), INT4 K^, FP8 V^ and the score correction.  Output, mask, sm_scale, p_r as for
 * sage_attn_fwd_kvquantized_gqa.
 */
int sage_attn_fwd_q4(const void *q, const float *q_mean, const int8_t *k_i4, const uint8_t *v_fp8,
                     const float *k_scale, const float *v_scale, const float *dsx, void *out,
                     int B, int Hq, int Hkv, int Nq, int Nk, int d, int causal, float sm_scale, float p_r,
                     sage_dtype dt, void *stream);

/*
 * The whole forward pass of the 4+8 variant: sage_quant_kv4 + sage_quant_q4 (means only) + sage_delta_s +
 * sage_attn_fwd_q4 with the default ranges; workspace >= sage_workspace_bytes_4bit(), 256-byte aligned.
 */
int sage_attn_fwd_4bit(const void *q, const void *k, const void *v, void *out,
                       int B, int Hq, int Hkv, int Nq, int Nk, int d, int causal, float sm_scale,
                       void *stream, sage_dtype dt, void *workspace, size_t workspace_bytes);

/* ---- decode-shaped calls ---------------------------------------------- */

/*
 * Attention of few query rows over a long, already quantised key sequence: calls whose (head, query tile) pairs
 * alone cannot fill the GPU (the paper does not treat this shape; a key step is evaluated exactly as in
 * sage_attn_fwd_kvquantized_gqa, Sec. 2.1 / Sec. 3.1).  The keys are cut into ranges of `split_keys` keys that are
 * evaluated independently -- each from an empty running maximum, so P~ is rounded to FP8 against the maximum of
 * its RANGE -- and then combined as partial softmax sums (m = max m_s, l = sum 2^(m_s - m) l_s, O likewise).  With
 * one range (split_keys >= Nk) the result is that of sage_attn_fwd_kvquantized_gqa bit for bit; with more it differs
 * from it by FP8 rounding decisions only.
 * Up to (Hq/Hkv) * Nq = 64 query rows per K/V head, the rows of all query heads that share a K/V head are packed
 * into MFMA tiles of 16 and one wavefront takes one (K/V head, range, row tile), reading K^ and V^ straight from
 * global memory; above that the prefill kernel runs with its key steps cut into ranges, one workgroup per
 * (head, query tile, range).
 *   q, out      device, [B,Hq,Nq,d] contiguous, 16-bit type `dt`; Q is quantised inside (per head and block of 128
 *               rows, as everywhere)
 *   k_i8 .. v_scale   device, as produced by sage_quant_k / sage_quant_v (or sage_quant_kv) for [B,Hkv,Nk,d]
 *   causal      mask aligned to the end of both sequences (key n visible to row r iff n <= r + Nk - Nq)
 *   split_keys  keys per range: a positive multiple of 128, or 0 for the library's choice, which
 *               sage_decode_split_keys(B, Hq, Hkv, Nq, Nk) reports (about four wavefronts, or workgroups, per CU
 *               over the launch); a caller whose results must not depend on the batch size passes its own
 *   workspace   device, 256-byte aligned, >= sage_decode_workspace_bytes(B, Hq, Hkv, Nq, Nk, d, split_keys): the
 *               ranges' partial results; nothing in it has to be initialised
 * Returns SAGE_EINVAL for a split_keys that is negative or no multiple of 128 and for the argument errors of the
 * other entry points; SAGE_EWORKSPACE; SAGE_EHIP.  Two launches (ranges, combination); allocates nothing, does not
 * synchronise.
 */
int sage_decode_split_keys(int B, int Hq, int Hkv, int Nq, int Nk);
size_t sage_decode_workspace_bytes(int B, int Hq, int Hkv, int Nq, int Nk, int d, int split_keys);
int sage_attn_fwd_decode(const void *q, const int8_t *k_i8, const uint8_t *v_fp8,
                         const float *k_scale, const float *v_scale, void *out,
                         int B, int Hq, int Hkv, int Nq, int Nk, int d, int causal, float sm_scale, float p_r,
                         int split_keys, sage_dtype dt, void *stream, void *workspace, size_t workspace_bytes);

/* ---- measurement aid -------------------------------------------------- */

/*
 * Not a step of the method: launches a kernel that only issues the matrix instructions of the attention
 * kernel, back to back on independent accumulators (4 wavefronts per workgroup, 8 accumulators each,
 * `iters` rounds), so that a benchmark can time it (events on `stream`) and state throughput against the
 * matrix-pipe rate the GPU at hand sustains, next to the published peak.
 *   kind   0: INT8 16x16x64 (the Q^ K^T product), 1: FP8 16x16x128 (the P^ V^ product),
 *          2: the older FP8 16x16x32 form, 3: the attention kernel's mix (two of kind 0 per one of kind 1)
 *   sink   device, one float (never written in practice; keeps the arithmetic alive)
 *   ops_per_launch  host, receives the operation count (2 per multiply-add) of the launch
 * Returns SAGE_EINVAL for a bad argument, SAGE_EHIP if the launch failed.
 */
int sage_diag_mfma_rate(int kind, int iters, int workgroups, float *sink, double *ops_per_launch, void *stream);

/*
 * Not a step of the method: selects, process-wide, which kernels the K/V quantisers (sage_quant_kv,
 * sage_quant_kv_static, sage_quant_kv4 and the whole-pass entry points) launch.  Both choices compute the same
 * codes, scales and mean (Sec. 2.1, Sec. 3).
 *   path        0 (default): by shape — the single-read kernel (K and V are read once: the workgroups of a head
 *               keep 64 KiB of tokens each in registers, exchange their partial column statistics through the
 *               workspace and then write the codes) when a head is at most 128 such workgroups (32768 tokens at
 *               d = 128, 65536 at d = 64), the three launches (statistics, finalize, codes; K and V read twice)
 *               above that; 1: always the three launches; 2: always the single-read kernel (calls then fail with
 *               SAGE_EHIP above 256 workgroups per head)
 *   wait_ticks  how long a workgroup of the single-read kernel waits for the partials of its partners before it
 *               computes the head's statistic alone from global memory (same result), in ticks of the GPU's
 *               constant 100 MHz clock; negative: it does not wait at all (for tests of that branch); the
 *               default is 50 000 (0.5 ms; partners normally arrive within microseconds)
 * Returns SAGE_EINVAL for a path outside 0..2.  For benchmarks and tests; a production caller leaves it alone.
 */
int sage_diag_quant_kv_path(int path, long long wait_ticks);

#ifdef __cplusplus
}
#endif
#endif /* SAGE_H */
