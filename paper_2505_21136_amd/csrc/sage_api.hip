// C ABI of libsage (declared in include/sage.h): argument checks, workspace
// carving and kernel launches.  No allocation, no synchronisation; the only
// state is the last HIP error code of the calling thread (for sage_strerror).
// A call that enqueues kernels first discards whatever error an earlier,
// unrelated HIP call of this thread left pending, so that SAGE_EHIP always
// speaks of this call's own launches.
#include "../../include/sage.h"
#include "sage_internal.h"

#include <math.h>

#include <mutex>

namespace {

thread_local hipError_t g_last_hip_error = hipSuccess;

// Scratch of sage_quant_kv_static: device memory that belongs to the library's code object, one copy per
// GPU, alive until the process ends.  In host code the array's NAME is only a handle for
// hipGetSymbolAddress; the address kernels can use is looked up once per device and kept in
// g_scratch_ptr, and only that pointer is ever handed to a launch.
static __device__ __align__(256) unsigned char scratch[SAGE_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// The current device's copy of `scratch` (NULL + error code on failure).  Allocates nothing.
hipError_t static_scratch(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned256(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }
bool shape_ok(int B, int H, int N, int d) {
    return B >= 1 && H >= 1 && N >= 1 && N <= (1 << 22) && (d == 64 || d == 128) && (size_t)B * H <= 65535u;
}
bool gqa_ok(int B, int Hq, int Hkv, int Nq, int Nk, int d, int causal) {
    return shape_ok(B, Hq, Nq, d) && shape_ok(B, Hkv, Nk, d) && Hq % Hkv == 0 && (!causal || Nk >= Nq);
}
bool dtype_ok(sage_dtype dt) { return dt == SAGE_F16 || dt == SAGE_BF16; }

// Caller-supplied element strides (batch, head, token); NULL selects contiguous [B,H,N,d].
// Inputs: non-negative multiples of 8 elements (rows stay 16-byte aligned; 0 broadcasts), at most 2^40.
bool read_strides(const int64_t *s, int H, int N, int d, sage::Strides *out) {
    if (!s) {
        *out = sage::contiguous_bhnd(H, N, d);
        return true;
    }
    for (int i = 0; i < 3; ++i)
        if (s[i] < 0 || s[i] % 8 != 0 || s[i] > ((int64_t)1 << 40)) return false;  // (bounded: offsets stay far from 2^63)
    *out = sage::Strides{s[0], s[1], s[2]};
    return true;
}
// Output: additionally no two (b, h, n) rows may overlap -- sorted by stride, every stride must
// cover the extent of the next smaller one (dimensions of extent 1 do not matter).
bool write_strides_ok(const sage::Strides &st, int B, int H, int N, int d) {
    int64_t stride[3] = {st.b, st.h, st.n};
    int64_t extent[3] = {B, H, N};
    for (int i = 0; i < 3; ++i)
        for (int j = i + 1; j < 3; ++j)
            if (stride[j] < stride[i]) {
                const int64_t ts = stride[i], te = extent[i];
                stride[i] = stride[j], extent[i] = extent[j];
                stride[j] = ts, extent[j] = te;
            }
    int64_t span = d;  // elements covered by everything below the current dimension
    for (int i = 0; i < 3; ++i) {
        if (extent[i] == 1) continue;
        if (stride[i] < span) return false;
        span = stride[i] * extent[i];
    }
    return true;
}
int from_hip(hipError_t e) {
    if (e == hipSuccess) return SAGE_OK;
    g_last_hip_error = e;
    return SAGE_EHIP;
}
// Called after the argument checks, right before the first launch of an entry point.
void discard_pending_hip_error() { (void)hipGetLastError(); }
// sm_scale as given when it is a positive finite number, 1/sqrt(d) otherwise (0, negative, NaN, infinity)
float scale_or_default(float sm_scale, int d) {
    return (isfinite(sm_scale) && sm_scale > 0.0f) ? sm_scale : 1.0f / sqrtf((float)d);
}

// Carving of the sage_attn_fwd workspace.
struct FwdWorkspace {
    int8_t *k_i8;
    uint8_t *v_fp8;
    float *k_scale, *v_scale, *k_mean;
    void *quant;
    size_t quant_bytes;
    size_t bytes;
};
FwdWorkspace fwd_layout(void *base, int B, int Hq, int Hkv, int Nq, int Nk, int d) {
    (void)Hq, (void)Nq;  // Q is quantised inside the attention kernel: nothing of it is staged
    const size_t Ek = (size_t)B * Hkv * Nk * d, BHk = (size_t)B * Hkv;
    char *p = static_cast<char *>(base);
    size_t off = 0;
    FwdWorkspace w;
    w.k_i8 = reinterpret_cast<int8_t *>(p + off);
    off += align256(Ek);
    w.v_fp8 = reinterpret_cast<uint8_t *>(p + off);
    off += align256(sage_v_fp8_bytes(B, Hkv, Nk, d));
    w.k_scale = reinterpret_cast<float *>(p + off);
    off += align256(BHk * sage::cdiv(Nk, sage::kBK) * sizeof(float));
    w.v_scale = reinterpret_cast<float *>(p + off);
    off += align256(BHk * d * sizeof(float));
    w.k_mean = reinterpret_cast<float *>(p + off);
    off += align256(BHk * d * sizeof(float));
    w.quant = p + off;
    w.quant_bytes = sage::quant_scratch_layout(nullptr, B, Hkv, Nk, d).bytes;
    off += w.quant_bytes;
    w.bytes = off;
    return w;
}

// Carving of the sage_attn_fwd_4bit workspace: the 8+8 layout plus the block means of Q and the score correction.
struct Fwd4Workspace {
    FwdWorkspace base;
    float *q_mean, *dsx;
    size_t bytes;
};
Fwd4Workspace fwd4_layout(void *base, int B, int Hq, int Hkv, int Nq, int Nk, int d) {
    Fwd4Workspace w;
    w.base = fwd_layout(base, B, Hq, Hkv, Nq, Nk, d);
    char *p = static_cast<char *>(base);
    size_t off = w.base.bytes;
    const size_t BHq = (size_t)B * Hq, nQ = (size_t)sage::cdiv(Nq, sage::kBQ), nT = (size_t)sage::cdiv(Nk, sage::kW);
    w.q_mean = reinterpret_cast<float *>(p + off);
    off += align256(BHq * nQ * d * sizeof(float));
    w.dsx = reinterpret_cast<float *>(p + off);
    off += align256(BHq * nQ * nT * 128 * sizeof(float));
    w.bytes = off;
    return w;
}

}  // namespace

extern "C" {

int sage_get_params(sage_params *out) {
    if (!out) return SAGE_EINVAL;
    out->bq = SAGE_BQ;
    out->bk = SAGE_BK;
    out->w = SAGE_W;
    out->v_tile = SAGE_VTILE;
    out->p_r = 224.0f;
    out->v_r = 4.5f;
    return SAGE_OK;
}

const char *sage_strerror(int code) {
    switch (code) {
        case SAGE_OK: return "success";
        case SAGE_EINVAL:
            return "invalid argument (NULL or misaligned pointer, d not 64/128, size out of range, bad dtype or FP8 "
                   "range, Hq not a multiple of Hkv, causal with Nk < Nq)";
        case SAGE_EWORKSPACE: return "workspace missing, misaligned or too small";
        case SAGE_EHIP: return hipGetErrorString(g_last_hip_error);
        case SAGE_ESCRATCH:
            return "problem too large for the library's static scratch (sage_quant_workspace_bytes() exceeds "
                   "SAGE_STATIC_SCRATCH_BYTES): use sage_quant_kv with a caller-supplied workspace";
        default: return "unknown error code";
    }
}

size_t sage_v_fp8_bytes(int B, int H, int N, int d) {
    if (!shape_ok(B, H, N, d)) return 0;
    return (size_t)B * H * sage::cdiv(N, SAGE_VTILE) * d * SAGE_VTILE;
}

size_t sage_quant_workspace_bytes(int B, int H, int N, int d) {
    if (!shape_ok(B, H, N, d)) return 0;
    return sage::quant_scratch_layout(nullptr, B, H, N, d).bytes;
}

size_t sage_workspace_bytes(int B, int H, int N, int d) { return sage_workspace_bytes_gqa(B, H, H, N, N, d); }

size_t sage_workspace_bytes_gqa(int B, int Hq, int Hkv, int Nq, int Nk, int d) {
    if (!gqa_ok(B, Hq, Hkv, Nq, Nk, d, 0)) return 0;
    return fwd_layout(nullptr, B, Hq, Hkv, Nq, Nk, d).bytes;
}

int sage_quant_q(const void *q, int8_t *q_i8, float *q_scale, int B, int H, int N, int d, sage_dtype dt,
                 void *stream) {
    if (!shape_ok(B, H, N, d) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!q || !q_i8 || !q_scale || !aligned16(q) || !aligned16(q_i8)) return SAGE_EINVAL;
    discard_pending_hip_error();
    return from_hip(sage::launch_quant_q(q, sage::contiguous_bhnd(H, N, d), q_i8, q_scale, B, H, N, d, dt == SAGE_BF16,
                                         static_cast<hipStream_t>(stream)));
}

int sage_quant_k(const void *k, int8_t *k_i8, float *k_scale, float *k_mean, int B, int H, int N, int d,
                 sage_dtype dt, void *stream, void *workspace, size_t workspace_bytes) {
    if (!shape_ok(B, H, N, d) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!k || !k_i8 || !k_scale || !k_mean || !aligned16(k) || !aligned16(k_i8)) return SAGE_EINVAL;
    if (!workspace || !aligned256(workspace) || workspace_bytes < sage_quant_workspace_bytes(B, H, N, d))
        return SAGE_EWORKSPACE;
    const sage::QuantScratch ws = sage::quant_scratch_layout(workspace, B, H, N, d);
    discard_pending_hip_error();
    return from_hip(sage::launch_quant_k(k, sage::contiguous_bhnd(H, N, d), k_i8, k_scale, k_mean, B, H, N, d,
                                         dt == SAGE_BF16, static_cast<hipStream_t>(stream), ws));
}

int sage_quant_qk(const void *q, const void *k, int8_t *q_i8, int8_t *k_i8, float *q_scale, float *k_scale,
                  float *k_mean, int B, int H, int N, int d, sage_dtype dt, void *stream, void *workspace,
                  size_t workspace_bytes) {
    // every argument is checked before anything is enqueued
    if (!shape_ok(B, H, N, d) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!q || !k || !q_i8 || !k_i8 || !q_scale || !k_scale || !k_mean) return SAGE_EINVAL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(q_i8) || !aligned16(k_i8)) return SAGE_EINVAL;
    if (!workspace || !aligned256(workspace) || workspace_bytes < sage_quant_workspace_bytes(B, H, N, d))
        return SAGE_EWORKSPACE;
    const int rc = sage_quant_k(k, k_i8, k_scale, k_mean, B, H, N, d, dt, stream, workspace, workspace_bytes);
    if (rc != SAGE_OK) return rc;
    return sage_quant_q(q, q_i8, q_scale, B, H, N, d, dt, stream);
}

int sage_quant_v(const void *v, uint8_t *v_fp8, float *v_scale, float v_r, int B, int H, int N, int d,
                 sage_dtype dt, void *stream, void *workspace, size_t workspace_bytes) {
    if (!shape_ok(B, H, N, d) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!v || !v_fp8 || !v_scale || !(v_r > 0.0f) || !(v_r <= 448.0f)) return SAGE_EINVAL;
    if (!aligned16(v) || !aligned16(v_fp8) || !aligned16(v_scale)) return SAGE_EINVAL;
    if (!workspace || !aligned256(workspace) || workspace_bytes < sage_quant_workspace_bytes(B, H, N, d))
        return SAGE_EWORKSPACE;
    const sage::QuantScratch ws = sage::quant_scratch_layout(workspace, B, H, N, d);
    discard_pending_hip_error();
    return from_hip(sage::launch_quant_v(v, sage::contiguous_bhnd(H, N, d), v_fp8, v_scale, v_r, B, H, N, d,
                                         dt == SAGE_BF16, static_cast<hipStream_t>(stream), ws));
}

int sage_quant_kv(const void *k, const void *v, int8_t *k_i8, float *k_scale, float *k_mean, uint8_t *v_fp8,
                  float *v_scale, float v_r, int B, int H, int N, int d, sage_dtype dt, void *stream, void *workspace,
                  size_t workspace_bytes) {
    if (!shape_ok(B, H, N, d) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!k || !v || !k_i8 || !k_scale || !k_mean || !v_fp8 || !v_scale) return SAGE_EINVAL;
    if (!(v_r > 0.0f) || !(v_r <= 448.0f)) return SAGE_EINVAL;
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_i8) || !aligned16(v_fp8) || !aligned16(v_scale))
        return SAGE_EINVAL;
    if (!workspace || !aligned256(workspace) || workspace_bytes < sage_quant_workspace_bytes(B, H, N, d))
        return SAGE_EWORKSPACE;
    const sage::QuantScratch ws = sage::quant_scratch_layout(workspace, B, H, N, d);
    const sage::Strides st = sage::contiguous_bhnd(H, N, d);
    discard_pending_hip_error();
    return from_hip(sage::launch_quant_kv(k, st, v, st, k_i8, k_scale, k_mean, v_fp8, v_scale, v_r, B, H, N, d,
                                          dt == SAGE_BF16, static_cast<hipStream_t>(stream), ws));
}

int sage_quant_kv_static(const void *k, const void *v, int8_t *k_i8, float *k_scale, float *k_mean, uint8_t *v_fp8,
                         float *v_scale, float v_r, int B, int H, int N, int d, sage_dtype dt, void *stream) {
    if (!shape_ok(B, H, N, d) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!k || !v || !k_i8 || !k_scale || !k_mean || !v_fp8 || !v_scale) return SAGE_EINVAL;
    if (!(v_r > 0.0f) || !(v_r <= 448.0f)) return SAGE_EINVAL;
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_i8) || !aligned16(v_fp8) || !aligned16(v_scale))
        return SAGE_EINVAL;
    if (sage_quant_workspace_bytes(B, H, N, d) > (size_t)SAGE_STATIC_SCRATCH_BYTES) return SAGE_ESCRATCH;
    discard_pending_hip_error();
    void *ptr = nullptr;
    const hipError_t e = static_scratch(&ptr);
    if (e != hipSuccess) return from_hip(e);
    // nothing in the scratch has to be cleared by the caller: the three launches write every partial statistic
    // and reciprocal before they read it, and the single-read kernel's launcher clears the partial buffers with a
    // fill kernel of its own in front
    const sage::QuantScratch ws = sage::quant_scratch_layout(ptr, B, H, N, d);
    const sage::Strides st = sage::contiguous_bhnd(H, N, d);
    return from_hip(sage::launch_quant_kv(k, st, v, st, k_i8, k_scale, k_mean, v_fp8, v_scale, v_r, B, H, N, d,
                                          dt == SAGE_BF16, static_cast<hipStream_t>(stream), ws));
}

/* ---- the 4+8 variant ---------------------------------------------------------------------------------- */

size_t sage_workspace_bytes_4bit(int B, int Hq, int Hkv, int Nq, int Nk, int d) {
    if (!gqa_ok(B, Hq, Hkv, Nq, Nk, d, 0)) return 0;
    return fwd4_layout(nullptr, B, Hq, Hkv, Nq, Nk, d).bytes;
}

size_t sage_delta_s_bytes(int B, int Hq, int Nq, int Nk) {
    if (B < 1 || Hq < 1 || Nq < 1 || Nk < 1 || Nq > (1 << 22) || Nk > (1 << 22) || (size_t)B * Hq > 65535u) return 0;
    return (size_t)B * Hq * sage::cdiv(Nq, sage::kBQ) * sage::cdiv(Nk, sage::kW) * 128 * sizeof(float);
}

int sage_quant_q4(const void *q, float *q_mean, int8_t *q_i4, float *q_scale, int B, int H, int N, int d,
                  sage_dtype dt, void *stream) {
    if (!shape_ok(B, H, N, d) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!q || !q_mean || !aligned16(q) || !aligned16(q_mean)) return SAGE_EINVAL;
    if ((q_i4 == nullptr) != (q_scale == nullptr) || (q_i4 && !aligned16(q_i4))) return SAGE_EINVAL;
    discard_pending_hip_error();
    return from_hip(sage::launch_quant_q4(q, sage::contiguous_bhnd(H, N, d), q_mean, q_i4, q_scale, B, H, N, d,
                                          dt == SAGE_BF16, static_cast<hipStream_t>(stream)));
}

int sage_quant_kv4(const void *k, const void *v, int8_t *k_i4, float *k_scale, float *k_mean, uint8_t *v_fp8,
                   float *v_scale, float v_r, int B, int H, int N, int d, sage_dtype dt, void *stream, void *workspace,
                   size_t workspace_bytes) {
    if (!shape_ok(B, H, N, d) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!k || !v || !k_i4 || !k_scale || !k_mean || !v_fp8 || !v_scale) return SAGE_EINVAL;
    if (!(v_r > 0.0f) || !(v_r <= 448.0f)) return SAGE_EINVAL;
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_i4) || !aligned16(v_fp8) || !aligned16(v_scale) ||
        !aligned16(k_mean))
        return SAGE_EINVAL;
    if (!workspace || !aligned256(workspace) || workspace_bytes < sage_quant_workspace_bytes(B, H, N, d))
        return SAGE_EWORKSPACE;
    const sage::QuantScratch ws = sage::quant_scratch_layout(workspace, B, H, N, d);
    const sage::Strides st = sage::contiguous_bhnd(H, N, d);
    discard_pending_hip_error();
    return from_hip(sage::launch_quant_kv(k, st, v, st, k_i4, k_scale, k_mean, v_fp8, v_scale, v_r, B, H, N, d,
                                          dt == SAGE_BF16, static_cast<hipStream_t>(stream), ws, true));
}

int sage_delta_s(const void *k, const float *k_mean, const float *q_mean, float *dsx, int B, int Hq, int Hkv, int Nq,
                 int Nk, int d, int causal, float sm_scale, sage_dtype dt, void *stream) {
    if (!gqa_ok(B, Hq, Hkv, Nq, Nk, d, causal) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!k || !k_mean || !q_mean || !dsx) return SAGE_EINVAL;
    if (!aligned16(k) || !aligned16(k_mean) || !aligned16(q_mean) || !aligned16(dsx)) return SAGE_EINVAL;
    sm_scale = scale_or_default(sm_scale, d);
    discard_pending_hip_error();
    return from_hip(sage::launch_delta_s(k, sage::contiguous_bhnd(Hkv, Nk, d), k_mean, q_mean, dsx, B, Hq, Hkv, Nq, Nk,
                                         d, causal != 0, sm_scale, dt == SAGE_BF16, static_cast<hipStream_t>(stream)));
}

int sage_attn_fwd_q4(const void *q, const float *q_mean, const int8_t *k_i4, const uint8_t *v_fp8,
                     const float *k_scale, const float *v_scale, const float *dsx, void *out, int B, int Hq, int Hkv,
                     int Nq, int Nk, int d, int causal, float sm_scale, float p_r, sage_dtype dt, void *stream) {
    if (!gqa_ok(B, Hq, Hkv, Nq, Nk, d, causal) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!q || !q_mean || !k_i4 || !v_fp8 || !k_scale || !v_scale || !dsx || !out) return SAGE_EINVAL;
    if (!aligned16(q) || !aligned16(q_mean) || !aligned16(k_i4) || !aligned16(v_fp8) || !aligned16(v_scale) ||
        !aligned16(dsx) || !aligned16(out))
        return SAGE_EINVAL;
    if (!(p_r > 0.0f) || !(p_r <= 448.0f)) return SAGE_EINVAL;
    sm_scale = scale_or_default(sm_scale, d);
    const sage::Strides st = sage::contiguous_bhnd(Hq, Nq, d);
    discard_pending_hip_error();
    return from_hip(sage::launch_attn(q, true, st, k_i4, v_fp8, nullptr, k_scale, v_scale, out, st, B, Hq, Hkv, Nq, Nk, d,
                                      causal != 0, sm_scale, p_r, dt == SAGE_BF16, static_cast<hipStream_t>(stream),
                                      q_mean, dsx));
}

int sage_attn_fwd_4bit(const void *q, const void *k, const void *v, void *out, int B, int Hq, int Hkv, int Nq, int Nk,
                       int d, int causal, float sm_scale, void *stream, sage_dtype dt, void *workspace,
                       size_t workspace_bytes) {
    if (!gqa_ok(B, Hq, Hkv, Nq, Nk, d, causal) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!q || !k || !v || !out) return SAGE_EINVAL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return SAGE_EINVAL;
    if (!workspace || !aligned256(workspace) || workspace_bytes < sage_workspace_bytes_4bit(B, Hq, Hkv, Nq, Nk, d))
        return SAGE_EWORKSPACE;
    sm_scale = scale_or_default(sm_scale, d);
    const Fwd4Workspace w = fwd4_layout(workspace, B, Hq, Hkv, Nq, Nk, d);
    const sage::QuantScratch qws = sage::quant_scratch_layout(w.base.quant, B, Hkv, Nk, d);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool bf16 = dt == SAGE_BF16;
    const sage::Strides qs = sage::contiguous_bhnd(Hq, Nq, d), ks = sage::contiguous_bhnd(Hkv, Nk, d);
    discard_pending_hip_error();
    hipError_t e = sage::launch_quant_kv(k, ks, v, ks, w.base.k_i8, w.base.k_scale, w.base.k_mean, w.base.v_fp8,
                                         w.base.v_scale, 4.5f, B, Hkv, Nk, d, bf16, s, qws, true);
    if (e == hipSuccess) e = sage::launch_quant_q4(q, qs, w.q_mean, nullptr, nullptr, B, Hq, Nq, d, bf16, s);
    if (e == hipSuccess)
        e = sage::launch_delta_s(k, ks, w.base.k_mean, w.q_mean, w.dsx, B, Hq, Hkv, Nq, Nk, d, causal != 0, sm_scale, bf16,
                                 s);
    if (e == hipSuccess)
        e = sage::launch_attn(q, true, qs, w.base.k_i8, w.base.v_fp8, nullptr, w.base.k_scale, w.base.v_scale, out, qs, B,
                              Hq, Hkv, Nq, Nk, d, causal != 0, sm_scale, 224.0f, bf16, s, w.q_mean, w.dsx);
    return from_hip(e);
}

int sage_attn_fwd_quantized_gqa(const int8_t *q_i8, const int8_t *k_i8, const uint8_t *v_fp8, const float *q_scale,
                                const float *k_scale, const float *v_scale, void *out, int B, int Hq, int Hkv,
                                int Nq, int Nk, int d, int causal, float sm_scale, float p_r, sage_dtype out_dt,
                                void *stream) {
    if (!gqa_ok(B, Hq, Hkv, Nq, Nk, d, causal) || !dtype_ok(out_dt)) return SAGE_EINVAL;
    if (!q_i8 || !k_i8 || !v_fp8 || !q_scale || !k_scale || !v_scale || !out) return SAGE_EINVAL;
    if (!aligned16(q_i8) || !aligned16(k_i8) || !aligned16(v_fp8) || !aligned16(v_scale) || !aligned16(out))
        return SAGE_EINVAL;
    if (!(p_r > 0.0f) || !(p_r <= 448.0f)) return SAGE_EINVAL;
    sm_scale = scale_or_default(sm_scale, d);
    const sage::Strides st = sage::contiguous_bhnd(Hq, Nq, d);
    discard_pending_hip_error();
    return from_hip(sage::launch_attn(q_i8, false, st, k_i8, v_fp8, q_scale, k_scale, v_scale, out, st, B, Hq, Hkv, Nq,
                                      Nk, d, causal != 0, sm_scale, p_r, out_dt == SAGE_BF16,
                                      static_cast<hipStream_t>(stream)));
}

int sage_attn_fwd_kvquantized_gqa(const void *q, const int8_t *k_i8, const uint8_t *v_fp8, const float *k_scale,
                                  const float *v_scale, void *out, int B, int Hq, int Hkv, int Nq, int Nk, int d,
                                  int causal, float sm_scale, float p_r, sage_dtype dt, void *stream) {
    if (!gqa_ok(B, Hq, Hkv, Nq, Nk, d, causal) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!q || !k_i8 || !v_fp8 || !k_scale || !v_scale || !out) return SAGE_EINVAL;
    if (!aligned16(q) || !aligned16(k_i8) || !aligned16(v_fp8) || !aligned16(v_scale) || !aligned16(out))
        return SAGE_EINVAL;
    if (!(p_r > 0.0f) || !(p_r <= 448.0f)) return SAGE_EINVAL;
    sm_scale = scale_or_default(sm_scale, d);
    const sage::Strides st = sage::contiguous_bhnd(Hq, Nq, d);
    discard_pending_hip_error();
    return from_hip(sage::launch_attn(q, true, st, k_i8, v_fp8, nullptr, k_scale, v_scale, out, st, B, Hq, Hkv, Nq, Nk,
                                      d, causal != 0, sm_scale, p_r, dt == SAGE_BF16,
                                      static_cast<hipStream_t>(stream)));
}

/* ---- decode-shaped calls -------------------------------------------------------------------------------- */

namespace {
constexpr int kDecodeRows = 64;  // query rows per K/V head the packed decode kernel takes
bool decode_ok(int B, int Hq, int Hkv, int Nq, int Nk, int d, int causal, int split_keys) {
    return gqa_ok(B, Hq, Hkv, Nq, Nk, d, causal) && split_keys >= 0 && split_keys % sage::kW == 0;
}
bool packed(int Hq, int Hkv, int Nq) { return (Hq / Hkv) * Nq <= kDecodeRows; }
int decode_steps(int B, int Hq, int Hkv, int Nq, int Nk, int split_keys) {
    if (split_keys > 0) return split_keys / sage::kW;
    return packed(Hq, Hkv, Nq) ? sage::decode_auto_steps_per_split(B, Hkv, Nk)
                               : sage::ranges_auto_steps_per_split(B, Hq, Nq, Nk);
}
sage::DecodeScratch decode_layout(void *base, int B, int Hq, int Hkv, int Nq, int Nk, int d, int steps) {
    return packed(Hq, Hkv, Nq)
               ? sage::decode_scratch_layout(base, B, Hkv, Nk, d, steps, sage::cdiv((Hq / Hkv) * Nq, 16))
               : sage::ranges_scratch_layout(base, B, Hq, Nq, Nk, d, steps);
}
}  // namespace

int sage_decode_split_keys(int B, int Hq, int Hkv, int Nq, int Nk) {
    if (!gqa_ok(B, Hq, Hkv, Nq, Nk, 128, 0)) return 0;
    return decode_steps(B, Hq, Hkv, Nq, Nk, 0) * sage::kW;
}

size_t sage_decode_workspace_bytes(int B, int Hq, int Hkv, int Nq, int Nk, int d, int split_keys) {
    if (!decode_ok(B, Hq, Hkv, Nq, Nk, d, 0, split_keys)) return 0;
    return decode_layout(nullptr, B, Hq, Hkv, Nq, Nk, d, decode_steps(B, Hq, Hkv, Nq, Nk, split_keys)).bytes;
}

int sage_attn_fwd_decode(const void *q, const int8_t *k_i8, const uint8_t *v_fp8, const float *k_scale,
                         const float *v_scale, void *out, int B, int Hq, int Hkv, int Nq, int Nk, int d, int causal,
                         float sm_scale, float p_r, int split_keys, sage_dtype dt, void *stream, void *workspace,
                         size_t workspace_bytes) {
    if (!decode_ok(B, Hq, Hkv, Nq, Nk, d, causal, split_keys) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!q || !k_i8 || !v_fp8 || !k_scale || !v_scale || !out) return SAGE_EINVAL;
    if (!aligned16(q) || !aligned16(k_i8) || !aligned16(v_fp8) || !aligned16(v_scale) || !aligned16(out))
        return SAGE_EINVAL;
    if (!(p_r > 0.0f) || !(p_r <= 448.0f)) return SAGE_EINVAL;
    const int steps = decode_steps(B, Hq, Hkv, Nq, Nk, split_keys);
    const sage::DecodeScratch ws = decode_layout(workspace, B, Hq, Hkv, Nq, Nk, d, steps);
    if (!workspace || !aligned256(workspace) || workspace_bytes < ws.bytes) return SAGE_EWORKSPACE;
    sm_scale = scale_or_default(sm_scale, d);
    discard_pending_hip_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (packed(Hq, Hkv, Nq))
        return from_hip(sage::launch_decode(q, k_i8, v_fp8, k_scale, v_scale, out, B, Hq, Hkv, Nq, Nk, d, causal != 0,
                                            sm_scale, p_r, steps, dt == SAGE_BF16, s, ws));
    return from_hip(sage::launch_attn_ranges(q, k_i8, v_fp8, k_scale, v_scale, out, B, Hq, Hkv, Nq, Nk, d, causal != 0,
                                             sm_scale, p_r, steps, dt == SAGE_BF16, s, ws));
}

int sage_attn_fwd_quantized(const int8_t *q_i8, const int8_t *k_i8, const uint8_t *v_fp8, const float *q_scale,
                            const float *k_scale, const float *v_scale, void *out, int B, int H, int N, int d,
                            int causal, float sm_scale, float p_r, sage_dtype out_dt, void *stream) {
    return sage_attn_fwd_quantized_gqa(q_i8, k_i8, v_fp8, q_scale, k_scale, v_scale, out, B, H, H, N, N, d, causal,
                                       sm_scale, p_r, out_dt, stream);
}

int sage_attn_fwd_strided(const void *q, const void *k, const void *v, void *out, int B, int Hq, int Hkv, int Nq,
                          int Nk, int d, const int64_t *q_strides, const int64_t *k_strides, const int64_t *v_strides,
                          const int64_t *out_strides, int causal, float sm_scale, void *stream, sage_dtype dt,
                          void *workspace, size_t workspace_bytes) {
    if (!gqa_ok(B, Hq, Hkv, Nq, Nk, d, causal) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!q || !k || !v || !out) return SAGE_EINVAL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return SAGE_EINVAL;
    sage::Strides qs, ks, vs, os;
    if (!read_strides(q_strides, Hq, Nq, d, &qs) || !read_strides(k_strides, Hkv, Nk, d, &ks) ||
        !read_strides(v_strides, Hkv, Nk, d, &vs) || !read_strides(out_strides, Hq, Nq, d, &os))
        return SAGE_EINVAL;
    if (!write_strides_ok(os, B, Hq, Nq, d)) return SAGE_EINVAL;
    if (!workspace || !aligned256(workspace) || workspace_bytes < sage_workspace_bytes_gqa(B, Hq, Hkv, Nq, Nk, d))
        return SAGE_EWORKSPACE;
    sm_scale = scale_or_default(sm_scale, d);
    const FwdWorkspace w = fwd_layout(workspace, B, Hq, Hkv, Nq, Nk, d);
    const sage::QuantScratch qws = sage::quant_scratch_layout(w.quant, B, Hkv, Nk, d);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool bf16 = dt == SAGE_BF16;
    discard_pending_hip_error();
    hipError_t e = sage::launch_quant_kv(k, ks, v, vs, w.k_i8, w.k_scale, w.k_mean, w.v_fp8, w.v_scale, 4.5f, B, Hkv, Nk,
                                         d, bf16, s, qws);
    // Q is quantised inside the attention kernel: Q^ and delta_Q never touch memory
    if (e == hipSuccess)
        e = sage::launch_attn(q, true, qs, w.k_i8, w.v_fp8, nullptr, w.k_scale, w.v_scale, out, os, B, Hq, Hkv, Nq, Nk, d,
                              causal != 0, sm_scale, 224.0f, bf16, s);
    return from_hip(e);
}

int sage_attn_fwd_gqa(const void *q, const void *k, const void *v, void *out, int B, int Hq, int Hkv, int Nq, int Nk,
                      int d, int causal, float sm_scale, void *stream, sage_dtype dt, void *workspace,
                      size_t workspace_bytes) {
    return sage_attn_fwd_strided(q, k, v, out, B, Hq, Hkv, Nq, Nk, d, nullptr, nullptr, nullptr, nullptr, causal,
                                 sm_scale, stream, dt, workspace, workspace_bytes);
}

int sage_attn_fwd(const void *q, const void *k, const void *v, void *out, int B, int H, int N, int d, int causal,
                  float sm_scale, void *stream, sage_dtype dt, void *workspace, size_t workspace_bytes) {
    return sage_attn_fwd_gqa(q, k, v, out, B, H, H, N, N, d, causal, sm_scale, stream, dt, workspace, workspace_bytes);
}

}  // extern "C"
