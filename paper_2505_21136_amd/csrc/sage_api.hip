// C ABI of libsage (declared in include/sage.h): argument checks, workspace
// carving and kernel launches.  No allocation, no synchronisation, no state.
#include "../../include/sage.h"
#include "sage_internal.h"

#include <math.h>

namespace {

thread_local hipError_t g_last_hip_error = hipSuccess;

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned256(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }
bool shape_ok(int B, int H, int N, int d) {
    return B >= 1 && H >= 1 && N >= 1 && N <= (1 << 22) && (d == 64 || d == 128) && (size_t)B * H <= 65535u;
}
bool dtype_ok(sage_dtype dt) { return dt == SAGE_F16 || dt == SAGE_BF16; }
int from_hip(hipError_t e) {
    if (e == hipSuccess) return SAGE_OK;
    g_last_hip_error = e;
    return SAGE_EHIP;
}

// Carving of the sage_attn_fwd workspace.
struct FwdWorkspace {
    int8_t *q_i8, *k_i8;
    uint8_t *v_fp8;
    float *q_scale, *k_scale, *v_scale, *k_mean;
    void *quant;
    size_t bytes;
};
FwdWorkspace fwd_layout(void *base, int B, int H, int N, int d) {
    const size_t BH = (size_t)B * H, E = BH * N * d;
    char *p = static_cast<char *>(base);
    size_t off = 0;
    FwdWorkspace w;
    w.q_i8 = reinterpret_cast<int8_t *>(p + off);
    off += align256(E);
    w.k_i8 = reinterpret_cast<int8_t *>(p + off);
    off += align256(E);
    w.v_fp8 = reinterpret_cast<uint8_t *>(p + off);
    off += align256(sage_v_fp8_bytes(B, H, N, d));
    w.q_scale = reinterpret_cast<float *>(p + off);
    off += align256(BH * sage::cdiv(N, sage::kBQ) * sizeof(float));
    w.k_scale = reinterpret_cast<float *>(p + off);
    off += align256(BH * sage::cdiv(N, sage::kBK) * sizeof(float));
    w.v_scale = reinterpret_cast<float *>(p + off);
    off += align256(BH * d * sizeof(float));
    w.k_mean = reinterpret_cast<float *>(p + off);
    off += align256(BH * d * sizeof(float));
    w.quant = p + off;
    off += sage::quant_scratch_layout(nullptr, B, H, N, d).bytes;
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
        case SAGE_EINVAL: return "invalid argument (NULL or misaligned pointer, d not 64/128, size < 1, bad dtype or range)";
        case SAGE_EWORKSPACE: return "workspace missing, misaligned or too small";
        case SAGE_EHIP: return hipGetErrorString(g_last_hip_error);
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

size_t sage_workspace_bytes(int B, int H, int N, int d) {
    if (!shape_ok(B, H, N, d)) return 0;
    return fwd_layout(nullptr, B, H, N, d).bytes;
}

int sage_quant_qk(const void *q, const void *k, int8_t *q_i8, int8_t *k_i8, float *q_scale, float *k_scale,
                  float *k_mean, int B, int H, int N, int d, sage_dtype dt, void *stream, void *workspace,
                  size_t workspace_bytes) {
    if (!shape_ok(B, H, N, d) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!q || !k || !q_i8 || !k_i8 || !q_scale || !k_scale || !k_mean) return SAGE_EINVAL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(q_i8) || !aligned16(k_i8)) return SAGE_EINVAL;
    if (!workspace || !aligned256(workspace) || workspace_bytes < sage_quant_workspace_bytes(B, H, N, d))
        return SAGE_EWORKSPACE;
    const sage::QuantScratch ws = sage::quant_scratch_layout(workspace, B, H, N, d);
    return from_hip(sage::launch_quant_qk(q, k, q_i8, k_i8, q_scale, k_scale, k_mean, B, H, N, d,
                                          dt == SAGE_BF16, static_cast<hipStream_t>(stream), ws));
}

int sage_quant_v(const void *v, uint8_t *v_fp8, float *v_scale, float v_r, int B, int H, int N, int d,
                 sage_dtype dt, void *stream, void *workspace, size_t workspace_bytes) {
    if (!shape_ok(B, H, N, d) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!v || !v_fp8 || !v_scale || !(v_r > 0.0f) || !(v_r <= 448.0f)) return SAGE_EINVAL;
    if (!aligned16(v) || !aligned16(v_fp8) || !aligned16(v_scale)) return SAGE_EINVAL;
    if (!workspace || !aligned256(workspace) || workspace_bytes < sage_quant_workspace_bytes(B, H, N, d))
        return SAGE_EWORKSPACE;
    const sage::QuantScratch ws = sage::quant_scratch_layout(workspace, B, H, N, d);
    return from_hip(sage::launch_quant_v(v, v_fp8, v_scale, v_r, B, H, N, d, dt == SAGE_BF16,
                                         static_cast<hipStream_t>(stream), ws));
}

int sage_attn_fwd_quantized(const int8_t *q_i8, const int8_t *k_i8, const uint8_t *v_fp8, const float *q_scale,
                            const float *k_scale, const float *v_scale, void *out, int B, int H, int N, int d,
                            int causal, float sm_scale, float p_r, sage_dtype out_dt, void *stream) {
    if (!shape_ok(B, H, N, d) || !dtype_ok(out_dt)) return SAGE_EINVAL;
    if (!q_i8 || !k_i8 || !v_fp8 || !q_scale || !k_scale || !v_scale || !out) return SAGE_EINVAL;
    if (!aligned16(q_i8) || !aligned16(k_i8) || !aligned16(v_fp8) || !aligned16(v_scale) || !aligned16(out))
        return SAGE_EINVAL;
    if (!(p_r > 0.0f) || !(p_r <= 448.0f)) return SAGE_EINVAL;
    if (!(sm_scale > 0.0f)) sm_scale = 1.0f / sqrtf((float)d);  // also catches NaN
    return from_hip(sage::launch_attn(q_i8, k_i8, v_fp8, q_scale, k_scale, v_scale, out, B, H, N, d, causal != 0,
                                      sm_scale, p_r, out_dt == SAGE_BF16, static_cast<hipStream_t>(stream)));
}

int sage_attn_fwd(const void *q, const void *k, const void *v, void *out, int B, int H, int N, int d, int causal,
                  float sm_scale, void *stream, sage_dtype dt, void *workspace, size_t workspace_bytes) {
    if (!shape_ok(B, H, N, d) || !dtype_ok(dt)) return SAGE_EINVAL;
    if (!q || !k || !v || !out) return SAGE_EINVAL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return SAGE_EINVAL;
    if (!workspace || !aligned256(workspace) || workspace_bytes < sage_workspace_bytes(B, H, N, d))
        return SAGE_EWORKSPACE;
    const FwdWorkspace w = fwd_layout(workspace, B, H, N, d);
    const size_t qbytes = sage_quant_workspace_bytes(B, H, N, d);
    int rc = sage_quant_qk(q, k, w.q_i8, w.k_i8, w.q_scale, w.k_scale, w.k_mean, B, H, N, d, dt, stream, w.quant,
                           qbytes);
    if (rc != SAGE_OK) return rc;
    rc = sage_quant_v(v, w.v_fp8, w.v_scale, 4.5f, B, H, N, d, dt, stream, w.quant, qbytes);
    if (rc != SAGE_OK) return rc;
    return sage_attn_fwd_quantized(w.q_i8, w.k_i8, w.v_fp8, w.q_scale, w.k_scale, w.v_scale, out, B, H, N, d,
                                   causal, sm_scale, 224.0f, dt, stream);
}

}  // extern "C"
