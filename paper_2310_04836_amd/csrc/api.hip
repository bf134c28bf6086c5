// extern "C" boundary of libdgq.so: argument validation on the host, then one launcher.
// Every check happens before anything is enqueued.
#include <atomic>
#include <mutex>
#include <cmath>
#include <cstdio>

#include "dgq_device.hpp"

namespace {

thread_local int g_last_hip_error = 0;

// Scratch of dgq_linear_a8w4_noalloc: the INT32 partial sums of a K split, for callers that cannot
// bring a workspace.  Every GPU the library runs on holds its own copy of this array, at its own
// address, until the process ends.  In host code the NAME below is only a handle for
// hipGetSymbolAddress; kernels are given the address that call returns for the current device.
constexpr size_t kScratchBytes = (size_t)40 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];   // device address of `scratch` per GPU, set once
std::mutex g_scratch_mutex;

hipError_t scratch_of_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[dev].load(std::memory_order_acquire);
        if (!p) {
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (!p) return hipErrorInvalidSymbol;
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return hipSuccess;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

dgq_status check_shape(int N, int K, int group)
{
    if (group != 64 && group != 128) return DGQ_ERR_SHAPE;
    if (K < 128 || K > 131072 || (K % 128) != 0) return DGQ_ERR_SHAPE;
    if (N < 16 || (N % 16) != 0) return DGQ_ERR_SHAPE;
    // cell and element indices are computed in 32 bits in places; keep K*N below 2^36
    if ((long long)K * (long long)N > (1LL << 36)) return DGQ_ERR_SHAPE;
    return DGQ_OK;
}

dgq_status hip_result(hipError_t e)
{
    if (e == hipSuccess) return DGQ_OK;
    g_last_hip_error = (int)e;
    return DGQ_ERR_HIP;
}

// 0 = by M, 1 = weight-streaming kernels, 2 = tiled kernel, 3 = the streaming kernel that
// re-reads activations every step (never chosen by M).
enum { kPathAuto = 0, kPathStream = 1, kPathTiled = 2, kPathStreamGeneric = 3 };

int pick_path(int M, int forced)
{
    if (forced == kPathTiled) return kPathTiled;
    if (forced == kPathStreamGeneric) return kPathStreamGeneric;
    if (forced == kPathStream) return M <= dgq::kDecodeMaxM ? kPathStream : kPathStreamGeneric;
    return M <= dgq::kDecodeMaxM ? kPathStream : kPathTiled;
}

size_t workspace_needed(int path, int M, int N, int K)
{
    if (path == kPathStream) return dgq::decode_workspace_bytes(M, N, K);
    if (path == kPathTiled) return dgq::tiled_workspace_bytes(M, N, K);
    return 0;
}

dgq_status run_linear(dgq::LinearArgs &a, int forced, void *workspace, size_t workspace_bytes, void *stream)
{
    if (forced < kPathAuto || forced > kPathStreamGeneric) return DGQ_ERR_RANGE;
    if ((forced == kPathStream || forced == kPathStreamGeneric) && a.M > dgq::kStreamMaxM) return DGQ_ERR_SHAPE;
    const int path = pick_path(a.M, forced);
    if (path == kPathStreamGeneric && a.zp) return DGQ_ERR_SHAPE;  // that kernel knows the constant zero point only
    const size_t need = workspace_needed(path, a.M, a.N, a.K);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return DGQ_ERR_WORKSPACE;
        if (!aligned16(workspace)) return DGQ_ERR_ALIGN;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (path) {
    case kPathStream: return hip_result(dgq::launch_linear_decode(a, workspace, st));
    case kPathStreamGeneric: return hip_result(dgq::launch_linear_stream(a, st));
    default: return hip_result(dgq::launch_linear_tiled(a, workspace, st));
    }
}

// The one-call form quantizes inside the decode kernel when one workgroup covers all of K.
bool quantizes_in_kernel(int M, int K, int forced)
{
    if (pick_path(M, forced) != kPathStream) return false;
    return dgq::decode_plan(K).ksplit == 1 && (long long)M * (K + 16) <= dgq::kQuantDecodeStageBytes;
}

inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

// gamma != nullptr: RMSNorm (with eps) in front of the quantizer
dgq_status quant_linear(const uint16_t *x, const uint16_t *gamma, float eps, const void *qweight, const void *scales,
                        int zp_form, const float *s1, uint16_t *out, float *sx_out, int M, int N, int K, int group,
                        void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x || !qweight || !scales || !s1 || !out) return DGQ_ERR_NULL;
    if (M < 1) return DGQ_ERR_SHAPE;
    if (dgq_status st = check_shape(N, K, group)) return st;
    if (gamma && K > 24576) return DGQ_ERR_SHAPE;
    if (gamma && (!(eps >= 0.0f) || !(eps < 1.0f))) return DGQ_ERR_RANGE;
    if (!aligned16(x) || !aligned16(qweight) || !aligned16(scales) || !aligned16(out) || !aligned16(gamma) ||
        (reinterpret_cast<uintptr_t>(s1) & 3u) || (reinterpret_cast<uintptr_t>(sx_out) & 3u))
        return DGQ_ERR_ALIGN;
    const int forced = kPathAuto;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (quantizes_in_kernel(M, K, forced) && (!gamma || dgq::decode_plan(K).spw <= dgq::kRmsDecodeMaxStepsPerWave)) {
        dgq::LinearArgs a{nullptr, nullptr, static_cast<const uint4 *>(qweight), static_cast<const uint32_t *>(scales),
                          s1, out, nullptr, M, N, K, group, zp_form, x, sx_out, gamma, eps};
        return hip_result(dgq::launch_linear_decode(a, nullptr, st));
    }
    // two launches, xq and sx in the workspace: [what the linear needs, its arrival counters first][xq: M*K][sx: 4*M]
    const int path = pick_path(M, forced);
    if (path == kPathStreamGeneric && zp_form) return DGQ_ERR_SHAPE;
    const size_t lin_bytes = round256(workspace_needed(path, M, N, K));
    const size_t xq_bytes = round256((size_t)M * K), sx_bytes = round256((size_t)M * sizeof(float));
    if (!workspace || workspace_bytes < lin_bytes + xq_bytes + sx_bytes) return DGQ_ERR_WORKSPACE;
    if (!aligned16(workspace)) return DGQ_ERR_ALIGN;
    char *ws = static_cast<char *>(workspace);
    int8_t *xq = reinterpret_cast<int8_t *>(ws + lin_bytes);
    float *sx = sx_out ? sx_out : reinterpret_cast<float *>(ws + lin_bytes + xq_bytes);
    dgq::LinearArgs a{xq, sx, static_cast<const uint4 *>(qweight), static_cast<const uint32_t *>(scales),
                      s1, out, nullptr, M, N, K, group, zp_form, nullptr, nullptr, nullptr, 0.0f};
    const hipError_t qe = gamma ? dgq::launch_rmsnorm_quant_act(x, gamma, M, K, eps, xq, sx, st)
                                : dgq::launch_quant_act(x, M, K, xq, sx, st);
    if (dgq_status q = hip_result(qe)) return q;
    return run_linear(a, kPathAuto, ws, lin_bytes, stream);
}

}  // namespace

extern "C" {

const char *dgq_status_string(dgq_status st)
{
    switch (st) {
    case DGQ_OK: return "ok";
    case DGQ_ERR_NULL: return "a required pointer is NULL";
    case DGQ_ERR_SHAPE: return "M, N, K or group breaks a shape rule";
    case DGQ_ERR_ALIGN: return "a device pointer is not 16-byte aligned";
    case DGQ_ERR_RANGE: return "value out of range";
    case DGQ_ERR_WORKSPACE: return "workspace too small";
    case DGQ_ERR_HIP: return "a HIP call failed (see dgq_last_hip_error)";
    default: return "unknown dgq status";
    }
}

int dgq_last_hip_error(void) { return g_last_hip_error; }

int dgq_layout_version(void) { return DGQ_LAYOUT_VERSION; }

dgq_status dgq_packed_sizes(int K, int N, int group, size_t *qweight_bytes, size_t *scales_bytes)
{
    if (!qweight_bytes || !scales_bytes) return DGQ_ERR_NULL;
    if (dgq_status st = check_shape(N, K, group)) return st;
    const size_t ng = (size_t)K / group;
    *qweight_bytes = (size_t)K * (size_t)N / 2;
    *scales_bytes = ((size_t)N / 16) * ((ng + 3) / 4) * 64;
    return DGQ_OK;
}

dgq_status dgq_linear_workspace_bytes(int M, int N, int K, int group, size_t *bytes)
{
    if (!bytes) return DGQ_ERR_NULL;
    if (M < 1) return DGQ_ERR_SHAPE;
    if (dgq_status st = check_shape(N, K, group)) return st;
    // Partial sums go through global memory when several workgroups split K: the decode kernel
    // with a K too long for one workgroup, and the tiled kernel where its plan splits K.
    *bytes = workspace_needed(pick_path(M, kPathAuto), M, N, K);
    return DGQ_OK;
}

dgq_status dgq_linear_acc_workspace_bytes(int M, int N, int K, int group, int path, size_t *bytes)
{
    if (!bytes) return DGQ_ERR_NULL;
    if (M < 1) return DGQ_ERR_SHAPE;
    if (path < kPathAuto || path > kPathStreamGeneric) return DGQ_ERR_RANGE;
    if (dgq_status st = check_shape(N, K, group)) return st;
    if ((path == kPathStream || path == kPathStreamGeneric) && M > dgq::kStreamMaxM) return DGQ_ERR_SHAPE;
    *bytes = workspace_needed(pick_path(M, path), M, N, K);
    return DGQ_OK;
}

dgq_status dgq_pack_weights(const int8_t *w4, const uint8_t *s2, int K, int N, int group, void *qweight,
                            void *scales, int32_t *bad_count, void *stream)
{
    if (!w4 || !s2 || !qweight || !scales) return DGQ_ERR_NULL;
    if (dgq_status st = check_shape(N, K, group)) return st;
    if (!aligned16(w4) || !aligned16(s2) || !aligned16(qweight) || !aligned16(scales)) return DGQ_ERR_ALIGN;
    if (bad_count && (reinterpret_cast<uintptr_t>(bad_count) & 3u)) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_pack(w4, s2, K, N, group, qweight, scales, bad_count,
                                       static_cast<hipStream_t>(stream)));
}

dgq_status dgq_unpack_weights(const void *qweight, const void *scales, int K, int N, int group, int8_t *w_s8,
                              void *stream)
{
    if (!qweight || !scales || !w_s8) return DGQ_ERR_NULL;
    if (dgq_status st = check_shape(N, K, group)) return st;
    if (!aligned16(qweight) || !aligned16(scales) || !aligned16(w_s8)) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_unpack(qweight, scales, 0, K, N, group, w_s8, static_cast<hipStream_t>(stream)));
}

dgq_status dgq_packed_sizes_zp(int K, int N, int group, size_t *qweight_bytes, size_t *scales_zp_bytes)
{
    if (!qweight_bytes || !scales_zp_bytes) return DGQ_ERR_NULL;
    if (dgq_status st = check_shape(N, K, group)) return st;
    const size_t ng = (size_t)K / group;
    *qweight_bytes = (size_t)K * (size_t)N / 2;
    *scales_zp_bytes = ((size_t)N / 16) * ((ng + 1) / 2) * 64;
    return DGQ_OK;
}

dgq_status dgq_pack_weights_zp(const uint8_t *w_u4, const uint8_t *s2, const uint8_t *zp, int K, int N, int group,
                               void *qweight, void *scales_zp, int32_t *bad_count, void *stream)
{
    if (!w_u4 || !s2 || !zp || !qweight || !scales_zp) return DGQ_ERR_NULL;
    if (dgq_status st = check_shape(N, K, group)) return st;
    if (!aligned16(w_u4) || !aligned16(s2) || !aligned16(zp) || !aligned16(qweight) || !aligned16(scales_zp))
        return DGQ_ERR_ALIGN;
    if (bad_count && (reinterpret_cast<uintptr_t>(bad_count) & 3u)) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_pack_zp(w_u4, s2, zp, K, N, group, qweight, scales_zp, bad_count,
                                          static_cast<hipStream_t>(stream)));
}

dgq_status dgq_unpack_weights_zp(const void *qweight, const void *scales_zp, int K, int N, int group, int8_t *w_s8,
                                 void *stream)
{
    if (!qweight || !scales_zp || !w_s8) return DGQ_ERR_NULL;
    if (dgq_status st = check_shape(N, K, group)) return st;
    if (!aligned16(qweight) || !aligned16(scales_zp) || !aligned16(w_s8)) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_unpack(qweight, scales_zp, 1, K, N, group, w_s8, static_cast<hipStream_t>(stream)));
}

dgq_status dgq_quantize_weights_rtn(const uint16_t *W, int K, int N, int group, int8_t *w4, uint8_t *s2,
                                    float *s1, void *stream)
{
    if (!W || !w4 || !s2 || !s1) return DGQ_ERR_NULL;
    if (dgq_status st = check_shape(N, K, group)) return st;
    if (!aligned16(W) || !aligned16(w4) || !aligned16(s2) || !aligned16(s1)) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_quantize_rtn(W, K, N, group, w4, s2, s1, static_cast<hipStream_t>(stream)));
}

dgq_status dgq_quantize_weights_grid(const uint16_t *W, int K, int N, int group, int n_alpha, float step,
                                     uint8_t *w_u4, uint8_t *zp, uint8_t *s2, float *s1, void *workspace,
                                     size_t workspace_bytes, void *stream)
{
    if (!W || !w_u4 || !zp || !s2 || !s1 || !workspace) return DGQ_ERR_NULL;
    if (dgq_status st = check_shape(N, K, group)) return st;
    if (n_alpha < 1 || n_alpha > 1024 || !(step >= 0.0f) || !((float)(n_alpha - 1) * step < 1.0f)) return DGQ_ERR_RANGE;
    if (workspace_bytes < (size_t)(K / group) * (size_t)N * sizeof(float)) return DGQ_ERR_WORKSPACE;
    if (!aligned16(W) || !aligned16(w_u4) || !aligned16(zp) || !aligned16(s2) || !aligned16(s1) || !aligned16(workspace))
        return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_quantize_grid(W, K, N, group, n_alpha, step, w_u4, zp, s2, s1,
                                                static_cast<float *>(workspace), static_cast<hipStream_t>(stream)));
}

dgq_status dgq_quantize_weights_grid_act_workspace_bytes(int M, int K, int N, int group, size_t *bytes)
{
    if (!bytes) return DGQ_ERR_NULL;
    if (M < 1 || M > 4096) return DGQ_ERR_SHAPE;
    if (dgq_status st = check_shape(N, K, group)) return st;
    *bytes = dgq::quantize_grid_act_workspace_bytes(M, K, N, group);
    return DGQ_OK;
}

dgq_status dgq_quantize_weights_grid_act(const uint16_t *W, const uint16_t *X, const int8_t *xq, const float *sx, int M,
                                         int K, int N, int group, int n_alpha, float step, uint8_t *w_u4, uint8_t *zp,
                                         uint8_t *s2, float *s1, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!W || !X || !xq || !sx || !w_u4 || !zp || !s2 || !s1 || !workspace) return DGQ_ERR_NULL;
    if (M < 1 || M > 4096) return DGQ_ERR_SHAPE;
    if (dgq_status st = check_shape(N, K, group)) return st;
    if (n_alpha < 1 || n_alpha > 1024 || !(step >= 0.0f) || !((float)(n_alpha - 1) * step < 1.0f)) return DGQ_ERR_RANGE;
    if (workspace_bytes < dgq::quantize_grid_act_workspace_bytes(M, K, N, group)) return DGQ_ERR_WORKSPACE;
    if (!aligned16(W) || !aligned16(X) || !aligned16(xq) || !aligned16(w_u4) || !aligned16(zp) || !aligned16(s2) ||
        !aligned16(s1) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(sx) & 3u))
        return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_quantize_grid_act(W, X, xq, sx, M, K, N, group, n_alpha, step, w_u4, zp, s2, s1,
                                                    static_cast<float *>(workspace), static_cast<hipStream_t>(stream)));
}

dgq_status dgq_quant_act(const uint16_t *x, int M, int K, int8_t *xq, float *sx, void *stream)
{
    if (!x || !xq || !sx) return DGQ_ERR_NULL;
    if (M < 1 || K < 128 || K > 131072 || (K % 128) != 0) return DGQ_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(xq) || (reinterpret_cast<uintptr_t>(sx) & 3u)) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_quant_act(x, M, K, xq, sx, static_cast<hipStream_t>(stream)));
}

static dgq_status linear_fp16(const int8_t *xq, const float *sx, const void *qweight, const void *scales,
                              int zp_form, const float *s1, uint16_t *out, int M, int N, int K, int group,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    if (!xq || !sx || !qweight || !scales || !s1 || !out) return DGQ_ERR_NULL;
    if (M < 1) return DGQ_ERR_SHAPE;
    if (dgq_status st = check_shape(N, K, group)) return st;
    if (!aligned16(xq) || !aligned16(qweight) || !aligned16(scales) || !aligned16(out) ||
        (reinterpret_cast<uintptr_t>(sx) & 3u) || (reinterpret_cast<uintptr_t>(s1) & 3u))
        return DGQ_ERR_ALIGN;
    dgq::LinearArgs a{xq, sx, static_cast<const uint4 *>(qweight), static_cast<const uint32_t *>(scales),
                      s1, out, nullptr, M, N, K, group, zp_form};
    return run_linear(a, kPathAuto, workspace, workspace_bytes, stream);
}

static dgq_status linear_acc(const int8_t *xq, const void *qweight, const void *scales, int zp_form,
                             int32_t *acc_out, int M, int N, int K, int group, int path, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    if (!xq || !qweight || !scales || !acc_out) return DGQ_ERR_NULL;
    if (M < 1) return DGQ_ERR_SHAPE;
    if (dgq_status st = check_shape(N, K, group)) return st;
    if (!aligned16(xq) || !aligned16(qweight) || !aligned16(scales) || !aligned16(acc_out)) return DGQ_ERR_ALIGN;
    dgq::LinearArgs a{xq, nullptr, static_cast<const uint4 *>(qweight), static_cast<const uint32_t *>(scales),
                      nullptr, nullptr, acc_out, M, N, K, group, zp_form};
    return run_linear(a, path, workspace, workspace_bytes, stream);
}

dgq_status dgq_smooth_scales(const uint16_t *X, int M, int K, float pct, float *k, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    if (!X || !k || !workspace) return DGQ_ERR_NULL;
    if (M < 1 || M > 65535 || K < 128 || K > 131072 || (K % 128) != 0) return DGQ_ERR_SHAPE;
    if (!(pct > 0.0f) || !(pct <= 1.0f)) return DGQ_ERR_RANGE;
    if (workspace_bytes < (size_t)K * sizeof(float)) return DGQ_ERR_WORKSPACE;
    if (!aligned16(X) || !aligned16(k) || !aligned16(workspace)) return DGQ_ERR_ALIGN;
    int r = (int)std::ceil(pct * (float)K);   // fp32 product, as the definition is stated
    if (r < 1) r = 1;
    if (r > K) r = K;
    return hip_result(dgq::launch_smooth_scales(X, M, K, r, k, static_cast<float *>(workspace),
                                                static_cast<hipStream_t>(stream)));
}

dgq_status dgq_smooth_apply(const uint16_t *W, const uint16_t *X, const float *k, int M, int K, int N,
                            uint16_t *Wout, uint16_t *Xout, void *stream)
{
    if (!k || (!W && !X) || (W && !Wout) || (X && !Xout)) return DGQ_ERR_NULL;
    if (K < 1 || K > 131072 || (W && N < 1) || (X && M < 1)) return DGQ_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(Wout) |
         reinterpret_cast<uintptr_t>(Xout)) & 1u)
        return DGQ_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(k) & 3u) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_smooth_apply(W, X, k, M, K, N, Wout, Xout, static_cast<hipStream_t>(stream)));
}

dgq_status dgq_rmsnorm_quant_act(const uint16_t *x, const uint16_t *gamma, int M, int K, float eps, int8_t *xq,
                                 float *sx, void *stream)
{
    if (!x || !gamma || !xq || !sx) return DGQ_ERR_NULL;
    if (M < 1 || K < 128 || K > 24576 || (K % 128) != 0) return DGQ_ERR_SHAPE;
    if (!(eps >= 0.0f) || !(eps < 1.0f)) return DGQ_ERR_RANGE;
    if (!aligned16(x) || !aligned16(gamma) || !aligned16(xq) || (reinterpret_cast<uintptr_t>(sx) & 3u))
        return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_rmsnorm_quant_act(x, gamma, M, K, eps, xq, sx, static_cast<hipStream_t>(stream)));
}

dgq_status dgq_silu_mul_quant_act(const uint16_t *gate_up, int M, int I, int8_t *xq, float *sx, void *stream)
{
    if (!gate_up || !xq || !sx) return DGQ_ERR_NULL;
    if (M < 1 || I < 128 || I > 24576 || (I % 128) != 0) return DGQ_ERR_SHAPE;
    if (!aligned16(gate_up) || !aligned16(xq) || (reinterpret_cast<uintptr_t>(sx) & 3u)) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_silu_mul_quant_act(gate_up, M, I, xq, sx, static_cast<hipStream_t>(stream)));
}

dgq_status dgq_quant_act_static(const uint16_t *x, int M, int K, float scale, int8_t *xq, float *sx, void *stream)
{
    if (!x || !xq || !sx) return DGQ_ERR_NULL;
    if (M < 1 || K < 128 || K > 131072 || (K % 128) != 0) return DGQ_ERR_SHAPE;
    if (!(scale > 0.0f) || !(scale < 3.0e38f)) return DGQ_ERR_RANGE;
    if (!aligned16(x) || !aligned16(xq) || (reinterpret_cast<uintptr_t>(sx) & 3u)) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_quant_act_static(x, M, K, scale, xq, sx, static_cast<hipStream_t>(stream)));
}

dgq_status dgq_linear_a8w4(const int8_t *xq, const float *sx, const void *qweight, const void *scales,
                           const float *s1, uint16_t *out, int M, int N, int K, int group, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    return linear_fp16(xq, sx, qweight, scales, 0, s1, out, M, N, K, group, workspace, workspace_bytes, stream);
}

dgq_status dgq_linear_a8w4_noalloc(const int8_t *xq, const float *sx, const void *qweight, const void *scales,
                                   const float *s1, uint16_t *out, int M, int N, int K, int group, void *stream)
{
    if (!xq || !sx || !qweight || !scales || !s1 || !out) return DGQ_ERR_NULL;
    if (M < 1) return DGQ_ERR_SHAPE;
    if (dgq_status st = check_shape(N, K, group)) return st;
    const size_t need = workspace_needed(pick_path(M, kPathAuto), M, N, K);
    if (need > kScratchBytes) return DGQ_ERR_WORKSPACE;
    void *ws = nullptr;
    if (need > 0) {
        if (dgq_status st = hip_result(scratch_of_current_device(&ws))) return st;
    }
    return linear_fp16(xq, sx, qweight, scales, 0, s1, out, M, N, K, group, ws, need, stream);
}

dgq_status dgq_linear_a8w4_acc(const int8_t *xq, const void *qweight, const void *scales, int32_t *acc_out,
                               int M, int N, int K, int group, int path, void *workspace, size_t workspace_bytes,
                               void *stream)
{
    return linear_acc(xq, qweight, scales, 0, acc_out, M, N, K, group, path, workspace, workspace_bytes, stream);
}

dgq_status dgq_linear_a8w4_zp(const int8_t *xq, const float *sx, const void *qweight, const void *scales_zp,
                              const float *s1, uint16_t *out, int M, int N, int K, int group, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    return linear_fp16(xq, sx, qweight, scales_zp, 1, s1, out, M, N, K, group, workspace, workspace_bytes, stream);
}

dgq_status dgq_linear_a8w4_zp_acc(const int8_t *xq, const void *qweight, const void *scales_zp, int32_t *acc_out,
                                  int M, int N, int K, int group, int path, void *workspace, size_t workspace_bytes,
                                  void *stream)
{
    return linear_acc(xq, qweight, scales_zp, 1, acc_out, M, N, K, group, path, workspace, workspace_bytes, stream);
}

static dgq_status quant_linear_workspace(int M, int N, int K, int group, bool rms, size_t *bytes)
{
    if (!bytes) return DGQ_ERR_NULL;
    if (M < 1) return DGQ_ERR_SHAPE;
    if (dgq_status st = check_shape(N, K, group)) return st;
    const int forced = kPathAuto;
    if (quantizes_in_kernel(M, K, forced) && (!rms || dgq::decode_plan(K).spw <= dgq::kRmsDecodeMaxStepsPerWave))
        *bytes = 0;
    else
        *bytes = round256((size_t)M * K) + round256((size_t)M * sizeof(float)) +
                 round256(workspace_needed(pick_path(M, forced), M, N, K));
    return DGQ_OK;
}

dgq_status dgq_quant_linear_workspace_bytes(int M, int N, int K, int group, size_t *bytes)
{
    return quant_linear_workspace(M, N, K, group, false, bytes);
}

dgq_status dgq_rmsnorm_quant_linear_workspace_bytes(int M, int N, int K, int group, size_t *bytes)
{
    return quant_linear_workspace(M, N, K, group, true, bytes);
}

dgq_status dgq_quant_linear_a8w4(const uint16_t *x, const void *qweight, const void *scales, const float *s1,
                                 uint16_t *out, float *sx_out, int M, int N, int K, int group, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    return quant_linear(x, nullptr, 0.0f, qweight, scales, 0, s1, out, sx_out, M, N, K, group, workspace,
                        workspace_bytes, stream);
}

dgq_status dgq_rmsnorm_quant_linear_a8w4(const uint16_t *x, const uint16_t *gamma, float eps, const void *qweight,
                                         const void *scales, const float *s1, uint16_t *out, float *sx_out, int M,
                                         int N, int K, int group, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!gamma) return DGQ_ERR_NULL;
    return quant_linear(x, gamma, eps, qweight, scales, 0, s1, out, sx_out, M, N, K, group, workspace,
                        workspace_bytes, stream);
}

dgq_status dgq_rmsnorm_quant_linear_a8w4_zp(const uint16_t *x, const uint16_t *gamma, float eps, const void *qweight,
                                            const void *scales_zp, const float *s1, uint16_t *out, float *sx_out,
                                            int M, int N, int K, int group, void *workspace, size_t workspace_bytes,
                                            void *stream)
{
    if (!gamma) return DGQ_ERR_NULL;
    return quant_linear(x, gamma, eps, qweight, scales_zp, 1, s1, out, sx_out, M, N, K, group, workspace,
                        workspace_bytes, stream);
}

dgq_status dgq_quant_linear_a8w4_zp(const uint16_t *x, const void *qweight, const void *scales_zp, const float *s1,
                                    uint16_t *out, float *sx_out, int M, int N, int K, int group, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    return quant_linear(x, nullptr, 0.0f, qweight, scales_zp, 1, s1, out, sx_out, M, N, K, group, workspace,
                        workspace_bytes, stream);
}

dgq_status dgq_quant_linear_plan(int M, int N, int K, int group, char *buf, size_t buf_bytes)
{
    if (!buf) return DGQ_ERR_NULL;
    if (M < 1 || buf_bytes < 96) return DGQ_ERR_SHAPE;
    if (dgq_status st = check_shape(N, K, group)) return st;
    if (quantizes_in_kernel(M, K, kPathAuto)) {
        const dgq::DecodePlan p = dgq::decode_plan(K);
        std::snprintf(buf, buf_bytes, "quant_linear_decode_%skernel<%d, %d, %d>", dgq::decode_streams_weights(N, K) ? "nt_" : "",
                      p.spw, p.pf, group);
        return DGQ_OK;
    }
    return dgq_linear_plan(M, N, K, group, buf, buf_bytes);
}

dgq_status dgq_linear_plan(int M, int N, int K, int group, char *buf, size_t buf_bytes)
{
    if (!buf) return DGQ_ERR_NULL;
    if (M < 1 || buf_bytes < 96) return DGQ_ERR_SHAPE;
    if (dgq_status st = check_shape(N, K, group)) return st;
    switch (pick_path(M, kPathAuto)) {
    case kPathStream: {
        const dgq::DecodePlan p = dgq::decode_plan(K);
        if (dgq::decode_streams_weights(N, K))
            std::snprintf(buf, buf_bytes, "linear_decode_nt_kernel<%d, %d, %d, %s>", p.spw, p.pf, group,
                          p.ksplit > 1 ? "true" : "false");
        else
            std::snprintf(buf, buf_bytes, "linear_decode_kernel<%d, %d, %d, false, %s>", p.spw, p.pf, group,
                          p.ksplit > 1 ? "true" : "false");
        break;
    }
    case kPathStreamGeneric: {
        const dgq::StreamPlan p = dgq::stream_plan(M, N, K);
        std::snprintf(buf, buf_bytes, "linear_stream_kernel<%d, %d, %d, %d, false>", p.mtiles, group, p.waves, p.depth);
        break;
    }
    default:
        dgq::tiled_plan_name(M, N, K, group, buf, buf_bytes);
    }
    return DGQ_OK;
}

static dgq_status bmm_check(const void *a, const void *b, int batch, int M, int N, int K)
{
    if (!a || !b) return DGQ_ERR_NULL;
    // INT32 sums cannot wrap: 128 * 128 * K < 2^31; the batch is a grid dimension
    if (batch < 1 || batch > 65535 || M < 1 || N < 1 || K < 16 || K > 65536 || (K % 16) != 0) return DGQ_ERR_SHAPE;
    if ((long long)M > (1LL << 24) || (long long)N > (1LL << 24)) return DGQ_ERR_SHAPE;
    if (!aligned16(a) || !aligned16(b)) return DGQ_ERR_ALIGN;
    return DGQ_OK;
}

dgq_status dgq_bmm_s8(const int8_t *a, const int8_t *b, const float *sa, const float *sb, uint16_t *out, int batch,
                      int M, int N, int K, void *stream)
{
    if (!out) return DGQ_ERR_NULL;
    if (dgq_status st = bmm_check(a, b, batch, M, N, K)) return st;
    if (!aligned16(out) || (reinterpret_cast<uintptr_t>(sa) & 3u) || (reinterpret_cast<uintptr_t>(sb) & 3u)) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_bmm_s8(a, b, sa, sb, out, nullptr, batch, M, N, K, static_cast<hipStream_t>(stream)));
}

dgq_status dgq_bmm_s8_acc(const int8_t *a, const int8_t *b, int32_t *acc_out, int batch, int M, int N, int K, void *stream)
{
    if (!acc_out) return DGQ_ERR_NULL;
    if (dgq_status st = bmm_check(a, b, batch, M, N, K)) return st;
    if (!aligned16(acc_out)) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_bmm_s8(a, b, nullptr, nullptr, nullptr, acc_out, batch, M, N, K, static_cast<hipStream_t>(stream)));
}

dgq_status dgq_probe_read(const void *src, size_t bytes, uint32_t *sink, int workgroups, void *stream)
{
    if (!src || !sink) return DGQ_ERR_NULL;
    if (bytes < 16 || workgroups < 1 || workgroups > 65536) return DGQ_ERR_SHAPE;
    if (!aligned16(src) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_probe_read(src, bytes, sink, workgroups, static_cast<hipStream_t>(stream)));
}

dgq_status dgq_probe_mfma(const void *operands, size_t bytes, int iters, uint32_t *sink, int workgroups, void *stream)
{
    if (!operands || !sink) return DGQ_ERR_NULL;
    if (bytes < 96 || iters < 1 || iters > (1 << 24) || workgroups < 1 || workgroups > 65536) return DGQ_ERR_SHAPE;
    if (!aligned16(operands) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return DGQ_ERR_ALIGN;
    return hip_result(dgq::launch_probe_mfma(operands, bytes, iters, sink, workgroups, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
