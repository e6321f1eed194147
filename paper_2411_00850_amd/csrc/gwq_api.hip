// C ABI of libgwq: host-side validation and dispatch.  Every check runs before the first HIP call,
// so argument errors are reported on machines without a GPU as well.
#include <string.h>

#include <mutex>

#include "gwq_internal.h"

// Scratch of gwq_linear_static: one copy per GPU, held until the process ends.  In host code this name is
// only a handle for hipGetSymbolAddress; the device address is asked once per device (static_scratch below).
static __device__ __align__(256) unsigned char scratch[GWQ_STATIC_SCRATCH_BYTES];

namespace {

std::mutex g_scratch_mutex;
void *g_scratch_ptr[64];                                // per device: address of its copy of `scratch`

// Device address of the current device's copy of `scratch`.
hipError_t static_scratch(unsigned char **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<unsigned char *>(g_scratch_ptr[dev]);
    return hipSuccess;
}

// Measurement hooks of gwq_tuning_set: process-wide, read once per call.
std::atomic<int> g_decode_waves{0};   // 0 = heuristic
std::atomic<int> g_gemm_ms{0};        // rows of Y per GEMM block; 0 = heuristic
std::atomic<int> g_decode_stream{0};  // 0 = heuristic, 1 = never the streaming kernel, 2 = wherever it can run
std::atomic<int> g_decode_tiles{0};   // tiles per block of the streaming kernel; 0 = heuristic
std::atomic<int> g_decode_lean{0};    // largest M of the kernel that keeps X[M][K] in LDS; 0 = built-in
std::atomic<int> g_decode_pairs{0};   // two tiles per block in that kernel for 5 <= M <= 8: 0 = heuristic, 1 = never, 2 = wherever it fits
std::atomic<int> g_pack_full{0};      // 1: gwq_pack always runs its passes over all scores (never the candidate list)

gwq::DecodeTuning decode_tuning() { return gwq::DecodeTuning{g_decode_waves, g_decode_stream, g_decode_tiles, g_decode_lean, g_decode_pairs}; }

gwq_status check_shape(int64_t N, int64_t K, int bits, int group, uint32_t ppm)
{
    if (bits != 3 && bits != 4) return GWQ_ERR_UNSUPPORTED;
    if (group != 16 && group != 32 && group != 64 && group != gwq::kGroup) return GWQ_ERR_UNSUPPORTED;
    if (N < 1 || K < gwq::kGroup || K > 65536 || K % gwq::kGroup != 0) return GWQ_ERR_SHAPE;
    if (N * K >= ((int64_t)1 << 32)) return GWQ_ERR_SHAPE;
    if (K / group > 2048) return GWQ_ERR_SHAPE;          // a tile's scales and zero points (48 bytes per group) are staged in LDS
    if (ppm > 1000000u) return GWQ_ERR_SHAPE;
    return GWQ_OK;
}

int64_t outlier_count(int64_t N, int64_t K, uint32_t ppm)
{
    return ((int64_t)ppm * N * K + 999999) / 1000000;
}

gwq_status check_packed(const gwq_packed *P)
{
    if (!P) return GWQ_ERR_NULL;
    gwq_status s = check_shape(P->N, P->K, P->bits, P->group, P->outlier_ppm);
    if (s != GWQ_OK) return s;
    if (P->n_outliers != outlier_count(P->N, P->K, P->outlier_ppm)) return GWQ_ERR_SHAPE;
    if (!P->qweight || !P->scales || !P->zeros || !P->row_ptr || !P->col_idx || !P->out_val) return GWQ_ERR_NULL;
    if ((uintptr_t)P->row_ptr & 3) return GWQ_ERR_SHAPE;
    if ((uintptr_t)P->index & 15) return GWQ_ERR_SHAPE;  // optional, but aligned when present
    return GWQ_OK;
}

// Shared argument checks of the gwq_linear variants.
gwq_status check_xy(const gwq_packed *P, const void *X_f16, int32_t M, const void *Y_f16)
{
    gwq_status s = check_packed(P);
    if (s != GWQ_OK) return s;
    if (!X_f16 || !Y_f16) return GWQ_ERR_NULL;
    if (M < 1 || (int64_t)M * P->N >= ((int64_t)1 << 40)) return GWQ_ERR_SHAPE;
    if (((uintptr_t)X_f16 | (uintptr_t)P->qweight | (uintptr_t)P->scales | (uintptr_t)P->zeros |
         (uintptr_t)P->col_idx | (uintptr_t)P->out_val) & 15)
        return GWQ_ERR_SHAPE;
    return GWQ_OK;
}

// The same plus the index: `index` is the workspace (whose head becomes the index) or the prebuilt index.
gwq_status check_linear(const gwq_packed *P, const void *X_f16, int32_t M, const void *Y_f16, const void *index,
                        size_t index_bytes)
{
    gwq_status s = check_xy(P, X_f16, M, Y_f16);
    if (s != GWQ_OK) return s;
    if (M > 16 && (!index || index_bytes < gwq::gemm_index_bytes(P->N, P->K, P->group))) return GWQ_ERR_WORKSPACE;
    if (M > 16 && ((uintptr_t)index & 15)) return GWQ_ERR_SHAPE;
    return GWQ_OK;
}

}  // namespace

namespace gwq {

int device_cus()
{
    static std::atomic<int> cus[64];                    // 0 = not asked yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cus[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
        cus[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

hipError_t allow_dynamic_lds(const void *kernel, int bytes, std::atomic<uint32_t> &done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) dev = -1;
    const bool tracked = dev >= 0 && dev < 32;
    if (tracked && (done.load(std::memory_order_acquire) >> dev & 1u)) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && tracked) done.fetch_or(1u << dev, std::memory_order_release);
    return e;
}

}  // namespace gwq

extern "C" {

gwq_status gwq_layout(int32_t N, int32_t K, int32_t bits, int32_t group, uint32_t outlier_ppm,
                      int32_t M_max, gwq_sizes *out)
{
    if (!out) return GWQ_ERR_NULL;
    gwq_status s = check_shape(N, K, bits, group, outlier_ppm);
    if (s != GWQ_OK) return s;
    if (M_max < 0) return GWQ_ERR_SHAPE;
    const int64_t blocks = (int64_t)N * (K / gwq::kGroup), groups = (int64_t)N * (K / group);
    const int64_t k_out = outlier_count(N, K, outlier_ppm);
    memset(out, 0, sizeof(*out));
    out->qweight = (size_t)blocks * gwq::words_per_group(bits) * 4;
    // Read with wide (partly unaligned) loads by the kernels: whole 16-byte vectors plus one spare.
    out->scales = ((size_t)groups * 2 + 15) / 16 * 16 + 16;
    out->zeros = ((size_t)groups + 15) / 16 * 16 + 16;
    out->row_ptr = (size_t)(N + 1) * 4;
    out->col_idx = ((size_t)k_out * 2 + 15) / 16 * 16 + 16;
    out->out_val = out->col_idx;
    out->pack_workspace = gwq::pack_workspace_bytes(N, K);
    out->linear_index = gwq::gemm_index_bytes(N, K, group);
    out->linear_scratch = gwq::gemm_scratch_bytes(N, M_max);
    out->linear_workspace = M_max > 16 ? out->linear_index + out->linear_scratch : 0;
    out->n_outliers = k_out;
    out->quality_workspace = gwq::quality_workspace_bytes(N);
    return GWQ_OK;
}

gwq_status gwq_pack(const void *W_f16, const void *score, int32_t score_dtype, gwq_packed *dst,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    if (!W_f16 || !score) return GWQ_ERR_NULL;
    gwq_status s = check_packed(dst);
    if (s != GWQ_OK) return s;
    if (score_dtype != GWQ_SCORE_F32 && score_dtype != GWQ_SCORE_F16) return GWQ_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < gwq::pack_workspace_bytes(dst->N, dst->K)) return GWQ_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 3) || ((uintptr_t)W_f16 & 15) || ((uintptr_t)score & 15)) return GWQ_ERR_SHAPE;
    hipError_t e = gwq::launch_pack(W_f16, score, score_dtype == GWQ_SCORE_F16, *dst,
                                    static_cast<uint32_t *>(workspace), g_pack_full != 0, static_cast<hipStream_t>(stream));
    if (e == hipSuccess && dst->index) e = gwq::launch_gemm_index(*dst, dst->index, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GWQ_OK : GWQ_ERR_DEVICE;
}

gwq_status gwq_quality(const gwq_packed *P, const void *W_f16, const void *score, int32_t score_dtype,
                       double *out_f64, void *workspace, size_t workspace_bytes, void *stream)
{
    gwq_status s = check_packed(P);
    if (s != GWQ_OK) return s;
    if (!W_f16 || !score || !out_f64) return GWQ_ERR_NULL;
    if (score_dtype != GWQ_SCORE_F32 && score_dtype != GWQ_SCORE_F16) return GWQ_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < gwq::quality_workspace_bytes(P->N)) return GWQ_ERR_WORKSPACE;
    if (((uintptr_t)W_f16 & 15) || ((uintptr_t)score & 15) || ((uintptr_t)workspace & 7) || ((uintptr_t)out_f64 & 7))
        return GWQ_ERR_SHAPE;
    hipError_t e = gwq::launch_quality(*P, W_f16, score, score_dtype == GWQ_SCORE_F16, workspace, out_f64,
                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GWQ_OK : GWQ_ERR_DEVICE;
}

gwq_status gwq_score(const void *dY_f16, const void *X_f16, int32_t M, int32_t N, int32_t K, float alpha,
                     float beta, float *score_f32, void *stream)
{
    if (!dY_f16 || !X_f16 || !score_f32) return GWQ_ERR_NULL;
    if (M < 1 || N < 1 || N > (1 << 24) || K < gwq::kGroup || K % gwq::kGroup || K > 65536) return GWQ_ERR_SHAPE;
    if (((uintptr_t)X_f16 & 15) || ((uintptr_t)score_f32 & 3) || ((uintptr_t)dY_f16 & (N % 8 ? 1 : 15)))
        return GWQ_ERR_SHAPE;
    hipError_t e = gwq::launch_score(dY_f16, X_f16, M, N, K, alpha, beta, score_f32, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GWQ_OK : GWQ_ERR_DEVICE;
}

gwq_status gwq_linear(const gwq_packed *P, const void *X_f16, int32_t M, void *Y_f16, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    gwq_status s = check_linear(P, X_f16, M, Y_f16, workspace, workspace_bytes);
    if (s != GWQ_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (M <= 16) {
        e = gwq::launch_decode(1, &P, &X_f16, M, &Y_f16, decode_tuning(), st);
    } else {
        // The workspace holds the index, then (whatever is left) the partial sums of a K-split launch.
        // A layer that carries its index (filled by gwq_pack) is not indexed again.
        const size_t ib = gwq::gemm_index_bytes(P->N, P->K, P->group);
        e = P->index ? hipSuccess : gwq::launch_gemm_index(*P, workspace, st);
        if (e == hipSuccess)
            e = gwq::launch_gemm(*P, X_f16, M, Y_f16, P->index ? P->index : workspace,
                                 static_cast<char *>(workspace) + ib, workspace_bytes - ib, g_gemm_ms, st);
    }
    return e == hipSuccess ? GWQ_OK : GWQ_ERR_DEVICE;
}

gwq_status gwq_linear_bf16(const gwq_packed *P, const void *X_bf16, int32_t M, void *Y_bf16, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    gwq_status s = check_linear(P, X_bf16, M, Y_bf16, workspace, workspace_bytes);
    if (s != GWQ_OK) return s;
    if (P->group != gwq::kGroup) return GWQ_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (M <= 16) {
        gwq::DecodeTuning t = decode_tuning();
        t.bf16 = true;
        e = gwq::launch_decode(1, &P, &X_bf16, M, &Y_bf16, t, st);
    } else {
        const size_t ib = gwq::gemm_index_bytes(P->N, P->K, P->group);
        e = P->index ? hipSuccess : gwq::launch_gemm_index(*P, workspace, st);
        if (e == hipSuccess)
            e = gwq::launch_gemm(*P, X_bf16, M, Y_bf16, P->index ? P->index : workspace,
                                 static_cast<char *>(workspace) + ib, workspace_bytes - ib, g_gemm_ms, st, nullptr, true);
    }
    return e == hipSuccess ? GWQ_OK : GWQ_ERR_DEVICE;
}

gwq_status gwq_linear_index(const gwq_packed *P, void *index, size_t index_bytes, void *stream)
{
    gwq_status s = check_packed(P);
    if (s != GWQ_OK) return s;
    if (!index || index_bytes < gwq::gemm_index_bytes(P->N, P->K, P->group)) return GWQ_ERR_WORKSPACE;
    if ((uintptr_t)index & 15) return GWQ_ERR_SHAPE;
    hipError_t e = gwq::launch_gemm_index(*P, index, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GWQ_OK : GWQ_ERR_DEVICE;
}

gwq_status gwq_linear_indexed(const gwq_packed *P, const void *X_f16, int32_t M, void *Y_f16, const void *index,
                              size_t index_bytes, void *scratch, size_t scratch_bytes, void *stream)
{
    gwq_status s = check_linear(P, X_f16, M, Y_f16, index, index_bytes);
    if (s != GWQ_OK) return s;
    if (scratch && ((uintptr_t)scratch & 15)) return GWQ_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = M <= 16 ? gwq::launch_decode(1, &P, &X_f16, M, &Y_f16, decode_tuning(), st)
                           : gwq::launch_gemm(*P, X_f16, M, Y_f16, index, scratch, scratch ? scratch_bytes : 0,
                                              g_gemm_ms, st);
    return e == hipSuccess ? GWQ_OK : GWQ_ERR_DEVICE;
}

gwq_status gwq_linear_static(const gwq_packed *P, const void *X_f16, int32_t M, void *Y_f16, void *stream)
{
    gwq_status s = check_xy(P, X_f16, M, Y_f16);
    if (s != GWQ_OK) return s;
    // What gwq_linear would want as its workspace for this M (host arithmetic only).
    const size_t ib = (M > 16 && !P->index) ? gwq::gemm_index_bytes(P->N, P->K, P->group) : 0;
    const size_t sb = M > 16 ? gwq::gemm_scratch_bytes(P->N, M) : 0;
    if (ib + sb > GWQ_STATIC_SCRATCH_BYTES) return GWQ_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (M <= 16)                                        // the decode kernels use no scratch
        return gwq::launch_decode(1, &P, &X_f16, M, &Y_f16, decode_tuning(), st) == hipSuccess ? GWQ_OK : GWQ_ERR_DEVICE;
    unsigned char *base = nullptr;
    if (static_scratch(&base) != hipSuccess) return GWQ_ERR_DEVICE;
    // Same layout as gwq_linear's workspace: the index (when the layer carries none), then the partial sums.
    hipError_t e = P->index ? hipSuccess : gwq::launch_gemm_index(*P, base, st);
    if (e == hipSuccess)
        e = gwq::launch_gemm(*P, X_f16, M, Y_f16, P->index ? P->index : base, base + ib, sb, g_gemm_ms, st);
    return e == hipSuccess ? GWQ_OK : GWQ_ERR_DEVICE;
}

gwq_status gwq_linear_batch(int32_t count, const gwq_packed *const *P, const void *const *X_f16, int32_t M,
                            void *const *Y_f16, void *stream)
{
    if (!P || !X_f16 || !Y_f16) return GWQ_ERR_NULL;
    if (count < 1 || count > GWQ_MAX_BATCH || M < 1 || M > 16) return GWQ_ERR_SHAPE;
    for (int32_t i = 0; i < count; ++i) {
        gwq_status s = check_packed(P[i]);
        if (s != GWQ_OK) return s;
        if (!X_f16[i] || !Y_f16[i]) return GWQ_ERR_NULL;
        if (P[i]->bits != P[0]->bits) return GWQ_ERR_UNSUPPORTED;
        if (((uintptr_t)X_f16[i] | (uintptr_t)P[i]->qweight | (uintptr_t)P[i]->scales | (uintptr_t)P[i]->zeros |
             (uintptr_t)P[i]->col_idx | (uintptr_t)P[i]->out_val) & 15)
            return GWQ_ERR_SHAPE;
    }
    // One launch per distinct K, in order of first appearance: a launch runs as many waves per block as
    // its longest rows need, and the surplus waves of a layer with shorter rows would only repeat work.
    bool done[GWQ_MAX_BATCH] = {};
    for (int32_t i = 0; i < count; ++i) {
        if (done[i]) continue;
        const gwq_packed *p[GWQ_MAX_BATCH];
        const void *x[GWQ_MAX_BATCH];
        void *y[GWQ_MAX_BATCH];
        int n = 0;
        for (int32_t j = i; j < count; ++j)
            if (!done[j] && P[j]->K == P[i]->K && P[j]->group == P[i]->group) {
                p[n] = P[j]; x[n] = X_f16[j]; y[n] = Y_f16[j];
                done[j] = true;
                ++n;
            }
        hipError_t e = gwq::launch_decode(n, p, x, M, y, decode_tuning(), static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return GWQ_ERR_DEVICE;
    }
    return GWQ_OK;
}

gwq_status gwq_linear_gate_up(const gwq_packed *P_gate, const gwq_packed *P_up, const void *X_f16, int32_t M, void *H_f16,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    gwq_status s = check_xy(P_gate, X_f16, M, H_f16);
    if (s != GWQ_OK) return s;
    s = check_xy(P_up, X_f16, M, H_f16);
    if (s != GWQ_OK) return s;
    if (M > 16 || P_gate->N != P_up->N || P_gate->K != P_up->K) return GWQ_ERR_SHAPE;
    if (P_gate->bits != P_up->bits || P_gate->group != P_up->group) return GWQ_ERR_UNSUPPORTED;
    if ((uintptr_t)workspace & 15) return GWQ_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const gwq_packed *p[2] = {P_gate, P_up};
    const void *x[2] = {X_f16, X_f16};
    if (M <= 4) {                                       // one launch: the second run of each block writes H
        void *y[2] = {H_f16, H_f16};
        gwq::DecodeTuning t = decode_tuning();
        t.gated_pairs = true;
        hipError_t e = gwq::launch_decode(2, p, x, M, y, t, st);
        if (e == hipSuccess) return GWQ_OK;
        if (e != hipErrorNotSupported) return GWQ_ERR_DEVICE;
    }
    // Larger batches (and rows too long for the kernel above): the two products into the workspace, then H.
    const size_t each = (size_t)M * P_gate->N * 2;
    if (!workspace || workspace_bytes < 2 * each) return GWQ_ERR_WORKSPACE;
    void *y[2] = {workspace, static_cast<char *>(workspace) + each};
    hipError_t e = gwq::launch_decode(2, p, x, M, y, decode_tuning(), st);
    if (e == hipSuccess) e = gwq::launch_silu_mul(y[0], y[1], H_f16, (size_t)M * P_gate->N, st);
    return e == hipSuccess ? GWQ_OK : GWQ_ERR_DEVICE;
}

gwq_status gwq_linear_plan(int32_t count, const gwq_packed *const *P, int32_t M, int32_t with_scratch, char *text,
                           size_t text_bytes)
{
    if (!P || !text) return GWQ_ERR_NULL;
    if (count < 1 || count > GWQ_MAX_BATCH || M < 1 || text_bytes < 1 || (M > 16 && count != 1)) return GWQ_ERR_SHAPE;
    for (int32_t i = 0; i < count; ++i) {
        gwq_status s = check_packed(P[i]);
        if (s != GWQ_OK) return s;
        if (P[i]->bits != P[0]->bits || P[i]->group != P[0]->group) return GWQ_ERR_UNSUPPORTED;
        if (P[i]->K != P[0]->K) return GWQ_ERR_SHAPE;
    }
    gwq::PlanText plan;
    plan.text[0] = 0;
    hipError_t e;
    if (M <= 16) {
        const void *x[GWQ_MAX_BATCH] = {};
        void *y[GWQ_MAX_BATCH] = {};
        e = gwq::launch_decode(count, P, x, M, y, decode_tuning(), nullptr, &plan);
    } else {
        // the pointer only says whether partial sums may be used; nothing is launched
        e = gwq::launch_gemm(*P[0], nullptr, M, nullptr, nullptr, with_scratch ? &plan : nullptr,
                             with_scratch ? gwq::gemm_scratch_bytes(P[0]->N, M) : 0, g_gemm_ms, nullptr, &plan);
    }
    if (e != hipSuccess) return GWQ_ERR_DEVICE;
    strncpy(text, plan.text, text_bytes - 1);
    text[text_bytes - 1] = 0;
    return GWQ_OK;
}

gwq_status gwq_probe_stream(const void *src, size_t bytes, void *sink, void *stream)
{
    if (!src || !sink) return GWQ_ERR_NULL;
    if (bytes < 16 || bytes % 16 || bytes >= ((size_t)1 << 40) || ((uintptr_t)src & 15) || ((uintptr_t)sink & 3)) return GWQ_ERR_SHAPE;
    return gwq::launch_probe_stream(src, bytes, sink, static_cast<hipStream_t>(stream)) == hipSuccess ? GWQ_OK : GWQ_ERR_DEVICE;
}

gwq_status gwq_probe_mfma(int32_t blocks, int32_t iters, void *sink, void *stream)
{
    if (!sink) return GWQ_ERR_NULL;
    if (blocks < 1 || blocks > (1 << 20) || iters < 1 || ((uintptr_t)sink & 3)) return GWQ_ERR_SHAPE;
    return gwq::launch_probe_mfma(blocks, iters, sink, static_cast<hipStream_t>(stream)) == hipSuccess ? GWQ_OK : GWQ_ERR_DEVICE;
}

gwq_status gwq_tuning_set(const char *key, int32_t value)
{
    if (!key) return GWQ_ERR_NULL;
    if (!strcmp(key, "decode_waves")) {
        if (value < 0 || value > 16) return GWQ_ERR_UNSUPPORTED;
        g_decode_waves = value;
        return GWQ_OK;
    }
    if (!strcmp(key, "decode_stream")) {
        if (value < 0 || value > 2) return GWQ_ERR_UNSUPPORTED;
        g_decode_stream = value;
        return GWQ_OK;
    }
    if (!strcmp(key, "decode_tiles")) {
        if (value < 0 || value > 4096) return GWQ_ERR_UNSUPPORTED;
        g_decode_tiles = value;
        return GWQ_OK;
    }
    if (!strcmp(key, "decode_lean_rows")) {
        if (value < 0 || value > 8) return GWQ_ERR_UNSUPPORTED;
        g_decode_lean = value;
        return GWQ_OK;
    }
    if (!strcmp(key, "decode_pairs")) {
        if (value < 0 || value > 2) return GWQ_ERR_UNSUPPORTED;
        g_decode_pairs = value;
        return GWQ_OK;
    }
    if (!strcmp(key, "pack_full_passes")) {
        if (value < 0 || value > 1) return GWQ_ERR_UNSUPPORTED;
        g_pack_full = value;
        return GWQ_OK;
    }
    if (!strcmp(key, "gemm_rows")) {
        if (value != 0 && value != 32 && value != 64 && value != 128 && value != 256) return GWQ_ERR_UNSUPPORTED;
        g_gemm_ms = value;
        return GWQ_OK;
    }
    return GWQ_ERR_UNSUPPORTED;
}

const char *gwq_status_string(gwq_status status)
{
    switch (status) {
    case GWQ_OK: return "ok";
    case GWQ_ERR_NULL: return "null pointer";
    case GWQ_ERR_SHAPE: return "bad shape, size or alignment";
    case GWQ_ERR_UNSUPPORTED: return "unsupported bits, group, type or option";
    case GWQ_ERR_WORKSPACE: return "workspace missing or too small";
    case GWQ_ERR_DEVICE: return "HIP call failed";
    }
    return "unknown status";
}

const char *gwq_version(void) { return "gwq-gfx950 0.1"; }

}  // extern "C"
