// Internal declarations shared by the HIP translation units of libgwq (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "gwq.h"

namespace gwq {

constexpr int kGroup = 128;        // codes per quantisation group along K
constexpr int kSelBins = 2048;     // bins of one radix-select pass
constexpr int kMaxBatch = GWQ_MAX_BATCH;   // layers per grouped decode launch

__host__ __device__ constexpr int words_per_group(int bits) { return bits == 4 ? 16 : 13; }

// Compute units of the current device, asked once per device (256 on MI355X; 256 if the query fails).
int device_cus();

// Lets `kernel` use up to `bytes` of dynamic LDS on the current device.  `done` is the caller's per-kernel
// record (bit d: done on device d); the HIP call is idempotent, so a race between threads is harmless.
hipError_t allow_dynamic_lds(const void *kernel, int bytes, std::atomic<uint32_t> &done);

// ---- gwq_pack workspace: uint32 words -------------------------------------------------------
// [0, 3*kSelBins)        histograms of the three radix-select passes
// kWsPrefix              key bits fixed by the passes done so far
// kWsRemaining           how many entries are still to be taken among keys matching the prefix
// kWsRows + 0*N ..       per row: count of keys above the threshold
// kWsRows + 1*N ..       per row: count of keys equal to the threshold
// kWsRows + 2*N ..       per row: how many of its threshold ties are kept
// kWsRows + 3*N ..       kSelBins words: histogram of the second digit over the candidates (below)
// then                   per row: number of candidates; then the candidates' keys, [N][pack_candidates_per_row(K)]
// kWsCandOverflow        nonzero when some row had more candidates than its share of the list holds
// Candidates are the keys whose first digit equals the threshold's: after the first pass over the scores only
// they can still decide the threshold, so the second and third digit and the per-row counts are worked out on
// that short list instead of in three more passes over all scores.  Every row has its own part of the list (no
// counter shared between blocks).  When a row's part does not hold its candidates (scores with very many equal or
// nearly equal magnitudes) the full passes run instead; both ways give the same result.
constexpr int kWsPrefix = 3 * kSelBins;
constexpr int kWsRemaining = kWsPrefix + 1;
constexpr int kWsCandOverflow = kWsPrefix + 3;
constexpr int kWsRows = kWsPrefix + 16;

inline int pack_candidates_per_row(int64_t K) { return K / 32 < 32 ? 32 : (int)(K / 32); }
inline size_t pack_workspace_bytes(int64_t N, int64_t K)
{
    return (size_t)(kWsRows + 3 * N + kSelBins + N + N * pack_candidates_per_row(K)) * 4 + 256;
}

// Launchers (defined in the .hip files).  Each enqueues on `stream` and returns the last HIP error.
// full_passes: measurement and test hook - never use the candidate list (always the passes over all scores).
hipError_t launch_pack(const void *W, const void *score, int score_is_f16, const gwq_packed &P,
                       uint32_t *ws, bool full_passes, hipStream_t stream);
// Measurement overrides of the decode launch (0 = built-in choice): waves per block of the kernel for M <= 4;
// streaming kernel 1 = never, 2 = for every M <= 16 it can take; its tiles per block.
struct DecodeTuning {
    int waves, stream, tiles;
    int lean_rows = 0;          // largest M the kernel with X[M][K] in LDS takes (0 = built-in choice, at most 8)
    int pairs = 0;              // that kernel with two tiles per block for 5 <= M <= 8: 0 = built-in choice, 1 = never, 2 = wherever it fits
    bool gated_pairs = false;   // layers (2i, 2i+1) are gate and up of a gated pair: one launch writes silu(gate) * up into Y[2i+1]
    bool bf16 = false;          // X and Y are bfloat16 (groups of 128 only; the kernel for any M <= 16 takes these)
};
// With `describe` set a launcher only writes there which kernel, template arguments and launch shape it
// would use for these arguments, and launches nothing.
struct PlanText {
    char text[192];
};
hipError_t launch_decode(int count, const gwq_packed *const *P, const void *const *X, int M, void *const *Y,
                         const DecodeTuning &tune, hipStream_t stream, PlanText *describe = nullptr);
// index: gemm_index_bytes(N, K, group) bytes, 16-byte aligned (one record per channel and block of 128 codes:
// index of the block's first outlier, scale, zero point; for groups below 128 also a scale / zero-point pair
// per 16 columns; a multiple of 256 bytes).  scratch: gemm_scratch_bytes(N, M_max)
// bytes for the partial sums of launches that also split K (may be NULL: then K is never split).
size_t gemm_index_bytes(int64_t N, int64_t K, int group);
size_t gemm_scratch_bytes(int64_t N, int64_t M_max);
hipError_t launch_gemm_index(const gwq_packed &P, void *index, hipStream_t stream);        // fills the records
hipError_t launch_gemm(const gwq_packed &P, const void *X, int M, void *Y, const void *index, void *scratch,
                       size_t scratch_bytes, int ms_override, hipStream_t stream,
                       PlanText *describe = nullptr, bool bf16 = false);                   // reads them; bf16: X, Y bfloat16

// workspace: quality_workspace_bytes(N) bytes, 8-byte aligned (one partial result per channel); out: 3 doubles.
size_t quality_workspace_bytes(int64_t N);
hipError_t launch_quality(const gwq_packed &P, const void *W, const void *score, int score_is_f16, void *workspace,
                          double *out, hipStream_t stream);

// Measurement probes (gwq_probe.hip): one plain streaming read of `bytes` (a multiple of 16); `blocks` blocks of
// four waves that issue 8 * iters 32x32x16 FP16 MFMAs each out of registers.  sink: 4 bytes, practically never written.
hipError_t launch_probe_stream(const void *src, size_t bytes, void *sink, hipStream_t stream);
hipError_t launch_probe_mfma(int blocks, int iters, void *sink, hipStream_t stream);

// H = silu(G) * U elementwise over `count` FP16 values (the unfused form of the gated pair, for M > 4).
hipError_t launch_silu_mul(const void *G, const void *U, void *H, size_t count, hipStream_t stream);

// score = beta * score + alpha * dY^T X (dY [M][N], X [M][K] FP16; score [N][K] FP32); K a multiple of 128.
hipError_t launch_score(const void *dY, const void *X, int M, int N, int K, float alpha, float beta, float *score,
                        hipStream_t stream);

}  // namespace gwq
