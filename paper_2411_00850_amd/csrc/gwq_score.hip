// gwq_score on gfx950: the score that gwq_pack ranks, produced on the device for one linear layer.
// The score is the gradient of the loss with respect to the weights (Sec. 3.1, Eq. 2); for Y = X W^T
// without bias the chain rule gives, from the gradient dY of the loss with respect to Y,
//   g[n][k] = sum_m dY[m][n] * X[m][k]
// and the entry point writes score = beta * score + alpha * g, so that the mean over calibration
// samples (Sec. 4.4) is a sequence of calls with alpha = 1 / samples.
//
// A dense contraction over the samples m with both operands stored m-major, bound by MFMA.  A block of
// four waves owns a 128 (n) x 128 (k) tile of the score and walks m in steps of 64; a wave owns 64 x 64
// of it as 2 x 2 tiles of v_mfma_f32_32x32x16_f16 (FP32 accumulators, exact FP16 products).  The MFMA
// wants, per lane, eight consecutive m of one n (or k), while memory has eight consecutive n of one m:
// a thread loads 16 bytes of four consecutive rows m, regroups them in registers into eight 8-byte
// pieces "four m of one n" and stores those, so the LDS copy is transposed, [n][m] and [k][m], 128
// bytes per row, and fragment reads are plain 16-byte reads.  The eight 16-byte units of a row are
// XOR-permuted by (row + row / 8) mod 8: fragment reads (32 rows x one unit) are free of bank
// conflicts, the transposing stores (16 rows 8 apart x 4 pieces) two-way.  Two LDS buffers, one block
// barrier per step; global loads run two steps ahead in two register sets.
#include "gwq_internal.h"

namespace gwq {
namespace {

typedef _Float16 half8s __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kTile = 128;         // tile edge along n and along k
constexpr int kStepM = 64;         // samples per step
constexpr int kScoreThreads = 256;
constexpr int kUnitsPerBuf = kTile * 8;                 // 16-byte units of one operand's tile (128 rows x 64 halves)
constexpr size_t kScoreLds = (size_t)2 * 2 * kUnitsPerBuf * 16;   // two buffers x two operands = 64 KB

__device__ inline int unit_of(int row, int c) { return row * 8 + (c ^ ((row + (row >> 3)) & 7)); }

struct RowSet {
    uint4 a[4], b[4];             // 8 halves of dY and of X from four consecutive rows m
};

template <bool N8>
__global__ __launch_bounds__(kScoreThreads, N8 ? 2 : 1) void score_kernel(const _Float16 *__restrict__ dY,
                                                              const _Float16 *__restrict__ X, int M, int N, int K,
                                                              int tiles_k, float alpha, float beta,
                                                              float *__restrict__ score)
{
    extern __shared__ uint4 lds[];                      // [buffer][operand][unit]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = (blockIdx.x / tiles_k) * kTile, k0 = (blockIdx.x % tiles_k) * kTile;
    const int chunk = tid & 15, quad = tid >> 4;        // staging: columns 8 * chunk .. + 7 of rows 4 * quad .. + 3
    const int wn = wave >> 1, wk = wave & 1;
    const int steps = (M + kStepM - 1) / kStepM;

    // Requests for step t.  Rows beyond M and columns beyond N read a valid address; what they return is
    // masked off when the set is staged (touching a loaded value here would wait for it here).
    auto fetch = [&](int t, RowSet &r) {
        const int nn = n0 + 8 * chunk, kk = k0 + 8 * chunk;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = t * kStepM + 4 * quad + i;
            const size_t mrow = m < M ? m : 0;
            r.b[i] = *reinterpret_cast<const uint4 *>(X + mrow * K + kk);
            if (N8) {                                   // N is a multiple of 8: a chunk is inside or outside
                r.a[i] = *reinterpret_cast<const uint4 *>(dY + mrow * N + (nn < N ? nn : 0));
            } else {                                    // rows of dY are not 16-byte aligned: element by element
                uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    w[j >> 1] |= (uint32_t)__builtin_bit_cast(uint16_t, dY[mrow * N + (nn + j < N ? nn + j : 0)]) << (16 * (j & 1));
                r.a[i] = uint4{w[0], w[1], w[2], w[3]};
            }
        }
    };
    // Transposing store of the register set of step t into buffer `buf`: for each of the thread's eight
    // columns the four rows' halves as one 8-byte piece at [column][4 * quad .. + 3].
    auto stage = [&](int buf, int t, const RowSet &r) {
        char *a_base = reinterpret_cast<char *>(lds + (size_t)(2 * buf) * kUnitsPerBuf);
        char *b_base = reinterpret_cast<char *>(lds + (size_t)(2 * buf + 1) * kUnitsPerBuf);
        const int m = t * kStepM + 4 * quad;
        const uint32_t rows01 = (m < M ? 0xFFFFu : 0u) | (m + 1 < M ? 0xFFFF0000u : 0u);
        const uint32_t rows23 = (m + 2 < M ? 0xFFFFu : 0u) | (m + 3 < M ? 0xFFFF0000u : 0u);
        auto put = [&](char *base, const uint4 *v, int cols_left) {
            const uint32_t w[4][4] = {{v[0].x, v[0].y, v[0].z, v[0].w}, {v[1].x, v[1].y, v[1].z, v[1].w},
                                      {v[2].x, v[2].y, v[2].z, v[2].w}, {v[3].x, v[3].y, v[3].z, v[3].w}};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;   // the same half of two words
                const uint32_t col = j < cols_left ? 0xFFFFFFFFu : 0u;
                uint2 piece;
                piece.x = __builtin_amdgcn_perm(w[1][j >> 1], w[0][j >> 1], sel) & rows01 & col;
                piece.y = __builtin_amdgcn_perm(w[3][j >> 1], w[2][j >> 1], sel) & rows23 & col;
                const int row = 8 * chunk + j;
                *reinterpret_cast<uint2 *>(base + (size_t)unit_of(row, quad >> 1) * 16 + 8 * (quad & 1)) = piece;
            }
        };
        put(a_base, r.a, N - (n0 + 8 * chunk));
        put(b_base, r.b, 8);
    };

    float16v acc[2][2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[s][t][v] = 0.f;

    auto multiply = [&](int buf) {
        const uint4 *a_base = lds + (size_t)(2 * buf) * kUnitsPerBuf;
        const uint4 *b_base = lds + (size_t)(2 * buf + 1) * kUnitsPerBuf;
#pragma unroll
        for (int kb = 0; kb < kStepM / 16; ++kb) {
            const int c = 2 * kb + (lane >> 5);         // the lane's eight samples: 16 * kb + 8 * (lane / 32) ..
            uint4 fa[2], fb[2];
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                fa[s] = a_base[unit_of(wn * 64 + s * 32 + (lane & 31), c)];
                fb[s] = b_base[unit_of(wk * 64 + s * 32 + (lane & 31), c)];
            }
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    acc[s][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8s, fa[s]),
                                                                       __builtin_bit_cast(half8s, fb[t]), acc[s][t], 0, 0, 0);
        }
    };

    // Set (t & 1) holds step t until it is staged.  Requests past the last step repeat the last one
    // (in bounds, never staged): no load sits inside a branch, so none is waited for early.
    RowSet set0, set1;
    const int last = steps - 1;
    fetch(0, set0);
    fetch(last < 1 ? last : 1, set1);
    stage(0, 0, set0);
    fetch(last < 2 ? last : 2, set0);
    __syncthreads();
    for (int t = 0; t < steps; t += 2) {
        multiply(0);
        if (t + 1 < steps) stage(1, t + 1, set1);
        fetch(last < t + 3 ? last : t + 3, set1);
        __syncthreads();
        if (t + 1 >= steps) break;
        multiply(1);
        if (t + 2 < steps) stage(0, t + 2, set0);
        fetch(last < t + 4 ? last : t + 4, set0);
        __syncthreads();
    }

    // D layout of a 32x32 tile: column (k) = lane % 32, row (n) = 8 * (v / 4) + 4 * (lane / 32) + v % 4.
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int k = k0 + wk * 64 + t * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int n = n0 + wn * 64 + s * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (n < N) {
                    float *p = score + (size_t)n * K + k;
                    float g = alpha * acc[s][t][v];
                    if (beta != 0.f) g += beta * *p;
                    *p = g;
                }
            }
        }
}

}  // namespace

hipError_t launch_score(const void *dY, const void *X, int M, int N, int K, float alpha, float beta, float *score,
                        hipStream_t st)
{
    const int tiles_k = K / kTile, tiles_n = (N + kTile - 1) / kTile;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&score_kernel<true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kScoreLds);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&score_kernel<false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kScoreLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const _Float16 *d = static_cast<const _Float16 *>(dY), *x = static_cast<const _Float16 *>(X);
    if (N % 8 == 0)
        score_kernel<true><<<tiles_n * tiles_k, kScoreThreads, kScoreLds, st>>>(d, x, M, N, K, tiles_k, alpha, beta, score);
    else
        score_kernel<false><<<tiles_n * tiles_k, kScoreThreads, kScoreLds, st>>>(d, x, M, N, K, tiles_k, alpha, beta, score);
    return hipGetLastError();
}

}  // namespace gwq
