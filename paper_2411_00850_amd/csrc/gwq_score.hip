// gwq_score on gfx950: the score that gwq_pack ranks, produced on the device for one linear layer.
// The score is the gradient of the loss with respect to the weights (Sec. 3.1, Eq. 2); for Y = X W^T
// without bias the chain rule gives, from the gradient dY of the loss with respect to Y,
//   g[n][k] = sum_m dY[m][n] * X[m][k]
// and the entry point writes score = beta * score + alpha * g, so that the mean over calibration
// samples (Sec. 4.3, ablation on the number of calibration samples) is a sequence of calls with alpha = 1 / samples.
//
// A dense contraction over the samples m with both operands stored m-major, bound by MFMA.  A block of
// four waves owns a 128 (n) x 128 (k) tile of the score and walks m in steps of 64; a wave owns 64 x 64
// of it as 2 x 2 tiles of v_mfma_f32_32x32x16_f16 (FP32 accumulators, exact FP16 products).  The MFMA
// wants, per lane, eight consecutive m of one n (or k), while memory has eight consecutive n of one m:
// a thread loads 16 bytes of four consecutive rows m, regroups them in registers into eight 8-byte
// pieces "four m of one n" and stores those, so the LDS copy is transposed, [n][m] and [k][m], 128
// bytes per row, and fragment reads are plain 16-byte reads.  The eight 16-byte units of a row are
// XOR-permuted by row so that both the fragment reads (16 consecutive rows x one unit) and the
// transposing stores (rows 8 apart) are free of bank conflicts.  Two LDS buffers, one block barrier
// per step; global loads run a step ahead in two register sets; the stores of the next step are
// spread behind the MFMA batches of the current one.
#include <type_traits>

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

// 16-byte unit c of row `row` of a tile in LDS (rows of 128 bytes: two rows span the 64 banks).  The XOR
// term has bit 0 = row bit 3 and bits 2..1 = row bits 2..1 ^ row bits 5..4: the 16 consecutive rows of a
// fragment read meet 16 different (row parity, unit) pairs, and so do the 16 rows, 8 apart and of both
// parities, that the lanes of a transposing store write.
__device__ inline int unit_of(int row, int c)
{
    return row * 8 + (c ^ (((((row >> 1) ^ (row >> 4)) & 3) << 1) | ((row >> 3) & 1)));
}

struct RowSet {
    uint4 a[4], b[4];             // 8 halves of dY and of X from four consecutive rows m
};

template <bool N8>
__global__ __launch_bounds__(kScoreThreads, N8 ? 2 : 1) void score_kernel(const _Float16 *__restrict__ dY,
                                                              const _Float16 *__restrict__ X, int M, int N, int K,
                                                              int tiles_n, int tiles_k, float alpha, float beta,
                                                              float *__restrict__ score)
{
    extern __shared__ uint4 lds[];                      // [buffer][operand][unit]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Workgroups go round-robin to the 8 XCDs, each with an L2 of its own: XCD x takes the x-th eighth of
    // the tiles, in an order that walks k inside bands of 8 tile rows, so that the blocks an XCD runs at
    // one time form a patch of about 8 x 8 tiles and share their operands' tiles in its L2.
    const int per_xcd = (tiles_n * tiles_k + 7) >> 3;
    const int lin = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (lin >= tiles_n * tiles_k) return;               // whole block, before any barrier
    const int band = lin / (8 * tiles_k), in_band = lin - band * 8 * tiles_k;
    const int band_rows = tiles_n - 8 * band < 8 ? tiles_n - 8 * band : 8;
    const int n0 = (8 * band + in_band % band_rows) * kTile, k0 = (in_band / band_rows) * kTile;
    // Staging: a thread takes columns 8 * chunk .. + 7 of rows 4 * quad .. + 3.  Lanes 16 apart and lanes 32
    // apart both differ in the 8-byte half of a unit they store to, and a lane with chunk >= 8 stores the
    // odd column while the others store the even one: whichever lanes the LDS serves together, their
    // stores fall into different banks.
    const int chunk = lane & 15, quad = 4 * wave + 2 * (lane >> 5) + (((lane >> 4) ^ (lane >> 5)) & 1);
    const int flip = chunk >> 3;
    const int wn = wave >> 1, wk = wave & 1;
    const int steps = (M + kStepM - 1) / kStepM;

    // Requests for step t.  Rows beyond M and columns beyond N read a valid address.  Columns beyond N
    // only reach rows of the tile that are never stored; rows beyond M are zeroed in X when the set is
    // staged (touching a loaded value here would wait for it here), which makes their products zero.
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
    // columns the four rows' halves as one 8-byte piece at [column][4 * quad .. + 3].  Done in four parts
    // (columns 2 * part and 2 * part + 1 of both operands), one behind each batch of MFMAs, whose shadow
    // hides them.
    auto stage_part = [&](int buf, int t, const RowSet &r, int part) {
        char *a_base = reinterpret_cast<char *>(lds + (size_t)(2 * buf) * kUnitsPerBuf);
        char *b_base = reinterpret_cast<char *>(lds + (size_t)(2 * buf + 1) * kUnitsPerBuf);
        const int m = t * kStepM + 4 * quad;
        const uint32_t rows01 = (m < M ? 0xFFFFu : 0u) | (m + 1 < M ? 0xFFFF0000u : 0u);
        const uint32_t rows23 = (m + 2 < M ? 0xFFFFu : 0u) | (m + 3 < M ? 0xFFFF0000u : 0u);
        auto put = [&](char *base, const uint4 *v, uint32_t mask01, uint32_t mask23) {
            const uint32_t w[4][4] = {{v[0].x, v[0].y, v[0].z, v[0].w}, {v[1].x, v[1].y, v[1].z, v[1].w},
                                      {v[2].x, v[2].y, v[2].z, v[2].w}, {v[3].x, v[3].y, v[3].z, v[3].w}};
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int j = 2 * part + jj;            // column j ^ flip: the same word of the loaded 16 bytes
                const uint32_t sel = ((j & 1) ^ flip) ? 0x07060302u : 0x05040100u;   // the same half of two words
                uint2 piece;
                piece.x = __builtin_amdgcn_perm(w[1][j >> 1], w[0][j >> 1], sel) & mask01;
                piece.y = __builtin_amdgcn_perm(w[3][j >> 1], w[2][j >> 1], sel) & mask23;
                const int row = 8 * chunk + (j ^ flip);
                *reinterpret_cast<uint2 *>(base + (size_t)unit_of(row, quad >> 1) * 16 + 8 * (quad & 1)) = piece;
            }
        };
        put(a_base, r.a, 0xFFFFFFFFu, 0xFFFFFFFFu);
        put(b_base, r.b, rows01, rows23);
    };

    float16v acc[2][2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[s][t][v] = 0.f;

    // One step: the MFMAs of buffer `buf` and the staging of step `next`, held in `r`, into the other
    // buffer.  Behind the last step this stages a repeat of it that nobody reads: no branch.
    auto step = [&](int buf, int next, const RowSet &r) {
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
            stage_part(buf ^ 1, next, r, kb);
        }
    };

    // Set (t & 1) holds step t until it is staged.  Requests past the last step repeat the last one
    // (in bounds): no load sits inside a branch, so none is waited for early.
    RowSet set0, set1;
    const int last = steps - 1;
    fetch(0, set0);
    fetch(last < 1 ? last : 1, set1);
#pragma unroll
    for (int part = 0; part < 4; ++part) stage_part(0, 0, set0, part);
    fetch(last < 2 ? last : 2, set0);
    __syncthreads();
    for (int t = 0; t < steps; t += 2) {
        step(0, t + 1, set1);
        fetch(last < t + 3 ? last : t + 3, set1);
        __syncthreads();
        if (t + 1 >= steps) break;
        step(1, t + 2, set0);
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
    static std::atomic<uint32_t> lds_allowed[2];        // per kernel
    {
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&score_kernel<true>), (int)kScoreLds, lds_allowed[0]);
        if (e == hipSuccess)
            e = allow_dynamic_lds(reinterpret_cast<const void *>(&score_kernel<false>), (int)kScoreLds, lds_allowed[1]);
        if (e != hipSuccess) return e;
    }
    const _Float16 *d = static_cast<const _Float16 *>(dY), *x = static_cast<const _Float16 *>(X);
    const int blocks = (tiles_n * tiles_k + 7) / 8 * 8;
    if (N % 8 == 0)
        score_kernel<true><<<blocks, kScoreThreads, kScoreLds, st>>>(d, x, M, N, K, tiles_n, tiles_k, alpha, beta, score);
    else
        score_kernel<false><<<blocks, kScoreThreads, kScoreLds, st>>>(d, x, M, N, K, tiles_n, tiles_k, alpha, beta, score);
    return hipGetLastError();
}

}  // namespace gwq
