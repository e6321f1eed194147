// gwq_quality on gfx950: the two figures of merit of a packed layer against the weights it was made
// from (Sec. 3.1): the squared error || W - W_Q ||^2 that the quantiser minimises (Eq. 4) and the
// first-order change g^T (W - W_Q) of the loss (Eq. 3 and 5), plus max |W - W_Q|.  W_Q is the decoded
// layer: s * (q - z) (Sec. 3.2, Eq. 10) where a weight was quantised, the stored FP16 value where it
// was kept as an outlier.
//
// One block per output channel.  The codes are read through the format's definition (position of a
// code inside its word), not through the magic-number decoders of the linear kernels, and every
// difference is formed in fp64 from exact operands (an FP16 weight, an FP16 scale times a small
// integer: all multiples of 2^-24 below 2^21), so it is the exact value.  The sums are fp64 and run in
// a fixed order: threads over their strided columns, a shuffle tree, the block's waves in order, and a
// second kernel over the channels; no floating-point atomics, results identical from run to run.
// Bound by HBM: W (2 bytes), the score (4 or 2) and the packed layer (about 0.5) per weight, read once.
#include "gwq_internal.h"

namespace gwq {
namespace {

constexpr int kQThreads = 256;

struct Merit {
    double sq, first, mx;
};

__device__ inline void merit_add(Merit &a, const Merit &b)
{
    a.sq += b.sq;
    a.first += b.first;
    a.mx = a.mx > b.mx ? a.mx : b.mx;
}

__device__ inline Merit merit_shuffle_down(const Merit &m, int delta)
{
    return Merit{__shfl_down(m.sq, delta), __shfl_down(m.first, delta), __shfl_down(m.mx, delta)};
}

// Fixed-order sum over the block: lanes by a shuffle tree, then the waves in order.  Valid in thread 0.
__device__ inline Merit block_sum(Merit m, Merit *wave_part)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) merit_add(m, merit_shuffle_down(m, d));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) wave_part[wave] = m;
    __syncthreads();
    if (threadIdx.x == 0)
        for (int w = 1; w < kQThreads / 64; ++w) merit_add(m, wave_part[w]);
    return m;
}

// What a thread fetches for eight consecutive columns k0 .. k0 + 7 of its channel: the weights, the
// scores, the group's scale and zero point, and the words that hold the eight codes - one word at 4
// bits; at 3 bits the slot's three words and the group's tail word.
template <int BITS, bool F16> struct Chunk {
    uint4 w;
    uint4 g[F16 ? 1 : 2];
    uint32_t code[BITS == 4 ? 1 : 4];
    uint16_t scale;
    uint8_t zero;
};

// Code t (0..7) of a chunk that starts at position c0 (a multiple of 8) of its 32-code slot `slot`,
// from the layout of the packed format: even positions in the low half of a word, odd ones in the
// high half, `bits` bits apiece, ascending; 3-bit words hold ten codes and codes 30 and 31 of a slot
// sit in the tail word at bits 3*slot and 16 + 3*slot.
template <int BITS> __device__ inline int code_of(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t tail, int slot, int c0, int t)
{
    if (BITS == 4) return (int)((w0 >> (16 * (t & 1) + 4 * (t >> 1))) & 15u);
    const int c = c0 + t;
    if (c >= 30) return (int)((tail >> (16 * (c & 1) + 3 * slot)) & 7u);
    const uint32_t word = c < 10 ? w0 : c < 20 ? w1 : w2;
    const int p = c < 10 ? c : c < 20 ? c - 10 : c - 20;
    return (int)((word >> (16 * (p & 1) + 3 * (p >> 1))) & 7u);
}

template <int BITS, bool F16>
__global__ __launch_bounds__(kQThreads) void quality_kernel(const uint32_t *__restrict__ qweight,
                                                            const uint16_t *__restrict__ scales,
                                                            const uint8_t *__restrict__ zeros,
                                                            const int32_t *__restrict__ row_ptr,
                                                            const uint16_t *__restrict__ col_idx,
                                                            const uint16_t *__restrict__ out_val,
                                                            const _Float16 *__restrict__ W, const void *__restrict__ score,
                                                            int K, int group, Merit *__restrict__ partial)
{
    __shared__ uint32_t kept[65536 / 32];               // one bit per column: kept as an outlier
    __shared__ Merit wave_part[kQThreads / 64];
    const int n = blockIdx.x, tid = threadIdx.x;
    const int gpr = K / kGroup, spr = K / group;        // blocks of 128 codes and scale groups per row
    const size_t row = (size_t)n * K;
    Merit m{0.0, 0.0, 0.0};

    // Requests for the chunk at k0 (clamped to the row: a chunk past its end is fetched again and not used).
    auto fetch = [&](int k0, Chunk<BITS, F16> &c) {
        k0 = k0 < K ? k0 : K - 8;
        const int g = k0 / kGroup, slot = (k0 % kGroup) >> 5, j8 = (k0 & 31) >> 3;
        const uint32_t *words = qweight + ((size_t)n * gpr + g) * words_per_group(BITS);
        c.w = *reinterpret_cast<const uint4 *>(W + row + k0);
        if (F16) {
            c.g[0] = *reinterpret_cast<const uint4 *>(static_cast<const _Float16 *>(score) + row + k0);
        } else {
            c.g[0] = *reinterpret_cast<const uint4 *>(static_cast<const float *>(score) + row + k0);
            c.g[F16 ? 0 : 1] = *reinterpret_cast<const uint4 *>(static_cast<const float *>(score) + row + k0 + 4);
        }
        if (BITS == 4) {
            c.code[0] = words[4 * slot + j8];
        } else {
            c.code[0] = words[3 * slot]; c.code[BITS == 4 ? 0 : 1] = words[3 * slot + 1]; c.code[BITS == 4 ? 0 : 2] = words[3 * slot + 2];
            c.code[BITS == 4 ? 0 : 3] = words[12];
        }
        c.scale = scales[(size_t)n * spr + k0 / group];
        c.zero = zeros[(size_t)n * spr + k0 / group];
    };
    auto consume = [&](int k0, const Chunk<BITS, F16> &c) {
        if (k0 >= K) return;
        const int slot = (k0 % kGroup) >> 5, c0 = k0 & 31;
        const double s = (double)(float)__builtin_bit_cast(_Float16, c.scale);
        const int z = c.zero;
        const uint32_t w2[4] = {c.w.x, c.w.y, c.w.z, c.w.w};
        uint32_t g4[8];
        g4[0] = c.g[0].x; g4[1] = c.g[0].y; g4[2] = c.g[0].z; g4[3] = c.g[0].w;
        if (!F16) { g4[4] = c.g[F16 ? 0 : 1].x; g4[5] = c.g[F16 ? 0 : 1].y; g4[6] = c.g[F16 ? 0 : 1].z; g4[7] = c.g[F16 ? 0 : 1].w; }
        const uint32_t kept8 = (kept[k0 >> 5] >> (k0 & 31)) & 0xFFu;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (kept8 >> t & 1) continue;
            const double w = (double)(float)__builtin_bit_cast(_Float16, (uint16_t)(w2[t >> 1] >> (16 * (t & 1))));
            const double g = F16 ? (double)(float)__builtin_bit_cast(_Float16, (uint16_t)(g4[t >> 1] >> (16 * (t & 1))))
                                 : (double)__builtin_bit_cast(float, g4[t]);
            const double d = w - s * (double)(code_of<BITS>(c.code[0], c.code[BITS == 4 ? 0 : 1], c.code[BITS == 4 ? 0 : 2],
                                                           c.code[BITS == 4 ? 0 : 3], slot, c0, t) - z);
            m.sq += d * d;
            m.first += g * d;
            m.mx = m.mx > fabs(d) ? m.mx : fabs(d);
        }
    };

    // The first two chunks are on their way while the channel's outliers are looked at.
    constexpr int kStride = 8 * kQThreads;
    Chunk<BITS, F16> a, b;
    fetch(8 * tid, a);
    fetch(8 * tid + kStride, b);

    for (int i = tid; i < K / 32; i += kQThreads) kept[i] = 0u;
    __syncthreads();
    // The channel's outliers: mark their columns and take their own difference (zero when the stored
    // value is the weight's copy, as gwq_pack writes it).
    for (int j = row_ptr[n] + tid; j < row_ptr[n + 1]; j += kQThreads) {
        const int c = col_idx[j];
        atomicOr(&kept[c >> 5], 1u << (c & 31));
        const double d = (double)(float)W[row + c] - (double)(float)__builtin_bit_cast(_Float16, out_val[j]);
        const double g = F16 ? (double)(float)static_cast<const _Float16 *>(score)[row + c]
                             : (double)static_cast<const float *>(score)[row + c];
        m.sq += d * d;
        m.first += g * d;
        m.mx = m.mx > fabs(d) ? m.mx : fabs(d);
    }
    __syncthreads();
    // Everything else, eight consecutive columns per thread and chunk, two chunks in flight.
    for (int k0 = 8 * tid; k0 < K; k0 += 2 * kStride) {
        consume(k0, a);
        fetch(k0 + 2 * kStride, a);
        consume(k0 + kStride, b);
        fetch(k0 + 3 * kStride, b);
    }
    m = block_sum(m, wave_part);
    if (tid == 0) partial[n] = m;
}

// out[0..2] = the channels' partial results added in the order of n: thread t takes channels
// t, t + 256, ..., then the block's fixed-order sum.
__global__ __launch_bounds__(kQThreads) void quality_reduce_kernel(const Merit *__restrict__ partial, int N,
                                                                   double *__restrict__ out)
{
    __shared__ Merit wave_part[kQThreads / 64];
    Merit m{0.0, 0.0, 0.0};
    // Eight channels' partial results requested at a time (the additions keep their order).
    int n = threadIdx.x;
    for (; n + 7 * kQThreads < N; n += 8 * kQThreads) {
        Merit p[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) p[i] = partial[n + i * kQThreads];
#pragma unroll
        for (int i = 0; i < 8; ++i) merit_add(m, p[i]);
    }
    for (; n < N; n += kQThreads) merit_add(m, partial[n]);
    m = block_sum(m, wave_part);
    if (threadIdx.x == 0) {
        out[0] = m.sq;
        out[1] = m.first;
        out[2] = m.mx;
    }
}

}  // namespace

size_t quality_workspace_bytes(int64_t N) { return (size_t)N * sizeof(Merit); }

hipError_t launch_quality(const gwq_packed &P, const void *W, const void *score, int score_is_f16, void *workspace,
                          double *out, hipStream_t st)
{
    Merit *partial = static_cast<Merit *>(workspace);
    const _Float16 *w = static_cast<const _Float16 *>(W);
#define GWQ_QUALITY(B, F) \
    quality_kernel<B, F><<<P.N, kQThreads, 0, st>>>(P.qweight, P.scales, P.zeros, P.row_ptr, P.col_idx, P.out_val, w, \
                                                    score, P.K, P.group, partial)
    if (P.bits == 4) {
        if (score_is_f16) GWQ_QUALITY(4, true); else GWQ_QUALITY(4, false);
    } else {
        if (score_is_f16) GWQ_QUALITY(3, true); else GWQ_QUALITY(3, false);
    }
#undef GWQ_QUALITY
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    quality_reduce_kernel<<<1, kQThreads, 0, st>>>(partial, P.N, out);
    return hipGetLastError();
}

}  // namespace gwq
