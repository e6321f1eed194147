// gwq_pack on gfx950: outlier selection (Sec. 3.2, Eq. 8) as a three-pass (FP16 scores: two-pass) radix select over the
// bit patterns of |score|, CSR build in flat-index order, then per (row, group of 16 to 128) the scale,
// zero point and codes of Eq. 6, 7 and 9 and the word layout documented in gwq.h.
//
// Everything is integer work or exactly specified IEEE arithmetic (fp64 division, round half to
// even), so the output is a function of the inputs alone.  Integer atomics are used for the
// histograms (order-independent); there are no floating-point atomics.
#include "gwq_internal.h"

#pragma clang fp contract(off)

namespace gwq {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kElemsPerThread = 8;
constexpr int kElemsPerIter = kThreads * kElemsPerThread;   // 2048 = 16 groups

// Ranking key: bit pattern of |score| as binary32 (monotone in the magnitude, NaN on top).
__device__ inline uint32_t key_from_f32(uint32_t bits) { return bits & 0x7FFFFFFFu; }

__device__ inline uint32_t key_from_f16(uint16_t h)
{
    const uint32_t e = (h >> 10) & 0x1F, f = h & 0x3FF;
    if (e == 31) return 0x7F800000u | (f << 13);                 // inf / NaN keep their payload
    const float v = (float)__builtin_bit_cast(_Float16, (uint16_t)(h & 0x7FFF));  // exact widening
    return __builtin_bit_cast(uint32_t, v);
}

// Digit of a key in pass 0, 1, 2 (11 + 11 + 9 bits of the 31-bit key) and the bits above it.
template <int PASS> __device__ inline uint32_t digit_of(uint32_t key)
{
    return PASS == 0 ? key >> 20 : PASS == 1 ? (key >> 9) & 0x7FFu : key & 0x1FFu;
}
template <int PASS> __device__ inline bool prefix_matches(uint32_t key, uint32_t prefix)
{
    return PASS == 0 ? true : PASS == 1 ? (key >> 20) == (prefix >> 20) : (key >> 9) == (prefix >> 9);
}

template <bool F16> __device__ inline void load_keys8(const void *score, size_t idx, uint32_t key[8])
{
    if (F16) {
        const uint4 v = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(score) + idx);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            key[2 * i] = key_from_f16((uint16_t)(w[i] & 0xFFFF));
            key[2 * i + 1] = key_from_f16((uint16_t)(w[i] >> 16));
        }
    } else {
        const uint4 *p = reinterpret_cast<const uint4 *>(static_cast<const uint32_t *>(score) + idx);
        const uint4 a = p[0], b = p[1];
        key[0] = key_from_f32(a.x); key[1] = key_from_f32(a.y);
        key[2] = key_from_f32(a.z); key[3] = key_from_f32(a.w);
        key[4] = key_from_f32(b.x); key[5] = key_from_f32(b.y);
        key[6] = key_from_f32(b.z); key[7] = key_from_f32(b.w);
    }
}

__global__ void init_ws_kernel(uint32_t *ws, uint32_t k_out, int N)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < kWsRows; i += gridDim.x * blockDim.x)
        ws[i] = 0;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < kSelBins; i += gridDim.x * blockDim.x)
        ws[kWsRows + 3 * N + i] = 0;                    // the candidates' histogram
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        // With nothing to select the threshold sits above every key, so no entry qualifies.
        ws[kWsPrefix] = k_out ? 0u : 0xFFFFFFFFu;
        ws[kWsRemaining] = k_out;
    }
}

// One radix-select pass: histogram of this pass's digit over the keys that match the prefix.
// `total` is a multiple of 8 (K is a multiple of 128).  The grid is kept small (two blocks per CU):
// every block flushes its non-empty bins with global atomics, in the first pass a few hundred bins
// per block and all blocks on the same addresses, which with 2048 blocks took longer than the pass
// over the keys.
// Which way a launch belongs to: both ways are enqueued (the choice is made on the device, by the pass that
// collects the candidates) and the kernels of the way not taken return at once.
enum When { kAlways = 0, kWithCandidates = 1, kWithoutCandidates = 2 };
__device__ inline bool not_my_turn(const uint32_t *ws, int when)
{
    const bool overflow = ws[kWsCandOverflow] != 0;
    return (when == kWithCandidates && overflow) || (when == kWithoutCandidates && !overflow);
}

// With candidates (PASS 2 only, per_row > 0): when the candidates fitted, the third digit is counted over them instead
// (one wave per row of the list, global atomics: they are few), and the scores are not read.
template <int PASS, bool F16>
__global__ __launch_bounds__(kThreads) void hist_kernel(const void *score, size_t total, uint32_t *ws, int when, int N = 0,
                                                        int per_row = 0)
{
    if (PASS == 2 && per_row > 0 && ws[kWsCandOverflow] == 0) {
        const uint32_t prefix = ws[kWsPrefix];
        const uint32_t *counts = ws + kWsRows + 3 * N + kSelBins, *keys = counts + N;
        const int lane = threadIdx.x & 63;
        for (int n = blockIdx.x * kWaves + (threadIdx.x >> 6); n < N; n += gridDim.x * kWaves) {
            const uint32_t count = counts[n];
            for (uint32_t i = lane; i < count; i += 64) {
                const uint32_t key = keys[(size_t)n * per_row + i];
                if (prefix_matches<2>(key, prefix)) atomicAdd(&ws[2 * kSelBins + digit_of<2>(key)], 1u);
            }
        }
        return;
    }
    if (not_my_turn(ws, when)) return;
    __shared__ uint32_t h[kSelBins];
    for (int i = threadIdx.x; i < kSelBins; i += kThreads) h[i] = 0;
    __syncthreads();
    const uint32_t prefix = ws[kWsPrefix];
    const size_t stride = (size_t)gridDim.x * kThreads * 8;
    for (size_t idx = ((size_t)blockIdx.x * kThreads + threadIdx.x) * 8; idx < total; idx += stride) {
        uint32_t key[8];
        load_keys8<F16>(score, idx, key);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (prefix_matches<PASS>(key[i], prefix)) atomicAdd(&h[digit_of<PASS>(key[i])], 1u);
    }
    __syncthreads();
    uint32_t *g = ws + PASS * kSelBins;
    for (int i = threadIdx.x; i < kSelBins; i += kThreads)
        if (h[i]) atomicAdd(&g[i], h[i]);
}

// Pick the digit d of this pass: (#keys with digit > d) < remaining <= (#keys with digit >= d).
// One block of kSelBins / 2 threads; suffix sums by a doubling scan in LDS.
// hist: word offset of the histogram in ws; hist_candidates (when not negative): the one to read instead when the
// candidates fitted.
template <int PASS> __global__ __launch_bounds__(kSelBins / 2) void pick_kernel(uint32_t *ws, int hist, int hist_candidates)
{
    __shared__ uint32_t a[2][kSelBins + 1];
    const uint32_t *g = ws + (hist_candidates >= 0 && ws[kWsCandOverflow] == 0 ? hist_candidates : hist);
    const int t = threadIdx.x;
    a[0][t] = g[t];
    a[0][t + kSelBins / 2] = g[t + kSelBins / 2];
    __syncthreads();
    int cur = 0;
    for (int d = 1; d < kSelBins; d <<= 1) {           // a[cur][i] becomes sum of bins i .. end
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int i = t + r * (kSelBins / 2);
            a[cur ^ 1][i] = a[cur][i] + (i + d < kSelBins ? a[cur][i + d] : 0u);
        }
        __syncthreads();
        cur ^= 1;
    }
    const uint32_t remaining = ws[kWsRemaining];
    const uint32_t prefix = ws[kWsPrefix];
    __syncthreads();
    if (remaining == 0) return;
    constexpr int shift = PASS == 0 ? 20 : PASS == 1 ? 9 : 0;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int i = t + r * (kSelBins / 2);
        const uint32_t ge = a[cur][i];
        const uint32_t gt = i + 1 < kSelBins ? a[cur][i + 1] : 0u;
        if (gt < remaining && remaining <= ge) {       // true for exactly one bin
            ws[kWsPrefix] = prefix | ((uint32_t)i << shift);
            ws[kWsRemaining] = remaining - gt;
        }
    }
}

__device__ inline uint32_t wave_inclusive_scan(uint32_t v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(v, d);
        if (lane >= d) v += t;
    }
    return v;
}

// Exclusive scan of one value per thread over the block, plus the block total.
__device__ inline uint32_t block_exclusive_scan(uint32_t v, uint32_t *smem, uint32_t &total)
{
    const uint32_t inc = wave_inclusive_scan(v);
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 63) smem[w] = inc;
    __syncthreads();
    uint32_t base = 0, sum = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) {
        const uint32_t s = smem[i];
        if (i < w) base += s;
        sum += s;
    }
    total = sum;
    return base + inc - v;
}

// Per row: how many keys are above the threshold and how many are equal to it.
// With candidates (per_row > 0) and when they fitted: only the row's candidates are looked at - the keys with a larger
// first digit are counted already (candidates_kernel) - and the scores are not read.
template <bool F16>
__global__ __launch_bounds__(kThreads) void row_count_kernel(const void *score, int K, uint32_t *ws, int N, int per_row)
{
    __shared__ uint32_t red[2][kWaves];
    const int n = blockIdx.x;
    const uint32_t thr = ws[kWsPrefix];
    if (per_row > 0 && ws[kWsCandOverflow] == 0) {
        if (threadIdx.x >= 64) return;                  // a row's candidates are few: one wave
        const uint32_t *counts = ws + kWsRows + 3 * N + kSelBins, *keys = counts + N + (size_t)n * per_row;
        const uint32_t count = counts[n];
        uint32_t gt = 0, eq = 0;
        for (uint32_t i = threadIdx.x; i < count; i += 64) {
            const uint32_t key = keys[i];
            gt += key > thr;
            eq += key == thr;
        }
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) { gt += __shfl_xor(gt, d); eq += __shfl_xor(eq, d); }
        if (threadIdx.x == 0) { ws[kWsRows + n] += gt; ws[kWsRows + N + n] = eq; }
        return;
    }
    uint32_t gt = 0, eq = 0;
    for (int k = threadIdx.x * 8; k < K; k += kElemsPerIter) {
        uint32_t key[8];
        load_keys8<F16>(score, (size_t)n * K + k, key);
#pragma unroll
        for (int i = 0; i < 8; ++i) { gt += key[i] > thr; eq += key[i] == thr; }
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) { gt += __shfl_xor(gt, d); eq += __shfl_xor(eq, d); }
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = gt; red[1][threadIdx.x >> 6] = eq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t a = 0, b = 0;
        for (int i = 0; i < kWaves; ++i) { a += red[0][i]; b += red[1][i]; }
        ws[kWsRows + n] = a;
        ws[kWsRows + N + n] = b;
    }
}

// The second pass over the scores when candidates are collected: per row the count of keys whose first digit is above
// the threshold's (they are above the threshold whatever its other digits are), and the keys whose first digit equals
// it - the candidates - written to the row's part of the list and entered into the histogram of the second digit.  A
// row with more candidates than its part holds raises the overflow flag (then the full passes run).
template <bool F16>
__global__ __launch_bounds__(kThreads) void candidates_kernel(const void *score, int K, uint32_t *ws, int N, int per_row,
                                                              int force_overflow)
{
    __shared__ uint32_t red[kWaves];
    __shared__ uint32_t count_s;
    const int n = blockIdx.x;
    if (threadIdx.x == 0) count_s = 0;
    __syncthreads();
    const uint32_t p0 = ws[kWsPrefix] >> 20;
    uint32_t *hist = ws + kWsRows + 3 * N, *counts = hist + kSelBins, *keys = counts + N + (size_t)n * per_row;
    uint32_t gt = 0;
    for (int k = threadIdx.x * 8; k < K; k += kElemsPerIter) {
        uint32_t key[8];
        load_keys8<F16>(score, (size_t)n * K + k, key);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t d0 = key[i] >> 20;
            gt += d0 > p0;
            // One LDS atomic per wave and position: the first candidate lane reserves the slots, the others take
            // theirs by their rank among the wave's candidate lanes.
            const bool cand = d0 == p0;
            const unsigned long long m = __ballot(cand);
            if (m) {
                const int leader = __builtin_ctzll(m);
                uint32_t first = 0;
                if ((int)(threadIdx.x & 63) == leader) first = atomicAdd(&count_s, (uint32_t)__builtin_popcountll(m));
                first = __shfl(first, leader);
                if (cand) {
                    const uint32_t slot = first + (uint32_t)__builtin_popcountll(m & ((1ull << (threadIdx.x & 63)) - 1ull));
                    if (slot < (uint32_t)per_row) {
                        keys[slot] = key[i];
                        atomicAdd(&hist[digit_of<1>(key[i])], 1u);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) gt += __shfl_xor(gt, d);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = gt;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t a = 0;
        for (int i = 0; i < kWaves; ++i) a += red[i];
        ws[kWsRows + n] = a;                            // row_count_kernel adds the candidates above the threshold (or counts anew)
        ws[kWsRows + N + n] = 0;
        const uint32_t count = count_s;
        counts[n] = count < (uint32_t)per_row ? count : (uint32_t)per_row;
        if (force_overflow || count > (uint32_t)per_row) ws[kWsCandOverflow] = 1u;
    }
}

// Ties at the threshold are kept in flat-index order until `remaining` of them are taken;
// row_ptr is the running count of kept entries.  One block; a thread takes kRowsPerThread
// consecutive rows per round, so that a round of two block scans covers 2048 rows.  The rows' counts go
// through LDS: read from memory with consecutive threads on consecutive rows, handed to the thread that owns them.
constexpr int kRowsPerThread = 8;
__global__ __launch_bounds__(kThreads) void row_scan_kernel(uint32_t *ws, int N, int32_t *row_ptr)
{
    constexpr int kRound = kThreads * kRowsPerThread;
    __shared__ uint32_t smem[kWaves];
    __shared__ uint32_t s_gt[kRound], s_eq[kRound];
    const uint32_t need = ws[kWsRemaining];
    uint32_t eq_before = 0, kept_before = 0;
    for (int n0 = 0; n0 < N; n0 += kRound) {
        __syncthreads();                                // the round before is done with the LDS arrays
#pragma unroll
        for (int i = 0; i < kRowsPerThread; ++i) {
            const int l = i * kThreads + threadIdx.x, n = n0 + l;
            s_gt[l] = n < N ? ws[kWsRows + n] : 0u;
            s_eq[l] = n < N ? ws[kWsRows + N + n] : 0u;
        }
        __syncthreads();
        const int local = threadIdx.x * kRowsPerThread, base = n0 + local;
        uint32_t gt[kRowsPerThread], eq[kRowsPerThread], eq_sum = 0;
#pragma unroll
        for (int i = 0; i < kRowsPerThread; ++i) {
            gt[i] = s_gt[local + i];
            eq[i] = s_eq[local + i];
            eq_sum += eq[i];
        }
        uint32_t eq_total, kept_total;
        uint32_t eq_rank = eq_before + block_exclusive_scan(eq_sum, smem, eq_total);
        uint32_t take[kRowsPerThread], kept_sum = 0;
#pragma unroll
        for (int i = 0; i < kRowsPerThread; ++i) {
            take[i] = eq_rank >= need ? 0u : (need - eq_rank < eq[i] ? need - eq_rank : eq[i]);
            eq_rank += eq[i];
            kept_sum += gt[i] + take[i];
        }
        uint32_t pos = kept_before + block_exclusive_scan(kept_sum, smem, kept_total);
        // results back through LDS, written out with consecutive threads on consecutive rows
#pragma unroll
        for (int i = 0; i < kRowsPerThread; ++i) {
            s_gt[local + i] = take[i];
            s_eq[local + i] = pos;
            pos += gt[i] + take[i];
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kRowsPerThread; ++i) {
            const int l = i * kThreads + threadIdx.x, n = n0 + l;
            if (n < N) { ws[kWsRows + 2 * N + n] = s_gt[l]; row_ptr[n] = (int32_t)s_eq[l]; }
        }
        eq_before += eq_total;
        kept_before += kept_total;
    }
    if (threadIdx.x == 0) row_ptr[N] = (int32_t)kept_before;
}

__device__ inline double half_bits_to_double(uint16_t h)
{
    return (double)(float)__builtin_bit_cast(_Float16, h);
}

// Eq. 6 / Eq. 7 for one group from its masked min and max (both already widened to contain 0).
template <int BITS> __device__ inline void scale_and_zero(float mn, float mx, uint16_t &s_bits, int &z)
{
    constexpr int maxq = (1 << BITS) - 1;
    const double R = (double)mx - (double)mn;
    if (R == 0.0) { s_bits = 0x3C00; z = 0; return; }
    // First guess near R/maxq, then walk to the smallest FP16 s with s*maxq >= R; the walk makes
    // the result independent of how the guess was rounded.
    uint16_t sb = __builtin_bit_cast(uint16_t, (_Float16)(float)(R / maxq));
    if (sb == 0) sb = 1;
    while (sb < 0x7BFF && half_bits_to_double(sb) * maxq < R) ++sb;
    while (sb > 1 && half_bits_to_double((uint16_t)(sb - 1)) * maxq >= R) --sb;
    const double zr = rint(-(double)mn / half_bits_to_double(sb));
    z = !(zr > 0.0) ? 0 : (zr > maxq ? maxq : (int)zr);
    s_bits = sb;
}

// One block per output channel n.  Walks the row in flat-index order: marks the kept entries,
// appends them to the CSR arrays, and quantises each group (16 to 128 weights: 2 to 16 consecutive threads) and packs each block of 128 codes.
template <int BITS, bool F16>
__global__ __launch_bounds__(kThreads) void encode_kernel(const uint16_t *__restrict__ W,
                                                          const void *__restrict__ score, int N, int K,
                                                          int group, const uint32_t *__restrict__ ws,
                                                          const int32_t *__restrict__ row_ptr,
                                                          uint32_t *__restrict__ qweight,
                                                          uint16_t *__restrict__ scales,
                                                          uint8_t *__restrict__ zeros,
                                                          uint16_t *__restrict__ col_idx,
                                                          uint16_t *__restrict__ out_val)
{
    constexpr int maxq = (1 << BITS) - 1;
    constexpr int wpg = words_per_group(BITS);
    __shared__ uint32_t smem[kWaves];
    __shared__ uint8_t code_lds[BITS == 3 ? kElemsPerIter : 8];

    const int n = blockIdx.x, tid = threadIdx.x;
    const int gpr = K / kGroup;
    const int spr = K / group, lanes = group / 8;       // scale groups per row; threads that share one
    const uint32_t thr = ws[kWsPrefix];
    const uint32_t take = ws[kWsRows + 2 * N + n];
    uint32_t ties_seen = 0, gt_seen = 0;                // of the chunks before the current one
    const uint32_t out_pos = (uint32_t)row_ptr[n];

    for (int k0 = 0; k0 < K; k0 += kElemsPerIter) {
        const int k = k0 + tid * 8;
        const bool active = k < K;          // a group is 16 consecutive threads: all or none active
        uint16_t w[8];
        uint32_t key[8];
        uint32_t gt_mask = 0, eq_mask = 0;
        if (active) {
            const uint4 v = *reinterpret_cast<const uint4 *>(W + (size_t)n * K + k);
            const uint32_t vw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) { w[2 * i] = (uint16_t)(vw[i] & 0xFFFF); w[2 * i + 1] = (uint16_t)(vw[i] >> 16); }
            load_keys8<F16>(score, (size_t)n * K + k, key);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                gt_mask |= (uint32_t)(key[i] > thr) << i;
                eq_mask |= (uint32_t)(key[i] == thr) << i;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = 0;
        }

        // One scan for both counts (each at most 2048 per chunk: 16 bits apiece): the keys above the
        // threshold and the threshold ties before this thread, in flat-index order.  The first `take`
        // ties of the row are kept, so of the ties before this thread min(their number, take) are, and
        // the thread's first kept entry goes behind those and the larger keys before it.
        uint32_t both_total;
        const uint32_t both = block_exclusive_scan((uint32_t)__popc(gt_mask) | (uint32_t)__popc(eq_mask) << 16, smem, both_total);
        const uint32_t tie_rank = ties_seen + (both >> 16);
        uint32_t sel_mask = gt_mask;
        {
            uint32_t r = tie_rank;
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (eq_mask >> i & 1) { if (r < take) sel_mask |= 1u << i; ++r; }
        }
        uint32_t pos = out_pos + gt_seen + (both & 0xFFFFu) + (tie_rank < take ? tie_rank : take);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (sel_mask >> i & 1) { col_idx[pos] = (uint16_t)(k + i); out_val[pos] = w[i]; ++pos; }
        ties_seen += both_total >> 16;
        gt_seen += both_total & 0xFFFFu;

        // Masked min / max of the group (range always contains 0), reduced over the group's 2 to 16 lanes.
        float mn = 0.f, mx = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (!(sel_mask >> i & 1)) {
                const float v = (float)__builtin_bit_cast(_Float16, w[i]);
                mn = v < mn ? v : mn;
                mx = v > mx ? v : mx;
            }
#pragma unroll
        for (int d = 1; d < 16; d <<= 1) {
            const float a = __shfl_xor(mn, d), b = __shfl_xor(mx, d);
            mn = d < lanes && a < mn ? a : mn;
            mx = d < lanes && b > mx ? b : mx;
        }
        uint16_t s_bits;
        int z;
        scale_and_zero<BITS>(mn, mx, s_bits, z);

        // Eq. 9 per weight; an outlier takes the code z.  The quotient is taken in FP32 (a correctly
        // rounded division, as the oracle's is in fp64): for FP16 operands w = mw 2^a and s = ms 2^b with
        // 11-bit mw, ms the exact quotient is either a half-integer, which FP32 holds exactly, or at
        // least 1 / (4 ms) >= 2^-13 away from one while below 2^6 in magnitude, far more than the 2^-18
        // an FP32 rounding can move it: both precisions round to the same integer.  Quotients too large
        // for that argument are clamped to 0 or maxq either way.
        const float s32 = (float)__builtin_bit_cast(_Float16, s_bits);
        uint32_t code[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float qr = rintf((float)__builtin_bit_cast(_Float16, w[i]) / s32) + (float)z;
            const int q = !(qr > 0.f) ? 0 : (qr > (float)maxq ? maxq : (int)qr);
            code[i] = (sel_mask >> i & 1) ? (uint32_t)z : (uint32_t)q;
        }

        const int g = k / kGroup;           // block of 128 codes within the row
        const int j = tid & 15;             // this thread's 8 codes are k_local = 8j .. 8j+7
        if (BITS == 4) {
            uint32_t word = 0;
#pragma unroll
            for (int t = 0; t < 8; ++t) word |= code[t] << (16 * (t & 1) + 4 * (t >> 1));
            if (active) qweight[((size_t)n * gpr + g) * wpg + j] = word;
        } else {
            __syncthreads();                // previous iteration's readers are done
#pragma unroll
            for (int t = 0; t < 8; ++t) code_lds[tid * 8 + t] = (uint8_t)code[t];
            __syncthreads();
            const uint8_t *c = code_lds + (tid >> 4) * kGroup;
            if (active && j < 13) {
                uint32_t word = 0;
                if (j < 12) {
                    const int base = 32 * (j / 3) + 10 * (j % 3);
#pragma unroll
                    for (int t = 0; t < 10; ++t) word |= (uint32_t)c[base + t] << (16 * (t & 1) + 3 * (t >> 1));
                } else {
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        word |= (uint32_t)c[32 * b + 30] << (3 * b) | (uint32_t)c[32 * b + 31] << (16 + 3 * b);
                }
                qweight[((size_t)n * gpr + g) * wpg + j] = word;
            }
        }
        if (active && (tid & (lanes - 1)) == 0) {
            scales[(size_t)n * spr + k / group] = s_bits;
            zeros[(size_t)n * spr + k / group] = (uint8_t)z;
        }
    }
}

template <bool F16>
hipError_t run_select(const void *score, int N, int K, uint32_t *ws, int32_t *row_ptr, bool any, bool full_passes,
                      hipStream_t st)
{
    const size_t total = (size_t)N * K;
    const size_t want = (total / 8 + kThreads - 1) / kThreads;
    const int blocks = (int)(want < 512 ? (want ? want : 1) : 512);
    const int per_row = pack_candidates_per_row(K);
    if (any) {
        // With nothing to keep the threshold set by init_ws_kernel already sits above every key.
        hist_kernel<0, F16><<<blocks, kThreads, 0, st>>>(score, total, ws, kAlways);
        pick_kernel<0><<<1, kSelBins / 2, 0, st>>>(ws, 0, -1);
        // Second pass over the scores: the first digit's share of the per-row counts, and the candidates.
        candidates_kernel<F16><<<N, kThreads, 0, st>>>(score, K, ws, N, per_row, full_passes ? 1 : 0);
        // Every launch from here on takes the candidates where they fitted and the scores where not; the one pass
        // that only the second way needs returns at once on the first.
        hist_kernel<1, F16><<<blocks, kThreads, 0, st>>>(score, total, ws, kWithoutCandidates);
        pick_kernel<1><<<1, kSelBins / 2, 0, st>>>(ws, 1 * kSelBins, kWsRows + 3 * N);
        // (The key of an FP16 score is its exact binary32 widening, whose low 13 bits are zero, payloads of NaNs
        // included: the third digit is 0 for every key, so FP16 scores are selected by two digits.)
        if (!F16) {
            hist_kernel<2, F16><<<blocks, kThreads, 0, st>>>(score, total, ws, kAlways, N, per_row);
            pick_kernel<2><<<1, kSelBins / 2, 0, st>>>(ws, 2 * kSelBins, -1);
        }
        row_count_kernel<F16><<<N, kThreads, 0, st>>>(score, K, ws, N, per_row);
    } else {
        row_count_kernel<F16><<<N, kThreads, 0, st>>>(score, K, ws, N, 0);
    }
    row_scan_kernel<<<1, kThreads, 0, st>>>(ws, N, row_ptr);
    return hipGetLastError();
}

template <int BITS, bool F16>
hipError_t run_encode(const void *W, const void *score, const gwq_packed &P, const uint32_t *ws, hipStream_t st)
{
    encode_kernel<BITS, F16><<<P.N, kThreads, 0, st>>>(static_cast<const uint16_t *>(W), score, P.N, P.K, P.group, ws,
                                                       P.row_ptr, P.qweight, P.scales, P.zeros, P.col_idx,
                                                       P.out_val);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_pack(const void *W, const void *score, int score_is_f16, const gwq_packed &P,
                       uint32_t *ws, bool full_passes, hipStream_t st)
{
    init_ws_kernel<<<8, kThreads, 0, st>>>(ws, (uint32_t)P.n_outliers, P.N);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = score_is_f16 ? run_select<true>(score, P.N, P.K, ws, P.row_ptr, P.n_outliers > 0, full_passes, st)
                     : run_select<false>(score, P.N, P.K, ws, P.row_ptr, P.n_outliers > 0, full_passes, st);
    if (e != hipSuccess) return e;
    if (P.bits == 4)
        return score_is_f16 ? run_encode<4, true>(W, score, P, ws, st) : run_encode<4, false>(W, score, P, ws, st);
    return score_is_f16 ? run_encode<3, true>(W, score, P, ws, st) : run_encode<3, false>(W, score, P, ws, st);
}

}  // namespace gwq
