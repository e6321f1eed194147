// gwq_linear for M > 16 on gfx950: an MFMA GEMM that dequantises the packed weights on the fly.
//
//   Y[m][n] = sum_k X[m][k] * What[n][k],  What = s*(q - z) (Sec. 3.2, Eq. 10) with the FP16
//   outliers written over their (zero-decoding) codes.
//
// A block of 8 waves owns a BM x 128 tile of Y (BM = 256, or 128 for small M) and walks K in steps
// of 64 (half a group).  Per step the block stages X[BM][64] and the dequantised weights
// What[128][64] as FP16 in LDS (double-buffered): a thread turns its codes into FP16 (exact q - z,
// one multiply by the scale), stores them, and then overwrites the positions of the channel's
// outliers.  The waves (4 along m, 2 along n) multiply 32x32x16 FP16 MFMA tiles with FP32
// accumulators and store FP16.
//
// Two waves share a SIMD because a wave can issue next to nothing while one of its own MFMAs runs
// (measured: about a quarter of the MFMA's 32 cycles): the staging work of one wave hides behind
// the MFMAs of the other.  LDS stores are the scarcest resource (about 64 bytes per clock and CU,
// a quarter of the load rate), so no lane ever stores data that is not needed.
//
// Everything a step needs from memory is requested two steps (X) or one group (codes, scale, zero
// point, outliers) ahead, with addresses that do not depend on loaded data, so no wave waits for
// memory inside the loop.  For the outliers this needs to know, per channel and group, how many
// CSR entries fall into the group: a small kernel counts them into the workspace first (one byte
// per channel and group); the running sum is the index of the group's first entry, and its first
// eight entries are fetched ahead by the channel's threads with unaligned loads (longer runs take a
// slow path).  Scales, zero points and counts are fetched four groups at a time, again with one
// unaligned load each.  The staging work of the next step is cut into pieces issued between the
// MFMA batches of the current one.
#include <type_traits>

#include "gwq_dequant.h"
#include "gwq_internal.h"

namespace gwq {
namespace {

typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kThreads = 512;
constexpr int kBN = 128;
constexpr int kBK = 64;
constexpr int kLd = kBK + 8;            // LDS row stride in halves: 144 bytes, conflict-free b128 reads
constexpr int kAhead = 8;               // outlier entries per (channel, group) fetched ahead

// ------------------------------------------------------------------------------------------------
// Outlier counts per (channel, group), saturating at 255.  One wave per channel.
__global__ __launch_bounds__(256) void group_count_kernel(const int32_t *__restrict__ row_ptr,
                                                          const uint16_t *__restrict__ col_idx, int N, int gpr,
                                                          uint8_t *__restrict__ cnt)
{
    __shared__ uint32_t c[4][512];                      // gpr <= 512 (K <= 65536)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.x * 4 + wave;
    for (int g = lane; g < gpr; g += 64) c[wave][g] = 0;
    __syncthreads();
    if (n < N) {
        const int j1 = row_ptr[n + 1];
        for (int j = row_ptr[n] + lane; j < j1; j += 64) atomicAdd(&c[wave][col_idx[j] >> 7], 1u);
    }
    __syncthreads();
    if (n < N)
        for (int g = lane; g < gpr; g += 64) cnt[(size_t)n * gpr + g] = (uint8_t)(c[wave][g] < 255u ? c[wave][g] : 255u);
}

// ------------------------------------------------------------------------------------------------
template <int BITS> struct SlotRegs;
template <> struct SlotRegs<4> { uint32_t w[4]; };
template <> struct SlotRegs<3> { uint32_t w[3], tail; };

template <int BITS> __device__ inline void load_slot(SlotRegs<BITS> &r, const uint32_t *group, int slot);
template <> __device__ inline void load_slot<4>(SlotRegs<4> &r, const uint32_t *group, int slot)
{
    const uint4 v = *reinterpret_cast<const uint4 *>(group + 4 * slot);
    r.w[0] = v.x; r.w[1] = v.y; r.w[2] = v.z; r.w[3] = v.w;
}
template <> __device__ inline void load_slot<3>(SlotRegs<3> &r, const uint32_t *group, int slot)
{
    const uint32_t *p = group + 3 * slot;
    r.w[0] = p[0]; r.w[1] = p[1]; r.w[2] = p[2];
    r.tail = group[12] >> (3 * slot);
}

// Loads of 8 / 4 bytes at 2-byte / 1-byte alignment (gfx950 global memory takes unaligned addresses).
struct __attribute__((packed, aligned(2))) U64a2 { uint32_t lo, hi; };
struct __attribute__((packed, aligned(2))) U32a2 { uint32_t v; };
struct __attribute__((packed, aligned(1))) U32a1 { uint32_t v; };

// What a thread fetches for one group of its channel.
//   4-bit: thread q of the channel's four owns columns 16q .. 16q+15 of every step: two words per
//   half of the group, and entries 2q, 2q+1 of the group's first eight outliers.
//   3-bit (words do not end on 16-column boundaries): thread (s, r) owns slot 2r + s of the group,
//   i.e. columns 32s .. 32s+31 of the steps of parity r, and entries 4s .. 4s+3; it idles in the
//   steps of the other parity.
template <int BITS> struct GroupRegs;
template <> struct GroupRegs<4> {
    uint32_t w[2][2];
    uint32_t col, val;
};
template <> struct GroupRegs<3> {
    SlotRegs<3> slot;
    uint32_t col_lo, col_hi, val_lo, val_hi;
};
// Scales, zero points and outlier counts of four consecutive groups of channel n.  (Plain words:
// the unaligned loads go through temporaries, so these stay in registers.)
struct MetaRegs {
    uint64_t sc;
    uint32_t zp, cnt;
};

// Fragment j (8 codes -> 8 FP16 values s*(q - z)) of a slot.
__device__ inline u32x4 dequant_word(uint32_t w, uint32_t z, uint32_t s2, const DecodeConsts &d)
{
    const ZeroConsts<4> c(z);
    u32x4 f = decode_word4(w, c, d);
    f.x = pk_mul(f.x, s2); f.y = pk_mul(f.y, s2); f.z = pk_mul(f.z, s2); f.w = pk_mul(f.w, s2);
    return f;
}
__device__ inline void dequant_all(const SlotRegs<3> &r, uint32_t z, uint32_t s2, const DecodeConsts &d, u32x4 f[4])
{
    decode_slot3(r.w, r.tail, z, d, f);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f[j].x = pk_mul(f[j].x, s2); f[j].y = pk_mul(f[j].y, s2);
        f[j].z = pk_mul(f[j].z, s2); f[j].w = pk_mul(f[j].w, s2);
    }
}

// MSW = 32-row sub-tiles per wave along m; the block tile is BM = 128 * MSW rows by 128 channels,
// worked on by 8 waves (4 along m, 2 along n), two per SIMD: a wave cannot issue anything else for
// most of the time one of its MFMAs runs, so the staging work of one wave overlaps the MFMAs of
// the other wave on its SIMD, not its own.
template <int BITS, int MSW>
__global__ __launch_bounds__(kThreads) void gemm_kernel(const uint32_t *__restrict__ qweight,
                                                        const uint16_t *__restrict__ scales,
                                                        const uint8_t *__restrict__ zeros,
                                                        const int32_t *__restrict__ row_ptr,
                                                        const uint16_t *__restrict__ col_idx,
                                                        const uint16_t *__restrict__ out_val,
                                                        const uint8_t *__restrict__ grp_cnt,
                                                        const _Float16 *__restrict__ X, _Float16 *__restrict__ Y,
                                                        int N, int K, int M, int tiles_m, int tiles_n, int last_entry)
{
    constexpr int BM = 128 * MSW;
    constexpr int wpg = words_per_group(BITS);
    constexpr int kAPasses = BM / 64;                   // 512 threads move 64 rows x 128 bytes per pass
    extern __shared__ _Float16 lds[];                   // [2][BM + 128][kLd]
    constexpr int kBufHalves = (BM + kBN) * kLd;        // one buffer: X rows, then weight rows

    // Tile order: bands of two m-tiles, n fastest inside a band; when the tile count divides by 8
    // every XCD (blocks go round-robin over the 8 XCDs) gets one contiguous run of that order.
    int id = blockIdx.x;
    const int total = tiles_m * tiles_n;
    if (total % 8 == 0) id = (id % 8) * (total / 8) + id / 8;
    const int band_m = tiles_m >= 2 ? 2 : 1;
    const int per_band = band_m * tiles_n;
    int mt, nt;
    {
        const int band = id / per_band, in_band = id % per_band;
        const int rows_here = (band + 1) * band_m <= tiles_m ? band_m : tiles_m - band * band_m;
        nt = in_band / rows_here;
        mt = band * band_m + in_band % rows_here;
    }
    const int m0 = mt * BM, n0 = nt * kBN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int gpr = K / kGroup;
    const int nk = K / kBK;                             // steps; two per group

    // Staging roles.  X: 8 threads cover one 128-byte row of a step.  Weights: the four threads of
    // channel n are neighbours in a wave (see GroupRegs for what each owns).
    const int a_row = tid >> 3, a_chunk = tid & 7;
    const int b_n_local = tid >> 2, b_q = tid & 3, b_s = (tid >> 1) & 1, b_r = tid & 1;
    int b_n = n0 + b_n_local;
    const bool b_valid = b_n < N;
    b_n = b_valid ? b_n : N - 1;                        // clamped: loads stay in bounds, tile row unused
    const DecodeConsts dc(BITS);

    const _Float16 *a_src[kAPasses];
#pragma unroll
    for (int p = 0; p < kAPasses; ++p) {
        int m = m0 + p * 64 + a_row;
        m = m < M ? m : M - 1;
        a_src[p] = X + (size_t)m * K + 8 * a_chunk;
    }
    const uint32_t row_group = (uint32_t)b_n * gpr;
    const uint32_t *q_row = qweight + (size_t)row_group * wpg;
    _Float16 *const a_dst = lds + a_row * kLd + 8 * a_chunk;            // + buffer, + pass * 64 rows
    _Float16 *const b_dst = lds + (BM + b_n_local) * kLd;               // + buffer

    auto issue_a = [&](int step, u32x4 dst[kAPasses]) {
        const int k0 = (step < nk ? step : nk - 1) * kBK;
#pragma unroll
        for (int p = 0; p < kAPasses; ++p) dst[p] = *reinterpret_cast<const u32x4 *>(a_src[p] + k0);
    };
    // first = CSR index of the group's first entry (it depends on counts fetched long before).
    auto issue_group = [&](int g, int first, GroupRegs<BITS> &G) {
        g = g < gpr ? g : gpr - 1;
        const uint32_t *grp = q_row + (uint32_t)g * wpg;
        if constexpr (BITS == 4) {
            const uint2 v0 = *reinterpret_cast<const uint2 *>(grp + 4 * (b_q >> 1) + 2 * (b_q & 1));
            const uint2 v1 = *reinterpret_cast<const uint2 *>(grp + 8 + 4 * (b_q >> 1) + 2 * (b_q & 1));
            G.w[0][0] = v0.x; G.w[0][1] = v0.y; G.w[1][0] = v1.x; G.w[1][1] = v1.y;
            const int j = first + 2 * b_q < last_entry ? first + 2 * b_q : last_entry;   // arrays carry 16 spare bytes
            G.col = reinterpret_cast<const U32a2 *>(col_idx + j)->v;
            G.val = reinterpret_cast<const U32a2 *>(out_val + j)->v;
        } else {
            load_slot<3>(G.slot, grp, 2 * b_r + b_s);
            const int j = first + 4 * b_s < last_entry ? first + 4 * b_s : last_entry;
            const U64a2 c = *reinterpret_cast<const U64a2 *>(col_idx + j), v = *reinterpret_cast<const U64a2 *>(out_val + j);
            G.col_lo = c.lo; G.col_hi = c.hi; G.val_lo = v.lo; G.val_hi = v.hi;
        }
    };
    // Groups 4q .. 4q+3 (reads past the row or the array stay inside the padded buffers).
    auto issue_meta = [&](int q, MetaRegs &Q) {
        const int g = 4 * q < gpr ? 4 * q : 0;
        const U64a2 sc = *reinterpret_cast<const U64a2 *>(scales + row_group + g);
        Q.sc = (uint64_t)sc.hi << 32 | sc.lo;
        Q.zp = reinterpret_cast<const U32a1 *>(zeros + row_group + g)->v;
        Q.cnt = reinterpret_cast<const U32a1 *>(grp_cnt + row_group + g)->v;
    };
    auto meta_scale = [](const MetaRegs &Q, int g) -> uint32_t {
        const uint32_t h = (uint32_t)(Q.sc >> (16 * (g & 3))) & 0xFFFFu;      // a shift, not a choice of fields
        return h | h << 16;
    };
    auto meta_zero = [](const MetaRegs &Q, int g) -> uint32_t { return (Q.zp >> (8 * (g & 3))) & 0xFFu; };
    auto meta_count = [&](const MetaRegs &Q, int g) -> int { return b_valid ? (int)((Q.cnt >> (8 * (g & 3))) & 0xFFu) : 0; };

    // Staging of step `step` into buffer `buf`, in pieces that the step function spreads over its
    // MFMA batches.  stage_x: X rows of passes p0 .. p1-1 go to LDS, and the registers are refilled
    // with the rows of two steps later.  stage_w: half of this thread's weight fragments.
    // stage_outliers: this thread's entries, then (one thread per channel) the rare rest.
    auto stage_x = [&](int p0, int p1, int step, int buf, u32x4 a_regs[kAPasses]) {
        _Float16 *A = a_dst + buf * kBufHalves;
        const int k2 = (step + 2 < nk ? step + 2 : nk - 1) * kBK;
#pragma unroll
        for (int p = p0; p < p1 && p < kAPasses; ++p) {
            *reinterpret_cast<u32x4 *>(A + p * 64 * kLd) = a_regs[p];
            a_regs[p] = *reinterpret_cast<const u32x4 *>(a_src[p] + k2);
        }
    };
    auto stage_w = [&](int pair, int step, int buf, const GroupRegs<BITS> &G, const MetaRegs &Q) {
        _Float16 *brow = b_dst + buf * kBufHalves;
        const int g = step >> 1;
        const uint32_t s2 = meta_scale(Q, g), z = meta_zero(Q, g);
        if constexpr (BITS == 4) {
            *reinterpret_cast<u32x4 *>(brow + 16 * b_q + 8 * pair) = dequant_word(G.w[step & 1][pair], z, s2, dc);
        } else {
            if (pair == 0 && b_r == (step & 1)) {
                u32x4 f[4];
                dequant_all(G.slot, z, s2, dc, f);
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(brow + 32 * b_s + 8 * j) = f[j];
            }
        }
    };
    // Outliers of this channel inside the step's 64 columns replace their decoded zeros.  The
    // writers of those zeros are lanes of the same wave and their stores were issued earlier, so
    // the order is kept.  4-bit: an entry that is not ours to write goes to the row's padding
    // (predication would fence the MFMAs off).
    auto stage_outliers = [&](int step, int buf, const GroupRegs<BITS> &G, const MetaRegs &Q, int first) {
        _Float16 *brow = b_dst + buf * kBufHalves;
        const int g = step >> 1;
        const int cnt = step < nk ? meta_count(Q, g) : 0;       // nothing to patch behind the last step
        const uint32_t k_lo = (uint32_t)(step * kBK);
        bool rest;                                              // this thread takes the entries past the eighth
        if constexpr (BITS == 4) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t col = ((G.col >> (16 * i)) & 0xFFFFu) - k_lo;
                const uint32_t dst = (2 * b_q + i < cnt && col < (uint32_t)kBK) ? col : kBK + b_q;
                brow[dst] = __builtin_bit_cast(_Float16, (uint16_t)(G.val >> (16 * i)));
            }
            rest = b_q == 0;
        } else {
            const bool mine = b_r == (step & 1);
            if (mine) {
                const uint32_t cs[2] = {G.col_lo, G.col_hi}, vs[2] = {G.val_lo, G.val_hi};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t col = ((cs[i >> 1] >> (16 * (i & 1))) & 0xFFFFu) - k_lo;
                    if (4 * b_s + i < cnt && col < (uint32_t)kBK)
                        brow[col] = __builtin_bit_cast(_Float16, (uint16_t)(vs[i >> 1] >> (16 * (i & 1))));
                }
            }
            rest = mine && b_s == 0;
        }
        if (rest)
            for (int i = kAhead; i < cnt; ++i) {        // rare: more than kAhead outliers in one group
                const uint32_t c = (uint32_t)col_idx[first + i] - k_lo;
                if (c < (uint32_t)kBK) brow[c] = __builtin_bit_cast(_Float16, out_val[first + i]);
            }
    };

    float16v acc[MSW][2];
#pragma unroll
    for (int i = 0; i < MSW; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int fi = lane & 31, fk = lane >> 5;           // fragment row and k-block of this lane
    const _Float16 *a_frag = lds + (wm * (BM / 4) + fi) * kLd + 8 * fk;
    const _Float16 *b_frag = lds + (BM + wn * 64 + fi) * kLd + 8 * fk;

    // Fragments of the k-batch being multiplied and of the one after it (16 columns each).
    u32x4 fa[2][MSW], fb[2][2];
    auto read_frags = [&](int buf, int s, u32x4 a[MSW], u32x4 b[2]) {
        const _Float16 *A = a_frag + buf * kBufHalves, *B = b_frag + buf * kBufHalves;
#pragma unroll
        for (int i = 0; i < MSW; ++i) a[i] = *reinterpret_cast<const u32x4 *>(A + i * 32 * kLd + 16 * s);
#pragma unroll
        for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const u32x4 *>(B + j * 32 * kLd + 16 * s);
    };
    auto mfma_rows = [&](int s, int i0, int i1) {
#pragma unroll
        for (int i = i0; i < i1; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, fa[s & 1][i]),
                                                                   __builtin_bit_cast(half8, fb[s & 1][j]),
                                                                   acc[i][j], 0, 0, 0);
    };
    auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
    // Scheduling pattern for the region since the last fence: `count` times one MFMA followed by
    // `others` of the staging instructions (vector ALU, scalar ALU, global loads, LDS writes).
    auto interleave = [](auto count, auto others) {
#pragma unroll
        for (int k = 0; k < decltype(count)::value; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002 | 0x004 | 0x020 | 0x200, decltype(others)::value, 0);
        }
    };
    using std::integral_constant;

    // One step.  On entry the fragments of its first k-batch are in fa[0], fb[0].  Each k-batch
    // first requests the fragments of the batch after it, then multiplies with a piece of the
    // staging of step + 1 (into the other buffer, from a_regs, G, Q) scheduled among its MFMAs:
    // the weights in batches 0 and 1, the outliers and the X rows in batch 2.  The block's barrier
    // sits in the middle of the last batch: behind it the first fragments of step + 1 are requested
    // while the rest of the batch still multiplies.
    auto step_fn = [&](int step, int buf, u32x4 a_regs[kAPasses], const GroupRegs<BITS> &G, const MetaRegs &Q,
                       int first) {
        constexpr int kMfma = 2 * MSW;                          // MFMAs of one batch
        constexpr int h = MSW >= 2 ? MSW / 2 : 1;               // rows of the last batch ahead of the barrier
        // LDS stores are the slow kind of LDS traffic (a 16-byte store per lane keeps the unit busy
        // four times as long as a load), so they are spread evenly: fragment loads queued behind a
        // burst of stores would come back late.
        read_frags(buf, 1, fa[1], fb[1]);
        fence();
        mfma_rows(0, 0, MSW);
        stage_w(0, step + 1, buf ^ 1, G, Q);
        stage_x(0, 1, step + 1, buf ^ 1, a_regs);
        interleave(integral_constant<int, kMfma>{}, integral_constant<int, 32 / kMfma>{});
        fence();
        read_frags(buf, 2, fa[0], fb[0]);
        fence();
        mfma_rows(1, 0, MSW);
        stage_w(1, step + 1, buf ^ 1, G, Q);
        stage_x(1, 2, step + 1, buf ^ 1, a_regs);
        interleave(integral_constant<int, kMfma>{}, integral_constant<int, 32 / kMfma>{});
        fence();
        read_frags(buf, 3, fa[1], fb[1]);
        fence();
        mfma_rows(2, 0, MSW);
        stage_outliers(step + 1, buf ^ 1, G, Q, first);
        stage_x(2, 3, step + 1, buf ^ 1, a_regs);
        fence();
        mfma_rows(3, 0, h);
        stage_x(3, kAPasses, step + 1, buf ^ 1, a_regs);
        fence();
        __syncthreads();
        read_frags(buf ^ 1, 0, fa[0], fb[0]);
        fence();
        mfma_rows(3, h, MSW);
    };

    // Prologue: metadata of groups 0..7, codes and outliers of groups 0 and 1, the X rows of
    // steps 0 and 1; step 0 staged.
    MetaRegs Qc, Qn;                                    // groups 4q .. 4q+3 and the four after them
    GroupRegs<BITS> Gc, Gn;                             // current group, next group
    u32x4 a0[kAPasses], a1[kAPasses];                   // X rows of the even / odd step being staged
    int first_c = b_valid ? row_ptr[b_n] : 0;           // CSR index of the current group's first entry
    issue_meta(0, Qc);
    issue_meta(1, Qn);
    issue_a(0, a0);
    issue_a(1, a1);
    issue_group(0, first_c, Gc);
    int first_n = first_c + meta_count(Qc, 0);
    issue_group(1, first_n, Gn);
    stage_w(0, 0, 0, Gc, Qc);
    stage_w(1, 0, 0, Gc, Qc);
    stage_outliers(0, 0, Gc, Qc, first_c);
    stage_x(0, kAPasses, 0, 0, a0);                     // refills a0 with the rows of step 2
    __syncthreads();
    read_frags(0, 0, fa[0], fb[0]);

    // Main loop, one group (two steps) per trip.  Entering trip g: buffer 0 holds step 2g, a1
    // holds the X rows of step 2g + 1, a0 those of step 2g + 2 (in flight), Gc is group g, Gn is
    // group g + 1 (in flight), Qc covers group g, Qn the four groups after Qc's.
    for (int g = 0; g < gpr; ++g) {
        step_fn(2 * g, 0, a1, Gc, Qc, first_c);         // stages step 2g + 1 (second half of group g)
        // Second half: stage step 2g + 2 = first half of group g + 1, then move on to it.
        const bool roll = (g & 3) == 3;                 // group g + 1 starts the next four
        MetaRegs Qs;                                    // selected by value: a reference would pin both in memory
        Qs.sc = roll ? Qn.sc : Qc.sc;
        Qs.zp = roll ? Qn.zp : Qc.zp; Qs.cnt = roll ? Qn.cnt : Qc.cnt;
        step_fn(2 * g + 1, 1, a0, Gn, Qs, first_n);
        Gc = Gn;
        if (roll) {
            Qc = Qn;
            issue_meta((g + 1) / 4 + 1, Qn);
        }
        first_c = first_n;
        first_n = first_c + meta_count(Qc, g + 1);
        issue_group(g + 2, first_n, Gn);
    }

    // D layout of the 32x32 tile: column = lane % 32, row = 8*(v/4) + 4*(lane/32) + v%4.
#pragma unroll
    for (int i = 0; i < MSW; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn * 64 + j * 32 + fi;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * (BM / 4) + i * 32 + 8 * (v >> 2) + 4 * fk + (v & 3);
                if (m < M && n < N) Y[(size_t)m * N + n] = (_Float16)acc[i][j][v];
            }
        }
}

template <int BITS, int MSW>
hipError_t launch_ms(const gwq_packed &P, const void *X, int M, void *Y, uint8_t *grp_cnt, hipStream_t st)
{
    constexpr int BM = 128 * MSW;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (P.N + kBN - 1) / kBN;
    const size_t lds = (size_t)2 * (BM + kBN) * kLd * sizeof(_Float16);
    static bool attr_set = false;                       // per instantiation; idempotent HIP call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel<BITS, MSW>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    gemm_kernel<BITS, MSW><<<tiles_m * tiles_n, kThreads, lds, st>>>(
        P.qweight, P.scales, P.zeros, P.row_ptr, P.col_idx, P.out_val, grp_cnt, static_cast<const _Float16 *>(X),
        static_cast<_Float16 *>(Y), P.N, P.K, M, tiles_m, tiles_n, P.n_outliers > 0 ? (int)P.n_outliers - 1 : 0);
    return hipGetLastError();
}

}  // namespace

size_t gemm_workspace_bytes(int64_t N, int64_t K) { return (size_t)(N * (K / kGroup) + 255) / 256 * 256 + 256; }

hipError_t launch_gemm(const gwq_packed &P, const void *X, int M, void *Y, void *workspace, int ms_override,
                       hipStream_t st)
{
    uint8_t *cnt = static_cast<uint8_t *>(workspace);
    group_count_kernel<<<(P.N + 3) / 4, 256, 0, st>>>(P.row_ptr, P.col_idx, P.N, P.K / kGroup, cnt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // Rows per tile: 256 unless M is small (the override is in rows: 64 and 128 both mean 128).
    const int msw = ms_override ? (ms_override >= 4 ? 2 : 1) : M <= 128 ? 1 : 2;
    if (P.bits == 4) return msw == 1 ? launch_ms<4, 1>(P, X, M, Y, cnt, st) : launch_ms<4, 2>(P, X, M, Y, cnt, st);
    return msw == 1 ? launch_ms<3, 1>(P, X, M, Y, cnt, st) : launch_ms<3, 2>(P, X, M, Y, cnt, st);
}

}  // namespace gwq
