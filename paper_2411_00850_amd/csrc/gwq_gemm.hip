// gwq_linear for M > 16 on gfx950: an MFMA GEMM that dequantises the packed weights on the fly.
//
//   Y[m][n] = sum_k X[m][k] * What[n][k],  What = s*(q - z) (Sec. 3.2, Eq. 10) with the FP16
//   outliers written over their (zero-decoding) codes.
//
// A block owns a BM x 128 tile of Y (BM = 256; 128, 64 or 32 for small M) and walks K in steps of 64 (half
// a group).  Per step X[BM][64] and the dequantised weights What[128][64] are staged as FP16 in LDS
// (three buffers each) and multiplied with 32x32x16 FP16 MFMA tiles, FP32 accumulators, FP16 store.
//
// The 16 waves of a block have three roles, four waves per SIMD:
//   * 8 consumers (4 along m, 2 along n; 2 x 4 or 1 x 4 in the blocks for small M) do nothing but read
//     fragments from LDS, two k-batches ahead, and issue MFMAs;
//   * 4 producers stage the weights of the next step: codes to FP16 (exact q - z, one multiply by
//     the scale) to LDS, then the channel's outliers over their decoded zeros;
//   * 4 loaders copy the X rows of the step after next from memory straight into LDS (loads with
//     an LDS destination: no registers, no LDS store instructions).
// A wave can issue next to nothing while one of its own MFMAs runs (measured: about a quarter of
// the MFMA's 32 cycles are free), so staging done by the multiplying waves themselves is time added
// to theirs; done by other waves of the SIMD it is hidden.  What the roles share is the LDS: per
// step 128 KB of fragment reads, 32 KB of X and 16 KB of weights written, which together keep it
// busy about as long as the step's MFMAs take.
//
// Everything a step needs from memory is requested two steps ahead, with addresses that do not
// depend on data requested in the same trip, so nobody waits for memory inside the loop.  For the
// outliers this needs to know, per channel and group, where the group's CSR entries start: a small
// kernel writes that index, with the group's scale and zero point, one 8-byte record per channel
// and group (per call into the workspace, or once per layer: gwq_linear_index); a group's first
// eight entries are fetched ahead by the channel's two threads with unaligned loads (longer runs
// take a slow path).
//
// Launches with fewer tiles than CUs also split K over up to eight blocks per tile; their FP32
// partial sums go to scratch and splitk_reduce_kernel adds them in a fixed order.
#include <stdio.h>

#include <type_traits>

#include "gwq_dequant.h"
#include "gwq_internal.h"

namespace gwq {
namespace {

typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kConsumers = 8, kProducers = 4, kLoaders = 4;     // waves
constexpr int kThreads = 64 * (kConsumers + kProducers + kLoaders);
constexpr int kBN = 128;
constexpr int kBK = 64;
constexpr int kLd = kBK + 8;            // LDS row stride in halves: 144 bytes, conflict-free b128 reads
constexpr int kAhead = 8;               // outlier entries per (channel, group) fetched ahead

// ------------------------------------------------------------------------------------------------
// Per (channel, group) record for the GEMM's producers: the CSR index of the group's first outlier
// and the group's scale and zero point, so that one 8-byte load fetches everything a group needs
// besides its codes.  gpr + 1 records per channel; the last one holds the channel's end index.
// One wave per channel.
struct GroupRecord {
    int32_t first;
    uint32_t scale_zero;                                // scale bits | zero point << 16
};

__global__ __launch_bounds__(256) void group_index_kernel(const int32_t *__restrict__ row_ptr,
                                                          const uint16_t *__restrict__ col_idx,
                                                          const uint16_t *__restrict__ scales,
                                                          const uint8_t *__restrict__ zeros, int N, int gpr,
                                                          uint32_t scale_cap, GroupRecord *__restrict__ rec)
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
    if (n >= N) return;
    // Exclusive prefix over the groups: lane l owns groups 8l .. 8l+7.
    uint32_t mine[8], sum = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int g = 8 * lane + i;
        mine[i] = g < gpr ? c[wave][g] : 0u;
        sum += mine[i];
    }
    uint32_t incl = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
    }
    uint32_t first = (uint32_t)row_ptr[n] + incl - sum;
    GroupRecord *out = rec + (size_t)n * (gpr + 1);
    const size_t row_group = (size_t)n * gpr;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int g = 8 * lane + i;
        if (g < gpr) {
            // The GEMM multiplies FP16 operands s * (q - z): a scale is capped at the largest FP16 value whose
            // product with 2^bits - 1 is still finite (only ranges beyond 65460 reach it; positive FP16
            // patterns order like integers).
            const uint32_t sc = scales ? scales[row_group + g] : 0u, zp = scales ? zeros[row_group + g] : 0u;
            out[g] = GroupRecord{(int32_t)first, (sc < scale_cap ? sc : scale_cap) | zp << 16};
        }
        first += mine[i];
    }
    if (lane == 0) out[gpr] = GroupRecord{row_ptr[n + 1], 0u};
}

// Layers quantised in groups of fewer than 128 weights (16, 32 or 64): per channel and block of 128 codes,
// eight words scale bits | zero point << 16, one per 16 columns (a group's pair repeated over its columns),
// so that a producer finds the two pairs of a slot's halves with one 8-byte load, whatever the group size.
__global__ __launch_bounds__(256) void fine_index_kernel(const uint16_t *__restrict__ scales, const uint8_t *__restrict__ zeros,
                                                         size_t count, int K, int group, uint32_t scale_cap,
                                                         uint32_t *__restrict__ fine)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;           // (channel, 16-column piece)
    if (i >= count) return;
    const size_t n = i / (K / 16), piece = i % (K / 16);
    const size_t g = n * (K / group) + piece * 16 / group;
    const uint32_t sc = scales[g];
    fine[i] = (sc < scale_cap ? sc : scale_cap) | (uint32_t)zeros[g] << 16;
}

// ------------------------------------------------------------------------------------------------
template <int BITS> struct SlotRegs;
template <> struct SlotRegs<4> { uint32_t w[4]; };
template <> struct SlotRegs<3> { uint32_t w[3], fourth; };    // fourth: the word after the slot's three (slot 3: the tail word)

template <int BITS> __device__ inline void load_slot(SlotRegs<BITS> &r, const uint32_t *group, int slot);
template <> __device__ inline void load_slot<4>(SlotRegs<4> &r, const uint32_t *group, int slot)
{
    const uint4 v = *reinterpret_cast<const uint4 *>(group + 4 * slot);
    r.w[0] = v.x; r.w[1] = v.y; r.w[2] = v.z; r.w[3] = v.w;
}
template <> __device__ inline void load_slot<3>(SlotRegs<3> &r, const uint32_t *group, int slot)
{
    // one 16-byte load at 4-byte alignment; it stays inside the group's 13 words for every slot
    const U128a4 v = *reinterpret_cast<const U128a4 *>(group + 3 * slot);
    r.w[0] = v.x; r.w[1] = v.y; r.w[2] = v.z; r.fourth = v.w;
}

// A 16-bit load that is complete when it returns, invisible to the compiler's bookkeeping of
// outstanding loads: for the rare path inside the staging loop, whose loads would otherwise make
// the compiler wait for every prefetch in flight at each trip of the loop.
__device__ inline uint32_t load_u16_now(const uint16_t *p)
{
    uint32_t v;
    asm volatile("global_load_ushort %0, %1, off\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
    return v;
}

// A load of 8 bytes at 2-byte alignment (gfx950 global memory takes unaligned addresses).
struct __attribute__((packed, aligned(2))) U64a2 { uint32_t lo, hi; };

// What producer thread (n, h) fetches for one group of channel n: its two slots (h and 2 + h: columns
// 32h .. 32h+31 of the group's two steps), entries 4h .. 4h+3 of the group's first eight outliers
// as packed 16-bit pairs, and the record of the group after it.
template <int BITS> struct GroupRegs {
    SlotRegs<BITS> slot[2];
    uint32_t col_lo, col_hi, val_lo, val_hi;
    int32_t next_first;
    uint32_t next_scale_zero;
    uint32_t sub[4];                                    // small groups only: scale | zero << 16 of the halves of the two slots
};

// Fragment j (8 codes -> 8 FP16 values s*(q - z)) of a slot.
__device__ inline u32x4 dequant_frag(const SlotRegs<4> &r, int j, uint32_t z, uint32_t s2, const DecodeConsts &d)
{
    const ZeroConsts<4> c(z);
    u32x4 f = decode_word4(r.w[j], c, d);
    f.x = pk_mul(f.x, s2); f.y = pk_mul(f.y, s2); f.z = pk_mul(f.z, s2); f.w = pk_mul(f.w, s2);
    return f;
}
__device__ inline void dequant_all(const SlotRegs<3> &r, uint32_t tail_pair, uint32_t z, uint32_t s2, const DecodeConsts &d,
                                   u32x4 f[4])
{
    decode_slot3(r.w, tail_pair, z, d, f);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f[j].x = pk_mul(f[j].x, s2); f[j].y = pk_mul(f[j].y, s2);
        f[j].z = pk_mul(f[j].z, s2); f[j].w = pk_mul(f[j].w, s2);
    }
}

// bfloat16 operands: the eight exact FP16 integers q - z of a fragment times the scale in FP32, rounded once to
// bfloat16 (round to nearest even).
__device__ inline uint32_t scale_pair_bf16(uint32_t h2, float s)
{
    const half2v h = __builtin_bit_cast(half2v, h2);
    const __bf16 lo = (__bf16)((float)h.x * s), hi = (__bf16)((float)h.y * s);
    return (uint32_t)__builtin_bit_cast(uint16_t, lo) | (uint32_t)__builtin_bit_cast(uint16_t, hi) << 16;
}
__device__ inline u32x4 scale_frag_bf16(u32x4 f, float s)
{
    return u32x4{scale_pair_bf16(f.x, s), scale_pair_bf16(f.y, s), scale_pair_bf16(f.z, s), scale_pair_bf16(f.w, s)};
}
// An FP16 bit pattern as the nearest bfloat16's (the stored outliers, for bfloat16 MFMA operands).
__device__ inline uint16_t half_bits_to_bf16_bits(uint32_t h)
{
    return __builtin_bit_cast(uint16_t, (__bf16)(float)__builtin_bit_cast(_Float16, (uint16_t)h));
}

// X rows lie in LDS 128 bytes apart, so the 16-byte chunk c of row r is kept at position
// c ^ x_swizzle(r): the 16 rows a fragment read touches per cycle then hit 16 different bank groups,
// whichever of the two plausible lane groupings the hardware uses.
__device__ inline int x_swizzle(int r)
{
    const int t = (r >> 1) & 7;
    return (t & 3) << 1 | t >> 2;
}
template <int N> __device__ inline void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// The consumer waves form a WM x WN grid (WN = 2 or 4 along n), each with MSW 32-row sub-tiles along m
// and 128 / 32 / WN 32-column sub-tiles along n: the block tile is BM = 32 * MSW * WM rows by 128
// channels - 256 rows (MSW 2, 4 x 2 waves) for large M, 128 (MSW 1, 4 x 2), 64 (2 x 4) and 32 rows
// (1 x 4, four consumer waves idle) for small M, where a step is bounded by LDS traffic and the staged
// weights are then read by fewer rows of waves.  When the tiles alone would leave most of the chip idle (few rows, few channels), K is
// split as well: `splits` blocks share a tile, block s of them takes groups s * split_groups onwards
// and writes its FP32 sums to partial[s][M][N] instead of Y; splitk_reduce_kernel adds them up in
// the order of s.
// FINE: the layer's groups are smaller than 128; the producers take scale and zero point per half slot from `fine`
// (fine_index_kernel) instead of the group's record.
// BF16: X and Y are bfloat16 and the MFMAs take bfloat16 operands: the producers round s * (q - z), formed in FP32, and
// the stored outliers to bfloat16 (groups of 128 only).
template <int BITS, int MSW, int WN, int WM, bool FINE, bool BF16>
__global__ __launch_bounds__(kThreads) void gemm_kernel(const uint32_t *__restrict__ qweight,
                                                        const uint16_t *__restrict__ col_idx,
                                                        const uint16_t *__restrict__ out_val,
                                                        const GroupRecord *__restrict__ rec,
                                                        const uint32_t *__restrict__ fine,
                                                        const _Float16 *__restrict__ X, _Float16 *__restrict__ Y,
                                                        float *__restrict__ partial, int split_groups,
                                                        int N, int K, int M, int tiles_m, int tiles_n, int last_entry)
{
    static_assert(WM * WN <= kConsumers, "consumer waves");
    static_assert(!(FINE && BF16), "bfloat16 activations: groups of 128 only");
    typedef std::conditional_t<BF16, __bf16, _Float16> act_t;
    constexpr int BM = 32 * MSW * WM;                   // WM x WN consumer waves work; with fewer than eight the rest idle
    constexpr int NB = kBN / 32 / WN;                   // 32-column sub-tiles per consumer wave
    constexpr int wpg = words_per_group(BITS);
    // LDS: three X buffers of BM rows x 128 bytes (unpadded: the loads that fill them write whole
    // kilobytes; the 16-byte chunks of a row are permuted instead, see x_swizzle), then three weight
    // buffers of 128 rows x kLd halves.  Step t uses buffers t % 3.
    extern __shared__ _Float16 lds[];
    constexpr int kXBufHalves = BM * kBK;
    constexpr int kWBufHalves = kBN * kLd;
    _Float16 *const lds_w = lds + 3 * kXBufHalves;

    // Tile order: bands of two m-tiles, n fastest inside a band; when the tile count divides by 8
    // every XCD (blocks go round-robin over the 8 XCDs) gets one contiguous run of that order.
    const int total = tiles_m * tiles_n;
    const int split = blockIdx.x / total;
    int id = blockIdx.x % total;
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

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int gpr = K / kGroup;                         // groups per row of the matrix
    const int g_first = split * split_groups;           // this block's groups: g_first .. g_first + gl - 1
    const int gl = gpr - g_first < split_groups ? gpr - g_first : split_groups;
    const int nk = 2 * gl;                              // steps; two per group
    const int k_first = g_first * kGroup;

    // Every wave passes the block's barrier exactly 1 + nk times: once when step 0 is staged, then
    // once per step (the consumers between the step's second and third k-batch).  Barrier t, the one
    // of step t, says: step t + 1 is staged, and nobody reads the buffers of step t any more (its
    // last fragments are in registers).
    if (wave >= kConsumers && wave < kConsumers + kProducers) {
        // ======================================= producers =====================================
        const int ptid = tid - 64 * kConsumers;
        const int b_n_local = ptid >> 1, b_h = ptid & 1;
        int b_n = n0 + b_n_local;
        const bool b_valid = b_n < N;
        b_n = b_valid ? b_n : N - 1;                    // clamped: loads stay in bounds, tile row unused
        const DecodeConsts dc(BITS);

        const uint32_t *q_row = qweight + ((size_t)b_n * gpr + g_first) * wpg;       // group numbers below are local
        const GroupRecord *r_row = rec + (size_t)b_n * (gpr + 1) + g_first;
        const uint32_t *f_row = fine + ((size_t)b_n * gpr + g_first) * 8 + 2 * b_h;
        _Float16 *const b_dst = lds_w + b_n_local * kLd;                    // + buffer

        // Requests for group g (clamped: the last trips ask for groups past the row's end and use
        // none of it); first = CSR index of its first entry.
        auto issue_group = [&](int g, int first, GroupRegs<BITS> &G) {
            g = g < gl ? g : gl - 1;
            const uint32_t *grp = q_row + (uint32_t)g * wpg;
            load_slot<BITS>(G.slot[0], grp, b_h);
            load_slot<BITS>(G.slot[1], grp, 2 + b_h);
            const int j = first + 4 * b_h < last_entry ? first + 4 * b_h : last_entry;   // arrays carry 16 spare bytes
            const U64a2 c = *reinterpret_cast<const U64a2 *>(col_idx + j), v = *reinterpret_cast<const U64a2 *>(out_val + j);
            G.col_lo = c.lo; G.col_hi = c.hi; G.val_lo = v.lo; G.val_hi = v.hi;
            const GroupRecord r = r_row[g + 1];
            G.next_first = r.first; G.next_scale_zero = r.scale_zero;
            if constexpr (FINE) {
                const uint2 a = *reinterpret_cast<const uint2 *>(f_row + (uint32_t)g * 8);
                const uint2 c2 = *reinterpret_cast<const uint2 *>(f_row + (uint32_t)g * 8 + 4);
                G.sub[0] = a.x; G.sub[1] = a.y; G.sub[2] = c2.x; G.sub[3] = c2.y;
            }
        };

        // Staging of step `step` (of a group with scale and zero point sz, `cnt` outliers from CSR
        // index `first`) into buffer `buf`: this thread's 32 columns of weights, then its four
        // outlier entries (anywhere in the step's 64 columns: the thread that decoded those columns
        // is the lane next to this one and its stores were issued before).  The outlier stores are
        // unconditional: an entry that is absent or outside this step goes to column 64, the row's
        // padding.  (Stores under a condition would sit in branches, and there the compiler waits
        // for every load in flight before it touches a loaded value.)
        uint32_t out_col[4];                            // columns of the group's entries; 0x10000 = no entry
        auto stage = [&](int step, int buf, const GroupRegs<BITS> &G, uint32_t sz, int first, int cnt) {
            _Float16 *brow = b_dst + buf * kWBufHalves;
            const int half = step & 1;
            const uint32_t s2 = (sz & 0xFFFFu) * 0x10001u, z = sz >> 16;
            if constexpr (BF16) {
                const float sf = (float)__builtin_bit_cast(_Float16, (uint16_t)(sz & 0xFFFFu));
                u32x4 f[4];
                if constexpr (BITS == 4) {
                    decode_slot4(G.slot[half].w, z, dc, f);
                } else {
                    const uint32_t tail = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)G.slot[1].fourth, 0xF5, 0xF, 0xF, false);
                    decode_slot3(G.slot[half].w, tail >> (3 * (2 * half + b_h)), z, dc, f);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(brow + 32 * b_h + 8 * j) = scale_frag_bf16(f[j], sf);
            } else if constexpr (FINE) {
                const uint32_t lo = G.sub[2 * half], hi = G.sub[2 * half + 1];
                u32x4 f[4];
                if constexpr (BITS == 4) {
                    decode_slot4_halves(G.slot[half].w, lo >> 16, hi >> 16, dc, f);
                } else {
                    const uint32_t tail = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)G.slot[1].fourth, 0xF5, 0xF, 0xF, false);
                    decode_slot3_halves(G.slot[half].w, tail >> (3 * (2 * half + b_h)), lo >> 16, hi >> 16, dc, f);
                }
                scale_halves(f, (lo & 0xFFFFu) * 0x10001u, (hi & 0xFFFFu) * 0x10001u);
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(brow + 32 * b_h + 8 * j) = f[j];
            } else if constexpr (BITS == 4) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    *reinterpret_cast<u32x4 *>(brow + 32 * b_h + 8 * j) = dequant_frag(G.slot[half], j, z, s2, dc);
            } else {
                // The group's tail word is the fourth word of slot 3, which the odd thread of the
                // channel has loaded: both threads of the pair read it from there (quad_perm 1,1,3,3).
                const uint32_t tail = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)G.slot[1].fourth, 0xF5, 0xF, 0xF, false);
                u32x4 f[4];
                dequant_all(G.slot[half], tail >> (3 * (2 * half + b_h)), z, s2, dc, f);
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(brow + 32 * b_h + 8 * j) = f[j];
            }
            cnt = step < nk ? cnt : 0;
            const uint32_t k_lo = (uint32_t)(k_first + step * kBK);
            const uint32_t cs[2] = {G.col_lo, G.col_hi}, vs[2] = {G.val_lo, G.val_hi};
            if (half == 0) {                            // the group's first step: keep the columns for its second
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    out_col[i] = 4 * b_h + i < cnt ? (cs[i >> 1] >> (16 * (i & 1))) & 0xFFFFu : 0x10000u;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t t = out_col[i] - k_lo;   // >= 64 for 0x10000 (k_lo <= 65536 - 64) and for other steps' columns
                const uint32_t vbits = (vs[i >> 1] >> (16 * (i & 1))) & 0xFFFFu;
                brow[t < (uint32_t)kBK ? t : (uint32_t)kBK] = __builtin_bit_cast(_Float16, BF16 ? half_bits_to_bf16_bits(vbits) : (uint16_t)vbits);
            }
            if (b_h == 0)
                for (int i = kAhead; i < cnt; ++i) {    // rare: more than kAhead outliers in one group
                    const uint32_t c = load_u16_now(col_idx + first + i) - k_lo;
                    if (c < (uint32_t)kBK) {
                        const uint32_t vbits = load_u16_now(out_val + first + i);
                        brow[c] = __builtin_bit_cast(_Float16, BF16 ? half_bits_to_bf16_bits(vbits) : (uint16_t)vbits);
                    }
                }
        };

        // Prologue: records of groups 0 and 1, codes and outliers of groups 0 and 1; step 0 staged.
        GroupRegs<BITS> G0, G1;                         // even groups, odd groups
        const GroupRecord r0 = r_row[0], r1 = r_row[1];
        int first_c = r0.first, first_n = r1.first;     // current group, next group
        uint32_t sz_c = r0.scale_zero, sz_n = r1.scale_zero;
        issue_group(0, first_c, G0);
        issue_group(1, first_n, G1);
        stage(0, 0, G0, sz_c, first_c, first_n - first_c);
        __syncthreads();
        int wbuf = 1;                                   // weight buffer of step 2g + 1: (2g + 1) % 3

        // One group (two steps) per trip.  Entering trip g: step 2g is staged, Gcur is group g
        // and Gnxt group g + 1 (in flight, with the record of group g + 2).  As soon as Gcur's second
        // half is staged its registers are refilled with group g + 2, two steps before its first
        // use, so the two register sets swap roles from trip to trip and a set is never copied (a
        // copy would have to wait for loads that were only just issued).  The body has no branch
        // around a request: the compiler's count of loads in flight stays exact.
        // (The scheduling fences keep every request where it is written: left alone, the compiler moves
        // loads down towards their use, and then waits for them.)
        auto trip = [&](int g, GroupRegs<BITS> &Gcur, GroupRegs<BITS> &Gnxt) {
            stage(2 * g + 1, wbuf, Gcur, sz_c, first_c, first_n - first_c);   // second half of group g
            wbuf = wbuf == 2 ? 0 : wbuf + 1;
            __builtin_amdgcn_sched_barrier(0);
            const int first_nn = Gnxt.next_first;       // group g + 2
            const uint32_t sz_nn = Gnxt.next_scale_zero;
            issue_group(g + 2, first_nn, Gcur);
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            stage(2 * g + 2, wbuf, Gnxt, sz_n, first_n, first_nn - first_n);  // first half of group g + 1 (past the end: unused)
            wbuf = wbuf == 2 ? 0 : wbuf + 1;
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            first_c = first_n; sz_c = sz_n;
            first_n = first_nn; sz_n = sz_nn;
        };
        int g = 0;
        for (; g + 1 < gl; g += 2) {
            trip(g, G0, G1);
            trip(g + 1, G1, G0);
        }
        if (g < gl) trip(g, G0, G1);
        return;
    }

    if (wave >= kConsumers) {
        // ========================================= loaders =====================================
        // Four waves copy the X rows of every step from memory straight into LDS: a load with an
        // LDS destination writes lane l's 16 bytes at (wave-uniform base) + 16 l, so one instruction
        // fills eight consecutive 128-byte rows, lane l fetching the chunk that belongs at position
        // l % 8 of its row.  Step t + 2 is requested when barrier t - 1 has released its buffer;
        // before barrier t everything but those newest requests has arrived.
        // The step's base address is wave-uniform (advanced by scalar adds); a lane adds its row offset.
        constexpr int kInstr = BM / 8 / kLoaders;       // per wave and step
        const int lw = wave - kConsumers - kProducers, lr = lane >> 3;
        uint32_t row_off[kInstr];                       // bytes from the tile's first row and the step's first column
#pragma unroll
        for (int j = 0; j < kInstr; ++j) {
            const int r = 8 * (lw * kInstr + j) + lr;
            const int rc = m0 + r < M ? r : M - 1 - m0;
            row_off[j] = (uint32_t)rc * (uint32_t)K * 2u + 16u * (uint32_t)((lane & 7) ^ x_swizzle(r));
        }
        const char *tile = reinterpret_cast<const char *>(X + (size_t)m0 * K + k_first);
        typedef __attribute__((address_space(3))) unsigned char lds_byte;
        const uint32_t lds_x = (uint32_t)(uintptr_t)(lds_byte *)lds + (uint32_t)(lw * kInstr) * 1024u;   // LDS byte offset of the wave's first KB
        auto issue_x = [&](int step, int buf) {
            const char *src = tile + (size_t)step * (kBK * 2);
            const uint32_t dst = lds_x + (uint32_t)buf * (uint32_t)(kXBufHalves * 2);
#pragma unroll
            // Written out instead of __builtin_amdgcn_global_load_lds: with the scalar base and a 32-bit lane offset
            // the load needs no address arithmetic; the builtin forms a 64-bit address per lane and load, and the
            // whole GEMM measured 4.5 % slower with it (7B layer, M = 2048: 895 against 935 TFLOP/s on one machine).
            // m0 (the LDS base of the wave's 1 KB) is written here only and nothing else in a loader wave reads it (no
            // other LDS-destination load, no indexed register move, no message); the compiler does not accept m0 in
            // a clobber list (it warns that the register is reserved), so this is stated rather than declared.
            for (int j = 0; j < kInstr; ++j)
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                             :: "s"(dst + j * 1024u), "v"(row_off[j]), "s"(src) : "memory");
        };
        issue_x(0, 0);
        issue_x(1, 1);                                  // nk >= 2
        wait_vm<kInstr>();
        __builtin_amdgcn_s_barrier();                   // no fence: the explicit waits are the ordering
        int buf = 2;                                    // buffer of step t + 2
        for (int t = 0; t < nk; ++t) {
            issue_x(t + 2 < nk ? t + 2 : nk - 1, buf);  // past the end: the last step again, unused
            wait_vm<kInstr>();
            __builtin_amdgcn_s_barrier();
            buf = buf == 2 ? 0 : buf + 1;
        }
        wait_vm<0>();                                   // nothing may still be writing this block's LDS when it ends
        return;
    }

    // ========================================= consumers =======================================
    const int wm = wave / WN, wn = wave % WN;           // WM x WN waves, each 32 MSW rows by 32 NB columns
    if (wm >= WM) {                                     // a consumer wave without a sub-tile only keeps the barrier count
        for (int t = 0; t < 1 + nk; ++t) __syncthreads();
        return;
    }
    float16v acc[MSW][NB];
#pragma unroll
    for (int i = 0; i < MSW; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int fi = lane & 31, fk = lane >> 5;           // fragment row and k-block of this lane
    const _Float16 *b_frag = lds_w + (wn * (32 * NB) + fi) * kLd + 8 * fk;
    const _Float16 *a_frag[4];                          // per k-batch: the row's chunk 2s + fk, where the permutation puts it
#pragma unroll
    for (int s = 0; s < 4; ++s) a_frag[s] = lds + (wm * (32 * MSW) + fi) * kBK + 8 * ((2 * s + fk) ^ x_swizzle(fi));

    // Fragments of three k-batches (16 columns each): the one being multiplied and the two after
    // it.  With every wave of the block reading, a fragment takes longer to arrive than one batch
    // of MFMAs lasts, so it is requested two batches ahead.  Batch s of step t uses register set
    // (t + s) % 3 and LDS buffers t % 3: the loop is unrolled over three steps and all of that is
    // static.  Barrier t (step t + 1 is staged; steps up to t - 1 are read) comes after batch 1 of
    // step t, just in time for the request of step t + 1's first fragments.
    u32x4 fa[3][MSW], fb[3][NB];
    auto read_frags = [&](int buf, int s, int set) {
        const _Float16 *A = a_frag[s] + buf * kXBufHalves, *B = b_frag + buf * kWBufHalves;
#pragma unroll
        for (int i = 0; i < MSW; ++i) fa[set][i] = *reinterpret_cast<const u32x4 *>(A + i * 32 * kBK);
#pragma unroll
        for (int j = 0; j < NB; ++j) fb[set][j] = *reinterpret_cast<const u32x4 *>(B + j * 32 * kLd + 16 * s);
    };
    auto mfma_batch = [&](int set) {
#pragma unroll
        for (int i = 0; i < MSW; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
                if constexpr (BF16)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[set][i]),
                                                                        __builtin_bit_cast(bf16x8, fb[set][j]),
                                                                        acc[i][j], 0, 0, 0);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, fa[set][i]),
                                                                       __builtin_bit_cast(half8, fb[set][j]),
                                                                       acc[i][j], 0, 0, 0);
    };
    auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
    // One step whose number is p modulo 3.
    auto one_step = [&](auto phase) {
        constexpr int p = decltype(phase)::value, q = (p + 1) % 3;
        read_frags(p, 2, (p + 2) % 3);
        fence();
        mfma_batch(p);
        fence();
        read_frags(p, 3, p);                            // set (p + 3) % 3, free again
        fence();
        mfma_batch((p + 1) % 3);
        fence();
        __syncthreads();
        read_frags(q, 0, (p + 1) % 3);                  // batch 0 of the next step: set (q + 0) % 3
        fence();
        mfma_batch((p + 2) % 3);
        fence();
        read_frags(q, 1, (p + 2) % 3);
        fence();
        mfma_batch(p);
        fence();
    };

    __syncthreads();                                    // barrier -1: step 0 is staged
    read_frags(0, 0, 0);
    read_frags(0, 1, 1);
    int step = 0;
    for (; step + 3 <= nk; step += 3) {
        one_step(std::integral_constant<int, 0>{});
        one_step(std::integral_constant<int, 1>{});
        one_step(std::integral_constant<int, 2>{});
    }
    if (step < nk) one_step(std::integral_constant<int, 0>{});
    if (step + 1 < nk) one_step(std::integral_constant<int, 1>{});

    // D layout of the 32x32 tile: column = lane % 32, row = 8*(v/4) + 4*(lane/32) + v%4.
#pragma unroll
    for (int i = 0; i < MSW; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int n = n0 + wn * (32 * NB) + j * 32 + fi;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * (32 * MSW) + i * 32 + 8 * (v >> 2) + 4 * fk + (v & 3);
                if (m < M && n < N) {
                    if (partial) partial[((size_t)split * M + m) * N + n] = acc[i][j][v];
                    else reinterpret_cast<act_t *>(Y)[(size_t)m * N + n] = (act_t)acc[i][j][v];
                }
            }
        }
}

// Y = sum over the splits of partial[s], added in the order of s (so the result does not depend on
// which block finished first), rounded to FP16 once.
template <typename act_t>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partial, act_t *__restrict__ Y,
                                                            size_t count, int splits)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float sum = partial[i];
    for (int s = 1; s < splits; ++s) sum += partial[(size_t)s * count + i];
    Y[i] = (act_t)sum;
}

// How many ways K is split for a launch of `tiles` tiles over rows of `gpr` groups: as many as keep
// the block count within the CU count, at least two groups each, at most kMaxSplits.
// kCUs is the compute-unit count of the MI355X, which the scratch size reported by gwq_layout (a pure host
// call) is based on; a launch plans with the current device's count, never beyond kCUs.
constexpr int kMaxSplits = 8, kSplitBelowTiles = 160, kCUs = 256;
size_t record_bytes(int64_t N, int64_t K) { return ((size_t)(N * (K / kGroup + 1)) * sizeof(GroupRecord) + 255) / 256 * 256; }
int launch_cus()
{
    const int n = device_cus();
    return n < kCUs ? n : kCUs;
}
int choose_splits(int tiles, int gpr, int cus)
{
    if (tiles >= kSplitBelowTiles) return 1;
    int s = cus / tiles;
    s = s < kMaxSplits ? s : kMaxSplits;
    s = s < gpr / 2 ? s : gpr / 2;
    return s < 1 ? 1 : s;
}

struct SplitPlan {
    int splits, split_groups;
};
SplitPlan plan_split(int tiles, int gpr, bool have_scratch, int cus)
{
    int splits = have_scratch ? choose_splits(tiles, gpr, cus) : 1;
    const int split_groups = (gpr + splits - 1) / splits;
    splits = (gpr + split_groups - 1) / split_groups;   // no empty split
    return SplitPlan{splits, split_groups};
}

// Rows of Y per block for a launch the caller did not fix the shape of.  Beyond M = 512 the 256-row
// tile, which has the most MFMA work per staged weight.  Below, the shape with the smallest expected
// duration under a linear model fitted to measurements (288 launches: 11 matrices from 2048 x 2048 to
// 8192 x 8192 and 4096 x 11008, M = 17 .. 512, every shape; it picks the measured best or a shape
// within 3 % of it on all but the 2048 x 2048 matrix): a launch takes, in microseconds,
//   rounds * (block + steps * step)  +  (K split ? 2.8 + 0.47 per MB of FP32 partial sums : 0)
// with rounds = ceil(blocks / 256 CUs), steps = K-steps of one block, and per shape the cost of a step
// (what its LDS traffic takes) and of a block's start and end.  Small tiles win where M leaves the
// larger ones mostly empty, or where they avoid the split of K and its second pass; large tiles win
// once the chip is full, since each stages the same weights for more rows.
struct ShapeCost {
    int rows;
    float step_us, block_us;
};
constexpr ShapeCost kShapeCost[4] = {{32, 0.42f, 0.9f}, {64, 0.49f, 0.45f}, {128, 0.60f, 1.6f}, {256, 0.87f, 2.2f}};
int choose_rows(int M, int N, int K, bool have_scratch)
{
    if (M > 512) return 256;
    const int gpr = K / kGroup, tiles_n = (N + kBN - 1) / kBN, cus = launch_cus();
    int best = 256;
    float best_us = 0.f;
    for (const ShapeCost &c : kShapeCost) {
        if (c.rows > 32 && c.rows >= 2 * M) continue;   // a tile at most half full: the next smaller holds M too
        const int tiles = (M + c.rows - 1) / c.rows * tiles_n;
        const SplitPlan sp = plan_split(tiles, gpr, have_scratch, cus);
        const int rounds = (tiles * sp.splits + cus - 1) / cus;
        float us = rounds * (c.block_us + 2 * sp.split_groups * c.step_us);
        if (sp.splits > 1) us += 2.8f + 0.47f * (4e-6f * sp.splits * M * N);
        if (best_us == 0.f || us < best_us) best = c.rows, best_us = us;
    }
    return best;
}

template <int BITS, int MSW, int WN, int WM, bool FINE, bool BF16>
hipError_t launch_ms(const gwq_packed &P, const void *X, int M, void *Y, const GroupRecord *rec, float *partial,
                     size_t partial_bytes, hipStream_t st, PlanText *describe)
{
    constexpr int BM = 32 * MSW * WM;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (P.N + kBN - 1) / kBN;
    const int gpr = P.K / kGroup;
    const SplitPlan sp = plan_split(tiles_m * tiles_n, gpr, partial != nullptr, launch_cus());
    int splits = sp.splits, split_groups = sp.split_groups;
    if (splits > 1 && (size_t)splits * M * P.N * sizeof(float) > partial_bytes) splits = 1, split_groups = gpr;
    if (splits == 1) partial = nullptr;
    const size_t lds = ((size_t)3 * BM * kBK + (size_t)3 * kBN * kLd) * sizeof(_Float16);
    if (describe) {
        snprintf(describe->text, sizeof(describe->text), "gemm_kernel<%d,%d,%d,%d,%s,%s> tile %dx%d grid %d block %d lds %zu k_splits %d",
                 BITS, MSW, WN, WM, FINE ? "true" : "false", BF16 ? "true" : "false", BM, kBN, tiles_m * tiles_n * splits, kThreads, lds, splits);
        return hipSuccess;
    }
    static std::atomic<uint32_t> lds_allowed{0};        // per instantiation
    {
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&gemm_kernel<BITS, MSW, WN, WM, FINE, BF16>), (int)lds, lds_allowed);
        if (e != hipSuccess) return e;
    }
    // The half-slot pairs of a layer with small groups follow the records.
    const uint32_t *fine = reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(rec) + record_bytes(P.N, P.K));
    gemm_kernel<BITS, MSW, WN, WM, FINE, BF16><<<tiles_m * tiles_n * splits, kThreads, lds, st>>>(
        P.qweight, P.col_idx, P.out_val, rec, fine, static_cast<const _Float16 *>(X),
        static_cast<_Float16 *>(Y), partial, split_groups, P.N, P.K, M, tiles_m, tiles_n,
        P.n_outliers > 0 ? (int)P.n_outliers - 1 : 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || splits == 1) return e;
    const size_t count = (size_t)M * P.N;
    if (BF16) splitk_reduce_kernel<__bf16><<<(unsigned)((count + 255) / 256), 256, 0, st>>>(partial, static_cast<__bf16 *>(Y), count, splits);
    else splitk_reduce_kernel<_Float16><<<(unsigned)((count + 255) / 256), 256, 0, st>>>(partial, static_cast<_Float16 *>(Y), count, splits);
    return hipGetLastError();
}

}  // namespace

size_t gemm_index_bytes(int64_t N, int64_t K, int group)
{
    return record_bytes(N, K) + (group < kGroup ? ((size_t)N * (K / 16) * 4 + 255) / 256 * 256 : 0);
}

// Scratch for the FP32 partial sums of a K-split launch with up to M_max rows.  Splitting stops
// where splits x tiles reaches the CU count, so splits * M * N never exceeds that many tiles' worth.
size_t gemm_scratch_bytes(int64_t N, int64_t M_max)
{
    if (M_max <= 16) return 0;
    const size_t by_rows = (size_t)kMaxSplits * (size_t)M_max * (size_t)N * sizeof(float);
    const size_t by_tiles = (size_t)kCUs * 256 * kBN * sizeof(float);
    return by_rows < by_tiles ? by_rows : by_tiles;
}

hipError_t launch_gemm_index(const gwq_packed &P, void *workspace, hipStream_t st)
{
    // 4364 * 15 = 65460 and 9352 * 7 = 65464: the last scales on the FP16 grid that keep s * (q - z) finite.
    const uint32_t scale_cap = P.bits == 4 ? 0x6C43u : 0x7091u;
    if (P.group == kGroup) {
        group_index_kernel<<<(P.N + 3) / 4, 256, 0, st>>>(P.row_ptr, P.col_idx, P.scales, P.zeros, P.N, P.K / kGroup,
                                                         scale_cap, static_cast<GroupRecord *>(workspace));
        return hipGetLastError();
    }
    // Small groups: the records carry the outlier index alone (scale and zero point come from the pairs behind them).
    group_index_kernel<<<(P.N + 3) / 4, 256, 0, st>>>(P.row_ptr, P.col_idx, nullptr, nullptr, P.N, P.K / kGroup,
                                                     scale_cap, static_cast<GroupRecord *>(workspace));
    const size_t count = (size_t)P.N * (P.K / 16);
    fine_index_kernel<<<(unsigned)((count + 255) / 256), 256, 0, st>>>(
        P.scales, P.zeros, count, P.K, P.group, scale_cap,
        reinterpret_cast<uint32_t *>(static_cast<char *>(workspace) + record_bytes(P.N, P.K)));
    return hipGetLastError();
}

hipError_t launch_gemm(const gwq_packed &P, const void *X, int M, void *Y, const void *index, void *scratch,
                       size_t scratch_bytes, int ms_override, hipStream_t st, PlanText *describe, bool bf16)
{
    if (bf16 && P.group != kGroup) return hipErrorNotSupported;
    const GroupRecord *rec = static_cast<const GroupRecord *>(index);
    float *part = static_cast<float *>(scratch);
    // Rows per tile (the override is in rows): 256 (consumer waves 4 x 2, 64 x 64 each), 128 (4 x 2, 32 x 64
    // each), 64 (2 x 4, 32 x 32 each) or 32 (1 x 4, four consumer waves idle).  In the small shapes the
    // weights a block stages are read from LDS by two rows of waves, or one, instead of four, and the
    // LDS is what bounds a step.
    const int rows = ms_override ? ms_override : choose_rows(M, (int)P.N, (int)P.K, part != nullptr);
    const int shape = rows == 256 ? 2 : rows == 128 ? 1 : rows == 64 ? 0 : 3;
#define GWQ_GEMM(B, F, A) \
    return shape == 2   ? launch_ms<B, 2, 2, 4, F, A>(P, X, M, Y, rec, part, scratch_bytes, st, describe) \
           : shape == 1 ? launch_ms<B, 1, 2, 4, F, A>(P, X, M, Y, rec, part, scratch_bytes, st, describe) \
           : shape == 0 ? launch_ms<B, 1, 4, 2, F, A>(P, X, M, Y, rec, part, scratch_bytes, st, describe) \
                        : launch_ms<B, 1, 4, 1, F, A>(P, X, M, Y, rec, part, scratch_bytes, st, describe)
    if (bf16) {
        if (P.bits == 4) GWQ_GEMM(4, false, true);
        GWQ_GEMM(3, false, true);
    }
    if (P.group == kGroup) {
        if (P.bits == 4) GWQ_GEMM(4, false, false);
        GWQ_GEMM(3, false, false);
    }
    if (P.bits == 4) GWQ_GEMM(4, true, false);
    GWQ_GEMM(3, true, false);
#undef GWQ_GEMM
}

}  // namespace gwq
