// gwq_linear for M <= 16 on gfx950: a bandwidth-bound fused dequantise-and-multiply.
//
//   Y[m][n] = sum_g s[n][g] * sum_{k in g} X[m][k] * (q[n][k] - z[n][g])   (Sec. 3.2, Eq. 10)
//           + sum_{j in CSR row n} out_val[j] * X[m][col_idx[j]]            (the FP16 outliers)
//
// Mapping.  A block owns 16 output channels; its waves split K by whole groups of 128.  A wave
// feeds v_mfma_f32_16x16x32_f16 with X as the 16 x 32 operand (rows m) and the dequantised codes
// as the 32 x 16 operand (columns n): lane (r = lane % 16, b = lane / 16) owns slot b of each
// group of channel n0 + r, i.e. 32 consecutive codes = one 16-byte load (at 3 bits: the slot's
// three words plus the word behind them, which for slot 3 is the tail word all four slots share;
// the other lanes of the channel fetch it from that lane).  Codes become the exact FP16 integers q - z with one
// AND-OR and one packed add per pair; the group scale is applied to the four FP32 results per
// lane after the group's four MFMAs.  The lanes then add their channel's outliers, the waves'
// partial sums meet in LDS in a fixed order, and one thread per output rounds to FP16 and stores.
// No atomics, no second pass: results are run-to-run identical.
//
// What bounds it.  A matrix is only a few microseconds of HBM time, and at that scale these matter
// more than arithmetic:
//   * every byte must be requested early: loads are unconditional (clamped addresses), issued
//     before anything consumes them, and nothing is converted or combined right behind a load
//     (loads retire in order, so waiting for a young one waits for all older ones);
//   * the address unit of a CU handles a scattered or sub-dword load lane by lane (about 64 cycles
//     per instruction against 16 for a coalesced 16-byte load), so everything except the code
//     stream is fetched with block-wide coalesced 16-byte loads into LDS: the block's scales and
//     zero points (contiguous for 16 consecutive channels), X, and the block's contiguous CSR
//     segment (kept in LDS as one word per entry, column and value together), whose bounds come
//     in through the scalar cache;
//   * the instructions a wave issues: wave-uniform values are kept in scalar registers, offsets
//     are compile-time constants, and nothing in the multiply is predicated.
// Three kernels: the lean one for M <= 8 with all of X in LDS, the streaming one for M <= 16 and K <= 4096 where a
// block has several tiles (X in registers, its transpose in LDS), the wide one for everything else (X through LDS
// in phases of K).
#include <stdio.h>

#include <type_traits>

#include "gwq_dequant.h"
#include "gwq_internal.h"

namespace gwq {
namespace {

typedef float float4v __attribute__((ext_vector_type(4)));

// Optional build (-DGWQ_STAMP, a separate library: see build.py): wave 0 of every block records the
// shader clock at the kernel's milestones, read back with gwq_debug_read_stamps.  Not part of the product.
#ifdef GWQ_STAMP
constexpr int kStampSlots = 16, kStampBlocks = 2048;
__device__ unsigned long long g_stamps[kStampBlocks * kStampSlots];
#define GWQ_STAMP_AT(i) \
    do { \
        if (tid == 0) { \
            const unsigned blk = (blockIdx.y * gridDim.x + blockIdx.x) % kStampBlocks; \
            g_stamps[blk * kStampSlots + (i)] = (i) == 0 ? wall_clock64() : clock64(); \
        } \
    } while (0)
// The same for the lean kernel, held in scalar registers until the end so that no store disturbs the run:
// slot 0 of a block's record is the wall clock, slots 1 .. from its first wave, 8 + those of its last wave.
#define GWQ_TS_DECL unsigned long long ts_[8] = {}; const unsigned long long ts_wall_ = wall_clock64()
#define GWQ_TS(i) ts_[i] = clock64()
#define GWQ_TS_FLUSH(first, last) \
    do { \
        if ((tid & 63) == 0 && ((first) || (last))) { \
            const unsigned blk = (blockIdx.y * gridDim.x + blockIdx.x) % kStampBlocks; \
            if (first) g_stamps[blk * kStampSlots] = ts_wall_; \
            for (int i_ = 0; i_ < 7; ++i_) g_stamps[blk * kStampSlots + ((last) && !(first) ? 8 : 1) + i_] = ts_[i_]; \
        } \
    } while (0)
#else
#define GWQ_STAMP_AT(i) do { } while (0)
#define GWQ_TS_DECL do { } while (0)
#define GWQ_TS(i) do { } while (0)
#define GWQ_TS_FLUSH(first, last) do { } while (0)
#endif


// Sixteen bytes per lane from memory straight into LDS, no registers in between: lane l's bytes land at LDS byte
// `lds_byte` + 16 l (wave-uniform, in m0 while the instruction issues; the old m0 is put back), read from `base` +
// the lane's 32-bit byte offset.  The load counts in vmcnt like any other but the compiler does not see it: whoever
// reads the LDS bytes waits with wait_all_loads() first.  (Extra loads in flight only make the compiler's own
// waits, which count from the youngest load backwards, wait for more than they need.)
__device__ inline void load_to_lds_16(uint32_t lds_byte, uint32_t lane_byte_offset, const void *base)
{
    uint32_t keep;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep) : "s"(lds_byte), "v"(lane_byte_offset), "s"(base) : "memory");
}
__device__ inline void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ inline const uint32_t *at_byte(const uint32_t *base, uint32_t byte_off)
{
    return reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(base) + byte_off);
}

// Eight CSR entries as staged in LDS: one word per entry, column in the low half and FP16 value in
// the high half, so that an entry costs its reader one LDS read instead of two.
__device__ inline void store_entries(u32x4 *dst, u32x4 col, u32x4 val)
{
    dst[0] = u32x4{(col.x & 0xFFFFu) | val.x << 16, col.x >> 16 | (val.x & 0xFFFF0000u),
                   (col.y & 0xFFFFu) | val.y << 16, col.y >> 16 | (val.y & 0xFFFF0000u)};
    dst[1] = u32x4{(col.z & 0xFFFFu) | val.z << 16, col.z >> 16 | (val.z & 0xFFFF0000u),
                   (col.w & 0xFFFFu) | val.w << 16, col.w >> 16 | (val.w & 0xFFFF0000u)};
}

// Registers of one slot (32 codes) as loaded from memory; offsets are bytes from qweight.
template <int BITS> struct Slot;
template <> struct Slot<4> {
    uint4 w;
    __device__ inline void load(const uint32_t *q, uint32_t group_off, int b)
    {
        w = *reinterpret_cast<const uint4 *>(at_byte(q, group_off + 16 * b));
    }
    // The same for a group that may lie past the last one: the read stops at `end` (bytes of qweight).
    __device__ inline void load_clamped(const uint32_t *q, uint32_t group_off, int b, uint32_t end)
    {
        const uint32_t off = group_off + 16 * b;
        w = *reinterpret_cast<const uint4 *>(at_byte(q, off < end - 16 ? off : end - 16));
    }
    // An empty statement that reads and "rewrites" the registers: the compiler waits for their load here and not later.
    __device__ inline void claim() { asm volatile("" : "+v"(w.x), "+v"(w.y), "+v"(w.z), "+v"(w.w)); }
    __device__ inline void decode(uint32_t z, int /*b*/, const DecodeConsts &d, u32x4 f[4], int /*tail_lane4*/) const
    {
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
        decode_slot4(ww, z, d, f);
    }
    // Zero points of the slot's two halves (groups of 16).
    __device__ inline void decode_halves(uint32_t z_lo, uint32_t z_hi, int /*b*/, const DecodeConsts &d, u32x4 f[4],
                                         int /*tail_lane4*/) const
    {
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
        decode_slot4_halves(ww, z_lo, z_hi, d, f);
    }
    __device__ inline void decode_bf16(int /*b*/, const DecodeConstsBf16 &d, u32x4 f[4], int /*tail_lane4*/) const
    {
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
        decode_slot4_bf16(ww, d, f);
    }
};
// 3-bit: a group is 13 words, slot b owns words 3b .. 3b+2 and two codes of word 12 (the tail).  One
// 16-byte load at byte 12b (4-byte aligned; gfx950 global memory takes that) brings a lane its three
// words and one more: for slot 3 that fourth word is the tail, which the other three lanes of the
// channel then fetch from it with a cross-lane read - one memory instruction per group instead of two.
template <> struct Slot<3> {
    uint32_t w[3], fourth;
    __device__ inline void load(const uint32_t *q, uint32_t group_off, int b)
    {
        const U128a4 v = *reinterpret_cast<const U128a4 *>(at_byte(q, group_off + 12 * b));
        w[0] = v.x; w[1] = v.y; w[2] = v.z; fourth = v.w;
    }
    __device__ inline void load_clamped(const uint32_t *q, uint32_t group_off, int b, uint32_t end)
    {
        const uint32_t off = group_off + 12 * b;
        const U128a4 v = *reinterpret_cast<const U128a4 *>(at_byte(q, off < end - 16 ? off : end - 16));
        w[0] = v.x; w[1] = v.y; w[2] = v.z; fourth = v.w;
    }
    __device__ inline void claim() { asm volatile("" : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(fourth)); }
    // tail_lane4 = 4 * (lane | 48): the byte index of the lane that holds slot 3 of the same channel.
    __device__ inline void decode(uint32_t z, int b, const DecodeConsts &d, u32x4 f[4], int tail_lane4) const
    {
        const uint32_t tail = (uint32_t)__builtin_amdgcn_ds_bpermute(tail_lane4, (int)fourth);
        decode_slot3(w, tail >> (3 * b), z, d, f);
    }
    __device__ inline void decode_halves(uint32_t z_lo, uint32_t z_hi, int b, const DecodeConsts &d, u32x4 f[4],
                                         int tail_lane4) const
    {
        const uint32_t tail = (uint32_t)__builtin_amdgcn_ds_bpermute(tail_lane4, (int)fourth);
        decode_slot3_halves(w, tail >> (3 * b), z_lo, z_hi, d, f);
    }
    __device__ inline void decode_bf16(int b, const DecodeConstsBf16 &d, u32x4 f[4], int tail_lane4) const
    {
        const uint32_t tail = (uint32_t)__builtin_amdgcn_ds_bpermute(tail_lane4, (int)fourth);
        decode_slot3_bf16(w, tail >> (3 * b), d, f);
    }
};

constexpr int kPre = 4;        // outlier entries a lane handles without a loop
constexpr int kXPad = 8;       // halves between the rows of X in LDS: the 16 rows of an MFMA operand hit different banks

// One layer of a launch, and the launch: up to kMaxBatch layers, layer i = blockIdx.y.  Passed by
// value (kernel argument segment) and read through the scalar cache: the descriptor's offset follows
// from blockIdx.y alone, so one scalar load separates the start of a wave from its first vector load.
struct DecodeProblem {
    const uint32_t *qweight;
    const uint16_t *scales;
    const uint8_t *zeros;
    const int32_t *row_ptr;
    const uint16_t *col_idx;
    const uint16_t *out_val;
    const _Float16 *X;
    _Float16 *Y;
    int N, K, sc_last_vec, zp_last_vec, csr_last_vec;
    int group_shift;            // log2 of the layer's group size: 7, or 4 .. 6 (the wide kernel alone takes those)
};
struct DecodeBatch {
    int M, nwaves;
    int wide_window = 8;        // wide kernel: CSR entries staged per thread, 8, or 4 where the LDS is short
    DecodeProblem p[kMaxBatch];
};

// ---- M <= 4 with X[M][K] in LDS: the lean kernel ------------------------------------------------
//
// A kernel this short is bounded as much by the instructions a wave issues as by the bytes it moves,
// so this one is straight-line code with compile-time offsets:
//   * wave w owns exactly the U groups [wU, wU + U) of the block's 16 channels (the launcher starts
//     ceil(gpr / U) waves); its index and everything derived from it live in scalar registers;
//   * groups at or beyond gpr exist only in the last wave.  Their codes are whatever follows in
//     memory (the next channel; the address is only kept from passing the end of qweight) and
//     they meet zeros in the LDS copy of X, whose rows are padded to waves * U groups.  Their
//     scale and zero point are whatever follows in LDS, at most U - 1 places on, and that must
//     be a finite scale and a zero point below 2^bits: a NaN scale, or a byte from 192 to 207 as
//     a 3-bit zero point (it carries the decoder's constant -(16 + z) into the NaN patterns),
//     would turn the exact zero of such a group into a NaN.  What follows is the next channel's
//     (fine), for channel 15 the zero points read as scales (tiny finite numbers) or the spare
//     slot, and for the last channel of a ragged N the padding of the caller's buffers; the
//     spare slot and that padding are replaced by zeros when the arrays are staged;
//   * a launch over several layers has as many waves as its longest rows need; the surplus waves of
//     a shorter layer repeat wave 0's work and drop the result.
//
// Dynamic LDS, in this order: X [MS][k_pad] halves | scales [16][gpr] halves | zero points [16][gpr]
// bytes | 16 spare bytes | CSR entries (column | value << 16), blockDim * 8 + 8 zero entries |
// partial sums [waves][MS][64] floats.  blockDim >= 3 gpr holds by construction (64 ceil(gpr / U)
// threads, U <= 16), so one 16-byte vector per thread stages all scales and zero points.
//
// MODE 0 stores Y.  MODE 1 and 2 are the two halves of the gated pair H = silu(X Wg^T) * (X Wu^T): the
// first run keeps its FP32 sums in LDS (behind the partial sums), the second combines them with its own
// and stores H, so the pair costs one launch and never writes the two products.
__device__ inline float silu(float x)
{
    // x * sigmoid(x); exp2 and the reciprocal are the hardware's approximations (about 1 ulp each)
    return x * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.44269504088896340736f * x));
}

//
// PAIR (five to eight rows, plain products): two neighbouring tiles per block, one set of waves each, one copy of X
// between them; each set stages every second row of X and half the CSR window.  What a tile costs beyond four rows
// is mostly its copy of X, read from L2 by every block.
// FINE: groups below 128.  The staged metadata is [16][spr] (up to three vectors per thread); a lane takes scale and
// zero point per half slot, with the indices of a group at or beyond gpr clamped into the row and its scales masked,
// and multiplies FP16 operands s * (q - z), as the wide kernel does for such layers.
// BF16: X and Y are bfloat16; operands 128 + q and a second set of MFMAs against ones, as in the wide kernel.
template <int BITS, int U, int MS, int MODE, bool FINE = false, bool BF16 = false, bool PAIR = false>
__device__ __forceinline__ void decode_small_body(const DecodeBatch &batch, const int layer)
{
    static_assert(!PAIR || (MODE == 0 && !FINE && !BF16 && MS > 4), "paired tiles: plain products of more than four rows");
    static_assert(!FINE || MODE == 0, "gated pairs: groups of 128 only");
    static_assert(!BF16 || (MODE == 0 && !FINE), "bfloat16 activations: plain products with groups of 128 only");
    typedef std::conditional_t<BF16, __bf16, _Float16> act_t;          // X and Y; both 16 bits wide
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const DecodeProblem &pr = batch.p[layer];
    const int N = pr.N, K = pr.K;
    const uint32_t *__restrict__ qweight = pr.qweight;
    const uint16_t *__restrict__ scales = pr.scales;
    const uint8_t *__restrict__ zeros = pr.zeros;
    const int32_t *__restrict__ row_ptr = pr.row_ptr;
    const uint16_t *__restrict__ col_idx = pr.col_idx;
    const uint16_t *__restrict__ out_val = pr.out_val;
    const act_t *__restrict__ X = reinterpret_cast<const act_t *>(pr.X);
    act_t *__restrict__ Y = reinterpret_cast<act_t *>(pr.Y);
    const int sc_last_vec = pr.sc_last_vec, zp_last_vec = pr.zp_last_vec, csr_last_vec = pr.csr_last_vec;
    const int shift = FINE ? pr.group_shift : 7;
    // The whole descriptor is requested in one go and only then looked at (the empty statement
    // keeps the compiler from moving the other loads behind the branch on N).
    asm volatile("" ::"s"(qweight), "s"(scales), "s"(zeros), "s"(row_ptr), "s"(col_idx), "s"(out_val), "s"(X), "s"(Y),
                 "s"(K), "s"(sc_last_vec), "s"(zp_last_vec), "s"(csr_last_vec), "s"(shift));
    if ((int)blockIdx.x * (PAIR ? 32 : 16) >= N) return;    // the grid is as wide as the largest layer

    // PAIR: the block's waves form two sets that work on two neighbouring 16-channel tiles with one copy of X
    // between them (each set stages every second row of it): half the reads of X per tile, which is what rows
    // five to eight cost over fewer.  Below, tid, wave, nwaves and nthreads are those of the set; everything
    // per tile in LDS exists once per set.  A set whose tile lies beyond N works on the last tile and stores nothing.
    const int lane = threadIdx.x & 63;
    const int block_wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int nwaves = PAIR ? batch.nwaves / 2 : batch.nwaves, nthreads = nwaves * 64;
    const int set = PAIR ? block_wave / nwaves : 0;
    const int wave = block_wave - set * nwaves;
    const int tid = (int)threadIdx.x - set * nthreads;
    const int tile = PAIR ? 2 * (int)blockIdx.x + set : (int)blockIdx.x;
    const bool tile_live = !PAIR || tile * 16 < N;
    const int block = tile_live ? tile : (N - 1) / 16;
    GWQ_TS_DECL;
    GWQ_TS(0);                                          // descriptor has arrived
    const int r = lane & 15, b = lane >> 4;
    const int tail_lane4 = 4 * (lane | 48);             // where the 3-bit tail word of this lane's channel arrives
    const int gpr = K / kGroup;
    const int spr = K >> shift;                         // scale / zero-point pairs per channel
    const int my_waves = (gpr + U - 1) / U;             // waves of this layer that own groups
    const bool active = wave < my_waves;
    const int g_begin = active ? wave * U : 0;
    const int k_pad = my_waves * U * kGroup + kXPad;    // row stride of the LDS copy of X
    const int row0 = block * 16;
    const int n = row0 + r;
    const int n_c = n < N ? n : N - 1;                  // clamped channel: its results are not stored

    act_t *xs = reinterpret_cast<act_t *>(lds_raw);
    // Staged CSR entries: eight per thread; in a pair four (the first half of the set's threads bring them), which
    // is what lets two blocks share a CU at eight rows and K = 4096.
    const int window = PAIR ? 4 * nthreads : 8 * nthreads;
    const uint32_t set_bytes = PAIR ? 48u * spr + 16u + 4u * window + 32u + (uint32_t)nwaves * MS * 64u : 0u;
    const uint32_t sc_off = (uint32_t)MS * k_pad * 2 + (uint32_t)set * set_bytes;
    const uint32_t zp_off = sc_off + 32 * spr;
    const uint32_t spare_off = zp_off + 16 * spr;
    const uint32_t ent_off = spare_off + 16;
    const uint32_t red_off = ent_off + 4 * window + 32;
    float *red = reinterpret_cast<float *>(lds_raw + red_off);

    // CSR bounds of the block and of this lane's channel.  The block's bounds are read through a pointer to
    // constant memory (nothing in the launch writes row_ptr): with a wave-uniform index that is a scalar
    // load, which nobody waits for until the segment is requested, behind the code stream.  (Through the plain
    // pointer the compiler issues a vector load and waits for it on the spot to make the value uniform -
    // a whole memory round trip before the first code is requested.)
    const int last_row = row0 + 16 < N ? row0 + 16 : N;
    const __attribute__((address_space(4))) int32_t *row_ptr_k =
        (const __attribute__((address_space(4))) int32_t *)(uintptr_t)row_ptr;
    const int e_begin = row_ptr_k[row0], e_end = row_ptr_k[last_row];
    const int rp0 = row_ptr[n_c], rp1 = row_ptr[n_c + 1];

    // Staging loads, all 16-byte and coalesced.  (1) X: each wave brings the columns of its own
    // groups; vectors beyond K are loaded from column 0 and replaced by zeros when stored.
    constexpr int kQ = U / 4;                           // 64-vector rounds covering U groups
    constexpr int kXRows = PAIR ? (MS + 1) / 2 : MS;    // rows of X a wave stages: all, or every second one from `set`
    u32x4 xstage[kXRows * kQ];
#pragma unroll
    for (int ei = 0; ei < kXRows; ++ei)
#pragma unroll
        for (int i = 0; i < kQ; ++i) {
            const int e = PAIR ? (2 * ei + set < MS ? 2 * ei + set : 0) : ei;
            const int kv = g_begin * (kGroup / 8) + lane + 64 * i;
            xstage[ei * kQ + i] = reinterpret_cast<const u32x4 *>(X)[e * (K / 8) + (kv < K / 8 ? kv : 0)];
        }
    // (2) The block's scales (32 gpr bytes) and zero points (16 gpr bytes), contiguous in memory for
    // 16 consecutive channels: thread t < 2 gpr takes a scales vector, the next gpr threads a
    // zero-point vector, any further thread re-reads vector 0 (and stores zeros into the spare slot).
    // The LDS copies of the two arrays are adjacent, so thread t stores to vector t of that range
    // (the spare slot follows at vector 3 gpr).
    u32x4 meta;
    int meta_valid;                                     // bytes of `meta` that lie inside the array
    u32x4 meta_fine[FINE ? 3 : 1];                      // small groups: vectors tid, tid + blockDim, tid + 2 blockDim of 3 spr
    if constexpr (FINE) {
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int t = tid + i * nthreads;
            const bool is_zp = t >= 2 * spr;
            const int u_sc = block * 2 * spr + t, u_zp = block * spr + (t - 2 * spr);
            const int v_sc = u_sc < sc_last_vec ? u_sc : sc_last_vec;
            const int v_zp = u_zp < zp_last_vec ? u_zp : zp_last_vec;
            const u32x4 *src = is_zp ? reinterpret_cast<const u32x4 *>(zeros) : reinterpret_cast<const u32x4 *>(scales);
            meta_fine[i] = src[is_zp ? (t < 3 * spr ? v_zp : 0) : v_sc];
        }
        meta = meta_fine[0];
        meta_valid = 16;
    } else {
        const bool is_sc = tid < 2 * gpr, is_zp = !is_sc && tid < 3 * gpr;
        const int u_sc = block * 2 * gpr + tid, u_zp = block * gpr + (tid - 2 * gpr);
        const int v_sc = u_sc < sc_last_vec ? u_sc : sc_last_vec;
        const int v_zp = u_zp < zp_last_vec ? u_zp : zp_last_vec;
        const int v = is_sc ? v_sc : is_zp ? v_zp : 0;
        const u32x4 *src = is_zp ? reinterpret_cast<const u32x4 *>(zeros) : reinterpret_cast<const u32x4 *>(scales);
        meta = src[v];
        meta_valid = is_sc ? 2 * N * gpr - 16 * u_sc : is_zp ? N * gpr - 16 * u_zp : 0;
    }
    const uint32_t meta_dst = sc_off + 16 * (tid < 3 * gpr ? tid : 3 * gpr);

    // Every wave has queued its staging loads before any wave queues code: the memory pipe of the
    // CU serves requests in order, and the first barrier below waits for the slowest staging load.
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);

    // The code stream.  The first kAhead groups are requested here, each further one while the
    // group kAhead places before it is being multiplied: a wave that had all its requests queued
    // at once would sit in the queue while its early groups wait in registers.
    constexpr uint32_t group_bytes = words_per_group(BITS) * 4;
    constexpr int kAhead = U < 4 ? U : 4;
    const uint32_t code_off = ((uint32_t)n_c * gpr + g_begin) * group_bytes;
    const uint32_t code_end = (uint32_t)N * gpr * group_bytes;
    Slot<BITS> slot[U];
#pragma unroll
    for (int u = 0; u < kAhead; ++u) slot[u].load_clamped(qweight, code_off + u * group_bytes, b, code_end);

    // Nothing that consumes a load may be scheduled above this point.
    __builtin_amdgcn_sched_barrier(0);
    GWQ_TS(1);                                          // staging and the first codes requested
    const DecodeConsts dc(BITS);
#pragma unroll
    for (int ei = 0; ei < kXRows; ++ei)
#pragma unroll
        for (int i = 0; i < kQ; ++i) {
            const int e = PAIR ? (2 * ei + set < MS ? 2 * ei + set : 0) : ei;   // past the last row: row 0 again, same bytes
            const int kv = g_begin * (kGroup / 8) + lane + 64 * i;
            reinterpret_cast<u32x4 *>(xs)[e * (k_pad / 8) + kv] =
                kv < K / 8 ? xstage[ei * kQ + i] : u32x4{0u, 0u, 0u, 0u};
        }
    // Bytes beyond the end of scales or zeros (the last block of a ragged N, and the spare slot) are
    // stored as zeros: the groups at or beyond gpr of the last channel and of channel 15 read them.
    if constexpr (FINE) {
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int t = tid + i * nthreads;
            if (t < 3 * spr) *reinterpret_cast<u32x4 *>(lds_raw + sc_off + 16 * t) = meta_fine[i];
        }
    } else {
        if (meta_valid < 16) {
            uint32_t *m = reinterpret_cast<uint32_t *>(&meta);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int nb = meta_valid - 4 * i;
                m[i] &= nb >= 4 ? ~0u : nb <= 0 ? 0u : (1u << (8 * nb)) - 1u;
            }
        }
        *reinterpret_cast<u32x4 *>(lds_raw + meta_dst) = meta;
    }
    __syncthreads();
    GWQ_TS(2);                                          // X, scales and zero points are in LDS

    // (3) The block's CSR segment [e_begin, e_end), from the 16-byte boundary below e_begin:
    // thread t brings entries e0 + 8t .. e0 + 8t + 7.  Entries beyond blockDim * 8 stay in memory.
    // Requested only now: its bounds have arrived in the meantime, and it is used last.
    const int e0 = e_begin & ~7;
    u32x4 seg_col, seg_val;
    {
        const int v_end = e_end > e0 ? (e_end - 1) / 8 : e0 / 8;     // last vector the block needs
        int v = e0 / 8 + tid;
        v = v < v_end ? v : v_end;                      // idle threads repeat it: no extra traffic
        v = v < csr_last_vec ? v : csr_last_vec;
        seg_col = reinterpret_cast<const u32x4 *>(col_idx)[v];
        seg_val = reinterpret_cast<const u32x4 *>(out_val)[v];
    }
    const int staged_end = e0 + window < e_end ? e0 + window : e_end;
    __builtin_amdgcn_sched_barrier(0);

    // A lane's MFMA results are rows 4b .. 4b+3 of its channel: rows below MS are kept.
    constexpr int RA = MS < 4 ? MS : 4;
    float acc[RA];
#pragma unroll
    for (int e = 0; e < RA; ++e) acc[e] = 0.f;
    {
        const int x_row = r < MS ? r : 0;
        const act_t *x_lane = xs + (uint32_t)x_row * k_pad + g_begin * kGroup + 32 * b;
        const uint16_t *sc_lane = reinterpret_cast<const uint16_t *>(lds_raw + sc_off) + r * gpr + g_begin;
        const uint8_t *zp_lane = lds_raw + zp_off + r * gpr + g_begin;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (u + kAhead < U) {
                slot[u + kAhead].load_clamped(qweight, code_off + (u + kAhead) * group_bytes, b, code_end);
                __builtin_amdgcn_sched_barrier(0);      // the request stays ahead of this group's arithmetic
            }
            u32x4 xa[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) xa[j] = *reinterpret_cast<const u32x4 *>(x_lane + u * kGroup + 8 * j);
            u32x4 wb[4];
            float4v part = float4v{0.f, 0.f, 0.f, 0.f};
            if constexpr (FINE) {
                constexpr uint32_t cap = BITS == 4 ? 0x6C43u : 0x7091u;     // largest scale with s * (2^bits - 1) finite in FP16
                const uint16_t *sc_row = reinterpret_cast<const uint16_t *>(lds_raw + sc_off) + r * spr;
                const uint8_t *zp_row = lds_raw + zp_off + r * spr;
                const int g = g_begin + u;
                const uint32_t keep = g < gpr ? ~0u : 0u;                   // uniform over the wave
                const int c0 = (g < gpr ? g : gpr - 1) * kGroup + 32 * b;   // first column of the lane's slot
                const int i_lo = c0 >> shift, i_hi = (c0 + 16) >> shift;
                uint32_t s_lo = sc_row[i_lo], s_hi = sc_row[i_hi];
                s_lo = (s_lo < cap ? s_lo : cap) & keep;
                s_hi = (s_hi < cap ? s_hi : cap) & keep;
                const uint32_t z_lo = BITS == 3 ? zp_row[i_lo] & keep : zp_row[i_lo];
                const uint32_t z_hi = BITS == 3 ? zp_row[i_hi] & keep : zp_row[i_hi];
                slot[u].decode_halves(z_lo, z_hi, b, dc, wb, tail_lane4);
                scale_halves(wb, s_lo * 0x10001u, s_hi * 0x10001u);
            } else if constexpr (BF16) {
                const DecodeConstsBf16 dbf(BITS);
                const u32x4 ones = u32x4{kBf16Ones, kBf16Ones, kBf16Ones, kBf16Ones};
                slot[u].decode_bf16(b, dbf, wb, tail_lane4);
                float4v xsum = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    part = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xa[j]),
                                                                   __builtin_bit_cast(bf16x8, wb[j]), part, 0, 0, 0);
                    xsum = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xa[j]),
                                                                   __builtin_bit_cast(bf16x8, ones), xsum, 0, 0, 0);
                }
                const float zc = -(float)(128u + zp_lane[u]);
#pragma unroll
                for (int e = 0; e < RA; ++e) part[e] = __builtin_fmaf(zc, xsum[e], part[e]);
            } else {
                slot[u].decode(zp_lane[u], b, dc, wb, tail_lane4);
            }
            if constexpr (!BF16)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    part = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, xa[j]),
                                                                  __builtin_bit_cast(half8, wb[j]), part, 0, 0, 0);
            const float s = FINE ? 1.f : (float)__builtin_bit_cast(_Float16, sc_lane[u]);
#pragma unroll
            for (int e = 0; e < RA; ++e) acc[e] = __builtin_fmaf(s, part[e], acc[e]);
        }
    }

    GWQ_TS(3);                                          // all codes multiplied
    // The CSR segment has arrived by now: publish it, followed by one vector of zero entries that
    // lanes without an entry read instead.
    if (!PAIR || 8 * tid < window) store_entries(reinterpret_cast<u32x4 *>(lds_raw + ent_off) + 2 * tid, seg_col, seg_val);
    if (tid == 0) {
        reinterpret_cast<u32x4 *>(lds_raw + ent_off)[window / 4] = u32x4{0u, 0u, 0u, 0u};
        reinterpret_cast<u32x4 *>(lds_raw + ent_off)[window / 4 + 1] = u32x4{0u, 0u, 0u, 0u};
    }
    __syncthreads();

    // Outliers: the 4 * waves lanes of a channel split its entries and sum rows m = 0 .. MS-1.
    // Entry j sits at LDS index j - e0 when j < staged_end.
    const int o_stride = 4 * nwaves;
    const bool o_live = n < N && tile_live;
    const int o_end = o_live ? (rp1 < staged_end ? rp1 : staged_end) : 0;   // end of the lane's staged entries
    const uint32_t *entries = reinterpret_cast<const uint32_t *>(lds_raw + ent_off);
    float oacc[MS];
#pragma unroll
    for (int e = 0; e < MS; ++e) oacc[e] = 0.f;
    auto add_outlier = [&](uint32_t col, uint16_t val_bits) {
        const _Float16 v = __builtin_bit_cast(_Float16, val_bits);
#pragma unroll
        for (int e = 0; e < MS; ++e) oacc[e] = __builtin_fmaf((float)v, (float)xs[(uint32_t)e * k_pad + col], oacc[e]);
    };
    auto staged = [&](int idx) {
        const uint32_t entry = entries[idx];
        add_outlier(entry & 0xFFFFu, (uint16_t)(entry >> 16));
    };
    const int j_first = rp0 + 4 * wave + b;
#pragma unroll
    for (int i = 0; i < kPre; ++i) {
        const int j = j_first + i * o_stride;
        staged(j < o_end ? j - e0 : window);            // the zero entry when the lane has none
    }
    if (j_first + kPre * o_stride < o_end || (o_live && rp1 > staged_end)) {
        int j = j_first + kPre * o_stride;
        for (; j < o_end; j += o_stride) staged(j - e0);
        // Entries that did not fit the staged window (very long rows) come straight from memory.
        j = j_first;
        if (j < staged_end) j += ((staged_end - j + o_stride - 1) / o_stride) * o_stride;
        if (o_live)
            for (; j < rp1; j += o_stride) add_outlier(col_idx[j], out_val[j]);
    }

    // Fixed-order reduction over the waves and the four lanes of a channel, then FP16 store.
    // Lane b of a wave that owns groups holds the dense results of rows 4b .. 4b+3.
    GWQ_TS(4);                                          // outliers added
    if constexpr (MS > 4) {
        // More than four rows: the four lanes of a channel meet first (in the order b = 0, 1, 2, 3 for every
        // lane), so that a wave leaves 16 partial sums per row instead of 64 and two blocks fit the LDS of a CU.
#pragma unroll
        for (int e = 0; e < MS; ++e) {
            float v = ((active && b == (e >> 2)) ? acc[e & 3] : 0.f) + oacc[e];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            if (lane < 16) red[(wave * MS + e) * 16 + lane] = v;
        }
        __syncthreads();
        GWQ_TS(5);
        for (int idx = tid; idx < MS * 16; idx += nthreads) {
            const int e = idx >> 4, c = idx & 15;
            float sum = 0.f;
            for (int w = 0; w < nwaves; ++w) sum += red[(w * MS + e) * 16 + c];
            if (tile_live && row0 + c < N) Y[(size_t)e * N + row0 + c] = (act_t)sum;
        }
        GWQ_TS(6);
        GWQ_TS_FLUSH(wave == 0, wave == nwaves - 1);
        return;
    }
#pragma unroll
    for (int e = 0; e < MS; ++e) {
        const float dense = (active && b == (e >> 2)) ? acc[e & 3] : 0.f;
        red[(wave * MS + e) * 64 + lane] = dense + oacc[e];
    }
    __syncthreads();
    GWQ_TS(5);                                          // partial sums of all waves are in LDS
    // Wave e (or the wave that reaches it by striding) sums row e: every lane adds its column of
    // partial sums over the waves, then the four lanes of a channel meet.
    for (int e = wave; e < MS; e += nwaves) {
        float s0 = 0.f, s1 = 0.f;
        int w = 0;
        for (; w + 1 < nwaves; w += 2) {
            s0 += red[(w * MS + e) * 64 + lane];
            s1 += red[((w + 1) * MS + e) * 64 + lane];
        }
        if (w < nwaves) s0 += red[(w * MS + e) * 64 + lane];
        float sum = s0 + s1;
        sum += __shfl_xor(sum, 16);
        sum += __shfl_xor(sum, 32);
        float *stash = red + nwaves * MS * 64 + e * 16 + (lane & 15);   // written and read by the same thread
        if (MODE == 1) {
            if (lane < 16) *stash = sum;
        } else {
            if (MODE == 2) sum = silu(*stash) * sum;
            if (lane < 16 && row0 + lane < N) Y[(size_t)e * N + row0 + lane] = (act_t)sum;
        }
    }
    GWQ_TS(6);                                          // stored
    GWQ_TS_FLUSH(wave == 0, wave == nwaves - 1);
}

template <int BITS, int U, int MS, bool FINE = false, bool BF16 = false, bool PAIR = false>
__global__ __launch_bounds__(1024) void decode_small_kernel(const DecodeBatch batch)
{
    decode_small_body<BITS, U, MS, 0, FINE, BF16, PAIR>(batch, blockIdx.y);
}

// Grid row y multiplies layers 2y (gate) and 2y + 1 (up, whose Y receives H) of the batch, one after the other
// in the same block; the barrier between them keeps the second run's staging out of the first run's LDS reads.
template <int BITS, int U, int MS>
__global__ __launch_bounds__(1024) void decode_small_gate_up_kernel(const DecodeBatch batch)
{
    decode_small_body<BITS, U, MS, 1>(batch, 2 * blockIdx.y);
    __syncthreads();
    decode_small_body<BITS, U, MS, 2>(batch, 2 * blockIdx.y + 1);
}

// ---- any M <= 16, X staged through LDS in chunks of K: the wide kernel ---------------------------
//
// For the batches the lean kernel does not take.  The block walks K in phases of `chunk` columns
// (waves * U groups): per phase every wave stages the X columns of its own U groups (all M rows,
// zeros beyond K) and requests their codes, multiplies, and then adds the outliers of its channels
// that fall into the chunk, with X gathered from LDS.  A lane keeps the four result rows
// 4b .. 4b+3 of its MFMA tiles; the outliers of a channel are split over the waves, every lane
// walking its share of the (column-sorted) row once with a cursor.  Nothing in the multiply is
// predicated: groups at or beyond gpr meet zeros in X, their codes are whatever follows in memory
// (the address is kept inside qweight), and their scale and zero point are replaced by 0 (ANDed
// with a wave-uniform mask; a select would make the compiler branch around the LDS reads): in the
// last phase such a group can lie up to a whole chunk beyond gpr, so what it finds in LDS may be
// anything, and a NaN scale, or a 3-bit zero point that carries the decoder's constants into the
// NaN patterns, would turn its exact zero into a NaN.  (The 4-bit decoder's constants are finite
// for every byte, so there the scale alone is masked.)  At most 8 waves.  X goes from memory straight into LDS
// (load_to_lds_16), a row's share of the wave per instruction.
//
// MR = 8 or 16: rows the MFMA tiles and the outlier lanes are laid out for (M <= MR; rows M .. MR-1 are not staged:
// their lanes read row 0 and their results are dropped).  With 8, the lanes b >= 2 have no rows of their own and
// take every second outlier entry of their channel instead.
// COPIES = 2 (M <= 8 with several phases): two LDS copies of a phase's X, the next phase's requested as soon as the
// block is through this phase's barrier, so that it arrives during the multiply and the outliers.
// Dynamic LDS: X [COPIES][M][chunk] halves | scales [16][gpr] halves | zero points [16][gpr] bytes | 96 guard bytes |
// CSR entries (column | value << 16), blockDim * 8 or * 4 | partial sums [waves][4][64] floats.
//
// FINE: layers whose groups are smaller than 128 (16, 32 or 64; Sec. 3.2 names 16).  The staged metadata
// is [16][spr] with spr = K / group; a lane's slot of 32 codes lies in one group or, at 16, in two, so the
// lane takes scale and zero point per half slot and multiplies them in before the MFMA, which sums over all
// four slots of a block of 128: the operands are s * (q - z) rounded to FP16, as in the kernel for M > 16, and
// the scale is capped likewise so that they stay finite.
//
// BF16: X and Y are bfloat16 (groups of 128 only).  The MFMA operands are the exact values 128 + q; a second set of
// MFMAs against ones gives the group's sum of x per row, and the lane folds s * (sum - (128 + z) * sum_x) into its
// FP32 result, so the weights enter exactly, as in the FP16 kernel.
constexpr int kWideGuard = 96;

template <int BITS, int U, int MR, bool FINE, bool BF16, int COPIES>
__global__ __launch_bounds__(512) void decode_wide_kernel(const DecodeBatch batch)
{
    static_assert(COPIES == 1 || COPIES == 2, "copies of a phase's X in LDS");
    static_assert(!(FINE && BF16), "bfloat16 activations: groups of 128 only");
    typedef std::conditional_t<BF16, __bf16, _Float16> act_t;          // X and Y; both 16 bits wide
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const DecodeProblem &pr = batch.p[blockIdx.y];
    const int N = pr.N, K = pr.K;
    const uint32_t *__restrict__ qweight = pr.qweight;
    const uint16_t *__restrict__ scales = pr.scales;
    const uint8_t *__restrict__ zeros = pr.zeros;
    const int32_t *__restrict__ row_ptr = pr.row_ptr;
    const uint16_t *__restrict__ col_idx = pr.col_idx;
    const uint16_t *__restrict__ out_val = pr.out_val;
    const act_t *__restrict__ X = reinterpret_cast<const act_t *>(pr.X);
    act_t *__restrict__ Y = reinterpret_cast<act_t *>(pr.Y);
    const int sc_last_vec = pr.sc_last_vec, zp_last_vec = pr.zp_last_vec, csr_last_vec = pr.csr_last_vec;
    const int shift = FINE ? pr.group_shift : 7;
    // The whole descriptor is requested in one go and only then looked at.
    asm volatile("" ::"s"(qweight), "s"(scales), "s"(zeros), "s"(row_ptr), "s"(col_idx), "s"(out_val), "s"(X), "s"(Y),
                 "s"(K), "s"(sc_last_vec), "s"(zp_last_vec), "s"(csr_last_vec), "s"(shift));
    if ((int)blockIdx.x * 16 >= N) return;              // the grid is as wide as the largest layer needs

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int M = batch.M, nwaves = batch.nwaves, nthreads = nwaves * 64;
    const int r = lane & 15, b = lane >> 4;
    const int tail_lane4 = 4 * (lane | 48);             // where the 3-bit tail word of this lane's channel arrives
    const int gpr = K / kGroup;
    const int spr = K >> shift;                         // scale / zero-point pairs per channel
    const int chunk_groups = nwaves * U;                // groups per phase
    const int chunk = chunk_groups * kGroup;            // columns per phase
    const int x_stride = chunk + kXPad;                 // row stride of the LDS copy of X
    const int phases = (gpr + chunk_groups - 1) / chunk_groups;

    // With two copies of a phase's X the next phase's columns arrive while this phase's are multiplied and its
    // outliers added (taken for M <= 8, where the copies cost one phase more; at 16 rows they would double the
    // phases, and a phase's outlier loop costs the same whatever its share of K).  When the copies hold all of X
    // between them, later tiles of the block do not stage it again.
    act_t *xs = reinterpret_cast<act_t *>(lds_raw);
    constexpr int x_copies = COPIES;
    const uint32_t x_copy = (uint32_t)M * x_stride;     // halves per copy
    const uint32_t sc_off = (uint32_t)x_copies * x_copy * 2;
    const uint32_t zp_off = sc_off + 32 * spr;
    const uint32_t guard_off = zp_off + 16 * spr;
    const uint32_t ent_off = guard_off + kWideGuard;
    const int window = batch.wide_window * nthreads;    // staged CSR entries: the first 8 or 4 per thread
    const uint32_t red_off = ent_off + 4 * window;
    float *red = reinterpret_cast<float *>(lds_raw + red_off);

    const DecodeConsts dc(BITS);
    constexpr uint32_t group_bytes = words_per_group(BITS) * 4;
    const uint32_t code_end = (uint32_t)N * gpr * group_bytes;
    constexpr int kQ = (U + 3) / 4;                     // 64-vector rounds covering U groups (U = 2: half a round)
    const int x_row = r < M ? r : 0;
    const act_t *x_lane = xs + (uint32_t)x_row * x_stride + wave * (U * kGroup) + 32 * b;
    // Outliers: lane (r, b) adds rows rb .. rb + 3 of its share of channel r's entries.  With 16 rows staged the four
    // lanes of a channel take the same entries, four rows each; with 8 the lanes b >= 2, whose MFMA rows do not
    // exist, take every second entry instead (their sums meet those of lanes b - 2 in the final reduction).
    constexpr bool kFold = MR == 8;
    const int rb = kFold ? 4 * (b & 1) : 4 * b;
    const int o_stride = kFold ? 2 * nwaves : nwaves;
    const act_t *x_out[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) x_out[e] = xs + (uint32_t)(rb + e < M ? rb + e : 0) * x_stride;   // rows m >= M are not stored
    const uint32_t *entries = reinterpret_cast<const uint32_t *>(lds_raw + ent_off);

    // A block takes the 16-channel tiles blockIdx.x, blockIdx.x + gridDim.x, ...: when all of K is
    // one or two phases, the copies of X staged for the first tile serve the others too.  The codes of a
    // phase are requested before the outliers of the phase (or tile) before it are added: by then
    // the registers that take them are free.
    Slot<BITS> slot[U];
    auto load_codes = [&](int tile, int ph) {
        int nn = tile * 16 + r;
        nn = nn < N ? nn : N - 1;
        const uint32_t code_off = ((uint32_t)nn * gpr + (ph * nwaves + wave) * U) * group_bytes;
#pragma unroll
        for (int u = 0; u < U; ++u) slot[u].load_clamped(qweight, code_off + u * group_bytes, b, code_end);
    };
    GWQ_STAMP_AT(0);
    GWQ_STAMP_AT(1);                                    // descriptor has arrived
    load_codes(blockIdx.x, 0);
    for (int block = blockIdx.x; block * 16 < N; block += gridDim.x) {
    const bool stage_x = phases > x_copies || block == (int)blockIdx.x;
    const int row0 = block * 16;
    const int n = row0 + r;
    const int n_c = n < N ? n : N - 1;                  // clamped channel: its results are not stored

    // CSR bounds of the block (scalar loads through the constant address space) and of this lane's channel.
    const int last_row = row0 + 16 < N ? row0 + 16 : N;
    const __attribute__((address_space(4))) int32_t *row_ptr_k =
        (const __attribute__((address_space(4))) int32_t *)(uintptr_t)row_ptr;
    const int e_begin = row_ptr_k[row0], e_end = row_ptr_k[last_row];
    const int rp0 = row_ptr[n_c], rp1 = row_ptr[n_c + 1];

    // The block's scales (32 spr bytes) and zero points (16 spr bytes), contiguous in memory for 16
    // consecutive channels and adjacent in LDS: vector t of that range, t < 2 spr a scales vector.
    auto meta_vec = [&](int t) -> u32x4 {
        const bool is_sc = t < 2 * spr;
        const int v_sc = block * 2 * spr + t < sc_last_vec ? block * 2 * spr + t : sc_last_vec;
        const int v_zp = block * spr + (t - 2 * spr) < zp_last_vec ? block * spr + (t - 2 * spr) : zp_last_vec;
        const u32x4 *src = is_sc ? reinterpret_cast<const u32x4 *>(scales) : reinterpret_cast<const u32x4 *>(zeros);
        return src[is_sc ? v_sc : (t < 3 * spr ? v_zp : 0)];
    };
    const u32x4 meta0 = meta_vec(tid);
    // The block's CSR segment [e_begin, e_end), from the 16-byte boundary below e_begin: thread t
    // brings entries e0 + 8t .. e0 + 8t + 7.  Entries beyond the staged window (blockDim * 8, or * 4) stay in memory.
    const int e0 = e_begin & ~7;
    u32x4 seg_col, seg_val;
    {
        const int v_end = e_end > e0 ? (e_end - 1) / 8 : e0 / 8;     // last vector the block needs
        int v = e0 / 8 + tid;
        v = v < v_end ? v : v_end;                      // idle threads repeat it: no extra traffic
        v = v < csr_last_vec ? v : csr_last_vec;
        seg_col = reinterpret_cast<const u32x4 *>(col_idx)[v];
        seg_val = reinterpret_cast<const u32x4 *>(out_val)[v];
    }
    const int staged_end = e0 + window < e_end ? e0 + window : e_end;

    const bool o_live = n < N && rb < M;
    int j = rp0 + (kFold ? 2 * wave + (b >> 1) : wave); // cursor into this lane's share of the channel's outliers
    const int j_end = o_live ? rp1 : 0;
    float4v acc = float4v{0.f, 0.f, 0.f, 0.f};
    float4v oacc = float4v{0.f, 0.f, 0.f, 0.f};         // outlier sums, apart from the MFMA results where lanes fold
    float4v &osum = kFold ? oacc : acc;

    // X columns of this wave's groups in phase ph, row by row, straight into LDS copy ph % 2: a row's share is 512
    // bytes to 2 KB in memory and in the LDS copy alike, so lane l brings vector l of it.  Vectors beyond K are
    // loaded from column 0 and overwritten with zeros once they have landed (zero_x_tail, after the wait).
    typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
    const uint32_t lds_row0 = (uint32_t)(uintptr_t)(lds_byte_t *)lds_raw + 16u * (uint32_t)(wave * (U * kGroup / 8));
    auto request_x = [&](int ph) {
        const int g_begin = (ph * nwaves + wave) * U;
        const uint32_t copy_bytes = (uint32_t)(ph & (x_copies - 1)) * x_copy * 2u;
#pragma unroll
        for (int e = 0; e < MR; ++e)
            if (e < M) {
#pragma unroll
                for (int i = 0; i < kQ; ++i) {
                    const int kv = g_begin * (kGroup / 8) + lane + 64 * i;
                    if (lane + 64 * i < 16 * U)
                        load_to_lds_16(lds_row0 + copy_bytes + 16u * (uint32_t)(e * (x_stride / 8) + 64 * i),
                                       16u * (uint32_t)(e * (K / 8) + (kv < K / 8 ? kv : 0)), X);
                }
            }
    };
    auto zero_x_tail = [&](int ph) {
        const int g_begin = (ph * nwaves + wave) * U;
        if ((g_begin + U) * (kGroup / 8) <= K / 8) return;      // uniform: only the wave that holds the end of K goes on
        u32x4 *copy = reinterpret_cast<u32x4 *>(xs + (uint32_t)(ph & (x_copies - 1)) * x_copy);
#pragma unroll
        for (int e = 0; e < MR; ++e)
            if (e < M) {
#pragma unroll
                for (int i = 0; i < kQ; ++i) {
                    const int kv = g_begin * (kGroup / 8) + lane + 64 * i;
                    if (lane + 64 * i < 16 * U && kv >= K / 8)
                        copy[e * (x_stride / 8) + wave * (U * kGroup / 8) + lane + 64 * i] = u32x4{0u, 0u, 0u, 0u};
                }
            }
    };
    if (COPIES == 2 && stage_x) request_x(0);
    __builtin_amdgcn_sched_barrier(0);

    for (int ph = 0; ph < phases; ++ph) {
        const int g_begin = (ph * nwaves + wave) * U;
        const uint32_t copy_off = (uint32_t)(ph & (x_copies - 1)) * x_copy;    // halves
        const act_t *const xl = x_lane + copy_off;      // this phase's copy of X
        const act_t *xo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) xo[e] = x_out[e] + copy_off;
        if (COPIES == 1 && stage_x) request_x(ph);      // one copy: free since the barrier that ended the phase before
        __builtin_amdgcn_sched_barrier(0);
        if (ph == 0) {                                  // what was requested above for the whole tile
            if (tid < 3 * spr) *reinterpret_cast<u32x4 *>(lds_raw + sc_off + 16 * tid) = meta0;
            for (int t = tid + nthreads; t < 3 * spr; t += nthreads)
                *reinterpret_cast<u32x4 *>(lds_raw + sc_off + 16 * t) = meta_vec(t);
            if (tid < kWideGuard / 4) reinterpret_cast<uint32_t *>(lds_raw + guard_off)[tid] = 0u;
            if (8 * tid < window) store_entries(reinterpret_cast<u32x4 *>(lds_raw + ent_off) + 2 * tid, seg_col, seg_val);
        }
        if (stage_x) {
            wait_all_loads();                           // X of this phase (and, older than it, this phase's codes)
            zero_x_tail(ph);
        }
        // X of the phase and, first time, the tile's metadata are in LDS; every wave is done with the phase before,
        // so the other copy of X (if there are two) is free.
        __syncthreads();
        // The next phase's X is requested now and arrives while this phase is worked on.  The compiler does not see
        // these loads: its own wait for this phase's codes must come before them (it counts from the youngest load
        // backwards and would wait for them too), hence the empty statements that claim the code registers here,
        // where everything older has arrived anyway.
        if constexpr (COPIES == 2) {
#pragma unroll
            for (int u = 0; u < U; ++u) slot[u].claim();
            __builtin_amdgcn_sched_barrier(0);
            if (stage_x && ph + 1 < phases) request_x(ph + 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (block == (int)blockIdx.x && ph < 3) GWQ_STAMP_AT(2 + 3 * ph);    // X of the phase is in LDS

        if constexpr (FINE) {
            const uint16_t *sc_row = reinterpret_cast<const uint16_t *>(lds_raw + sc_off) + r * spr;
            const uint8_t *zp_row = lds_raw + zp_off + r * spr;
            constexpr uint32_t cap = BITS == 4 ? 0x6C43u : 0x7091u;         // largest scale with s * (2^bits - 1) finite in FP16
#pragma unroll
            for (int u = 0; u < U; ++u) {
                u32x4 xa[4];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) xa[jj] = *reinterpret_cast<const u32x4 *>(xl + u * kGroup + 8 * jj);
                const int g = g_begin + u;
                const uint32_t keep = g < gpr ? ~0u : 0u;                   // uniform over the wave
                const int c0 = (g < gpr ? g : gpr - 1) * kGroup + 32 * b;   // first column of the lane's slot
                const int i_lo = c0 >> shift, i_hi = (c0 + 16) >> shift;
                uint32_t s_lo = sc_row[i_lo], s_hi = sc_row[i_hi];
                s_lo = (s_lo < cap ? s_lo : cap) & keep;
                s_hi = (s_hi < cap ? s_hi : cap) & keep;
                const uint32_t z_lo = BITS == 3 ? zp_row[i_lo] & keep : zp_row[i_lo];
                const uint32_t z_hi = BITS == 3 ? zp_row[i_hi] & keep : zp_row[i_hi];
                u32x4 wb[4];
                slot[u].decode_halves(z_lo, z_hi, b, dc, wb, tail_lane4);
                scale_halves(wb, s_lo * 0x10001u, s_hi * 0x10001u);
                float4v part = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    part = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, xa[jj]),
                                                                  __builtin_bit_cast(half8, wb[jj]), part, 0, 0, 0);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] += part[e];
            }
        } else if constexpr (BF16) {
            const uint16_t *sc_lane = reinterpret_cast<const uint16_t *>(lds_raw + sc_off) + r * gpr + g_begin;
            const uint8_t *zp_lane = lds_raw + zp_off + r * gpr + g_begin;
            const DecodeConstsBf16 dbf(BITS);
            const u32x4 ones = u32x4{kBf16Ones, kBf16Ones, kBf16Ones, kBf16Ones};
#pragma unroll
            for (int u = 0; u < U; ++u) {
                u32x4 xa[4];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) xa[jj] = *reinterpret_cast<const u32x4 *>(xl + u * kGroup + 8 * jj);
                const uint32_t keep = g_begin + u < gpr ? ~0u : 0u; // uniform over the wave: a scalar mask
                const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)(sc_lane[u] & keep));
                const float zc = -(float)(128u + zp_lane[u]);       // any byte gives a finite constant
                u32x4 wb[4];
                slot[u].decode_bf16(b, dbf, wb, tail_lane4);
                float4v part = float4v{0.f, 0.f, 0.f, 0.f}, xsum = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    part = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xa[jj]),
                                                                   __builtin_bit_cast(bf16x8, wb[jj]), part, 0, 0, 0);
                    xsum = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xa[jj]),
                                                                   __builtin_bit_cast(bf16x8, ones), xsum, 0, 0, 0);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] = __builtin_fmaf(s, __builtin_fmaf(zc, xsum[e], part[e]), acc[e]);
            }
        } else {
            const uint16_t *sc_lane = reinterpret_cast<const uint16_t *>(lds_raw + sc_off) + r * gpr + g_begin;
            const uint8_t *zp_lane = lds_raw + zp_off + r * gpr + g_begin;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                u32x4 xa[4];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) xa[jj] = *reinterpret_cast<const u32x4 *>(xl + u * kGroup + 8 * jj);
                const uint32_t keep = g_begin + u < gpr ? ~0u : 0u; // uniform over the wave: a scalar mask
                const _Float16 s = __builtin_bit_cast(_Float16, (uint16_t)(sc_lane[u] & keep));
                const uint32_t z = BITS == 3 ? zp_lane[u] & keep : zp_lane[u];
                u32x4 wb[4];
                slot[u].decode(z, b, dc, wb, tail_lane4);
                float4v part = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    part = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, xa[jj]),
                                                                  __builtin_bit_cast(half8, wb[jj]), part, 0, 0, 0);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] = __builtin_fmaf((float)s, part[e], acc[e]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (block == (int)blockIdx.x && ph < 3) GWQ_STAMP_AT(3 + 3 * ph);    // multiplied
        if (ph + 1 < phases) load_codes(block, ph + 1);
        else if ((block + (int)gridDim.x) * 16 < N) load_codes(block + gridDim.x, 0);
        __builtin_amdgcn_sched_barrier(0);

        // Outliers of the chunk's columns [c0, c1): the lane's entries are sorted by column, so it
        // takes them while they are below c1, four at a time (their columns, values and the X
        // values they select are independent LDS reads; one entry per trip would wait for two
        // dependent reads each time).  An entry that is not taken reads index 0 and adds zero; as the
        // entries are sorted, the taken ones are a prefix of the four.  Entries past the staged
        // window come from memory (two loops: one address space each).
        const int c0 = ph * chunk, c1 = c0 + chunk;
        const int j_staged = j_end < staged_end ? j_end : staged_end;
        for (;;) {
            int col[4];
            float val[4];
            bool ok[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int idx = j + i * o_stride;
                const bool in = idx < j_staged;
                const int li = in ? idx - e0 : 0;
                const uint32_t entry = entries[li];
                const int c = (int)(entry & 0xFFFFu);
                ok[i] = in && c < c1;
                val[i] = ok[i] ? (float)__builtin_bit_cast(_Float16, (uint16_t)(entry >> 16)) : 0.f;
                col[i] = ok[i] ? c - c0 : 0;
            }
            __builtin_amdgcn_sched_barrier(0);          // all four reads above are in flight together, ...
            act_t xv[4][4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e) xv[i][e] = xo[e][col[i]];
            __builtin_amdgcn_sched_barrier(0);          // ... and so are these sixteen
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e) osum[e] = __builtin_fmaf(val[i], (float)xv[i][e], osum[e]);
            j += ((int)ok[0] + (int)ok[1] + (int)ok[2] + (int)ok[3]) * o_stride;
            if (!ok[3]) break;
        }
        while (j >= staged_end && j < j_end) {          // very long rows only
            const int col = col_idx[j];
            if (col >= c1) break;
            const float v = (float)__builtin_bit_cast(_Float16, out_val[j]);
#pragma unroll
            for (int e = 0; e < 4; ++e) osum[e] = __builtin_fmaf(v, (float)xo[e][col - c0], osum[e]);
            j += o_stride;
        }
        if (block == (int)blockIdx.x && ph < 3) GWQ_STAMP_AT(4 + 3 * ph);    // outliers added
        if (x_copies == 1 && ph + 1 < phases) __syncthreads();                // everybody is done with the only copy of X
    }

    // Fixed-order reduction over the waves, then FP16 store.  Folded lanes (b >= 2 with 8 rows staged) hand over their
    // outlier sums alone: their MFMA rows are copies of row 0.
#pragma unroll
    for (int e = 0; e < 4; ++e) red[(wave * 4 + e) * 64 + lane] = !kFold ? acc[e] : b >= 2 ? oacc[e] : acc[e] + oacc[e];
    __syncthreads();
    for (int idx = tid; idx < 256; idx += nthreads) {
        const int e = idx >> 6, l = idx & 63;
        if (kFold && l >= 32) continue;
        float sum = 0.f;
        for (int w = 0; w < nwaves; ++w) sum += kFold ? red[w * 256 + idx] + red[w * 256 + idx + 32] : red[w * 256 + idx];
        const int nn = row0 + (l & 15), m = 4 * (l >> 4) + e;
        if (nn < N && m < M) Y[(size_t)m * N + nn] = (act_t)sum;
    }
    if (block == (int)blockIdx.x) GWQ_STAMP_AT(12);     // first tile stored
    }   // tiles
}

// ---- any M <= 16 with K <= 4096: the streaming kernel --------------------------------------------
//
// The wide kernel above pays for X twice: every group's MFMA operands are read from LDS (4 KB of LDS
// reads per KB of codes), and every outlier entry gathers its X values with one 2-byte LDS read per
// row.  It also stages X per tile and stops at several block-wide barriers per tile.  This kernel
// keeps X where each use wants it:
//   * wave w owns groups [4w, 4w + 4) of every tile, so the X operands of its MFMAs never change: they
//     are loaded once per block (one coalesced 1 KB load per row) and kept in registers (64 per lane);
//   * the outliers read a transposed copy XT[k][MR] in LDS (MR = 4, 8 or 16 rows, staged once per
//     block): the lanes (r, b) of channel r take one entry each and fetch four rows of its column with
//     one 8-byte read.  With MR = 16 the four lanes of a channel share an entry (four rows each), with
//     fewer rows they take different entries;
//   * a block walks `tiles_per_block` consecutive 16-channel tiles.  Codes, scales, zero points and CSR
//     bounds of a tile are requested three tiles ahead into one of three register sets (the loop is
//     unrolled over them), its CSR segment two tiles ahead; one block barrier per tile publishes the
//     segment and the next tile's scales and zero points in LDS (the block fetches those together, 48 gpr
//     contiguous bytes) and the previous tile's partial sums, which a quarter or half of the block then
//     adds in a fixed order while the others go on.
// XT is written by the waves from their X operands, with the matrix cores doing the transposition: an
// operand times a 32 x 16 selection matrix (a single 1.0 per column) returns sixteen of the operand's 32
// columns in the MFMA result layout, where lane (n, q) holds rows 4q .. 4q+3 of column n - the 8 bytes one
// outlier read fetches.  X is therefore read from memory once per block (every block needs all of it, and
// at M = 16 the blocks' reads of X are four times the bytes of the codes).  Column k keeps its rows at byte
// k * 2 MR, with one address bit flipped where bit 5 of k is set, so that the two half-groups of lanes of
// a store instruction (columns 32 apart) fall into different banks.
//
// Dynamic LDS: XT [K][MR] halves | CSR entries (column | value << 16) [2][ent_cap] + 8 zero words |
// partial sums [2][waves][4][64] floats | scales [16][gpr] halves and zero points [16][gpr] bytes of two tiles.
constexpr int kStreamU = 4;                             // groups per wave


// A load that is complete when it returns, invisible to the compiler's bookkeeping of outstanding loads
// (for the rare path below, whose loads would otherwise make every trip wait for all prefetches).
__device__ inline uint32_t load_u16_now(const uint16_t *p)
{
    uint32_t v;
    asm volatile("global_load_ushort %0, %1, off\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
    return v;
}

// Byte offset in XT of rows 4q .. 4q+3 of column `col` (MR rows of FP16 per column).
template <int MR> __device__ inline uint32_t xt_offset(uint32_t col, int q)
{
    constexpr uint32_t flip = MR == 16 ? 16u : MR == 8 ? 128u : 64u;
    return (col * (2 * MR) + 8 * q) ^ ((col & 32u) ? flip : 0u);
}

// Everything a wave needs from memory for one tile.
template <int BITS> struct TileRegs {
    Slot<BITS> slot[kStreamU];
    u32x4 meta;                                         // this thread's 16 bytes of the tile's scales and zero points
    int rp0, rp1;                                       // CSR range of this lane's channel
    int e_begin, e_end;                                 // CSR range of the tile (wave-uniform)
    u32x4 seg_col, seg_val;                             // this thread's eight entries of the tile's segment
};

template <int BITS, int MR>
__global__ __launch_bounds__(512) void decode_stream_kernel(const DecodeBatch batch, const int tiles_per_block,
                                                            const int ent_cap)
{
    constexpr int U = kStreamU, RB = MR / 4, SPLIT = 4 / RB;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const DecodeProblem &pr = batch.p[blockIdx.y];
    const int N = pr.N, K = pr.K;
    const uint32_t *__restrict__ qweight = pr.qweight;
    const uint16_t *__restrict__ scales = pr.scales;
    const uint8_t *__restrict__ zeros = pr.zeros;
    const int32_t *__restrict__ row_ptr = pr.row_ptr;
    const uint16_t *__restrict__ col_idx = pr.col_idx;
    const uint16_t *__restrict__ out_val = pr.out_val;
    const _Float16 *__restrict__ X = pr.X;
    _Float16 *__restrict__ Y = pr.Y;
    const int csr_last_vec = pr.csr_last_vec, sc_last_vec = pr.sc_last_vec, zp_last_vec = pr.zp_last_vec;
    asm volatile("" ::"s"(qweight), "s"(scales), "s"(zeros), "s"(row_ptr), "s"(col_idx), "s"(out_val), "s"(X), "s"(Y),
                 "s"(K), "s"(csr_last_vec), "s"(sc_last_vec), "s"(zp_last_vec));
    const int tiles = (N + 15) >> 4;
    const int tile0 = (int)blockIdx.x * tiles_per_block;
    if (tile0 >= tiles) return;                         // the grid is as wide as the largest layer needs
    const int nt = tiles - tile0 < tiles_per_block ? tiles - tile0 : tiles_per_block;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int M = batch.M, nwaves = batch.nwaves, nthreads = nwaves * 64;
    const int r = lane & 15, b = lane >> 4;
    const int tail_lane4 = 4 * (lane | 48);
    const int gpr = K / kGroup, K8 = K >> 3;
    const int g0 = wave * U;
    GWQ_STAMP_AT(0);                                    // wall clock (100 MHz) at the start
    GWQ_STAMP_AT(1);

    unsigned char *const xt = lds_raw;
    uint32_t *const ent = reinterpret_cast<uint32_t *>(lds_raw + (uint32_t)K * (2 * MR));
    float *const red = reinterpret_cast<float *>(reinterpret_cast<unsigned char *>(ent) + 8 * (uint32_t)ent_cap + 32);
    const int zero_entry = 2 * ent_cap;                 // an entry with value 0 in column 0
    unsigned char *const meta_lds = reinterpret_cast<unsigned char *>(red) + 2 * (uint32_t)nwaves * 1024;
    const uint32_t meta_bytes = 48u * gpr;              // scales [16][gpr] halves, then zero points [16][gpr] bytes

    const DecodeConsts dc(BITS);
    constexpr uint32_t group_bytes = words_per_group(BITS) * 4;
    const uint32_t code_end = (uint32_t)N * gpr * group_bytes;

    // row_ptr again as a pointer to constant memory (nothing in this launch writes it): a load through it with a
    // wave-uniform index is a scalar load, which does not queue behind the vector loads in flight.
    const __attribute__((address_space(4))) int32_t *row_ptr_k =
        (const __attribute__((address_space(4))) int32_t *)(uintptr_t)row_ptr;
    // Requests for tile number `it` of this block (clamped: past the last one it is the last again): the
    // CSR bounds of the tile (scalar loads), then everything the lanes need.
    auto issue_bounds = [&](TileRegs<BITS> &T, int it) {
        const int row0 = (tile0 + (it < nt ? it : nt - 1)) * 16;
        const int last_row = row0 + 16 < N ? row0 + 16 : N;
        T.e_begin = row_ptr_k[row0];                    // uniform addresses in the constant address space: scalar loads
        T.e_end = row_ptr_k[last_row];
    };
    auto issue_tile = [&](TileRegs<BITS> &T, int it) {
        const int n = (tile0 + (it < nt ? it : nt - 1)) * 16 + r;
        const int n_c = n < N ? n : N - 1;
        const uint32_t first_group = (uint32_t)n_c * gpr + g0;
#pragma unroll
        for (int u = 0; u < U; ++u) T.slot[u].load_clamped(qweight, (first_group + u) * group_bytes, b, code_end);
        T.rp0 = row_ptr[n_c];
        T.rp1 = row_ptr[n_c + 1];
    };
    // The tile's scales (32 gpr bytes) and zero points (16 gpr bytes) are contiguous in memory for 16 consecutive
    // channels: thread t < 3 gpr brings vector t of them (one coalesced load of a wave or two, where a load per
    // lane of its own four scales and zero points costs the CU's address unit four times as long); the
    // other threads repeat vector 0.
    auto issue_meta = [&](TileRegs<BITS> &T, int it) {
        const int tile = tile0 + (it < nt ? it : nt - 1);
        const bool is_sc = tid < 2 * gpr, is_zp = !is_sc && tid < 3 * gpr;
        const int v_sc = tile * 2 * gpr + tid < sc_last_vec ? tile * 2 * gpr + tid : sc_last_vec;
        const int v_zp = tile * gpr + (tid - 2 * gpr) < zp_last_vec ? tile * gpr + (tid - 2 * gpr) : zp_last_vec;
        const u32x4 *src = is_zp ? reinterpret_cast<const u32x4 *>(zeros) : reinterpret_cast<const u32x4 *>(scales);
        T.meta = src[is_sc ? v_sc : is_zp ? v_zp : 0];
    };
    auto store_meta = [&](const TileRegs<BITS> &T, int it) {
        if (tid < 3 * gpr) *reinterpret_cast<u32x4 *>(meta_lds + (it & 1) * meta_bytes + 16 * tid) = T.meta;
    };
    // The tile's CSR segment [e_begin, e_end) from the 16-byte boundary below e_begin: thread t brings
    // entries e0 + 8t .. e0 + 8t + 7 (idle threads repeat the last vector: no extra traffic).
    auto issue_seg = [&](TileRegs<BITS> &T) {
        const int e0 = T.e_begin & ~7;
        const int v_end = T.e_end > e0 ? (T.e_end - 1) / 8 : e0 / 8;
        int v = e0 / 8 + tid;
        v = v < v_end ? v : v_end;
        v = v < csr_last_vec ? v : csr_last_vec;
        T.seg_col = reinterpret_cast<const u32x4 *>(col_idx)[v];
        T.seg_val = reinterpret_cast<const u32x4 *>(out_val)[v];
    };

    // Order of the first requests: the first tile's scales and zero points, X, tiles 0, 1 and 2 - none of which
    // waits for anything - and, once the CSR bounds of the first two tiles have come in through the scalar cache
    // (requested first of all), their segments.  X is consumed before the first tile, with everything behind it
    // still in flight.
    TileRegs<BITS> A, B, C;
    issue_bounds(A, 0);
    issue_bounds(B, 1);
    issue_bounds(C, 2);
    issue_meta(A, 0);

    // X for this wave's MFMAs.  Its four groups are 512 consecutive columns, 1 KB of a row: one coalesced
    // load per row (a load in operand layout touches sixteen rows at once and costs the address unit four times
    // as long).  The rows then pass through the part of LDS that will hold this wave's columns of XT (at most MR KB,
    // private to the wave until the first block barrier) to reach the lanes that use them.
    u32x4 xrow[MR];
    {
        const int kv = g0 * (kGroup / 8) + lane;
#pragma unroll
        for (int e = 0; e < MR; ++e)
            xrow[e] = reinterpret_cast<const u32x4 *>(X)[(e < M ? e : 0) * K8 + (kv < K8 ? kv : 0)];
    }
    __builtin_amdgcn_sched_barrier(0);
    issue_tile(A, 0);
    issue_meta(B, 1);
    issue_tile(B, 1);
    issue_meta(C, 2);
    issue_tile(C, 2);
    __builtin_amdgcn_sched_barrier(0);
    issue_seg(A);
    issue_seg(B);
    __builtin_amdgcn_sched_barrier(0);
    GWQ_STAMP_AT(2);                                    // everything requested

    if (tid < 8) ent[zero_entry + tid] = 0u;
    store_meta(A, 0);

    // The rows lie back to back in the wave's part (256 bytes per group that exists), the 16-byte pieces of row e
    // permuted by e (piece c at position c ^ e), so that the sixteen rows of one piece - what an operand read
    // fetches - fall into different banks.  Rows at or beyond M and groups at or beyond gpr are zeros.
    u32x4 xa[U][4];
    {
        const int ng = gpr - g0 < U ? gpr - g0 : U;     // this wave's groups that exist (uniform; at least one)
        const uint32_t row_bytes = 256u * ng;
        unsigned char *const mine = xt + (uint32_t)g0 * (kGroup * 2 * MR);
        if (lane < 16 * ng)
#pragma unroll
            for (int e = 0; e < MR; ++e)
                *reinterpret_cast<u32x4 *>(mine + e * row_bytes + ((lane ^ e) << 4)) = e < M ? xrow[e] : u32x4{0u, 0u, 0u, 0u};
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool live = u < ng && r < MR;         // other lanes multiply zeros
            const uint32_t keep = live ? ~0u : 0u;
            const int rr = live ? r : 0, piece0 = live ? 16 * u + 4 * b : 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const u32x4 v = *reinterpret_cast<const u32x4 *>(mine + rr * row_bytes + (((piece0 + j) ^ rr) << 4));
                xa[u][j] = v & u32x4{keep, keep, keep, keep};
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    __builtin_amdgcn_sched_barrier(0);
    GWQ_STAMP_AT(3);                                    // X has arrived

    if (tid < 8) ent[zero_entry + tid] = 0u;
    store_meta(A, 0);

    // XT from the operands.  Operand (u, j) holds, as its MFMA column 8 b' + t, the X column
    // 128 (g0 + u) + 32 b' + 8 j + t; selection matrix s picks MFMA columns 16 s .. 16 s + 15, so lane
    // (n = r, q = b) receives rows 4q .. 4q+3 of X column 128 (g0 + u) + 64 s + 32 (n / 8) + 8 j + n % 8.
    {
        u32x4 sel[2];
#pragma unroll
        for (int sq = 0; sq < 2; ++sq) {
            const int at = b == 2 * sq + (r >> 3) ? (r & 7) : -1;    // position of this lane's 1.0, if it has one
            sel[sq] = u32x4{at == 0 ? 0x3C00u : at == 1 ? 0x3C000000u : 0u, at == 2 ? 0x3C00u : at == 3 ? 0x3C000000u : 0u,
                            at == 4 ? 0x3C00u : at == 5 ? 0x3C000000u : 0u, at == 6 ? 0x3C00u : at == 7 ? 0x3C000000u : 0u};
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (g0 + u < gpr) {                         // uniform over the wave
                // eight independent MFMAs back to back, then their results: nothing waits for the one before it
                float4v t[4][2];
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int sq = 0; sq < 2; ++sq)
                        t[j][sq] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                            __builtin_bit_cast(half8, xa[u][j]), __builtin_bit_cast(half8, sel[sq]),
                            float4v{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int sq = 0; sq < 2; ++sq) {
                        const uint32_t col = (uint32_t)(g0 + u) * kGroup + 64 * sq + 32 * (r >> 3) + 8 * j + (r & 7);
                        const half2v lo = half2v{(_Float16)t[j][sq][0], (_Float16)t[j][sq][1]};
                        const half2v hi = half2v{(_Float16)t[j][sq][2], (_Float16)t[j][sq][3]};
                        if (b < RB)
                            *reinterpret_cast<uint2 *>(xt + xt_offset<MR>(col, b)) =
                                uint2{__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
                    }
                __builtin_amdgcn_sched_barrier(0);
            }
    }

    __syncthreads();                                    // tile 0's scales and zero points are in LDS (and XT, for later)
    GWQ_STAMP_AT(4);                                    // XT written
    const int xq = b % RB;                              // which four rows of XT this lane adds
    const int sub = wave * SPLIT + b / RB;              // this lane's share of its channel's entries
    const int stride = nwaves * SPLIT;
    const int red_groups = nthreads >= 512 ? 2 : 1;     // sets of 256 threads that take turns adding partial sums

    // Adds the partial sums of tile number `it` (written before the last barrier) and stores its outputs.
    auto reduce_tile = [&](int it) {
        const float *src = red + (it & 1) * (nwaves * 256);
        const int row0 = (tile0 + it) * 16;
        auto one = [&](int idx) {
            const int e = idx >> 6, l = idx & 63, bq = l >> 4;
            if (bq >= RB) return;
            float sum = 0.f;
            for (int w = 0; w < nwaves; ++w)
#pragma unroll
                for (int sp = 0; sp < SPLIT; ++sp) sum += src[(w * 4 + e) * 64 + (l & 15) + 16 * (bq + RB * sp)];
            const int nn = row0 + (l & 15), m = 4 * bq + e;
            if (nn < N && m < M) Y[(size_t)m * N + nn] = (_Float16)sum;
        };
        if (nthreads >= 256) {
            const int grp = it % red_groups;
            if ((tid >> 8) == grp) one(tid & 255);
        } else {
            for (int idx = tid; idx < 256; idx += nthreads) one(idx);
        }
    };

    // One tile: T holds it, T1 and T2 are the sets of the next tile (its scales and zero points go to LDS here) and
    // of the one after (its CSR segment is requested here).  Requests are unconditional (past the block's last
    // tile they repeat it): a trip always leaves the same queue of requests behind, which is what lets the waits
    // inside the loop be exact.
    auto step = [&](TileRegs<BITS> &T, TileRegs<BITS> &T1, TileRegs<BITS> &T2, int it) {
        const int buf = it & 1;
        const int e0 = T.e_begin & ~7;
        const int staged_end = e0 + ent_cap < T.e_end ? e0 + ent_cap : T.e_end;
        // Real copies into other registers: the set is refilled below while these are still needed, and a
        // refilled value must land in the register the next trip reads it from (otherwise the compiler moves
        // it there at the end of the trip, and a move of a value still on its way waits for it).
        int rp0, rp1;
        asm volatile("v_mov_b32 %0, %2\n\tv_mov_b32 %1, %3" : "=&v"(rp0), "=&v"(rp1) : "v"(T.rp0), "v"(T.rp1));
        if (it == 0) GWQ_STAMP_AT(5);                   // tile 0 has arrived

        const uint16_t *sc_lane = reinterpret_cast<const uint16_t *>(meta_lds + buf * meta_bytes) + r * gpr + g0;
        const uint8_t *zp_lane = meta_lds + buf * meta_bytes + 32 * gpr + r * gpr + g0;
        float4v acc = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t keep = g0 + u < gpr ? ~0u : 0u;      // uniform over the wave
            const _Float16 s = __builtin_bit_cast(_Float16, (uint16_t)(sc_lane[u] & keep));
            const uint32_t z = BITS == 3 ? zp_lane[u] & keep : zp_lane[u];
            u32x4 wb[4];
            T.slot[u].decode(z, b, dc, wb, tail_lane4);
            float4v part = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j)
                part = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, xa[u][j]),
                                                              __builtin_bit_cast(half8, wb[j]), part, 0, 0, 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = __builtin_fmaf((float)s, part[e], acc[e]);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (it == 0) GWQ_STAMP_AT(6);                   // multiplied
        u32x4 seg_col = T.seg_col, seg_val = T.seg_val;
        issue_seg(T2);
        issue_bounds(T, it + 3);
        issue_meta(T, it + 3);
        issue_tile(T, it + 3);
        __builtin_amdgcn_sched_barrier(0);
        if (8 * tid < ent_cap) store_entries(reinterpret_cast<u32x4 *>(ent + buf * ent_cap) + 2 * tid, seg_col, seg_val);
        store_meta(T1, it + 1);
        if (it == 0) GWQ_STAMP_AT(7);                   // its CSR segment has arrived
        __syncthreads();                                // this tile's entries and the previous tile's sums are in LDS
        if (it == 0) GWQ_STAMP_AT(8);                   // through the barrier
        if (it > 0) reduce_tile(it - 1);

        // Outliers: entry j of the channel sits at LDS index j - e0 while j < staged_end.
        const int n = (tile0 + it) * 16 + r;
        const int j_end = n < N ? rp1 : rp0;
        const int j_staged = j_end < staged_end ? j_end : staged_end;
        for (int j = rp0 + sub; j < j_staged; j += 4 * stride) {
            uint32_t entry[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int idx = j + i * stride;
                entry[i] = ent[idx < j_staged ? buf * ent_cap + idx - e0 : zero_entry];
            }
            uint2 xv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t col = entry[i] & 0xFFFFu;
                xv[i] = *reinterpret_cast<const uint2 *>(xt + xt_offset<MR>(col, xq));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float v = (float)__builtin_bit_cast(_Float16, (uint16_t)(entry[i] >> 16));
                const half2v x01 = __builtin_bit_cast(half2v, xv[i].x), x23 = __builtin_bit_cast(half2v, xv[i].y);
                acc[0] = __builtin_fmaf(v, (float)x01[0], acc[0]);
                acc[1] = __builtin_fmaf(v, (float)x01[1], acc[1]);
                acc[2] = __builtin_fmaf(v, (float)x23[0], acc[2]);
                acc[3] = __builtin_fmaf(v, (float)x23[1], acc[3]);
            }
        }
        if (j_end > staged_end) {                       // rows longer than the staged window: straight from memory
            int j = rp0 + sub;
            if (j < staged_end) j += (staged_end - j + stride - 1) / stride * stride;
            for (; j < j_end; j += stride) {
                const uint32_t col = load_u16_now(col_idx + j);
                const float v = (float)__builtin_bit_cast(_Float16, (uint16_t)load_u16_now(out_val + j));
                const uint2 x = *reinterpret_cast<const uint2 *>(xt + xt_offset<MR>(col, xq));
                const half2v x01 = __builtin_bit_cast(half2v, x.x), x23 = __builtin_bit_cast(half2v, x.y);
                acc[0] = __builtin_fmaf(v, (float)x01[0], acc[0]);
                acc[1] = __builtin_fmaf(v, (float)x01[1], acc[1]);
                acc[2] = __builtin_fmaf(v, (float)x23[0], acc[2]);
                acc[3] = __builtin_fmaf(v, (float)x23[1], acc[3]);
            }
        }
        float *dst = red + buf * (nwaves * 256) + wave * 256 + lane;
#pragma unroll
        for (int e = 0; e < 4; ++e) dst[e * 64] = acc[e];
        if (it == 0) GWQ_STAMP_AT(9);                   // outliers added
    };

    // The first three trips stand outside the loop: after them the requests in flight are those a trip of
    // the loop leaves behind, in the same order, so the loop's waits hold from its first trip on.
    step(A, B, C, 0);
    if (nt > 1) {
        step(B, C, A, 1);
        if (nt > 2) {
            step(C, A, B, 2);
            int it = 3;
            for (; it + 3 <= nt; it += 3) {
                step(A, B, C, it);
                step(B, C, A, it + 1);
                step(C, A, B, it + 2);
            }
            if (it < nt) {
                step(A, B, C, it);
                if (it + 1 < nt) step(B, C, A, it + 1);
            }
        }
    }
    GWQ_STAMP_AT(10);                                   // all tiles done
    __syncthreads();
    GWQ_STAMP_AT(11);
    reduce_tile(nt - 1);
    GWQ_STAMP_AT(12);                                   // stored
}

constexpr size_t kMaxLds = 160 * 1024;                  // LDS a block may use on gfx950
constexpr size_t kXLdsBudget = 128 * 1024;              // X[M][k_pad] is staged in LDS up to this size
constexpr int kLeanRows = 8;                            // the lean kernel takes M up to here (where X fits the LDS)

template <auto Kernel>
hipError_t launch_kernel(const DecodeBatch &batch, int count, int blocks, int nwaves, size_t lds, hipStream_t st)
{
    static std::atomic<uint32_t> lds_allowed{0};        // per kernel
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(Kernel), (int)kMaxLds, lds_allowed);
    if (e != hipSuccess) return e;
    Kernel<<<dim3(blocks, count), nwaves * 64, lds, st>>>(batch);
    return hipGetLastError();
}

template <int BITS>
hipError_t launch_small(const DecodeBatch &batch, int count, int blocks, int nwaves, int u, int ms, size_t lds,
                        bool gated_pairs, bool fine, bool bf16, bool pair, hipStream_t st)
{
    if (pair) {                                         // nwaves: both sets of waves
#define GWQ_SMALL_PAIR(UU, MM) \
    if (u == UU && ms == MM && !gated_pairs && !fine && !bf16) \
        return launch_kernel<&decode_small_kernel<BITS, UU, MM, false, false, true>>(batch, count, blocks, nwaves, lds, st)
        GWQ_SMALL_PAIR(4, 5); GWQ_SMALL_PAIR(4, 6); GWQ_SMALL_PAIR(4, 7); GWQ_SMALL_PAIR(4, 8);
        GWQ_SMALL_PAIR(8, 5); GWQ_SMALL_PAIR(8, 6); GWQ_SMALL_PAIR(8, 7); GWQ_SMALL_PAIR(8, 8);
#undef GWQ_SMALL_PAIR
        return hipErrorInvalidValue;
    }
    if (bf16) {
#define GWQ_SMALL_BF16(UU, MM) \
    if (u == UU && ms == MM && !gated_pairs && !fine) \
        return launch_kernel<&decode_small_kernel<BITS, UU, MM, false, true>>(batch, count, blocks, nwaves, lds, st)
        GWQ_SMALL_BF16(4, 1); GWQ_SMALL_BF16(4, 2); GWQ_SMALL_BF16(4, 3); GWQ_SMALL_BF16(4, 4);
        GWQ_SMALL_BF16(4, 5); GWQ_SMALL_BF16(4, 6); GWQ_SMALL_BF16(4, 7); GWQ_SMALL_BF16(4, 8);
        GWQ_SMALL_BF16(8, 1); GWQ_SMALL_BF16(8, 2); GWQ_SMALL_BF16(8, 3); GWQ_SMALL_BF16(8, 4);
        GWQ_SMALL_BF16(8, 5); GWQ_SMALL_BF16(8, 6); GWQ_SMALL_BF16(8, 7); GWQ_SMALL_BF16(8, 8);
        GWQ_SMALL_BF16(16, 1);                           // (16, 2) would need more than the 128 registers of a 16-wave block
#undef GWQ_SMALL_BF16
        return hipErrorInvalidValue;
    }
    if (fine) {
#define GWQ_SMALL_FINE(UU, MM) \
    if (u == UU && ms == MM && !gated_pairs) return launch_kernel<&decode_small_kernel<BITS, UU, MM, true>>(batch, count, blocks, nwaves, lds, st)
        GWQ_SMALL_FINE(4, 1); GWQ_SMALL_FINE(4, 2); GWQ_SMALL_FINE(4, 3); GWQ_SMALL_FINE(4, 4);
        GWQ_SMALL_FINE(4, 5); GWQ_SMALL_FINE(4, 6); GWQ_SMALL_FINE(4, 7); GWQ_SMALL_FINE(4, 8);
        GWQ_SMALL_FINE(8, 1); GWQ_SMALL_FINE(8, 2); GWQ_SMALL_FINE(8, 3); GWQ_SMALL_FINE(8, 4);
        GWQ_SMALL_FINE(8, 5); GWQ_SMALL_FINE(8, 6); GWQ_SMALL_FINE(8, 7); GWQ_SMALL_FINE(8, 8);
#undef GWQ_SMALL_FINE
        return hipErrorInvalidValue;
    }
#define GWQ_SMALL(UU, MM) \
    if (u == UU && ms == MM) \
        return gated_pairs ? launch_kernel<&decode_small_gate_up_kernel<BITS, UU, MM>>(batch, count / 2, blocks, nwaves, lds, st) \
                           : launch_kernel<&decode_small_kernel<BITS, UU, MM>>(batch, count, blocks, nwaves, lds, st)
#define GWQ_SMALL_PLAIN(UU, MM) \
    if (u == UU && ms == MM && !gated_pairs) return launch_kernel<&decode_small_kernel<BITS, UU, MM>>(batch, count, blocks, nwaves, lds, st)
    GWQ_SMALL(4, 1); GWQ_SMALL(4, 2); GWQ_SMALL(4, 3); GWQ_SMALL(4, 4);
    GWQ_SMALL(8, 1); GWQ_SMALL(8, 2); GWQ_SMALL(8, 3); GWQ_SMALL(8, 4);
    GWQ_SMALL(16, 1); GWQ_SMALL(16, 2);
    GWQ_SMALL_PLAIN(4, 5); GWQ_SMALL_PLAIN(4, 6); GWQ_SMALL_PLAIN(4, 7); GWQ_SMALL_PLAIN(4, 8);
    GWQ_SMALL_PLAIN(8, 5); GWQ_SMALL_PLAIN(8, 6); GWQ_SMALL_PLAIN(8, 7); GWQ_SMALL_PLAIN(8, 8);
#undef GWQ_SMALL
#undef GWQ_SMALL_PLAIN
    return hipErrorInvalidValue;
}

}  // namespace

// Decode launch over `count` layers (same bits, same M): grid row i works on layer i; the grid is as
// wide as the layer with most channels needs and the surplus blocks of smaller layers exit at once.
hipError_t launch_decode(int count, const gwq_packed *const *P, const void *const *X, int M, void *const *Y,
                         const DecodeTuning &tune, hipStream_t st, PlanText *describe)
{
    const int waves_override = tune.waves;
    DecodeBatch batch;
    batch.M = M;
    int blocks = 0, max_gpr = 1, max_spr = 1;
    bool fine = false;                                  // groups below 128 (the caller passes layers of one group size)
    for (int i = 0; i < count; ++i) {
        const gwq_packed &L = *P[i];
        const int gpr = L.K / kGroup;
        DecodeProblem &d = batch.p[i];
        d.qweight = L.qweight; d.scales = L.scales; d.zeros = L.zeros;
        d.row_ptr = L.row_ptr; d.col_idx = L.col_idx; d.out_val = L.out_val;
        d.X = static_cast<const _Float16 *>(X[i]);       // bfloat16 when tune.bf16: the wide kernel reinterprets
        d.Y = static_cast<_Float16 *>(Y[i]);
        d.N = L.N; d.K = L.K;
        // Last 16-byte vector of each staged array (the buffers are padded, so clamped reads stay inside).
        int shift = 7;
        while ((1 << shift) > L.group) --shift;
        d.group_shift = shift;
        if (L.group < kGroup) fine = true;
        const int64_t groups = (int64_t)L.N * (L.K / L.group);
        if (L.K / L.group > max_spr) max_spr = L.K / L.group;
        d.sc_last_vec = (int)((groups * 2 + 15) / 16) - 1;
        d.zp_last_vec = (int)((groups + 15) / 16) - 1;
        d.csr_last_vec = (int)((L.n_outliers * 2 + 15) / 16);
        if ((L.N + 15) / 16 > blocks) blocks = (L.N + 15) / 16;
        if (gpr > max_gpr) max_gpr = gpr;
    }
    for (int i = count; i < kMaxBatch; ++i) batch.p[i] = batch.p[0];
    const int bits = P[0]->bits;
    const size_t meta = (size_t)48 * max_spr + 16;

    // The lean kernel: M <= 4, every wave owning exactly U groups, at most 16 waves, X in LDS.
    if (tune.bf16 && fine) return hipErrorNotSupported;
    const int lean_rows = tune.lean_rows > 0 ? tune.lean_rows : kLeanRows;
    if (M <= lean_rows && (M <= 4 || !tune.gated_pairs) && !(fine && tune.gated_pairs) && !(tune.bf16 && tune.gated_pairs) &&
        !(tune.stream == 2 && !fine && max_gpr <= 8 * kStreamU)) {
        int u = max_gpr > 128 ? 16 : max_gpr > 16 ? 8 : 4;
        if (waves_override > 0) {                       // the most waves that do not exceed the request
            u = 4;
            while (u < 16 && (max_gpr + u - 1) / u > waves_override) u *= 2;
        }
        while (u < 16 && (max_gpr + u - 1) / u > 16) u *= 2;
        const int nwaves = (max_gpr + u - 1) / u;
        const size_t x_bytes = (size_t)M * (nwaves * u * kGroup + kXPad) * 2;
        const size_t lds = x_bytes + meta + 2 * (16 * (size_t)nwaves * 64 + 16) + (size_t)nwaves * M * (M > 4 ? 64 : 256) + 64 * (size_t)M;
        // Beyond four rows X is most of a block's LDS: the kernel is taken where two blocks still share a CU, or
        // where the launch is at most three rounds of single blocks (more rounds: a kernel whose blocks stage X
        // once for several tiles is faster).
        int total_blocks = 0;
        for (int i = 0; i < count; ++i) total_blocks += (P[i]->N + 15) / 16;
        const bool roomy = M <= 4 || 2 * lds <= kMaxLds || total_blocks <= 3 * device_cus();
        // Small groups: at most three metadata vectors per thread (3 spr <= 3 blockDim).
        const bool fine_ok = !fine || (u <= 8 && max_spr <= 64 * nwaves);
        // Beyond four rows, two neighbouring tiles per block with one copy of X between them (half the reads of X
        // per tile) where the launch still has two blocks for every CU and two such blocks share a CU's LDS.
        const size_t set_bytes = meta + (size_t)16 * nwaves * 64 + 32 + (size_t)nwaves * M * 64;
        const size_t lds_pair = x_bytes + 2 * set_bytes;
        const bool pair = M > 4 && !fine && !tune.bf16 && !tune.gated_pairs && u <= 8 && 2 * nwaves <= 16 &&
                          x_bytes <= kXLdsBudget && 2 * lds_pair <= kMaxLds && tune.pairs != 1 &&
                          (tune.pairs == 2 || total_blocks >= 4 * device_cus());
        if (pair) {
            batch.nwaves = 2 * nwaves;
            const int grid = (blocks + 1) / 2;
            if (describe) {
                snprintf(describe->text, sizeof(describe->text), "decode_small_kernel<%d,%d,%d,false,false,true> grid %dx%d block %d lds %zu",
                         bits, u, M, grid, count, 128 * nwaves, lds_pair);
                return hipSuccess;
            }
            return bits == 4 ? launch_small<4>(batch, count, grid, 2 * nwaves, u, M, lds_pair, false, false, false, true, st)
                             : launch_small<3>(batch, count, grid, 2 * nwaves, u, M, lds_pair, false, false, false, true, st);
        }
        if (nwaves <= 16 && (u < 16 || M <= (tune.bf16 ? 1 : 2)) && x_bytes <= kXLdsBudget && lds <= kMaxLds && (M <= 4 || u <= 8) && roomy && fine_ok) {
            batch.nwaves = nwaves;
            if (describe) {
                snprintf(describe->text, sizeof(describe->text), "%s<%d,%d,%d%s> grid %dx%d block %d lds %zu",
                         tune.gated_pairs ? "decode_small_gate_up_kernel" : "decode_small_kernel", bits, u, M,
                         tune.bf16 ? ",false,true" : fine ? ",true" : "", blocks, tune.gated_pairs ? count / 2 : count,
                         64 * nwaves, lds);
                return hipSuccess;
            }
            return bits == 4 ? launch_small<4>(batch, count, blocks, nwaves, u, M, lds, tune.gated_pairs, fine, tune.bf16, false, st)
                             : launch_small<3>(batch, count, blocks, nwaves, u, M, lds, tune.gated_pairs, fine, tune.bf16, false, st);
        }
    }
    if (tune.gated_pairs) return hipErrorNotSupported;  // only the kernel above multiplies gated pairs

    // The streaming kernel: rows of at most 32 groups (8 waves of 4), XT[K][rows] in LDS.  By default for
    // the batches the lean kernel does not take.
    if (!fine && !tune.bf16 && tune.stream != 1 && (M > 4 || tune.stream == 2) && max_gpr <= 8 * kStreamU) {
        const int nwaves = (max_gpr + kStreamU - 1) / kStreamU, nthreads = 64 * nwaves;
        const int mr = M <= 4 ? 4 : M <= 8 ? 8 : 16;
        const size_t xt = (size_t)max_gpr * kGroup * 2 * mr, red = (size_t)2 * nwaves * 1024;
        const size_t meta_lds = (size_t)2 * 48 * max_gpr + 16;   // scales and zero points of two tiles
        const size_t avail = kMaxLds - xt - red - meta_lds - 32;
        int ent_cap = (int)(avail / 8) & ~7;
        if (ent_cap > 8 * nthreads) ent_cap = 8 * nthreads;
        if (ent_cap >= 64) {
            const size_t lds = xt + (size_t)8 * ent_cap + 32 + red + meta_lds;
            // Blocks a CU holds at once: the kernel's registers allow eight waves.
            int bpc = (int)(kMaxLds / lds);
            if (bpc > 8 / nwaves) bpc = 8 / nwaves;
            if (bpc < 1) bpc = 1;
            const int slots = device_cus() * bpc;
            // The fewest tiles per block with which all layers' blocks are resident at once.
            int tpb = tune.tiles;
            if (tpb <= 0)
                for (tpb = 1;; ++tpb) {
                    int total = 0;
                    for (int i = 0; i < count; ++i) total += ((P[i]->N + 15) / 16 + tpb - 1) / tpb;
                    if (total <= slots) break;
                }
            // A block that gets a single tile has nothing to pipeline and pays the set-up of XT for it: the wide
            // kernel is faster there (4096 channels on 256 CUs).
            const bool take = tune.stream == 2 || tune.tiles > 0 || tpb >= 2;
            batch.nwaves = nwaves;
            const int grid = (blocks + tpb - 1) / tpb;
            if (take && describe) {
                snprintf(describe->text, sizeof(describe->text),
                         "decode_stream_kernel<%d,%d> grid %dx%d block %d lds %zu tiles_per_block %d", bits, mr, grid,
                         count, nthreads, lds, tpb);
                return hipSuccess;
            }
            hipError_t e = hipErrorInvalidValue;
#define GWQ_STREAM(B, RR) \
    if (take && bits == B && mr == RR) { \
        static std::atomic<uint32_t> lds_allowed{0}; \
        e = allow_dynamic_lds(reinterpret_cast<const void *>(&decode_stream_kernel<B, RR>), (int)kMaxLds, lds_allowed); \
        if (e != hipSuccess) return e; \
        decode_stream_kernel<B, RR><<<dim3(grid, count), nthreads, lds, st>>>(batch, tpb, ent_cap); \
        return hipGetLastError(); \
    }
            GWQ_STREAM(4, 4) GWQ_STREAM(4, 8) GWQ_STREAM(4, 16) GWQ_STREAM(3, 4) GWQ_STREAM(3, 8) GWQ_STREAM(3, 16)
#undef GWQ_STREAM
            if (take) return e;
        }
    }

    // The wide kernel.  Among the shapes (U, waves <= 8) whose LDS footprint fits, the one with the
    // fewest phases, then the most waves, then the shorter waves.
    {
        int best_u = 0, best_w = 0, best_ph = 1 << 30, best_window = 8, best_copies = 1;
        size_t best_lds = 0;
        // The staged window of CSR entries is 8 per thread (a tile has about 650 at 1 %, the window 4096 with eight
        // waves); where that costs a phase, 4 per thread are tried as well.
        for (int window = 8; window >= 4; window -= 4)
            for (int u = 2; u <= (M <= 8 ? 8 : 4); u *= 2)   // 16 rows of 8 groups would not fit the registers
                for (int w = 1; w <= 8; ++w) {
                    const int ph = (max_gpr + w * u - 1) / (w * u);
                    // Several phases at M <= 8: two copies, the next phase's X arrives during this one (4096 x 11008,
                    // M = 8: 14.1 against 16.2 us; at M = 16 the copies double the phases: 20.1 against 16.4 us).
                    const size_t copies = ph > 1 && M <= 8 ? 2 : 1;
                    if ((u == 2 && copies == 1) || (u == 8 && copies == 2)) continue;    // forms that are not built
                    const size_t lds = copies * M * (w * u * kGroup + kXPad) * 2 + (size_t)48 * max_spr + kWideGuard +
                                       (size_t)window * 4 * w * 64 + (size_t)w * 1024;
                    if (lds > kMaxLds) continue;
                    if (ph < best_ph || (ph == best_ph && window == best_window && w > best_w)) {
                        best_ph = ph; best_u = u; best_w = w; best_lds = lds; best_window = window; best_copies = (int)copies;
                    }
                }
        if (best_u) {
            batch.nwaves = best_w;
            batch.wide_window = best_window;
            const int mr = M <= 8 ? 8 : 16;
            // One resident block per CU (X fills most of the LDS): when one or two phases cover K, all of X stays
            // in LDS, and fewer blocks that loop over tiles stage it once each.
            if (best_ph <= best_copies) {
                const int cus = device_cus();
                const int cap = cus / count > 0 ? cus / count : 1;
                if (blocks > cap) blocks = cap;
            }
            if (describe) {
                snprintf(describe->text, sizeof(describe->text), "decode_wide_kernel<%d,%d,%d,%s,%s,%d> grid %dx%d block %d lds %zu phases %d",
                         bits, best_u, mr, fine ? "true" : "false", tune.bf16 ? "true" : "false", best_copies, blocks, count,
                         64 * best_w, best_lds, best_ph);
                return hipSuccess;
            }
#define GWQ_WIDE(B, UU, RR, CC) \
    if (bits == B && best_u == UU && mr == RR && best_copies == CC) \
        return tune.bf16 ? launch_kernel<&decode_wide_kernel<B, UU, RR, false, true, CC>>(batch, count, blocks, best_w, best_lds, st) \
               : fine    ? launch_kernel<&decode_wide_kernel<B, UU, RR, true, false, CC>>(batch, count, blocks, best_w, best_lds, st) \
                         : launch_kernel<&decode_wide_kernel<B, UU, RR, false, false, CC>>(batch, count, blocks, best_w, best_lds, st)
            GWQ_WIDE(4, 4, 8, 1); GWQ_WIDE(4, 4, 16, 1); GWQ_WIDE(4, 8, 8, 1); GWQ_WIDE(4, 2, 8, 2); GWQ_WIDE(4, 4, 8, 2);
            GWQ_WIDE(3, 4, 8, 1); GWQ_WIDE(3, 4, 16, 1); GWQ_WIDE(3, 8, 8, 1); GWQ_WIDE(3, 2, 8, 2); GWQ_WIDE(3, 4, 8, 2);
#undef GWQ_WIDE
        }
    }

    return hipErrorInvalidValue;                        // unreachable: one wave of four groups always fits
}

namespace {
__global__ __launch_bounds__(256) void silu_mul_kernel(const _Float16 *__restrict__ G, const _Float16 *__restrict__ U,
                                                       _Float16 *__restrict__ H, size_t count)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) H[i] = (_Float16)(silu((float)G[i]) * (float)U[i]);
}
}  // namespace

hipError_t launch_silu_mul(const void *G, const void *U, void *H, size_t count, hipStream_t st)
{
    silu_mul_kernel<<<(unsigned)((count + 255) / 256), 256, 0, st>>>(static_cast<const _Float16 *>(G), static_cast<const _Float16 *>(U),
                                                                   static_cast<_Float16 *>(H), count);
    return hipGetLastError();
}

}  // namespace gwq

#ifdef GWQ_STAMP
// Copies the first `count` recorded stamps to the host (waits for the device first).
extern "C" int gwq_debug_read_stamps(unsigned long long *host, int count)
{
    if (count > gwq::kStampBlocks * gwq::kStampSlots) count = gwq::kStampBlocks * gwq::kStampSlots;
    if (hipDeviceSynchronize() != hipSuccess) return -1;
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(gwq::g_stamps), sizeof(unsigned long long) * count) == hipSuccess ? count : -1;
}
#endif
