// gwq_linear for M > 16 on gfx950: an MFMA GEMM that dequantises the packed weights on the fly.
//
//   Y[m][n] = sum_k X[m][k] * What[n][k],  What = s*(q - z) (Sec. 3.2, Eq. 10) with the FP16
//   outliers written over their (zero-decoding) codes.
//
// A block owns a BM x 128 tile of Y (BM = 256, or 128 for small M) and walks K in steps of 64 (half
// a group).  Per step X[BM][64] and the dequantised weights What[128][64] are staged as FP16 in LDS
// (double-buffered) and multiplied with 32x32x16 FP16 MFMA tiles, FP32 accumulators, FP16 store.
//
// The 12 waves of a block have two roles, three waves per SIMD:
//   * 8 consumers (4 along m, 2 along n) do nothing but read fragments from LDS and issue MFMAs;
//   * 4 producers stage the next step: X rows from memory to LDS, codes to FP16 (exact q - z, one
//     multiply by the scale) to LDS, then the channel's outliers over their decoded zeros.
// A wave can issue next to nothing while one of its own MFMAs runs (measured: about a quarter of
// the MFMA's 32 cycles are free), so staging done by the multiplying waves themselves is time added
// to theirs; done by other waves of the SIMD it is hidden.  LDS stores are the scarcest resource
// (about 64 bytes per clock and CU, a quarter of the load rate), so nothing is stored twice.
//
// Everything a step needs from memory is requested two steps (X) or one group (codes, scale, zero
// point, outliers) ahead, with addresses that do not depend on loaded data, so no producer waits
// for memory inside the loop.  For the outliers this needs to know, per channel and group, how many
// CSR entries fall into the group: a small kernel counts them into the workspace first (one byte
// per channel and group); the running sum is the index of the group's first entry, and its first
// eight entries are fetched ahead by the channel's two threads with unaligned loads (longer runs
// take a slow path).  Scales, zero points and counts are fetched four groups at a time, again with
// one unaligned load each.
#include "gwq_dequant.h"
#include "gwq_internal.h"

namespace gwq {
namespace {

typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kConsumers = 8, kProducers = 4;          // waves
constexpr int kThreads = 64 * (kConsumers + kProducers);
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

// A 16-bit load that is complete when it returns, invisible to the compiler's bookkeeping of
// outstanding loads: for the rare path inside the staging loop, whose loads would otherwise make
// the compiler wait for every prefetch in flight at each trip of the loop.
__device__ inline uint32_t load_u16_now(const uint16_t *p)
{
    uint32_t v;
    asm volatile("global_load_ushort %0, %1, off\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
    return v;
}

// Loads of 8 / 4 bytes at 2-byte / 1-byte alignment (gfx950 global memory takes unaligned addresses).
struct __attribute__((packed, aligned(2))) U64a2 { uint32_t lo, hi; };
struct __attribute__((packed, aligned(2))) U32a2 { uint32_t v; };
struct __attribute__((packed, aligned(1))) U32a1 { uint32_t v; };

// What producer thread (n, h) fetches for one group of channel n: its two slots (h and 2 + h: columns
// 32h .. 32h+31 of the group's two steps) and entries 4h .. 4h+3 of the group's first eight outliers,
// as packed 16-bit pairs.
template <int BITS> struct GroupRegs {
    SlotRegs<BITS> slot[2];
    uint32_t col_lo, col_hi, val_lo, val_hi;
};
// Scales, zero points and outlier counts of four consecutive groups of channel n.  (Plain words:
// the unaligned loads go through temporaries, so these stay in registers.)
struct MetaRegs {
    uint64_t sc;
    uint32_t zp, cnt;
};

// Fragment j (8 codes -> 8 FP16 values s*(q - z)) of a slot.
__device__ inline u32x4 dequant_frag(const SlotRegs<4> &r, int j, uint32_t z, uint32_t s2, const DecodeConsts &d)
{
    const ZeroConsts<4> c(z);
    u32x4 f = decode_word4(r.w[j], c, d);
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

// MSW = 32-row sub-tiles per consumer wave along m; the block tile is BM = 128 * MSW rows by 128
// channels.
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

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int gpr = K / kGroup;
    const int nk = K / kBK;                             // steps; two per group

    // Both roles pass the block's barrier exactly 1 + nk times: once when step 0 is staged, then
    // once per step (the consumers in the middle of the step's last k-batch).
    if (wave >= kConsumers) {
        // ======================================= producers =====================================
        constexpr int kAPasses = BM / 32;               // 256 threads move 32 rows x 128 bytes per pass
        const int ptid = tid - 64 * kConsumers;
        const int a_row = ptid >> 3, a_chunk = ptid & 7;   // 8 threads cover one 128-byte row of a step
        const int b_n_local = ptid >> 1, b_h = ptid & 1;
        int b_n = n0 + b_n_local;
        const bool b_valid = b_n < N;
        b_n = b_valid ? b_n : N - 1;                    // clamped: loads stay in bounds, tile row unused
        const DecodeConsts dc(BITS);

        const _Float16 *a_src[kAPasses];
#pragma unroll
        for (int p = 0; p < kAPasses; ++p) {
            int m = m0 + p * 32 + a_row;
            m = m < M ? m : M - 1;
            a_src[p] = X + (size_t)m * K + 8 * a_chunk;
        }
        const uint32_t row_group = (uint32_t)b_n * gpr;
        const uint32_t *q_row = qweight + (size_t)row_group * wpg;
        _Float16 *const a_dst = lds + a_row * kLd + 8 * a_chunk;            // + buffer, + pass * 32 rows
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
            load_slot<BITS>(G.slot[0], grp, b_h);
            load_slot<BITS>(G.slot[1], grp, 2 + b_h);
            const int j = first + 4 * b_h < last_entry ? first + 4 * b_h : last_entry;   // arrays carry 16 spare bytes
            const U64a2 c = *reinterpret_cast<const U64a2 *>(col_idx + j), v = *reinterpret_cast<const U64a2 *>(out_val + j);
            G.col_lo = c.lo; G.col_hi = c.hi; G.val_lo = v.lo; G.val_hi = v.hi;
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

        // Staging of step `step` into buffer `buf`: this thread's 32 columns of weights, then its four
        // outlier entries (anywhere in the step's 64 columns: the thread that decoded those columns
        // is the lane next to this one and its stores were issued before), then the X rows, whose
        // registers are refilled with the rows of two steps later.
        auto stage = [&](int step, int buf, u32x4 a_regs[kAPasses], const GroupRegs<BITS> &G, const MetaRegs &Q,
                         int first) {
            _Float16 *A = a_dst + buf * kBufHalves, *brow = b_dst + buf * kBufHalves;
            const int half = step & 1, g = step >> 1;
            const uint32_t s2 = meta_scale(Q, g), z = meta_zero(Q, g);
            if constexpr (BITS == 4) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    *reinterpret_cast<u32x4 *>(brow + 32 * b_h + 8 * j) = dequant_frag(G.slot[half], j, z, s2, dc);
            } else {
                u32x4 f[4];
                dequant_all(G.slot[half], z, s2, dc, f);
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(brow + 32 * b_h + 8 * j) = f[j];
            }
            const int cnt = meta_count(Q, g);
            const uint32_t k_lo = (uint32_t)(step * kBK);
            const uint32_t cs[2] = {G.col_lo, G.col_hi}, vs[2] = {G.val_lo, G.val_hi};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t col = ((cs[i >> 1] >> (16 * (i & 1))) & 0xFFFFu) - k_lo;
                if (4 * b_h + i < cnt && col < (uint32_t)kBK)
                    brow[col] = __builtin_bit_cast(_Float16, (uint16_t)(vs[i >> 1] >> (16 * (i & 1))));
            }
            if (b_h == 0)
                for (int i = kAhead; i < cnt; ++i) {    // rare: more than kAhead outliers in one group
                    const uint32_t c = load_u16_now(col_idx + first + i) - k_lo;
                    if (c < (uint32_t)kBK) brow[c] = __builtin_bit_cast(_Float16, (uint16_t)load_u16_now(out_val + first + i));
                }
            const int k2 = (step + 2 < nk ? step + 2 : nk - 1) * kBK;
#pragma unroll
            for (int p = 0; p < kAPasses; ++p) {
                *reinterpret_cast<u32x4 *>(A + p * 32 * kLd) = a_regs[p];
                a_regs[p] = *reinterpret_cast<const u32x4 *>(a_src[p] + k2);
            }
        };

        // Prologue: metadata of groups 0..7, codes and outliers of groups 0 and 1, the X rows of
        // steps 0 and 1; step 0 staged.
        MetaRegs Qc, Qn;                                // groups 4q .. 4q+3 and the four after them
        GroupRegs<BITS> G0, G1;                         // even groups, odd groups
        u32x4 a0[kAPasses], a1[kAPasses];               // X rows of the even / odd step being staged
        int first_c = b_valid ? row_ptr[b_n] : 0;       // CSR index of the current group's first entry
        issue_meta(0, Qc);
        issue_meta(1, Qn);
        issue_a(0, a0);
        issue_a(1, a1);
        issue_group(0, first_c, G0);
        int first_n = first_c + meta_count(Qc, 0);
        issue_group(1, first_n, G1);
        stage(0, 0, a0, G0, Qc, first_c);               // refills a0 with the rows of step 2
        __syncthreads();

        // One group (two steps) per trip.  Entering trip g: buffer 0 holds step 2g, a1 holds the X
        // rows of step 2g + 1, a0 those of step 2g + 2 (in flight), Gcur is group g, Gnxt is group
        // g + 1 (in flight), Qc covers group g, Qn the four groups after Qc's.  Gcur is refilled with
        // group g + 2 at the end, so the two register sets swap roles from trip to trip and a set
        // is never copied (a copy would have to wait for loads that were only just issued).
        // (The scheduling fences keep every request where it is written: left alone, the compiler moves
        // loads down towards their use, and then waits for them.)
        auto trip = [&](int g, GroupRegs<BITS> &Gcur, GroupRegs<BITS> &Gnxt) {
            stage(2 * g + 1, 1, a1, Gcur, Qc, first_c); // second half of group g, while step 2g multiplies
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            const bool roll = (g & 3) == 3;             // group g + 1 starts the next four
            if (g + 1 < gpr) {
                MetaRegs Qs;                            // selected by value: a reference would pin both in memory
                Qs.sc = roll ? Qn.sc : Qc.sc;
                Qs.zp = roll ? Qn.zp : Qc.zp; Qs.cnt = roll ? Qn.cnt : Qc.cnt;
                stage(2 * g + 2, 0, a0, Gnxt, Qs, first_n);   // first half of group g + 1, while step 2g + 1 multiplies
            }
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            if (roll) {
                Qc = Qn;
                issue_meta((g + 1) / 4 + 1, Qn);
            }
            first_c = first_n;
            first_n = first_c + meta_count(Qc, g + 1);
            issue_group(g + 2, first_n, Gcur);
            __builtin_amdgcn_sched_barrier(0);
        };
        int g = 0;
        for (; g + 1 < gpr; g += 2) {                   // no path skips half of the body: the compiler's count of
            trip(g, G0, G1);                            // loads in flight at the top of the loop stays exact
            trip(g + 1, G1, G0);
        }
        if (g < gpr) trip(g, G0, G1);
        return;
    }

    // ========================================= consumers =======================================
    const int wm = wave >> 1, wn = wave & 1;            // 4 x 2 waves, each (BM / 4) x 64
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

    __syncthreads();                                    // step 0 is staged
    read_frags(0, 0, fa[0], fb[0]);
    // One step: each k-batch first requests the fragments of the batch after it, then multiplies.
    // The barrier sits in the middle of the last batch: behind it the first fragments of the next
    // step are requested while the rest of the batch still multiplies.
    constexpr int h = MSW >= 2 ? MSW / 2 : 1;           // rows of the last batch ahead of the barrier
    for (int step = 0; step < nk; ++step) {
        const int buf = step & 1;
        read_frags(buf, 1, fa[1], fb[1]);
        fence();
        mfma_rows(0, 0, MSW);
        fence();
        read_frags(buf, 2, fa[0], fb[0]);
        fence();
        mfma_rows(1, 0, MSW);
        fence();
        read_frags(buf, 3, fa[1], fb[1]);
        fence();
        mfma_rows(2, 0, MSW);
        fence();
        mfma_rows(3, 0, h);
        fence();
        __syncthreads();
        read_frags(buf ^ 1, 0, fa[0], fb[0]);
        fence();
        mfma_rows(3, h, MSW);
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
