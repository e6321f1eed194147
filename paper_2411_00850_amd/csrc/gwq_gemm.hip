// gwq_linear for M > 16 on gfx950: an MFMA GEMM that dequantises the packed weights on the fly.
//
//   Y[m][n] = sum_k X[m][k] * What[n][k],  What = s*(q - z) (Sec. 3.2, Eq. 10) with the FP16
//   outliers written over their (zero-decoding) codes.
//
// A block of 4 waves owns a BM x 128 tile of Y and walks K in steps of 64 (half a group).  Per
// step the block stages X[BM][64] and the dequantised weights What[128][64] as FP16 in LDS
// (double-buffered).  Thread (n = tid / 2, h = tid % 2) owns 32 columns of the step for channel n:
// it turns 32 codes into FP16 (exact q - z, one multiply by the scale), stores them, and then
// overwrites the positions of channel n's outliers that fall into those columns.  The waves
// (2 x 2) multiply 32x32x16 FP16 MFMA tiles with FP32 accumulators and store FP16.
//
// Everything a step needs from memory is requested one step (X) or one group (codes, scale, zero
// point, outliers) ahead, with addresses that do not depend on loaded data, so the only wave of a
// SIMD never waits for memory inside the loop.  For the outliers this needs to know, per channel
// and group, how many CSR entries fall into the group: a small kernel counts them into the
// workspace first (one byte per channel and group); the running sum is the index of the group's
// first entry, and its first three entries are fetched ahead (longer runs take a slow path).
// The staging work of the next step is cut into four parts issued between the four MFMA batches
// of the current one.
#include "gwq_dequant.h"
#include "gwq_internal.h"

namespace gwq {
namespace {

typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kBN = 128;
constexpr int kBK = 64;
constexpr int kLd = kBK + 8;            // LDS row stride in halves: 144 bytes, conflict-free b128 reads
constexpr int kAhead = 3;               // outlier entries per (channel, group) fetched ahead

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

// Everything thread (n, h) needs for one group of channel n: its two slots (h and 2 + h), scale,
// zero point, the number of outliers in the group and the first kAhead of them.
template <int BITS> struct GroupRegs {
    SlotRegs<BITS> slot[2];
    uint16_t sc;
    uint8_t zp, cnt;
    uint16_t col[kAhead], val[kAhead];
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

// MS = 32-row sub-tiles per wave along m; the block tile is BM = 64 * MS rows by 128 channels.
template <int BITS, int MS>
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
    constexpr int BM = 64 * MS;
    constexpr int wpg = words_per_group(BITS);
    constexpr int kAPasses = BM / 32;                   // 256 threads move 32 rows x 128 bytes per pass
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

    // Staging roles.
    const int a_row = tid >> 3, a_chunk = tid & 7;      // 8 threads cover one 128-byte row of a step
    const int b_n_local = tid >> 1, b_h = tid & 1;
    int b_n = n0 + b_n_local;
    const bool b_valid = b_n < N;
    b_n = b_valid ? b_n : N - 1;                        // clamped: loads stay in bounds, tile row unused
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
    // first = CSR index of the group's first entry (data-independent of anything in flight).
    auto issue_group = [&](int g, int first, GroupRegs<BITS> &G) {
        g = g < gpr ? g : gpr - 1;
        const uint32_t *grp = q_row + (uint32_t)g * wpg;
        load_slot<BITS>(G.slot[0], grp, b_h);
        load_slot<BITS>(G.slot[1], grp, 2 + b_h);
        G.sc = scales[row_group + g];
        G.zp = zeros[row_group + g];
        const uint8_t cnt_raw = grp_cnt[row_group + g];
        G.cnt = b_valid ? cnt_raw : (uint8_t)0;
#pragma unroll
        for (int i = 0; i < kAhead; ++i) {
            const int j = first + i < last_entry ? first + i : last_entry;
            G.col[i] = col_idx[j];
            G.val[i] = out_val[j];
        }
    };

    // Store part `part` (0..3) of step `step` into buffer `buf`: a quarter of the X rows and one
    // 8-column fragment of this thread's weights; part 3 also writes the outliers.
    auto store_part = [&](int part, int step, int buf, const u32x4 a_regs[kAPasses], const GroupRegs<BITS> &G,
                          int first) {
        _Float16 *A = a_dst + buf * kBufHalves, *brow = b_dst + buf * kBufHalves;
        const int half = step & 1;
        constexpr int per = kAPasses >= 4 ? kAPasses / 4 : 1;
#pragma unroll
        for (int p = part * per; p < (part + 1) * per && p < kAPasses; ++p)
            *reinterpret_cast<u32x4 *>(A + p * 32 * kLd) = a_regs[p];
        const uint32_t s2 = (uint32_t)G.sc | (uint32_t)G.sc << 16;
        if constexpr (BITS == 4) {
            *reinterpret_cast<u32x4 *>(brow + 32 * b_h + 8 * part) = dequant_frag(G.slot[half], part, G.zp, s2, dc);
        } else {
            if (part == 0) {
                u32x4 f[4];
                dequant_all(G.slot[half], G.zp, s2, dc, f);
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(brow + 32 * b_h + 8 * j) = f[j];
            }
        }
        if (part == 3) {
            // Outliers of this channel inside this thread's 32 columns replace their decoded zeros.
            const int k_lo = step * kBK + 32 * b_h;
#pragma unroll
            for (int i = 0; i < kAhead; ++i) {
                const uint32_t c = (uint32_t)G.col[i] - (uint32_t)k_lo;
                if (i < G.cnt && c < 32u) brow[32 * b_h + c] = __builtin_bit_cast(_Float16, G.val[i]);
            }
            for (int i = kAhead; i < G.cnt; ++i) {      // rare: more than kAhead outliers in one group
                const uint32_t c = (uint32_t)col_idx[first + i] - (uint32_t)k_lo;
                if (c < 32u) brow[32 * b_h + c] = __builtin_bit_cast(_Float16, out_val[first + i]);
            }
        }
    };

    float16v acc[MS][2];
#pragma unroll
    for (int i = 0; i < MS; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int fi = lane & 31, fk = lane >> 5;           // fragment row and k-block of this lane
    const _Float16 *a_frag = lds + (wm * (BM / 2) + fi) * kLd + 8 * fk;
    const _Float16 *b_frag = lds + (BM + wn * 64 + fi) * kLd + 8 * fk;

    // One step: MFMA on buffer `buf` in four k-batches, the staging of step + 1 (from a_regs, G)
    // into the other buffer spread between them.
    auto step_fn = [&](int step, int buf, const u32x4 a_regs[kAPasses], const GroupRegs<BITS> &G, int first) {
        const _Float16 *A = a_frag + buf * kBufHalves, *B = b_frag + buf * kBufHalves;
        const bool stage = step + 1 < nk;
#pragma unroll
        for (int s = 0; s < kBK / 16; ++s) {
            u32x4 a[MS], b[2];
#pragma unroll
            for (int i = 0; i < MS; ++i) a[i] = *reinterpret_cast<const u32x4 *>(A + i * 32 * kLd + 16 * s);
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const u32x4 *>(B + j * 32 * kLd + 16 * s);
#pragma unroll
            for (int i = 0; i < MS; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a[i]),
                                                                       __builtin_bit_cast(half8, b[j]), acc[i][j], 0, 0, 0);
            if (stage) store_part(s, step + 1, buf ^ 1, a_regs, G, first);
        }
    };

    // Prologue: group 0 and the X rows of steps 0 and 1; step 0 staged; group 1 requested.
    GroupRegs<BITS> Gc, Gn;                             // current group, next group
    u32x4 a0[kAPasses], a1[kAPasses];                   // X rows of the even / odd step being staged
    int first_c = b_valid ? row_ptr[b_n] : 0;           // CSR index of the current group's first entry
    issue_group(0, first_c, Gc);
    issue_a(0, a0);
    issue_a(1, a1);
    int first_n = first_c + Gc.cnt;
    issue_group(1, first_n, Gn);
#pragma unroll
    for (int part = 0; part < 4; ++part) store_part(part, 0, 0, a0, Gc, first_c);
    issue_a(2, a0);
    __syncthreads();

    // Main loop, one group (two steps) per trip.  Entering trip g: buffer 0 holds step 2g, a1
    // holds the X rows of step 2g + 1, a0 those of step 2g + 2 (in flight), Gc is group g, Gn is
    // group g + 1 (in flight).
    for (int g = 0; g < gpr; ++g) {
        step_fn(2 * g, 0, a1, Gc, first_c);             // stages step 2g + 1 (second half of group g)
        issue_a(2 * g + 3, a1);
        __syncthreads();
        // Second half: stage step 2g + 2 = first half of group g + 1, then move on to it.
        step_fn(2 * g + 1, 1, a0, Gn, first_n);
        issue_a(2 * g + 4, a0);
        Gc = Gn;
        first_c = first_n;
        first_n = first_c + Gc.cnt;
        issue_group(g + 2, first_n, Gn);
        __syncthreads();
    }

    // D layout of the 32x32 tile: column = lane % 32, row = 8*(v/4) + 4*(lane/32) + v%4.
#pragma unroll
    for (int i = 0; i < MS; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn * 64 + j * 32 + fi;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * (BM / 2) + i * 32 + 8 * (v >> 2) + 4 * fk + (v & 3);
                if (m < M && n < N) Y[(size_t)m * N + n] = (_Float16)acc[i][j][v];
            }
        }
}

template <int BITS, int MS>
hipError_t launch_ms(const gwq_packed &P, const void *X, int M, void *Y, uint8_t *grp_cnt, hipStream_t st)
{
    constexpr int BM = 64 * MS;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (P.N + kBN - 1) / kBN;
    const size_t lds = (size_t)2 * (BM + kBN) * kLd * sizeof(_Float16);
    static bool attr_set = false;                       // per instantiation; idempotent HIP call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel<BITS, MS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    gemm_kernel<BITS, MS><<<tiles_m * tiles_n, kThreads, lds, st>>>(
        P.qweight, P.scales, P.zeros, P.row_ptr, P.col_idx, P.out_val, grp_cnt, static_cast<const _Float16 *>(X),
        static_cast<_Float16 *>(Y), P.N, P.K, M, tiles_m, tiles_n, P.n_outliers > 0 ? (int)P.n_outliers - 1 : 0);
    return hipGetLastError();
}

}  // namespace

size_t gemm_workspace_bytes(int64_t N, int64_t K) { return (size_t)(N * (K / kGroup) + 255) / 256 * 256; }

hipError_t launch_gemm(const gwq_packed &P, const void *X, int M, void *Y, void *workspace, hipStream_t st)
{
    uint8_t *cnt = static_cast<uint8_t *>(workspace);
    group_count_kernel<<<(P.N + 3) / 4, 256, 0, st>>>(P.row_ptr, P.col_idx, P.N, P.K / kGroup, cnt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int ms = M <= 64 ? 1 : M <= 128 ? 2 : 4;
    if (P.bits == 4)
        return ms == 1 ? launch_ms<4, 1>(P, X, M, Y, cnt, st) : ms == 2 ? launch_ms<4, 2>(P, X, M, Y, cnt, st)
                                                                         : launch_ms<4, 4>(P, X, M, Y, cnt, st);
    return ms == 1 ? launch_ms<3, 1>(P, X, M, Y, cnt, st) : ms == 2 ? launch_ms<3, 2>(P, X, M, Y, cnt, st)
                                                                     : launch_ms<3, 4>(P, X, M, Y, cnt, st);
}

}  // namespace gwq
