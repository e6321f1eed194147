// gwq_linear for M > 16 on gfx950: an MFMA GEMM that dequantises the packed weights on the fly.
//
//   Y[m][n] = sum_k X[m][k] * What[n][k],  What = s*(q - z) (Sec. 3.2, Eq. 10) with the FP16
//   outliers written over their (zero-decoding) codes.
//
// A block of 4 waves owns a BM x 128 tile of Y and walks K in steps of 64 (half a group).  Per
// step the block stages X[BM][64] and the dequantised weights What[128][64] as FP16 in LDS
// (double-buffered; the next step's global loads are in flight while the current one computes).
// Thread (n = tid / 2, h = tid % 2) owns slot h of the step for channel n: it turns 32 codes into
// FP16 (AND-OR into the mantissa of a power of two, exact subtract of the zero point, one
// multiply by the scale), stores them, and then overwrites the positions of channel n's outliers
// that fall into its 32 columns, walking the channel's sorted CSR row with a cursor.  The waves
// (2 x 2) multiply 32x32x16 FP16 MFMA tiles with FP32 accumulators and store FP16.
#include "gwq_internal.h"

namespace gwq {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kBN = 128;
constexpr int kBK = 64;
constexpr int kLd = kBK + 8;            // LDS row stride in halves: 144 bytes, conflict-free b128 reads

union Frag {
    half8 h;
    half2v h2[4];
    uint4 u;
};

__device__ inline half2v splat(float v)
{
    half2v r;
    r.x = (_Float16)v;
    r.y = (_Float16)v;
    return r;
}
__device__ inline half2v code_pair(uint32_t x, uint32_t mask, uint32_t magic)
{
    return __builtin_bit_cast(half2v, (x & mask) | magic);
}

template <int BITS> struct SlotRegs;
template <> struct SlotRegs<4> { uint4 w; };
template <> struct SlotRegs<3> { uint32_t w[3], tail; };

template <int BITS>
__device__ inline void load_slot(SlotRegs<BITS> &r, const uint32_t *group, int slot);
template <> __device__ inline void load_slot<4>(SlotRegs<4> &r, const uint32_t *group, int slot)
{
    r.w = *reinterpret_cast<const uint4 *>(group + 4 * slot);
}
template <> __device__ inline void load_slot<3>(SlotRegs<3> &r, const uint32_t *group, int slot)
{
    const uint32_t *p = group + 3 * slot;
    r.w[0] = p[0]; r.w[1] = p[1]; r.w[2] = p[2];
    r.tail = group[12];
}

// 32 codes -> 32 FP16 values s*(q - z), as four 16-byte fragments in k order.
__device__ inline void dequant_slot(const SlotRegs<4> &r, int /*slot*/, int z, float s, Frag f[4])
{
    const half2v c1024 = splat(-(1024.f + z)), c64 = splat(-(64.f + z)), sc = splat(s);
    const uint32_t ww[4] = {r.w.x, r.w.y, r.w.z, r.w.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t x = ww[j], y = x >> 8;
        f[j].h2[0] = (code_pair(x, 0x000F000Fu, 0x64006400u) + c1024) * sc;
        f[j].h2[1] = (code_pair(x, 0x00F000F0u, 0x54005400u) + c64) * sc;
        f[j].h2[2] = (code_pair(y, 0x000F000Fu, 0x64006400u) + c1024) * sc;
        f[j].h2[3] = (code_pair(y, 0x00F000F0u, 0x54005400u) + c64) * sc;
    }
}
__device__ inline void dequant_slot(const SlotRegs<3> &r, int slot, int z, float s, Frag f[4])
{
    const half2v c1024 = splat(-(1024.f + z)), c128 = splat(-(128.f + z)), c16 = splat(-(16.f + z)), sc = splat(s);
    half2v p[16];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const uint32_t x = r.w[i], y = x >> 9;
        p[5 * i + 0] = (code_pair(x, 0x00070007u, 0x64006400u) + c1024) * sc;
        p[5 * i + 1] = (code_pair(x, 0x00380038u, 0x58005800u) + c128) * sc;
        p[5 * i + 2] = (code_pair(x, 0x01C001C0u, 0x4C004C00u) + c16) * sc;
        p[5 * i + 3] = (code_pair(y, 0x00070007u, 0x64006400u) + c1024) * sc;
        p[5 * i + 4] = (code_pair(y, 0x00380038u, 0x58005800u) + c128) * sc;
    }
    p[15] = (code_pair(r.tail >> (3 * slot), 0x00070007u, 0x64006400u) + c1024) * sc;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) f[j].h2[e] = p[4 * j + e];
}

// MS = 32-row sub-tiles per wave along m; the block tile is BM = 64 * MS rows by 128 channels.
template <int BITS, int MS>
__global__ __launch_bounds__(kThreads) void gemm_kernel(const uint32_t *__restrict__ qweight,
                                                        const uint16_t *__restrict__ scales,
                                                        const uint8_t *__restrict__ zeros,
                                                        const int32_t *__restrict__ row_ptr,
                                                        const uint16_t *__restrict__ col_idx,
                                                        const uint16_t *__restrict__ out_val,
                                                        const _Float16 *__restrict__ X, _Float16 *__restrict__ Y,
                                                        int N, int K, int M, int tiles_m, int tiles_n)
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
    const int nk = K / kBK;

    // Global -> register staging.
    const int a_row = tid >> 3, a_chunk = tid & 7;      // 8 threads cover one 128-byte row of the step
    const int b_n_local = tid >> 1, b_h = tid & 1;
    int b_n = n0 + b_n_local;
    const bool b_valid = b_n < N;
    b_n = b_valid ? b_n : N - 1;
    uint4 a_regs[kAPasses];
    SlotRegs<BITS> b_regs;
    float b_scale = 0.f;
    int b_zero = 0;

    // Outlier cursor of this thread's channel.
    int cur = b_valid ? row_ptr[b_n] : 0;
    const int cur_end = b_valid ? row_ptr[b_n + 1] : 0;
    int next_col = cur < cur_end ? (int)col_idx[cur] : 0x7FFFFFFF;

    auto load_tile = [&](int it) {
        const int k0 = it * kBK;
#pragma unroll
        for (int p = 0; p < kAPasses; ++p) {
            int m = m0 + p * 32 + a_row;
            m = m < M ? m : M - 1;
            a_regs[p] = *reinterpret_cast<const uint4 *>(X + (size_t)m * K + k0 + 8 * a_chunk);
        }
        const int g = it >> 1, slot = 2 * (it & 1) + b_h;
        load_slot<BITS>(b_regs, qweight + ((size_t)b_n * gpr + g) * wpg, slot);
        b_scale = (float)__builtin_bit_cast(_Float16, scales[(size_t)b_n * gpr + g]);
        b_zero = zeros[(size_t)b_n * gpr + g];
    };
    auto store_tile = [&](int it, int buf) {
        _Float16 *A = lds + buf * kBufHalves, *B = A + BM * kLd;
#pragma unroll
        for (int p = 0; p < kAPasses; ++p)
            *reinterpret_cast<uint4 *>(A + (p * 32 + a_row) * kLd + 8 * a_chunk) = a_regs[p];
        Frag f[4];
        dequant_slot(b_regs, 2 * (it & 1) + b_h, b_zero, b_scale, f);
        _Float16 *brow = B + b_n_local * kLd;
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<uint4 *>(brow + 32 * b_h + 8 * j) = f[j].u;
        // Outliers of this channel inside this thread's 32 columns replace their decoded zeros.
        const int k_lo = it * kBK + 32 * b_h, k_hi = k_lo + 32;
        while (next_col < k_hi) {
            if (next_col >= k_lo) brow[next_col - it * kBK] = __builtin_bit_cast(_Float16, out_val[cur]);
            ++cur;
            next_col = cur < cur_end ? (int)col_idx[cur] : 0x7FFFFFFF;
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

    load_tile(0);
    store_tile(0, 0);
    __syncthreads();
    for (int it = 0; it < nk; ++it) {
        const int buf = it & 1;
        if (it + 1 < nk) load_tile(it + 1);
        const _Float16 *A = lds + buf * kBufHalves + (wm * (BM / 2) + fi) * kLd + 8 * fk;
        const _Float16 *B = lds + buf * kBufHalves + (BM + wn * 64 + fi) * kLd + 8 * fk;
#pragma unroll
        for (int s = 0; s < kBK / 16; ++s) {
            Frag a[MS], b[2];
#pragma unroll
            for (int i = 0; i < MS; ++i) a[i].u = *reinterpret_cast<const uint4 *>(A + i * 32 * kLd + 16 * s);
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j].u = *reinterpret_cast<const uint4 *>(B + j * 32 * kLd + 16 * s);
#pragma unroll
            for (int i = 0; i < MS; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i].h, b[j].h, acc[i][j], 0, 0, 0);
        }
        if (it + 1 < nk) store_tile(it + 1, buf ^ 1);
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
hipError_t launch_ms(const gwq_packed &P, const void *X, int M, void *Y, hipStream_t st)
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
        P.qweight, P.scales, P.zeros, P.row_ptr, P.col_idx, P.out_val, static_cast<const _Float16 *>(X),
        static_cast<_Float16 *>(Y), P.N, P.K, M, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const gwq_packed &P, const void *X, int M, void *Y, hipStream_t st)
{
    const int ms = M <= 64 ? 1 : M <= 128 ? 2 : 4;
    if (P.bits == 4) return ms == 1 ? launch_ms<4, 1>(P, X, M, Y, st) : ms == 2 ? launch_ms<4, 2>(P, X, M, Y, st) : launch_ms<4, 4>(P, X, M, Y, st);
    return ms == 1 ? launch_ms<3, 1>(P, X, M, Y, st) : ms == 2 ? launch_ms<3, 2>(P, X, M, Y, st) : launch_ms<3, 4>(P, X, M, Y, st);
}

}  // namespace gwq
