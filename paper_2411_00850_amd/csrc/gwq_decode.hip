// gwq_linear for M <= 16 on gfx950: a bandwidth-bound fused dequantise-and-multiply.
//
//   Y[m][n] = sum_g s[n][g] * sum_{k in g} X[m][k] * (q[n][k] - z[n][g])   (Sec. 3.2, Eq. 10)
//           + sum_{j in CSR row n} out_val[j] * X[m][col_idx[j]]            (the FP16 outliers)
//
// Mapping.  A block owns 16*T output channels; its waves split K by whole groups of 128.  A wave
// feeds v_mfma_f32_16x16x32_f16 with X as the 16 x 32 operand (rows m, zero beyond M) and the
// dequantised codes as the 32 x 16 operand (columns n): lane (r = lane % 16, b = lane / 16) owns
// slot b of each group of channel n0 + r, i.e. 32 consecutive codes = one 16-byte load (4-bit) or
// a 12-byte load plus the shared tail word (3-bit).  Codes become the exact FP16 integers q - z
// with one AND-OR and one packed add per pair (the code bits are dropped into the mantissa of a
// power of two); the group scale is applied to the four FP32 results per lane after the group's
// four MFMAs.  Each lane then adds its channel's outliers for its own four m, the waves' partial
// sums meet in LDS in a fixed order, and one thread per output rounds to FP16 and stores.
// No atomics, no second pass: results are run-to-run identical.
#include "gwq_internal.h"

namespace gwq {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));

union Frag {
    half8 h;
    half2v h2[4];
    uint4 u;
};

__device__ inline half2v bits_to_half2(uint32_t x) { return __builtin_bit_cast(half2v, x); }

__device__ inline half2v splat(float v)
{
    half2v r;
    r.x = (_Float16)v;
    r.y = (_Float16)v;
    return r;
}

// (x & mask) | magic reinterpreted as two FP16 values: 2^e + code, exactly.
__device__ inline half2v code_pair(uint32_t x, uint32_t mask, uint32_t magic)
{
    return bits_to_half2((x & mask) | magic);
}

// 32 codes of one slot -> four MFMA operands holding q - z.
template <int BITS> struct Slot;

template <> struct Slot<4> {
    uint4 w;
    __device__ inline void load(const uint32_t *group, int b) { w = *reinterpret_cast<const uint4 *>(group + 4 * b); }
    __device__ inline void dequant(int z, int /*b*/, Frag f[4]) const
    {
        const half2v c1024 = splat(-(1024.f + z)), c64 = splat(-(64.f + z));
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t x = ww[j], y = x >> 8;
            f[j].h2[0] = code_pair(x, 0x000F000Fu, 0x64006400u) + c1024;   // 1024 + q
            f[j].h2[1] = code_pair(x, 0x00F000F0u, 0x54005400u) + c64;     // 64 + q
            f[j].h2[2] = code_pair(y, 0x000F000Fu, 0x64006400u) + c1024;
            f[j].h2[3] = code_pair(y, 0x00F000F0u, 0x54005400u) + c64;
        }
    }
};

template <> struct Slot<3> {
    uint32_t w[3], tail;
    __device__ inline void load(const uint32_t *group, int b)
    {
        const uint32_t *p = group + 3 * b;
        w[0] = p[0]; w[1] = p[1]; w[2] = p[2];
        tail = group[12];
    }
    __device__ inline void dequant(int z, int b, Frag f[4]) const
    {
        const half2v c1024 = splat(-(1024.f + z)), c128 = splat(-(128.f + z)), c16 = splat(-(16.f + z));
        half2v p[16];
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const uint32_t x = w[i], y = x >> 9;
            p[5 * i + 0] = code_pair(x, 0x00070007u, 0x64006400u) + c1024;   // 1024 + q
            p[5 * i + 1] = code_pair(x, 0x00380038u, 0x58005800u) + c128;    // 128 + q
            p[5 * i + 2] = code_pair(x, 0x01C001C0u, 0x4C004C00u) + c16;     // 16 + q
            p[5 * i + 3] = code_pair(y, 0x00070007u, 0x64006400u) + c1024;
            p[5 * i + 4] = code_pair(y, 0x00380038u, 0x58005800u) + c128;
        }
        p[15] = code_pair(tail >> (3 * b), 0x00070007u, 0x64006400u) + c1024;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) f[j].h2[e] = p[4 * j + e];
    }
};

template <int BITS, int T>
__global__ __launch_bounds__(1024) void decode_kernel(const uint32_t *__restrict__ qweight,
                                                      const uint16_t *__restrict__ scales,
                                                      const uint8_t *__restrict__ zeros,
                                                      const int32_t *__restrict__ row_ptr,
                                                      const uint16_t *__restrict__ col_idx,
                                                      const uint16_t *__restrict__ out_val,
                                                      const _Float16 *__restrict__ X, _Float16 *__restrict__ Y,
                                                      int N, int K, int M, int groups_per_wave)
{
    extern __shared__ float red[];                      // [waves][T][4][64]
    constexpr int wpg = words_per_group(BITS);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int r = lane & 15, b = lane >> 4;
    const int gpr = K / kGroup;
    const int row0 = blockIdx.x * (16 * T);

    size_t row_off[T];                                  // group index of (channel, group 0)
#pragma unroll
    for (int t = 0; t < T; ++t) {
        int n = row0 + 16 * t + r;
        n = n < N ? n : N - 1;                          // clamped: loads stay in bounds, result unused
        row_off[t] = (size_t)n * gpr;
    }
    float4v acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t) acc[t] = float4v{0.f, 0.f, 0.f, 0.f};

    const int g_begin = wave * groups_per_wave;
    const int g_end = g_begin + groups_per_wave < gpr ? g_begin + groups_per_wave : gpr;
    const bool has_x = r < M;
    const _Float16 *xp = X + (size_t)(has_x ? r : 0) * K + 32 * b;

    for (int g = g_begin; g < g_end; ++g) {
        Frag xa[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            xa[j].u = has_x ? *reinterpret_cast<const uint4 *>(xp + (size_t)g * kGroup + 8 * j) : uint4{0, 0, 0, 0};
        Slot<BITS> slot[T];
        float s[T];
        int z[T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            slot[t].load(qweight + (row_off[t] + g) * wpg, b);
            s[t] = (float)__builtin_bit_cast(_Float16, scales[row_off[t] + g]);
            z[t] = zeros[row_off[t] + g];
        }
#pragma unroll
        for (int t = 0; t < T; ++t) {
            Frag wb[4];
            slot[t].dequant(z[t], b, wb);
            float4v part = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j)
                part = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[j].h, wb[j].h, part, 0, 0, 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[t][e] = __builtin_fmaf(s[t], part[e], acc[t][e]);
        }
    }

    // FP16 outliers of this lane's channel, for the lane's own rows m = 4b .. 4b+3.
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int n = row0 + 16 * t + r;
        if (n < N && 4 * b < M) {
            const int j1 = row_ptr[n + 1];
            for (int j = row_ptr[n] + wave; j < j1; j += nwaves) {
                const int col = col_idx[j];
                const float v = (float)__builtin_bit_cast(_Float16, out_val[j]);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (4 * b + e < M) acc[t][e] = __builtin_fmaf(v, (float)X[(size_t)(4 * b + e) * K + col], acc[t][e]);
            }
        }
    }

    // Fixed-order reduction over the waves, then FP16 store.
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) red[((wave * T + t) * 4 + e) * 64 + lane] = acc[t][e];
    __syncthreads();
    for (int idx = threadIdx.x; idx < T * 256; idx += blockDim.x) {
        float sum = 0.f;
        for (int w = 0; w < nwaves; ++w) sum += red[w * T * 256 + idx];
        const int t = idx >> 8, e = (idx >> 6) & 3, l = idx & 63;
        const int n = row0 + 16 * t + (l & 15), m = 4 * (l >> 4) + e;
        if (n < N && m < M) Y[(size_t)m * N + n] = (_Float16)sum;
    }
}

template <int BITS, int T>
hipError_t launch_t(const gwq_packed &P, const void *X, int M, void *Y, int nwaves, int gpw, hipStream_t st)
{
    const int blocks = (P.N + 16 * T - 1) / (16 * T);
    const size_t lds = (size_t)nwaves * T * 1024;
    decode_kernel<BITS, T><<<blocks, nwaves * 64, lds, st>>>(P.qweight, P.scales, P.zeros, P.row_ptr, P.col_idx,
                                                            P.out_val, static_cast<const _Float16 *>(X),
                                                            static_cast<_Float16 *>(Y), P.N, P.K, M, gpw);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_decode(const gwq_packed &P, const void *X, int M, void *Y, int tiles_override,
                         int waves_override, hipStream_t st)
{
    const int gpr = P.K / kGroup;
    int T = tiles_override ? tiles_override : 1;
    const int blocks = (P.N + 16 * T - 1) / (16 * T);
    // Enough waves to keep every CU's memory pipeline full: about 16 per CU over 256 CUs.
    int nwaves = waves_override ? waves_override : (4096 + blocks - 1) / blocks;
    if (nwaves > 16) nwaves = 16;
    if (nwaves > gpr) nwaves = gpr;
    if (nwaves < 1) nwaves = 1;
    if (nwaves * T > 32) nwaves = 32 / T;               // LDS reduction buffer stays <= 32 KB
    const int gpw = (gpr + nwaves - 1) / nwaves;
    nwaves = (gpr + gpw - 1) / gpw;                     // drop waves that would own no group
#define GWQ_DISPATCH(B, TT) \
    if (P.bits == B && T == TT) return launch_t<B, TT>(P, X, M, Y, nwaves, gpw, st)
    GWQ_DISPATCH(4, 1); GWQ_DISPATCH(4, 2); GWQ_DISPATCH(4, 4);
    GWQ_DISPATCH(3, 1); GWQ_DISPATCH(3, 2); GWQ_DISPATCH(3, 4);
#undef GWQ_DISPATCH
    return hipErrorInvalidValue;
}

}  // namespace gwq
