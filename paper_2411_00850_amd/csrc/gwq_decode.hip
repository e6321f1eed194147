// gwq_linear for M <= 16 on gfx950: a bandwidth-bound fused dequantise-and-multiply.
//
//   Y[m][n] = sum_g s[n][g] * sum_{k in g} X[m][k] * (q[n][k] - z[n][g])   (Sec. 3.2, Eq. 10)
//           + sum_{j in CSR row n} out_val[j] * X[m][col_idx[j]]            (the FP16 outliers)
//
// Mapping.  A block owns 16 output channels; its waves split K by whole groups of 128.  A wave
// feeds v_mfma_f32_16x16x32_f16 with X as the 16 x 32 operand (rows m, zero beyond M) and the
// dequantised codes as the 32 x 16 operand (columns n): lane (r = lane % 16, b = lane / 16) owns
// slot b of each group of channel n0 + r, i.e. 32 consecutive codes = one 16-byte load (4-bit) or
// a 12-byte load plus the shared tail word (3-bit).  Codes become the exact FP16 integers q - z
// with one AND-OR and one packed add per pair (the code bits are dropped into the mantissa of a
// power of two); the group scale is applied to the four FP32 results per lane after the group's
// four MFMAs.  Each lane then adds its channel's outliers for its own four m, the waves' partial
// sums meet in LDS in a fixed order, and one thread per output rounds to FP16 and stores.
// No atomics, no second pass: results are run-to-run identical.
//
// Latency.  At these sizes a whole matrix is only a few microseconds of HBM time, so the kernel is
// organised around having every byte requested as early as possible: a wave issues the code loads
// of U groups at once (and of the next U before it computes the current ones), the scales and
// zero points of those groups come in as one load per lane and are handed round with
// ds_bpermute, and the dependent chain of the outliers (row_ptr -> col/val -> X[col]) is started
// before the dense loop so that it overlaps the code stream.
#include "gwq_dequant.h"
#include "gwq_internal.h"

namespace gwq {
namespace {

typedef float float4v __attribute__((ext_vector_type(4)));

// Every load below is unconditional with a clamped (always valid) index, and nothing is combined
// or converted until it is consumed: a conditional load, or arithmetic right behind a load, makes
// the wave wait for that load - and, because loads retire in order, for every older one too.

__device__ inline const uint32_t *at_byte(const uint32_t *base, uint32_t byte_off)
{
    return reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(base) + byte_off);
}

// Registers of one slot (32 codes) as loaded from memory; `off` is a byte offset from qweight.
template <int BITS> struct Slot;
template <> struct Slot<4> {
    uint4 w;
    __device__ inline void load(const uint32_t *q, uint32_t group_off, int b)
    {
        w = *reinterpret_cast<const uint4 *>(at_byte(q, group_off + 16 * b));
    }
    __device__ inline void decode(uint32_t z, int /*b*/, const DecodeConsts &d, u32x4 f[4]) const
    {
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
        decode_slot4(ww, z, d, f);
    }
};
template <> struct Slot<3> {
    uint32_t w[3], tail;
    __device__ inline void load(const uint32_t *q, uint32_t group_off, int b)
    {
        const uint32_t *p = at_byte(q, group_off + 12 * b);
        w[0] = p[0]; w[1] = p[1]; w[2] = p[2];
        tail = *at_byte(q, group_off + 48);
    }
    __device__ inline void decode(uint32_t z, int b, const DecodeConsts &d, u32x4 f[4]) const
    {
        decode_slot3(w, tail >> (3 * b), z, d, f);
    }
};

constexpr int kPre = 4;        // outlier entries per lane fetched ahead of the dense loop

// Codes, scales and zero points of one chunk of U (4 or 8) groups of one channel.
template <int BITS, int U> struct Chunk {
    Slot<BITS> slot[U];
    uint16_t sc[U / 4];        // lane (r, b) holds the scale and zero point of groups g0 + b (+ 4)
    uint8_t zp[U / 4];

    // row_group = index of (channel, group 0); g_last = last valid group of this wave (clamp).
    __device__ inline void load(const uint32_t *qweight, const uint16_t *scales, const uint8_t *zeros,
                                uint32_t row_group, int g0, int g_last, int b)
    {
        constexpr uint32_t group_bytes = words_per_group(BITS) * 4;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = g0 + u < g_last ? g0 + u : g_last;
            slot[u].load(qweight, (row_group + g) * group_bytes, b);
        }
#pragma unroll
        for (int h = 0; h < U / 4; ++h) {
            const int g = g0 + 4 * h + b < g_last ? g0 + 4 * h + b : g_last;
            sc[h] = scales[row_group + g];
            zp[h] = zeros[row_group + g];
        }
    }
};

// BITS: 3 or 4.  U: groups per chunk.  PIPE: a wave owns more than U groups and double-buffers its
// chunks.  MS: 1..4 = M is exactly MS and X[M][K] is staged in LDS once per block, the four lanes
// of a channel sharing its outliers (only without PIPE); 0 = any M <= 16, X read from global memory.
//
// Rows m >= M of the X operand are never zeroed: lanes r >= M re-read row 0, which only produces
// result rows m >= M, and those are not stored.
template <int BITS, int U, bool PIPE, int MS>
__global__ __launch_bounds__(1024) void decode_kernel(const uint32_t *__restrict__ qweight,
                                                      const uint16_t *__restrict__ scales,
                                                      const uint8_t *__restrict__ zeros,
                                                      const int32_t *__restrict__ row_ptr,
                                                      const uint16_t *__restrict__ col_idx,
                                                      const uint16_t *__restrict__ out_val,
                                                      const _Float16 *__restrict__ X, _Float16 *__restrict__ Y,
                                                      int N, int K, int M, int groups_per_wave, int last_entry)
{
    constexpr bool SMALLM = MS > 0;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int r = lane & 15, b = lane >> 4;
    const int gpr = K / kGroup;
    const int row0 = blockIdx.x * 16;
    const int n = row0 + r;
    const int n_c = n < N ? n : N - 1;                  // clamped channel: its results are not stored
    _Float16 *xs = reinterpret_cast<_Float16 *>(lds_raw);                          // [MS][K]
    float *red = reinterpret_cast<float *>(lds_raw + (size_t)MS * K * 2);          // [waves][4][64]

    // Outlier chain, step 1: CSR row bounds of this lane's channel (the first loads issued).
    const int rp0 = row_ptr[n_c], rp1 = row_ptr[n_c + 1];

    const int g_begin = wave * groups_per_wave;
    const int g_end = g_begin + groups_per_wave < gpr ? g_begin + groups_per_wave : gpr;
    const int g_last = g_end - 1;                       // >= g_begin: the launcher gives every wave a group

    // X for LDS staging is requested next: it returns before the code stream does, and its
    // consumers must not have to wait for the (younger) code loads.  Each wave stages the columns
    // of its own groups (the waves partition K), U/4 16-byte vectors per lane and row; lanes past
    // the end of a short slice repeat its last vector.
    constexpr int kXVecs = SMALLM ? MS * (U / 4) : 1;
    u32x4 xstage[kXVecs];
    uint32_t xvec[kXVecs];                              // vector index inside X / xs
    if (SMALLM) {
        const int slice_vecs = (g_end - g_begin) * (kGroup / 8);
#pragma unroll
        for (int e = 0; e < MS; ++e)
#pragma unroll
            for (int i = 0; i < U / 4; ++i) {
                const int q = lane + 64 * i < slice_vecs ? lane + 64 * i : slice_vecs - 1;
                xvec[e * (U / 4) + i] = (uint32_t)e * (K / 8) + g_begin * (kGroup / 8) + q;
                xstage[e * (U / 4) + i] = reinterpret_cast<const u32x4 *>(X)[xvec[e * (U / 4) + i]];
            }
    }

    // The code stream: everything below overlaps its HBM latency.
    const uint32_t row_group = (uint32_t)n_c * gpr;
    Chunk<BITS, U> cur;
    cur.load(qweight, scales, zeros, row_group, g_begin, g_last, b);

    // Outlier chain, step 2: the first kPre entries of this lane.  SMALLM: the four lanes of a
    // channel split its entries; otherwise lane (r, b) takes every entry for rows m = 4b .. 4b+3.
    const int o_stride = SMALLM ? 4 * nwaves : nwaves;
    const int o_first = SMALLM ? 4 * wave + b : wave;
    const bool o_live = n < N && (SMALLM || 4 * b < M);
    uint16_t pre_col[kPre], pre_val[kPre];
    bool pre_ok[kPre];
#pragma unroll
    for (int i = 0; i < kPre; ++i) {
        const int j = rp0 + o_first + i * o_stride;
        pre_ok[i] = o_live && j < rp1;
        const int jc = j < last_entry ? j : last_entry;     // always a valid slot of the arrays
        pre_col[i] = col_idx[jc];
        pre_val[i] = out_val[jc];
    }

    // Nothing that consumes a load may be scheduled above this point.
    __builtin_amdgcn_sched_barrier(0);
    const DecodeConsts dc(BITS);
    if (SMALLM) {
#pragma unroll
        for (int i = 0; i < kXVecs; ++i) reinterpret_cast<u32x4 *>(xs)[xvec[i]] = xstage[i];
        __syncthreads();
    }

    float4v acc = float4v{0.f, 0.f, 0.f, 0.f};
    const int x_row = r < M ? r : 0;
    const _Float16 *xsrc = (SMALLM ? xs : X) + (uint32_t)x_row * K + 32 * b;
    // Groups past the wave's last one (a short final wave) are computed on the clamped, repeated
    // data and dropped by a zero scale: no branch sits between the loads and their use.
    auto compute = [&](const Chunk<BITS, U> &c, int g0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool valid = g0 + u <= g_last;        // wave-uniform
            const int g = valid ? g0 + u : g_last;
            u32x4 xa[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                xa[j] = *reinterpret_cast<const u32x4 *>(xsrc + (uint32_t)g * kGroup + 8 * j);
            const uint32_t mine = (uint32_t)c.sc[u >> 2] | (uint32_t)c.zp[u >> 2] << 16;
            const uint32_t sz = __builtin_amdgcn_ds_bpermute((r + 16 * (u & 3)) * 4, mine);
            const float s = valid ? (float)__builtin_bit_cast(_Float16, (uint16_t)(sz & 0xFFFF)) : 0.f;
            u32x4 wb[4];
            c.slot[u].decode(sz >> 16, b, dc, wb);
            float4v part = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j)
                part = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, xa[j]),
                                                              __builtin_bit_cast(half8, wb[j]), part, 0, 0, 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = __builtin_fmaf(s, part[e], acc[e]);
        }
    };

    if (PIPE) {
        for (int g0 = g_begin; g0 <= g_last; g0 += U) {
            Chunk<BITS, U> nxt;
            const bool more = g0 + U <= g_last;
            if (more) nxt.load(qweight, scales, zeros, row_group, g0 + U, g_last, b);
            compute(cur, g0);
            if (more) cur = nxt;
        }
    } else {
        compute(cur, g_begin);
    }

    // Outlier chain, step 3: X at the prefetched columns, then any entries beyond the window.
    // SMALLM: every lane sums its share of the channel's entries for rows m = 0 .. MS-1 in `oacc`;
    // otherwise the lane covers rows m = 4b .. 4b+3, the rows of its MFMA results.
    float4v oacc = float4v{0.f, 0.f, 0.f, 0.f};
    auto add_outlier = [&](uint32_t col, uint16_t val_bits, bool ok) {
        const float v = ok ? (float)__builtin_bit_cast(_Float16, val_bits) : 0.f;
        if (SMALLM) {
#pragma unroll
            for (int e = 0; e < MS; ++e) oacc[e] = __builtin_fmaf(v, (float)xs[(uint32_t)e * K + col], oacc[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int m = 4 * b + e < M ? 4 * b + e : 0;         // rows m >= M are not stored
                oacc[e] = __builtin_fmaf(v, (float)X[(uint32_t)m * K + col], oacc[e]);
            }
        }
    };
#pragma unroll
    for (int i = 0; i < kPre; ++i) add_outlier(pre_col[i], pre_val[i], pre_ok[i]);
    if (o_live)
        for (int j = rp0 + o_first + kPre * o_stride; j < rp1; j += o_stride) add_outlier(col_idx[j], out_val[j], true);

    // Fixed-order reduction over the waves (and, for SMALLM, over the four lanes of a channel),
    // then FP16 store.  SMALLM: only lanes b = 0 hold dense results for rows m < 4.
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float dense = (!SMALLM || b == 0) ? acc[e] : 0.f;
        red[(wave * 4 + e) * 64 + lane] = dense + oacc[e];
    }
    __syncthreads();
    if (SMALLM) {
        if (threadIdx.x < 16 * MS) {                    // (e, r)
            const int e = threadIdx.x >> 4, rr = threadIdx.x & 15;
            float sum = 0.f;
            for (int w = 0; w < nwaves; ++w)
#pragma unroll
                for (int bb = 0; bb < 4; ++bb) sum += red[(w * 4 + e) * 64 + 16 * bb + rr];
            if (row0 + rr < N) Y[(size_t)e * N + row0 + rr] = (_Float16)sum;
        }
    } else {
        for (int idx = threadIdx.x; idx < 256; idx += blockDim.x) {
            float sum = 0.f;
            for (int w = 0; w < nwaves; ++w) sum += red[w * 256 + idx];
            const int e = idx >> 6, l = idx & 63;
            const int nn = row0 + (l & 15), m = 4 * (l >> 4) + e;
            if (nn < N && m < M) Y[(size_t)m * N + nn] = (_Float16)sum;
        }
    }
}

constexpr size_t kXLdsBudget = 64 * 1024;               // X[M][K] is staged in LDS up to this size

template <int BITS, int U, bool PIPE, int MS>
hipError_t launch_v(const gwq_packed &P, const void *X, int M, void *Y, int nwaves, int gpw, hipStream_t st)
{
    const int blocks = (P.N + 15) / 16;
    const size_t lds = (size_t)nwaves * 1024 + (size_t)MS * P.K * 2;
    static bool attr_set = false;                       // per instantiation; idempotent HIP call
    if (MS > 0 && !attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&decode_kernel<BITS, U, PIPE, MS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)(kXLdsBudget + 16 * 1024));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int last_entry = P.n_outliers > 0 ? (int)P.n_outliers - 1 : 0;
    decode_kernel<BITS, U, PIPE, MS><<<blocks, nwaves * 64, lds, st>>>(
        P.qweight, P.scales, P.zeros, P.row_ptr, P.col_idx, P.out_val, static_cast<const _Float16 *>(X),
        static_cast<_Float16 *>(Y), P.N, P.K, M, gpw, last_entry);
    return hipGetLastError();
}

template <int BITS, int MS>
hipError_t launch_m(const gwq_packed &P, const void *X, int M, void *Y, int nwaves, int gpw, hipStream_t st)
{
    if (gpw <= 4) return launch_v<BITS, 4, false, MS>(P, X, M, Y, nwaves, gpw, st);
    if (gpw <= 8) return launch_v<BITS, 8, false, MS>(P, X, M, Y, nwaves, gpw, st);
    return launch_v<BITS, 4, true, 0>(P, X, M, Y, nwaves, gpw, st);
}

template <int BITS>
hipError_t launch_b(const gwq_packed &P, const void *X, int M, void *Y, int nwaves, int gpw, hipStream_t st)
{
    const bool stage = M <= 4 && (size_t)M * P.K * 2 <= kXLdsBudget;
    if (stage && M == 1) return launch_m<BITS, 1>(P, X, M, Y, nwaves, gpw, st);
    if (stage && M == 2) return launch_m<BITS, 2>(P, X, M, Y, nwaves, gpw, st);
    if (stage && M == 3) return launch_m<BITS, 3>(P, X, M, Y, nwaves, gpw, st);
    if (stage && M == 4) return launch_m<BITS, 4>(P, X, M, Y, nwaves, gpw, st);
    return launch_m<BITS, 0>(P, X, M, Y, nwaves, gpw, st);
}

}  // namespace

hipError_t launch_decode(const gwq_packed &P, const void *X, int M, void *Y, int waves_override, hipStream_t st)
{
    const int gpr = P.K / kGroup;
    // One chunk of eight groups per wave where the row is long enough, at most 16 waves per block.
    int nwaves = waves_override ? waves_override : (gpr + 7) / 8;
    if (nwaves > 16) nwaves = 16;
    if (nwaves > gpr) nwaves = gpr;
    if (nwaves < 1) nwaves = 1;
    const int gpw = (gpr + nwaves - 1) / nwaves;
    nwaves = (gpr + gpw - 1) / gpw;                     // drop waves that would own no group
    return P.bits == 4 ? launch_b<4>(P, X, M, Y, nwaves, gpw, st) : launch_b<3>(P, X, M, Y, nwaves, gpw, st);
}

}  // namespace gwq
