// gwq_linear for M <= 16 on gfx950: a bandwidth-bound fused dequantise-and-multiply.
//
//   Y[m][n] = sum_g s[n][g] * sum_{k in g} X[m][k] * (q[n][k] - z[n][g])   (Sec. 3.2, Eq. 10)
//           + sum_{j in CSR row n} out_val[j] * X[m][col_idx[j]]            (the FP16 outliers)
//
// Mapping.  A block owns 16 output channels; its waves split K by whole groups of 128.  A wave
// feeds v_mfma_f32_16x16x32_f16 with X as the 16 x 32 operand (rows m) and the dequantised codes
// as the 32 x 16 operand (columns n): lane (r = lane % 16, b = lane / 16) owns slot b of each
// group of channel n0 + r, i.e. 32 consecutive codes = one 16-byte load (4-bit) or a 12-byte
// load plus the shared tail word (3-bit).  Codes become the exact FP16 integers q - z with one
// AND-OR and one packed add per pair; the group scale is applied to the four FP32 results per
// lane after the group's four MFMAs.  The lanes then add their channel's outliers, the waves'
// partial sums meet in LDS in a fixed order, and one thread per output rounds to FP16 and stores.
// No atomics, no second pass: results are run-to-run identical.
//
// What bounds it.  A matrix is only a few microseconds of HBM time, and at that scale two things
// matter more than arithmetic:
//   * every byte must be requested at once: all loads are unconditional (clamped indices), issued
//     before anything consumes them, and nothing is converted or combined right behind a load
//     (loads retire in order, so waiting for a young one waits for all older ones);
//   * the address unit of a CU handles a scattered or sub-dword load lane by lane (about 64 cycles
//     per instruction against 16 for a coalesced 16-byte load), so everything except the code
//     stream is fetched with block-wide coalesced 16-byte loads into LDS: the block's scales and
//     zero points (contiguous for 16 consecutive channels), X (when it fits) and the block's
//     contiguous CSR segment, whose bounds come in through the scalar cache.
#include "gwq_dequant.h"
#include "gwq_internal.h"

namespace gwq {
namespace {

typedef float float4v __attribute__((ext_vector_type(4)));

__device__ inline const uint32_t *at_byte(const uint32_t *base, uint32_t byte_off)
{
    return reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(base) + byte_off);
}

// Registers of one slot (32 codes) as loaded from memory; offsets are bytes from qweight.
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

// Codes of one chunk of U groups of one channel.
template <int BITS, int U> struct Chunk {
    Slot<BITS> slot[U];
    // row_group = index of (channel, group 0); groups past g_last repeat g_last (always valid).
    __device__ inline void load(const uint32_t *qweight, uint32_t row_group, int g0, int g_last, int b)
    {
        constexpr uint32_t group_bytes = words_per_group(BITS) * 4;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = g0 + u < g_last ? g0 + u : g_last;
            slot[u].load(qweight, (row_group + g) * group_bytes, b);
        }
    }
};

constexpr int kPre = 4;        // outlier entries a lane handles without a loop
constexpr int kMetaRounds = 2; // 16-byte vectors of scales / zero points a thread stages

// One layer of a launch, and the launch: up to kMaxBatch layers, blocks [block_end[i-1], block_end[i])
// belong to layer i.  Passed by value (kernel argument segment), read through the scalar cache.
struct DecodeProblem {
    const uint32_t *qweight;
    const uint16_t *scales;
    const uint8_t *zeros;
    const int32_t *row_ptr;
    const uint16_t *col_idx;
    const uint16_t *out_val;
    const _Float16 *X;
    _Float16 *Y;
    int N, K, groups_per_wave, sc_last_vec, zp_last_vec, csr_last_vec;
};
struct DecodeBatch {
    int count, M;
    int block_end[kMaxBatch];
    DecodeProblem p[kMaxBatch];
};

// BITS: 3 or 4.  U: groups per chunk (4 or 8).  PIPE: a wave owns more than U groups (up to 16 when
// MS > 0) and double-buffers chunks of U = 4.  MS: 1..4 = M is exactly MS and X[M][K] is staged in
// LDS, the four lanes of a channel sharing its outliers; 0 = any M <= 16, X read from global memory.
//
// Rows m >= M of the X operand are never zeroed: lanes r >= M re-read row 0, which only produces
// result rows m >= M, and those are not stored.
//
// Dynamic LDS, in this order: X [MS][K] halves | scales [16][gpr] halves | zero points [16][gpr]
// bytes | 16 spare bytes | CSR columns, blockDim * 8 entries | CSR values, same | partial sums
// [waves][4][64] floats.  The launcher guarantees kMetaRounds * blockDim >= 3 * gpr.
template <int BITS, int U, bool PIPE, int MS>
__global__ __launch_bounds__(1024) void decode_kernel(const DecodeBatch batch)
{
    constexpr bool SMALLM = MS > 0;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    // Which layer this block works on (uniform).
    int layer = 0;
    while (layer + 1 < batch.count && (int)blockIdx.x >= batch.block_end[layer]) ++layer;
    const DecodeProblem &pr = batch.p[layer];
    const int block = blockIdx.x - (layer ? batch.block_end[layer - 1] : 0);
    const uint32_t *__restrict__ qweight = pr.qweight;
    const uint16_t *__restrict__ scales = pr.scales;
    const uint8_t *__restrict__ zeros = pr.zeros;
    const int32_t *__restrict__ row_ptr = pr.row_ptr;
    const uint16_t *__restrict__ col_idx = pr.col_idx;
    const uint16_t *__restrict__ out_val = pr.out_val;
    const _Float16 *__restrict__ X = pr.X;
    _Float16 *__restrict__ Y = pr.Y;
    const int N = pr.N, K = pr.K, M = batch.M, groups_per_wave = pr.groups_per_wave;
    const int sc_last_vec = pr.sc_last_vec, zp_last_vec = pr.zp_last_vec, csr_last_vec = pr.csr_last_vec;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nthreads = blockDim.x, nwaves = nthreads >> 6;
    const int r = lane & 15, b = lane >> 4;
    const int gpr = K / kGroup;
    const int row0 = block * 16;
    const int n = row0 + r;
    const int n_c = n < N ? n : N - 1;                  // clamped channel: its results are not stored

    _Float16 *xs = reinterpret_cast<_Float16 *>(lds_raw);
    const uint32_t sc_off = (uint32_t)MS * K * 2;
    const uint32_t zp_off = sc_off + 32 * gpr;
    const uint32_t spare_off = zp_off + 16 * gpr;
    const uint32_t col_off = spare_off + 16;
    const uint32_t val_off = col_off + 16 * nthreads;
    const uint32_t red_off = val_off + 16 * nthreads;
    const uint16_t *sc_lds = reinterpret_cast<const uint16_t *>(lds_raw + sc_off);
    const uint8_t *zp_lds = lds_raw + zp_off;
    const uint16_t *col_lds = reinterpret_cast<const uint16_t *>(lds_raw + col_off);
    const uint16_t *val_lds = reinterpret_cast<const uint16_t *>(lds_raw + val_off);
    float *red = reinterpret_cast<float *>(lds_raw + red_off);

    // CSR bounds of the block (uniform: scalar loads) and of this lane's channel.
    const int last_row = row0 + 16 < N ? row0 + 16 : N;
    const int e_begin = row_ptr[row0], e_end = row_ptr[last_row];
    const int rp0 = row_ptr[n_c], rp1 = row_ptr[n_c + 1];

    // This wave's groups [g_begin, g_last]; a wave past the end of K (has_groups false) walks the
    // last group with a zero scale.
    const bool has_groups = wave * groups_per_wave < gpr;
    const int g_begin = has_groups ? wave * groups_per_wave : gpr - 1;
    const int g_end = g_begin + groups_per_wave < gpr ? g_begin + groups_per_wave : gpr;
    const int g_last = g_end - 1;

    // Staging loads, all 16-byte and coalesced.  (1) X: each wave brings the columns of its own
    // groups (the waves partition K); lanes past the end of a short slice repeat its last vector.
    constexpr int kSliceQuads = PIPE ? 4 : U / 4;       // 64-vector rounds covering a wave's slice
    constexpr int kXVecs = SMALLM ? MS * kSliceQuads : 1;
    u32x4 xstage[kXVecs];
    uint32_t xvec[kXVecs];
    if (SMALLM) {
        const int slice_vecs = (g_end - g_begin) * (kGroup / 8);
#pragma unroll
        for (int e = 0; e < MS; ++e)
#pragma unroll
            for (int i = 0; i < kSliceQuads; ++i) {
                const int q = lane + 64 * i < slice_vecs ? lane + 64 * i : slice_vecs - 1;
                xvec[e * kSliceQuads + i] = (uint32_t)e * (K / 8) + g_begin * (kGroup / 8) + q;
                xstage[e * kSliceQuads + i] = reinterpret_cast<const u32x4 *>(X)[xvec[e * kSliceQuads + i]];
            }
    }
    // (2) The block's scales (32 * gpr bytes) and zero points (16 * gpr bytes), contiguous in
    // memory for 16 consecutive channels: vector t < 2 gpr is a scales vector, the next gpr are
    // zero-point vectors, any further thread re-reads vector 0 into the spare slot.
    uint32_t meta_dst[kMetaRounds];
    u32x4 meta[kMetaRounds];
#pragma unroll
    for (int i = 0; i < kMetaRounds; ++i) {
        const int t = tid + i * nthreads;
        const bool is_sc = t < 2 * gpr, is_zp = !is_sc && t < 3 * gpr;
        int v = is_sc ? block * 2 * gpr + t : block * gpr + (t - 2 * gpr);
        const int last = is_sc ? sc_last_vec : zp_last_vec;
        v = (is_sc || is_zp) ? (v < last ? v : last) : 0;
        const u32x4 *src = is_zp ? reinterpret_cast<const u32x4 *>(zeros) : reinterpret_cast<const u32x4 *>(scales);
        meta[i] = src[v];
        meta_dst[i] = is_sc ? sc_off + 16 * t : is_zp ? zp_off + 16 * (t - 2 * gpr) : spare_off;
    }

    // The code stream: everything else overlaps its HBM latency.
    const uint32_t row_group = (uint32_t)n_c * gpr;
    Chunk<BITS, U> cur;
    cur.load(qweight, row_group, g_begin, g_last, b);

    // (3) The block's CSR segment [e_begin, e_end), from the 16-byte boundary below e_begin:
    // thread t brings entries e0 + 8t .. e0 + 8t + 7.  Entries beyond blockDim * 8 stay in memory.
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
    const int staged_end = e0 + 8 * nthreads < e_end ? e0 + 8 * nthreads : e_end;

    // Nothing that consumes a load may be scheduled above this point.
    __builtin_amdgcn_sched_barrier(0);
    const DecodeConsts dc(BITS);
    if (SMALLM) {
#pragma unroll
        for (int i = 0; i < kXVecs; ++i) reinterpret_cast<u32x4 *>(xs)[xvec[i]] = xstage[i];
    }
#pragma unroll
    for (int i = 0; i < kMetaRounds; ++i) *reinterpret_cast<u32x4 *>(lds_raw + meta_dst[i]) = meta[i];
    __syncthreads();

    float4v acc = float4v{0.f, 0.f, 0.f, 0.f};
    const int x_row = r < M ? r : 0;
    const _Float16 *xsrc = (SMALLM ? xs : X) + (uint32_t)x_row * K + 32 * b;
    // Groups past the wave's last one (a short final wave) are computed on the clamped, repeated
    // data and dropped by a zero scale: no branch sits between the loads and their use.
    auto compute = [&](const Chunk<BITS, U> &c, int g0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool valid = has_groups && g0 + u <= g_last;      // wave-uniform
            const int g = valid ? g0 + u : g_last;
            u32x4 xa[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                xa[j] = *reinterpret_cast<const u32x4 *>(xsrc + (uint32_t)g * kGroup + 8 * j);
            const float s_raw = (float)__builtin_bit_cast(_Float16, sc_lds[r * gpr + g]);
            const float s = valid ? s_raw : 0.f;
            const uint32_t z = zp_lds[r * gpr + g];
            u32x4 wb[4];
            c.slot[u].decode(z, b, dc, wb);
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
            if (more) nxt.load(qweight, row_group, g0 + U, g_last, b);
            compute(cur, g0);
            if (more) cur = nxt;
        }
    } else {
        compute(cur, g_begin);
    }

    // The CSR segment has arrived by now: publish it.
    reinterpret_cast<u32x4 *>(lds_raw + col_off)[tid] = seg_col;
    reinterpret_cast<u32x4 *>(lds_raw + val_off)[tid] = seg_val;
    __syncthreads();

    // Outliers.  SMALLM: the four lanes of a channel split its entries and sum rows m = 0 .. MS-1;
    // otherwise lane (r, b) takes every entry of its channel for rows m = 4b .. 4b+3, the rows of
    // its MFMA results.  Entry j sits at LDS index j - e0 when j < staged_end.
    const int o_stride = SMALLM ? 4 * nwaves : nwaves;
    const int o_first = SMALLM ? 4 * wave + b : wave;
    const bool o_live = n < N && (SMALLM || 4 * b < M);
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
    for (int i = 0; i < kPre; ++i) {
        const int j = rp0 + o_first + i * o_stride;
        const bool ok = o_live && j < rp1 && j < staged_end;
        const int idx = ok ? j - e0 : 0;
        add_outlier(col_lds[idx], val_lds[idx], ok);
    }
    if (o_live) {
        int j = rp0 + o_first + kPre * o_stride;
        for (; j < rp1 && j < staged_end; j += o_stride) add_outlier(col_lds[j - e0], val_lds[j - e0], true);
        // Entries that did not fit the staged window (very long rows) come straight from memory.
        j = rp0 + o_first;
        if (j < staged_end) j += ((staged_end - j + o_stride - 1) / o_stride) * o_stride;
        for (; j < rp1; j += o_stride) add_outlier(col_idx[j], out_val[j], true);
    }

    // Fixed-order reduction over the waves (and, for SMALLM, over the four lanes of a channel),
    // then FP16 store.  SMALLM: only lanes b = 0 hold dense results for rows m < 4.
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float dense = (!SMALLM || b == 0) ? acc[e] : 0.f;
        red[(wave * 4 + e) * 64 + lane] = dense + oacc[e];
    }
    __syncthreads();
    if (SMALLM) {
        if (tid < 16 * MS) {                            // (e, r)
            const int e = tid >> 4, rr = tid & 15;
            float sum = 0.f;
            for (int w = 0; w < nwaves; ++w)
#pragma unroll
                for (int bb = 0; bb < 4; ++bb) sum += red[(w * 4 + e) * 64 + 16 * bb + rr];
            if (row0 + rr < N) Y[(size_t)e * N + row0 + rr] = (_Float16)sum;
        }
    } else {
        for (int idx = tid; idx < 256; idx += nthreads) {
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
hipError_t launch_v(const DecodeBatch &batch, int blocks, int nwaves, size_t lds, hipStream_t st)
{
    static bool attr_set = false;                       // per instantiation; idempotent HIP call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&decode_kernel<BITS, U, PIPE, MS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    decode_kernel<BITS, U, PIPE, MS><<<blocks, nwaves * 64, lds, st>>>(batch);
    return hipGetLastError();
}

template <int BITS, int MS>
hipError_t launch_m(const DecodeBatch &batch, int blocks, int nwaves, int max_gpw, size_t lds, hipStream_t st)
{
    if (max_gpw <= 4) return launch_v<BITS, 4, false, MS>(batch, blocks, nwaves, lds, st);
    if (max_gpw <= 8) return launch_v<BITS, 8, false, MS>(batch, blocks, nwaves, lds, st);
    // Long rows: double-buffered chunks; X is staged only while its staging registers stay few.
    if constexpr (MS == 1 || MS == 2) {
        if (max_gpw <= 16) return launch_v<BITS, 4, true, MS>(batch, blocks, nwaves, lds, st);
    }
    return launch_v<BITS, 4, true, 0>(batch, blocks, nwaves, lds, st);
}

}  // namespace

// Decode launch over `count` layers (same bits, same M): one grid, layer i owning ceil(N_i / 16) blocks.
hipError_t launch_decode(int count, const gwq_packed *const *P, const void *const *X, int M, void *const *Y,
                         int waves_override, hipStream_t st)
{
    DecodeBatch batch;
    batch.count = count;
    batch.M = M;
    // Waves per block: one chunk of eight groups per wave where the rows are long enough, at most 16,
    // and enough threads to stage every layer's 3 * gpr vectors of scales and zero points.
    int nwaves = 1, max_k = 0;
    for (int i = 0; i < count; ++i) {
        const int gpr = P[i]->K / kGroup;
        int w = waves_override ? waves_override : (gpr + 7) / 8;
        const int min_waves = (3 * gpr + 64 * kMetaRounds - 1) / (64 * kMetaRounds);
        if (w < min_waves) w = min_waves;
        if (w > 16) w = 16;
        if (w > gpr && gpr >= min_waves) w = gpr;
        if (count == 1) {                               // a single layer drops waves that would own no group
            const int gpw = (gpr + w - 1) / w, needed = (gpr + gpw - 1) / gpw;
            if (needed >= min_waves) w = needed;
        }
        if (w > nwaves) nwaves = w;
        if (P[i]->K > max_k) max_k = P[i]->K;
    }
    int blocks = 0, max_gpw = 1;
    size_t max_meta = 0;
    for (int i = 0; i < count; ++i) {
        const gwq_packed &L = *P[i];
        const int gpr = L.K / kGroup;
        if (nwaves * 64 * kMetaRounds < 3 * gpr) return hipErrorInvalidValue;      // K <= 65536 keeps this false
        DecodeProblem &d = batch.p[i];
        d.qweight = L.qweight; d.scales = L.scales; d.zeros = L.zeros;
        d.row_ptr = L.row_ptr; d.col_idx = L.col_idx; d.out_val = L.out_val;
        d.X = static_cast<const _Float16 *>(X[i]);
        d.Y = static_cast<_Float16 *>(Y[i]);
        d.N = L.N; d.K = L.K;
        d.groups_per_wave = (gpr + nwaves - 1) / nwaves;
        if (d.groups_per_wave > max_gpw) max_gpw = d.groups_per_wave;
        // Last 16-byte vector of each staged array (the buffers are padded, so clamped reads stay inside).
        const int64_t groups = (int64_t)L.N * gpr;
        d.sc_last_vec = (int)((groups * 2 + 15) / 16) - 1;
        d.zp_last_vec = (int)((groups + 15) / 16) - 1;
        d.csr_last_vec = (int)((L.n_outliers * 2 + 15) / 16);
        blocks += (L.N + 15) / 16;
        batch.block_end[i] = blocks;
        if ((size_t)48 * gpr > max_meta) max_meta = (size_t)48 * gpr;
    }
    for (int i = count; i < kMaxBatch; ++i) { batch.block_end[i] = blocks; batch.p[i] = batch.p[0]; }

    int ms = (M <= 4 && (size_t)M * max_k * 2 <= kXLdsBudget) ? M : 0;
    if (max_gpw > 8 && !((ms == 1 || ms == 2) && max_gpw <= 16)) ms = 0;            // mirrors launch_m
    const size_t lds = (size_t)ms * max_k * 2 + max_meta + 16 + 32 * (size_t)nwaves * 64 + (size_t)nwaves * 1024;
    const int bits = P[0]->bits;
#define GWQ_MS(B, MM) if (bits == B && ms == MM) return launch_m<B, MM>(batch, blocks, nwaves, max_gpw, lds, st)
    GWQ_MS(4, 0); GWQ_MS(4, 1); GWQ_MS(4, 2); GWQ_MS(4, 3); GWQ_MS(4, 4);
    GWQ_MS(3, 0); GWQ_MS(3, 1); GWQ_MS(3, 2); GWQ_MS(3, 3); GWQ_MS(3, 4);
#undef GWQ_MS
    return hipErrorInvalidValue;
}

}  // namespace gwq
