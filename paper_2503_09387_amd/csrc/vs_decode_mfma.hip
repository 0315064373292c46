// Decode attention for bf16 storage on gfx950 (VideoScan Section 3.3, decoding phase;
// Eq. 1 of Section 3.1): one query token per stream over that stream's retained rows.
//
// The step is bound by reading K and V once from HBM, so the work is cut by ROWS, not by
// stream: every (stream, KV head, chunk of `chunk_rows` rows) is one workgroup, whatever
// the stream's length.  Inside a workgroup each of the 4 wavefronts walks its own 32-row
// tiles with no workgroup barrier in the loop:
//   * K rows go straight from global memory into the A operand of
//     v_mfma_f32_16x16x32_bf16 (S^T = K Q^T; the G query heads of the KV head are the
//     columns, padded to 16);
//   * V rows are loaded coalesced, parked row-major in a wave-private LDS buffer and come
//     back transposed through ds_read_b64_tr_b16 for O^T += V^T P^T;
//   * the next tile's 16 KB are already in flight while the current tile is computed;
//   * the softmax reference maximum is refreshed only when a score exceeds it by more than
//     2^8, which needs one ballot per tile instead of two cross-lane reductions and one
//     accumulator rescale.
// The row appended in this step is read from k_new / v_new (never from the slab, which one
// workgroup per KV head updates on the side).  Wave results are merged in LDS; chunk
// results by a second small kernel.  (Merging inside the attention kernel, by the last
// workgroup to arrive, was measured and rejected: partials must then be written through to
// device-coherent memory or the L2 flushed per workgroup, because the 8 XCDs' L2 caches are
// not coherent with each other inside a kernel, and either costs more than the 2.4 us of a
// second launch.)
#include "vs_internal.h"

namespace vs {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int TR = 32;      // rows per wave tile
constexpr int VSTR = 144;   // LDS row stride of the V tile in elements (288 B)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazyMax = 8.0f;  // scores may exceed the reference maximum by 2^8 before it is refreshed

struct DecodeParams {
    __bf16* k_slab;
    __bf16* v_slab;
    const __bf16* q;
    const __bf16* k_new;  // may be null
    const __bf16* v_new;
    __bf16* out;
    float* part_o;        // [stream][max_chunks][Hkv][G][D]
    float* part_ml;       // [stream][max_chunks][Hkv][G][2]
    int64_t stream_stride;   // elements between streams in the slabs
    int n_streams, G, Hq, Hkv, chunk_rows, max_chunks;
    float scale_log2e;
    LenTable lens;           // valid rows per stream, the appended row included
};

__device__ __forceinline__ bf16x4 lds_read_tr(const __bf16* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        (__attribute__((address_space(3))) bf16x4*)(p));
}

// One tile (32 rows) of one wave: scores, lazy-reference softmax, value accumulation.
// K0..K7 are the staged K operands (rows r0+i16 and r0+16+i16, four 32-wide slices each),
// the V tile has already been parked in the wave's LDS buffer.
#define VS_TILE_COMPUTE(R0, K00, K01, K02, K03, K10, K11, K12, K13)                                   \
    do {                                                                                              \
        f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = sa;                                                     \
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, K00), qf0, sa, 0, 0, 0); \
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, K10), qf0, sb, 0, 0, 0); \
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, K01), qf1, sa, 0, 0, 0); \
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, K11), qf1, sb, 0, 0, 0); \
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, K02), qf2, sa, 0, 0, 0); \
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, K12), qf2, sb, 0, 0, 0); \
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, K03), qf3, sa, 0, 0, 0); \
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, K13), qf3, sb, 0, 0, 0); \
        float z[8];                                                                                   \
        _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                               \
            z[e] = ((R0) + 4 * kq + e < row_end) ? sa[e] * p.scale_log2e : -INFINITY;                 \
            z[4 + e] = ((R0) + 16 + 4 * kq + e < row_end) ? sb[e] * p.scale_log2e : -INFINITY;        \
        }                                                                                             \
        float mx = fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])),                                 \
                         fmaxf(fmaxf(z[4], z[5]), fmaxf(z[6], z[7])));                                \
        if (__any(mx > m_ref + kLazyMax)) { /* rare after the first tile: refresh the reference */    \
            mx = fmaxf(mx, __shfl_xor(mx, 16));                                                       \
            mx = fmaxf(mx, __shfl_xor(mx, 32));                                                       \
            const float m_new = fmaxf(m_ref, mx); /* finite: the tile has a valid row */              \
            const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new); /* 0 on the first tile */      \
            m_ref = m_new;                                                                            \
            l_run *= alpha;                                                                           \
            o0 *= alpha; o1 *= alpha; o2 *= alpha; o3 *= alpha;                                       \
            o4 *= alpha; o5 *= alpha; o6 *= alpha; o7 *= alpha;                                       \
        }                                                                                             \
        bf16x8 pf;                                                                                    \
        _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                               \
            const float pe = __builtin_amdgcn_exp2f(z[e] - m_ref);                                    \
            l_run += pe;                                                                              \
            pf[e] = (__bf16)pe;                                                                       \
        }                                                                                             \
        VS_PV(o0, 0); VS_PV(o1, 1); VS_PV(o2, 2); VS_PV(o3, 3);                                       \
        VS_PV(o4, 4); VS_PV(o5, 5); VS_PV(o6, 6); VS_PV(o7, 7);                                       \
    } while (0)

#define VS_PV(ACC, DB)                                                                          \
    do {                                                                                        \
        const bf16x4 lo = lds_read_tr(vrd + 16 * (DB));                                         \
        const bf16x4 hi4 = lds_read_tr(vrd + 16 * VSTR + 16 * (DB));                            \
        ACC = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                                          \
            __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7), pf, ACC, 0, 0, 0);        \
    } while (0)

#define VS_KPTR(row) (((row) == new_row ? knew : kslab + (int64_t)(row) * row_stride) + 8 * kq)
#define VS_VPTR(row) (((row) == new_row ? vnew : vslab + (int64_t)(row) * row_stride) + 8 * i16)
#define VS_LD(ptr) (*reinterpret_cast<const uint4*>(ptr))
// loads one tile into the register set named by suffix X: 8 K operands (rows r+i16 and
// r+16+i16) and 8 V row pieces (individually named registers, so that nothing lands in scratch)
#define VS_FETCH(tile, X)                                                            \
    do {                                                                             \
        const int fr0 = row_begin + (tile) * TR;                                     \
        const __bf16* kpa_ = VS_KPTR(min(fr0 + i16, last));                          \
        const __bf16* kpb_ = VS_KPTR(min(fr0 + 16 + i16, last));                     \
        k0##X = VS_LD(kpa_); k1##X = VS_LD(kpa_ + 32); k2##X = VS_LD(kpa_ + 64); k3##X = VS_LD(kpa_ + 96); \
        k4##X = VS_LD(kpb_); k5##X = VS_LD(kpb_ + 32); k6##X = VS_LD(kpb_ + 64); k7##X = VS_LD(kpb_ + 96); \
        v0##X = VS_LD(VS_VPTR(min(fr0 + kq, last)));                                 \
        v1##X = VS_LD(VS_VPTR(min(fr0 + 4 + kq, last)));                             \
        v2##X = VS_LD(VS_VPTR(min(fr0 + 8 + kq, last)));                             \
        v3##X = VS_LD(VS_VPTR(min(fr0 + 12 + kq, last)));                            \
        v4##X = VS_LD(VS_VPTR(min(fr0 + 16 + kq, last)));                            \
        v5##X = VS_LD(VS_VPTR(min(fr0 + 20 + kq, last)));                            \
        v6##X = VS_LD(VS_VPTR(min(fr0 + 24 + kq, last)));                            \
        v7##X = VS_LD(VS_VPTR(min(fr0 + 28 + kq, last)));                            \
    } while (0)
#define VS_PARK_ROW(n, reg) *reinterpret_cast<uint4*>(&vs_w[(4 * (n) + kq) * VSTR + 8 * i16]) = reg
#define VS_PARK(X)                                                                   \
    do {                                                                             \
        VS_PARK_ROW(0, v0##X); VS_PARK_ROW(1, v1##X); VS_PARK_ROW(2, v2##X); VS_PARK_ROW(3, v3##X); \
        VS_PARK_ROW(4, v4##X); VS_PARK_ROW(5, v5##X); VS_PARK_ROW(6, v6##X); VS_PARK_ROW(7, v7##X); \
    } while (0)
#define VS_TILE(R0, X) VS_TILE_COMPUTE(R0, k0##X, k1##X, k2##X, k3##X, k4##X, k5##X, k6##X, k7##X)

// Grid (chunk, KV head, stream).  Partials go to slot = stream * max_chunks + chunk.
template <int MODE, int DEPTH>
__global__ __launch_bounds__(kThreads, DEPTH == 1 ? 3 : 2) void decode_mfma_kernel(DecodeParams p) {
    __shared__ __attribute__((aligned(16))) char smem[kWaves * TR * VSTR * 2];       // per-wave V tiles
    __shared__ __attribute__((aligned(16))) float sm_o[kWaves * kMaxGroup * D];        // wave results
    __shared__ float sm_ml[kWaves * kMaxGroup * 2];

    const int chunk = blockIdx.x, g = blockIdx.y, s = blockIdx.z;
    const int len = p.lens.v[s];
    const int row_begin = chunk * p.chunk_rows;
    if (row_begin >= len) return;  // this stream has fewer chunks than the longest one
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, kq = lane >> 4;
    const int n_chunks = (len + p.chunk_rows - 1) / p.chunk_rows;
    const int row_end = min(len, row_begin + p.chunk_rows);
    const int n_tiles = (row_end - row_begin + TR - 1) / TR;
    const int last = row_end - 1;
    const int new_row = p.k_new ? len - 1 : -1;
    const int64_t row_stride = (int64_t)p.Hkv * D;
    __bf16* kslab = p.k_slab + (int64_t)s * p.stream_stride + (int64_t)g * D;
    __bf16* vslab = p.v_slab + (int64_t)s * p.stream_stride + (int64_t)g * D;
    const __bf16* knew = p.k_new ? p.k_new + ((int64_t)s * p.Hkv + g) * D : nullptr;
    const __bf16* vnew = p.v_new ? p.v_new + ((int64_t)s * p.Hkv + g) * D : nullptr;
    __bf16* vs_w = reinterpret_cast<__bf16*>(smem) + wave * (TR * VSTR);
    const __bf16* vrd = &vs_w[(4 * kq + (i16 >> 2)) * VSTR + 4 * (i16 & 3)];

    // two tiles per wave are requested before anything else happens
    const uint4 zz = make_uint4(0, 0, 0, 0);
    uint4 k0a = zz, k1a = zz, k2a = zz, k3a = zz, k4a = zz, k5a = zz, k6a = zz, k7a = zz;
    uint4 v0a = zz, v1a = zz, v2a = zz, v3a = zz, v4a = zz, v5a = zz, v6a = zz, v7a = zz;
    uint4 k0b = zz, k1b = zz, k2b = zz, k3b = zz, k4b = zz, k5b = zz, k6b = zz, k7b = zz;
    uint4 v0b = zz, v1b = zz, v2b = zz, v3b = zz, v4b = zz, v5b = zz, v6b = zz, v7b = zz;
    if (wave < n_tiles) VS_FETCH(wave, a);
    if (DEPTH == 2 && wave + kWaves < n_tiles) VS_FETCH(wave + kWaves, b);

    // the step's new row also goes into the slab (nobody reads it from there in this launch)
    if (new_row >= 0 && chunk == n_chunks - 1 && tid < 32) {
        const int c = tid & 15;
        const uint4* src = reinterpret_cast<const uint4*>(tid < 16 ? knew : vnew) + c;
        uint4* dst = reinterpret_cast<uint4*>((tid < 16 ? kslab : vslab) + (int64_t)new_row * row_stride) + c;
        *dst = *src;
    }

    // Q^T fragments (B operand): lane (col = i16, k = 8*kq..8*kq+7), zero beyond the G heads
    bf16x8 qf0, qf1, qf2, qf3;
    {
        const __bf16* qrow = p.q + ((int64_t)s * p.Hq + (int64_t)g * p.G + min(i16, p.G - 1)) * D + 8 * kq;
        const unsigned int keep = i16 < p.G ? 0xffffffffu : 0u;
        uint4 a = VS_LD(qrow), b = VS_LD(qrow + 32), c = VS_LD(qrow + 64), d = VS_LD(qrow + 96);
        a.x &= keep; a.y &= keep; a.z &= keep; a.w &= keep;
        b.x &= keep; b.y &= keep; b.z &= keep; b.w &= keep;
        c.x &= keep; c.y &= keep; c.z &= keep; c.w &= keep;
        d.x &= keep; d.y &= keep; d.z &= keep; d.w &= keep;
        qf0 = __builtin_bit_cast(bf16x8, a);
        qf1 = __builtin_bit_cast(bf16x8, b);
        qf2 = __builtin_bit_cast(bf16x8, c);
        qf3 = __builtin_bit_cast(bf16x8, d);
    }

    f32x4 o0 = {0.f, 0.f, 0.f, 0.f}, o1 = o0, o2 = o0, o3 = o0, o4 = o0, o5 = o0, o6 = o0, o7 = o0;
    float m_ref = -INFINITY, l_run = 0.f;  // m_ref: softmax reference (log2 units), uniform per head column

    // no workgroup barrier in this loop: the LDS buffer is private to the wave, whose LDS
    // operations execute in program order
    for (int t = wave; t < n_tiles; t += DEPTH * kWaves) {
        if (DEPTH == 1) {
            VS_PARK(a);
            VS_TILE(row_begin + t * TR, a);
            if (t + kWaves < n_tiles) VS_FETCH(t + kWaves, a);
            continue;
        }
        if (MODE == 1) {  // experiment: consume the loads without computing
            o0[0] += __builtin_bit_cast(float, k0a.x ^ k1a.x ^ k2a.x ^ k3a.x ^ k4a.x ^ k5a.x ^ k6a.x ^ k7a.x ^ v0a.x ^ v1a.x ^ v2a.x ^ v3a.x ^ v4a.x ^ v5a.x ^ v6a.x ^ v7a.x);
            if (t + 2 * kWaves < n_tiles) VS_FETCH(t + 2 * kWaves, a);
            if (t + kWaves < n_tiles) {
                o1[0] += __builtin_bit_cast(float, k0b.x ^ k1b.x ^ k2b.x ^ k3b.x ^ k4b.x ^ k5b.x ^ k6b.x ^ k7b.x ^ v0b.x ^ v1b.x ^ v2b.x ^ v3b.x ^ v4b.x ^ v5b.x ^ v6b.x ^ v7b.x);
                if (t + 3 * kWaves < n_tiles) VS_FETCH(t + 3 * kWaves, b);
            }
            continue;
        }
        VS_PARK(a);
        VS_TILE(row_begin + t * TR, a);
        if (t + 2 * kWaves < n_tiles) VS_FETCH(t + 2 * kWaves, a);
        if (t + kWaves < n_tiles) {
            VS_PARK(b);
            VS_TILE(row_begin + (t + kWaves) * TR, b);
            if (t + 3 * kWaves < n_tiles) VS_FETCH(t + 3 * kWaves, b);
        }
    }

    if (MODE == 2) {  // experiment: no merge, minimal output
        if (o0[0] + l_run == 123.f) p.out[0] = (__bf16)o0[1];
        return;
    }
    // ---- merge the 4 waves (one barrier: the merge buffer does not alias the V tiles).
    //      lane (head = i16, kq) holds dims 16*db + 4*kq + e ----
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    if (i16 < p.G) {
        float* dst = &sm_o[(wave * kMaxGroup + i16) * D + 4 * kq];
        *reinterpret_cast<f32x4*>(dst + 0) = o0;
        *reinterpret_cast<f32x4*>(dst + 16) = o1;
        *reinterpret_cast<f32x4*>(dst + 32) = o2;
        *reinterpret_cast<f32x4*>(dst + 48) = o3;
        *reinterpret_cast<f32x4*>(dst + 64) = o4;
        *reinterpret_cast<f32x4*>(dst + 80) = o5;
        *reinterpret_cast<f32x4*>(dst + 96) = o6;
        *reinterpret_cast<f32x4*>(dst + 112) = o7;
        if (kq == 0) {
            sm_ml[(wave * kMaxGroup + i16) * 2 + 0] = m_ref;
            sm_ml[(wave * kMaxGroup + i16) * 2 + 1] = l_run;
        }
    }
    __syncthreads();
    const int64_t slot = (int64_t)s * p.max_chunks + chunk;
    if (tid < p.G * (D / 4)) {  // one thread per (head, 4 dims)
        const int h = tid / (D / 4), d4 = (tid - h * (D / 4)) * 4;
        float mw[kWaves], mstar = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            mw[w] = sm_ml[(w * kMaxGroup + h) * 2];
            mstar = fmaxf(mstar, mw[w]);
        }
        f32x4 num = {0.f, 0.f, 0.f, 0.f};
        float den = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float wt = (mw[w] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw[w] - mstar);
            num += *reinterpret_cast<const f32x4*>(&sm_o[(w * kMaxGroup + h) * D + d4]) * wt;
            den += wt * sm_ml[(w * kMaxGroup + h) * 2 + 1];
        }
        if (n_chunks == 1) {
            const float inv = 1.0f / den;
            bf16x4 r;
#pragma unroll
            for (int j = 0; j < 4; ++j) r[j] = (__bf16)(num[j] * inv);
            *reinterpret_cast<bf16x4*>(&p.out[((int64_t)s * p.Hq + (int64_t)g * p.G + h) * D + d4]) = r;
        } else {
            const int64_t pr = (slot * p.Hkv + g) * p.G + h;
            *reinterpret_cast<f32x4*>(&p.part_o[pr * D + d4]) = num;
            if (d4 == 0) {
                p.part_ml[pr * 2 + 0] = mstar;
                p.part_ml[pr * 2 + 1] = den;
            }
        }
    }
}
#undef VS_TILE_COMPUTE
#undef VS_PV
#undef VS_KPTR
#undef VS_VPTR
#undef VS_LD
#undef VS_FETCH
#undef VS_PARK
#undef VS_PARK_ROW
#undef VS_TILE

// Merge of a stream's chunk partials (streams with a single chunk were written directly).
// Grid (streams, query heads); thread = output dim.  The chunk loop is unrolled by 4 with all
// loads issued before they are used, so the latency of one round trip covers four chunks.
__global__ __launch_bounds__(D) void decode_combine_kernel(DecodeParams p) {
    const int s = blockIdx.x, hq = blockIdx.y, d = threadIdx.x;
    const int len = p.lens.v[s];
    const int n_chunks = (len + p.chunk_rows - 1) / p.chunk_rows;
    if (n_chunks == 1) return;
    const int g = hq / p.G, h = hq - g * p.G;
    const int64_t cstride = (int64_t)p.Hkv * p.G;  // partial rows between consecutive chunks
    const int64_t base = ((int64_t)s * p.max_chunks * p.Hkv + g) * p.G + h;
    __shared__ float red[D / 64];
    float mx = -INFINITY;
    for (int c = d; c < n_chunks; c += D) mx = fmaxf(mx, p.part_ml[(base + c * cstride) * 2]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if ((d & 63) == 0) red[d >> 6] = mx;
    __syncthreads();
    const float mstar = fmaxf(red[0], red[1]);
    float num = 0.f, den = 0.f;
    int c = 0;
    for (; c + 4 <= n_chunks; c += 4) {
        float m4[4], l4[4], o4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t pr = base + (c + u) * cstride;
            m4[u] = p.part_ml[pr * 2];
            l4[u] = p.part_ml[pr * 2 + 1];
            o4[u] = p.part_o[pr * D + d];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float wt = __builtin_amdgcn_exp2f(m4[u] - mstar);
            num += wt * o4[u];
            den += wt * l4[u];
        }
    }
    for (; c < n_chunks; ++c) {
        const int64_t pr = base + c * cstride;
        const float wt = __builtin_amdgcn_exp2f(p.part_ml[pr * 2] - mstar);
        num += wt * p.part_o[pr * D + d];
        den += wt * p.part_ml[pr * 2 + 1];
    }
    p.out[((int64_t)s * p.Hq + hq) * D + d] = (__bf16)(num / den);
}

int pick_chunk_rows(const vs_shape& s, int n_streams, const LenTable& lens) {
    if (g_tune_decode_chunk_rows) return g_tune_decode_chunk_rows;
    int64_t total = 0;
    for (int i = 0; i < n_streams; ++i) total += lens.v[i];
    const int64_t target_groups = 1024;  // about four workgroups per compute unit
    int64_t rows = (total * s.n_kv_heads) / target_groups;
    rows -= rows % (TR * kWaves);
    if (rows < TR * kWaves) rows = TR * kWaves;
    if (rows > 4 * TR * kWaves) rows = 4 * TR * kWaves;
    return (int)rows;
}

}  // namespace

size_t decode_mfma_workspace_bytes(const vs_shape& s, int32_t n_streams, int32_t max_rows) {
    const int64_t chunks_per_stream = (int64_t)max_rows / (TR * kWaves) + 1;
    const int64_t slots = chunks_per_stream * n_streams;
    return (size_t)(slots * s.n_q_heads * (D + 2) * sizeof(float));
}

hipError_t launch_decode_mfma(const vs_shape& s, int32_t n_streams, void* k_slab, void* v_slab,
                              int32_t capacity, const LenTable& lens, const void* q,
                              const void* k_new, const void* v_new, void* out, void* /*counters*/,
                              void* workspace, hipStream_t st) {
    DecodeParams p;
    p.k_slab = (__bf16*)k_slab;
    p.v_slab = (__bf16*)v_slab;
    p.q = (const __bf16*)q;
    p.k_new = (const __bf16*)k_new;
    p.v_new = (const __bf16*)v_new;
    p.out = (__bf16*)out;
    p.stream_stride = (int64_t)capacity * s.n_kv_heads * D;
    p.n_streams = n_streams;
    p.G = s.n_q_heads / s.n_kv_heads;
    p.Hq = s.n_q_heads;
    p.Hkv = s.n_kv_heads;
    p.chunk_rows = pick_chunk_rows(s, n_streams, lens);
    p.scale_log2e = s.softmax_scale * kLog2e;
    p.lens = lens;
    int max_len = 1;
    for (int i = 0; i < n_streams; ++i) max_len = lens.v[i] > max_len ? lens.v[i] : max_len;
    p.max_chunks = (max_len + p.chunk_rows - 1) / p.chunk_rows;
    p.part_o = (float*)workspace;
    p.part_ml = p.part_o + (int64_t)n_streams * p.max_chunks * s.n_q_heads * D;
    const dim3 grid(p.max_chunks, s.n_kv_heads, n_streams);
    if (g_tune_debug_mode == 1) decode_mfma_kernel<1, 2><<<grid, kThreads, 0, st>>>(p);
    else if (g_tune_debug_mode == 2) decode_mfma_kernel<2, 2><<<grid, kThreads, 0, st>>>(p);
    else if (g_tune_debug_mode == 3) decode_mfma_kernel<0, 1><<<grid, kThreads, 0, st>>>(p);
    else decode_mfma_kernel<0, 2><<<grid, kThreads, 0, st>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.max_chunks == 1 || g_tune_skip_merge) return e;
    decode_combine_kernel<<<dim3(n_streams, s.n_q_heads), D, 0, st>>>(p);
    return hipGetLastError();
}

}  // namespace vs
