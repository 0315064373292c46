// Decode attention for bf16 storage on gfx950 (VideoScan Section 3.3, decoding phase;
// Eq. 1 of Section 3.1): one query token per stream over that stream's retained rows.
//
// The step is bound by reading K and V once from HBM, so the work is cut by ROWS, not by
// stream: the 32-row tiles of all streams are laid end to end and every workgroup of the
// launch takes an equal, contiguous share of them (a share that crosses from one stream into
// the next is worked off as two segments).  A workgroup reads WHOLE rows: its wavefronts are
// the KV heads (wavefront w walks the share for head w), so together they stream contiguous
// memory, which HBM serves measurably faster than one head's 256 bytes out of every 1 KB.
// (With fewer than 4 KV heads the spare wavefronts take sub-ranges of the share; with more,
// blockIdx.y selects the group of 4 heads.)  The grid is one workgroup per compute unit, so
// they all run at once and stream for the whole launch.  A wavefront works alone, with no
// barrier anywhere in the kernel:
//   * K rows go straight from global memory into the A operand of
//     v_mfma_f32_16x16x32_bf16 (S^T = K Q^T; the G query heads of the KV head are the
//     columns, padded to 16);
//   * V rows are loaded coalesced, parked row-major in a wave-private LDS buffer and come
//     back transposed through ds_read_b64_tr_b16 for O^T += V^T P^T;
//   * the next tile's 16 KB are already in flight while the current tile is computed;
//   * the softmax reference maximum is refreshed only when a score exceeds it by more than
//     2^8, which needs one ballot per tile instead of two cross-lane reductions and one
//     accumulator rescale.
// The row appended in this step is read from k_new / v_new (never from the slab, which the
// wavefront that owns the stream's last tile updates on the side).  Every wavefront leaves a
// normalised partial result (fp16 with a power-of-two scale per row) with its reference and sum; a second small kernel merges
// them (a launch that follows another on the same stream starts within about a microsecond of
// it; what the merge costs is its one round trip to memory).  Merging inside the attention
// kernel, by the last wavefront of a stream to arrive, would need the partials of workgroups on
// all 8 XCDs, whose L2 caches are not coherent with each other inside a kernel: they would
// have to be written through and re-read at device scope, which on the prefill kernel cost
// more than the second launch does here.
#include "vs_internal.h"

namespace vs {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
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
    // partial results: [slot][Hkv][nsub][G][D] normalised, slot = workgroup + stream of the segment; stored
    // as fp16 after multiplying the row by the power of two that brings its largest entry into
    // [2^14, 2^15) (11 significant bits whatever the size of the values, in the bytes of bf16)
    _Float16* part_o;
    float* part_ml;       // [slot][Hkv][nsub][G][4]: reference (log2 units), sum, inverse of the row's scale, unused
    int64_t stream_stride;   // elements between streams in the slabs
    int n_streams, G, Hq, Hkv;
    int nh, nsub;            // KV heads per workgroup (1, 2 or 4) and sub-ranges per share (4 / nh)
    int n_wg;                // workgroups along x
    int total_tiles;         // tile_prefix[n_streams]
    int share_q, share_r;    // total_tiles = n_wg * share_q + share_r: the first share_r workgroups take share_q + 1 tiles
    float scale_log2e;
    LenTable lens;           // valid rows per stream, the appended row included
    int tile_prefix[kMaxStreamsPerLaunch + 1];  // tiles of the streams before this one
    int first_wg[kMaxStreamsPerLaunch];  // first workgroup (along x) that holds tiles of the stream, and how many do:
    int n_wgs[kMaxStreamsPerLaunch];     // what the merge kernel walks
};

// first flat tile of workgroup w (w = n_wg gives the end)
__device__ __forceinline__ int wg_first_tile(const DecodeParams& p, int w) {
    return w * p.share_q + min(w, p.share_r);
}

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
// every K/V byte is read once by one wavefront: the loads are marked non-temporal
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_nt(const void* p) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}
#define VS_LD(ptr) ld_nt(ptr)
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

// Grid (n_wg, Hkv / nh).
__global__ __launch_bounds__(kThreads, 2) void decode_mfma_kernel(DecodeParams p) {
    __shared__ __attribute__((aligned(16))) char smem[kWaves * TR * VSTR * 2];  // per-wave V tiles

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, kq = lane >> 4;
    const int g = blockIdx.y * p.nh + wave % p.nh;  // this wavefront's KV head
    const int sub = wave / p.nh;                     // and its sub-range of every segment
    const int64_t row_stride = (int64_t)p.Hkv * D;
    const int flat_end = wg_first_tile(p, blockIdx.x + 1);
    int flat = wg_first_tile(p, blockIdx.x);
    // Lane i holds the end of stream i in flat tiles and its length: one fetch at the start, and
    // whatever a segment needs of a stream is then read out of these registers (a fetch per
    // segment would sit between the workgroup's start and its first K/V loads).
    static_assert(kMaxStreamsPerLaunch <= 64, "one lane per stream");
    const int end_of = p.tile_prefix[min(lane, kMaxStreamsPerLaunch - 1) + 1];
    const int len_of = p.lens.v[min(lane, kMaxStreamsPerLaunch - 1)];
    // stream of the first tile: the number of streams that end at or before it
    int s = __builtin_popcountll(__ballot(end_of <= flat));
    __bf16* vs_w = reinterpret_cast<__bf16*>(smem) + wave * (TR * VSTR);
    const __bf16* vrd = &vs_w[(4 * kq + (i16 >> 2)) * VSTR + 4 * (i16 & 3)];

  for (; flat < flat_end; ++s) {
    // ---- one segment: tiles [seg_a, seg_b) of stream s; this wavefront takes the sub-range
    //      [tile_a, tile_b) of it for head g ----
    const int len = __builtin_amdgcn_readlane(len_of, s);
    const int first_of = s ? __builtin_amdgcn_readlane(end_of, s - 1) : 0;
    const int stream_tiles = __builtin_amdgcn_readlane(end_of, s) - first_of;
    const int seg_a = flat - first_of;
    const int seg_b = min(stream_tiles, flat_end - first_of);
    const bool whole_stream = seg_a == 0 && seg_b == stream_tiles && p.nsub == 1;
    const int tile_a = seg_a + (seg_b - seg_a) * sub / p.nsub;
    const int tile_b = seg_a + (seg_b - seg_a) * (sub + 1) / p.nsub;
    const int row_begin = tile_a * TR;
    const int row_end = min(len, tile_b * TR);
    const int n_tiles = tile_b - tile_a;
    const int last = max(row_end - 1, 0);
    const int new_row = p.k_new ? len - 1 : -1;
    __bf16* kslab = p.k_slab + (int64_t)s * p.stream_stride + (int64_t)g * D;
    __bf16* vslab = p.v_slab + (int64_t)s * p.stream_stride + (int64_t)g * D;
    const __bf16* knew = p.k_new ? p.k_new + ((int64_t)s * p.Hkv + g) * D : nullptr;
    const __bf16* vnew = p.v_new ? p.v_new + ((int64_t)s * p.Hkv + g) * D : nullptr;

    // two tiles are requested before anything else happens
    const uint4 zz = make_uint4(0, 0, 0, 0);
    uint4 k0a = zz, k1a = zz, k2a = zz, k3a = zz, k4a = zz, k5a = zz, k6a = zz, k7a = zz;
    uint4 v0a = zz, v1a = zz, v2a = zz, v3a = zz, v4a = zz, v5a = zz, v6a = zz, v7a = zz;
    uint4 k0b = zz, k1b = zz, k2b = zz, k3b = zz, k4b = zz, k5b = zz, k6b = zz, k7b = zz;
    uint4 v0b = zz, v1b = zz, v2b = zz, v3b = zz, v4b = zz, v5b = zz, v6b = zz, v7b = zz;
    if (0 < n_tiles) VS_FETCH(0, a);
    if (1 < n_tiles) VS_FETCH(1, b);

    // the step's new row also goes into the slab (nobody reads it from there in this launch):
    // done by the wavefront whose range ends with the stream's last tile
    if (new_row >= 0 && n_tiles > 0 && tile_b == stream_tiles && lane < 32) {
        const int c = lane & 15;
        const uint4* src = reinterpret_cast<const uint4*>(lane < 16 ? knew : vnew) + c;
        uint4* dst = reinterpret_cast<uint4*>((lane < 16 ? kslab : vslab) + (int64_t)new_row * row_stride) + c;
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

    // the LDS buffer is private to the wave, whose LDS operations execute in program order
    for (int t = 0; t < n_tiles; t += 2) {
        VS_PARK(a);
        VS_TILE(row_begin + t * TR, a);
        if (t + 2 < n_tiles) VS_FETCH(t + 2, a);
        if (t + 1 < n_tiles) {
            VS_PARK(b);
            VS_TILE(row_begin + (t + 1) * TR, b);
            if (t + 3 < n_tiles) VS_FETCH(t + 3, b);
        }
    }

    // ---- this wavefront's result: lane (head = i16, kq) holds dims 16*db + 4*kq + e ----
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    {
        const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;
        const int head = min(i16, p.G - 1);  // (lanes beyond the G heads compute along and store nothing)
        if (whole_stream) {
            __bf16* dst = p.out + ((int64_t)s * p.Hq + (int64_t)g * p.G + head) * D + 4 * kq;
#define VS_OUT(ACC, DB)                                                                  \
            do {                                                                         \
                bf16x4 r_;                                                               \
                _Pragma("unroll") for (int j = 0; j < 4; ++j) r_[j] = (__bf16)(ACC[j] * inv); \
                if (i16 < p.G) *reinterpret_cast<bf16x4*>(dst + 16 * (DB)) = r_;         \
            } while (0)
            VS_OUT(o0, 0); VS_OUT(o1, 1); VS_OUT(o2, 2); VS_OUT(o3, 3);
            VS_OUT(o4, 4); VS_OUT(o5, 5); VS_OUT(o6, 6); VS_OUT(o7, 7);
#undef VS_OUT
        } else {
            // the row's largest entry: this lane holds 32 of its dims, lanes +-16, +-32 the rest
            float big = 0.f;
#define VS_BIG(ACC) big = fmaxf(fmaxf(fmaxf(big, fabsf(ACC[0])), fmaxf(fabsf(ACC[1]), fabsf(ACC[2]))), fabsf(ACC[3]))
            VS_BIG(o0); VS_BIG(o1); VS_BIG(o2); VS_BIG(o3); VS_BIG(o4); VS_BIG(o5); VS_BIG(o6); VS_BIG(o7);
#undef VS_BIG
            big *= inv;
            big = fmaxf(big, __shfl_xor(big, 16));
            big = fmaxf(big, __shfl_xor(big, 32));
            const int expo = (int)((__float_as_uint(big) >> 23) & 255u);
            const int se = min(max(127 + 14 + 127 - expo, 1), 254);  // biased exponent of the scale
            const float scale = __uint_as_float((unsigned)se << 23), inv_scale = __uint_as_float((unsigned)(254 - se) << 23);
            const int64_t pr = ((((int64_t)blockIdx.x + s) * p.Hkv + g) * p.nsub + sub) * p.G + head;
            _Float16* dst = p.part_o + pr * D + 4 * kq;
            if (kq == 0 && i16 < p.G) *reinterpret_cast<float4*>(p.part_ml + pr * 4) = make_float4(m_ref, l_run, inv_scale, 0.f);
#define VS_OUT(ACC, DB)                                                                  \
            do {                                                                         \
                f16x4 r_;                                                                \
                _Pragma("unroll") for (int j = 0; j < 4; ++j) r_[j] = (_Float16)((ACC[j] * inv) * scale); \
                if (i16 < p.G) *reinterpret_cast<f16x4*>(dst + 16 * (DB)) = r_;          \
            } while (0)
            VS_OUT(o0, 0); VS_OUT(o1, 1); VS_OUT(o2, 2); VS_OUT(o3, 3);
            VS_OUT(o4, 4); VS_OUT(o5, 5); VS_OUT(o6, 6); VS_OUT(o7, 7);
#undef VS_OUT
        }
    }
    flat = first_of + seg_b;  // next segment: the next stream
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

// Merge of a stream's partials (a stream that one wavefront per head covered alone was written
// directly).  Grid (streams, query heads), one wavefront each = 4 groups of 16 lanes: a lane owns
// 8 output dims and the partials group, group + 4, ..; up to kCombineDepth of them per lane are
// requested at once (one round trip to memory for up to 64 partials), merged in the lane in index
// order, and the four groups are then merged with two lane exchanges.  No LDS, no barrier.
constexpr int kCombineGroups = 4, kCombineDepth = 16;
__global__ __launch_bounds__(64) void decode_combine_kernel(DecodeParams p) {
    const int s = blockIdx.x, hq = blockIdx.y;
    const int w_first = p.first_wg[s], n_wgs = p.n_wgs[s];
    if (n_wgs == 1 && p.nsub == 1) return;
    const int g = hq / p.G, h = hq - g * p.G;
    const int lane = threadIdx.x, pg = lane >> 4, t = lane & 15, d8 = t * 8;
    const int n_parts = n_wgs * p.nsub;
    // partial c of the stream: workgroup w_first + c / nsub, sub-range c % nsub
    const int64_t slot_rows = (int64_t)p.Hkv * p.nsub * p.G;
    auto row_of = [&](int c) {
        const int w = p.nsub == 1 ? c : c / p.nsub, sub = p.nsub == 1 ? 0 : c - w * p.nsub;
        return ((int64_t)(w_first + w + s) * slot_rows) + ((int64_t)g * p.nsub + sub) * p.G + h;
    };
    float acc[8], den = 0.f, mref = -INFINITY;
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    for (int c0 = pg; c0 < n_parts; c0 += kCombineGroups * kCombineDepth) {
        float4 ml[kCombineDepth];  // reference, sum, inverse scale of the stored row
        f16x8 o[kCombineDepth];
#pragma unroll
        for (int u = 0; u < kCombineDepth; ++u) {
            const int c = min(c0 + kCombineGroups * u, n_parts - 1);  // (past the end: a valid row, ignored below)
            const int64_t pr = row_of(c);
            ml[u] = *reinterpret_cast<const float4*>(p.part_ml + pr * 4);
            o[u] = *reinterpret_cast<const f16x8*>(p.part_o + pr * D + d8);
        }
#pragma unroll
        for (int u = 0; u < kCombineDepth; ++u)
            if (c0 + kCombineGroups * u >= n_parts) ml[u] = make_float4(-INFINITY, 0.f, 0.f, 0.f);
        float mx = mref;
#pragma unroll
        for (int u = 0; u < kCombineDepth; ++u) mx = fmaxf(mx, ml[u].x);
        if (mx == -INFINITY) continue;
        const float sc = (mref == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mref - mx);
        den *= sc;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] *= sc;
        mref = mx;
#pragma unroll
        for (int u = 0; u < kCombineDepth; ++u) {
            const float wt = (ml[u].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ml[u].x - mx) * ml[u].y;
            den += wt;
            const float wo = wt * ml[u].z;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += wo * (float)o[u][j];
        }
    }
    // the four groups: (0, 1) and (2, 3) first, then the pairs
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const float m2 = __shfl_xor(mref, off), d2 = __shfl_xor(den, off);
        const float mx = fmaxf(mref, m2);
        const float a0 = (mref == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mref - mx);
        const float a1 = (m2 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m2 - mx);
        // (both lanes of a pair must add in the same order to end up with the same bits: the lower group first)
        const bool low = (lane & off) == 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float x2 = __shfl_xor(acc[j], off);
            acc[j] = low ? acc[j] * a0 + x2 * a1 : x2 * a1 + acc[j] * a0;
        }
        den = low ? den * a0 + d2 * a1 : d2 * a1 + den * a0;
        mref = mx;
    }
    if (pg != 0) return;
    const float inv = 1.0f / den;
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = (__bf16)(acc[j] * inv);
    *reinterpret_cast<bf16x8*>(p.out + ((int64_t)s * p.Hq + hq) * D + d8) = r;
}

constexpr int kDecodeMaxWorkgroups = 1024;

// KV heads per workgroup (one wavefront each): the largest of 1, 2, 4 that divides Hkv; the
// other wavefronts take sub-ranges of the share.  One rule for the sizing and the launch.
int heads_per_workgroup(int n_kv_heads) { return n_kv_heads % 4 == 0 ? 4 : (n_kv_heads % 2 == 0 ? 2 : 1); }

// Rows of partial results: a slot per (workgroup + stream of the segment), each with one row per
// (KV head, sub-range, query head of the group).
int64_t partial_rows(const vs_shape& s, int32_t n_streams) {
    const int G = s.n_q_heads / s.n_kv_heads, nsub = kWaves / heads_per_workgroup(s.n_kv_heads);
    return ((int64_t)kDecodeMaxWorkgroups + n_streams) * s.n_kv_heads * nsub * G;
}

}  // namespace

size_t decode_mfma_workspace_bytes(const vs_shape& s, int32_t n_streams, int32_t /*max_rows*/) {
    return (size_t)(partial_rows(s, n_streams) * (D * sizeof(_Float16) + 4 * sizeof(float)));
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
    p.nh = heads_per_workgroup(s.n_kv_heads);
    p.nsub = kWaves / p.nh;
    p.scale_log2e = s.softmax_scale * kLog2e;
    p.lens = lens;
    p.tile_prefix[0] = 0;
    for (int i = 0; i < n_streams; ++i) p.tile_prefix[i + 1] = p.tile_prefix[i] + (lens.v[i] + TR - 1) / TR;
    for (int i = n_streams; i < kMaxStreamsPerLaunch; ++i) p.tile_prefix[i + 1] = 0x7fffffff;  // never "before" a tile
    p.total_tiles = p.tile_prefix[n_streams];
    // Shares of equal size in tiles, one workgroup per compute unit (measured on cfg4: 256 workgroups
    // 30.0 us, 512 30.7 us, and anything in between worse, because some compute units then hold two
    // workgroups and the others one; fewer shares also mean fewer partial results to merge); the
    // tuning knob gives the rows per share instead.
    const int groups_y = s.n_kv_heads / p.nh;
    const int max_x = groups_y < 256 ? 256 / groups_y : 1;
    int64_t tiles_per_wg = g_tune_decode_chunk_rows ? g_tune_decode_chunk_rows / TR : (p.total_tiles + max_x - 1) / max_x;
    if (tiles_per_wg < p.nsub) tiles_per_wg = p.nsub;
    int64_t n_wg = (p.total_tiles + tiles_per_wg - 1) / tiles_per_wg;
    if (n_wg > kDecodeMaxWorkgroups) n_wg = kDecodeMaxWorkgroups;
    if (n_wg < 1) n_wg = 1;
    p.n_wg = (int)n_wg;
    p.share_q = p.total_tiles / p.n_wg;
    p.share_r = p.total_tiles % p.n_wg;
    // which workgroups hold a stream: the largest w with first tile <= the stream's first / last tile
    {
        const int big = p.share_r * (p.share_q + 1);  // tiles held by the workgroups with one tile more
        auto owner = [&](int tile) {
            return tile < big ? tile / (p.share_q + 1) : p.share_r + (tile - big) / (p.share_q > 0 ? p.share_q : 1);
        };
        for (int i = 0; i < kMaxStreamsPerLaunch; ++i) {
            p.first_wg[i] = 0;
            p.n_wgs[i] = 1;
            if (i < n_streams && p.tile_prefix[i + 1] > p.tile_prefix[i]) {
                p.first_wg[i] = owner(p.tile_prefix[i]);
                p.n_wgs[i] = owner(p.tile_prefix[i + 1] - 1) - p.first_wg[i] + 1;
            }
        }
    }
    // the largest slot a wavefront can name is (n_wg - 1) + (n_streams - 1)
    const int64_t rows = partial_rows(s, n_streams);
    if ((int64_t)(p.n_wg + n_streams - 1) * s.n_kv_heads * p.nsub * p.G > rows) return hipErrorInvalidValue;
    p.part_ml = (float*)workspace;
    p.part_o = (_Float16*)(p.part_ml + rows * 4);
    const dim3 grid(p.n_wg, groups_y);
    decode_mfma_kernel<<<grid, kThreads, 0, st>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    decode_combine_kernel<<<dim3(n_streams, s.n_q_heads), 64, 0, st>>>(p);
    return hipGetLastError();
}

}  // namespace vs
