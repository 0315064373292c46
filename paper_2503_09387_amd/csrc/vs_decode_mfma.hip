// Decode attention for bf16 storage on gfx950 (VideoScan Section 3.3, decoding phase;
// Eq. 1 of Section 3.1): one query token per stream over that stream's retained rows.
//
// The step is bound by reading K and V once from HBM, so the work is cut by ROWS, not by
// stream: every (stream, KV head, chunk of `chunk_rows` rows) is one workgroup, whatever
// the stream's length.  Inside a workgroup each of the 4 wavefronts walks its own 32-row
// tiles: K goes straight from global memory into the A operand of
// v_mfma_f32_16x16x32_bf16 (S^T = K Q^T, the G query heads of the KV head are the
// columns), V is staged row-major in a per-wave LDS buffer and comes back transposed
// through ds_read_b64_tr_b16 for O^T += V^T P^T.  Wave results are merged in LDS, chunk
// results by a second small kernel.
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

struct ChunkTable {
    int32_t start[kMaxStreamsPerLaunch + 1];  // first chunk slot of each stream
};

struct DecodeParams {
    const __bf16* k_slab;
    const __bf16* v_slab;
    const __bf16* q;
    __bf16* out;
    float* part_o;   // [slot][Hkv][G][D]
    float* part_ml;  // [slot][Hkv][G][2]
    int64_t stream_stride;  // elements between streams in the slabs
    int n_streams, G, Hq, Hkv, chunk_rows;
    float scale_log2e;
    LenTable lens;
    ChunkTable chunks;
};

__device__ __forceinline__ bf16x4 lds_read_tr(const __bf16* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        (__attribute__((address_space(3))) bf16x4*)(p));
}

__global__ __launch_bounds__(kThreads) void decode_mfma_kernel(DecodeParams p) {
    // per-wave V tiles; reused afterwards for the cross-wave merge
    constexpr int kTileBytes = kWaves * TR * VSTR * 2;
    constexpr int kMergeBytes = kWaves * 16 * D * 4 + kWaves * 16 * 2 * 4;
    __shared__ __attribute__((aligned(16))) char smem[kTileBytes > kMergeBytes ? kTileBytes : kMergeBytes];
    __bf16* vs_all = reinterpret_cast<__bf16*>(smem);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, kq = lane >> 4;
    const int slot = blockIdx.x, g = blockIdx.y;
    int s = 0;
    while (s + 1 < p.n_streams && p.chunks.start[s + 1] <= slot) ++s;
    const int chunk = slot - p.chunks.start[s];
    const int len = p.lens.v[s];
    const int row_begin = chunk * p.chunk_rows;
    const int row_end = min(len, row_begin + p.chunk_rows);  // > row_begin by construction
    const int n_tiles = (row_end - row_begin + TR - 1) / TR;
    const int64_t row_stride = (int64_t)p.Hkv * D;
    const __bf16* kbase = p.k_slab + (int64_t)s * p.stream_stride + (int64_t)g * D;
    const __bf16* vbase = p.v_slab + (int64_t)s * p.stream_stride + (int64_t)g * D;
    __bf16* vs_w = vs_all + wave * (TR * VSTR);

    // Q^T fragments (B operand): lane (col = i16, k = 8*kq..8*kq+7), zero beyond the G heads
    bf16x8 qf[4];
    {
        const __bf16* qrow = p.q + ((int64_t)s * p.Hq + (int64_t)g * p.G + min(i16, p.G - 1)) * D;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 v = *reinterpret_cast<const bf16x8*>(qrow + 32 * kk + 8 * kq);
            if (i16 >= p.G)
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = (__bf16)0.f;
            qf[kk] = v;
        }
    }

    f32x4 o[8];
#pragma unroll
    for (int db = 0; db < 8; ++db) o[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;

    uint4 kreg[2][4], vreg[8];
    auto fetch = [&](int tile) {
        const int r0 = row_begin + tile * TR;
        const int last = row_end - 1;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int row = min(r0 + 16 * c + i16, last);
            const __bf16* kr = kbase + (int64_t)row * row_stride + 8 * kq;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) kreg[c][kk] = *reinterpret_cast<const uint4*>(kr + 32 * kk);
        }
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int row = min(r0 + 4 * n + kq, last);
            vreg[n] = *reinterpret_cast<const uint4*>(vbase + (int64_t)row * row_stride + 8 * i16);
        }
    };

    // every wave runs the same number of iterations (workgroup barriers inside the loop);
    // a wave whose tile lies beyond the chunk works on clamped rows with all scores masked
    const int n_iter = (n_tiles + kWaves - 1) / kWaves;
    fetch(min(wave, n_tiles - 1));
    for (int it = 0; it < n_iter; ++it) {
        const int tile = it * kWaves + wave;
        const int r0 = row_begin + tile * TR;
        __syncthreads();
#pragma unroll
        for (int n = 0; n < 8; ++n)
            *reinterpret_cast<uint4*>(&vs_w[(4 * n + kq) * VSTR + 8 * i16]) = vreg[n];
        bf16x8 kf[2][4];
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) kf[c][kk] = __builtin_bit_cast(bf16x8, kreg[c][kk]);
        __syncthreads();
        if (it + 1 < n_iter) fetch(min(tile + kWaves, n_tiles - 1));

        // S^T (16 keys x 16 heads) for the two 16-row halves of the tile
        f32x4 sc[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            sc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                sc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[c][kk], qf[kk], sc[c], 0, 0, 0);
        }
        // lane (head = i16, kq) holds keys r0 + 16c + 4kq + e
        float mx = -INFINITY;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = r0 + 16 * c + 4 * kq + e;
                if (row >= row_end) sc[c][e] = -INFINITY;
                mx = fmaxf(mx, sc[c][e]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx * p.scale_log2e);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        m_run = m_new;
        bf16x8 pf;
        float rs = 0.f;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float pe = __builtin_amdgcn_exp2f(fmaf(sc[c][e], p.scale_log2e, -m_use));
                rs += pe;
                pf[4 * c + e] = (__bf16)pe;
            }
        l_run = l_run * alpha + rs;
#pragma unroll
        for (int db = 0; db < 8; ++db) o[db] *= alpha;
        // O^T (16 dims x 16 heads per block) += V^T P^T over the tile's 32 keys
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            const int col = 16 * db + 4 * (i16 & 3);
            const int vr = 4 * kq + (i16 >> 2);
            const bf16x4 lo = lds_read_tr(&vs_w[vr * VSTR + col]);
            const bf16x4 hi4 = lds_read_tr(&vs_w[(vr + 16) * VSTR + col]);
            const bf16x8 a = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
            o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pf, o[db], 0, 0, 0);
        }
    }

    // ---- merge the 4 waves: lane (head = i16, kq) holds dims 16*db + 4*kq + e ----
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    __syncthreads();  // V tiles are dead, the buffer becomes [wave][head][D] + stats
    float* sm_o = reinterpret_cast<float*>(smem);
    float* sm_ml = sm_o + kWaves * 16 * D;
    if (i16 < p.G) {
#pragma unroll
        for (int db = 0; db < 8; ++db)
            *reinterpret_cast<f32x4*>(&sm_o[(wave * 16 + i16) * D + 16 * db + 4 * kq]) = o[db];
        if (kq == 0) {
            sm_ml[(wave * 16 + i16) * 2 + 0] = m_run;
            sm_ml[(wave * 16 + i16) * 2 + 1] = l_run;
        }
    }
    __syncthreads();
    const int n_chunks = p.chunks.start[s + 1] - p.chunks.start[s];
    for (int idx = tid; idx < p.G * D; idx += kThreads) {
        const int h = idx / D, d = idx - h * D;
        float mstar = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) mstar = fmaxf(mstar, sm_ml[(w * 16 + h) * 2]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float mw = sm_ml[(w * 16 + h) * 2];
            const float wt = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - mstar);
            num += wt * sm_o[(w * 16 + h) * D + d];
            den += wt * sm_ml[(w * 16 + h) * 2 + 1];
        }
        if (n_chunks == 1) {
            p.out[((int64_t)s * p.Hq + (int64_t)g * p.G + h) * D + d] = (__bf16)(num / den);
        } else {
            const int64_t pr = ((int64_t)slot * p.Hkv + g) * p.G + h;
            p.part_o[pr * D + d] = num;
            if (d == 0) {
                p.part_ml[pr * 2 + 0] = mstar;
                p.part_ml[pr * 2 + 1] = den;
            }
        }
    }
}

// Merge of a stream's chunk partials.  Grid (streams, Hq), one thread per output dim.
__global__ __launch_bounds__(D) void decode_combine_kernel(DecodeParams p) {
    const int s = blockIdx.x, hq = blockIdx.y, d = threadIdx.x;
    const int c0 = p.chunks.start[s], c1 = p.chunks.start[s + 1];
    if (c1 - c0 == 1) return;  // written directly by the attention kernel
    const int g = hq / p.G, h = hq - g * p.G;
    float mstar = -INFINITY;
    for (int c = c0; c < c1; ++c)
        mstar = fmaxf(mstar, p.part_ml[(((int64_t)c * p.Hkv + g) * p.G + h) * 2]);
    float num = 0.f, den = 0.f;
    for (int c = c0; c < c1; ++c) {
        const int64_t pr = ((int64_t)c * p.Hkv + g) * p.G + h;
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
    int64_t rows = (total * s.n_kv_heads + target_groups - 1) / target_groups;
    rows = ((rows + TR * kWaves - 1) / (TR * kWaves)) * (TR * kWaves);
    if (rows < TR * kWaves) rows = TR * kWaves;
    return (int)rows;
}

}  // namespace

size_t decode_mfma_workspace_bytes(const vs_shape& s, int32_t n_streams, int32_t max_rows) {
    const int64_t chunks_per_stream = (int64_t)max_rows / (TR * kWaves) + 1;
    const int64_t slots = chunks_per_stream * n_streams;
    return (size_t)(slots * s.n_q_heads * (D + 2) * sizeof(float));
}

hipError_t launch_decode_mfma(const vs_shape& s, int32_t n_streams, const void* k_slab,
                              const void* v_slab, int32_t capacity, const LenTable& lens,
                              const void* q, void* out, void* workspace, hipStream_t st) {
    DecodeParams p;
    p.k_slab = (const __bf16*)k_slab;
    p.v_slab = (const __bf16*)v_slab;
    p.q = (const __bf16*)q;
    p.out = (__bf16*)out;
    p.stream_stride = (int64_t)capacity * s.n_kv_heads * D;
    p.n_streams = n_streams;
    p.G = s.n_q_heads / s.n_kv_heads;
    p.Hq = s.n_q_heads;
    p.Hkv = s.n_kv_heads;
    p.chunk_rows = pick_chunk_rows(s, n_streams, lens);
    p.scale_log2e = s.softmax_scale * kLog2e;
    p.lens = lens;
    int slots = 0;
    bool any_split = false;
    for (int i = 0; i < n_streams; ++i) {
        p.chunks.start[i] = slots;
        const int n = (lens.v[i] + p.chunk_rows - 1) / p.chunk_rows;
        any_split |= n > 1;
        slots += n;
    }
    for (int i = n_streams; i <= kMaxStreamsPerLaunch; ++i) p.chunks.start[i] = slots;
    p.part_o = (float*)workspace;
    p.part_ml = p.part_o + (int64_t)slots * s.n_q_heads * D;
    decode_mfma_kernel<<<dim3(slots, s.n_kv_heads), kThreads, 0, st>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !any_split) return e;
    decode_combine_kernel<<<dim3(n_streams, s.n_q_heads), D, 0, st>>>(p);
    return hipGetLastError();
}

}  // namespace vs
