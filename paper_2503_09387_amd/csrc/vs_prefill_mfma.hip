// Frame prefill attention for bf16 storage on gfx950 (VideoScan Section 3.3, prefilling
// phase; Eq. 1 of Section 3.1; carrier token last in the run, Section 3.2).
//
// Work layout
//   * The G = Hq/Hkv query heads of one KV head are packed into one row dimension:
//     packed row r = t*G + hl (token-major), M = T*G rows per KV head.  A row tile of
//     BM = 128*NQ rows is owned by one workgroup of 4 wavefronts, 32*NQ rows each.
//   * Keys are the virtual sequence [len cache rows | T frame rows]; row t sees keys
//     j <= len + t.  The sequence is walked in tiles of 64 keys staged through LDS; the
//     tiles a row tile can see are divided among `nsplit` workgroups, whose partial
//     (max, sum, accumulator) triples are merged by a second small kernel.
//   * Scores are computed transposed, S^T = K Q^T (v_mfma_f32_32x32x16_bf16), so that a
//     lane owns one query column: softmax statistics stay in the lane, and the
//     probabilities are already laid out as the B operand of O^T += V^T P^T.  V^T comes
//     out of row-major LDS through the transposing read ds_read_b64_tr_b16.
//   * Workgroup id = row_tile * (nsplit*Hkv) + (split*Hkv + kv_head): with nsplit*Hkv a
//     multiple of 8, all workgroups that read one K/V slice run on one XCD (ids are
//     dealt round-robin to the 8 XCDs) and share its L2.
#include "vs_internal.h"

namespace vs {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int BN = 64;     // keys per tile
constexpr int KSTR = 136;  // LDS row stride of the K tile in elements (272 B)
constexpr int VSTR = 160;  // LDS row stride of the V tile in elements (320 B)
constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

struct PrefillParams {
    const __bf16* kc;
    const __bf16* vc;
    const __bf16* q;
    const __bf16* kf;
    const __bf16* vf;
    __bf16* out;
    float* part_o;   // [nsplit*Hkv][m_pad][D]
    float* part_ml;  // [nsplit*Hkv][m_pad][2]
    __bf16* k_append_dst;
    __bf16* v_append_dst;
    int L, T, G, Hq, Hkv;
    int M, m_pad, nsplit;
    float scale_log2e;
};

__device__ __forceinline__ float xhalf(float x) {  // value held by lane ^ 32
    return __shfl_xor(x, 32);
}

__device__ __forceinline__ bf16x4 lds_read_tr(const __bf16* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        (__attribute__((address_space(3))) bf16x4*)(p));
}

template <int NQ>
__global__ __launch_bounds__(kThreads) void prefill_mfma_kernel(PrefillParams p) {
    constexpr int BM = 128 * NQ;
    __shared__ __attribute__((aligned(16))) __bf16 Ks[BN * KSTR];
    __shared__ __attribute__((aligned(16))) __bf16 Vs[BN * VSTR];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const int C = p.nsplit * p.Hkv;
    const int rt = blockIdx.x / C;
    const int c = blockIdx.x % C;
    const int split = c / p.Hkv, g = c % p.Hkv;
    const int L = p.L, T = p.T, G = p.G;
    const int64_t kv_row_stride = (int64_t)p.Hkv * D;

    // fused carrier compaction: one workgroup copies the last frame row into the cache
    if (p.k_append_dst && blockIdx.x == 0) {
        const int n16 = (int)(kv_row_stride / 8);  // 16-byte chunks per row
        const uint4* ksrc = reinterpret_cast<const uint4*>(p.kf + (int64_t)(T - 1) * kv_row_stride);
        const uint4* vsrc = reinterpret_cast<const uint4*>(p.vf + (int64_t)(T - 1) * kv_row_stride);
        for (int ch = tid; ch < n16; ch += kThreads) {
            reinterpret_cast<uint4*>(p.k_append_dst)[ch] = ksrc[ch];
            reinterpret_cast<uint4*>(p.v_append_dst)[ch] = vsrc[ch];
        }
    }

    const int row0 = rt * BM;
    const int wrow0 = row0 + wave * 32 * NQ;
    const int last_row = min(row0 + BM, p.M) - 1;
    const int tmax = last_row / G;                        // < T
    const int n_tiles = (L + tmax + 1 + BN - 1) / BN;     // key tiles this row tile can see
    const int tile_begin = (int)((int64_t)n_tiles * split / p.nsplit);
    const int tile_end = (int)((int64_t)n_tiles * (split + 1) / p.nsplit);

    // ---- Q fragments: B operand of S^T = K Q^T, lane (col q = l32, k = 8*hi..8*hi+7) ----
    bf16x8 qf[NQ][8];
    int tq[NQ];  // token index of this lane's query row (for the causal test)
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int r = wrow0 + 32 * nq + l32;
        const int rr = min(r, p.M - 1);
        const int t = rr / G, hl = rr - t * G;
        tq[nq] = t;
        const __bf16* qrow = p.q + ((int64_t)t * p.Hq + (int64_t)g * G + hl) * D;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            qf[nq][kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * hi);
    }

    f32x16 o[NQ][4];
    float m_run[NQ], l_run[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        m_run[nq] = -INFINITY;
        l_run[nq] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[nq][db][e] = 0.f;
    }

    // ---- global -> register staging of one K/V tile: 4 x 16 B of K and of V per thread ----
    uint4 kreg[4], vreg[4];
    auto fetch = [&](int tile) {
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            const int ch = tid + kThreads * n;
            const int row = ch >> 4, c16 = ch & 15;
            const int j = tile * BN + row;
            uint4 kz = make_uint4(0, 0, 0, 0), vz = kz;
            if (j < L) {
                const int64_t off = ((int64_t)j * p.Hkv + g) * D + c16 * 8;
                kz = *reinterpret_cast<const uint4*>(p.kc + off);
                vz = *reinterpret_cast<const uint4*>(p.vc + off);
            } else if (j < L + T) {
                const int64_t off = ((int64_t)(j - L) * p.Hkv + g) * D + c16 * 8;
                kz = *reinterpret_cast<const uint4*>(p.kf + off);
                vz = *reinterpret_cast<const uint4*>(p.vf + off);
            }
            kreg[n] = kz;
            vreg[n] = vz;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            const int ch = tid + kThreads * n;
            const int row = ch >> 4, c16 = ch & 15;
            *reinterpret_cast<uint4*>(&Ks[row * KSTR + c16 * 8]) = kreg[n];
            *reinterpret_cast<uint4*>(&Vs[row * VSTR + c16 * 8]) = vreg[n];
        }
    };

    if (tile_begin < tile_end) fetch(tile_begin);

    for (int tile = tile_begin; tile < tile_end; ++tile) {
        __syncthreads();  // everyone is done reading the previous tile
        stage();
        __syncthreads();
        if (tile + 1 < tile_end) fetch(tile + 1);

        // ---- S^T = K Q^T : rows = 64 keys (2 blocks of 32), cols = this wave's queries ----
        f32x16 s[NQ][2];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) s[nq][b][e] = 0.f;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[(32 * b + l32) * KSTR + 16 * kk + 8 * hi]);
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq)
                    s[nq][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[nq][kk], s[nq][b], 0, 0, 0);
            }
        }

        // ---- causal / tail mask: key j visible to token t iff j <= L + t ----
        const int j0 = tile * BN;
        if (j0 + BN > L) {
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
                const int jmax = L + tq[nq];
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int j = j0 + 32 * b + 8 * (e >> 2) + 4 * hi + (e & 3);
                        if (j > jmax) s[nq][b][e] = -INFINITY;
                    }
            }
        }

        // ---- running-max softmax, one query column per lane (both lane halves hold the
        //      same column and split its keys) ----
        bf16x8 pf[NQ][4];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            float mx = -INFINITY;
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[nq][b][e]);
            mx = fmaxf(mx, xhalf(mx));
            const float m_new = fmaxf(m_run[nq], mx * p.scale_log2e);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run[nq] - m_use);
            m_run[nq] = m_new;
            float rs = 0.f;
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float pe = __builtin_amdgcn_exp2f(fmaf(s[nq][b][e], p.scale_log2e, -m_use));
                    s[nq][b][e] = pe;
                    rs += pe;
                }
            l_run[nq] = l_run[nq] * alpha + rs;  // this lane's half of the keys; halves are added at the end
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[nq][db][e] *= alpha;
            // probabilities -> bf16 B operands: k-slot 4c+j of step t is key 16t + 8c + 4hi + j,
            // i.e. registers 8*(t&1) .. 8*(t&1)+7 of score block t>>1
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[nq][t][e] = (__bf16)s[nq][t >> 1][8 * (t & 1) + e];
        }

        // ---- O^T += V^T P^T : rows = 128 dims (4 blocks of 32), contraction over 64 keys ----
        const int i16 = lane & 15, dh = (lane >> 4) & 1;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const int col = 32 * db + 16 * dh + 4 * (i16 & 3);
                const int r0 = 16 * t + 4 * hi + (i16 >> 2);
                const bf16x4 lo = lds_read_tr(&Vs[r0 * VSTR + col]);
                const bf16x4 hi4 = lds_read_tr(&Vs[(r0 + 8) * VSTR + col]);
                const bf16x8 a = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq)
                    o[nq][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[nq][t], o[nq][db], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: lane (q = l32, hi) holds dims 32*db + 8*(e>>2) + 4*hi + (e&3) ----
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int r = wrow0 + 32 * nq + l32;
        const float l_tot = l_run[nq] + xhalf(l_run[nq]);
        if (r >= p.M) continue;
        if (p.nsplit == 1) {
            const int t = r / G, hl = r - t * G;
            __bf16* orow = p.out + ((int64_t)t * p.Hq + (int64_t)g * G + hl) * D;
            const float inv = 1.0f / l_tot;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    bf16x4 w;
#pragma unroll
                    for (int j = 0; j < 4; ++j) w[j] = (__bf16)(o[nq][db][4 * e4 + j] * inv);
                    *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * e4 + 4 * hi) = w;
                }
        } else {
            const int64_t prow = (int64_t)c * p.m_pad + r;
            float* po = p.part_o + prow * D;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    f32x4 w;
#pragma unroll
                    for (int j = 0; j < 4; ++j) w[j] = o[nq][db][4 * e4 + j];
                    *reinterpret_cast<f32x4*>(po + 32 * db + 8 * e4 + 4 * hi) = w;
                }
            if (hi == 0) {
                p.part_ml[prow * 2 + 0] = m_run[nq];
                p.part_ml[prow * 2 + 1] = l_tot;
            }
        }
    }
}

// Merge of the per-split partials: out = sum_s 2^(m_s - m*) O_s / sum_s 2^(m_s - m*) l_s.
// Block = 8 packed rows x 32 threads, 4 dims per thread.
__global__ __launch_bounds__(kThreads) void prefill_combine_kernel(PrefillParams p) {
    const int g = blockIdx.y;
    const int r = blockIdx.x * 8 + (threadIdx.x >> 5);
    const int d4 = (threadIdx.x & 31) * 4;
    if (r >= p.M) return;
    float mstar = -INFINITY;
    for (int s = 0; s < p.nsplit; ++s)
        mstar = fmaxf(mstar, p.part_ml[((int64_t)(s * p.Hkv + g) * p.m_pad + r) * 2]);
    float denom = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < p.nsplit; ++s) {
        const int64_t prow = (int64_t)(s * p.Hkv + g) * p.m_pad + r;
        const float ms = p.part_ml[prow * 2], ls = p.part_ml[prow * 2 + 1];
        const float w = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - mstar);
        denom += w * ls;
        const f32x4 po = *reinterpret_cast<const f32x4*>(p.part_o + prow * D + d4);
        acc += po * w;
    }
    const float inv = 1.0f / denom;
    const int t = r / p.G, hl = r - t * p.G;
    bf16x4 w4;
#pragma unroll
    for (int j = 0; j < 4; ++j) w4[j] = (__bf16)(acc[j] * inv);
    *reinterpret_cast<bf16x4*>(p.out + ((int64_t)t * p.Hq + (int64_t)g * p.G + hl) * D + d4) = w4;
}

struct Plan {
    int nq, bm, n_row_tiles, m_pad, nsplit;
};

Plan make_plan(const vs_shape& s, int n_tokens, int len) {
    const int G = s.n_q_heads / s.n_kv_heads;
    const int M = n_tokens * G;
    Plan pl;
    pl.nq = g_tune_prefill_row_blocks ? g_tune_prefill_row_blocks : 1;
    pl.bm = 128 * pl.nq;
    pl.n_row_tiles = (M + pl.bm - 1) / pl.bm;
    pl.m_pad = pl.n_row_tiles * pl.bm;
    const int units = pl.n_row_tiles * s.n_kv_heads;
    const int max_tiles = (len + n_tokens + BN - 1) / BN;
    int ns = (512 + units - 1) / units;  // aim at two workgroups per compute unit
    if (ns > max_tiles) ns = max_tiles;
    if (ns > kMaxPrefillSplits) ns = kMaxPrefillSplits;
    if (ns < 1) ns = 1;
    // keep nsplit*Hkv a multiple of 8 when splitting, so K/V sharers land on one XCD
    int gcd8 = 8, h = s.n_kv_heads;
    while (h % gcd8 != 0) gcd8 >>= 1;
    const int step = 8 / gcd8;
    if (ns >= step) ns -= ns % step;
    if (g_tune_prefill_splits) ns = g_tune_prefill_splits < max_tiles ? g_tune_prefill_splits : (max_tiles > 0 ? max_tiles : 1);
    pl.nsplit = ns;
    return pl;
}

}  // namespace

size_t prefill_mfma_workspace_bytes(const vs_shape& s, int32_t max_q_tokens) {
    const int G = s.n_q_heads / s.n_kv_heads;
    const int64_t M = (int64_t)max_q_tokens * G;
    const int64_t m_pad = ((M + 255) / 256) * 256;
    const int64_t slots = (int64_t)kMaxPrefillSplits * s.n_kv_heads * m_pad;
    return (size_t)(slots * (D + 2) * sizeof(float));
}

hipError_t launch_prefill_mfma(const vs_shape& s, const void* kc, const void* vc, int32_t len,
                               const void* q, const void* kf, const void* vf, int32_t n_tokens,
                               void* out, void* k_append_dst, void* v_append_dst, void* /*counters*/,
                               void* workspace, hipStream_t st) {
    const Plan pl = make_plan(s, n_tokens, len);
    PrefillParams p;
    p.kc = (const __bf16*)kc;
    p.vc = (const __bf16*)vc;
    p.q = (const __bf16*)q;
    p.kf = (const __bf16*)kf;
    p.vf = (const __bf16*)vf;
    p.out = (__bf16*)out;
    p.k_append_dst = (__bf16*)k_append_dst;
    p.v_append_dst = (__bf16*)v_append_dst;
    p.L = len;
    p.T = n_tokens;
    p.G = s.n_q_heads / s.n_kv_heads;
    p.Hq = s.n_q_heads;
    p.Hkv = s.n_kv_heads;
    p.M = n_tokens * p.G;
    p.m_pad = pl.m_pad;
    p.nsplit = pl.nsplit;
    p.scale_log2e = s.softmax_scale * kLog2e;
    const int64_t slots = (int64_t)pl.nsplit * s.n_kv_heads * pl.m_pad;
    p.part_o = (float*)workspace;
    p.part_ml = p.part_o + slots * D;
    const int grid = pl.n_row_tiles * pl.nsplit * s.n_kv_heads;
    if (pl.nq == 1) prefill_mfma_kernel<1><<<grid, kThreads, 0, st>>>(p);
    else prefill_mfma_kernel<2><<<grid, kThreads, 0, st>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.nsplit == 1) return e;
    prefill_combine_kernel<<<dim3((p.M + 7) / 8, s.n_kv_heads), kThreads, 0, st>>>(p);
    return hipGetLastError();
}

}  // namespace vs
