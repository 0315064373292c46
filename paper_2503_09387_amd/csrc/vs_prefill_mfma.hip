// Frame prefill attention for bf16 storage on gfx950 (VideoScan Section 3.3, prefilling
// phase; Eq. 1 of Section 3.1; carrier token last in the run, Section 3.2).
//
// Work layout
//   * The G = Hq/Hkv query heads of one KV head are packed into one row dimension:
//     packed row r = t*G + hl (token-major), M = T*G rows per KV head.  A row tile is
//     BM = 128 rows: 4 wavefronts ("row group"), 32 rows each.
//   * Keys are the virtual sequence [len cache rows | T frame rows]; row t sees keys
//     j <= len + t.  The sequence is walked in tiles of 64 keys staged through LDS,
//     double-buffered (one barrier per tile) with the next tile's global loads in flight in
//     registers.
//   * Too few rows exist to fill 256 compute units, so the key tiles a row tile can see are
//     split twice: across `nsplit` workgroups, and inside a workgroup across KVG "key
//     groups" of 4 wavefronts each that take alternate tiles and are merged through LDS at
//     the end.  With KVG = 2 a workgroup has 8 wavefronts (2 per SIMD) and the number of
//     partial results that must travel through memory halves.  The per-workgroup partials
//     (reference, sum, normalised accumulator in bf16) are merged by a second small kernel.
//   * Scores are computed transposed, S^T = K Q^T (v_mfma_f32_32x32x16_bf16), so that a
//     lane owns one query column: softmax statistics stay in the lane, and the
//     probabilities are already laid out as the B operand of O^T += V^T P^T.  V^T comes
//     out of row-major LDS through the transposing read ds_read_b64_tr_b16.
//   * Softmax uses a stale reference: probabilities are first computed against the reference
//     left by earlier tiles (no maximum, no rescale); only if one of them comes out above
//     2^8, or a row has no reference yet, are the scores recomputed, the true maximum taken
//     and the accumulators rescaled.  After the first tile that is rare.
//   * Workgroup id = row_tile * (nsplit*Hkv) + (split*Hkv + kv_head): with nsplit*Hkv a
//     multiple of 8, all workgroups that read one K/V slice run on one XCD (ids are
//     dealt round-robin to the 8 XCDs) and share its L2.
#include "vs_internal.h"

namespace vs {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 128;
constexpr int BM = 128;    // packed query rows per workgroup
constexpr int BN = 64;     // keys per tile
constexpr int KSTR = 136;  // LDS row stride of the K tile in elements (272 B)
constexpr int VSTR = 160;  // LDS row stride of the V tile in elements (320 B)
constexpr int kGroupThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kStageBytes = BN * KSTR * 2 + BN * VSTR * 2;  // one K tile + one V tile
constexpr int kGroupLds = 2 * kStageBytes;                  // two stages per key group

struct PrefillParams {
    const __bf16* kc;
    const __bf16* vc;
    const __bf16* q;
    const __bf16* kf;
    const __bf16* vf;
    __bf16* out;
    // partial accumulators, normalised, in register order:
    // [nsplit*Hkv][row tiles][4 waves][4 dim blocks][2][64 lanes] x 8 bf16
    __bf16* part_o;
    float* part_ml;  // [nsplit*Hkv][m_pad][2]: reference (log2 units), row sum
    __bf16* k_append_dst;
    __bf16* v_append_dst;
    int L, T, G, Hq, Hkv;
    int M, m_pad, nsplit, n_row_tiles;
    float scale_log2e;
    unsigned long long* dbg;  // tuning aid: per-workgroup timestamps, normally null
};

__device__ __forceinline__ float xhalf(float x) {  // value held by lane ^ 32
    return __shfl_xor(x, 32);
}

__device__ __forceinline__ bf16x4 lds_read_tr(const __bf16* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        (__attribute__((address_space(3))) bf16x4*)(p));
}

template <int KVG>
__global__ __launch_bounds__(kGroupThreads * KVG, KVG == 1 ? 2 : 1) void prefill_mfma_kernel(PrefillParams p) {
    extern __shared__ __attribute__((aligned(16))) char dyn_smem[];  // per key group: two stages of (K tile, V tile)

    const unsigned long long t_start = p.dbg ? wall_clock64() : 0;
    const int tid = threadIdx.x;
    const int kg = tid / kGroupThreads;        // key group of this wave
    const int gtid = tid - kg * kGroupThreads;  // thread index inside the key group
    const int lane = tid & 63, rg = (tid >> 6) & 3;  // rg: which 32 rows of the tile
    const int l32 = lane & 31, hi = lane >> 5;
    const int C = p.nsplit * p.Hkv;
    const int rt = blockIdx.x / C;
    const int c = blockIdx.x % C;
    const int split = c / p.Hkv, g = c % p.Hkv;
    const int L = p.L, T = p.T, G = p.G;
    const int64_t kv_row_stride = (int64_t)p.Hkv * D;
    char* const my_smem = dyn_smem + kg * kGroupLds;

    const int row0 = rt * BM;
    const int wrow0 = row0 + rg * 32;
    const int last_row = min(row0 + BM, p.M) - 1;
    const int tmax = last_row / G;                        // < T
    const int n_tiles = (L + tmax + 1 + BN - 1) / BN;     // key tiles this row tile can see
    const int tile_begin = (int)((int64_t)n_tiles * split / p.nsplit);
    const int tile_end = (int)((int64_t)n_tiles * (split + 1) / p.nsplit);
    // key group kg takes tiles tile_begin + kg, + KVG, ...; every group runs n_steps barriers
    const int n_steps = (tile_end - tile_begin + KVG - 1) / KVG;
    const int my_first = tile_begin + kg;

    // ---- global -> register staging of one K/V tile: 4 x 16 B of K and of V per thread ----
    uint4 kreg0, kreg1, kreg2, kreg3, vreg0, vreg1, vreg2, vreg3;
    const int srow = gtid >> 4, sc16 = gtid & 15;  // this thread stages rows srow + 16n, 16-byte piece sc16
#define VS_FETCH1(n, KR, VR)                                                             \
    do {                                                                                 \
        const int j = tile_ * BN + srow + 16 * (n);                                      \
        uint4 kz = make_uint4(0, 0, 0, 0), vz = kz;                                      \
        if (j < L) {                                                                     \
            const int64_t off = ((int64_t)j * p.Hkv + g) * D + sc16 * 8;                 \
            kz = *reinterpret_cast<const uint4*>(p.kc + off);                            \
            vz = *reinterpret_cast<const uint4*>(p.vc + off);                            \
        } else if (j < L + T) {                                                          \
            const int64_t off = ((int64_t)(j - L) * p.Hkv + g) * D + sc16 * 8;           \
            kz = *reinterpret_cast<const uint4*>(p.kf + off);                            \
            vz = *reinterpret_cast<const uint4*>(p.vf + off);                            \
        }                                                                                \
        KR = kz;                                                                         \
        VR = vz;                                                                         \
    } while (0)
#define VS_FETCH(tile)                                                                   \
    do {                                                                                 \
        const int tile_ = (tile);                                                        \
        VS_FETCH1(0, kreg0, vreg0); VS_FETCH1(1, kreg1, vreg1);                          \
        VS_FETCH1(2, kreg2, vreg2); VS_FETCH1(3, kreg3, vreg3);                          \
    } while (0)
#define VS_STAGE1(n, KR, VR)                                                             \
    do {                                                                                 \
        *reinterpret_cast<uint4*>(&ks_[(srow + 16 * (n)) * KSTR + sc16 * 8]) = KR;       \
        *reinterpret_cast<uint4*>(&vs_[(srow + 16 * (n)) * VSTR + sc16 * 8]) = VR;       \
    } while (0)
#define VS_STAGE(buf)                                                                    \
    do {                                                                                 \
        __bf16* ks_ = reinterpret_cast<__bf16*>(my_smem + (buf) * kStageBytes);          \
        __bf16* vs_ = ks_ + BN * KSTR;                                                   \
        VS_STAGE1(0, kreg0, vreg0); VS_STAGE1(1, kreg1, vreg1);                          \
        VS_STAGE1(2, kreg2, vreg2); VS_STAGE1(3, kreg3, vreg3);                          \
    } while (0)

    // the first key tile is requested before anything else (tiles past the range read as
    // zeros and are fully masked, so a group without work in a step stays harmless)
    kreg0 = kreg1 = kreg2 = kreg3 = vreg0 = vreg1 = vreg2 = vreg3 = make_uint4(0, 0, 0, 0);
    if (my_first < tile_end) VS_FETCH(my_first);

    // fused carrier compaction: one workgroup copies the last frame row into the cache
    if (p.k_append_dst && blockIdx.x == 0) {
        const int n16 = (int)(kv_row_stride / 8);  // 16-byte chunks per row
        const uint4* ksrc = reinterpret_cast<const uint4*>(p.kf + (int64_t)(T - 1) * kv_row_stride);
        const uint4* vsrc = reinterpret_cast<const uint4*>(p.vf + (int64_t)(T - 1) * kv_row_stride);
        for (int ch = tid; ch < n16; ch += kGroupThreads * KVG) {
            reinterpret_cast<uint4*>(p.k_append_dst)[ch] = ksrc[ch];
            reinterpret_cast<uint4*>(p.v_append_dst)[ch] = vsrc[ch];
        }
    }

    // ---- Q fragments: B operand of S^T = K Q^T, lane (col q = l32, k = 8*hi..8*hi+7) ----
    bf16x8 qf[8];
    const int r_mine = wrow0 + l32;
    int jmax;  // last key index visible to this lane's query row (causal test)
    {
        const int rr = min(r_mine, p.M - 1);
        const int t = rr / G, hl = rr - t * G;
        jmax = L + t;
        const __bf16* qrow = p.q + ((int64_t)t * p.Hq + (int64_t)g * G + hl) * D;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * hi);
    }

    f32x16 o[4];
    float m_ref = -INFINITY, l_run = 0.f;  // softmax reference (log2 units); this lane's share of the row sum
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][e] = 0.f;

    if (n_steps > 0) {
        VS_STAGE(0);
        if (my_first + KVG < tile_end) VS_FETCH(my_first + KVG);
    }

    const int i16 = lane & 15, dh = (lane >> 4) & 1;
    const int voff = (4 * hi + (i16 >> 2)) * VSTR + 16 * dh + 4 * (i16 & 3);  // this lane's corner of a V^T fragment

    // S^T for 32 keys (sub-block b of the staged tile): 8 K fragments against the Q fragments
    auto qk = [&](const __bf16* Ks, int b, f32x16& sc) {
#pragma unroll
        for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[(32 * b + l32) * KSTR + 16 * kk + 8 * hi]);
            sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], sc, 0, 0, 0);
        }
    };
    // key j = jb + 8*(e>>2) + 4*hi + (e&3) is visible to the row iff j <= jmax
    auto mask = [&](int jb, f32x16& sc) {
#pragma unroll
        for (int e = 0; e < 16; ++e)
            if (jb + 8 * (e >> 2) + 4 * hi + (e & 3) > jmax) sc[e] = -INFINITY;
    };
    // p = 2^(s*c - reference) in place; returns this lane's sum
    auto expo = [&](f32x16& sc) {
        const float m_sub = (m_ref == -INFINITY) ? 0.f : m_ref;
        float r0 = 0.f, r1 = 0.f;
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(sc[e], p.scale_log2e, -m_sub));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(sc[e + 1], p.scale_log2e, -m_sub));
            sc[e] = p0;
            sc[e + 1] = p1;
            r0 += p0;
            r1 += p1;
        }
        return r0 + r1;
    };
    // O^T += V^T P^T for the 32 keys of sub-block b.  k-slot 4c+j of step t is key
    // 16t + 8c + 4hi + j, i.e. probability registers 8t .. 8t+7 of the sub-block.
    auto pv = [&](const __bf16* Vs, int b, const f32x16& sc) {
        bf16x8 pf[2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const bf16x2 pr = __builtin_convertvector(f32x2{sc[8 * t + e], sc[8 * t + e + 1]}, bf16x2);
                pf[t][e] = pr[0];
                pf[t][e + 1] = pr[1];
            }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const bf16x4 lo = lds_read_tr(Vs + voff + (32 * b + 16 * t) * VSTR + 32 * db);
                const bf16x4 hi4 = lds_read_tr(Vs + voff + (32 * b + 16 * t + 8) * VSTR + 32 * db);
                const bf16x8 a = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[t], o[db], 0, 0, 0);
            }
        }
    };
    // Does the speculative pass (stale reference) have to be redone for this sub-block?  Yes if
    // some probability came out above 2^8 (or overflowed), or if a row that can see a key of this
    // sub-block has no reference yet.
    auto stale = [&](float rs, int jb) {
        return __any(!(rs <= 256.f) || (m_ref == -INFINITY && jb + 4 * hi <= jmax));
    };
    // Exact pass: recompute the raw scores, refresh the reference from their maximum, rescale the
    // accumulators and redo the probabilities.  Runs once at the start and then rarely.
    auto refresh = [&](const __bf16* Ks, int b, int jb, bool masked, f32x16& sc) {
        qk(Ks, b, sc);
        if (masked) mask(jb, sc);
        float mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sc[e]);
        mx = fmaxf(mx, xhalf(mx)) * p.scale_log2e;
        const float m_new = fmaxf(m_ref, mx);
        const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_ref - m_new);
        m_ref = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
        return expo(sc);
    };

    const unsigned long long t_loop = p.dbg ? wall_clock64() : 0;
    for (int step = 0; step < n_steps; ++step) {
        const int tile = my_first + step * KVG;  // may lie past tile_end for the last step of a group
        const int buf = step & 1;
        __syncthreads();  // stage `buf` is complete; nobody reads the other stage any more
        if (step + 1 < n_steps) {
            VS_STAGE(buf ^ 1);
            kreg0 = kreg1 = kreg2 = kreg3 = vreg0 = vreg1 = vreg2 = vreg3 = make_uint4(0, 0, 0, 0);
            if (tile + 2 * KVG < tile_end) VS_FETCH(tile + 2 * KVG);
        }
        if (KVG > 1 && tile >= tile_end) continue;  // this group idles in the last step
        const __bf16* Ks = reinterpret_cast<const __bf16*>(my_smem + buf * kStageBytes);
        const __bf16* Vs = Ks + BN * KSTR;
        const int j0 = tile * BN;
        const bool masked = j0 + BN > L;  // the tile holds frame rows (causal) or runs past the end

        // Two sub-blocks of 32 keys, ordered so that the exponentials of one (VALU) sit next to
        // the matrix products of the other (MFMA):  QK(0) | QK(1) + exp(0) | PV(0) + exp(1) | PV(1)
        f32x16 sa, sb;
        qk(Ks, 0, sa);
        if (masked) mask(j0, sa);
        qk(Ks, 1, sb);
        float rsa = expo(sa);
        if (masked) mask(j0 + 32, sb);
        if (stale(rsa, j0)) rsa = refresh(Ks, 0, j0, masked, sa);
        float rsb = expo(sb);
        pv(Vs, 0, sa);
        if (stale(rsb, j0 + 32)) {
            l_run += rsa;  // the refresh rescales l_run, so sub-block 0's sum goes in first
            rsa = 0.f;
            rsb = refresh(Ks, 1, j0 + 32, masked, sb);
        }
        pv(Vs, 1, sb);
        l_run += rsa + rsb;
    }
#undef VS_FETCH1
#undef VS_FETCH
#undef VS_STAGE1
#undef VS_STAGE

    const unsigned long long t_epi = p.dbg ? wall_clock64() : 0;
    float l_tot = l_run + xhalf(l_run);

    // ---- merge the key groups through LDS: group 1 hands (reference, sum, accumulator) to
    //      group 0, which holds the same rows in the same lanes ----
    if (KVG > 1) {
        __syncthreads();  // all tiles consumed, the stage buffers are free
        float* xo = reinterpret_cast<float*>(dyn_smem);  // [4 waves][16 x f32x4][64 lanes]
        float* xml = xo + 4 * 16 * 64 * 4;               // [4 waves][32 rows][2]
        if (kg == 1) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    f32x4 w;
#pragma unroll
                    for (int j = 0; j < 4; ++j) w[j] = o[db][4 * e4 + j];
                    *reinterpret_cast<f32x4*>(&xo[((rg * 16 + db * 4 + e4) * 64 + lane) * 4]) = w;
                }
            if (hi == 0) {
                xml[(rg * 32 + l32) * 2 + 0] = m_ref;
                xml[(rg * 32 + l32) * 2 + 1] = l_tot;
            }
        }
        __syncthreads();
        if (kg == 1) return;
        const float m1 = xml[(rg * 32 + l32) * 2 + 0], l1 = xml[(rg * 32 + l32) * 2 + 1];
        const float m_new = fmaxf(m_ref, m1);
        const float a0 = (m_ref == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_ref - m_new);
        const float a1 = (m1 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m1 - m_new);
        m_ref = m_new;
        l_tot = l_tot * a0 + l1 * a1;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const f32x4 w = *reinterpret_cast<const f32x4*>(&xo[((rg * 16 + db * 4 + e4) * 64 + lane) * 4]);
#pragma unroll
                for (int j = 0; j < 4; ++j) o[db][4 * e4 + j] = o[db][4 * e4 + j] * a0 + w[j] * a1;
            }
    }

    // ---- output: lane (q = l32, hi) holds dims 32*db + 8*(e>>2) + 4*hi + (e&3) ----
    const float inv = (l_tot > 0.f) ? 1.0f / l_tot : 0.f;
    if (p.nsplit == 1) {
        if (r_mine < p.M) {
            const int t = r_mine / G, hl = r_mine - t * G;
            __bf16* orow = p.out + ((int64_t)t * p.Hq + (int64_t)g * G + hl) * D;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    bf16x4 w;
#pragma unroll
                    for (int j = 0; j < 4; ++j) w[j] = (__bf16)(o[db][4 * e4 + j] * inv);
                    *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * e4 + 4 * hi) = w;
                }
        }
    } else {
        // normalised partials in register order: every store instruction writes 1 KB contiguous
        const int64_t unit = (int64_t)c * p.n_row_tiles + rt;
        bf16x8* po = reinterpret_cast<bf16x8*>(p.part_o) + (unit * 4 + rg) * (8 * 64) + lane;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                bf16x8 w;
#pragma unroll
                for (int j = 0; j < 8; ++j) w[j] = (__bf16)(o[db][8 * h2 + j] * inv);
                po[(db * 2 + h2) * 64] = w;
            }
        if (hi == 0) {
            const int64_t prow = (int64_t)c * p.m_pad + r_mine;
            p.part_ml[prow * 2 + 0] = m_ref;
            p.part_ml[prow * 2 + 1] = l_tot;
        }
    }
    if (p.dbg && tid == 0) {
        unsigned long long* d = p.dbg + (size_t)blockIdx.x * 4;
        d[0] = t_start; d[1] = t_loop; d[2] = t_epi; d[3] = wall_clock64();
    }
}

// Merge of the per-split partials: out = sum_s w_s l_s Ohat_s / sum_s w_s l_s with
// w_s = 2^(m_s - m*).  One 64-thread block per (row tile, row group, dim block, half): the same
// lane -> element mapping as the attention kernel, so the partials are read 1 KB at a time; all
// loads of up to 8 splits are issued before any is used.
__global__ __launch_bounds__(64) void prefill_combine_kernel(PrefillParams p) {
    const int lane = threadIdx.x, l32 = lane & 31, hi = lane >> 5;
    int b = blockIdx.x;
    const int h2 = b & 1; b >>= 1;
    const int db = b & 3; b >>= 2;
    const int rg = b & 3; b >>= 2;
    const int rt = b;
    const int g = blockIdx.y;
    if (rt * BM + rg * 32 >= p.M) return;  // whole block beyond the rows
    const int r = rt * BM + rg * 32 + l32;
    const int rr = min(r, p.M - 1);
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    float mstar = -INFINITY;
    for (int s = 0; s < p.nsplit; ++s)
        mstar = fmaxf(mstar, p.part_ml[((int64_t)(s * p.Hkv + g) * p.m_pad + rr) * 2]);
    float denom = 0.f;
    for (int s0 = 0; s0 < p.nsplit; s0 += 8) {
        float ms[8], ls[8];
        bf16x8 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int s = min(s0 + u, p.nsplit - 1);
            const int c = s * p.Hkv + g;
            const int64_t prow = (int64_t)c * p.m_pad + rr;
            ms[u] = p.part_ml[prow * 2];
            ls[u] = p.part_ml[prow * 2 + 1];
            const int64_t unit = (int64_t)c * p.n_row_tiles + rt;
            v[u] = (reinterpret_cast<const bf16x8*>(p.part_o) + (unit * 4 + rg) * (8 * 64) + lane)[(db * 2 + h2) * 64];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float w = (s0 + u < p.nsplit && ms[u] != -INFINITY) ? __builtin_amdgcn_exp2f(ms[u] - mstar) * ls[u] : 0.f;
            denom += w;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += w * (float)v[u][j];
        }
    }
    if (r >= p.M) return;
    const float inv = 1.0f / denom;
    const int t = r / p.G, hl = r - t * p.G;
    __bf16* orow = p.out + ((int64_t)t * p.Hq + (int64_t)g * p.G + hl) * D + 32 * db + 16 * h2 + 4 * hi;
    bf16x4 w0, w1;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        w0[j] = (__bf16)(acc[j] * inv);
        w1[j] = (__bf16)(acc[4 + j] * inv);
    }
    *reinterpret_cast<bf16x4*>(orow) = w0;
    *reinterpret_cast<bf16x4*>(orow + 8) = w1;
}

struct Plan {
    int kvg, n_row_tiles, m_pad, nsplit;
};

Plan make_plan(const vs_shape& s, int n_tokens, int len) {
    const int G = s.n_q_heads / s.n_kv_heads;
    const int M = n_tokens * G;
    Plan pl;
    pl.n_row_tiles = (M + BM - 1) / BM;
    pl.m_pad = pl.n_row_tiles * BM;
    const int units = pl.n_row_tiles * s.n_kv_heads;
    const int max_tiles = (len + n_tokens + BN - 1) / BN;
    // 8-wave workgroups (two key groups) when there are enough key tiles to share out
    pl.kvg = g_tune_prefill_kv_groups ? g_tune_prefill_kv_groups : (max_tiles >= 8 ? 2 : 1);
    int ns = (pl.kvg == 1 ? 512 : 256) / units;  // fill the chip in a single round
    if (ns > max_tiles / pl.kvg) ns = max_tiles / pl.kvg;
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

template <int KVG>
hipError_t launch_kvg(const PrefillParams& p, const Plan& pl, int n_kv_heads, hipStream_t st) {
    static bool attr_set = false;  // dynamic LDS above 64 KB has to be allowed once per kernel
    constexpr int kLds = KVG * kGroupLds;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_mfma_kernel<KVG>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int grid = pl.n_row_tiles * pl.nsplit * n_kv_heads;
    prefill_mfma_kernel<KVG><<<grid, kGroupThreads * KVG, kLds, st>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.nsplit == 1 || g_tune_skip_merge) return e;
    prefill_combine_kernel<<<dim3(pl.n_row_tiles * 4 * 4 * 2, n_kv_heads), 64, 0, st>>>(p);
    return hipGetLastError();
}

}  // namespace

size_t prefill_mfma_workspace_bytes(const vs_shape& s, int32_t max_q_tokens) {
    const int G = s.n_q_heads / s.n_kv_heads;
    const int64_t M = (int64_t)max_q_tokens * G;
    const int64_t m_pad = ((M + BM - 1) / BM) * BM;
    const int64_t slots = (int64_t)kMaxPrefillSplits * s.n_kv_heads * m_pad;
    return (size_t)(slots * (D * sizeof(__bf16) + 2 * sizeof(float))) + (1u << 20);  // + tuning-aid block
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
    p.n_row_tiles = pl.n_row_tiles;
    p.scale_log2e = s.softmax_scale * kLog2e;
    const int64_t slots = (int64_t)pl.nsplit * s.n_kv_heads * pl.m_pad;
    p.part_ml = (float*)workspace;
    p.part_o = (__bf16*)(p.part_ml + slots * 2);
    p.dbg = g_tune_debug_mode == 7
                ? (unsigned long long*)((char*)workspace + prefill_mfma_workspace_bytes(s, n_tokens) - (1 << 20))
                : nullptr;
    return pl.kvg == 1 ? launch_kvg<1>(p, pl, s.n_kv_heads, st) : launch_kvg<2>(p, pl, s.n_kv_heads, st);
}

}  // namespace vs
