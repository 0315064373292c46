// Frame prefill attention for bf16 storage on gfx950 (VideoScan Section 3.3, prefilling
// phase; Eq. 1 of Section 3.1; carrier token last in the run, Section 3.2).
//
// Work layout
//   * The G = Hq/Hkv query heads of one KV head are packed into one row dimension:
//     packed row r = t*G + hl (token-major), M = T*G rows per KV head.  A row tile is
//     BM = 128 rows: two wavefronts of 64 rows each (two "row groups" of 32 per wavefront,
//     so that every K / V^T fragment read from LDS feeds two matrix instructions).
//   * Keys are the virtual sequence [len cache rows | T frame rows]; row t sees keys
//     j <= len + t.  The sequence is walked in tiles of 64 keys.  A tile goes from global
//     memory straight into LDS (global_load_lds_dwordx4, no registers in between) into a ring
//     of two K and two V tiles per key group; the 16-byte pieces of a row are stored at a
//     slot permuted by the row number so that both the row-wise K reads and the transposing
//     V reads are free of bank conflicts without padding.  One barrier per tile.
//   * Too few rows exist to fill 256 compute units, so the key tiles a row tile can see are
//     split twice: across `nsplit` workgroups, and inside a workgroup across NKG "key groups"
//     of two wavefronts that are merged through LDS at the end (each group closes one half
//     of the rows).  Tiles are dealt to the (split, key group) lanes in whole tiles, equally
//     many per lane; the tiles that hold frame rows are spread over the lanes and come first
//     in their lane.  One wavefront per SIMD: it owns all 512 registers.
//   * The per-workgroup partials (reference, sum, normalised accumulator as scaled fp16) are merged
//     inside the launch (all splits of a row tile run on one XCD and count themselves in
//     through its L2): by the tile's workgroups together, each its share of the rows, once
//     the last of them has arrived (the others wait for it, a bounded number of looks at the
//     counter), or by that last one alone, or, where neither is possible, by a second small
//     kernel.  Same sums, same order, same bits.
//   * Scores are computed transposed, S^T = K Q^T (v_mfma_f32_32x32x16_bf16), so that a
//     lane owns one query column: softmax statistics stay in the lane, and the
//     probabilities are already laid out as the B operand of O^T += V^T P^T.  V^T comes
//     out of row-major LDS through the transposing read ds_read_b64_tr_b16.
//   * The matrix instructions, the LDS reads that feed them and the softmax arithmetic are
//     issued from generated blocks of inline assembly over fixed registers, as a software
//     pipeline over sub-blocks of 32 keys: scores of sub-block n+1, value product of n-1 and
//     softmax of n in one block, the ordinary instructions dealt out one by one behind the
//     matrix instructions (gen_prefill_asm.py documents registers and hazards).
//   * Softmax uses a stale reference: probabilities are computed against the reference
//     left by earlier sub-blocks (for the first: against 0); no maximum, no rescale.  Only if
//     a row sum comes out above 2^8, or a row without history underflows, is the sub-block
//     redone exactly from its raw scores (true maximum, accumulators rescaled).  After the
//     first sub-block that is rare.
//   * Workgroup ids are dealt to the 8 XCDs in turn, and each XCD has its own L2: ids are
//     chosen so that the workgroups of one KV head sit on as few XCDs as possible.
#include <type_traits>

#include "vs_internal.h"
#include "vs_prefill_map.h"

namespace vs {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 128;
constexpr int BM = 128;    // packed query rows per workgroup: two wavefronts of 64 rows
constexpr int BN = 64;     // keys per tile
constexpr int kRowBytes = D * 2;               // one K or V row of one head in LDS
constexpr int kTileBytes = BN * kRowBytes;     // 16 KB
constexpr int kStageBytes = 2 * kTileBytes;    // K tile then V tile
constexpr int kGroupLds = 2 * kStageBytes;     // two stages per key group
constexpr int kGroupThreads = 128;             // two wavefronts per key group
constexpr float kLog2e = 1.4426950408889634f;

struct PrefillParams {
    const __bf16* kc;
    const __bf16* vc;
    const __bf16* q;
    const __bf16* kf;
    const __bf16* vf;
    __bf16* out;
    // partial accumulators, normalised, in register order:
    // [nsplit*Hkv][row tiles][4 row groups of 32][4 dim blocks][2][64 lanes] x 8 bf16
    // (stored as fp16 after multiplying the row by a power of two that brings its largest entry
    // into [2^14, 2^15): 11 significant bits whatever the size of the values, in the bytes bf16
    // would take; the power's inverse travels with the row's reference and sum)
    _Float16* part_o;
    float* part_ml;  // [nsplit*Hkv][m_pad][4]: reference (log2 units), row sum, inverse of the row's scale, unused
    __bf16* k_append_dst;    // frame rows append_first .. T-1 are copied here (null: none)
    __bf16* v_append_dst;
    int append_first;        // T - 1: the carrier alone; 0: every row of the run (a question)
    int L, T, G, Hq, Hkv;
    int M, m_pad, nsplit, n_row_tiles;
    float scale_log2e;
    float inv_G, inv_nsplit;  // reciprocals for the index arithmetic of the prologue
    // Merging inside this kernel (see the end of the kernel): the workgroups of one (row tile,
    // KV head) unit are placed on one XCD and count their arrivals in `arrivals`; null = the
    // partial results are merged by prefill_combine_kernel.
    unsigned* arrivals;       // [Hkv][frames][row tiles], kCounterStrideBytes apart, zero between launches
    int xcd_shift;            // log2 of the number of XCDs workgroup ids are dealt to in turn
    int units_per_xcd;
    // the guard of that placement: the XCC_ID the probe read for every residue of the id (4 bits
    // each, residue 0 lowest), and the word in pinned host memory that a workgroup finding itself
    // on another XCD sets (the host looks at it before every launch)
    unsigned long long xcc_of_residue;
    unsigned* misplaced;
    // merge shared by a unit's workgroups (0: the last one to arrive merges alone), and how often a
    // waiting workgroup looks at the counter before it gives up
    int share_merge;
    int max_looks;
    float inv_row_tiles;
    // A run of F frames (semantic-aware mask, Section 3.4): frame a has its own T rows of q, kf,
    // vf and out, and sees L + a retained rows: the L rows of the cache and the carriers (last rows)
    // of the frames before it, which it reads from kf / vf; the launch also copies all F carriers
    // behind the cache's rows.  F = 1: the single frame.
    int F;
    float inv_frame_tiles;    // 1 / (F * row tiles)
};

typedef __attribute__((address_space(1))) const void* global_cptr;
typedef __attribute__((address_space(3))) void* lds_ptr;

__device__ __forceinline__ float xhalf(float x) {  // value held by lane ^ 32
    return __shfl_xor(x, 32);
}

__device__ __forceinline__ bf16x4 lds_read_tr(const char* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(p));
}

// 16 bytes per lane from global memory straight into LDS: lane i's bytes land at dst + 16*i
// (dst is the same for the whole wavefront); completion is counted by vmcnt.
__device__ __forceinline__ void load_to_lds16(const char* src, char* dst) {
    __builtin_amdgcn_global_load_lds((global_cptr)src, (lds_ptr)dst, 16, 0, 0);
}

// Power of two that brings a row whose largest absolute entry is `big` into fp16's top binade
// [2^14, 2^15), and its inverse; rows of zeros (and entries below 2^-112) take the largest power
// there is, NaN and infinity pass through as they are.
struct PartScale {
    float scale, inv_scale;
};
__device__ __forceinline__ PartScale part_scale(float big) {
    const int expo = (int)((__float_as_uint(big) >> 23) & 255u);           // biased exponent of big
    const int se = min(max(127 + 14 + 127 - expo, 1), 254);                // biased exponent of the scale
    PartScale r;
    r.scale = __uint_as_float((unsigned)se << 23);
    r.inv_scale = __uint_as_float((unsigned)(254 - se) << 23);
    return r;
}

// The matrix instructions are issued from hand-scheduled blocks of inline assembly
// (vs_prefill_asm.inc, written by gen_prefill_asm.py, which also documents the register plan):
// output accumulators and query fragments live in a[0:191] for the whole kernel and are never
// values the compiler sees; every block names those registers as clobbered.
#include "vs_prefill_asm.inc"

// The merge of any number of per-split partials of one row, eight of its features at a time: splits
// are taken in chunks of 8 in index order; everything of a chunk is requested before anything is used,
// and chunks are merged like sub-blocks of the online softmax, against a running reference (for up to
// 8 splits: one pass against their largest reference).  ml_of(u) -> (reference, sum, inverse scale, -)
// and v_of(u) -> the 8 stored features of split u.  One piece of code for the second kernel and for the
// in-kernel merge of more than 8 splits, so that both give the same bits.
// NC > 0: the loads of NC chunks at a time are requested before the first of them is used (one round
// trip for up to 8 NC splits); NC = 0: a chunk's loads at the start of its turn.  The arithmetic
// is the same either way.
template <int NC, typename MlOf, typename VOf>
__device__ __forceinline__ void merge_splits_chunked(int nsplit, MlOf ml_of, VOf v_of, float (&acc)[8], float& denom) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    float m_run = -INFINITY;
    denom = 0.f;
    // one chunk: references, sums, inverse scales and stored features of 8 splits (absent ones: -inf, 0, 0, 0)
    auto chunk = [&](const float (&ms)[8], const float (&ls)[8], const float (&isc)[8], const f16x8 (&v)[8]) {
        float m_new = m_run;
#pragma unroll
        for (int u = 0; u < 8; ++u) m_new = fmaxf(m_new, ms[u]);
        if (m_new == -INFINITY) return;  // nothing in these splits (and nothing before)
        const float keep = __builtin_amdgcn_exp2f(m_run - m_new);  // 0 for the first chunk with content
        denom *= keep;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] *= keep;
        m_run = m_new;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float w = (ms[u] != -INFINITY) ? __builtin_amdgcn_exp2f(ms[u] - m_new) * ls[u] : 0.f;
            denom += w;
            const float wo = w * isc[u];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += wo * (float)v[u][j];
        }
    };
    constexpr int kChunks = NC > 0 ? NC : 1;
    float ms[kChunks][8], ls[kChunks][8], isc[kChunks][8];
    f16x8 v[kChunks][8];
    auto fetch = [&](int c, int s0) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            ms[c][u] = -INFINITY;
            ls[c][u] = 0.f;
            isc[c][u] = 0.f;
            if (s0 + u < nsplit) {
                const float4 ml = ml_of(s0 + u);
                ms[c][u] = ml.x;
                ls[c][u] = ml.y;
                isc[c][u] = ml.z;
                v[c][u] = v_of(s0 + u);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) v[c][u][j] = (_Float16)0.f;
            }
        }
    };
    if constexpr (NC > 0) {
        for (int g0 = 0; g0 < nsplit; g0 += 8 * NC) {
#pragma unroll
            for (int c = 0; c < NC; ++c)
                if (g0 + 8 * c < nsplit) fetch(c, g0 + 8 * c);
#pragma unroll
            for (int c = 0; c < NC; ++c)
                if (g0 + 8 * c < nsplit) chunk(ms[c], ls[c], isc[c], v[c]);
        }
    } else {
        for (int s0 = 0; s0 < nsplit; s0 += 8) {
            fetch(0, s0);
            chunk(ms[0], ls[0], isc[0], v[0]);
        }
    }
}

template <int NKG>
__global__ __launch_bounds__(kGroupThreads * NKG) __attribute__((amdgpu_waves_per_eu(1, 1)))
void prefill_mfma_kernel(PrefillParams p) {
    extern __shared__ __attribute__((aligned(1024))) char dyn_smem[];  // per key group: two K tiles, two V tiles

    // All arguments the prologue needs are fetched here, at once (left to itself the compiler
    // fetches each one where it is first used, and waits there).
    const char* const kc = reinterpret_cast<const char*>(p.kc);
    const char* const vc = reinterpret_cast<const char*>(p.vc);
    const char* kf = reinterpret_cast<const char*>(p.kf);
    const char* vf = reinterpret_cast<const char*>(p.vf);
    const char* qbase = reinterpret_cast<const char*>(p.q);
    int L = p.L;
    const int T = p.T, G = p.G, M = p.M, Hkv = p.Hkv, nsplit = p.nsplit;
    const float inv_G = p.inv_G, inv_nsplit = p.inv_nsplit;
    asm volatile("" : : "s"(kc), "s"(vc), "s"(kf), "s"(vf), "s"(qbase), "s"(L), "s"(T), "s"(G), "s"(M), "s"(Hkv),
                 "s"(nsplit), "s"(inv_G), "s"(inv_nsplit), "s"(p.Hq), "s"(p.scale_log2e));
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rb = w & 1;   // which 64 rows of the tile
    const int kg = w >> 1;  // key group of this wave
    const int l32 = lane & 31, hi = lane >> 5;
    int g, split, rt, frame;
    if (p.arrivals) {
        // 1-D grid.  Workgroup ids are dealt to the XCDs in turn (id mod number of XCDs), and a
        // unit = (KV head, frame, row tile) is merged through the L2 its XCD's compute units share, so
        // all splits of a unit take ids of one residue: XCD x holds units x*units_per_xcd ..
        // (consecutive units: the same KV head, whose K/V that L2 then holds once), each with
        // nsplit consecutive slots.
        const PrefillSlot at = prefill_slot_of_id(blockIdx.x, p.n_row_tiles * p.F * Hkv, p.units_per_xcd, nsplit,
                                                  inv_nsplit, p.xcd_shift);
        if (at.unit < 0) return;  // spare ids
        // Guard: is this workgroup on the XCD that ids of its residue were seen on when the
        // device was probed?  If not, the splits of its unit may not share an L2, and the merge
        // below cannot be trusted: say so where the host sees it before its next launch.
        unsigned xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        if ((xcc & 15u) != (unsigned)((p.xcc_of_residue >> (4 * at.xcd)) & 15u) && threadIdx.x == 0)
            __hip_atomic_store(p.misplaced, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        const int unit = at.unit;
        split = at.split;
        g = div_small(unit, p.n_row_tiles * p.F, p.inv_frame_tiles);
        const int ft = unit - g * p.n_row_tiles * p.F;
        frame = div_small(ft, p.n_row_tiles, p.inv_row_tiles);
        rt = ft - frame * p.n_row_tiles;
    } else {
        // grid (Hkv, nsplit, frames x row tiles): x runs fastest in dispatch order, so with
        // nsplit*Hkv a multiple of the number of XCDs all workgroups that read one K/V slice
        // share an L2
        g = blockIdx.x, split = blockIdx.y;
        frame = div_small(blockIdx.z, p.n_row_tiles, p.inv_row_tiles);
        rt = blockIdx.z - frame * p.n_row_tiles;
    }
    // the frame's own tensors and retained rows: Lc rows in the cache, then the carriers of the
    // run's earlier frames (keys Lc .. L-1, read from the run's own K/V: row T-1 of frame j - Lc)
    const int Lc = L;
    const char* const kf0 = kf;
    const char* const vf0 = vf;
    L += frame;
    qbase += (int64_t)frame * T * p.Hq * (D * 2);
    kf += (int64_t)frame * T * Hkv * kRowBytes;
    vf += (int64_t)frame * T * Hkv * kRowBytes;
    __bf16* const out = p.out + (int64_t)frame * T * p.Hq * D;
    const int gf = g * p.F + frame, HF = Hkv * p.F;  // (head, frame) pairs index partial results and counters
    const int c = split * HF + gf;  // which partial result
    const int wg_id = rt * (nsplit * HF) + c;
    const int kv_row_bytes = Hkv * kRowBytes;
    char* const k_ring = dyn_smem + kg * kGroupLds;
    char* const v_ring = k_ring + 2 * kTileBytes;

    const int row0 = rt * BM;
    const int wrow0 = row0 + rb * 64;
    const int last_row = min(row0 + BM, M) - 1;
    const int tmax = div_small(last_row, G, inv_G);       // < T
    const int n_tiles = (L + tmax + BN) / BN;             // key tiles this row tile can see
    // The tiles are dealt to lanes = (split, key group) pairs, lane = split*NKG + kg.  Every lane
    // takes q or q+1 tiles (the first lanes one more), a contiguous run of plain cache tiles.
    // Tiles with frame rows cost more (causal mask, staging through the slower path), so they
    // are not left in one lane: they are handed out one at a time from the last lane backwards
    // and replace plain tiles there.  (With fewer tiles than that takes, every lane simply has
    // its contiguous run of whatever tiles fall into it.)  Tile number s of this lane:
    //     s < n_rest ? rest_first + s : run_first + (s - n_rest)
    // (frame tiles first: their slower staging then falls into the prologue, and the steady
    // state of the pipeline sees plain tiles only.)
    const int n_lanes = nsplit * NKG;
    const float inv_lanes = NKG == 1 ? inv_nsplit : 0.5f * inv_nsplit;
    const int n_plain = Lc / BN;            // tiles of cache rows only (<= n_tiles)
    const int n_frame = n_tiles - n_plain;
    const bool small = n_tiles < (1 << 22);
    const int q_all = small ? div_small(n_tiles, n_lanes, inv_lanes) : n_tiles / n_lanes;
    const int r_all = n_tiles - q_all * n_lanes;
    const int q_fr = small ? div_small(n_frame, n_lanes, inv_lanes) : n_frame / n_lanes;
    const int r_fr = n_frame - q_fr * n_lanes;
    const bool dealt = q_fr < q_all;        // every lane has room for its frame tiles
    auto tiles_before = [&](int i) { return i * q_all + min(i, r_all); };
    auto frame_before = [&](int i) { return i * q_fr + max(0, i - (n_lanes - r_fr)); };
    const int my_lane = split * NKG + kg;
    const int n_my = tiles_before(my_lane + 1) - tiles_before(my_lane);  // tiles of this lane
    const int n_steps = tiles_before(split * NKG + 1) - tiles_before(split * NKG);  // the workgroup's longest lane
    const int n_rest = dealt ? frame_before(my_lane + 1) - frame_before(my_lane) : 0;
    const int run_first = tiles_before(my_lane) - (dealt ? frame_before(my_lane) : 0);
    const int rest_first = n_plain + frame_before(my_lane);
    auto tile_of = [&](int s) { return s < n_rest ? rest_first + s : run_first + (s - n_rest); };

    // ---- global -> LDS staging --------------------------------------------------------------
    // A tile is 64 rows of 256 B.  One load instruction of a wavefront fills 1 KB = 4 rows
    // ("chunk"): lane i fills 16-byte slot i&15 of row i>>4.  Which 16-byte piece of the row a
    // slot holds is permuted so that the fragment reads below are free of bank conflicts:
    //   K: slot = piece ^ (row & 15)         (32 lanes read one piece of 32 consecutive rows)
    //   V: slot = piece ^ ((row & 3) << 1)   (a transposing read takes 32 B of each of 4 rows)
    // Wave rb of the key group loads chunks 8*rb .. 8*rb+7 of a tile.
    const int lr = lane >> 4, ls = lane & 15;
    int k_src_off[4];  // byte offset of this lane's piece from the chunk's first row, chunk & 3 = x
#pragma unroll
    for (int x = 0; x < 4; ++x) k_src_off[x] = lr * kv_row_bytes + ((ls ^ lr ^ (x << 2)) << 4);
    const int v_src_off = lr * kv_row_bytes + ((ls ^ (lr << 1)) << 4);
    int k_off[8], v_off[8];  // the same with the chunk's rows added: what the in-block staging loads use
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        k_off[u] = k_src_off[u & 3] + u * 4 * kv_row_bytes;
        v_off[u] = v_src_off + u * 4 * kv_row_bytes;
    }

    // tile number s of this group -> K ring (is_v = false) or V ring, slot s & 1
    auto issue = [&](int s, bool is_v) {
        if (s >= n_my) return;
        const int tile = tile_of(s);
        char* dst = (is_v ? v_ring : k_ring) + (s & 1) * kTileBytes + rb * (8 * 1024);
        const int j0 = tile * BN + rb * 32;  // first row this wave loads
        if (tile * BN + BN <= Lc) {
            const char* src = (is_v ? vc : kc) + ((int64_t)j0 * Hkv + g) * kRowBytes;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                load_to_lds16(src + (int64_t)u * 4 * kv_row_bytes + (is_v ? v_src_off : k_src_off[u & 3]), dst + u * 1024);
        } else {
            // the tile holds frame rows or runs past the end: rows past the last key re-read the
            // last row (finite values; every such key is masked)
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int j = min(j0 + 4 * u + lr, L + T - 1);
                const char* row = (j < Lc) ? (is_v ? vc : kc) + ((int64_t)j * Hkv + g) * kRowBytes
                                  : (j < L) ? (is_v ? vf0 : kf0) + (((int64_t)(j - Lc) * T + (T - 1)) * Hkv + g) * kRowBytes
                                            : (is_v ? vf : kf) + ((int64_t)(j - L) * Hkv + g) * kRowBytes;
                const int piece = is_v ? (ls ^ (lr << 1)) : (ls ^ lr ^ ((u & 3) << 2));
                load_to_lds16(row + (piece << 4), dst + u * 1024);
            }
        }
    };

    // ---- what the first two blocks need is requested before anything else is set up: K of
    //      the first tile and the query rows.  (A compute unit takes in 64 bytes per clock: the
    //      96 KB of these two are what the start of the pipeline waits for; K of the second
    //      tile and V of the first are requested later, from inside the first two blocks.)
    //      Q fragments are the B operand of S^T = K Q^T, lane (col q = l32, k = 8*hi..8*hi+7);
    //      the wave holds two row groups r = 0, 1 of 32 rows.  They are loaded straight into
    //      a[128:191] and stay there. ----
    issue(0, false);
    int r_mine[2], jmax[2];  // jmax: last key index visible to this lane's query row (causal test)
    {
        const char* qrow[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            r_mine[r] = wrow0 + 32 * r + l32;
            const int rr = min(r_mine[r], M - 1);
            const int t = div_small(rr, G, inv_G), hl = rr - t * G;
            jmax[r] = L + t;
            qrow[r] = qbase + ((int64_t)(t * p.Hq + g * G + hl) * D + 8 * hi) * 2;
        }
        asm volatile(VS_ASM_LOAD_Q : : [qa0] "v"(qrow[0]), [qa1] "v"(qrow[1]) : VS_CLOB_ACC);
    }
    asm volatile(VS_ASM_INIT_O : : : VS_CLOB_ACC, VS_CLOB_TMP);  // while the loads above are under way

    float m_ref[2] = {-INFINITY, -INFINITY};  // softmax reference (log2 units)
    float ms[2] = {0.f, 0.f};                 // what the blocks subtract: the reference, 0 while there is none
    float l_run[2] = {0.f, 0.f};              // this lane's share of the row sum

    // LDS read addresses (bytes inside a tile)
    unsigned k_rd[8];  // K fragment of step kk: row l32 (+32b), piece 2kk+hi
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) k_rd[kk] = l32 * kRowBytes + (((2 * kk + hi) ^ (l32 & 15)) << 4);
    const int i16 = lane & 15, dh = (lane >> 4) & 1;
    unsigned v_rd[2];  // V^T fragment corner, dim block parity x: row 4hi + (i16>>2), piece 4x + 2dh + ((i16&3)>>1)
#pragma unroll
    for (int x = 0; x < 2; ++x)
        v_rd[x] = (4 * hi + (i16 >> 2)) * kRowBytes + (((4 * x + 2 * dh + ((i16 & 3) >> 1)) ^ ((i16 >> 2) << 1)) << 4) + 8 * (i16 & 1);
    const unsigned k_ring_lds = (unsigned)(size_t)(lds_ptr)k_ring;  // LDS byte addresses of the rings
    const unsigned v_ring_lds = (unsigned)(size_t)(lds_ptr)v_ring;

    // ---- pipeline state lives in fixed registers between the blocks: raw scores of the
    // sub-block in flight S[parity][row group] in v[128:191], packed probabilities
    // P[parity][row group][step] in v[216:247] (sub-block n of this group uses parity n & 1).
    // Every block names them as clobbered, and the code between the blocks is small enough
    // that the compiler stays in the low registers there (the build checks the listing).
    // the read addresses of the tiles in use: K starts in slot 0, V in slot 0; they change slot
    // once per tile
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) k_rd[kk] += k_ring_lds;
    v_rd[0] += v_ring_lds;
    v_rd[1] += v_ring_lds;
    int k_hop = kTileBytes, v_hop = kTileBytes;  // to the other slot
#define VS_ADDR                                                                                  \
    [ka0] "v"(k_rd[0]), [ka1] "v"(k_rd[1]), [ka2] "v"(k_rd[2]), [ka3] "v"(k_rd[3]),              \
    [ka4] "v"(k_rd[4]), [ka5] "v"(k_rd[5]), [ka6] "v"(k_rd[6]), [ka7] "v"(k_rd[7]),              \
    [va0] "v"(v_rd[0]), [va1] "v"(v_rd[1])
#define VS_KOFF                                                                                  \
    [ko0] "v"(k_off[0]), [ko1] "v"(k_off[1]), [ko2] "v"(k_off[2]), [ko3] "v"(k_off[3]),          \
    [ko4] "v"(k_off[4]), [ko5] "v"(k_off[5]), [ko6] "v"(k_off[6]), [ko7] "v"(k_off[7])
#define VS_VOFF                                                                                  \
    [vo0] "v"(v_off[0]), [vo1] "v"(v_off[1]), [vo2] "v"(v_off[2]), [vo3] "v"(v_off[3]),          \
    [vo4] "v"(v_off[4]), [vo5] "v"(v_off[5]), [vo6] "v"(v_off[6]), [vo7] "v"(v_off[7])
    // what every block with a softmax part takes and returns: the sums, and the lanes that need the
    // closer look of commit()
#define VS_SM_OUT [sum0] "=&v"(sum0_), [sum1] "=&v"(sum1_), [flag] "=&s"(flag_)
#define VS_SM_IN [ms0] "v"(ms[0]), [ms1] "v"(ms[1]), [scale] "s"(p.scale_log2e), [l0] "v"(l_run[0]), [l1] "v"(l_run[1]), [k256] "s"(256.f)
#define VS_CLOBBERS VS_CLOB_ACC, VS_CLOB_S, VS_CLOB_FRAG, VS_CLOB_TMP, VS_CLOB_P, "vcc"

    // tile number s of this group: LDS byte addresses of its K and V tiles, first key index
    auto k_tile = [&](int s) { return k_ring_lds + (s & 1) * kTileBytes; };
    auto v_tile = [&](int s) { return v_ring_lds + (s & 1) * kTileBytes; };
    auto key0 = [&](int n) { return tile_of(n >> 1) * BN + 32 * (n & 1); };  // of sub-block n

    // Sub-block n has gone through the speculative softmax (reference possibly stale); its PV
    // product has not been issued.  Commit its row sums, or, if a probability came out above
    // 2^8 (or overflowed), redo it exactly from the raw scores: reference refreshed from their
    // maximum, accumulators and sums rescaled, probabilities rebuilt.
    // A row that has accumulated nothing yet runs against the made-up reference 0: there an
    // underflow (a lane that can see a key of the sub-block but whose sum vanished) also sends
    // the sub-block to the exact pass, which treats such a row as having no reference at all.
    auto commit = [&](int n, float sum0, float sum1, unsigned long long flag) {
        if (flag == 0) {  // the common case, decided inside the block
            l_run[0] += sum0;
            l_run[1] += sum1;
            return;
        }
        const int jl = key0(n) + 4 * hi;  // this lane's smallest key in the sub-block
        const bool redo = !(sum0 <= 256.f) || !(sum1 <= 256.f) ||
                          (l_run[0] == 0.f && jl <= jmax[0] && sum0 < 0x1p-40f) ||
                          (l_run[1] == 0.f && jl <= jmax[1] && sum1 < 0x1p-40f);
        if (!__any(redo)) {
            l_run[0] += sum0;
            l_run[1] += sum1;
            return;
        }
        const int par = n & 1, j0 = key0(n);
        float alpha[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            f32x16 x;  // raw scores S[par][r], fetched from their fixed registers
            if (par == 0 && r == 0) asm volatile("" : "={v[128:143]}"(x));
            if (par == 0 && r == 1) asm volatile("" : "={v[144:159]}"(x));
            if (par == 1 && r == 0) asm volatile("" : "={v[160:175]}"(x));
            if (par == 1 && r == 1) asm volatile("" : "={v[176:191]}"(x));
            const f32x16 x_raw = x;
            if (j0 + 32 > L) {
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (j0 + 8 * (e >> 2) + 4 * hi + (e & 3) > jmax[r]) x[e] = -INFINITY;
            }
            float mx = -INFINITY;
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, x[e]);
            mx = fmaxf(mx, xhalf(mx)) * p.scale_log2e;
            const float m_old = (l_run[r] + xhalf(l_run[r]) > 0.f) ? m_ref[r] : -INFINITY;  // the row's history
            const float m_new = fmaxf(m_old, mx);
            alpha[r] = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_old - m_new);
            m_ref[r] = m_new;
            const float m_sub = (m_new == -INFINITY) ? 0.f : m_new;
            ms[r] = m_sub;
            float sum = 0.f;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                bf16x8 pk8;
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(fmaf(x[8 * t + e], p.scale_log2e, -m_sub));
                    const float p1 = __builtin_amdgcn_exp2f(fmaf(x[8 * t + e + 1], p.scale_log2e, -m_sub));
                    const bf16x2 pk = __builtin_convertvector(f32x2{p0, p1}, bf16x2);
                    pk8[e] = pk[0];
                    pk8[e + 1] = pk[1];
                    sum += (float)pk[0] + (float)pk[1];
                }
                // P[par][r][t] goes back to its fixed registers 216 + 4*(4*par + 2*r + t)
                switch (4 * par + 2 * r + t) {
                    case 0: asm volatile("" : : "{v[216:219]}"(pk8)); break;
                    case 1: asm volatile("" : : "{v[220:223]}"(pk8)); break;
                    case 2: asm volatile("" : : "{v[224:227]}"(pk8)); break;
                    case 3: asm volatile("" : : "{v[228:231]}"(pk8)); break;
                    case 4: asm volatile("" : : "{v[232:235]}"(pk8)); break;
                    case 5: asm volatile("" : : "{v[236:239]}"(pk8)); break;
                    case 6: asm volatile("" : : "{v[240:243]}"(pk8)); break;
                    default: asm volatile("" : : "{v[244:247]}"(pk8)); break;
                }
            }
            l_run[r] = l_run[r] * alpha[r] + sum;
            // the raw scores stay where they are to the end: this keeps the compiler from working
            // in place inside the fixed registers
            if (par == 0 && r == 0) asm volatile("" : : "{v[128:143]}"(x_raw));
            if (par == 0 && r == 1) asm volatile("" : : "{v[144:159]}"(x_raw));
            if (par == 1 && r == 0) asm volatile("" : : "{v[160:175]}"(x_raw));
            if (par == 1 && r == 1) asm volatile("" : : "{v[176:191]}"(x_raw));
        }
        if (__any(alpha[0] != 1.f || alpha[1] != 1.f))
            asm volatile(VS_ASM_RESCALE : : [alpha0] "v"(alpha[0]), [alpha1] "v"(alpha[1]) : VS_CLOB_ACC, VS_CLOB_TMP);
    };

    // One pipeline step with a softmax part: runs the block `ASM` and commits sub-block n.
#define VS_STEP(ASM, n)                                                                              \
    do {                                                                                             \
        float sum0_, sum1_;                                                                          \
        unsigned long long flag_;                                                                    \
        asm volatile(ASM : VS_SM_OUT : VS_ADDR, VS_SM_IN : VS_CLOBBERS);                             \
        commit(n, sum0_, sum1_, flag_);                                                              \
    } while (0)
#define VS_STEP_MASKED(ASM, n)                                                                       \
    do {                                                                                             \
        float sum0_, sum1_;                                                                          \
        unsigned long long flag_;                                                                    \
        const int d0_ = jmax[0] - (key0(n) + 4 * hi), d1_ = jmax[1] - (key0(n) + 4 * hi);            \
        unsigned long long mk0_, mk1_;                                                               \
        asm volatile(ASM                                                                             \
                     : VS_SM_OUT, [mk0] "=&s"(mk0_), [mk1] "=&s"(mk1_)                               \
                     : VS_ADDR, VS_SM_IN, [d0] "v"(d0_), [d1] "v"(d1_)                               \
                     : VS_CLOBBERS);                                                                 \
        commit(n, sum0_, sum1_, flag_);                                                              \
    } while (0)

    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): K(0) and Q have landed
    __syncthreads();                     // K(0) of every group is staged
    if (n_my > 0) {
        // K of the group's second tile and V of its first are requested on the way: from inside
        // the first two blocks, between their matrix instructions, when they are plain cache tiles.
        // sub-block 0: raw scores
        if (n_my > 1 && tile_of(1) * BN + BN <= Lc) {
            const unsigned long long ksrc = (unsigned long long)(kc + ((int64_t)(tile_of(1) * BN + rb * 32) * Hkv + g) * kRowBytes);
            asm volatile(VS_ASM_QK0_LOADS
                         :
                         : VS_ADDR, VS_KOFF, "{s[88:89]}"(ksrc), [ldsk] "s"(k_tile(1) + rb * (8 * 1024))
                         : VS_CLOBBERS, "scc");
        } else {
            issue(1, false);
            asm volatile(VS_ASM_QK0 : : VS_ADDR : VS_CLOBBERS);
        }
        // step 0 = QK(1) | SM(0) against the reference 0 (fine whenever the scaled scores are
        // moderate; otherwise commit() redoes it exactly)
        m_ref[0] = m_ref[1] = 0.f;
        if (tile_of(0) * BN + BN <= Lc) {
            const unsigned long long vsrc = (unsigned long long)(vc + ((int64_t)(tile_of(0) * BN + rb * 32) * Hkv + g) * kRowBytes);
            float sum0_, sum1_;
            unsigned long long flag_;
            asm volatile(VS_ASM_FIRST_LOADS
                         : VS_SM_OUT
                         : VS_ADDR, VS_SM_IN, VS_VOFF, "{s[90:91]}"(vsrc), [ldsv] "s"(v_tile(0) + rb * (8 * 1024))
                         : VS_CLOBBERS, "scc");
            commit(0, sum0_, sum1_, flag_);
        } else {
            issue(0, true);
            if (key0(0) + 32 > L) VS_STEP_MASKED(VS_ASM_FIRST_MASKED, 0);
            else VS_STEP(VS_ASM_FIRST, 0);
        }
    }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) k_rd[kk] += k_hop;  // the loop starts on K of tile 1, V of tile 0
    k_hop = -k_hop;

    for (int s = 0; s < n_steps; ++s) {
        // steps 2s+1 and 2s+2 of this group: they read K of tile s+1 and V of tile s
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's share of K(s+1), V(s) has landed
        __syncthreads();                     // ... and everybody's; K slot s&1 and V slot (s+1)&1 are free
        // tiles to stage now: K of tile s+2, V of tile s+1.  When both lie inside the cache rows
        // the first block issues the loads itself, between its matrix instructions.
        // (the block that can do that is the unmasked one: tile s must be a plain tile too)
        const bool loads_inside = s + 2 < n_my && tile_of(s + 2) * BN + BN <= Lc && tile_of(s + 1) * BN + BN <= Lc &&
                                  tile_of(s) * BN + BN <= Lc;
        if (!loads_inside) {
            issue(s + 2, false);
            issue(s + 1, true);
        }
        if (NKG > 1 && s >= n_my) continue;  // this group idles in the last step
        const int n = 2 * s + 1;
        if (s + 1 < n_my) {
            // step 2s+1: QK(2s+2) | PV(2s) | SM(2s+1)
            if (key0(n) + 32 > L) {
                VS_STEP_MASKED(VS_ASM_ODD_MASKED, n);
            } else if (loads_inside) {
                // this wave's share: rows 32*rb .. 32*rb+31 of the two tiles, head g
                const unsigned long long ksrc = (unsigned long long)(kc +
                    ((int64_t)(tile_of(s + 2) * BN + rb * 32) * Hkv + g) * kRowBytes);
                const unsigned long long vsrc = (unsigned long long)(vc +
                    ((int64_t)(tile_of(s + 1) * BN + rb * 32) * Hkv + g) * kRowBytes);
                float sum0_, sum1_;
                unsigned long long flag_;
                asm volatile(VS_ASM_ODD_LOADS
                             : VS_SM_OUT
                             : VS_ADDR, VS_SM_IN, VS_KOFF, VS_VOFF, "{s[88:89]}"(ksrc), "{s[90:91]}"(vsrc),
                               [ldsk] "s"(k_tile(s) + rb * (8 * 1024)), [ldsv] "s"(v_tile(s + 1) + rb * (8 * 1024))
                             : VS_CLOBBERS, "scc");
                commit(n, sum0_, sum1_, flag_);
            } else {
                VS_STEP(VS_ASM_ODD, n);
            }
            // step 2s+2: QK(2s+3) | PV(2s+1) | SM(2s+2)
            if (key0(n + 1) + 32 > L) VS_STEP_MASKED(VS_ASM_EVEN_MASKED, n + 1);
            else VS_STEP(VS_ASM_EVEN, n + 1);
        } else {
            // the group's last tile: step 2s+1 = PV(2s) | SM(2s+1), then PV(2s+1)
            if (key0(n) + 32 > L) VS_STEP_MASKED(VS_ASM_ODD_LAST_MASKED, n);
            else VS_STEP(VS_ASM_ODD_LAST, n);
            asm volatile(VS_ASM_TAIL : : VS_ADDR : VS_CLOBBERS);
        }
        // the next step reads the other slots
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) k_rd[kk] += k_hop;
        v_rd[0] += v_hop;
        v_rd[1] += v_hop;
        k_hop = -k_hop;
        v_hop = -v_hop;
    }
#undef VS_ADDR
#undef VS_KOFF
#undef VS_VOFF
#undef VS_SM_OUT
#undef VS_SM_IN
#undef VS_CLOBBERS
#undef VS_STEP
#undef VS_STEP_MASKED

    asm volatile("; pipeline registers free");  // marker for the listing check of the build

    // fused compaction: the frame rows that stay (the carrier, or all rows of a question) are
    // copied into the cache, 16 bytes per thread, the workgroups of the launch taking turns (the
    // carrier's 1 KB is done by the first one alone; no workgroup of this launch reads the
    // cache rows written here)
    if (p.k_append_dst && p.F > 1) {
        // a run: row T-1 of every frame goes behind the cache's rows, frame f to row Lc + f
        const int c16 = kv_row_bytes / 16, n16 = p.F * c16;
        const int n_thr = kGroupThreads * NKG, n_wgs = p.n_row_tiles * nsplit * HF;
        for (int ch = wg_id * n_thr + tid; ch < n16; ch += n_wgs * n_thr) {
            const int f = ch / c16;
            const int64_t from = ((int64_t)f * T + (T - 1)) * c16 + (ch - f * c16);
            reinterpret_cast<uint4*>(p.k_append_dst)[ch] = reinterpret_cast<const uint4*>(kf0)[from];
            reinterpret_cast<uint4*>(p.v_append_dst)[ch] = reinterpret_cast<const uint4*>(vf0)[from];
        }
    } else if (p.k_append_dst) {
        const int n16 = (T - p.append_first) * (kv_row_bytes / 16);
        const uint4* ksrc = reinterpret_cast<const uint4*>(kf + (int64_t)p.append_first * kv_row_bytes);
        const uint4* vsrc = reinterpret_cast<const uint4*>(vf + (int64_t)p.append_first * kv_row_bytes);
        const int n_thr = kGroupThreads * NKG, n_wgs = p.n_row_tiles * nsplit * HF;
        for (int ch = wg_id * n_thr + tid; ch < n16; ch += n_wgs * n_thr) {
            reinterpret_cast<uint4*>(p.k_append_dst)[ch] = ksrc[ch];
            reinterpret_cast<uint4*>(p.v_append_dst)[ch] = vsrc[ch];
        }
    }
    f32x16 o[2][4];
    asm volatile(VS_ASM_READ_O
                 : "={v[0:15]}"(o[0][0]), "={v[16:31]}"(o[0][1]), "={v[32:47]}"(o[0][2]), "={v[48:63]}"(o[0][3]),
                   "={v[64:79]}"(o[1][0]), "={v[80:95]}"(o[1][1]), "={v[96:111]}"(o[1][2]), "={v[112:127]}"(o[1][3])
                 :
                 : VS_CLOB_ACC);
    float l_tot[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        l_tot[r] = l_run[r] + xhalf(l_run[r]);
        if (!(l_tot[r] > 0.f)) m_ref[r] = -INFINITY;  // nothing accumulated: the made-up reference must not count
    }

    // ---- output of one row group: lane (q = l32, hi) holds dims 32*db + 8*(e>>2) + 4*hi + (e&3) ----
    auto emit = [&](int r, const f32x16 (&oo)[4], float m_row, float l_row) {
        const float inv = (l_row > 0.f) ? 1.0f / l_row : 0.f;
        const int rg = rb * 2 + r;  // 32-row group inside the row tile
        if (p.nsplit == 1) {
            if (r_mine[r] < p.M) {
                const int t = r_mine[r] / G, hl = r_mine[r] - t * G;
                __bf16* orow = out + ((int64_t)t * p.Hq + (int64_t)g * G + hl) * D;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        bf16x4 wv;
#pragma unroll
                        for (int j = 0; j < 4; ++j) wv[j] = (__bf16)(oo[db][4 * e4 + j] * inv);
                        *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * e4 + 4 * hi) = wv;
                    }
            }
        } else {
            // normalised partials in register order: every store instruction writes 1 KB contiguous
            const int64_t unit = (int64_t)c * p.n_row_tiles + rt;
            f16x8* po = reinterpret_cast<f16x8*>(p.part_o) + (unit * 4 + rg) * (8 * 64) + lane;
            // the row's largest entry (this lane holds 64 of its 128 dims, lane ^ 32 the rest)
            float big = 0.f;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) big = fmaxf(big, fabsf(oo[db][e]));
            big *= inv;
            big = fmaxf(big, xhalf(big));
            const PartScale sc = part_scale(big);
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    f16x8 wv;
#pragma unroll
                    for (int j = 0; j < 8; ++j) wv[j] = (_Float16)((oo[db][8 * h2 + j] * inv) * sc.scale);  // (the second product is exact)
                    // (non-temporal also when this launch reads the partials back: the lines are then
                    // written through while the kernel runs, instead of being left for the write-back at
                    // its end: 0.3 us per launch)
                    __builtin_nontemporal_store(wv, &po[(db * 2 + h2) * 64]);
                }
            if (hi == 0) {
                const int64_t prow = (int64_t)c * p.m_pad + r_mine[r];
                *reinterpret_cast<float4*>(p.part_ml + prow * 4) = make_float4(m_row, l_row, sc.inv_scale, 0.f);
            }
        }
    };

    if (NKG == 1) {
        emit(0, o[0], m_ref[0], l_tot[0]);
        emit(1, o[1], m_ref[1], l_tot[1]);
    } else {
        // ---- merge the key groups through LDS.  The two wavefronts that hold the same 64 rows
        //      (same lanes) swap halves: the wavefront of key group kg keeps row group kg, hands
        //      the other one over, and finishes its own, so the closing work is shared. ----
        __syncthreads();  // all tiles consumed, the stage buffers are free
        float* xo = reinterpret_cast<float*>(dyn_smem);  // [4 waves][16 x f32x4][64 lanes]
        float* xml = xo + 4 * 16 * 64 * 4;               // [4 waves][32 rows][2]
        auto hand_over = [&](int r) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    f32x4 wv;
#pragma unroll
                    for (int j = 0; j < 4; ++j) wv[j] = o[r][db][4 * e4 + j];
                    *reinterpret_cast<f32x4*>(&xo[((w * 16 + db * 4 + e4) * 64 + lane) * 4]) = wv;
                }
            if (hi == 0) {
                xml[(w * 32 + l32) * 2 + 0] = m_ref[r];
                xml[(w * 32 + l32) * 2 + 1] = l_tot[r];
            }
        };
        auto take_over = [&](int r) {
            const int pw = w ^ 2;  // the partner: same rows, other key group
            const float m1 = xml[(pw * 32 + l32) * 2 + 0], l1 = xml[(pw * 32 + l32) * 2 + 1];
            const float m_new = fmaxf(m_ref[r], m1);
            const float a0 = (m_ref[r] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_ref[r] - m_new);
            const float a1 = (m1 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m1 - m_new);
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    const f32x4 wv = *reinterpret_cast<const f32x4*>(&xo[((pw * 16 + db * 4 + e4) * 64 + lane) * 4]);
#pragma unroll
                    for (int j = 0; j < 4; ++j) o[r][db][4 * e4 + j] = o[r][db][4 * e4 + j] * a0 + wv[j] * a1;
                }
            emit(r, o[r], m_new, l_tot[r] * a0 + l1 * a1);
        };
        if (kg == 0) hand_over(1); else hand_over(0);
        __syncthreads();
        if (kg == 0) take_over(0); else take_over(1);
    }

    if (p.arrivals) {
        // ---- merge of the splits inside this launch.  Every workgroup has stored its
        // partial result above (ordinary stores: they stay in the XCD's L2, and all splits
        // of the unit run on this XCD).  Once the stores of all its wavefronts have been
        // acknowledged the workgroup counts itself in.  Then either the workgroups of the unit
        // share the merge (below), or the one that finds all others counted reads their partials
        // back from L2 and writes the unit's output rows alone, and nobody waits for anybody.
        // Either way the sums run over the splits in index order and take a workgroup's own part
        // rounded as stored, so the result does not depend on which workgroup comes last, and
        // equals what prefill_combine_kernel computes. ----
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        __syncthreads();                     // also: the exchange area is free again
        unsigned* const box = reinterpret_cast<unsigned*>(dyn_smem);
        unsigned* const counter = p.arrivals + (int64_t)(gf * p.n_row_tiles + rt) * (kCounterStrideBytes / 4);
        // (an increment that wraps: 0, 1, .., nsplit - 1, 0: the counter is back at zero with the last
        // arrival, for the next launch and as the sign that all have arrived)
        if (tid == 0) *box = __builtin_amdgcn_atomic_inc32(counter, (unsigned)(nsplit - 1), __ATOMIC_RELAXED, "workgroup");
        __syncthreads();
        const unsigned before = *box;
        if (p.share_merge) {
            // ---- The merge shared by the workgroups of the unit.  Those that are not the last to
            // arrive look at the counter again, with read-modify-writes (adding a zero the compiler
            // cannot see), which are executed at the L2 like the count itself and never served by the
            // compute unit's cache, a bounded number of times: a zero says that the last one has
            // arrived.  Whoever knows that, knows that every partial result of the unit is complete
            // in this L2, and merges its own pieces: of the unit's 4 row groups x 8 pieces of 16
            // features per lane, wavefront w of split j takes those from (w nsplit + j) * ppw on, ppw = 1,
            // 2 or 4, so that the work is spread over the unit's compute units and (up to 8 splits) one
            // round trip brings in all a wavefront needs.  The sums are those of the
            // single-workgroup merge below and of prefill_combine_kernel, in the same order.  A
            // workgroup that has looked max_looks times in vain (its unit's workgroups are not all
            // running at once: the device is shared, or part of it is masked) reports through the
            // same host word as a misplaced one and leaves its pieces unmerged: the next call
            // returns VS_ERR_PLACEMENT and the library merges with the second kernel from then on. ----
            if (before + 1 != (unsigned)nsplit) {
                unsigned zero = 0;
                asm volatile("" : "+s"(zero));
                unsigned* const seen_box = box + 1;
                if (tid == 0) {
                    unsigned ok = 0;
                    for (int n = 0; n < p.max_looks && !ok; ++n) {
                        ok = __hip_atomic_fetch_add(counter, zero, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == 0u;
                        if (!ok) __builtin_amdgcn_s_sleep(2);
                    }
                    *seen_box = ok;
                    if (!ok) __hip_atomic_store(p.misplaced, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                }
                __syncthreads();
                if (!*seen_box) return;
            }
            // pieces per wavefront: the fewest that cover the 32 pieces with the unit's 2 NKG nsplit wavefronts
            const int ppw = NKG == 2 ? (nsplit >= 8 ? 1 : nsplit >= 4 ? 2 : 4) : (nsplit >= 16 ? 1 : nsplit >= 8 ? 2 : nsplit >= 4 ? 4 : 8);
            const int first = (w * nsplit + split) * ppw;            // of the unit's 4 x 8 pieces: dealt to the workgroups in turn
            if (first >= 32) return;
            const int rg = first >> 3, piece0 = first & 7;
            const int m = rt * BM + rg * 32 + l32;  // the lane's row of the packed rows
            const bool row_ok = m < M;
            const int t = row_ok ? div_small(m, G, inv_G) : 0, hl = m - t * G;
            __bf16* const orow = out + ((int64_t)t * p.Hq + (int64_t)g * G + hl) * D;
            const float* const ml0 = p.part_ml + ((int64_t)gf * p.m_pad + m) * 4;
            const int64_t ml_step = (int64_t)HF * p.m_pad * 4;  // floats between splits
            const f16x8* const po0 = reinterpret_cast<const f16x8*>(p.part_o) +
                                      (((int64_t)gf * p.n_row_tiles + rt) * 4 + rg) * (8 * 64) + piece0 * 64 + lane;
            const int64_t po_step = (int64_t)HF * p.n_row_tiles * 4 * (8 * 64);  // f16x8 between splits
            auto share = [&](auto ns_tag, auto pieces_tag) {
                constexpr int NS = decltype(ns_tag)::value, PIECES = decltype(pieces_tag)::value;
                float4 ml[NS];  // reference, sum, inverse scale of the stored row
                f16x8 v[NS][PIECES];
#pragma unroll
                for (int u = 0; u < NS; ++u) ml[u] = *reinterpret_cast<const float4*>(ml0 + u * ml_step);
#pragma unroll
                for (int u = 0; u < NS; ++u)
#pragma unroll
                    for (int k = 0; k < PIECES; ++k) v[u][k] = po0[u * po_step + k * 64];
                float m_star = -INFINITY;
#pragma unroll
                for (int u = 0; u < NS; ++u) m_star = fmaxf(m_star, ml[u].x);
                float wgt[NS], denom = 0.f;  // wgt: what the stored (scaled) row is multiplied by
#pragma unroll
                for (int u = 0; u < NS; ++u) {
                    const float ww = (ml[u].x != -INFINITY) ? __builtin_amdgcn_exp2f(ml[u].x - m_star) * ml[u].y : 0.f;
                    denom += ww;
                    wgt[u] = ww * ml[u].z;
                }
                const float inv = 1.0f / denom;
#pragma unroll
                for (int k = 0; k < PIECES; ++k) {
                    float acc[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
#pragma unroll
                    for (int u = 0; u < NS; ++u)
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[j] += wgt[u] * (float)v[u][k][j];
                    if (row_ok) {
                        // piece (db, h2) = (piece >> 1, piece & 1): dims 32 db + 16 h2 + 4 hi + 0..3, + 8
                        bf16x4 w0, w1;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            w0[j] = (__bf16)(acc[j] * inv);
                            w1[j] = (__bf16)(acc[4 + j] * inv);
                        }
                        __bf16* dst = orow + 16 * (piece0 + k) + 4 * hi;
                        *reinterpret_cast<bf16x4*>(dst) = w0;
                        *reinterpret_cast<bf16x4*>(dst + 8) = w1;
                    }
                }
            };
            using std::integral_constant;
            if (nsplit > 8) {  // piece by piece, splits in chunks of 8, exactly as prefill_combine_kernel does it
                auto ml_of = [&](int u) { return *reinterpret_cast<const float4*>(ml0 + u * ml_step); };
                for (int k = 0; k < ppw; ++k) {
                    float acc[8], denom;
                    auto v_of = [&](int u) { return po0[u * po_step + k * 64]; };
                    merge_splits_chunked<2>(nsplit, ml_of, v_of, acc, denom);
                    if (row_ok) {
                        const float inv = 1.0f / denom;
                        bf16x4 w0, w1;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            w0[j] = (__bf16)(acc[j] * inv);
                            w1[j] = (__bf16)(acc[4 + j] * inv);
                        }
                        __bf16* dst = orow + 16 * (piece0 + k) + 4 * hi;
                        *reinterpret_cast<bf16x4*>(dst) = w0;
                        *reinterpret_cast<bf16x4*>(dst + 8) = w1;
                    }
                }
                return;
            }
            if constexpr (NKG == 2) {
                switch (nsplit) {
                    case 2: share(integral_constant<int, 2>{}, integral_constant<int, 4>{}); break;
                    case 3: share(integral_constant<int, 3>{}, integral_constant<int, 4>{}); break;
                    case 4: share(integral_constant<int, 4>{}, integral_constant<int, 2>{}); break;
                    case 5: share(integral_constant<int, 5>{}, integral_constant<int, 2>{}); break;
                    case 6: share(integral_constant<int, 6>{}, integral_constant<int, 2>{}); break;
                    case 7: share(integral_constant<int, 7>{}, integral_constant<int, 2>{}); break;
                    default: share(integral_constant<int, 8>{}, integral_constant<int, 1>{}); break;
                }
            } else {
                switch (nsplit) {
                    case 2: share(integral_constant<int, 2>{}, integral_constant<int, 8>{}); break;
                    case 3: share(integral_constant<int, 3>{}, integral_constant<int, 8>{}); break;
                    case 4: share(integral_constant<int, 4>{}, integral_constant<int, 4>{}); break;
                    case 5: share(integral_constant<int, 5>{}, integral_constant<int, 4>{}); break;
                    case 6: share(integral_constant<int, 6>{}, integral_constant<int, 4>{}); break;
                    case 7: share(integral_constant<int, 7>{}, integral_constant<int, 4>{}); break;
                    default: share(integral_constant<int, 8>{}, integral_constant<int, 2>{}); break;
                }
            }
            return;
        }
        if (before + 1 == (unsigned)nsplit) {
            // the rows this wavefront has closed: row group kg of its 64 rows, or both
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                if (NKG == 2 && r != kg) continue;
                const int rg = rb * 2 + r;
                const bool row_ok = r_mine[r] < M;
                const int t = row_ok ? div_small(r_mine[r], G, inv_G) : 0, hl = r_mine[r] - t * G;
                __bf16* const orow = out + ((int64_t)t * p.Hq + (int64_t)g * G + hl) * D;
                const float* const ml0 = p.part_ml + ((int64_t)gf * p.m_pad + r_mine[r]) * 4;
                const int64_t ml_step = (int64_t)HF * p.m_pad * 4;       // floats between splits
                const f16x8* const po0 = reinterpret_cast<const f16x8*>(p.part_o) +
                                          (((int64_t)gf * p.n_row_tiles + rt) * 4 + rg) * (8 * 64) + lane;
                const int64_t po_step = (int64_t)HF * p.n_row_tiles * 4 * (8 * 64);  // f16x8 between splits
                // NS splits, the 8 pieces of a lane in PASSES rounds: everything of a round is
                // requested before anything is used (a round trip to L2 is what this tail costs)
                auto tail = [&](auto ns_tag, auto passes_tag) {
                    constexpr int NS = decltype(ns_tag)::value, PASSES = decltype(passes_tag)::value, PIECES = 8 / PASSES;
                    float4 ml[NS];  // reference, sum, inverse scale of the stored row
                    f16x8 v[NS][PIECES];
                    // (addresses are worked out here, per case: an opaque copy of the bases keeps the
                    // compiler from preparing those of all cases ahead of the switch)
                    const float* mlb = ml0;
                    const f16x8* pob = po0;
                    asm volatile("" : "+v"(mlb), "+v"(pob));
#pragma unroll
                    for (int u = 0; u < NS; ++u) ml[u] = *reinterpret_cast<const float4*>(mlb + u * ml_step);
#pragma unroll
                    for (int pass = 0; pass < PASSES; ++pass) {
#pragma unroll
                        for (int u = 0; u < NS; ++u)
#pragma unroll
                            for (int k = 0; k < PIECES; ++k) v[u][k] = pob[u * po_step + (pass * PIECES + k) * 64];
                        float m_star = -INFINITY;
#pragma unroll
                        for (int u = 0; u < NS; ++u) m_star = fmaxf(m_star, ml[u].x);
                        float wgt[NS], denom = 0.f;  // wgt: what the stored (scaled) row is multiplied by
#pragma unroll
                        for (int u = 0; u < NS; ++u) {
                            const float w = (ml[u].x != -INFINITY) ? __builtin_amdgcn_exp2f(ml[u].x - m_star) * ml[u].y : 0.f;
                            denom += w;
                            wgt[u] = w * ml[u].z;
                        }
                        const float inv = 1.0f / denom;
#pragma unroll
                        for (int k = 0; k < PIECES; ++k) {
                            float acc[8];
#pragma unroll
                            for (int j = 0; j < 8; ++j) acc[j] = 0.f;
#pragma unroll
                            for (int u = 0; u < NS; ++u)
#pragma unroll
                                for (int j = 0; j < 8; ++j) acc[j] += wgt[u] * (float)v[u][k][j];
                            if (row_ok) {
                                // piece (db, h2) = ((pass*PIECES + k) >> 1, & 1): dims 32 db + 16 h2 + 4 hi + 0..3, + 8
                                const int piece = pass * PIECES + k;
                                bf16x4 w0, w1;
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    w0[j] = (__bf16)(acc[j] * inv);
                                    w1[j] = (__bf16)(acc[4 + j] * inv);
                                }
                                __bf16* dst = orow + 16 * piece + 4 * hi;
                                *reinterpret_cast<bf16x4*>(dst) = w0;
                                *reinterpret_cast<bf16x4*>(dst + 8) = w1;
                            }
                        }
                    }
                };
                using std::integral_constant;
                constexpr int kPasses = NKG == 1 ? 2 : 1;  // (one key group: two row groups to do, fewer registers each)
                switch (nsplit) {
                    case 2: tail(integral_constant<int, 2>{}, integral_constant<int, kPasses>{}); break;
                    case 3: tail(integral_constant<int, 3>{}, integral_constant<int, kPasses>{}); break;
                    case 4: tail(integral_constant<int, 4>{}, integral_constant<int, kPasses>{}); break;
                    case 5: tail(integral_constant<int, 5>{}, integral_constant<int, kPasses>{}); break;
                    case 6: tail(integral_constant<int, 6>{}, integral_constant<int, kPasses>{}); break;
                    case 7: tail(integral_constant<int, 7>{}, integral_constant<int, 2>{}); break;
                    default: tail(integral_constant<int, 8>{}, integral_constant<int, 2>{}); break;
                }
                __builtin_amdgcn_sched_barrier(0);  // one row group at a time: its loads fill the registers
            }
        }
    }
}

// Merge of the per-split partials: out = sum_s w_s l_s Ohat_s / sum_s w_s l_s with
// w_s = 2^(m_s - m*).  One 64-thread block per (row tile, row group, dim block, half): the same
// lane -> element mapping as the attention kernel, so the partials are read 1 KB at a time; all
// loads of up to 8 splits, references and sums included, are issued before any is used.
__global__ __launch_bounds__(64) void prefill_combine_kernel(PrefillParams p) {
    const int lane = threadIdx.x, l32 = lane & 31, hi = lane >> 5;
    int b = blockIdx.x;
    const int h2 = b & 1; b >>= 1;
    const int db = b & 3; b >>= 2;
    const int rg = b & 3; b >>= 2;
    const int rt = b;
    const int g = blockIdx.y, frame = blockIdx.z;
    const int gf = g * p.F + frame, HF = p.Hkv * p.F;
    if (rt * BM + rg * 32 >= p.M) return;  // whole block beyond the rows
    const int r = rt * BM + rg * 32 + l32;
    const int rr = min(r, p.M - 1);
    float acc[8], denom;
    merge_splits_chunked<0>(
        p.nsplit,
        [&](int u) { return *reinterpret_cast<const float4*>(p.part_ml + ((int64_t)(u * HF + gf) * p.m_pad + rr) * 4); },
        [&](int u) {
            const int64_t unit = (int64_t)(u * HF + gf) * p.n_row_tiles + rt;
            return (reinterpret_cast<const f16x8*>(p.part_o) + (unit * 4 + rg) * (8 * 64) + lane)[(db * 2 + h2) * 64];
        },
        acc, denom);
    if (r >= p.M) return;
    const float inv = 1.0f / denom;
    const int t = r / p.G, hl = r - t * p.G;
    __bf16* orow = p.out + (int64_t)frame * p.T * p.Hq * D + ((int64_t)t * p.Hq + (int64_t)g * p.G + hl) * D +
                   32 * db + 16 * h2 + 4 * hi;
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
    bool merge_inside;  // the attention kernel merges the splits itself
};

// How this device deals workgroup ids to its XCDs, found once per device by xcd_probe_kernel:
// log2 of the number of XCDs if ids go to them in turn (id mod count), -1 if not (or not yet
// probed, or after a workgroup has reported that it ran elsewhere): then the splits are merged
// by the second kernel.
int g_xcd_shift[16] = {-1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1};
unsigned long long g_xcc_of_residue[16] = {};  // XCC_ID read for ids of residue r: bits 4r .. 4r+3
// One word of pinned host memory per device (allocated by the probe, kept until the process
// ends), set by any workgroup of an in-kernel-merge launch that finds itself on an XCD other
// than the probed one.
unsigned* g_misplaced[16] = {};      // as the host addresses it
unsigned* g_misplaced_dev[16] = {};  // as the kernels address it
// tests: 3 = the probe-derived table is handed to the kernels rotated by one XCD; 4 = workgroups that
// wait for the last of their unit do not look at all and give up
int g_tune_guard_test = 0;

__global__ void xcd_probe_kernel(unsigned* out) {
    unsigned x;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
    if (threadIdx.x == 0) out[blockIdx.x] = x & 15u;
}

Plan make_plan(const vs_shape& s, int n_tokens, int len, int n_frames) {
    const int G = s.n_q_heads / s.n_kv_heads;
    const int M = n_tokens * G;
    Plan pl;
    pl.n_row_tiles = (M + BM - 1) / BM;
    pl.m_pad = pl.n_row_tiles * BM;
    const int units = pl.n_row_tiles * s.n_kv_heads * n_frames;
    const int max_tiles = (len + n_frames - 1 + n_tokens + BN - 1) / BN;
    // 4-wave workgroups (two key groups) when there are enough key tiles to share out
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
    // More units than half the chip has compute units (runs of frames, long runs of tokens): the
    // workgroups go through the chip in several rounds, and more, shorter ones may end sooner
    // than few long ones with a thin last round.  Estimated time of a launch in units of one
    // pipeline step (one tile per key group, ~2 us): rounds x (steps of a workgroup + its fixed
    // cost of ~2.25 steps), plus the merge when there are splits.
    if (units > 128 && pl.kvg == 2) {
        float best = 0.f;
        for (int cand = 1; cand <= 8 && cand <= max_tiles / pl.kvg; ++cand) {
            const int rounds = (units * cand + 255) / 256;
            const int steps = ((max_tiles + cand - 1) / cand + pl.kvg - 1) / pl.kvg;
            const float cost = rounds * (steps + 2.25f) + (cand > 1 ? 1.25f : 0.f);
            if (cand == 1 || cost < best) {
                best = cost;
                ns = cand;
            }
        }
    }
    if (g_tune_prefill_splits) ns = g_tune_prefill_splits < max_tiles ? g_tune_prefill_splits : (max_tiles > 0 ? max_tiles : 1);
    pl.nsplit = ns;
    int dev = 0;
    // (more than 8 splits: only the shared merge knows how)
    pl.merge_inside = g_tune_prefill_merge != 2 && ns > 1 && (ns <= 8 || g_tune_prefill_merge != 1) &&
                      ns <= kMaxPrefillSplits && pl.n_row_tiles * n_frames <= kMaxRowTiles &&
                      hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 16 && g_xcd_shift[dev] >= 0 && g_misplaced[dev];
    return pl;
}

template <int KVG>
hipError_t launch_kvg(const PrefillParams& p, const Plan& pl, int n_kv_heads, hipStream_t st) {
    static bool attr_set_on[16] = {};  // dynamic LDS above 64 KB has to be allowed once per kernel and device
    constexpr int kLds = KVG * kGroupLds;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return hipErrorInvalidDevice;
    bool& attr_set = attr_set_on[dev];
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_mfma_kernel<KVG>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    // x runs fastest in dispatch order: all workgroups that read one K/V slice are neighbours
    const dim3 grid = p.arrivals ? dim3(prefill_grid_ids(pl.n_row_tiles * p.F * n_kv_heads, pl.nsplit, p.xcd_shift))
                                 : dim3(n_kv_heads, pl.nsplit, pl.n_row_tiles * p.F);
    prefill_mfma_kernel<KVG><<<grid, kGroupThreads * KVG, kLds, st>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.nsplit == 1 || p.arrivals) return e;
    prefill_combine_kernel<<<dim3(pl.n_row_tiles * 4 * 4 * 2, n_kv_heads, p.F), 64, 0, st>>>(p);
    return hipGetLastError();
}

}  // namespace

int xcd_shift_of_device(int dev) { return dev >= 0 && dev < 16 ? g_xcd_shift[dev] : -1; }

hipError_t probe_xcd_mapping(void* scratch, hipStream_t st) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= 16 || g_xcd_shift[dev] >= 0) return e;
    constexpr int kProbe = 64;
    unsigned ids[kProbe];
    xcd_probe_kernel<<<kProbe, 64, 0, st>>>((unsigned*)scratch);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = hipMemcpyAsync(ids, scratch, sizeof(ids), hipMemcpyDeviceToHost, st)) != hipSuccess) return e;
    if ((e = hipStreamSynchronize(st)) != hipSuccess) return e;
    for (int shift = 0; shift <= 4; ++shift) {
        const int n = 1 << shift;
        bool ok = true;
        for (int i = 0; i < kProbe && ok; ++i) ok = ids[i] == ids[i % n];          // period n
        for (int i = 0; i < n && ok; ++i)
            for (int j = 0; j < i && ok; ++j) ok = ids[i] != ids[j];                // n different XCDs
        if (ok) {
            unsigned long long table = 0;
            for (int i = 0; i < n; ++i) table |= (unsigned long long)(ids[i] & 15u) << (4 * i);
            if (!g_misplaced[dev]) {
                void* flag = nullptr;
                void* flag_dev = nullptr;
                if ((e = hipHostMalloc(&flag, 64, hipHostMallocMapped)) != hipSuccess) return e;
                *static_cast<unsigned*>(flag) = 0u;
                if ((e = hipHostGetDevicePointer(&flag_dev, flag, 0)) != hipSuccess) return e;
                g_misplaced[dev] = static_cast<unsigned*>(flag);
                g_misplaced_dev[dev] = static_cast<unsigned*>(flag_dev);
            }
            g_xcc_of_residue[dev] = table;
            g_xcd_shift[dev] = shift;
            break;
        }
    }
    return hipSuccess;
}

bool prefill_placement_fault(int dev) {
    if (dev < 0 || dev >= 16 || !g_misplaced[dev]) return false;
    if (*static_cast<volatile unsigned*>(g_misplaced[dev]) == 0u) return false;
    g_xcd_shift[dev] = -1;  // from now on the second kernel merges
    *static_cast<volatile unsigned*>(g_misplaced[dev]) = 0u;
    return true;
}

void prefill_guard_test_mode(int on) { g_tune_guard_test = on; }

bool xcd_placement_of_device(int dev, XcdPlacement* out) {
    if (dev < 0 || dev >= 16 || g_xcd_shift[dev] < 0 || !g_misplaced_dev[dev] || g_tune_prefill_merge == 2) return false;
    out->xcd_shift = g_xcd_shift[dev];
    out->xcc_of_residue = g_xcc_of_residue[dev];
    if (g_tune_guard_test == 3 && out->xcd_shift > 0)  // (as for the prefill: the table rotated by one XCD)
        out->xcc_of_residue = (out->xcc_of_residue >> 4) | ((out->xcc_of_residue & 15ull) << (4 * ((1 << out->xcd_shift) - 1)));
    out->misplaced = g_misplaced_dev[dev];
    out->max_looks = g_tune_guard_test == 4 ? 0 : 8192;
    return true;
}

size_t prefill_mfma_workspace_bytes(const vs_shape& s, int32_t max_q_tokens) {
    const int G = s.n_q_heads / s.n_kv_heads;
    const int64_t M = (int64_t)max_q_tokens * G;
    const int64_t m_pad = ((M + BM - 1) / BM) * BM;
    const int64_t slots = (int64_t)kMaxPrefillSplits * s.n_kv_heads * m_pad;
    return (size_t)(slots * (D * sizeof(_Float16) + 4 * sizeof(float)));
}

// Bytes the partial results of a run of n_frames frames can take (the plan's own choice of
// splits; a tuning override that asks for more is refused by the caller's size check).
size_t prefill_frames_workspace_bytes(const vs_shape& s, int32_t n_frames, int32_t n_tokens, int32_t nsplit) {
    const int G = s.n_q_heads / s.n_kv_heads;
    const int64_t M = (int64_t)n_tokens * G;
    const int64_t m_pad = ((M + BM - 1) / BM) * BM;
    const int64_t slots = (int64_t)nsplit * s.n_kv_heads * n_frames * m_pad;
    return (size_t)(slots * (D * sizeof(_Float16) + 4 * sizeof(float)));
}

int prefill_frames_splits(const vs_shape& s, int32_t n_frames, int32_t n_tokens, int32_t len) {
    return make_plan(s, n_tokens, len, n_frames).nsplit;
}

hipError_t launch_prefill_mfma(const vs_shape& s, const void* kc, const void* vc, int32_t len,
                               const void* q, const void* kf, const void* vf, int32_t n_tokens,
                               void* out, void* k_append_dst, void* v_append_dst, void* counters,
                               void* workspace, hipStream_t st, int32_t n_frames, bool append_all) {
    const Plan pl = make_plan(s, n_tokens, len, n_frames);
    PrefillParams p;
    p.kc = (const __bf16*)kc;
    p.vc = (const __bf16*)vc;
    p.q = (const __bf16*)q;
    p.kf = (const __bf16*)kf;
    p.vf = (const __bf16*)vf;
    p.out = (__bf16*)out;
    p.k_append_dst = (__bf16*)k_append_dst;
    p.v_append_dst = (__bf16*)v_append_dst;
    p.append_first = append_all ? 0 : n_tokens - 1;
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
    p.inv_G = 1.0f / (float)p.G;
    p.inv_nsplit = 1.0f / (float)pl.nsplit;
    p.arrivals = nullptr;
    p.xcd_shift = p.units_per_xcd = 0;
    p.xcc_of_residue = 0;
    p.misplaced = nullptr;
    p.share_merge = 0;
    p.max_looks = 0;
    p.inv_row_tiles = 1.0f / (float)pl.n_row_tiles;
    p.F = n_frames;
    p.inv_frame_tiles = 1.0f / (float)(pl.n_row_tiles * n_frames);
    if (pl.merge_inside && counters) {
        int dev = 0;
        (void)hipGetDevice(&dev);
        p.arrivals = (unsigned*)counters;
        p.xcd_shift = g_xcd_shift[dev];
        p.units_per_xcd = prefill_units_per_xcd(pl.n_row_tiles * s.n_kv_heads * n_frames, p.xcd_shift);
        p.xcc_of_residue = g_xcc_of_residue[dev];
        if (g_tune_guard_test == 3 && p.xcd_shift > 0)  // entry r names the XCD of residue r + 1: every workgroup is "misplaced"
            p.xcc_of_residue = (p.xcc_of_residue >> 4) | ((p.xcc_of_residue & 15ull) << (4 * ((1 << p.xcd_shift) - 1)));
        p.misplaced = g_misplaced_dev[dev];
        if (g_tune_prefill_merge != 1) {
            p.share_merge = 1;
            p.max_looks = g_tune_guard_test == 4 ? 0 : 8192;  // ~0.3 us a look: some milliseconds at most
        }
    }
    const int64_t slots = (int64_t)pl.nsplit * s.n_kv_heads * n_frames * pl.m_pad;
    p.part_ml = (float*)workspace;
    p.part_o = (_Float16*)(p.part_ml + slots * 4);
    return pl.kvg == 1 ? launch_kvg<1>(p, pl, s.n_kv_heads, st) : launch_kvg<2>(p, pl, s.n_kv_heads, st);
}

}  // namespace vs
