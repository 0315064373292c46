// The dense layers around the attention for a run of at most 192 token rows on gfx950
// (Section 3.1: Q = X W_Q, K = X W_K, V = X W_V; the rest of the decoder layer of the backbone the
// method is built on, Section 4.1: output projection, gated feed-forward, residual sums, RMS norm).
//
//   out [T][N] = X [T][K] . W [N][K]^T      bf16 operands, fp32 sums
//
// T <= 192 rows meet N weight rows: every weight is needed once, so the launch is bound by reading W
// from HBM, and behind that by what a compute unit can take in from L2, because every workgroup
// needs X for all of its K range.  A workgroup owns all 192 rows of a block of 64, 128 or 160
// output features (the wider the block, the fewer times X passes through a compute unit) and a
// contiguous share of K (split-K where N alone gives too few blocks for 256 compute units).
// 64 input features at a time, a tile of 192 rows of X and the block's rows of W goes from global
// memory straight into LDS, whole 128-byte lines per 8 lanes, into a ring of 3 or 4 buffers, one
// barrier per tile.  The 16-byte pieces of a row are stored permuted (piece ^ ((row >> 1) & 7))
// so that the fragment reads of v_mfma_f32_16x16x32_bf16 (16 rows x one piece) hit all banks.
// Of the 8 wavefronts, w multiplies the 16-row sub-tiles w&3, +4, +8 with all feature sub-tiles
// for half w>>2 of each tile's input features; the halves are added through LDS at the end.
//
// What happens to the sums (fp32) is the caller's choice:
//   store      out = bf16(sum)
//   residual   out = bf16(res + sum)                       (res [T][N], bf16)
//   gated      out [T][N/2]: feature 2j is the gate g, 2j+1 the value u of output j:
//              out_j = bf16(g / (1 + exp(-g)) * u)         (SiLU gate, as in the backbone)
// With split-K the workgroups leave their fp32 sums in the workspace, in register order (a store
// instruction writes 1 KB); the shares are added in index order, and the above done, either by a
// second small kernel or, when the caller provides arrival counters (the decoder layer does), inside
// the launch by the workgroups of a block together, each its rows, once the last of them has
// finished: the same sums in the same order.  Without split-K the multiplying kernel does it itself.
#include <hip/hip_runtime.h>

#include "vs_internal.h"
#include "vs_prefill_map.h"

namespace vs {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr;

constexpr int kRows = 192;      // rows of X a tile holds; rows from T on repeat row T-1
constexpr int kThreads = 512;

struct LinParams {
    const __bf16* x;    // [T][ldx]
    const __bf16* w;    // [N][K]
    const __bf16* res;  // [T][N] or null
    __bf16* out;        // [T][N], or [T][N/2] when gated
    // store mode may cut the features into up to three tensors (Q, K, V): features below seg_end[0]
    // go to out, those below seg_end[1] to out1 (row length seg_end[1] - seg_end[0]), the rest to out2
    __bf16* out1;
    __bf16* out2;
    int seg_end[2];
    float* ws;          // split-K shares, or null
    int T, N, K, ldx;
    int mode;           // vs_linear_mode
    int ksplit, tiles_per_split;
    // split-K shares added inside the launch (null: by linear_reduce_kernel).  All shares of a block
    // then run on one XCD and meet in its L2, exactly as the key splits of the prefill kernel do
    // (vs_prefill_map.h: unit = block, split = share), counted in and waited for in the same way.
    unsigned* arrivals;          // one counter per block, kCounterStrideBytes apart, zero between launches
    unsigned* misplaced;         // pinned host word through which a workgroup reports
    unsigned long long xcc_of_residue;
    int xcd_shift, units_per_xcd, n_blocks, max_looks;
    float inv_ksplit;
};

// s_waitcnt vmcnt(n) only (gfx9 encoding: vmcnt in bits 3:0 and 15:14; expcnt, lgkmcnt left at "no wait")
#define VS_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0F70)

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + __expf(-g)) * u; }

// The finished sums of a block of rows leave through LDS: the accumulators (lane (i16, kq) holds
// rows 4 kq + 0..3 of feature i16 of a 16 x 16 sub-tile) are put down as a row-major fp32 tile,
// and then every thread takes 8 neighbouring features of a row, does what the mode asks and
// writes 16 bytes (8 when gated), so that rows go out, and residual rows come in, in whole
// lines instead of two bytes at a time.  The tile's row length in floats is NT + 4: with it the
// 64 lanes of an accumulator store hit 64 different banks.
template <int NT>
__device__ __forceinline__ void put_acc(float* tile, f32x4 v, int row0, int col0, int lane) {
    const int i16 = lane & 15, kq = lane >> 4;
#pragma unroll
    for (int e = 0; e < 4; ++e) tile[(row0 + 4 * kq + e) * (NT + 4) + col0 + i16] = v[e];
}

// rows_local rows of the tile; local row r is row row_of(r) of the output.
template <int NT, typename RowOf>
__device__ __forceinline__ void write_tile(const LinParams& p, const float* tile, int rows_local, int n0, int tid,
                                           int n_threads, RowOf row_of) {
    constexpr int kChunks = NT / 8;
    for (int idx = tid; idx < rows_local * kChunks; idx += n_threads) {
        const int r = idx / kChunks, c8 = (idx - r * kChunks) * 8;
        const int m = row_of(r), n = n0 + c8;
        if (m >= p.T || n >= p.N) continue;
        const f32x4 lo = *reinterpret_cast<const f32x4*>(tile + r * (NT + 4) + c8);
        const f32x4 hi4 = *reinterpret_cast<const f32x4*>(tile + r * (NT + 4) + c8 + 4);
        float v[8] = {lo[0], lo[1], lo[2], lo[3], hi4[0], hi4[1], hi4[2], hi4[3]};
        if (p.mode == VS_LINEAR_GATED) {
            const int half = p.N >> 1;
            __bf16* dst = p.out + (int64_t)m * half + (n >> 1);
            if (n + 8 <= p.N && (half & 3) == 0) {
                bf16x4 y;
#pragma unroll
                for (int j = 0; j < 4; ++j) y[j] = (__bf16)silu_mul(v[2 * j], v[2 * j + 1]);
                *reinterpret_cast<bf16x4*>(dst) = y;
            } else {
                for (int j = 0; j < 4 && n + 2 * j + 1 < p.N; ++j) dst[j] = (__bf16)silu_mul(v[2 * j], v[2 * j + 1]);
            }
            continue;
        }
        // where feature n lives: tensor, its row length, column (a chunk of 8 never straddles two
        // tensors when their first features are multiples of 8; otherwise it goes out one by one)
        __bf16* base = p.out;
        int ld = p.seg_end[0], col = n, end = p.seg_end[0];
        if (n >= p.seg_end[0]) {
            const bool second = n < p.seg_end[1];
            base = second ? p.out1 : p.out2;
            ld = second ? p.seg_end[1] - p.seg_end[0] : p.N - p.seg_end[1];
            col = n - (second ? p.seg_end[0] : p.seg_end[1]);
            end = second ? p.seg_end[1] : p.N;
        }
        __bf16* dst = base + (int64_t)m * ld + col;
        if (n + 8 <= end && (ld & 7) == 0 && (col & 7) == 0) {
            if (p.mode == VS_LINEAR_RESIDUAL) {
                const bf16x8 rv = *reinterpret_cast<const bf16x8*>(p.res + (int64_t)m * p.N + n);
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] += (float)rv[j];
            }
            bf16x8 y;
#pragma unroll
            for (int j = 0; j < 8; ++j) y[j] = (__bf16)v[j];
            *reinterpret_cast<bf16x8*>(dst) = y;
        } else {
            for (int j = 0; j < 8 && n + j < p.N; ++j) {
                // (one by one, each feature to its own tensor)
                const int nn = n + j;
                __bf16* b1 = p.out;
                int l1 = p.seg_end[0], c1 = nn;
                if (nn >= p.seg_end[0]) {
                    const bool second = nn < p.seg_end[1];
                    b1 = second ? p.out1 : p.out2;
                    l1 = second ? p.seg_end[1] - p.seg_end[0] : p.N - p.seg_end[1];
                    c1 = nn - (second ? p.seg_end[0] : p.seg_end[1]);
                }
                float y = v[j];
                if (p.mode == VS_LINEAR_RESIDUAL) y += (float)p.res[(int64_t)m * p.N + nn];
                b1[(int64_t)m * l1 + c1] = (__bf16)y;
            }
        }
    }
}

template <int NSUB, int RING>
__global__ __launch_bounds__(kThreads) void linear_kernel(LinParams p) {
    constexpr int kTileN = 16 * NSUB;
    constexpr int kTileBytes = (kRows + kTileN) * 128;
    constexpr int kGroups = (kRows + kTileN) / 8;   // load instructions (8 rows each) per tile
    constexpr int kMaxMine = (kGroups + 7) / 8;     // ... of one wavefront, at most
    constexpr int kAccs = 3 * NSUB;
    extern __shared__ __attribute__((aligned(1024))) char ring[];  // RING tiles: 192 rows of X, then the rows of W

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, kq = lane >> 4;
    int blk = blockIdx.x, share = blockIdx.y;
    if (p.arrivals) {
        // 1-D grid: ids of one residue modulo the number of XCDs go to one XCD, and block b's shares
        // take consecutive slots of one residue
        const PrefillSlot at = prefill_slot_of_id(blockIdx.x, p.n_blocks, p.units_per_xcd, p.ksplit, p.inv_ksplit, p.xcd_shift);
        if (at.unit < 0) return;  // spare ids
        unsigned xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        if ((xcc & 15u) != (unsigned)((p.xcc_of_residue >> (4 * at.xcd)) & 15u) && threadIdx.x == 0)
            __hip_atomic_store(p.misplaced, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);  // (see vs_workspace_init)
        blk = at.unit;
        share = at.split;
    }
    const int n0 = blk * kTileN;
    const int n_tiles_all = p.K / 64;
    const int t_begin = share * p.tiles_per_split;
    const int n_tiles = max(0, min(p.tiles_per_split, n_tiles_all - t_begin));

    // ---- global -> LDS.  A load instruction of a wavefront fills 8 rows: lane l -> row l >> 3, 16-byte
    // slot l & 7, which holds piece (l & 7) ^ ((row >> 1) & 7) of the row.  Wavefront w issues row
    // groups w, w + 8, .. of the tile: 24 groups of X rows, then 2 NSUB of W rows. ----
    const int my_groups = (kGroups - w + 7) / 8;
    const char* src[kMaxMine];
#pragma unroll
    for (int u = 0; u < kMaxMine; ++u) {
        const int grp = min(w + 8 * u, kGroups - 1), r = grp * 8 + (lane >> 3);  // row within the tile (X rows, then W rows)
        const int piece = (lane & 7) ^ ((r >> 1) & 7);
        const __bf16* row = r < kRows ? p.x + (int64_t)min(r, p.T - 1) * p.ldx
                                      : p.w + (int64_t)min(n0 + r - kRows, p.N - 1) * p.K;
        src[u] = reinterpret_cast<const char*>(row) + piece * 16 + (int64_t)t_begin * 128;
    }
    // (written as assembly: for the builtin form of these loads the compiler waits for all of them
    // before any LDS read, whichever buffer it is from.  M0 is the LDS address of the wavefront's
    // 1 KB; a write of M0 is kept one instruction away from its use.  Every wavefront issues
    // kMaxMine loads per tile, the ones beyond its share repeating its last group into the same
    // place, so that the counts the waits below assume are the same for all.)
    const unsigned ring_lds = (unsigned)(size_t)(lds_ptr)ring;
    auto issue = [&](int t) {  // tile t of this share (clamped: past the end the last tile is fetched again)
        const int64_t off = (int64_t)min(t, n_tiles - 1) * 128;
        const unsigned base = ring_lds + (unsigned)(t % RING) * kTileBytes;
#pragma unroll
        for (int u = 0; u < kMaxMine; ++u) {
            const int grp = min(w + 8 * u, w + 8 * (my_groups - 1));
            const unsigned dst = base + (unsigned)grp * 1024;
            const char* const from = src[min(u, my_groups - 1)] + off;
            // groups from 24 on (u >= 3 for every wavefront) are rows of W: each byte of W is needed
            // once by one workgroup, so it is asked for as non-temporal and leaves the L2 to X
            if (u >= kRows / 64)
                asm volatile("s_mov_b32 m0, %[dst]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[a], off nt"
                             :
                             : [dst] "s"(dst), [a] "v"(from)
                             : "memory");
            else
                asm volatile("s_mov_b32 m0, %[dst]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[a], off"
                             :
                             : [dst] "s"(dst), [a] "v"(from)
                             : "memory");
        }
    };

    f32x4 acc[kAccs];
#pragma unroll
    for (int a = 0; a < kAccs; ++a) acc[a] = f32x4{0.f, 0.f, 0.f, 0.f};

    // fragment reads: lane (i16, kq): piece kh*4 + kq of row r.  This wavefront: row sub-tiles mg,
    // mg+4, mg+8 x all feature sub-tiles, for half kh of every tile's 64 input features
    const int mg = w & 3, kh = w >> 2;
    int a_off[3], b_off[NSUB];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int r = (mg + 4 * i) * 16 + i16;
        a_off[i] = r * 128 + (((kh * 4 + kq) ^ ((r >> 1) & 7)) << 4);
    }
#pragma unroll
    for (int ni = 0; ni < NSUB; ++ni) {
        const int r = kRows + ni * 16 + i16;
        b_off[ni] = r * 128 + (((kh * 4 + kq) ^ ((r >> 1) & 7)) << 4);
    }

    if (n_tiles > 0) {
#pragma unroll
        for (int t = 0; t < RING - 1; ++t) issue(t);
        for (int t = 0; t < n_tiles; ++t) {
            VS_WAIT_VM((RING - 2) * kMaxMine);  // this wavefront's part of tile t has landed
            __syncthreads();                     // everybody's has, and tile t-1 has been read by all
            issue(t + RING - 1);                 // into the buffer of tile t-1
            const char* buf = ring + (t % RING) * kTileBytes;
            // all fragments of the tile are requested before the first matrix instruction (the
            // wavefronts of a workgroup move in step, tile by tile: left to the compiler, which asks
            // for a fragment just before its use, every one of them waits out an LDS round trip)
            bf16x8 af[3], bfr[NSUB];
#pragma unroll
            for (int i = 0; i < 3; ++i) af[i] = *reinterpret_cast<const bf16x8*>(buf + a_off[i]);
#pragma unroll
            for (int ni = 0; ni < NSUB; ++ni) bfr[ni] = *reinterpret_cast<const bf16x8*>(buf + b_off[ni]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ni = 0; ni < NSUB; ++ni)
#pragma unroll
                for (int i = 0; i < 3; ++i)
                    acc[i * NSUB + ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[ni], acc[i * NSUB + ni], 0, 0, 0);
        }
        VS_WAIT_VM(0);  // the spare loads behind the last tile must not land in LDS after the workgroup has gone
    }

    // ---- the two halves of the input features are added (the ring is free now) ----
    __syncthreads();
    float* const xch = reinterpret_cast<float*>(ring) + ((size_t)mg * kAccs * 64 + lane) * 4;
    if (kh == 1) {
#pragma unroll
        for (int a = 0; a < kAccs; ++a) *reinterpret_cast<f32x4*>(xch + a * 256) = acc[a];
    }
    __syncthreads();
    if (kh == 0) {
#pragma unroll
        for (int a = 0; a < kAccs; ++a) acc[a] += *reinterpret_cast<const f32x4*>(xch + a * 256);
    }
    // lane (i16, kq) of accumulator (i, ni): rows (mg + 4 i)*16 + 4 kq + 0..3, feature n0 + 16 ni + i16
    if (p.ws) {
        if (kh != 0 && !p.arrivals) return;
        if (kh == 0) {
            // this share's sums, in register order: [split][block][mg][accumulator][lane] x 4 floats
            f32x4* dst = reinterpret_cast<f32x4*>(p.ws) + ((((int64_t)share * p.n_blocks + blk) * 4 + mg) * kAccs) * 64 + lane;
            if (p.arrivals) {  // (written through while the kernel runs, not left for the write-back at its end)
#pragma unroll
                for (int a = 0; a < kAccs; ++a) __builtin_nontemporal_store(acc[a], &dst[a * 64]);
            } else {
#pragma unroll
                for (int a = 0; a < kAccs; ++a) dst[a * 64] = acc[a];
            }
        }
        if (!p.arrivals) return;
        // ---- The shares are added inside this launch, by the workgroups of the block together.
        // Every workgroup's stores above are complete in its XCD's L2 before it counts itself in
        // (all wavefronts wait for their stores, then the barrier, then the atomic, executed at that
        // L2: an increment that wraps, so the counter is zero again with the last arrival).  Those
        // that are not last look at the counter again with read-modify-writes (adding a zero the
        // compiler cannot see), never served by the compute unit's cache, a bounded number of times,
        // until it reads zero; then every share of the block is complete in this L2 (these lines are
        // read nowhere else in the launch, so the loads miss in the compute unit's cache).
        // Workgroup j of the block then finishes the 16-row sub-tiles j, j + ksplit, ..: its wavefronts
        // add the shares of their (sub-tile, feature sub-tile) pairs in index order, as
        // linear_reduce_kernel does, and the rows leave through LDS as below.  A workgroup that has looked max_looks
        // times in vain reports through the host word of the placement guard and returns. ----
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        __syncthreads();                     // (also: the exchange area has been read)
        unsigned* const box = reinterpret_cast<unsigned*>(ring);
        unsigned* const counter = p.arrivals + (int64_t)blk * (kCounterStrideBytes / 4);
        if (tid == 0) *box = __builtin_amdgcn_atomic_inc32(counter, (unsigned)(p.ksplit - 1), __ATOMIC_RELAXED, "workgroup");
        __syncthreads();
        if (*box + 1 != (unsigned)p.ksplit) {
            unsigned zero = 0;
            asm volatile("" : "+s"(zero));
            if (tid == 0) {
                unsigned ok = 0;
                for (int n = 0; n < p.max_looks && !ok; ++n) {
                    ok = __hip_atomic_fetch_add(counter, zero, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == 0u;
                    if (!ok) __builtin_amdgcn_s_sleep(2);
                }
                box[1] = ok;
                if (!ok) __hip_atomic_store(p.misplaced, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
            __syncthreads();
            if (!box[1]) return;
        }
        // this workgroup's sub-tiles: rs = share, share + ksplit, .. below 12 and below T rows
        const int n_rs = min(kRows / 16, (p.T + 15) >> 4);
        const int n_mine = share < n_rs ? (n_rs - share + p.ksplit - 1) / p.ksplit : 0;
        float* const mine = reinterpret_cast<float*>(ring + 1024);  // [n_mine * 16][kTileN + 4]
        const int64_t step = (int64_t)p.n_blocks * 4 * kAccs * 64;    // f32x4 between shares
        const int items = n_mine * NSUB;                              // (sub-tile, feature sub-tile) pairs
        // two items per wavefront and pass, all their shares requested before any is used: with the
        // plans in use one pass, so one round trip to L2
        for (int it0 = w; it0 < items; it0 += 16) {
            const f32x4* src[2];
            int k_of[2], ni_of[2];
#pragma unroll
            for (int b2 = 0; b2 < 2; ++b2) {
                const int it = min(it0 + 8 * b2, items - 1);
                k_of[b2] = it / NSUB;
                ni_of[b2] = it - k_of[b2] * NSUB;
                const int rs = share + k_of[b2] * p.ksplit, mg_r = rs & 3, i_r = rs >> 2;  // accumulator row i_r of row group mg_r
                src[b2] = reinterpret_cast<const f32x4*>(p.ws) + (((int64_t)blk * 4 + mg_r) * kAccs + i_r * NSUB + ni_of[b2]) * 64 + lane;
            }
            f32x4 sum[2] = {src[0][0], src[1][0]};
            for (int s0 = 1; s0 < p.ksplit; s0 += 8) {
                f32x4 v[2][8];
#pragma unroll
                for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[b2][u] = src[b2][(int64_t)min(s0 + u, p.ksplit - 1) * step];
#pragma unroll
                for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (s0 + u < p.ksplit) sum[b2] += v[b2][u];
            }
#pragma unroll
            for (int b2 = 0; b2 < 2; ++b2)
                if (it0 + 8 * b2 < items) put_acc<kTileN>(mine, sum[b2], 16 * k_of[b2], 16 * ni_of[b2], lane);
        }
        __syncthreads();
        const int ks = p.ksplit;
        write_tile<kTileN>(p, mine, 16 * n_mine, n0, tid, kThreads,
                           [share, ks](int r) { return (share + (r >> 4) * ks) * 16 + (r & 15); });
        return;
    }
    __syncthreads();  // the exchange area has been read: the tile of sums may overwrite it
    float* const tile = reinterpret_cast<float*>(ring);  // [192][kTileN + 4]
    if (kh == 0) {
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int ni = 0; ni < NSUB; ++ni) put_acc<kTileN>(tile, acc[i * NSUB + ni], (mg + 4 * i) * 16, 16 * ni, lane);
    }
    __syncthreads();
    write_tile<kTileN>(p, tile, kRows, n0, tid, kThreads, [](int r) { return r; });
}

// Adds the split-K shares in index order and finishes the sums.  Grid (blocks, 4 row groups): a
// workgroup owns the 48 rows of sub-tiles mg, mg + 4, mg + 8 of a block; a wavefront takes
// accumulators wave, wave + 4, .. (all shares of one are requested at once).
template <int NSUB>
__global__ __launch_bounds__(256) void linear_reduce_kernel(LinParams p, int n_blocks) {
    constexpr int kAccs = 3 * NSUB, kTileN = 16 * NSUB;
    __shared__ __attribute__((aligned(16))) float tile[48 * (kTileN + 4)];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int blk = blockIdx.x, mg = blockIdx.y;
    for (int a = wave; a < kAccs; a += 4) {
        const f32x4* src = reinterpret_cast<const f32x4*>(p.ws) + (((int64_t)blk * 4 + mg) * kAccs + a) * 64 + lane;
        const int64_t step = (int64_t)n_blocks * 4 * kAccs * 64;
        f32x4 sum = src[0];
        for (int s0 = 1; s0 < p.ksplit; s0 += 8) {
            f32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[(int64_t)min(s0 + u, p.ksplit - 1) * step];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + u < p.ksplit) sum += v[u];
        }
        const int i = a / NSUB, ni = a - i * NSUB;
        put_acc<kTileN>(tile, sum, 16 * i, 16 * ni, lane);
    }
    __syncthreads();
    // local row r = 16 i + j is row (mg + 4 i) * 16 + j of the output
    write_tile<kTileN>(p, tile, 48, blk * kTileN, threadIdx.x, 256, [mg](int r) { return (mg + 4 * (r >> 4)) * 16 + (r & 15); });
}

// RMS norm of T rows of d numbers: out = x * gamma / sqrt(mean(x^2) + eps), fp32 arithmetic, one
// rounding.  One workgroup per row, 8 numbers per thread and pass.
__global__ __launch_bounds__(256) void rmsnorm_kernel(const __bf16* __restrict__ x, const __bf16* __restrict__ gamma,
                                                      __bf16* __restrict__ out, int d, float eps) {
    __shared__ float part[4];
    const int64_t row = blockIdx.x;
    const bf16x8* xr = reinterpret_cast<const bf16x8*>(x + row * d);
    const bf16x8* gr = reinterpret_cast<const bf16x8*>(gamma);
    bf16x8* orow = reinterpret_cast<bf16x8*>(out + row * d);
    const int n8 = d / 8;
    float ss = 0.f;
    for (int i = threadIdx.x; i < n8; i += 256) {
        const bf16x8 v = xr[i];
#pragma unroll
        for (int j = 0; j < 8; ++j) ss += (float)v[j] * (float)v[j];
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = (part[0] + part[1]) + (part[2] + part[3]);
    const float r = 1.0f / sqrtf(tot / (float)d + eps);
    for (int i = threadIdx.x; i < n8; i += 256) {
        const bf16x8 v = xr[i], g = gr[i];
        bf16x8 y;
#pragma unroll
        for (int j = 0; j < 8; ++j) y[j] = (__bf16)((float)v[j] * r * (float)g[j]);
        orow[i] = y;
    }
}

struct LinPlan {
    int nsub, ksplit, n_blocks, tiles_per_split;
};

// The chip the plan is made for: workgroup ids are dealt to 8 XCDs of 32 compute units in turn.  A
// split plan keeps all shares of a block on one XCD at once (ceil(blocks / 8) blocks x ksplit shares
// <= 32 workgroups per XCD), so that the shares can be added inside the launch; the plan does not
// depend on whether they will be, so both ways of adding them see the same shares.
constexpr int kPlanXcds = 8, kPlanCusPerXcd = 32;

// Block width and split of K: estimated time = rounds through the chip x (tiles of a workgroup x
// bytes a tile brings into its compute unit) at ~60 GB/s per compute unit, plus, with split-K,
// the trip of the shares through memory and their addition.
LinPlan make_lin_plan(int T, int N, int K) {
    (void)T;
    const int ktiles = K / 64;
    LinPlan best{4, 1, (N + 63) / 64, ktiles};
    double best_cost = 1e30;
    for (int nsub : {4, 7, 8, 10}) {
        const int blocks = (N + 16 * nsub - 1) / (16 * nsub);
        for (int ks = 1; ks <= 16 && ks <= ktiles; ++ks) {
            if (ks > 1 && (blocks * ks > kPlanXcds * kPlanCusPerXcd ||
                           ((blocks + kPlanXcds - 1) / kPlanXcds) * ks > kPlanCusPerXcd))
                break;
            const int tps = (ktiles + ks - 1) / ks;
            const int rounds = (blocks * ks + 255) / 256;
            double cost = rounds * (2.0 + tps * (kRows + 16.0 * nsub) * 128.0 / 60e3);  // us
            if (ks > 1) cost += 3.0 + (double)ks * kRows * (double)(blocks * 16 * nsub) * 4.0 * 2.0 / 4e6;
            if (cost < best_cost) {
                best_cost = cost;
                best = LinPlan{nsub, ks, blocks, tps};
            }
        }
    }
    return best;
}

template <int NSUB, int RING>
hipError_t launch_lin(const LinParams& p, const LinPlan& pl, int dev, hipStream_t st) {
    static bool attr_set_on[16] = {};  // dynamic LDS above 64 KB has to be allowed once per kernel and device
    constexpr int kLds = RING * (kRows + 16 * NSUB) * 128;
    if (!attr_set_on[dev]) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(&linear_kernel<NSUB, RING>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (err != hipSuccess) return err;
        attr_set_on[dev] = true;
    }
    if (p.arrivals) {  // 1-D grid, the shares of a block on one XCD; they are added inside the launch
        linear_kernel<NSUB, RING><<<prefill_grid_ids(pl.n_blocks, pl.ksplit, p.xcd_shift), kThreads, kLds, st>>>(p);
        return hipGetLastError();
    }
    linear_kernel<NSUB, RING><<<dim3(pl.n_blocks, pl.ksplit), kThreads, kLds, st>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.ksplit == 1) return e;
    linear_reduce_kernel<NSUB><<<dim3(pl.n_blocks, 4), 256, 0, st>>>(p, pl.n_blocks);
    return hipGetLastError();
}

}  // namespace

size_t linear_workspace_bytes(int32_t n_rows, int32_t K, int32_t N) {
    const LinPlan pl = make_lin_plan(n_rows, N, K);
    if (pl.ksplit == 1) return 0;
    return (size_t)pl.ksplit * pl.n_blocks * 4 * (3 * pl.nsub) * 64 * sizeof(f32x4);
}

hipError_t launch_linear(const void* x, int32_t ldx, const void* w, int32_t n_rows, int32_t K, int32_t N, int32_t mode,
                         const void* residual, void* out, void* workspace, hipStream_t st, void* out1, void* out2,
                         int32_t seg0, int32_t seg1, void* arrival_counters, int32_t n_counters) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return hipErrorInvalidDevice;
    const LinPlan pl = make_lin_plan(n_rows, N, K);
    LinParams p;
    p.x = (const __bf16*)x;
    p.w = (const __bf16*)w;
    p.res = (const __bf16*)residual;
    p.out = (__bf16*)out;
    p.out1 = (__bf16*)out1;
    p.out2 = (__bf16*)out2;
    p.seg_end[0] = out1 ? seg0 : N;
    p.seg_end[1] = out1 ? seg1 : N;
    p.ws = pl.ksplit > 1 ? (float*)workspace : nullptr;
    p.T = n_rows;
    p.N = N;
    p.K = K;
    p.ldx = ldx;
    p.mode = mode;
    p.ksplit = pl.ksplit;
    p.tiles_per_split = pl.tiles_per_split;
    p.n_blocks = pl.n_blocks;
    p.arrivals = nullptr;
    p.misplaced = nullptr;
    p.xcc_of_residue = 0;
    p.xcd_shift = p.units_per_xcd = p.max_looks = 0;
    p.inv_ksplit = 1.0f / (float)pl.ksplit;
    XcdPlacement where;
    if (arrival_counters && pl.ksplit > 1 && pl.n_blocks <= n_counters && xcd_placement_of_device(dev, &where) &&
        (1 << where.xcd_shift) == kPlanXcds) {
        p.arrivals = (unsigned*)arrival_counters;
        p.misplaced = where.misplaced;
        p.xcc_of_residue = where.xcc_of_residue;
        p.xcd_shift = where.xcd_shift;
        p.units_per_xcd = prefill_units_per_xcd(pl.n_blocks, where.xcd_shift);
        p.max_looks = where.max_looks;
    }
    switch (pl.nsub) {
        case 4: return launch_lin<4, 4>(p, pl, dev, st);
        case 7: return launch_lin<7, 4>(p, pl, dev, st);
        case 8: return launch_lin<8, 3>(p, pl, dev, st);
        default: return launch_lin<10, 3>(p, pl, dev, st);
    }
}

hipError_t launch_rmsnorm(const void* x, const void* gamma, int32_t n_rows, int32_t d, float eps, void* out,
                          hipStream_t st) {
    rmsnorm_kernel<<<n_rows, 256, 0, st>>>((const __bf16*)x, (const __bf16*)gamma, (__bf16*)out, d, eps);
    return hipGetLastError();
}

}  // namespace vs
