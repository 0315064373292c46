// The frame's rows and their Q/K/V projections for gfx950 (Section 3.1: Q = X W_Q, K = X W_K,
// V = X W_V; Section 3.3: the carrier's embedding is the mean of the frame's token embeddings;
// Section 3.2: it is the frame's last row).  One launch: X = [E ; mean(E)] is never written out,
// the outputs land in the layouts the frame prefill reads.
//
// M = N + 1 <= 192 rows meet n_out = (Hq + 2 Hkv) D weight rows of d numbers each: the weights
// (33 MB at the 7B shape) are what the launch has to pull in, once.  A workgroup owns 144 output
// features (9 sub-tiles of 16) and one slice of the d input features; 4 wavefronts share the rows
// (16-row sub-tiles w, w+4, w+8).  64 input features at a time, X and W tiles go through LDS
// (rows padded to 144 B: the 16 B fragment reads of 16 consecutive rows then fall into different
// banks), the next tiles travel in registers meanwhile.  The carrier row of an X tile is summed
// from the tile in LDS, in the order of mean_pool_kernel (16 row groups, then the groups in
// order, one division, one rounding to bf16), so it is the same bits as vs_carrier_mean_pool.
//
// The slices of a unit (= 144 output features) run on one XCD, whose L2 they share: every
// workgroup leaves its fp32 partial sums there in register order, counts itself in, and once
// all slices of the unit have arrived the workgroups of the unit add up one share each, slices in
// index order, and write bf16.  Waiting is bounded; see the comment at the protocol below.
#include <hip/hip_runtime.h>

#include "vs_internal.h"

namespace vs {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kSub = 9;             // 16-feature sub-tiles per workgroup
constexpr int kTileN = 16 * kSub;   // 144 output features
constexpr int kStepK = 64;          // input features per LDS tile
constexpr int kPitch = 72;          // elements per LDS row (144 B)
constexpr int kMaxM = 192;          // rows (12 sub-tiles, 3 per wavefront)
constexpr int kRowsPerWave = 3;
constexpr int kAcc = kRowsPerWave * kSub;  // accumulators of a wavefront
constexpr int kXLoads = kMaxM * 8 / 256;   // 16-byte pieces of an X tile per thread (6)
constexpr int kWLoads = (kTileN * 8 + 255) / 256;  // of a W tile (5, the last half used)
constexpr int kQkvPolls = 256;

struct QkvParams {
    const __bf16* e;   // [N][d]
    const __bf16* w;   // [n_out][d]
    __bf16* q;         // [M][nq]
    __bf16* k;         // [M][nk]
    __bf16* v;         // [M][nk]
    __bf16* c_out;     // [d] or null
    float* part;       // [nsplit][units][4 waves][kAcc][64 lanes] x 4 floats
    unsigned* arrivals;  // [units], zero between launches
    int N, M, d, n_out, nq, nk;
    int units, nsplit, n_steps;  // n_steps = d / 64
    int msub;                    // 16-row sub-tiles that hold rows < M
    int xcd_shift, units_per_xcd, share_polls;
};

__device__ __forceinline__ __bf16* dest(const QkvParams& p, int m, int n) {
    if (n < p.nq) return p.q + (int64_t)m * p.nq + n;
    n -= p.nq;
    if (n < p.nk) return p.k + (int64_t)m * p.nk + n;
    return p.v + (int64_t)m * p.nk + (n - p.nk);
}

__global__ __launch_bounds__(256) void frame_qkv_kernel(QkvParams p) {
    __shared__ __attribute__((aligned(16))) __bf16 xs[kMaxM * kPitch];
    __shared__ __attribute__((aligned(16))) __bf16 wsm[kTileN * kPitch];
    __shared__ float colsum[16][kStepK];
    __shared__ unsigned box[2];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, kq = lane >> 4;
    int unit, split;
    if (p.xcd_shift >= 0) {
        // ids are dealt to the XCDs in turn; XCD x holds units x*units_per_xcd .., each with
        // nsplit consecutive slots
        const int x = blockIdx.x & ((1 << p.xcd_shift) - 1), slot = blockIdx.x >> p.xcd_shift;
        const int j = slot / p.nsplit;
        unit = x * p.units_per_xcd + j;
        split = slot - j * p.nsplit;
        if (j >= p.units_per_xcd || unit >= p.units) return;  // spare ids
    } else {
        unit = blockIdx.x;
        split = 0;
    }
    const int n0 = unit * kTileN;
    const int s0 = (int)((int64_t)p.n_steps * split / p.nsplit), s1 = (int)((int64_t)p.n_steps * (split + 1) / p.nsplit);
    const int N = p.N, d = p.d;

    // rows of the X tile beyond the carrier are never written again: zero once
    for (int i = tid; i < (kMaxM - N) * kPitch; i += 256) xs[N * kPitch + i] = (__bf16)0.f;

    uint4 xr[kXLoads], wr[kWLoads];
    auto fetch = [&](int s) {
        const int k0 = s * kStepK;
#pragma unroll
        for (int i = 0; i < kXLoads; ++i) {
            const int idx = tid + 256 * i, r = idx >> 3, pc = idx & 7;
            xr[i] = make_uint4(0, 0, 0, 0);
            if (r < N) xr[i] = *reinterpret_cast<const uint4*>(p.e + (int64_t)r * d + k0 + pc * 8);
        }
#pragma unroll
        for (int i = 0; i < kWLoads; ++i) {
            const int idx = tid + 256 * i, r = idx >> 3, pc = idx & 7;
            wr[i] = make_uint4(0, 0, 0, 0);
            if (r < kTileN && n0 + r < p.n_out)
                wr[i] = *reinterpret_cast<const uint4*>(p.w + (int64_t)(n0 + r) * d + k0 + pc * 8);
        }
    };
    auto park = [&]() {
#pragma unroll
        for (int i = 0; i < kXLoads; ++i) {
            const int idx = tid + 256 * i, r = idx >> 3, pc = idx & 7;
            if (r < N) *reinterpret_cast<uint4*>(&xs[r * kPitch + pc * 8]) = xr[i];
        }
#pragma unroll
        for (int i = 0; i < kWLoads; ++i) {
            const int idx = tid + 256 * i, r = idx >> 3, pc = idx & 7;
            if (r < kTileN) *reinterpret_cast<uint4*>(&wsm[r * kPitch + pc * 8]) = wr[i];
        }
    };

    f32x4 acc[kAcc];
#pragma unroll
    for (int a = 0; a < kAcc; ++a) acc[a] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (s0 < s1) fetch(s0);
    for (int s = s0; s < s1; ++s) {
        park();
        __syncthreads();
        // ---- the carrier's piece of this tile: column means over the N token rows ----
        {
            const int col = tid & 63, g4 = tid >> 6;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int rg = g4 * 4 + u;
                float sum = 0.f;
                for (int r = rg; r < N; r += 16) sum += (float)xs[r * kPitch + col];
                colsum[rg][col] = sum;
            }
        }
        __syncthreads();
        if (tid < kStepK) {
            float tot = colsum[0][tid];
#pragma unroll
            for (int g = 1; g < 16; ++g) tot += colsum[g][tid];
            const __bf16 c = (__bf16)(tot / (float)N);
            xs[N * kPitch + tid] = c;
            if (p.c_out && unit == 0) p.c_out[s * kStepK + tid] = c;
        }
        __syncthreads();
        if (s + 1 < s1) fetch(s + 1);  // in flight while this tile is multiplied
        // ---- 2 steps of 32 input features ----
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            bf16x8 af[kRowsPerWave];
#pragma unroll
            for (int i = 0; i < kRowsPerWave; ++i)
                af[i] = *reinterpret_cast<const bf16x8*>(&xs[((w + 4 * i) * 16 + i16) * kPitch + st * 32 + kq * 8]);
#pragma unroll
            for (int ni = 0; ni < kSub; ++ni) {
                const bf16x8 bfr = *reinterpret_cast<const bf16x8*>(&wsm[(ni * 16 + i16) * kPitch + st * 32 + kq * 8]);
#pragma unroll
                for (int i = 0; i < kRowsPerWave; ++i)
                    acc[i * kSub + ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr, acc[i * kSub + ni], 0, 0, 0);
            }
        }
        __syncthreads();  // the tiles are free again
    }

    // lane (i16, kq) of accumulator (i, ni): rows (w + 4 i) * 16 + 4 kq + 0..3, feature n0 + 16 ni + i16
    auto write_out = [&](int wv, int a, const f32x4& val) {
        const int i = a / kSub, ni = a - i * kSub;
        const int n = n0 + 16 * ni + i16, m0 = (wv + 4 * i) * 16 + 4 * kq;
        if (n >= p.n_out) return;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (m0 + e < p.M) *dest(p, m0 + e, n) = (__bf16)val[e];
    };

    if (p.nsplit == 1) {
#pragma unroll
        for (int a = 0; a < kAcc; ++a)
            if (w + 4 * (a / kSub) < p.msub) write_out(w, a, acc[a]);
        return;
    }

    // ---- partial sums to L2, in register order (a store instruction writes 1 KB) ----
    const int64_t item_floats = 64 * 4;
    float* const mine = p.part + ((((int64_t)split * p.units + unit) * 4 + w) * kAcc) * item_floats + lane * 4;
#pragma unroll
    for (int a = 0; a < kAcc; ++a)
        if (w + 4 * (a / kSub) < p.msub) *reinterpret_cast<f32x4*>(mine + a * item_floats) = acc[a];

    // ---- the slices of the unit meet.  The unit's word: arrivals in bits 0..7, one bit per slice
    // that stopped waiting in 8..15, the number of workgroups that saw the full count while
    // waiting in 16..23, a count of polls in 24..31 (a poll has to be a read-modify-write, which
    // L2 executes: a load could be answered by the compute unit's own cache for ever).  A
    // workgroup that is not the last polls a bounded number of times; seeing the full count it
    // reports that and adds up its share; out of polls it sets its bit and leaves, unless the word
    // it gets back shows that the last one has come meanwhile.  The last to arrive learns from
    // the word who has left, does those shares besides its own, waits until the others still there
    // have reported (each does after a bounded number of its own steps) and zeroes the word. ----
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's partial sums are in L2
    __syncthreads();
    enum { kLeave = 0, kHelp = 1, kLast = 2 };
    constexpr unsigned kPollTick = 1u << 24;
    unsigned* const word = p.arrivals + unit;
    const unsigned ns = (unsigned)p.nsplit;
    if (tid == 0) {
        const unsigned before = __hip_atomic_fetch_add(word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        unsigned role = kLast, left = (before >> 8) & 0xffu;
        if ((before & 0xffu) + 1u != ns) {
            unsigned state = before;
            for (int polls = p.share_polls; polls > 0 && (state & 0xffu) != ns; --polls) {
                __builtin_amdgcn_s_sleep(4);
                state = __hip_atomic_fetch_add(word, kPollTick, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            if ((state & 0xffu) != ns)
                state = __hip_atomic_fetch_or(word, 0x100u << split, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            role = kLeave;
            if ((state & 0xffu) == ns) {
                role = kHelp;
                __hip_atomic_fetch_add(word, 0x10000u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            left = 0;
        }
        box[0] = role;
        box[1] = left;
    }
    __syncthreads();
    const unsigned role = box[0], left = box[1];
    if (role == kLeave) return;

    // share of slice j: items (wavefront wv, accumulator a), item = wv * kAcc + a, taken in turn
    // by the 4 * nsplit wavefronts of the unit; the slices are added in index order
    const int n_items = 4 * kAcc, unit_waves = 4 * p.nsplit;
    const float* const unit_part = p.part + ((int64_t)unit * 4 * kAcc) * item_floats + lane * 4;
    const int64_t split_stride = (int64_t)p.units * 4 * kAcc * item_floats;
    for (int j = 0; j < p.nsplit; ++j) {
        if (j != split && !(role == kLast && ((left >> j) & 1u))) continue;
        for (int item = j * 4 + w; item < n_items; item += unit_waves) {
            const int wv = item / kAcc, a = item - wv * kAcc;
            if (wv + 4 * (a / kSub) >= p.msub) continue;
            f32x4 part[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (u < p.nsplit) part[u] = *reinterpret_cast<const f32x4*>(unit_part + u * split_stride + item * item_floats);
            f32x4 sum = part[0];
#pragma unroll
            for (int u = 1; u < 8; ++u)
                if (u < p.nsplit) sum += part[u];
            write_out(wv, a, sum);
        }
    }
    if (role == kLast && tid == 0) {
        const unsigned expected = ns - 1u - (unsigned)__builtin_popcount(left);
        unsigned state;
        int guard = 1 << 16;
        do {
            state = __hip_atomic_fetch_add(word, kPollTick, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        } while (((state >> 16) & 0xffu) != expected && --guard > 0);
        __hip_atomic_store(word, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
}

struct QkvPlan {
    int units, nsplit, xcd_shift, units_per_xcd, share_polls, grid;
};

QkvPlan make_qkv_plan(int n_out, int d) {
    QkvPlan pl;
    pl.units = (n_out + kTileN - 1) / kTileN;
    pl.nsplit = 1;
    pl.xcd_shift = -1;
    pl.units_per_xcd = 0;
    pl.share_polls = 0;
    pl.grid = pl.units;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return pl;
    const int shift = xcd_shift_of_device(dev);
    if (shift < 0 || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return pl;
    const int n_xcd = 1 << shift, per_xcd = cus / n_xcd;
    const int upx = (pl.units + n_xcd - 1) / n_xcd;
    // as many slices as keep all workgroups of an XCD on its compute units at the same time
    int ns = upx > 0 ? per_xcd / upx : 1;
    if (ns > 8) ns = 8;
    if (ns > d / kStepK) ns = d / kStepK;
    if (g_tune_qkv_splits) ns = g_tune_qkv_splits < d / kStepK ? g_tune_qkv_splits : d / kStepK;
    if (ns < 2) return pl;
    pl.nsplit = ns;
    pl.xcd_shift = shift;
    pl.units_per_xcd = upx;
    pl.share_polls = (upx * ns <= per_xcd && !g_tune_qkv_nowait) ? kQkvPolls : 0;
    pl.grid = (upx * ns) << shift;
    return pl;
}

}  // namespace

size_t frame_qkv_workspace_bytes(int n_out, int /*d*/) {
    const int units = (n_out + kTileN - 1) / kTileN;
    return (size_t)8 * units * 4 * kAcc * 64 * 4 * sizeof(float);
}

hipError_t launch_frame_qkv(const vs_shape& s, const void* e, int32_t n_visual, int32_t d, const void* w,
                            void* q, void* k, void* v, void* c_out, void* arrivals, void* workspace,
                            hipStream_t st) {
    QkvParams p;
    p.e = (const __bf16*)e;
    p.w = (const __bf16*)w;
    p.q = (__bf16*)q;
    p.k = (__bf16*)k;
    p.v = (__bf16*)v;
    p.c_out = (__bf16*)c_out;
    p.part = (float*)workspace;
    p.arrivals = (unsigned*)arrivals;
    p.N = n_visual;
    p.M = n_visual + 1;
    p.d = d;
    p.nq = s.n_q_heads * s.head_dim;
    p.nk = s.n_kv_heads * s.head_dim;
    p.n_out = p.nq + 2 * p.nk;
    p.n_steps = d / kStepK;
    p.msub = (p.M + 15) / 16;
    const QkvPlan pl = make_qkv_plan(p.n_out, d);
    p.units = pl.units;
    p.nsplit = pl.nsplit;
    p.xcd_shift = pl.xcd_shift;
    p.units_per_xcd = pl.units_per_xcd;
    p.share_polls = pl.share_polls;
    frame_qkv_kernel<<<pl.grid, 256, 0, st>>>(p);
    return hipGetLastError();
}

}  // namespace vs
