// The frame's rows and their Q/K/V projections for gfx950 (Section 3.1: Q = X W_Q, K = X W_K,
// V = X W_V; Section 3.3: the carrier's embedding is the mean of the frame's token embeddings;
// Section 3.2: it is the frame's last row).  One launch; X = [E ; mean(E)] is never written out,
// the outputs land in the layouts the frame prefill reads.
//
// N + 1 <= 192 rows meet n_out = (Hq + 2 Hkv) D weight rows of d numbers each; the weights (33 MB
// at the 7B shape) are what the launch has to pull in from HBM, once.  A workgroup owns 32 output
// features and all of the d input features, so nothing has to be added up across workgroups; what
// bounds it is the 64 bytes per clock a compute unit takes in, because every workgroup reads all of
// E (from L2).  64 input features at a time, a tile of 192 rows of E and 32 rows of W (28 KB) goes
// from global memory straight into LDS, whole 128-byte lines per 8 lanes, into a ring of five
// buffers: four tiles are on their way while one is multiplied, with one barrier per tile.  The
// 16-byte pieces of a row are stored permuted (piece ^ ((row >> 1) & 7)) so that the fragment
// reads of v_mfma_f32_16x16x32_bf16 (16 rows x one piece) hit all banks.  Of the 8 wavefronts, w
// multiplies the 16-row sub-tiles w&3, +4, +8 with both 16-feature sub-tiles for half w>>2 of each
// tile's input features: two wavefronts per SIMD, each part of a tile read from LDS by one of
// them only; the halves are added through LDS at the end.
//
// The carrier's row is not multiplied at all: the projection is linear, so its Q/K/V are the means
// over the token rows of the fp32 sums the workgroup holds anyway (the mean enters unrounded).
// The carrier embedding itself, if asked for, is computed on the side: each workgroup takes a
// share of the d columns and adds the rows in the order of mean_pool_kernel (16 row groups, then
// the groups in order, one division, one rounding), so it is the same bits as vs_carrier_mean_pool.
#include <hip/hip_runtime.h>

#include "vs_internal.h"

namespace vs {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const void* global_cptr;
typedef __attribute__((address_space(3))) void* lds_ptr;

constexpr int kTileN = 32;       // output features per workgroup (2 sub-tiles of 16)
// rows of E a tile holds: ROWS = 176 (up to 175 tokens) or 192; rows from N on repeat row N-1
constexpr int kThreads = 512;
// RING tile buffers of (ROWS + 32) * 128 bytes: 6 x 26 KB or 5 x 28 KB
constexpr int kAccs = 3 * 2;

struct QkvParams {
    const __bf16* e;   // [N][d]
    const __bf16* w;   // [n_out][d]
    __bf16* q;         // [N + 1][nq]
    __bf16* k;         // [N + 1][nk]
    __bf16* v;         // [N + 1][nk]
    __bf16* c_out;     // [d] or null
    int N, d, n_out, nq, nk;
};

__device__ __forceinline__ __bf16* dest(const QkvParams& p, int m, int n) {
    if (n < p.nq) return p.q + (int64_t)m * p.nq + n;
    n -= p.nq;
    if (n < p.nk) return p.k + (int64_t)m * p.nk + n;
    return p.v + (int64_t)m * p.nk + (n - p.nk);
}

// s_waitcnt vmcnt(n) only (gfx9 encoding: vmcnt in bits 3:0 and 15:14; expcnt, lgkmcnt left at "no wait")
#define VS_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0F70)

template <int kRows, int kRing>
__global__ __launch_bounds__(kThreads) void frame_qkv_kernel(QkvParams p) {
    constexpr int kTileBytes = (kRows + kTileN) * 128;
    constexpr int kGroups = (kRows + kTileN) / 8;  // load instructions (8 rows each) per tile; a wavefront issues 4 or 3
    extern __shared__ __attribute__((aligned(1024))) char ring[];  // kRing tiles: 192 rows of E, then 32 rows of W
    __shared__ float colsum[4][kTileN];
    __shared__ float poolsum[16][32];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, kq = lane >> 4;
    const int N = p.N, d = p.d;
    const int n0 = blockIdx.x * kTileN;
    const int n_tiles = d / 64;

    // ---- global -> LDS.  A load instruction of a wavefront fills 8 rows: lane l -> row l >> 3, 16-byte
    // slot l & 7, which holds piece (l & 7) ^ ((row >> 1) & 7) of the row.  Wavefront w issues row
    // groups w, w + 8, .. of the tile: 24 groups of E rows, then 4 of W rows. ----
    const int my_groups = w + 24 < kGroups ? 4 : 3;
    const char* src[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int grp = min(w + 8 * u, kGroups - 1), r = grp * 8 + (lane >> 3);  // row within the tile (E rows, then W rows)
        const int piece = (lane & 7) ^ ((r >> 1) & 7);
        const __bf16* row = r < kRows ? p.e + (int64_t)min(r, N - 1) * d
                                      : p.w + (int64_t)min(n0 + r - kRows, p.n_out - 1) * d;
        src[u] = reinterpret_cast<const char*>(row) + piece * 16;
    }
    // (written as assembly: for the builtin form of these loads the compiler waits for all of them
    // before any LDS read, whichever buffer it is from.  M0 is the LDS address of the wavefront's
    // 1 KB; a write of M0 is kept one instruction away from its use.)
    const unsigned ring_lds = (unsigned)(size_t)(lds_ptr)ring;
    auto issue = [&](int t) {  // tile t (clamped: past the end the last tile is fetched again, so that
                               // the number of loads in flight stays what the waits below assume)
        const int64_t off = (int64_t)min(t, n_tiles - 1) * 128;
        const unsigned dst = ring_lds + (unsigned)(t % kRing) * kTileBytes + (unsigned)w * 1024;
        // the groups of W rows (those from kRows / 8 on) are asked for as non-temporal: every byte of W
        // is needed once, by one workgroup
        asm volatile(
            "s_mov_b32 m0, %[dst]\n\ts_nop 0\n\t"
            "global_load_lds_dwordx4 %[a0], off\n\ts_add_u32 m0, m0, 0x2000\n\ts_nop 0\n\t"
            "global_load_lds_dwordx4 %[a1], off"
            :
            : [dst] "s"(dst), [a0] "v"(src[0] + off), [a1] "v"(src[1] + off)
            : "memory");
        if (w + 16 >= kRows / 8)
            asm volatile("s_mov_b32 m0, %[dst]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[a2], off nt"
                         :
                         : [dst] "s"(dst + 2 * 0x2000), [a2] "v"(src[2] + off)
                         : "memory");
        else
            asm volatile("s_mov_b32 m0, %[dst]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[a2], off"
                         :
                         : [dst] "s"(dst + 2 * 0x2000), [a2] "v"(src[2] + off)
                         : "memory");
        if (my_groups == 4)
            asm volatile("s_mov_b32 m0, %[dst]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[a3], off nt"
                         :
                         : [dst] "s"(dst + 3 * 0x2000), [a3] "v"(src[3] + off)
                         : "memory");
    };

    f32x4 acc[kAccs];
#pragma unroll
    for (int a = 0; a < kAccs; ++a) acc[a] = f32x4{0.f, 0.f, 0.f, 0.f};

    // fragment reads: lane (i16, kq), step st of the tile: piece st*4 + kq of row r
    // this wavefront: row sub-tiles mg, mg+4, mg+8 x both feature sub-tiles, for half kh of every tile's
    // 64 input features (so that the wavefronts read different parts of a tile, not the same twice)
    const int mg = w & 3, kh = w >> 2;
    int a_row[3], b_row[2];
#pragma unroll
    for (int i = 0; i < 3; ++i) a_row[i] = (mg + 4 * i) * 16 + i16;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) b_row[ni] = kRows + ni * 16 + i16;

#pragma unroll
    for (int t = 0; t < kRing - 1; ++t) issue(t);
    for (int t = 0; t < n_tiles; ++t) {
        if (my_groups == 4) VS_WAIT_VM((kRing - 2) * 4);  // this wavefront's part of tile t has landed
        else VS_WAIT_VM((kRing - 2) * 3);
        __syncthreads();                           // everybody's has, and tile t-1 has been read by all
        issue(t + kRing - 1);                      // into the buffer of tile t-1
        const char* buf = ring + (t % kRing) * kTileBytes;
        {
            bf16x8 af[3], bfr[2];
#pragma unroll
            for (int i = 0; i < 3; ++i)
                af[i] = *reinterpret_cast<const bf16x8*>(buf + a_row[i] * 128 + (((kh * 4 + kq) ^ ((a_row[i] >> 1) & 7)) << 4));
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                bfr[ni] = *reinterpret_cast<const bf16x8*>(buf + b_row[ni] * 128 + (((kh * 4 + kq) ^ ((b_row[ni] >> 1) & 7)) << 4));
#pragma unroll
            for (int i = 0; i < 3; ++i)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    acc[i * 2 + ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[ni], acc[i * 2 + ni], 0, 0, 0);
        }
    }
    VS_WAIT_VM(0);  // the spare loads behind the last tile must not land in LDS after the workgroup has gone

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
        // lane (i16, kq) of accumulator (i, ni): rows (mg + 4 i)*16 + 4 kq + 0..3, feature n0 + 16 ni + i16.
        // Token rows go out; their column sums make the carrier's row.
        float csum[2] = {0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                const int n = n0 + 16 * ni + i16, m0 = (mg + 4 * i) * 16 + 4 * kq;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (m0 + e < N) {
                        csum[ni] += acc[i * 2 + ni][e];
                        if (n < p.n_out) *dest(p, m0 + e, n) = (__bf16)acc[i * 2 + ni][e];
                    }
                }
            }
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            csum[ni] += __shfl_xor(csum[ni], 16);
            csum[ni] += __shfl_xor(csum[ni], 32);
            if (kq == 0) colsum[mg][16 * ni + i16] = csum[ni];
        }
    }
    __syncthreads();
    if (tid < kTileN && n0 + tid < p.n_out)
        *dest(p, N, n0 + tid) =
            (__bf16)((((colsum[0][tid] + colsum[1][tid]) + colsum[2][tid]) + colsum[3][tid]) / (float)N);

    // ---- the carrier embedding, a share of the columns per workgroup ----
    if (p.c_out) {
        const int c_begin = (int)((int64_t)d * blockIdx.x / gridDim.x), c_end = (int)((int64_t)d * (blockIdx.x + 1) / gridDim.x);
        for (int c0 = c_begin; c0 < c_end; c0 += 32) {  // 32 columns x 16 row groups at a time
            const int col = c0 + (tid & 31), rg = tid >> 5;
            float sum = 0.f;
            if (col < c_end)
                for (int r = rg; r < N; r += 16) sum += (float)p.e[(int64_t)r * d + col];
            poolsum[rg][tid & 31] = sum;
            __syncthreads();
            if (tid < 32 && col < c_end) {
                float tot = poolsum[0][tid];
#pragma unroll
                for (int g = 1; g < 16; ++g) tot += poolsum[g][tid];
                p.c_out[col] = (__bf16)(tot / (float)N);
            }
            __syncthreads();
        }
    }
}

}  // namespace

template <int ROWS, int RING>
hipError_t launch_qkv_variant(const QkvParams& p, int dev, hipStream_t st) {
    static bool attr_set_on[16] = {};  // dynamic LDS above 64 KB has to be allowed once per kernel and device
    constexpr int kLds = RING * (ROWS + kTileN) * 128;
    if (!attr_set_on[dev]) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(&frame_qkv_kernel<ROWS, RING>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (err != hipSuccess) return err;
        attr_set_on[dev] = true;
    }
    frame_qkv_kernel<ROWS, RING><<<(p.n_out + kTileN - 1) / kTileN, kThreads, kLds, st>>>(p);
    return hipGetLastError();
}

hipError_t launch_frame_qkv(const vs_shape& s, const void* e, int32_t n_visual, int32_t d, const void* w,
                            void* q, void* k, void* v, void* c_out, hipStream_t st) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return hipErrorInvalidDevice;
    QkvParams p;
    p.e = (const __bf16*)e;
    p.w = (const __bf16*)w;
    p.q = (__bf16*)q;
    p.k = (__bf16*)k;
    p.v = (__bf16*)v;
    p.c_out = (__bf16*)c_out;
    p.N = n_visual;
    p.d = d;
    p.nq = s.n_q_heads * s.head_dim;
    p.nk = s.n_kv_heads * s.head_dim;
    p.n_out = p.nq + 2 * p.nk;
    // fewer rows per tile leave room for one more tile in flight
    return n_visual <= 175 ? launch_qkv_variant<176, 6>(p, dev, st) : launch_qkv_variant<192, 5>(p, dev, st);
}

}  // namespace vs
