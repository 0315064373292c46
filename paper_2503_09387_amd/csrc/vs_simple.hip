// fp32-arithmetic attention path (used for VS_F32 storage), row copies and the mean pool.
//
// The attention kernel here is the small, definition-shaped one: a workgroup per
// (query token, query head), scores for 256 keys at a time, running-max softmax
// (Eq. 1 of the VideoScan paper, Section 3.1) and a value accumulation with one
// thread per output coordinate.  It exists for fp32 storage, where the shapes are
// tiny and accuracy (1e-5) is what matters; the bf16 shapes go through the MFMA
// kernels.
#include "vs_internal.h"

namespace vs {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

template <bool kMax>
__device__ __forceinline__ float block_reduce(float x, float* red) {
    x = kMax ? wave_max(x) : wave_sum(x);
    const int w = threadIdx.x >> 6;
    __syncthreads();  // red may still be read from the previous reduction
    if ((threadIdx.x & 63) == 0) red[w] = x;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < kThreads / 64; ++i) r = kMax ? fmaxf(r, red[i]) : r + red[i];
    return r;
}

// Grid: (query tokens, query heads, streams).  Stream z reads its cache at
// kc + z*cache_stride (elements), valid rows lens.v[z] (or `len` when lens_used == 0).
// Frame rows (kf != nullptr) follow the cache rows; query token i sees frame rows 0..i.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void attn_simple_kernel(
    const T* __restrict__ kc, const T* __restrict__ vc, int64_t cache_stride, int32_t len,
    LenTable lens, int lens_used, const T* __restrict__ q, const T* __restrict__ kf,
    const T* __restrict__ vf, T* __restrict__ out, int Hq, int Hkv, float scale) {
    const int i = blockIdx.x, h = blockIdx.y, z = blockIdx.z;
    const int g = h / (Hq / Hkv);
    const int tid = threadIdx.x;
    const int L = lens_used ? lens.v[z] : len;
    const int n = L + (kf ? i + 1 : 0);
    const T* kcz = kc + (int64_t)z * cache_stride;
    const T* vcz = vc + (int64_t)z * cache_stride;
    const int64_t qrow = ((int64_t)z * gridDim.x + i) * Hq + h;

    __shared__ float s_q[D];
    __shared__ float s_p[kThreads];
    __shared__ float s_red[kThreads / 64];
    __shared__ float s_acc[kThreads];

    if (tid < D) s_q[tid] = to_f32(q[qrow * D + tid]);
    __syncthreads();

    constexpr int KG = kThreads / D;  // key groups in the value accumulation
    const int d = tid % D, kg = tid / D;
    float m = -INFINITY, l = 0.f, acc = 0.f;

    for (int base = 0; base < n; base += kThreads) {
        const int j = base + tid;
        float zj = -INFINITY;
        if (j < n) {
            const T* krow = (j < L) ? kcz + ((int64_t)j * Hkv + g) * D
                                    : kf + ((int64_t)(j - L) * Hkv + g) * D;
            float dot = 0.f;
#pragma unroll 8
            for (int e = 0; e < D; ++e) dot = fmaf(s_q[e], to_f32(krow[e]), dot);
            zj = dot * scale;
        }
        const float cmax = block_reduce<true>(zj, s_red);  // finite: key `base` is visible
        const float m_new = fmaxf(m, cmax);
        const float alpha = expf(m - m_new);                // 0 on the first chunk
        const float p = (j < n) ? expf(zj - m_new) : 0.f;
        const float csum = block_reduce<false>(p, s_red);
        l = l * alpha + csum;
        acc *= alpha;
        m = m_new;
        s_p[tid] = p;
        __syncthreads();
        const int cnt = min(kThreads, n - base);
        for (int jj = kg; jj < cnt; jj += KG) {
            const int jr = base + jj;
            const T* vrow = (jr < L) ? vcz + ((int64_t)jr * Hkv + g) * D
                                     : vf + ((int64_t)(jr - L) * Hkv + g) * D;
            acc = fmaf(s_p[jj], to_f32(vrow[d]), acc);
        }
        __syncthreads();
    }
    s_acc[tid] = acc;
    __syncthreads();
    if (tid < D) {
        float t = 0.f;
#pragma unroll
        for (int k = 0; k < KG; ++k) t += s_acc[k * D + tid];
        out[qrow * D + tid] = from_f32<T>(t / l);
    }
}

template <typename T>
hipError_t launch_attn_simple(const vs_shape& s, const void* kc, const void* vc, int64_t cache_stride,
                              int32_t len, const LenTable& lens, int lens_used, int n_streams,
                              const void* q, const void* kf, const void* vf, int32_t n_tokens,
                              void* out, hipStream_t st) {
    dim3 grid(n_tokens, s.n_q_heads, n_streams), block(kThreads);
#define VS_GO(DD)                                                                              \
    attn_simple_kernel<T, DD><<<grid, block, 0, st>>>(                                           \
        (const T*)kc, (const T*)vc, cache_stride, len, lens, lens_used, (const T*)q,             \
        (const T*)kf, (const T*)vf, (T*)out, s.n_q_heads, s.n_kv_heads, s.softmax_scale)
    if (s.head_dim == 64) VS_GO(64);
    else VS_GO(128);
#undef VS_GO
    return hipGetLastError();
}

// ---- row copies ------------------------------------------------------------
// Run i's chosen row (`row_bytes`, a multiple of 16) goes into row len_i of cache i, for K and
// for V.  The work is cut into items of 1 KB = one load of 16 bytes per lane of a wavefront:
// item t = ((which * n_caches + cache) * pieces + piece): all of K, then all of V.  A fixed grid of wavefronts walks the items
// kCopyDepth at a time, wavefront w taking batches w, w + n_waves, ...: the wavefronts that run
// at the same time work on neighbouring rows (one moving window over the slabs, which is what
// the address translation caches want), and a wavefront has the loads of a whole batch, plus
// the lengths its destinations depend on, requested before its first store.  Every byte is
// touched once: loads and stores are marked non-temporal (measured: 10 % faster).
constexpr int kCopyThreads = 256, kCopyDepth = 8, kCopyMaxWorkgroups = 2048;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
// kByValue: the lengths of at most 64 caches travel in the kernel arguments (lens); otherwise they
// are read from lens_device.
template <bool kOnePiece, bool kByValue>
__global__ __launch_bounds__(kCopyThreads) void append_rows_kernel(
    char* __restrict__ k_slab, char* __restrict__ v_slab, int64_t cache_stride_bytes, LenTable lens,
    const int32_t* __restrict__ lens_device, const char* __restrict__ k_src,
    const char* __restrict__ v_src, int64_t src_stride_bytes, int64_t src_row_offset_bytes,
    int32_t row_bytes, uint32_t n_items, uint32_t pieces) {
    const int lane = threadIdx.x & 63;
    const uint32_t n_waves = gridDim.x * (kCopyThreads / 64);
    const uint32_t wave = blockIdx.x * (kCopyThreads / 64) + (threadIdx.x >> 6);
    const uint32_t half_items = n_items >> 1;  // items of K
    for (uint64_t t0 = (uint64_t)wave * kCopyDepth; t0 < n_items; t0 += (uint64_t)n_waves * kCopyDepth) {
        // lane j (mod 8): the length that item t0 + j needs (items past the end repeat the last one)
        int32_t my_len = 0;
        {
            uint32_t t = (uint32_t)min(t0 + (lane & (kCopyDepth - 1)), (uint64_t)n_items - 1);
            if (t >= half_items) t -= half_items;
            const uint32_t cache = kOnePiece ? t : t / pieces;
            if (kByValue) {
#pragma unroll
                for (int i = 0; i < kMaxStreamsPerLaunch; ++i) my_len = cache == (uint32_t)i ? lens.v[i] : my_len;
            } else if (lane < kCopyDepth) {  // (one request of 32 bytes: the lengths may sit in pinned host memory)
                my_len = lens_device[cache];
            }
        }
        // every load is issued (from a clamped, valid address) before the first store; only the
        // stores are conditional
        u32x4 v[kCopyDepth];
        char* dst[kCopyDepth];
        bool ok[kCopyDepth];
#pragma unroll
        for (int u = 0; u < kCopyDepth; ++u) {
            uint32_t t = (uint32_t)min(t0 + u, (uint64_t)n_items - 1);
            const bool which = t >= half_items;
            if (which) t -= half_items;
            const uint32_t cache = kOnePiece ? t : t / pieces;
            const uint32_t piece = kOnePiece ? 0 : t - cache * pieces;
            const int64_t off = (int64_t)piece * 1024 + lane * 16;
            ok[u] = t0 + u < n_items && off < row_bytes;
            const int64_t off_in = min(off, (int64_t)row_bytes - 16);
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(
                (which ? v_src : k_src) + (int64_t)cache * src_stride_bytes + src_row_offset_bytes + off_in));
            dst[u] = (which ? v_slab : k_slab) + (int64_t)cache * cache_stride_bytes + off;
        }
        // (the compiler would otherwise move every load down to its store, one in flight at a time)
        static_assert(kCopyDepth == 8, "the statement below names eight values");
        asm volatile("" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]));
#pragma unroll
        for (int u = 0; u < kCopyDepth; ++u) {
            const int32_t len = __shfl(my_len, u);
            if (ok[u]) __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4*>(dst[u] + (int64_t)len * row_bytes));
        }
    }
}

// ---- mean pool ---------------------------------------------------------------
// Block: 16 column chunks (of VEC columns) x 16 row groups, so that a frame's rows are read
// with many loads in flight.  Row group r sums rows r, r+16, ... in order in fp32 (4 rows are
// loaded before they are added); the 16 partial sums are added in order 0..15; one rounding.
constexpr int kPoolCols = 16, kPoolRowGroups = 16;
template <typename T, int VEC>
__global__ __launch_bounds__(kPoolCols * kPoolRowGroups) void mean_pool_kernel(
    const T* __restrict__ e, int n, int d, T* __restrict__ c) {
    const int cl = threadIdx.x % kPoolCols, rg = threadIdx.x / kPoolCols;
    const int col = (blockIdx.x * kPoolCols + cl) * VEC;
    __shared__ float part[kPoolRowGroups][kPoolCols][VEC];
    float s[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) s[k] = 0.f;
    if (col < d) {
        int r = rg;
        for (; r + 3 * kPoolRowGroups < n; r += 4 * kPoolRowGroups) {
            alignas(16) T tmp[4][VEC];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                *reinterpret_cast<uint4*>(tmp[u]) =
                    *reinterpret_cast<const uint4*>(e + (int64_t)(r + u * kPoolRowGroups) * d + col);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int k = 0; k < VEC; ++k) s[k] += to_f32(tmp[u][k]);
        }
        for (; r < n; r += kPoolRowGroups) {
            alignas(16) T tmp[VEC];
            *reinterpret_cast<uint4*>(tmp) = *reinterpret_cast<const uint4*>(e + (int64_t)r * d + col);
#pragma unroll
            for (int k = 0; k < VEC; ++k) s[k] += to_f32(tmp[k]);
        }
    }
#pragma unroll
    for (int k = 0; k < VEC; ++k) part[rg][cl][k] = s[k];
    __syncthreads();
    if (rg == 0 && col < d) {
        alignas(16) T tmp[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            float tot = part[0][cl][k];
#pragma unroll
            for (int g = 1; g < kPoolRowGroups; ++g) tot += part[g][cl][k];
            tmp[k] = from_f32<T>(tot / (float)n);
        }
        *reinterpret_cast<uint4*>(c + col) = *reinterpret_cast<const uint4*>(tmp);
    }
}

__global__ __launch_bounds__(256) void zero_fill_kernel(uint32_t* p, size_t n) {
    const size_t i = blockIdx.x * (size_t)256 + threadIdx.x;
    if (i < n) p[i] = 0u;
}

}  // namespace

size_t control_block_bytes(const vs_shape& s) {
    const size_t n = prefill_counter_offset(s) + (size_t)kMaxRowTiles * s.n_kv_heads * kCounterStrideBytes;
    return (n + 255) & ~size_t(255);
}

hipError_t launch_zero_fill(void* p, size_t bytes, hipStream_t st) {
    const size_t n = bytes / 4;
    zero_fill_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>((uint32_t*)p, n);
    return hipGetLastError();
}

hipError_t launch_prefill_simple(const vs_shape& s, const void* kc, const void* vc, int32_t len,
                                 const void* q, const void* kf, const void* vf, int32_t n_tokens,
                                 void* out, hipStream_t st) {
    LenTable none{};
    if (s.dtype == VS_F32)
        return launch_attn_simple<float>(s, kc, vc, 0, len, none, 0, 1, q, kf, vf, n_tokens, out, st);
    return launch_attn_simple<__bf16>(s, kc, vc, 0, len, none, 0, 1, q, kf, vf, n_tokens, out, st);
}

hipError_t launch_decode_simple(const vs_shape& s, int32_t n_streams, const void* k_slab,
                                const void* v_slab, int32_t capacity, const LenTable& lens,
                                const void* q, void* out, hipStream_t st) {
    const int64_t stride = (int64_t)capacity * s.n_kv_heads * s.head_dim;
    if (s.dtype == VS_F32)
        return launch_attn_simple<float>(s, k_slab, v_slab, stride, 0, lens, 1, n_streams, q, nullptr,
                                         nullptr, 1, out, st);
    return launch_attn_simple<__bf16>(s, k_slab, v_slab, stride, 0, lens, 1, n_streams, q, nullptr,
                                      nullptr, 1, out, st);
}

hipError_t launch_append_rows(int32_t n_caches, void* k_slab, void* v_slab, int64_t cache_stride_bytes,
                              const LenTable* lens_by_value, const int32_t* lens_device,
                              const void* k_src, const void* v_src, int64_t src_stride_bytes,
                              int64_t src_row_offset_bytes, int32_t row_bytes, hipStream_t st) {
    LenTable t{};
    if (lens_by_value) t = *lens_by_value;
    const int64_t pieces = (row_bytes + 1023) / 1024;
    const int64_t n_items = (int64_t)n_caches * 2 * pieces;
    if (n_items < 1 || n_items > 0x7fffffff) return hipErrorInvalidValue;
    const int64_t per_wg = (int64_t)(kCopyThreads / 64) * kCopyDepth;
    int64_t n_wg = (n_items + per_wg - 1) / per_wg;
    if (n_wg > kCopyMaxWorkgroups) n_wg = kCopyMaxWorkgroups;
#define VS_GO(ONE, BYVAL)                                                                             \
    append_rows_kernel<ONE, BYVAL><<<(unsigned)n_wg, kCopyThreads, 0, st>>>(                           \
        (char*)k_slab, (char*)v_slab, cache_stride_bytes, t, lens_device, (const char*)k_src,          \
        (const char*)v_src, src_stride_bytes, src_row_offset_bytes, row_bytes, (uint32_t)n_items, (uint32_t)pieces)
    if (lens_device) {
        if (pieces == 1) VS_GO(true, false);
        else VS_GO(false, false);
    } else {
        if (n_caches > kMaxStreamsPerLaunch) return hipErrorInvalidValue;
        if (pieces == 1) VS_GO(true, true);
        else VS_GO(false, true);
    }
#undef VS_GO
    return hipGetLastError();
}

hipError_t launch_mean_pool(const void* e, int32_t n, int32_t d, int32_t dtype, void* c_out,
                            hipStream_t st) {
    if (dtype == VS_F32) {
        const int blocks = (d / 4 + kPoolCols - 1) / kPoolCols;
        mean_pool_kernel<float, 4><<<blocks, kPoolCols * kPoolRowGroups, 0, st>>>((const float*)e, n, d, (float*)c_out);
    } else {
        const int blocks = (d / 8 + kPoolCols - 1) / kPoolCols;
        mean_pool_kernel<__bf16, 8><<<blocks, kPoolCols * kPoolRowGroups, 0, st>>>((const __bf16*)e, n, d, (__bf16*)c_out);
    }
    return hipGetLastError();
}

}  // namespace vs
