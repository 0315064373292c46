// Memory bank of the semantic carriers (VideoScan Section 3.3, memory mechanism): at most M
// carriers are kept; when one arrives at a full bank, embeddings of adjacent carriers are
// compared and the older carrier of the most similar pair is dropped.  Reading of the passage:
// the sequence bank[0..M-1], incoming has M adjacent pairs (i, i+1); victim = the i with the
// largest cosine, of equal ones the smallest i (policy 1: the i whose cosine with the incoming
// carrier is largest).  A vector of norm 0 has cosine 0 with everything.
//
// Two steps on the device, no host round trip in between:
//   1. bank_cosine_kernel: one workgroup per pair, fp64 sums in a fixed order (the products of
//      bf16 or fp32 values are exact in fp64, so the cosines agree with a plain fp64 evaluation
//      to ~1e-13 and the victim is the same unless two cosines are that close);
//   2. bank_shift_kernel: every workgroup finds the victim from the M cosines (or reads the
//      index an earlier call left in device memory), then a table of per-carrier rows (the
//      embeddings, or one layer's K or V rows) drops that row, closes the gap and takes the
//      new row last.  A workgroup owns a 1 KB wide column block of one table: it loads up to
//      128 rows into registers, waits for all its wavefronts to have theirs, and stores them one
//      row up, so the move is in place and takes one round trip per 128 rows.
#include "vs_internal.h"

namespace vs {
namespace {

constexpr int kShiftThreads = 256;   // 4 rows of 64 16-byte pieces per step
constexpr int kShiftSteps = 32;      // rows per thread and pass: 128 rows per pass

__device__ __forceinline__ double block_sum(double x, double* lds) {  // fixed order, every thread gets the sum
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[w] = x;
    __syncthreads();
    return (lds[0] + lds[1]) + (lds[2] + lds[3]);
}

template <typename T>
__global__ __launch_bounds__(256) void bank_cosine_kernel(const T* __restrict__ e, const T* __restrict__ e_new,
                                                          int M, int d, int policy, double* __restrict__ cosines) {
    __shared__ double lds[4];
    const int i = blockIdx.x;
    const T* a = e + (int64_t)i * d;
    const T* b = (policy == 1 || i + 1 == M) ? e_new : e + (int64_t)(i + 1) * d;
    double ab = 0.0, aa = 0.0, bb = 0.0;
    for (int j = threadIdx.x; j < d; j += 256) {
        const double x = (double)to_f32(a[j]), y = (double)to_f32(b[j]);
        ab += x * y;
        aa += x * x;
        bb += y * y;
    }
    ab = block_sum(ab, lds);
    aa = block_sum(aa, lds);
    bb = block_sum(bb, lds);
    if (threadIdx.x == 0) cosines[i] = (aa > 0.0 && bb > 0.0) ? ab / (sqrt(aa) * sqrt(bb)) : 0.0;
}

struct ShiftTables {
    char* base[kBankMaxTables];           // table t: rows of row_bytes bytes
    const char* new_row[kBankMaxTables];  // the row that becomes the last one
};

struct ShiftParams {
    ShiftTables t;
    int64_t row_bytes;
    int first;              // rows in front of the carriers
    int M;                  // carriers of a full bank
    int append_at;          // >= 0: room left, the new row goes to first + append_at; -1: drop the victim
    const double* cosines;  // [M], or null: the victim's index is read from victim_io
    int* victim_io;         // device int (may be null when cosines are given)
};

__global__ __launch_bounds__(kShiftThreads) void bank_shift_kernel(ShiftParams p) {
    __shared__ int s_victim;
    __shared__ double s_cos[kShiftThreads / 64];
    __shared__ int s_idx[kShiftThreads / 64];
    const int tid = threadIdx.x;
    const int64_t col = (int64_t)blockIdx.x * 1024 + (tid & 63) * 16;  // this thread's 16 bytes of a row
    const int lr = tid >> 6;
    char* const base = p.t.base[blockIdx.y] + (int64_t)p.first * p.row_bytes;
    const char* const new_row = p.t.new_row[blockIdx.y];
    const bool in_row = col < p.row_bytes;
    if (p.append_at >= 0) {
        if (lr == 0 && in_row)
            *reinterpret_cast<uint4*>(base + (int64_t)p.append_at * p.row_bytes + col) =
                *reinterpret_cast<const uint4*>(new_row + col);
        if (p.victim_io && blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) *p.victim_io = -1;
        return;
    }
    int victim;
    if (p.cosines) {
        // largest cosine, of equal ones the smallest index: thread t looks at cosines t, t + 256, ..,
        // the candidates of a wavefront meet by lane exchanges, those of the wavefronts in LDS
        double best_cos = 0.0;
        int best = 0x7fffffff;  // (none yet)
        for (int i = tid; i < p.M; i += kShiftThreads) {
            const double c = p.cosines[i];
            if (best == 0x7fffffff || c > best_cos) {
                best = i;
                best_cos = c;
            }
        }
        auto better = [](double c_b, int i_b, double c_a, int i_a) {  // does candidate b beat candidate a?
            return i_b != 0x7fffffff && (i_a == 0x7fffffff || c_b > c_a || (c_b == c_a && i_b < i_a));
        };
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const double c_o = __shfl_xor(best_cos, off);
            const int i_o = __shfl_xor(best, off);
            if (better(c_o, i_o, best_cos, best)) {
                best_cos = c_o;
                best = i_o;
            }
        }
        if ((tid & 63) == 0) {
            s_cos[tid >> 6] = best_cos;
            s_idx[tid >> 6] = best;
        }
        __syncthreads();
        if (tid == 0) {
            for (int w2 = 1; w2 < kShiftThreads / 64; ++w2)
                if (better(s_cos[w2], s_idx[w2], best_cos, best)) {
                    best_cos = s_cos[w2];
                    best = s_idx[w2];
                }
            s_victim = best;
        }
        __syncthreads();
        victim = s_victim;
        if (p.victim_io && blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) *p.victim_io = victim;
    } else {
        victim = *p.victim_io;
    }
    victim = min(max(victim, 0), p.M - 1);  // (an index from device memory is not trusted to be in range)
    // rows victim+1 .. M-1 move to victim .. M-2, 128 rows per pass: all loads of a pass, a barrier,
    // all its stores (a later pass reads only rows that no earlier pass has written)
    for (int r0 = victim; r0 + 1 < p.M; r0 += 4 * kShiftSteps) {
        uint4 v[kShiftSteps];
#pragma unroll
        for (int u = 0; u < kShiftSteps; ++u) {
            const int r = r0 + 4 * u + lr;  // destination row
            if (r + 1 < p.M && in_row) v[u] = *reinterpret_cast<const uint4*>(base + (int64_t)(r + 1) * p.row_bytes + col);
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kShiftSteps; ++u) {
            const int r = r0 + 4 * u + lr;
            if (r + 1 < p.M && in_row) *reinterpret_cast<uint4*>(base + (int64_t)r * p.row_bytes + col) = v[u];
        }
        __syncthreads();
    }
    if (lr == 0 && in_row)
        *reinterpret_cast<uint4*>(base + (int64_t)(p.M - 1) * p.row_bytes + col) = *reinterpret_cast<const uint4*>(new_row + col);
}

}  // namespace

hipError_t launch_bank_cosines(const void* e, const void* e_new, int32_t M, int32_t d, int32_t dtype,
                               int32_t policy, double* cosines, hipStream_t st) {
    if (dtype == VS_F32)
        bank_cosine_kernel<float><<<M, 256, 0, st>>>((const float*)e, (const float*)e_new, M, d, policy, cosines);
    else
        bank_cosine_kernel<__bf16><<<M, 256, 0, st>>>((const __bf16*)e, (const __bf16*)e_new, M, d, policy, cosines);
    return hipGetLastError();
}

hipError_t launch_bank_shift(int32_t n_tables, void* const* bases, const void* const* new_rows, int64_t row_bytes,
                             int32_t first, int32_t M, int32_t append_at, const double* cosines, int32_t* victim_io,
                             hipStream_t st) {
    for (int32_t t0 = 0; t0 < n_tables; t0 += kBankMaxTables) {
        const int32_t n = n_tables - t0 < kBankMaxTables ? n_tables - t0 : kBankMaxTables;
        ShiftParams p;
        for (int32_t t = 0; t < n; ++t) {
            p.t.base[t] = (char*)bases[t0 + t];
            p.t.new_row[t] = (const char*)new_rows[t0 + t];
        }
        p.row_bytes = row_bytes;
        p.first = first;
        p.M = M;
        p.append_at = append_at;
        p.cosines = cosines;
        p.victim_io = victim_io;
        bank_shift_kernel<<<dim3((unsigned)((row_bytes + 1023) / 1024), (unsigned)n), kShiftThreads, 0, st>>>(p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace vs
