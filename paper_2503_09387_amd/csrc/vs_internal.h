// Internal declarations shared by the C-ABI layer and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "videoscan.h"

namespace vs {

constexpr int kMaxStreamsPerLaunch = 64;  // lengths travel by value in the kernel arguments
constexpr int kMaxPrefillSplits = 32;
constexpr int kMaxGroup = 8;              // query heads per KV head

// launch-plan overrides (0 = automatic), set through vs_set_tuning
extern int g_tune_prefill_splits;
extern int g_tune_prefill_kv_groups;
extern int g_tune_decode_chunk_rows;
extern int g_tune_prefill_merge;  // 0 automatic, 1 inside the kernel by the last workgroup alone, 2 always by the second kernel

struct LenTable {
    int32_t v[kMaxStreamsPerLaunch];
};

// ---- storage <-> fp32 -------------------------------------------------------
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(__bf16 x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ __bf16 from_f32<__bf16>(float x) { return (__bf16)x; }  // RNE

// ---- launchers (each validates nothing: the C-ABI layer has done it) ---------
// fp32-arithmetic reference-shaped path, any storage type (used for VS_F32).
hipError_t launch_prefill_simple(const vs_shape& s, const void* kc, const void* vc, int32_t len,
                                 const void* q, const void* kf, const void* vf, int32_t n_tokens,
                                 void* out, hipStream_t st);
hipError_t launch_decode_simple(const vs_shape& s, int32_t n_streams, const void* k_slab,
                                const void* v_slab, int32_t capacity, const LenTable& lens,
                                const void* q, void* out, hipStream_t st);

// bf16 MFMA prefill with split along cache rows; optional fused carrier append.
size_t prefill_mfma_workspace_bytes(const vs_shape& s, int32_t max_q_tokens);
// n_frames > 1: q, kf, vf, out hold a run of frames [n_frames][n_tokens][..] under the semantic-aware
// mask; k_append_dst / v_append_dst (row `len` of the cache) then receive all their carriers.
// append_all (single run only): every row of the run goes to the cache, not just the last.
hipError_t launch_prefill_mfma(const vs_shape& s, const void* kc, const void* vc, int32_t len,
                               const void* q, const void* kf, const void* vf, int32_t n_tokens,
                               void* out, void* k_append_dst, void* v_append_dst, void* counters,
                               void* workspace, hipStream_t st, int32_t n_frames = 1, bool append_all = false);
size_t prefill_frames_workspace_bytes(const vs_shape& s, int32_t n_frames, int32_t n_tokens, int32_t nsplit);
int prefill_frames_splits(const vs_shape& s, int32_t n_frames, int32_t n_tokens, int32_t len);

// bf16 split-row decode over ragged streams; appends (k_new, v_new) on the side when given.
// `counters` points at the front of an initialised workspace's control block: reserved for the decode
// kernels, which at present keep no state between or within launches there.
size_t decode_mfma_workspace_bytes(const vs_shape& s, int32_t n_streams, int32_t max_rows);
hipError_t launch_decode_mfma(const vs_shape& s, int32_t n_streams, void* k_slab, void* v_slab,
                              int32_t capacity, const LenTable& lens, const void* q,
                              const void* k_new, const void* v_new, void* out, void* counters,
                              void* workspace, hipStream_t st);

// Control block at the start of every workspace: [kMaxStreamsPerLaunch][Hkv] words reserved for decode
// (unused), then the prefill's arrival counters, one per unit = (KV head, frame, row tile), each alone
// in 128 bytes (the workgroups of a unit look at theirs while they wait for one another: counters of
// other units in the same line would queue behind those looks).  A counter wraps to zero with the last
// arrival, so all of them are zero between launches.
constexpr int kMaxRowTiles = 256;
constexpr int kCounterStrideBytes = 128;
size_t control_block_bytes(const vs_shape& s);
inline size_t prefill_counter_offset(const vs_shape& s) {  // from the start of the control block; a multiple of 128
    const size_t n = (size_t)kMaxStreamsPerLaunch * s.n_kv_heads * sizeof(unsigned int);
    return (n + 127) & ~size_t(127);
}
hipError_t launch_zero_fill(void* p, size_t bytes, hipStream_t st);
// log2 of the number of XCDs workgroup ids are dealt to in turn on this device, -1 if unknown
int xcd_shift_of_device(int dev);
// Finds out once per device how workgroup ids are dealt to the XCDs (scratch: 256 bytes of device
// memory; synchronises the stream the first time).
hipError_t probe_xcd_mapping(void* scratch, hipStream_t st);
// True once after a workgroup of an in-kernel-merge launch on this device has reported that it ran
// on another XCD than probed; in-kernel merging is then off for the device until it is probed again.
bool prefill_placement_fault(int dev);
void prefill_guard_test_mode(int on);
// What a kernel that merges inside the launch needs to know about the device: how many XCDs ids are
// dealt to in turn (log2), which XCD ids of residue r were seen on (4 bits each), the host word (as
// the kernels address it) through which a workgroup reports, and how often a waiting workgroup looks
// before it gives up.  False: not probed, a fault has been reported since, or merging inside kernels is
// switched off (VS_TUNE_PREFILL_MERGE = 2): merge with a second kernel.
struct XcdPlacement {
    int xcd_shift;
    unsigned long long xcc_of_residue;
    unsigned* misplaced;
    int max_looks;
};
bool xcd_placement_of_device(int dev, XcdPlacement* out);

// the body of vs_decode_attn (checks, launches, length bookkeeping) over any workspace
vs_status decode_entry(const vs_shape* shape, int32_t n_streams, void* k_slab, void* v_slab, int32_t capacity,
                       int32_t* lens, const void* q, const void* k_new, const void* v_new, void* out,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

// row copies
hipError_t launch_append_rows(int32_t n_caches, void* k_slab, void* v_slab, int64_t cache_stride_bytes,
                              const LenTable* lens_by_value, const int32_t* lens_device,
                              const void* k_src, const void* v_src, int64_t src_stride_bytes,
                              int64_t src_row_offset_bytes, int32_t row_bytes, hipStream_t st);

// memory bank (Section 3.3, memory mechanism)
constexpr int kBankMaxTables = 64;  // tables (layers x {K, V}) per launch: their pointers travel by value
hipError_t launch_bank_cosines(const void* e, const void* e_new, int32_t M, int32_t d, int32_t dtype,
                               int32_t policy, double* cosines, hipStream_t st);
hipError_t launch_bank_shift(int32_t n_tables, void* const* bases, const void* const* new_rows, int64_t row_bytes,
                             int32_t first, int32_t M, int32_t append_at, const double* cosines, int32_t* victim_io,
                             hipStream_t st);

hipError_t launch_mean_pool(const void* e, int32_t n, int32_t d, int32_t dtype, void* c_out,
                            hipStream_t st);

// frame rows and their Q/K/V projections (Sections 3.1 - 3.3)
hipError_t launch_frame_qkv(const vs_shape& s, const void* e, int32_t n_visual, int32_t d, const void* w,
                            void* q, void* k, void* v, void* c_out, hipStream_t st);

// dense layers around the attention (Sections 3.1, 4.1): out = X W^T with fp32 sums and a choice of what
// happens to them (vs_linear_mode); store mode may cut the output features into three tensors
// (out: features < seg0, out1: < seg1, out2: the rest).  workspace: linear_workspace_bytes.
size_t linear_workspace_bytes(int32_t n_rows, int32_t K, int32_t N);
// arrival_counters: the prefill's counters in an initialised control block (null: none).  With them, and
// at most kMaxRowTiles * Hkv blocks, the split-K shares are added inside the multiplying launch.
hipError_t launch_linear(const void* x, int32_t ldx, const void* w, int32_t n_rows, int32_t K, int32_t N, int32_t mode,
                         const void* residual, void* out, void* workspace, hipStream_t st, void* out1 = nullptr,
                         void* out2 = nullptr, int32_t seg0 = 0, int32_t seg1 = 0, void* arrival_counters = nullptr,
                         int32_t n_counters = 0);
hipError_t launch_rmsnorm(const void* x, const void* gamma, int32_t n_rows, int32_t d, float eps, void* out,
                          hipStream_t st);

}  // namespace vs
