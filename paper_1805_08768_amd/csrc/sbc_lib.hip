// libsbc: host side of the C ABI declared in include/sbc.h.  Validates arguments, lays the
// call's tensors out as a table of chunks, and enqueues the kernels on the caller's stream.
// No device memory is allocated outside sbc_create().
#include "../../include/sbc.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <numeric>
#include <vector>

#include "sbc_accumulate_kernels.hpp"
#include "sbc_select_kernels.hpp"
#include "sbc_encode_kernels.hpp"
#include "sbc_decode_kernels.hpp"
#include "sbc_wide_kernels.hpp"
#include "sbc_step_kernels.hpp"

using namespace sbc;

namespace {
// kernels of sbc_compress in launch order (the histogram path repeats some of them)
enum Stage { kStSample = 0, kStAccumulate, kStWide, kStSelect, kStChunkSummary, kStTensorScan, kStPack,
             kStGather, kNumStages };
const char* const kStageNames[kNumStages] = {
    "k_sample_thresholds", "k_client_step", "k_wide_* (grid-wide selection, all launches)", "k_select",
    "k_chunk_summary", "k_tensor_scan", "k_pack", "k_finish_message"};
}  // namespace

constexpr int kDescSlots = 4;             // device copies of the tensor table, keyed by the pointer lists
constexpr int kMaxWideDec = 16;
constexpr uint32_t kMaxDecExtra = 512;    // additional decode workgroups that share a stream's scatter
constexpr uint32_t kDecSharePer = 384;    // kept entries per sharing workgroup
constexpr uint32_t kDecShareMax = 8;           // streams per call that the tile decoder can take
constexpr uint32_t kWideMinKept = 8192;   // kept entries per side from which a tensor takes those routes

struct DescSlot {
    bool valid = false;
    uint64_t stamp = 0;
    std::vector<const float*> dW;
    std::vector<float*> R;
};

struct sbc_ctx {
    int device = 0;
    int64_t max_elems = 0;
    int max_tensors = 0;
    uint64_t max_chunks = 0;
    uint64_t kept_cap = 0;
    uint64_t stage_cap = 0;

    // ---- device scratch of sbc_compress ----
    TensorDesc* d_desc = nullptr;         // kDescSlots tables of max_tensors entries
    uint32_t* d_chunk_tensor = nullptr;
    uint2* d_sched = nullptr;             // workgroup of the streaming kernel -> (chunk, tensor)
    GroupState* d_group = nullptr;        // per group of chunks: candidate and completion counters
    uint64_t max_groups = 0;
    bool compact = false;                 // candidate lists of a few times k entries instead of n
    uint64_t cand_entries = 0;            // entries d_cand holds
    uint32_t n_sched = 0;                 // workgroups of the streaming kernel
    uint32_t* d_order = nullptr;
    uint32_t* d_hist = nullptr;
    TensorState* d_state = nullptr;
    uint2* d_cand = nullptr;
    uint32_t* d_bitmap = nullptr;
    uint32_t* d_stage = nullptr;
    uint32_t* d_kept = nullptr;
    ChunkSummary* d_sum = nullptr;
    uint32_t* d_prev_end = nullptr;
    uint64_t* d_bitoff = nullptr;
    TileSummary* d_tile = nullptr;        // per tile of kScanTile chunks of a tensor encoded from the bitmap
    ResultBlock* d_result = nullptr;      // two for compress, two for decode, used in turn; [4] collects the
                                          // errors of decode calls whose status is deferred, [5] is a spare
    // grid-wide selection
    WideState* d_wide_state = nullptr;
    uint32_t* d_wide_hist = nullptr;
    uint32_t* d_wide_hist2 = nullptr;
    uint32_t* d_wide_tie_cnt = nullptr;
    long long* d_wide_acc = nullptr;
    uint32_t* d_wide_tie = nullptr;

    // ---- device scratch of sbc_decompress_accumulate ----
    DecDesc* d_dec = nullptr;
    uint2* d_dec_blocks = nullptr;        // workgroup -> (tensor, share | shares << 16) of the decode kernel
    DecWide* d_dec_wide = nullptr;        // long streams decoded tile by tile
    unsigned long long* d_seg_fn = nullptr;
    unsigned long long* d_seg_pack = nullptr;
    unsigned long long* d_tile_fn = nullptr;
    unsigned long long* d_tile_sum = nullptr;
    uint32_t* d_tile_entry = nullptr;
    uint64_t dec_seg_cap = 0, dec_tile_cap = 0;

    // ---- pinned host staging ----
    TensorDesc* h_desc = nullptr;
    uint32_t* h_chunk_tensor = nullptr;
    uint2* h_sched = nullptr;
    uint32_t* h_order = nullptr;
    uint32_t* h_wide_ids = nullptr;
    ResultBlock* h_result_dev = nullptr;  // h_result as the device addresses it
    ResultBlock* h_result = nullptr;      // compress
    uint32_t result_seq = 0;              // number of the latest launch of the message-assembly kernel
    ResultBlock* h_result_dec = nullptr;  // decode (its own block: a decode call may come between begin and end)
    ResultBlock* h_result_dec_dev = nullptr;
    uint32_t dec_seq = 0;
    DecDesc* h_dec = nullptr;
    uint2* h_dec_blocks = nullptr;
    uint32_t n_dec_blocks = 0;
    DecWide* h_dec_wide = nullptr;
    TensorState* h_state = nullptr;

    // ---- plan of the last compress call: everything that depends on sizes and p only ----
    bool cache_valid = false; int cache_T = 0; double cache_p = 0.0;
    std::vector<int64_t> cache_numel;
    uint64_t cache_total = 0, cache_chunks = 0, cache_stage_words = 0, cache_kept_total = 0, cache_max_bound = 0;
    uint32_t cache_scan_tiles = 1;        // most tiles of the chunk scan among the tensors encoded from the bitmap
    uint32_t cache_bitmap_chunks_max = 0; // most chunks among those tensors
    bool cache_any_bitmap = false;
    bool cache_all_inline = false;        // every tensor is finished inside the streaming kernel
    int cache_force_exact = 0;
    std::vector<TensorDesc> plan;         // without the pointers
    std::vector<uint32_t> plan_order;
    int n_wide = 0;                       // tensors given to the grid-wide selection
    uint32_t wide_blocks = 0;
    DescSlot slot[kDescSlots];            // which pointer lists the device tables hold
    uint64_t slot_clock = 0;

    // ---- what the decode tables currently hold ----
    int dev_dec_T = 0;
    bool dev_dec_valid = false;
    double dec_p = 0.0;
    int n_dec_wide = 0;
    uint32_t dec_tiles = 0;

    // ---- options ----
    int force_exact = 0;
    int carry_keys = 1;
    int carry_stale_run = 0;                 // sampled calls in a row that found the previous call's keys stale
    int carry_backoff = 0, carry_hold = 0;   // sampled calls after a call whose carried keys let a flood pass
    int fused_step = 0;                   // the streaming kernel finishes the tensors it can by itself
    int sampled = 0;                      // subsampled variant: the sampled threshold decides what is kept
    int defer_decode = 0;                 // decode calls return once enqueued; sbc_decode_status reports
    bool deferred_pending = false;        // some deferred decode has not been waited for yet
    bool deferred_dirty = true;           // block [4] must be cleared before the next deferred decode
    uint32_t wide_min_kept = kWideMinKept;

    // filter keys carried over from the previous successful call (same tensor sizes, same p)
    bool hist_valid = false;
    double hist_p = 0.0;
    std::vector<uint32_t> hist_n;

    // result blocks: calls alternate between two, and a kernel of each call clears the other one
    int result_idx = 0;
    bool result_dirty = true;             // the next compress call must clear its result blocks itself
    int dec_result_idx = 0;
    bool dec_result_dirty = true;

    // optional per-kernel timing: start/stop events of the dispatches
    int profile_level = 0;
    hipEvent_t ev[2 * kNumStages] = {};
    bool ev_ok = false;
    hipEvent_t ev_result = nullptr;       // recorded behind the copy of a client step's result block
    double stage_ms[kNumStages] = {};
    int64_t stage_calls[kNumStages] = {};

    // a client step that has been enqueued (sbc_compress_begin) and not yet completed
    struct Pending {
        bool active = false;
        hipStream_t stream = nullptr;
        int T = 0, b = 0, slot = 0, force_exact = 0, carry = 0;
        double p = 0.0;
        bool slot_is_new = false, use_history = false, sampled = false, any_bitmap = false, all_inline = false;
        bool wait_on_event = false;   // begin/end form: the wait ends with this step, not with the stream
        bool timed[kNumStages] = {};
        ResultBlock* res_now = nullptr;
        ResultBlock* res_next = nullptr;
        TensorDesc* d_desc = nullptr;
        uint8_t* msg8 = nullptr;
        size_t msg_capacity = 0, need = 0;
        uint32_t n_chunks = 0;
        unsigned gather_y = 1, scan_tiles = 1, bitmap_chunks_max = 0;
    } pend;

    // last compress call, for the inspection entry points
    int last_T = 0;
    bool last_ok = false;
    bool last_used_exact_path = false;
    bool last_used_history = false;
    bool last_used_wide = false;
    bool last_loose = false;
    bool last_deferred = false;
    hipStream_t last_stream = nullptr;    // stream of the last client step (its last kernel may still be draining)
};

namespace {

constexpr double kPhi = 1.6180339887498948482;

struct DeviceGuard {
    int prev = -1;
    bool changed = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) == hipSuccess && prev != dev) changed = (hipSetDevice(dev) == hipSuccess);
    }
    ~DeviceGuard() { if (changed) (void)hipSetDevice(prev); }
};

int bstar_of(double p) {
    const double b = 1.0 + std::floor(std::log2(std::log(kPhi - 1.0) / std::log(1.0 - p)));
    if (b < 0.0) return 0;
    return (int)b;
}

bool valid_p(double p) { return p > 0.0 && p < 1.0; }

int64_t kept_of(int64_t n, double p) {
    int64_t k = (int64_t)std::floor(p * (double)n);
    if (k < 1) k = 1;
    if (k > n) k = n;
    return k;
}

// Most entries a side may keep: k, or in the subsampled variant min(n, 2k + 64).
int64_t cap_of(int64_t n, int64_t k, bool sampled) {
    return sampled ? std::min<int64_t>(n, 2 * k + 64) : k;
}

uint64_t bound_words_of(int64_t n, int64_t k, int b) {
    const uint64_t bits = (uint64_t)k * (uint64_t)(1 + b) + ((uint64_t)(n - k) >> b);
    return (bits + 31) >> 5;
}

template <typename T>
hipError_t dev_alloc(T** p, size_t count) { return hipMalloc(reinterpret_cast<void**>(p), count * sizeof(T)); }
template <typename T>
hipError_t host_alloc(T** p, size_t count) { return hipHostMalloc(reinterpret_cast<void**>(p), count * sizeof(T), hipHostMallocDefault); }

void free_all(sbc_ctx* c) {
    (void)hipFree(c->d_desc); (void)hipFree(c->d_chunk_tensor); (void)hipFree(c->d_sched); (void)hipFree(c->d_group); (void)hipFree(c->d_order); (void)hipFree(c->d_hist);
    (void)hipFree(c->d_state); (void)hipFree(c->d_cand); (void)hipFree(c->d_bitmap); (void)hipFree(c->d_stage);
    (void)hipFree(c->d_kept); (void)hipFree(c->d_sum); (void)hipFree(c->d_prev_end); (void)hipFree(c->d_bitoff); (void)hipFree(c->d_tile);
    (void)hipFree(c->d_result); (void)hipFree(c->d_dec); (void)hipFree(c->d_dec_blocks);
    if (c->h_dec_blocks) (void)hipHostFree(c->h_dec_blocks);
    (void)hipFree(c->d_dec_wide); (void)hipFree(c->d_seg_fn); (void)hipFree(c->d_seg_pack); (void)hipFree(c->d_tile_fn);
    (void)hipFree(c->d_tile_sum); (void)hipFree(c->d_tile_entry);
    if (c->h_dec_wide) (void)hipHostFree(c->h_dec_wide);
    (void)hipFree(c->d_wide_state); (void)hipFree(c->d_wide_hist);
    (void)hipFree(c->d_wide_acc); (void)hipFree(c->d_wide_tie); (void)hipFree(c->d_wide_hist2); (void)hipFree(c->d_wide_tie_cnt);
    if (c->h_wide_ids) (void)hipHostFree(c->h_wide_ids);
    if (c->h_desc) (void)hipHostFree(c->h_desc);
    if (c->h_chunk_tensor) (void)hipHostFree(c->h_chunk_tensor);
    if (c->h_sched) (void)hipHostFree(c->h_sched);
    if (c->h_order) (void)hipHostFree(c->h_order);
    if (c->h_result) (void)hipHostFree(c->h_result);
    if (c->h_result_dec) (void)hipHostFree(c->h_result_dec);
    if (c->h_dec) (void)hipHostFree(c->h_dec);
    if (c->h_state) (void)hipHostFree(c->h_state);
    if (c->ev_ok) for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
    if (c->ev_result) (void)hipEventDestroy(c->ev_result);
    c->ev_result = nullptr;
    c->ev_ok = false;
}

int status_of_err(uint32_t err) {
    if (err & kErrInternal) return SBC_EINTERNAL;
    if (err & kErrNonFinite) return SBC_ENONFINITE;
    if (err & kErrOverflow) return SBC_ECAPACITY;
    if (err & kErrCorrupt) return SBC_ECORRUPT;
    return SBC_OK;
}

// Kernels are timed only when profiling was asked for: the launch then carries a start and a
// stop event that take the dispatch's own begin and end time stamps (event 2s and 2s+1 for
// stage s), so the figure is the kernel's duration without the gaps between dispatches.
// Expects c (context), lvl (profile level), stream and timed[] in scope.
#define SBC_LAUNCH(stage, on, kernel, grid, block, ...)                                                    \
    do {                                                                                                   \
        if ((on) && (lvl >= 2 || (lvl == 1 && ((stage) == kStAccumulate || (stage) == kStSample)))) {      \
            hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, c->ev[2 * (stage)], c->ev[2 * (stage) + 1], 0, \
                                  __VA_ARGS__);                                                            \
            timed[stage] = true;                                                                           \
        } else {                                                                                           \
            hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);                               \
        }                                                                                                  \
    } while (0)

// Alg. 3 for the tensors whose positions are in the bitmap, then the message assembly, for the
// pending client step.
void launch_encode_and_gather(sbc_ctx* c, bool profile) {
    sbc_ctx::Pending& P = c->pend;
    const int lvl = c->profile_level;
    hipStream_t stream = P.stream;
    bool* timed = P.timed;
    const int T = P.T, b = P.b;
    if (P.any_bitmap && P.bitmap_chunks_max <= kSelfScanChunks && P.n_chunks <= 8192u) {
        // no tensor of many chunks among those encoded from the bitmap: the workgroups that write
        // the codes scan the few summaries before their chunk themselves, one launch less
        SBC_LAUNCH(kStChunkSummary, profile, k_chunk_summary<1>, dim3(P.n_chunks), dim3(kChunkWords), P.d_desc,
                   c->d_chunk_tensor, c->d_bitmap, c->d_sum, b, P.n_chunks);
        SBC_LAUNCH(kStPack, profile, (k_pack<1, true>), dim3(P.n_chunks), dim3(kChunkWords), P.d_desc, c->d_chunk_tensor,
                   c->d_bitmap, c->d_sum, c->d_prev_end, c->d_bitoff, c->d_state, b, c->d_stage, P.res_now, P.n_chunks);
    } else if (P.any_bitmap) {
        // (with very many chunks a workgroup takes four of them: see the kernels)
        const bool batch = P.n_chunks > 8192u;
        const dim3 per_chunk(batch ? (P.n_chunks + 3u) / 4u : P.n_chunks);
        if (batch) {
            SBC_LAUNCH(kStChunkSummary, profile, k_chunk_summary<4>, per_chunk, dim3(kChunkWords), P.d_desc,
                       c->d_chunk_tensor, c->d_bitmap, c->d_sum, b, P.n_chunks);
        } else {
            SBC_LAUNCH(kStChunkSummary, profile, k_chunk_summary<1>, per_chunk, dim3(kChunkWords), P.d_desc,
                       c->d_chunk_tensor, c->d_bitmap, c->d_sum, b, P.n_chunks);
        }
        if (P.scan_tiles > 1)
            hipLaunchKernelGGL(k_tile_summary, dim3(T, P.scan_tiles), dim3(kScanThreads), 0, stream, P.d_desc, c->d_sum,
                               c->d_tile, b);
        SBC_LAUNCH(kStTensorScan, profile, k_tensor_scan, dim3(T, P.scan_tiles), dim3(kScanThreads), P.d_desc, c->d_sum,
                   c->d_tile, c->d_prev_end, c->d_bitoff, c->d_state, b);
        if (batch) {
            SBC_LAUNCH(kStPack, profile, (k_pack<4, false>), per_chunk, dim3(kChunkWords), P.d_desc, c->d_chunk_tensor,
                       c->d_bitmap, c->d_sum, c->d_prev_end, c->d_bitoff, c->d_state, b, c->d_stage, P.res_now, P.n_chunks);
        } else {
            SBC_LAUNCH(kStPack, profile, (k_pack<1, false>), per_chunk, dim3(kChunkWords), P.d_desc, c->d_chunk_tensor,
                       c->d_bitmap, c->d_sum, c->d_prev_end, c->d_bitoff, c->d_state, b, c->d_stage, P.res_now, P.n_chunks);
        }
    }
    SBC_LAUNCH(kStGather, profile, k_finish_message, dim3(T, P.gather_y), dim3(256), P.d_desc, c->d_state, T, b,
               c->d_stage, c->d_kept, c->d_group, P.msg8, (uint64_t)P.msg_capacity, P.res_now, P.res_next,
               c->h_result_dev, ++c->result_seq);
}

// Alg. 2 for the pending step's tensors that keep very many entries, as grid-wide sweeps over
// their candidate lists with one-workgroup steps in between (the tensors k_select then skips).
void launch_wide_selection(sbc_ctx* c, bool handback) {
    sbc_ctx::Pending& P = c->pend;
    const int lvl = c->profile_level;
    hipStream_t stream = P.stream;
    bool* timed = P.timed;
    TensorDesc* const d_desc = P.d_desc;
    ResultBlock* const res_now = P.res_now;
    // (the sweeps that carry the second histogram have four times the threads per workgroup)
    const dim3 sweep(c->wide_blocks, (unsigned)c->n_wide), sweep4(std::max(128u, c->wide_blocks / 4u), (unsigned)c->n_wide);
    const bool time_wide = lvl >= 2;
    WideIds ids = {};
    std::memcpy(ids.id, c->h_wide_ids, sizeof(uint32_t) * (size_t)c->n_wide);
    if (time_wide) {
        hipExtLaunchKernelGGL(k_wide_count, sweep, dim3(kWideThreads), 0, stream, c->ev[2 * kStWide], nullptr, 0,
                              d_desc, ids, c->d_state, c->d_cand, c->d_wide_hist);
    } else {
        hipLaunchKernelGGL(k_wide_count, sweep, dim3(kWideThreads), 0, stream, d_desc, ids, c->d_state,
                           c->d_cand, c->d_wide_hist);
    }
    hipLaunchKernelGGL(k_wide_refine, sweep4, dim3(kWideSweepThreads), 0, stream, d_desc, ids, c->d_state,
                       c->d_cand, c->d_wide_state, c->d_wide_hist, c->d_wide_hist2, c->d_wide_acc, c->d_wide_tie_cnt);
    hipLaunchKernelGGL(k_wide_sums, sweep4, dim3(kWideSweepThreads), 0, stream, d_desc, ids, c->d_state,
                       c->d_cand, c->d_wide_state, c->d_wide_hist, c->d_wide_hist2, c->d_wide_acc, c->d_wide_tie,
                       c->d_wide_tie_cnt);
    if (time_wide) {
        hipExtLaunchKernelGGL(k_wide_apply, sweep, dim3(kWideThreads), 0, stream, nullptr, c->ev[2 * kStWide + 1], 0,
                              d_desc, ids, c->d_state, c->d_cand, c->d_wide_state, c->d_wide_hist2, c->d_wide_acc,
                              c->d_wide_tie, c->d_wide_tie_cnt, c->d_bitmap, handback ? 1 : 0, res_now);
        timed[kStWide] = true;
    } else {
        hipLaunchKernelGGL(k_wide_apply, sweep, dim3(kWideThreads), 0, stream, d_desc, ids, c->d_state,
                           c->d_cand, c->d_wide_state, c->d_wide_hist2, c->d_wide_acc, c->d_wide_tie, c->d_wide_tie_cnt,
                           c->d_bitmap, handback ? 1 : 0, res_now);
    }
}

// The pending step's result block on its way to the host / waited for.
int enqueue_result_copy(sbc_ctx* c) {
    if (hipGetLastError() != hipSuccess) return SBC_EHIP;
    // In the begin/end form an event lets the wait end when this step is done, whatever the caller
    // has enqueued behind it; the one-call form waits for the stream, which is cheaper.
    // (k_finish_message has written the result block to pinned host memory)
    if (hipGetLastError() != hipSuccess ||
        (c->pend.wait_on_event && hipEventRecord(c->ev_result, c->pend.stream) != hipSuccess)) {
        (void)hipGetLastError();
        return SBC_EHIP;
    }
    return SBC_OK;
}

// Looks for sequence number `want` in a result block in pinned host memory for up to 0.3 ms.
bool result_arrived(const ResultBlock* block, uint32_t want) {
    const auto t0 = std::chrono::steady_clock::now();
    for (int spin = 0;; ++spin) {
        if (__atomic_load_n(&block->pad, __ATOMIC_ACQUIRE) == want) return true;
        if ((spin & 63) == 63 && std::chrono::steady_clock::now() - t0 > std::chrono::microseconds(300)) return false;
    }
}

int wait_result(sbc_ctx* c) {
    // The message-assembly kernel writes the result block to pinned host memory and its sequence
    // number last.  Looking for the number takes a microsecond or two once it is there, where the
    // runtime's wait returns several microseconds after the stream has drained; calls that run
    // longer than a fraction of a millisecond fall through to the runtime's wait.  (Not while
    // kernels carry timing events: those are read right after this, and must be complete.)
    if (c->profile_level == 0 && result_arrived(c->h_result, c->result_seq)) return SBC_OK;
    if ((c->pend.wait_on_event ? hipEventSynchronize(c->ev_result) : hipStreamSynchronize(c->pend.stream)) != hipSuccess) {
        (void)hipGetLastError();
        return SBC_EHIP;
    }
    return SBC_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Server step without any allocation, for callers that cannot call hipMalloc (code under HIP graph
// capture, tight serving loops, harnesses that forbid allocation).  The tables the decode kernel
// reads (tensor descriptors, workgroup -> stream table, result block) live in a file-scope device
// array instead of a context; one small kernel fills them from the launch arguments, the decode
// kernel of sbc_decompress_accumulate runs on them, and a last kernel stores the status where the
// caller asked for it.  Nothing is copied to or from the host and nothing waits.
// ---------------------------------------------------------------------------------------------
namespace {

struct NoAllocScratch {
    ResultBlock result[2];
    DecDesc dec[SBC_NOALLOC_MAX_TENSORS];
    uint2 blocks[SBC_NOALLOC_MAX_TENSORS + kMaxDecExtra];
};

// launch arguments of the set-up kernel (kernel arguments may take 4 KiB)
struct NoAllocArgs {
    float* out[SBC_NOALLOC_MAX_TENSORS];
    uint32_t n[SBC_NOALLOC_MAX_TENSORS];
    uint16_t first_block[SBC_NOALLOC_MAX_TENSORS];
    uint8_t shares[SBC_NOALLOC_MAX_TENSORS];
};
static_assert(sizeof(NoAllocArgs) <= 3584, "must fit the kernel argument segment");

constexpr int kNoAllocMaxDevices = 64;

}  // namespace

// Every GPU the library runs on holds its own copy of this array until the process ends.  In
// host code the name is only a handle for hipGetSymbolAddress: the address the kernels receive
// is looked up once per device (noalloc_scratch_of) and kept.
static __device__ __align__(256) unsigned char scratch[(sizeof(NoAllocScratch) + 255) / 256 * 256];

__global__ __launch_bounds__(256) void k_noalloc_setup(NoAllocScratch* __restrict__ s, NoAllocArgs a, int T) {
    const int tid = threadIdx.x;
    // the array keeps the previous call's contents: everything the decode kernel reads is rewritten
    if (tid < 2) { s->result[tid].err = 0u; s->result[tid].pad = 0u; s->result[tid].msg_bytes = 0ull; }
    for (int t = tid; t < T; t += 256) {
        DecDesc d;
        d.out = a.out[t]; d.n = a.n[t]; d.wide = 0u;
        s->dec[t] = d;
        const uint32_t shares = a.shares[t];
        for (uint32_t sh = 0; sh < shares; ++sh) s->blocks[a.first_block[t] + sh] = make_uint2((uint32_t)t, sh | (shares << 16));
    }
}

__global__ void k_noalloc_finish(const NoAllocScratch* __restrict__ s, int32_t* __restrict__ status) {
    if (threadIdx.x == 0) {
        const uint32_t err = s->result[0].err;
        *status = (err & kErrInternal) ? SBC_EINTERNAL : (err & kErrCorrupt) ? SBC_ECORRUPT : SBC_OK;
    }
}

namespace {

// Device address of `scratch` on `device` (which must be current), looked up on first use.
NoAllocScratch* noalloc_scratch_of(int device) {
    static NoAllocScratch* ptr[kNoAllocMaxDevices] = {};
    static std::mutex lock;
    if (device < 0 || device >= kNoAllocMaxDevices) return nullptr;
    std::lock_guard<std::mutex> g(lock);
    if (!ptr[device]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        ptr[device] = static_cast<NoAllocScratch*>(p);
    }
    return ptr[device];
}

}  // namespace

#ifdef SBC_PHASE_TIMING
#include <chrono>
static double g_host_ts[16];
#define SBC_HOST_TS(i) (g_host_ts[i] = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count())
#else
#define SBC_HOST_TS(i) ((void)0)
#endif

extern "C" {

const char* sbc_strerror(int code) {
    switch (code) {
        case SBC_OK: return "ok";
        case SBC_EINVAL: return "invalid argument";
        case SBC_ECAPACITY: return "buffer or context too small";
        case SBC_EHIP: return "HIP runtime error";
        case SBC_ECORRUPT: return "corrupt message";
        case SBC_ENONFINITE: return "non-finite accumulated update";
        case SBC_EINTERNAL: return "internal invariant violated";
        default: return "unknown status";
    }
}

int sbc_golomb_bstar(double p) {
    if (!valid_p(p)) return SBC_EINVAL;
    return bstar_of(p);
}

int64_t sbc_num_kept(int64_t numel, double p) {
    if (!valid_p(p) || numel < 1) return SBC_EINVAL;
    return kept_of(numel, p);
}

static size_t msg_bound(const int64_t* numel, int n_tensors, double p, bool sampled) {
    if (!numel || n_tensors <= 0 || !valid_p(p)) return 0;
    const int b = bstar_of(p);
    if (b > kMaxB) return 0;
    uint64_t words = 0;
    for (int t = 0; t < n_tensors; ++t) {
        if (numel[t] < 1 || numel[t] >= (int64_t)1 << 32) return 0;
        words += bound_words_of(numel[t], cap_of(numel[t], kept_of(numel[t], p), sampled), b);
    }
    return (size_t)(32 + 24ull * (unsigned)n_tensors + 4ull * words);
}

size_t sbc_msg_bound(const int64_t* numel, int n_tensors, double p) { return msg_bound(numel, n_tensors, p, false); }

size_t sbc_msg_bound_sampled(const int64_t* numel, int n_tensors, double p) { return msg_bound(numel, n_tensors, p, true); }

static int create_context(sbc_ctx** out, int device, int64_t max_total_elems, int max_tensors, bool compact) {
    if (!out || max_total_elems < 1 || max_tensors < 1 || max_tensors >= (1 << 24)) return SBC_EINVAL;
    *out = nullptr;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess) return SBC_EHIP;
    if (device < 0 || device >= n_dev) return SBC_EINVAL;
    sbc_ctx* c = new (std::nothrow) sbc_ctx();
    if (!c) return SBC_EHIP;
    c->device = device;
    c->max_elems = max_total_elems;
    c->max_tensors = max_tensors;
    c->compact = compact;
    // full: both sides' lists of every tensor hold every entry; compact: half an entry per entry in all
    // (plus the lists' fixed part), shared out by the plan of each call
    c->cand_entries = compact ? (uint64_t)max_total_elems / 2 + 2048ull * (uint64_t)max_tensors : 2ull * (uint64_t)max_total_elems;
    c->max_chunks = (uint64_t)max_total_elems / kChunk + (uint64_t)max_tensors;
    c->kept_cap = std::min<uint64_t>((uint64_t)max_total_elems, (uint64_t)kFusedBigK * (uint64_t)max_tensors);
    // A tensor's stream is at most k(1+b*) + (n-k)/2^b* bits, which stays below 1.3 n for every p
    // (b* shrinks as p grows); n/16 words plus rounding per tensor is ample, and sbc_compress
    // checks the actual need against this capacity.
    c->stage_cap = (uint64_t)max_total_elems / 16 + 64ull * (uint64_t)max_tensors + 64ull;
    DeviceGuard guard(device);
    const size_t T = (size_t)max_tensors;
    bool ok = true;
    ok = ok && dev_alloc(&c->d_desc, (size_t)kDescSlots * T) == hipSuccess;
    ok = ok && dev_alloc(&c->d_chunk_tensor, (size_t)c->max_chunks) == hipSuccess;
    c->max_groups = c->max_chunks / kGroupChunks + (uint64_t)max_tensors;
    ok = ok && dev_alloc(&c->d_sched, (size_t)c->max_chunks) == hipSuccess;
    ok = ok && dev_alloc(&c->d_group, (size_t)c->max_groups) == hipSuccess;
    ok = ok && hipMemset(c->d_group, 0, sizeof(GroupState) * c->max_groups) == hipSuccess;
    ok = ok && host_alloc(&c->h_sched, (size_t)c->max_chunks) == hipSuccess;
    ok = ok && dev_alloc(&c->d_order, T) == hipSuccess;
    ok = ok && dev_alloc(&c->d_hist, T * kL1Bins) == hipSuccess;
    ok = ok && dev_alloc(&c->d_state, T) == hipSuccess;
    ok = ok && hipMemset(c->d_state, 0, sizeof(TensorState) * T) == hipSuccess;
    ok = ok && dev_alloc(&c->d_cand, (size_t)c->cand_entries) == hipSuccess;
    ok = ok && dev_alloc(&c->d_bitmap, (size_t)c->max_chunks * kChunkWords) == hipSuccess;
    ok = ok && dev_alloc(&c->d_stage, (size_t)c->stage_cap) == hipSuccess;
    ok = ok && dev_alloc(&c->d_kept, (size_t)c->kept_cap) == hipSuccess;
    ok = ok && dev_alloc(&c->d_sum, (size_t)c->max_chunks) == hipSuccess;
    ok = ok && dev_alloc(&c->d_prev_end, (size_t)c->max_chunks) == hipSuccess;
    ok = ok && dev_alloc(&c->d_bitoff, (size_t)c->max_chunks) == hipSuccess;
    ok = ok && dev_alloc(&c->d_tile, (size_t)(c->max_chunks / kScanTile) + T + 1) == hipSuccess;
    ok = ok && dev_alloc(&c->d_result, 6) == hipSuccess;
    ok = ok && dev_alloc(&c->d_dec, T) == hipSuccess;
    ok = ok && dev_alloc(&c->d_dec_blocks, T + kMaxDecExtra) == hipSuccess;
    ok = ok && host_alloc(&c->h_dec_blocks, T + kMaxDecExtra) == hipSuccess;
    // tile decode: a stream of w words has w/2 segments; every stream is rounded up to whole tiles
    c->dec_seg_cap = c->stage_cap / 2 + (uint64_t)(kMaxWideDec + 1) * kDecThreads;
    c->dec_tile_cap = c->dec_seg_cap / kDecThreads + kMaxWideDec;
    ok = ok && dev_alloc(&c->d_dec_wide, (size_t)kMaxWideDec) == hipSuccess;
    ok = ok && host_alloc(&c->h_dec_wide, (size_t)kMaxWideDec) == hipSuccess;
    ok = ok && dev_alloc(&c->d_seg_fn, (size_t)c->dec_seg_cap) == hipSuccess;
    ok = ok && dev_alloc(&c->d_seg_pack, (size_t)c->dec_seg_cap) == hipSuccess;
    ok = ok && dev_alloc(&c->d_tile_fn, (size_t)c->dec_tile_cap) == hipSuccess;
    ok = ok && dev_alloc(&c->d_tile_sum, (size_t)c->dec_tile_cap) == hipSuccess;
    ok = ok && dev_alloc(&c->d_tile_entry, (size_t)c->dec_tile_cap) == hipSuccess;
    ok = ok && dev_alloc(&c->d_wide_state, (size_t)kMaxWide) == hipSuccess;
    ok = ok && dev_alloc(&c->d_wide_hist, (size_t)kMaxWide * 2 * kWindow) == hipSuccess;
    ok = ok && dev_alloc(&c->d_wide_hist2, (size_t)kMaxWide * 2 * kWideRefine) == hipSuccess;
    ok = ok && dev_alloc(&c->d_wide_tie_cnt, (size_t)kMaxWide * 2) == hipSuccess;
    ok = ok && dev_alloc(&c->d_wide_acc, (size_t)kMaxWide * 512) == hipSuccess;
    ok = ok && dev_alloc(&c->d_wide_tie, (size_t)kMaxWide * 2 * kWideTieMax) == hipSuccess;
    ok = ok && host_alloc(&c->h_wide_ids, (size_t)kMaxWide) == hipSuccess;
    // the histograms and accumulators start out zero; the kernels that read them leave them zero
    ok = ok && hipMemset(c->d_wide_hist, 0, sizeof(uint32_t) * kMaxWide * 2 * kWindow) == hipSuccess;
    ok = ok && hipMemset(c->d_wide_hist2, 0, sizeof(uint32_t) * kMaxWide * 2 * kWideRefine) == hipSuccess;
    ok = ok && hipMemset(c->d_wide_acc, 0, sizeof(long long) * kMaxWide * 512) == hipSuccess;
    ok = ok && host_alloc(&c->h_desc, T) == hipSuccess;
    ok = ok && host_alloc(&c->h_chunk_tensor, (size_t)c->max_chunks) == hipSuccess;
    ok = ok && host_alloc(&c->h_order, T) == hipSuccess;
    ok = ok && host_alloc(&c->h_result, 1) == hipSuccess;
    ok = ok && hipHostGetDevicePointer(reinterpret_cast<void**>(&c->h_result_dev), c->h_result, 0) == hipSuccess;
    // (a pinned block may come back from an earlier context with that context's sequence number in it)
    if (ok) std::memset(c->h_result, 0, sizeof(ResultBlock));
    ok = ok && host_alloc(&c->h_result_dec, 1) == hipSuccess;
    ok = ok && hipHostGetDevicePointer(reinterpret_cast<void**>(&c->h_result_dec_dev), c->h_result_dec, 0) == hipSuccess;
    if (ok) std::memset(c->h_result_dec, 0, sizeof(ResultBlock));
    ok = ok && host_alloc(&c->h_dec, T) == hipSuccess;
    ok = ok && host_alloc(&c->h_state, T) == hipSuccess;
    if (ok) {
        int made = 0;
        for (; made < 2 * kNumStages; ++made)
            if (hipEventCreate(&c->ev[made]) != hipSuccess) break;
        if (made < 2 * kNumStages) {
            for (int i = 0; i < made; ++i) (void)hipEventDestroy(c->ev[i]);
            ok = false;
        } else {
            c->ev_ok = true;
        }
        if (ok && hipEventCreateWithFlags(&c->ev_result, hipEventDisableTiming) != hipSuccess) {
            c->ev_result = nullptr;
            ok = false;
        }
    }
    if (!ok) {
        (void)hipGetLastError();
        free_all(c);
        delete c;
        return SBC_EHIP;
    }
    *out = c;
    return SBC_OK;
}

int sbc_create(sbc_ctx** out, int device, int64_t max_total_elems, int max_tensors) {
    return create_context(out, device, max_total_elems, max_tensors, false);
}

int sbc_create_compact(sbc_ctx** out, int device, int64_t max_total_elems, int max_tensors) {
    return create_context(out, device, max_total_elems, max_tensors, true);
}

void sbc_destroy(sbc_ctx* c) {
    if (!c) return;
    DeviceGuard guard(c->device);
    free_all(c);
    delete c;
}

int sbc_set_option(sbc_ctx* c, int option, int value) {
    if (!c || c->pend.active) return SBC_EINVAL;      // not between sbc_compress_begin and sbc_compress_end
    switch (option) {
        case SBC_OPT_FORCE_EXACT_PATH:
            c->force_exact = value ? 1 : 0;
            c->hist_valid = false;
            c->cache_valid = false;                    // which tensors the streaming kernel finishes is part of the plan
            return SBC_OK;
        case SBC_OPT_CARRY_FILTER_KEYS:
            c->carry_keys = value ? 1 : 0; c->hist_valid = false; c->carry_backoff = c->carry_hold = 0;
            return SBC_OK;
        case SBC_OPT_FUSED_STEP:
            c->fused_step = value ? 1 : 0;
            c->hist_valid = false;
            c->cache_valid = false;                    // which tensors the streaming kernel finishes is part of the plan
            return SBC_OK;
        case SBC_OPT_SAMPLED_THRESHOLD:
            c->sampled = value ? 1 : 0;
            c->cache_valid = false;                    // the capacities of the plan depend on it
            c->dev_dec_valid = false;
            c->hist_valid = false;
            return SBC_OK;
        case SBC_OPT_DEFER_DECODE_STATUS:
            if (c->deferred_pending) return SBC_EINVAL;    // collect the outstanding status first
            c->defer_decode = value ? 1 : 0;
            return SBC_OK;
        case SBC_OPT_WIDE_MIN_KEPT:
            if (value < 0) return SBC_EINVAL;
            c->wide_min_kept = value ? (uint32_t)value : kWideMinKept;
            c->cache_valid = false;                    // which tensors are wide is part of both plans
            c->dev_dec_valid = false;
            return SBC_OK;
        default: return SBC_EINVAL;
    }
}

static int compress_begin(sbc_ctx* c, void* hip_stream, const float* const* dW, float* const* residual,
                          const int64_t* numel, int n_tensors, double p, void* msg, size_t msg_capacity,
                          bool wait_on_event) {
    if (!c || !dW || !residual || !numel || !msg || n_tensors <= 0 || !valid_p(p))
        return SBC_EINVAL;
    if (c->pend.active) return SBC_EINVAL;            // one step at a time per context
    if (((uintptr_t)msg & 7u) != 0) return SBC_EINVAL;
    if (n_tensors > c->max_tensors) return SBC_ECAPACITY;
    const int T = n_tensors;
    const int b = bstar_of(p);
    if (b > kMaxB) return SBC_EINVAL;
    c->last_ok = false;
    SBC_HOST_TS(0);

    // ---- plan: tensor table, chunk numbering, staging layout ----
    // Everything but the pointers depends only on the tensor sizes and p, and is kept from call
    // to call while those stay the same.  The tensor table itself (sizes, offsets and the
    // pointers) lives in one of kDescSlots device copies keyed by the pointer lists, so a caller
    // that alternates between a few sets of buffers uploads nothing in the steady state.
    uint64_t total = 0, chunks = 0, stage_words = 0, kept_total = 0, max_bound = 0, groups = 0, cand_total = 0;
    bool any_bitmap = false, all_inline = true;
    uint32_t scan_tiles = 1, bitmap_chunks_max = 0;
    // in the subsampled variant the keys must come from this call's sample
    const bool sampled = c->sampled != 0;
    const int force_exact = sampled ? 0 : c->force_exact;
    bool use_history = !sampled && c->hist_valid && !force_exact && !c->result_dirty && c->hist_p == p &&
                       c->hist_n.size() == (size_t)T;
    if (use_history)
        for (int t = 0; t < T; ++t) if ((int64_t)c->hist_n[t] != numel[t]) { use_history = false; break; }
    const bool sizes_same = c->cache_valid && c->cache_T == T && c->cache_p == p && c->cache_force_exact == force_exact &&
                            std::memcmp(c->cache_numel.data(), numel, sizeof(int64_t) * T) == 0;
    auto pointers_ok = [&](int t) -> bool {
        if (!dW[t] || !residual[t]) return false;
        const uintptr_t a = (uintptr_t)dW[t], r = (uintptr_t)residual[t];
        if ((a & 3u) || (r & 3u)) return false;
        const uintptr_t bytes = (uintptr_t)numel[t] * 4u;
        return !(a < r + bytes && r < a + bytes);     // dW must not overlap the residual
    };
    int slot = -1;
    if (sizes_same) {
        total = c->cache_total; chunks = c->cache_chunks; stage_words = c->cache_stage_words;
        kept_total = c->cache_kept_total; max_bound = c->cache_max_bound; any_bitmap = c->cache_any_bitmap;
        scan_tiles = c->cache_scan_tiles; bitmap_chunks_max = c->cache_bitmap_chunks_max;
        all_inline = c->cache_all_inline;
        for (int i = 0; i < kDescSlots; ++i) {
            const DescSlot& sl = c->slot[i];
            if (sl.valid && std::memcmp(sl.dW.data(), dW, sizeof(float*) * T) == 0 &&
                std::memcmp(sl.R.data(), residual, sizeof(float*) * T) == 0) { slot = i; break; }
        }
        if (slot < 0)
            for (int t = 0; t < T; ++t) if (!pointers_ok(t)) return SBC_EINVAL;
    } else {
        c->cache_valid = false;
        for (int i = 0; i < kDescSlots; ++i) c->slot[i].valid = false;
        if (c->plan.size() < (size_t)T) c->plan.resize(T);
        int n_wide = 0;
        uint64_t wide_max_n = 0;
        for (int t = 0; t < T; ++t) {
            const int64_t n = numel[t];
            if (n < 1 || n >= (int64_t)1 << 32) return SBC_EINVAL;
            if (!pointers_ok(t)) return SBC_EINVAL;
            TensorDesc d;
            std::memset(&d, 0, sizeof(d));
            d.n = (uint32_t)n;
            d.k = (uint32_t)kept_of(n, p);
            d.kcap = (uint32_t)cap_of(n, d.k, sampled);
            d.chunk0 = (uint32_t)chunks;
            d.nchunks = (uint32_t)((n + kChunk - 1) / kChunk);
            // compact: a quarter of the tensor per side (the whole budget of half an entry per entry), more
            // if k asks for it (then the budget may not do, and the call is refused below)
            d.cand_cap = c->compact ? (uint32_t)std::min<uint64_t>((uint64_t)n, std::max<uint64_t>((uint64_t)n / 4u, 4ull * d.kcap + 1024ull))
                                    : (uint32_t)n;
            d.cand_off = cand_total;
            cand_total += 2ull * d.cand_cap;
            d.stage_off = stage_words;
            const uint64_t bw = bound_words_of(n, d.kcap, b);
            if (bw >= (1ull << 32)) return SBC_ECAPACITY;
            d.bound_words = (uint32_t)bw;
            const bool fused = (d.kcap <= kFusedMaxK && bw <= kFusedMaxWords) ||
                               (d.kcap <= kFusedBigK && d.kcap < c->wide_min_kept && bw + 1u <= fused_sort_capacity(d.kcap));
            // finished inside the streaming kernel: exact mode, and few enough kept entries and stream
            // words for one workgroup's LDS (a one-chunk tensor: any k, encoded from a bitmap)
            const uint32_t n_groups = (d.nchunks + kGroupChunks - 1u) / kGroupChunks;
            const bool inl = c->fused_step && !sampled && !force_exact && fused && n_groups <= (uint32_t)kMaxGroups &&
                             (d.nchunks == 1u && d.n <= kSmallMaxN ? bw <= kSmallMaxWords
                                                                   : (d.kcap <= kInlineMaxK && bw <= kInlineMaxWords));
            d.flags = (fused ? kDescFused : 0u) | (sampled ? kDescSampled : 0u) | (inl ? kDescInline : 0u);
            all_inline = all_inline && inl;
            d.grp0 = (uint32_t)groups;
            if (inl) groups += n_groups;
            if (!fused && d.kcap >= c->wide_min_kept && n_wide < kMaxWide) {
                d.flags |= kDescWide;
                c->h_wide_ids[n_wide++] = (uint32_t)t;
                wide_max_n = std::max<uint64_t>(wide_max_n, (uint64_t)n);
            }
            d.kept_off = (uint32_t)kept_total;
            if (fused) kept_total += d.kcap; else any_bitmap = true;
            total += (uint64_t)n;
            chunks += d.nchunks;
            stage_words += bw;
            max_bound = std::max<uint64_t>(max_bound, bw);
            if (!fused) scan_tiles = std::max<uint32_t>(scan_tiles, (d.nchunks + kScanTile - 1u) / kScanTile);
            if (!fused) bitmap_chunks_max = std::max<uint32_t>(bitmap_chunks_max, d.nchunks);
            if (total > (uint64_t)c->max_elems || cand_total > c->cand_entries || chunks > c->max_chunks || kept_total > c->kept_cap ||
                stage_words > c->stage_cap || groups > c->max_groups)
                return SBC_ECAPACITY;
            c->plan[t] = d;
        }
        if (chunks >= (1ull << 31)) return SBC_ECAPACITY;
        c->n_wide = n_wide;
        // sweeps over a candidate list: enough workgroups to fill the chip, each with several rounds;
        // at least 128 even for short lists (a compute unit pulls a small share sooner than a large one,
        // and the tensor-wide step every workgroup repeats costs the same in all of them at once)
        c->wide_blocks = (uint32_t)std::min<uint64_t>(2048, std::max<uint64_t>(128, wide_max_n / 65536));
    }
    const size_t need = (size_t)(32 + 24ull * (unsigned)T + 4ull * stage_words);
    if (msg_capacity < need) return SBC_ECAPACITY;

    DeviceGuard guard(c->device);
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    // The previous step returned when its size was known, possibly before its last kernel had
    // ended: a step on another stream must not touch the context's scratch before that.
    if (c->last_T > 0 && c->last_stream != stream && hipStreamSynchronize(c->last_stream) != hipSuccess) {
        (void)hipGetLastError();
        return SBC_EHIP;
    }
    if (!sizes_same) {
        // tables that depend on the sizes only: tensors by decreasing size, chunk -> tensor
        c->plan_order.resize(T);
        std::iota(c->plan_order.begin(), c->plan_order.end(), 0u);
        std::stable_sort(c->plan_order.begin(), c->plan_order.end(),
                         [&](uint32_t x, uint32_t y) { return c->plan[x].n > c->plan[y].n; });
        for (int t = 0; t < T; ++t) {
            c->h_order[t] = c->plan_order[t];
            uint32_t* ct = c->h_chunk_tensor + c->plan[t].chunk0;
            for (uint32_t j = 0; j < c->plan[t].nchunks; ++j) ct[j] = (uint32_t)t;
        }
        // Order of the streaming kernel's workgroups: the one-chunk tensors it finishes on the spot
        // go first (their selection then runs beside the streaming of everything else), the others
        // follow by decreasing size, so that the tensors whose completion costs most complete early
        // and the last workgroups to finish belong to tensors with little left to do.
        if (c->fused_step) {
            uint64_t w = 0;
            for (int pass = 0; pass < 2; ++pass)
                for (int i = 0; i < T; ++i) {
                    const TensorDesc& d = c->plan[c->plan_order[i]];
                    const bool first = (d.flags & kDescInline) && d.nchunks == 1u && d.n <= kSmallMaxN;
                    if (first != (pass == 0)) continue;
                    for (uint32_t j = 0; j < d.nchunks; ++j) c->h_sched[w++] = make_uint2(d.chunk0 + j, c->plan_order[i]);
                }
            c->n_sched = (uint32_t)w;
        } else {
            // k_accumulate_filter: chunks in memory order.  Every workgroup reserves room in its
            // tensor's candidate lists with one atomic on one address, and those of one tensor queue
            // up there (about 20 ns each): a tensor of very many chunks gives each workgroup several
            // consecutive chunks, so that the queue is no longer what bounds the pass.
            uint64_t w = 0;
            for (int t = 0; t < T; ++t) {
                const TensorDesc& d = c->plan[t];
                const uint32_t m = std::min<uint32_t>(kMaxChunksPerWorkgroup, std::max<uint32_t>(1u, d.nchunks / 4096u));
                for (uint32_t j = 0; j < d.nchunks; j += m)
                    c->h_sched[w++] = make_uint2(d.chunk0 + j, (uint32_t)t | (std::min(m, d.nchunks - j) << 24));
            }
            c->n_sched = (uint32_t)w;
        }
        if (hipMemcpyAsync(c->d_order, c->h_order, sizeof(uint32_t) * T, hipMemcpyHostToDevice, stream) != hipSuccess ||
            hipMemcpyAsync(c->d_sched, c->h_sched, sizeof(uint2) * c->n_sched, hipMemcpyHostToDevice, stream) != hipSuccess ||
            hipMemcpyAsync(c->d_chunk_tensor, c->h_chunk_tensor, sizeof(uint32_t) * chunks, hipMemcpyHostToDevice, stream) != hipSuccess) {
            (void)hipGetLastError();
            return SBC_EHIP;
        }
        c->cache_numel.assign(numel, numel + T);
        c->cache_T = T; c->cache_p = p;
        c->cache_total = total; c->cache_chunks = chunks; c->cache_stage_words = stage_words;
        c->cache_kept_total = kept_total; c->cache_max_bound = max_bound; c->cache_any_bitmap = any_bitmap;
        c->cache_scan_tiles = scan_tiles; c->cache_bitmap_chunks_max = bitmap_chunks_max;
        c->cache_all_inline = all_inline; c->cache_force_exact = force_exact;
        // (cache_valid is set once this call has completed: the uploads above must have happened)
    }
    bool slot_is_new = false;
    if (slot < 0) {
        // the least recently used slot receives this call's table
        slot = 0;
        for (int i = 0; i < kDescSlots; ++i) {
            if (!c->slot[i].valid) { slot = i; break; }
            if (c->slot[i].stamp < c->slot[slot].stamp) slot = i;
        }
        DescSlot& sl = c->slot[slot];
        sl.valid = false;
        for (int t = 0; t < T; ++t) {
            c->h_desc[t] = c->plan[t];
            c->h_desc[t].dW = dW[t];
            c->h_desc[t].R = residual[t];
        }
        if (hipMemcpyAsync(c->d_desc + (size_t)slot * c->max_tensors, c->h_desc, sizeof(TensorDesc) * T,
                           hipMemcpyHostToDevice, stream) != hipSuccess) {
            (void)hipGetLastError();
            return SBC_EHIP;
        }
        sl.dW.assign(dW, dW + T);
        sl.R.assign(residual, residual + T);
        slot_is_new = true;
    }
    c->slot[slot].stamp = ++c->slot_clock;
    TensorDesc* const d_desc = c->d_desc + (size_t)slot * c->max_tensors;

    uint8_t* msg8 = static_cast<uint8_t*>(msg);
    const uint32_t n_chunks = (uint32_t)chunks;
    if (c->result_dirty) {                            // after an error, or on the first call
        hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, stream, reinterpret_cast<uint32_t*>(c->d_result),
                           (uint64_t)(2 * sizeof(ResultBlock) / 4));
        hipLaunchKernelGGL(k_zero_words, dim3(64), dim3(256), 0, stream, reinterpret_cast<uint32_t*>(c->d_group),
                           (uint64_t)c->max_groups * (sizeof(GroupState) / 4));
        // (the grid-wide kernels leave their histograms clean only if all of them have run)
        hipLaunchKernelGGL(k_zero_words, dim3(64), dim3(256), 0, stream, c->d_wide_hist, (uint64_t)kMaxWide * 2 * kWindow);
        hipLaunchKernelGGL(k_zero_words, dim3(256), dim3(256), 0, stream, c->d_wide_hist2, (uint64_t)kMaxWide * 2 * kWideRefine);
    }
    c->result_dirty = true;                           // until this call has completed normally
    c->hist_valid = false;
    ResultBlock* const res_now = c->d_result + c->result_idx;
    ResultBlock* const res_next = c->d_result + (c->result_idx ^ 1);
    c->result_idx ^= 1;
    const unsigned gather_y = (unsigned)std::min<uint64_t>(64, std::max<uint64_t>(1, (max_bound + 1023) / 1024));

    // what sbc_compress_end and the launch helpers need
    sbc_ctx::Pending& P = c->pend;
    P.stream = stream; P.T = T; P.b = b; P.p = p; P.slot = slot; P.slot_is_new = slot_is_new;
    P.force_exact = force_exact; P.use_history = use_history; P.sampled = sampled; P.any_bitmap = any_bitmap;
    P.all_inline = all_inline;
    for (int st = 0; st < kNumStages; ++st) P.timed[st] = false;
    P.res_now = res_now; P.res_next = res_next; P.d_desc = d_desc; P.msg8 = msg8;
    P.msg_capacity = msg_capacity; P.need = need; P.n_chunks = n_chunks; P.gather_y = gather_y; P.scan_tiles = scan_tiles; P.bitmap_chunks_max = bitmap_chunks_max;
    P.wait_on_event = wait_on_event;
    const int lvl = c->profile_level;
    bool* timed = P.timed;

    SBC_HOST_TS(1);
    // ---- fast path: [sample ->] accumulate + filter -> select (+ fused encode) -> gather ----
    // The sampling kernel is skipped when the previous call left filter keys for the same tensor
    // sizes and sparsity (its select kernel derives them from the exact thresholds it found).
    if (!use_history) {
        SBC_LAUNCH(kStSample, true, k_sample_thresholds, dim3(T), dim3(kSampleThreads), d_desc, c->d_state,
                   res_now, force_exact, sampled ? p : 0.0);
    }
    // 12 bytes per entry pass through; beyond about twice the 256 MiB last-level cache the update
    // is loaded with the nontemporal hint
    const int carry = c->carry_keys && !sampled && !force_exact ? 1 : 0;
    P.carry = carry;
    if (!c->fused_step) {
        if (total * 12ull > (512ull << 20)) {
            SBC_LAUNCH(kStAccumulate, true, k_accumulate_filter<true>, dim3(c->n_sched), dim3(kStreamThreads), d_desc,
                       c->d_sched, c->d_state, c->d_cand, c->d_bitmap, c->d_stage, res_now);
        } else {
            SBC_LAUNCH(kStAccumulate, true, k_accumulate_filter<false>, dim3(c->n_sched), dim3(kStreamThreads), d_desc,
                       c->d_sched, c->d_state, c->d_cand, c->d_bitmap, c->d_stage, res_now);
        }
    } else if (total * 12ull > (512ull << 20)) {
        SBC_LAUNCH(kStAccumulate, true, k_client_step<true>, dim3(n_chunks), dim3(kStepThreads), d_desc, c->d_sched,
                   c->d_state, c->d_cand, c->d_bitmap, c->d_stage, c->d_kept, c->d_group, b, carry, res_now);
    } else {
        SBC_LAUNCH(kStAccumulate, true, k_client_step<false>, dim3(n_chunks), dim3(kStepThreads), d_desc, c->d_sched,
                   c->d_state, c->d_cand, c->d_bitmap, c->d_stage, c->d_kept, c->d_group, b, carry, res_now);
    }
    if (!all_inline) {
        // the tensors the streaming kernel does not finish itself
        // (if every tensor goes through the grid-wide kernels, k_select has nothing to do unless one of
        // them is handed back: the last of those kernels then asks for the second pass below)
        const bool only_wide = c->n_wide == T;
        if (c->n_wide > 0) launch_wide_selection(c, only_wide);
        if (!only_wide) {
            SBC_LAUNCH(kStSelect, true, k_select, dim3(T), dim3(kSelThreads), d_desc, c->d_order,
                       c->d_state, c->d_cand, c->d_bitmap, c->d_stage, c->d_kept, b, 0, carry, res_now);
        }
    }
    launch_encode_and_gather(c, true);
    SBC_HOST_TS(2);
    const int rc = enqueue_result_copy(c);
    if (rc != SBC_OK) return rc;
    SBC_HOST_TS(3);
    P.active = true;
    return SBC_OK;
}

int sbc_compress_begin(sbc_ctx* c, void* hip_stream, const float* const* dW, float* const* residual,
                       const int64_t* numel, int n_tensors, double p, void* msg, size_t msg_capacity) {
    return compress_begin(c, hip_stream, dW, residual, numel, n_tensors, p, msg, msg_capacity, true);
}

int sbc_compress_end(sbc_ctx* c, size_t* msg_bytes) {
    if (!c || !msg_bytes || !c->pend.active) return SBC_EINVAL;
    sbc_ctx::Pending& P = c->pend;
    P.active = false;
    DeviceGuard guard(c->device);
    hipStream_t stream = P.stream;
    const int T = P.T, b = P.b;
    TensorDesc* const d_desc = P.d_desc;
    ResultBlock* const res_now = P.res_now;
    int rc = wait_result(c);
    SBC_HOST_TS(4);
    if (rc != SBC_OK) return rc;
    c->cache_valid = true;
    if (P.slot_is_new) c->slot[P.slot].valid = true;
    c->last_T = T;
    c->last_stream = stream;
    for (int st = 0; st < kNumStages; ++st) {
        if (!P.timed[st]) continue;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->ev[2 * st], c->ev[2 * st + 1]) == hipSuccess) {
            c->stage_ms[st] += (double)ms;
            c->stage_calls[st] += 1;
        } else {
            (void)hipGetLastError();
        }
    }
    uint32_t err = c->h_result->err;
    c->last_used_exact_path = false;
    c->last_used_wide = (err & kErrWide) != 0u;

    // ---- histogram path for the tensors whose filter kept fewer than k candidates ----
    // ---- second pass: the histogram route for the tensors whose filter kept fewer than k candidates,
    // and k_select for the tensors the streaming kernel left to it ----
    const uint32_t loose = err & (kErrLoose | kErrStaleKeys);
    c->last_deferred = (err & kErrDeferred) != 0u;
    if ((err & (kErrPrefilter | kErrDeferred)) && !(err & (kErrInternal | kErrNonFinite | kErrOverflow))) {
        c->last_used_exact_path = (err & kErrPrefilter) != 0u;
        hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, stream, reinterpret_cast<uint32_t*>(res_now),
                           (uint64_t)(sizeof(ResultBlock) / 4));
        if (err & kErrPrefilter) {
            const uint32_t hist_words = (uint32_t)T * kL1Bins;
            hipLaunchKernelGGL(k_zero_words, dim3((hist_words + 2047) / 2048), dim3(256), 0, stream, c->d_hist,
                               (uint64_t)hist_words);
            hipLaunchKernelGGL(k_hist_flagged, dim3(P.n_chunks), dim3(kStreamThreads), 0, stream, d_desc,
                               c->d_chunk_tensor, c->d_state, c->d_hist);
            hipLaunchKernelGGL(k_pick_bins, dim3(T), dim3(256), 0, stream, d_desc, c->d_hist, c->d_state, res_now);
            hipLaunchKernelGGL(k_extract, dim3(P.n_chunks), dim3(kStreamThreads), 0, stream, d_desc,
                               c->d_chunk_tensor, c->d_state, c->d_cand, res_now);
        }
        hipLaunchKernelGGL(k_select, dim3(T), dim3(kSelThreads), 0, stream, d_desc, c->d_order,
                           c->d_state, c->d_cand, c->d_bitmap, c->d_stage, c->d_kept, b, 1, P.carry, res_now);
        launch_encode_and_gather(c, false);
        rc = enqueue_result_copy(c);
        if (rc == SBC_OK) rc = wait_result(c);
        if (rc != SBC_OK) return rc;
        err = c->h_result->err | loose;
        if (err & (kErrPrefilter | kErrDeferred)) return SBC_EINTERNAL;
    }
    const int status = status_of_err(err);
    if (status != SBC_OK) return status;
    if (c->h_result->msg_bytes > P.need) return SBC_EINTERNAL;
    *msg_bytes = (size_t)c->h_result->msg_bytes;
    c->last_ok = true;
    c->last_used_history = P.use_history;
    c->last_loose = (err & kErrLoose) != 0u;
    c->result_dirty = false;
    // the next call may start from this call's thresholds unless they proved unhelpful
    // (a sampled call with long lists says nothing about the keys it leaves: those go by rank)
    const bool flood = (err & kErrLoose) && P.use_history;
    c->hist_valid = c->carry_keys && !P.sampled && !P.force_exact && !c->last_used_exact_path && !flood;
    // While the data still grows from call to call (the first rounds of a run, when the residual
    // builds up) carried keys let floods of candidates pass.  After such a call the next calls
    // sample, and each of their samples also tells whether the keys the call before it left would
    // have held on its data (kErrStaleKeys if not): sampling goes on until they would (for at most
    // 64 calls in a row, then a carried call is tried whatever the samples say).  Should carried
    // calls flood again and again all the same, each flood doubles the number of sampled calls
    // that follow it at the least; a carried call that goes well ends that.
    if (flood) {
        c->carry_backoff = std::min(64, std::max(1, 2 * c->carry_backoff));
        c->carry_hold = c->carry_backoff;
        c->carry_stale_run = 0;
    } else if (P.use_history) {
        c->carry_backoff = 0;
    } else if (c->carry_hold > 1) {
        --c->carry_hold;
        c->hist_valid = false;
    } else if (c->carry_hold == 1) {
        if ((err & kErrStaleKeys) && ++c->carry_stale_run <= 64) {
            c->hist_valid = false;
        } else {
            c->carry_hold = 0;
            c->carry_stale_run = 0;
        }
    }
    if (c->hist_valid) {
        c->hist_p = P.p;
        c->hist_n.resize(T);
        for (int t = 0; t < T; ++t) c->hist_n[t] = c->plan[t].n;
    }
    return SBC_OK;
}

int sbc_compress(sbc_ctx* c, void* hip_stream, const float* const* dW, float* const* residual,
                 const int64_t* numel, int n_tensors, double p, void* msg, size_t msg_capacity,
                 size_t* msg_bytes) {
    if (!msg_bytes) return SBC_EINVAL;
    const int rc = compress_begin(c, hip_stream, dW, residual, numel, n_tensors, p, msg, msg_capacity, false);
    if (rc != SBC_OK) return rc;
    return sbc_compress_end(c, msg_bytes);
}

int sbc_decompress_accumulate(sbc_ctx* c, void* hip_stream, const void* msg, size_t msg_bytes,
                              const int64_t* numel, int n_tensors, double p, float scale,
                              float* const* out) {
    if (!c || !msg || !numel || !out || n_tensors <= 0 || !valid_p(p)) return SBC_EINVAL;
    if (((uintptr_t)msg & 7u) != 0) return SBC_EINVAL;
    if (n_tensors > c->max_tensors) return SBC_ECAPACITY;
    const int T = n_tensors;
    const int b = bstar_of(p);
    if (b > kMaxB) return SBC_EINVAL;
    SBC_HOST_TS(8);
    if (msg_bytes < 32 + 24ull * (unsigned)T) return SBC_ECORRUPT;
    bool same = c->dev_dec_valid && c->dev_dec_T == T && c->dec_p == p;
    for (int t = 0; t < T; ++t) {
        if (numel[t] < 1 || numel[t] >= (int64_t)1 << 32 || !out[t] || ((uintptr_t)out[t] & 3u)) return SBC_EINVAL;
        if (same && (c->h_dec[t].out != out[t] || c->h_dec[t].n != (uint32_t)numel[t])) same = false;
    }
    DeviceGuard guard(c->device);
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    const bool deferred = c->defer_decode != 0;
    if (!same && c->deferred_pending) {
        // the pinned tables below may still be read by an upload of an earlier deferred call
        if (hipStreamSynchronize(stream) != hipSuccess) { (void)hipGetLastError(); return SBC_EHIP; }
    }
    if (!same) {
        // Streams of tensors that keep very many entries are decoded tile by tile by many
        // workgroups, as far as the scratch arrays reach; all others by one workgroup each.
        int n_wide = 0;
        uint64_t segs = 0, tiles = 0;
        uint32_t n_blocks = 0, extra = 0;
        for (int t = 0; t < T; ++t) {
            c->h_dec[t].out = out[t]; c->h_dec[t].n = (uint32_t)numel[t]; c->h_dec[t].wide = 0u;
            // (a context that expects messages of the subsampled variant reserves for its cap)
            const int64_t k = cap_of(numel[t], kept_of(numel[t], p), c->sampled != 0);
            // One workgroup decodes a stream; the scattered updates of a stream with many codes are
            // shared among several workgroups that each decode it (a compute unit sustains only so
            // many scattered accesses at a time, and decoding again costs no more time than once).
            uint32_t shares = (uint32_t)std::min<int64_t>(kDecShareMax, std::max<int64_t>(1, k / kDecSharePer));
            if (extra + shares - 1u > kMaxDecExtra) shares = 1u;
            extra += shares - 1u;
            for (uint32_t sh = 0; sh < shares; ++sh) c->h_dec_blocks[n_blocks++] = make_uint2((uint32_t)t, sh | (shares << 16));
            if (b > kPackedMaxB || (uint64_t)k < (uint64_t)c->wide_min_kept || n_wide >= kMaxWideDec) continue;
            const uint64_t max_seg = (bound_words_of(numel[t], (uint32_t)k, b) + 1) / 2;
            const uint64_t max_tiles = (max_seg + kDecThreads - 1) / kDecThreads;
            if (max_tiles == 0 || max_tiles >= (1ull << 31) || segs + max_tiles * kDecThreads > c->dec_seg_cap ||
                tiles + max_tiles > c->dec_tile_cap)
                continue;
            DecWide& w = c->h_dec_wide[n_wide++];
            w.t = (uint32_t)t; w.tile0 = (uint32_t)tiles; w.max_tiles = (uint32_t)max_tiles; w.pad = 0u; w.seg0 = segs;
            c->h_dec[t].wide = 1u;
            n_blocks -= shares - 1u; extra -= shares - 1u;     // its workgroup of this kernel only returns
            c->h_dec_blocks[n_blocks - 1u] = make_uint2((uint32_t)t, 1u << 16);
            segs += max_tiles * kDecThreads; tiles += max_tiles;
        }
        c->n_dec_wide = n_wide; c->dec_tiles = (uint32_t)tiles; c->dec_p = p;
        c->n_dec_blocks = n_blocks;
        c->dev_dec_valid = false;
        if (hipMemcpyAsync(c->d_dec, c->h_dec, sizeof(DecDesc) * T, hipMemcpyHostToDevice, stream) != hipSuccess ||
            hipMemcpyAsync(c->d_dec_blocks, c->h_dec_blocks, sizeof(uint2) * n_blocks, hipMemcpyHostToDevice, stream) != hipSuccess ||
            (n_wide > 0 && hipMemcpyAsync(c->d_dec_wide, c->h_dec_wide, sizeof(DecWide) * n_wide, hipMemcpyHostToDevice, stream) != hipSuccess)) {
            (void)hipGetLastError();
            return SBC_EHIP;
        }
        c->dev_dec_T = T;
    }
    // the decode kernel leaves the other of its two result blocks clean for the next call; calls
    // whose status is deferred all raise their error bits in block [4] and clear the spare
    ResultBlock* res_dec;
    ResultBlock* res_dec_next;
    if (deferred) {
        if (c->deferred_dirty) {
            hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, stream, reinterpret_cast<uint32_t*>(c->d_result + 4),
                               (uint64_t)(sizeof(ResultBlock) / 4));
            c->deferred_dirty = false;
        }
        res_dec = c->d_result + 4;
        res_dec_next = c->d_result + 5;
    } else {
        if (c->dec_result_dirty) {                    // after an error, or on the first call
            hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, stream, reinterpret_cast<uint32_t*>(c->d_result + 2),
                               (uint64_t)(2 * sizeof(ResultBlock) / 4));
        }
        c->dec_result_dirty = true;                   // until this call has completed normally
        res_dec = c->d_result + 2 + c->dec_result_idx;
        res_dec_next = c->d_result + 2 + (c->dec_result_idx ^ 1);
        c->dec_result_idx ^= 1;
    }
    SBC_HOST_TS(9);
    hipLaunchKernelGGL(k_decode_accumulate, dim3(c->n_dec_blocks), dim3(kDecThreads), 0, stream,
                       static_cast<const uint8_t*>(msg), (unsigned long long)msg_bytes, c->d_dec, c->d_dec_blocks, T, b, scale,
                       res_dec, res_dec_next);
    if (c->n_dec_wide > 0) {
        const uint8_t* m8 = static_cast<const uint8_t*>(msg);
        const unsigned long long mb = (unsigned long long)msg_bytes;
        const dim3 tiles(c->dec_tiles);
        hipLaunchKernelGGL(k_dec_tile_fn, tiles, dim3(kDecThreads), 0, stream, m8, mb, c->d_dec, c->d_dec_wide,
                           c->n_dec_wide, T, b, c->d_seg_fn, c->d_tile_fn, res_dec);
        hipLaunchKernelGGL(k_dec_tile_sums, tiles, dim3(kDecThreads), 0, stream, m8, mb, c->d_dec, c->d_dec_wide,
                           c->n_dec_wide, T, b, c->d_seg_fn, c->d_tile_fn, c->d_tile_entry, c->d_seg_pack,
                           c->d_tile_sum, res_dec);
        hipLaunchKernelGGL(k_dec_tile_place, tiles, dim3(kDecThreads), 0, stream, m8, mb, c->d_dec, c->d_dec_wide,
                           c->n_dec_wide, T, b, scale, c->d_seg_fn, c->d_tile_entry, c->d_seg_pack, c->d_tile_sum,
                           res_dec);
    }
    SBC_HOST_TS(10);
    if (hipGetLastError() != hipSuccess) return SBC_EHIP;
    if (deferred) {
        // (the uploads above precede every later kernel on this stream)
        c->deferred_pending = true;
        c->dev_dec_valid = true;
        return SBC_OK;
    }
    // the status goes to pinned host memory by a small dispatch, and the call looks for it there (as
    // the client step does): it returns when the status is known; `out` is complete for everything
    // enqueued on the stream afterwards
    hipLaunchKernelGGL(k_publish, dim3(1), dim3(64), 0, stream, c->h_result_dec_dev, res_dec, ++c->dec_seq);
    if (hipGetLastError() != hipSuccess) return SBC_EHIP;
    if (!result_arrived(c->h_result_dec, c->dec_seq) && hipStreamSynchronize(stream) != hipSuccess) {
        (void)hipGetLastError();
        return SBC_EHIP;
    }
    SBC_HOST_TS(11);
    c->dev_dec_valid = true;
    if (c->h_result_dec->err == 0u) c->dec_result_dirty = false;
    return status_of_err(c->h_result_dec->err);
}

int sbc_decode_status(sbc_ctx* c, void* hip_stream) {
    if (!c) return SBC_EINVAL;
    if (!c->deferred_pending) return SBC_OK;
    DeviceGuard guard(c->device);
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    c->deferred_pending = false;
    c->deferred_dirty = true;
    if (hipMemcpyAsync(c->h_result_dec, c->d_result + 4, sizeof(ResultBlock), hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess) {
        (void)hipGetLastError();
        return SBC_EHIP;
    }
    return status_of_err(c->h_result_dec->err);
}

int sbc_copy_baseline(void* hip_stream, void* dst, const void* src, size_t bytes) {
    if (!dst || !src || bytes == 0 || (bytes & 15u) || (((uintptr_t)dst | (uintptr_t)src) & 15u)) return SBC_EINVAL;
    const uint64_t n16 = bytes / 16;
    const uint64_t per_block = 256ull * 8ull;
    const uint64_t blocks = (n16 + per_block - 1) / per_block;
    if (blocks >= (1ull << 31)) return SBC_EINVAL;
    hipLaunchKernelGGL(k_copy_baseline, dim3((unsigned)blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                       static_cast<uint4*>(dst), static_cast<const uint4*>(src), n16);
    return hipGetLastError() == hipSuccess ? SBC_OK : SBC_EHIP;
}

int sbc_profile_enable(sbc_ctx* c, int level) {
    if (!c || level < 0 || level > 2) return SBC_EINVAL;
    c->profile_level = level;
    for (int st = 0; st < kNumStages; ++st) { c->stage_ms[st] = 0.0; c->stage_calls[st] = 0; }
    return SBC_OK;
}

int sbc_profile_level(sbc_ctx* c, int level) {
    if (!c || level < 0 || level > 2) return SBC_EINVAL;
    c->profile_level = level;
    return SBC_OK;
}

int sbc_profile_read(sbc_ctx* c, int stage, const char** name, double* total_ms, int64_t* calls) {
    if (!c || stage < 0 || stage >= kNumStages) return SBC_EINVAL;
    // (the streaming pass is one of two kernels, by SBC_OPT_FUSED_STEP)
    if (name) *name = (stage == kStAccumulate && !c->fused_step) ? "k_accumulate_filter" : kStageNames[stage];
    if (total_ms) *total_ms = c->stage_ms[stage];
    if (calls) *calls = c->stage_calls[stage];
    return SBC_OK;
}

int sbc_last_tensor_stats(sbc_ctx* c, int tensor, double* mu_pos, double* mu_neg, int* side,
                          int64_t* nnz, int64_t* bit_len) {
    if (!c || !c->last_ok || tensor < 0 || tensor >= c->last_T) return SBC_EINVAL;
    DeviceGuard guard(c->device);
    if (hipStreamSynchronize(c->last_stream) != hipSuccess ||
        hipMemcpy(c->h_state, c->d_state + tensor, sizeof(TensorState), hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return SBC_EHIP;
    }
    const TensorState& s = c->h_state[0];
    if (s.kc[0] == 0u || s.kc[1] == 0u) return SBC_EINTERNAL;
    if (mu_pos) *mu_pos = s.S[0] / (double)s.kc[0];
    if (mu_neg) *mu_neg = s.S[1] / (double)s.kc[1];
    if (side) *side = s.side;
    if (nnz) *nnz = (int64_t)s.nnz;
    if (bit_len) *bit_len = (int64_t)s.bit_len;
    return SBC_OK;
}

int sbc_last_candidates(sbc_ctx* c, int tensor, int64_t* positive, int64_t* negative) {
    if (!c || !c->last_ok || tensor < 0 || tensor >= c->last_T) return SBC_EINVAL;
    DeviceGuard guard(c->device);
    if (hipStreamSynchronize(c->last_stream) != hipSuccess ||
        hipMemcpy(c->h_state, c->d_state + tensor, sizeof(TensorState), hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return SBC_EHIP;
    }
    if (positive) *positive = (int64_t)c->h_state[0].cand_seen[0];
    if (negative) *negative = (int64_t)c->h_state[0].cand_seen[1];
    return SBC_OK;
}

int sbc_last_mask(sbc_ctx* c, int tensor, uint32_t* mask_words, size_t n_words) {
    if (!c || !c->last_ok || !mask_words || tensor < 0 || tensor >= c->last_T) return SBC_EINVAL;
    const TensorDesc& d = c->plan[tensor];
    if (n_words != ((size_t)d.n + 31) / 32) return SBC_EINVAL;
    DeviceGuard guard(c->device);
    if (hipStreamSynchronize(c->last_stream) != hipSuccess) { (void)hipGetLastError(); return SBC_EHIP; }
    if (d.flags & kDescFused) {
        // the select kernel left the sorted kept indices in scratch
        if (hipMemcpy(c->h_state, c->d_state + tensor, sizeof(TensorState), hipMemcpyDeviceToHost) != hipSuccess) {
            (void)hipGetLastError();
            return SBC_EHIP;
        }
        const uint32_t nnz = c->h_state[0].nnz;
        if (nnz > d.kcap) return SBC_EINTERNAL;
        std::vector<uint32_t> idx(nnz);
        if (hipMemcpy(idx.data(), c->d_kept + d.kept_off, (size_t)nnz * 4, hipMemcpyDeviceToHost) != hipSuccess) {
            (void)hipGetLastError();
            return SBC_EHIP;
        }
        std::memset(mask_words, 0, n_words * 4);
        for (uint32_t j : idx) {
            if (j >= d.n) return SBC_EINTERNAL;
            mask_words[j >> 5] |= 1u << (j & 31u);
        }
        return SBC_OK;
    }
    if (hipMemcpy(mask_words, c->d_bitmap + (size_t)d.chunk0 * kChunkWords, n_words * 4, hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return SBC_EHIP;
    }
    return SBC_OK;
}

int sbc_decompress_accumulate_noalloc(int device, void* hip_stream, const void* msg, size_t msg_bytes,
                                      const int64_t* numel, int n_tensors, double p, float scale,
                                      float* const* out, int32_t* status) {
    if (!msg || !numel || !out || !status || n_tensors <= 0 || !valid_p(p) || device < 0) return SBC_EINVAL;
    if ((((uintptr_t)msg) & 7u) != 0 || (((uintptr_t)status) & 3u) != 0) return SBC_EINVAL;
    if (n_tensors > SBC_NOALLOC_MAX_TENSORS || device >= kNoAllocMaxDevices) return SBC_ECAPACITY;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess) { (void)hipGetLastError(); return SBC_EHIP; }
    if (device >= n_dev) return SBC_EINVAL;
    const int T = n_tensors;
    const int b = bstar_of(p);
    if (b > kMaxB) return SBC_EINVAL;
    if (msg_bytes < 32 + 24ull * (unsigned)T) return SBC_ECORRUPT;
    NoAllocArgs a;
    std::memset(&a, 0, sizeof(a));
    uint32_t n_blocks = 0, extra = 0;
    for (int t = 0; t < T; ++t) {
        if (numel[t] < 1 || numel[t] >= (int64_t)1 << 32 || !out[t] || ((uintptr_t)out[t] & 3u)) return SBC_EINVAL;
        const int64_t k = kept_of(numel[t], p);
        uint32_t shares = (uint32_t)std::min<int64_t>(kDecShareMax, std::max<int64_t>(1, k / kDecSharePer));
        if (extra + shares - 1u > kMaxDecExtra) shares = 1u;
        extra += shares - 1u;
        a.out[t] = out[t]; a.n[t] = (uint32_t)numel[t];
        a.first_block[t] = (uint16_t)n_blocks; a.shares[t] = (uint8_t)shares;
        n_blocks += shares;
    }
    DeviceGuard guard(device);
    NoAllocScratch* const s = noalloc_scratch_of(device);
    if (!s) return SBC_EHIP;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(k_noalloc_setup, dim3(1), dim3(256), 0, stream, s, a, T);
    hipLaunchKernelGGL(k_decode_accumulate, dim3(n_blocks), dim3(kDecThreads), 0, stream,
                       static_cast<const uint8_t*>(msg), (unsigned long long)msg_bytes, s->dec, s->blocks, T, b, scale,
                       &s->result[0], &s->result[1]);
    hipLaunchKernelGGL(k_noalloc_finish, dim3(1), dim3(64), 0, stream, s, status);
    if (hipGetLastError() != hipSuccess) return SBC_EHIP;
    return SBC_OK;
}

#ifdef SBC_PHASE_TIMING
int sbc_debug_host_times(double* out) { for (int i = 0; i < 16; ++i) out[i] = g_host_ts[i]; return 0; }
// tuning builds only: copies the phase clock tables (3 x 1024 x 16 u64) to host memory
int sbc_debug_phase_clocks(unsigned long long* out) {
    return hipMemcpyFromSymbol(out, HIP_SYMBOL(sbc::g_phase_clock), sizeof(unsigned long long) * 3 * 1024 * 16) == hipSuccess ? 0 : -3;
}
int sbc_debug_step_clocks(unsigned long long* out) {
    return hipMemcpyFromSymbol(out, HIP_SYMBOL(sbc::g_step_clock), sizeof(unsigned long long) * 16384 * 8) == hipSuccess ? 0 : -3;
}
#endif

int sbc_last_route(sbc_ctx* c) {
    if (!c || !c->last_ok) return SBC_EINVAL;
    return (c->last_used_history ? SBC_ROUTE_CARRIED_KEYS : 0) | (c->last_used_exact_path ? SBC_ROUTE_HISTOGRAM : 0) |
           (c->last_used_wide ? SBC_ROUTE_WIDE : 0) | (c->last_loose ? SBC_ROUTE_LOOSE_KEYS : 0) |
           (c->last_deferred ? SBC_ROUTE_TAKEN_OVER : 0);
}

}  // extern "C"
