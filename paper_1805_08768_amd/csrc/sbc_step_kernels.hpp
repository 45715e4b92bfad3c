// The client step as one streaming kernel.
//
// k_client_step runs one workgroup per chunk of 8192 entries, in an order the host chooses
// (a schedule table: one-chunk tensors first, then the others by decreasing size):
//   * A = R + dW (Alg. 1, client line dW_i <- R_i + local update); entries at or beyond a side's
//     filter key are collected per wavefront with ballots (no LDS atomics) and appended to the
//     tensor's candidate lists; A is stored over R last, so that the only stores the workgroup
//     ever waits for are its few candidate entries;
//   * a tensor of one chunk is finished on the spot from the registers: it needs no filter key,
//     no candidate list and no other kernel;
//   * for the other tensors flagged kDescInline every workgroup, once its candidate stores have
//     completed, counts itself in; the workgroup that completes the count is the last of its
//     tensor and runs Alg. 2 and Alg. 3 for it from the candidate lists, while the workgroups of
//     other tensors keep streaming.  Nothing ever waits for another workgroup.
// Finishing a tensor (select_tensor): a histogram of the side keys over a window that spans the
// entries' own range finds the bin of the k-th most extreme entry of each side; the bin's
// few entries are ranked against each other by (key descending, index ascending), which gives the
// threshold key and the last index kept among equal values; exact integer sums; side and mean;
// the kept indices are sorted (from a bitmap for a one-chunk tensor, by buckets of leading index
// bits otherwise) and Golomb-coded in LDS.  Tie-heavy data, where a bin is too crowded to
// rank, takes a bisection over the key bits instead.
// Data that one workgroup writes and another reads inside this kernel (candidate entries, the
// counters) moves with device-scope atomic stores, loads and read-modify-writes only; everything
// else a finishing workgroup writes (stream words, kept indices, state) is read by the next
// kernel.  The residual update R[j] = A[j] - mu at the kept entries is left to that kernel too
// (k_finish_message): A[j] was stored by another workgroup through another L2, and two plain
// stores to one line from two L2s inside one kernel have no order.
//
// k_finish_message assembles the message, applies the residual update of the tensors finished
// here, resets the per-tensor counters and writes the call's result block to pinned host memory.
#pragma once

#include "sbc_device.hpp"
#include "sbc_select_kernels.hpp"

namespace sbc {

constexpr int kStepThreads = 256;
constexpr int kStepWaves = kStepThreads / 64;
constexpr int kSlots = kChunk / kStepThreads;            // 32 entries per thread
constexpr int kWaveQueue = 128;                          // candidates per side a wavefront can queue in LDS
constexpr uint32_t kInlineMaxK = 4224;                   // kept entries a finishing workgroup can sort and encode
constexpr uint32_t kInlineMaxWords = kFusedMaxWords;     // (k_select must be able to take the tensor over)
constexpr int kInlineBuckets = 1024;                     // index sort: buckets by leading index bits
constexpr uint32_t kSmallMaxWords = 512;                 // stream words of a one-chunk tensor (at most 1.3 bits per entry)
constexpr uint32_t kInlineMaxCand = 32768;               // longest list a finishing workgroup takes on
constexpr int kStepWindow = 1024;                        // bins of the side-key histogram
constexpr uint32_t kStepRankMax = 256;                   // a threshold bin of up to this many entries is ranked directly
constexpr uint32_t kSmallMaxN = 6144;                    // a one-chunk tensor of up to this size is finished from LDS
// LDS of a workgroup, in words: region A holds the histogram and the threshold bin, later the
// per-exponent sums, the sort arrays of a tensor that keeps few entries, or the bitmap and stream
// of a one-chunk tensor; region B holds a tensor's entries (a one-chunk tensor's keys, or the
// candidate lists when they fit).  The sort arrays of a tensor whose lists stay in memory take
// both regions, the streaming phase's queues and the keys of a chunk whose queues overflowed
// start at word 0.
constexpr uint32_t kLdsA = 2 * kStepWindow + 2 * 2 * kStepRankMax;       // 3072
constexpr uint32_t kLdsWords = 9600;
constexpr uint32_t kLdsB = kLdsWords - kLdsA;                             // 6528
static_assert(kSmallMaxN <= kLdsB, "a one-chunk tensor's keys fit region B");
static_assert(kInlineBuckets + 2 * kInlineMaxK + 2 <= kLdsWords, "sort arrays of the largest tensor fit");
static_assert(kChunk <= kLdsWords, "a chunk's keys fit");
static_assert(kChunkWords + kSmallMaxWords + 2 <= kLdsA && 1024 <= kLdsA, "small-tensor encoder and exponent sums fit region A");
static_assert(kInlineMaxWords <= kInlineMaxK, "the stream words reuse the grouping array");

// ---- device-scope accesses for data that crosses workgroups inside one kernel ----
__device__ __forceinline__ void store_shared_u64(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long load_shared_u64(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_cand(uint2* p, uint32_t key, uint32_t idx) {
    store_shared_u64(reinterpret_cast<unsigned long long*>(p), (unsigned long long)key | ((unsigned long long)idx << 32));
}
__device__ __forceinline__ uint2 load_cand(const uint2* p) {
    const unsigned long long v = load_shared_u64(reinterpret_cast<const unsigned long long*>(p));
    return make_uint2((uint32_t)v, (uint32_t)(v >> 32));
}
// every memory operation this wavefront has issued has completed
__device__ __forceinline__ void wait_all_memory() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory"); }

__device__ __forceinline__ uint32_t lane_rank(unsigned long long mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

struct StepShared {
    uint32_t lds[kLdsWords];
    unsigned long long red[2][kStepWaves];               // block sums, double buffered
    unsigned long long scratch64[kStepWaves];
    uint32_t scratch32[kStepWaves];
    uint32_t res[2][8];
    uint32_t ext[kStepWaves][4];                         // per wavefront: largest and smallest key of each side
    uint32_t wcnt[kStepWaves][2];                        // candidates queued per wavefront and side
    uint32_t base[2];
    uint32_t bcnt[2];
    uint32_t pick[2][2];
    uint32_t flag;
    double S[2];
    __device__ __forceinline__ uint2* wq(int wave, int side) { return reinterpret_cast<uint2*>(lds) + (wave * 2 + side) * kWaveQueue; }
    __device__ __forceinline__ uint32_t (*whist())[kStepWindow] { return reinterpret_cast<uint32_t (*)[kStepWindow]>(lds); }
    __device__ __forceinline__ uint2* bucket(int side) { return reinterpret_cast<uint2*>(lds + 2 * kStepWindow) + side * kStepRankMax; }
    __device__ __forceinline__ long long* acc(int side) { return reinterpret_cast<long long*>(lds) + side * 256; }
    __device__ __forceinline__ uint32_t* region_b() { return lds + kLdsA; }
};
static_assert(kStepWaves * 2 * kWaveQueue * 2 <= kLdsWords, "queues fit");

// Sum over the workgroup of one value per thread.  One barrier; the slots alternate so that the
// next call may write while slow wavefronts still read.
__device__ __forceinline__ unsigned long long block_sum(StepShared& sh, int& parity, unsigned long long v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    if ((threadIdx.x & 63) == 0) sh.red[parity][threadIdx.x >> 6] = v;
    __syncthreads();
    unsigned long long s = 0ull;
#pragma unroll
    for (int w = 0; w < kStepWaves; ++w) s += sh.red[parity][w];
    parity ^= 1;
    return s;
}

// ---- where a finishing workgroup finds the entries of its tensor ----
// for_each<S>(f): f(side key, index) for every entry of side S (0: positive, 1: negative, in its
// complemented key space) that this thread owns.

// candidate lists staged in LDS (region B): positive side first, then the negative side
struct LdsLists {
    const uint2* e[2];
    uint32_t cnt[2];
    template <int S, typename F>
    __device__ __forceinline__ void for_each(F f) const {
        const uint2* p = e[S];
        const uint32_t n = cnt[S];
#pragma unroll 4
        for (uint32_t i = threadIdx.x; i < n; i += kStepThreads) { const uint2 x = p[i]; f(x.x, x.y); }
    }
};

// candidate lists too long for LDS: read from memory in every sweep
struct MemLists {
    const uint2* g[2];
    uint32_t cnt[2];
    template <int S, typename F>
    __device__ __forceinline__ void for_each(F f) const {
        const uint2* __restrict__ p = g[S];
        const uint32_t n = cnt[S];
        for (uint32_t i0 = threadIdx.x; i0 < n; i0 += 8u * kStepThreads) {
            uint2 e[8];
#pragma unroll
            for (uint32_t u = 0; u < 8u; ++u) { const uint32_t i = i0 + u * kStepThreads; e[u] = load_cand(p + (i < n ? i : 0u)); }
#pragma unroll
            for (uint32_t u = 0; u < 8u; ++u) if (i0 + u * kStepThreads < n) f(e[u].x, e[u].y);
        }
    }
};

// a whole one-chunk tensor in LDS (region B): keys[i] is the plain key of entry i
struct LdsChunk {
    const uint32_t* keys;
    uint32_t n;
    template <int S, typename F>
    __device__ __forceinline__ void for_each(F f) const {
#pragma unroll 4
        for (uint32_t i = threadIdx.x; i < n; i += kStepThreads) { const uint32_t k = keys[i]; f(S ? ~k : k, i); }
    }
};

// ---- tie-heavy data: bisection instead of the histogram ----
// The exact need[s]-th largest key of each side by bisection over the 32 key bits, one count per
// bit; then, if fewer than all entries equal to it are kept, the index of the last one kept by
// bisection over the index bits.  Requires 1 <= need[s] <= entries of side s.  Contains barriers.
template <typename Src>
__device__ __forceinline__ void bisect_thresholds(StepShared& sh, int& parity, const Src& src, const uint32_t (&need)[2],
                                                  uint32_t (&tau)[2], uint32_t (&itau)[2]) {
    auto count_ge = [&](uint32_t tp, uint32_t tn) -> unsigned long long {
        uint32_t cp = 0u, cn = 0u;
        src.template for_each<0>([&](uint32_t key, uint32_t) { cp += key >= tp ? 1u : 0u; });
        src.template for_each<1>([&](uint32_t key, uint32_t) { cn += key >= tn ? 1u : 0u; });
        return block_sum(sh, parity, (unsigned long long)cp | ((unsigned long long)cn << 32));
    };
    uint32_t pre_p = 0u, pre_n = 0u;
#pragma nounroll
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t tp = pre_p | (1u << bit), tn = pre_n | (1u << bit);
        const unsigned long long tot = count_ge(tp, tn);
        if ((uint32_t)tot >= need[0]) pre_p = tp;
        if ((uint32_t)(tot >> 32) >= need[1]) pre_n = tn;
    }
    tau[0] = pre_p; tau[1] = pre_n;
    // (a key of 0xFFFFFFFF is a NaN pattern: the call fails as non-finite whatever is counted here)
    const unsigned long long ge = count_ge(pre_p, pre_n);
    const unsigned long long g = count_ge(pre_p == 0xFFFFFFFFu ? pre_p : pre_p + 1u, pre_n == 0xFFFFFFFFu ? pre_n : pre_n + 1u);
    const uint32_t gt[2] = {pre_p == 0xFFFFFFFFu ? 0u : (uint32_t)g, pre_n == 0xFFFFFFFFu ? 0u : (uint32_t)(g >> 32)};
    const uint32_t eq[2] = {(uint32_t)ge - gt[0], (uint32_t)(ge >> 32) - gt[1]};
    const uint32_t r[2] = {need[0] - gt[0], need[1] - gt[1]};          // entries equal to tau that are kept
    itau[0] = 0xFFFFFFFFu; itau[1] = 0xFFFFFFFFu;
    if (r[0] >= eq[0] && r[1] >= eq[1]) return;           // uniform: every tie is kept
    // the r-th smallest index among the ties: the largest j with fewer than r tie indices below it
    uint32_t jp = 0u, jn = 0u;
#pragma nounroll
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t tp = jp | (1u << bit), tn = jn | (1u << bit);
        uint32_t cp = 0u, cn = 0u;
        src.template for_each<0>([&](uint32_t key, uint32_t idx) { cp += (key == pre_p && idx < tp) ? 1u : 0u; });
        src.template for_each<1>([&](uint32_t key, uint32_t idx) { cn += (key == pre_n && idx < tn) ? 1u : 0u; });
        const unsigned long long tot = block_sum(sh, parity, (unsigned long long)cp | ((unsigned long long)cn << 32));
        if ((uint32_t)tot < r[0]) jp = tp;
        if ((uint32_t)(tot >> 32) < r[1]) jn = tn;
    }
    if (r[0] < eq[0]) itau[0] = jp;
    if (r[1] < eq[1]) itau[1] = jn;
}

struct Decision {
    int chosen;            // 0: positive side kept, 1: negative side
    float mu_signed;
    bool ok;
    bool defer;            // not ok because the tensor is better left to k_select (no error)
};

// --------------------------------------------------------------------------
// Alg. 2 for one tensor, by the whole workgroup, over the entries `src` yields: thresholds of both
// sides (exactly k kept entries per side, equal values to the lowest index), S+ and S- as exact
// integers, the side with the larger mean, the transmitted mean.  Records the results in the
// tensor's state; with `carry`, also the filter keys for a following call.  cnt[s]: entries of
// side s; lo_cur[s]: the filter key they passed.  Returns ok = false (after raising an error bit
// or flagging the tensor for k_select) if it cannot complete.  Contains barriers.
// --------------------------------------------------------------------------
template <typename Src, bool CAN_BISECT>
__device__ __forceinline__ Decision select_tensor(StepShared& sh, int& parity, const Src& src, const TensorDesc& d,
                                                  TensorState* __restrict__ st_t, const uint32_t (&cnt)[2],
                                                  const uint32_t (&lo_cur)[2], bool carry,
                                                  uint32_t (&tau)[2], uint32_t (&itau)[2],
                                                  ResultBlock* __restrict__ result) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t k = d.k;
    Decision dec;
    dec.chosen = 0; dec.mu_signed = 0.f; dec.ok = false; dec.defer = false;

    // ---- range of the side keys ----
    uint32_t mx[2] = {0u, 0u}, mn[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
    src.template for_each<0>([&](uint32_t key, uint32_t) { mx[0] = key > mx[0] ? key : mx[0]; mn[0] = key < mn[0] ? key : mn[0]; });
    src.template for_each<1>([&](uint32_t key, uint32_t) { mx[1] = key > mx[1] ? key : mx[1]; mn[1] = key < mn[1] ? key : mn[1]; });
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const uint32_t hi = __shfl_xor(mx[s], off, 64), lo = __shfl_xor(mn[s], off, 64);
            mx[s] = hi > mx[s] ? hi : mx[s];
            mn[s] = lo < mn[s] ? lo : mn[s];
        }
    }
    if (lane == 0) { sh.ext[wave][0] = mx[0]; sh.ext[wave][1] = mn[0]; sh.ext[wave][2] = mx[1]; sh.ext[wave][3] = mn[1]; }
    for (int i = tid; i < 2 * kStepWindow; i += kStepThreads) sh.lds[i] = 0u;
    if (tid < 2) sh.bcnt[tid] = 0u;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kStepWaves; ++w) {
        mx[0] = sh.ext[w][0] > mx[0] ? sh.ext[w][0] : mx[0]; mn[0] = sh.ext[w][1] < mn[0] ? sh.ext[w][1] : mn[0];
        mx[1] = sh.ext[w][2] > mx[1] ? sh.ext[w][2] : mx[1]; mn[1] = sh.ext[w][3] < mn[1] ? sh.ext[w][3] : mn[1];
    }
    if (mx[0] < mn[0] || mx[1] < mn[1]) {                 // uniform; a side without entries cannot happen (cnt >= k >= 1)
        if (tid == 0) atomicOr(&result->err, kErrInternal);
        return dec;
    }
    // bin of a key: its offset from the side's smallest key, scaled so that the largest lands in the window
    int shift[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint32_t span = mx[s] - mn[s];
        shift[s] = span ? max(0, 32 - __clz((int)span) - 10) : 0;
    }
    src.template for_each<0>([&](uint32_t key, uint32_t) { atomicAdd(&sh.whist()[0][(key - mn[0]) >> shift[0]], 1u); });
    src.template for_each<1>([&](uint32_t key, uint32_t) { atomicAdd(&sh.whist()[1][(key - mn[1]) >> shift[1]], 1u); });
    __syncthreads();

    // ---- bin of the k-th most extreme entry of each side; filter keys for a following call ----
    const bool both[2] = {true, true};
    uint32_t need[2] = {k, k}, digit[2];
    bool found[2];
    pick_wide_both<kStepWindow, kStepThreads>(sh.whist(), need, both, sh.res[0], sh.scratch64, digit, found);
    uint32_t next_key[2] = {lo_cur[0], lo_cur[1]};
    bool short_list[2] = {false, false};
    const uint32_t r_next = carried_rank(k);
    if (carry) {                                          // uniform
        // With the residual carried over, the k-th entry sits at the edge of a cliff (everything above
        // it has just been cut down to about mu), so a margin in value below it lets a flood of
        // entries pass, while a margin in rank does not: the key is the lower edge of the bin of this
        // call's r-th most extreme entry, r = 2 k + 4 sqrt(k) + 16 (if the next update is small beside
        // the residual, the k entries kept now are gone from above that key, and k more must
        // remain).  A list shorter than r says nothing about that entry: its place is extrapolated
        // from the k-th, once that is known.
        uint32_t need2[2] = {min(r_next, cnt[0]), min(r_next, cnt[1])}, digit2[2];
        bool found2[2];
        pick_wide_both<kStepWindow, kStepThreads>(sh.whist(), need2, both, sh.res[1], sh.scratch64, digit2, found2);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (cnt[s] >= r_next && found2[s]) next_key[s] = mn[s] + (digit2[s] << shift[s]);
            else short_list[s] = true;
        }
    }
    if (!found[0] || !found[1]) {                         // uniform; cannot happen: each side holds at least k entries
        if (tid == 0) atomicOr(&result->err, kErrInternal);
        return dec;
    }
    const uint32_t bsize[2] = {sh.whist()[0][digit[0]], sh.whist()[1][digit[1]]};
    itau[0] = 0xFFFFFFFFu; itau[1] = 0xFFFFFFFFu;
    if (bsize[0] <= kStepRankMax && bsize[1] <= kStepRankMax) {   // uniform
        // the usual case: the bin's few entries are copied out and ranked against each other by
        // (key descending, index ascending); the entry of rank need - 1 is the k-th of its side
        src.template for_each<0>([&](uint32_t key, uint32_t idx) {
            if (((key - mn[0]) >> shift[0]) == digit[0]) {
                const uint32_t q = atomicAdd(&sh.bcnt[0], 1u);
                if (q < kStepRankMax) sh.bucket(0)[q] = make_uint2(key, idx);
            }
        });
        src.template for_each<1>([&](uint32_t key, uint32_t idx) {
            if (((key - mn[1]) >> shift[1]) == digit[1]) {
                const uint32_t q = atomicAdd(&sh.bcnt[1], 1u);
                if (q < kStepRankMax) sh.bucket(1)[q] = make_uint2(key, idx);
            }
        });
        if (tid < 4) sh.pick[tid >> 1][tid & 1] = 0u;
        __syncthreads();
        bool ok = true;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const uint32_t m = sh.bcnt[s];
            if (m != bsize[s]) { ok = false; continue; }  // uniform; cannot happen
            for (uint32_t i = tid; i < m; i += kStepThreads) {
                const uint2 me2 = sh.bucket(s)[i];
                const unsigned long long me = ((unsigned long long)me2.x << 32) | (uint32_t)~me2.y;
                uint32_t ahead = 0u;
                for (uint32_t j = 0; j < m; ++j) {
                    const uint2 o = sh.bucket(s)[j];
                    ahead += ((((unsigned long long)o.x << 32) | (uint32_t)~o.y) > me) ? 1u : 0u;
                }
                if (ahead + 1u == need[s]) { sh.pick[s][0] = me2.x; sh.pick[s][1] = me2.y; }
            }
        }
        __syncthreads();
        tau[0] = sh.pick[0][0]; itau[0] = sh.pick[0][1];
        tau[1] = sh.pick[1][0]; itau[1] = sh.pick[1][1];
        if (!ok || tau[0] == 0u || tau[1] == 0u) {        // uniform; cannot happen
            if (tid == 0) atomicOr(&result->err, kErrInternal);
            return dec;
        }
    } else if (CAN_BISECT) {
        const uint32_t kk[2] = {k, k};
        bisect_thresholds(sh, parity, src, kk, tau, itau);
    } else {
        // tie-heavy data in lists too long for LDS: left to k_select
        dec.defer = true;
        return dec;
    }
    __syncthreads();                                      // the histogram's space is reused below

    // ---- S+ and S- (Alg. 2: the sums behind mu+ and mu-) as exact integers.  A kept entry whose
    // sign is the side's and whose exponent lies 0..24 above that of the threshold is added, shifted
    // to the threshold's scale, to one 64-bit integer (exact: 24 + 24 bits and at most 2^15
    // entries); anything else goes to one integer per fp32 exponent in LDS.  One rounding to fp64
    // per part, in a fixed order. ----
    const bool common[2] = {k <= 32768u && tau[0] > 0x80000000u, k <= 32768u && tau[1] >= 0x80000000u};
    uint32_t e_ref[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint32_t ex = (bits_of_key(s ? ~tau[s] : tau[s]) >> 23) & 0xFFu;
        e_ref[s] = ex ? ex : 1u;
    }
    long long part[2] = {0ll, 0ll};
    bool slow = !common[0] || !common[1];
    auto add_fast = [&](int s, uint32_t side_key) {
        const uint32_t u = bits_of_key(s ? ~side_key : side_key);
        uint32_t ex = (u >> 23) & 0xFFu;
        const long long m = (long long)(ex ? ((u & 0x7FFFFFu) | 0x800000u) : (u & 0x7FFFFFu));
        if (ex == 0u) ex = 1u;
        if (common[s] && ex >= e_ref[s] && ex - e_ref[s] <= 24u) part[s] += m << (ex - e_ref[s]);
        else slow = true;
    };
    src.template for_each<0>([&](uint32_t key, uint32_t idx) { if (cand_kept(key, idx, tau[0], itau[0])) add_fast(0, key); });
    src.template for_each<1>([&](uint32_t key, uint32_t idx) { if (cand_kept(key, idx, tau[1], itau[1])) add_fast(1, key); });
    const bool any_slow = __syncthreads_or(slow ? 1 : 0) != 0;
    const unsigned long long t0 = block_sum(sh, parity, (unsigned long long)part[0]);
    const unsigned long long t1 = block_sum(sh, parity, (unsigned long long)part[1]);
    double S[2];
    S[0] = ldexp((double)(long long)t0, (int)e_ref[0] - 150);
    S[1] = ldexp((double)(long long)t1, (int)e_ref[1] - 150);
    if (any_slow) {                                       // uniform
        for (int i = tid; i < 512; i += kStepThreads) sh.acc(0)[i] = 0ll;
        __syncthreads();
        auto add_slow = [&](int s, uint32_t side_key) {
            const uint32_t u = bits_of_key(s ? ~side_key : side_key);
            uint32_t ex = (u >> 23) & 0xFFu;
            long long m = (long long)(ex ? ((u & 0x7FFFFFu) | 0x800000u) : (u & 0x7FFFFFu));
            if (ex == 0u) ex = 1u;
            if (common[s] && ex >= e_ref[s] && ex - e_ref[s] <= 24u) return;
            if (((u >> 31) != 0u) != (s != 0)) m = -m;       // the negative side sums -A
            if (m != 0ll) atomicAdd(reinterpret_cast<unsigned long long*>(&sh.acc(s)[ex]), (unsigned long long)m);
        };
        src.template for_each<0>([&](uint32_t key, uint32_t idx) { if (cand_kept(key, idx, tau[0], itau[0])) add_slow(0, key); });
        src.template for_each<1>([&](uint32_t key, uint32_t idx) { if (cand_kept(key, idx, tau[1], itau[1])) add_slow(1, key); });
        __syncthreads();
        if (tid < 128) {
            // fixed order: lane l of wavefront s adds exponents 4l..4l+3 ascending, then a fixed tree
            const int s = tid >> 6;
            double v = 0.0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int ex = 4 * lane + j;
                v += ldexp((double)sh.acc(s)[ex], ex - 150);
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
            if (lane == 0) sh.S[s] = v;
        }
        __syncthreads();
        S[0] = sh.S[0] + S[0];
        S[1] = sh.S[1] + S[1];
        __syncthreads();                                  // acc shares its space with what follows
    }

    // ---- Alg. 2's comparison of the means (S+ and S- are correctly rounded sums, so the means are
    // those of an exactly rounded summation; equal means keep the positive side) ----
    dec.chosen = (S[0] / (double)k >= S[1] / (double)k) ? 0 : 1;
    const float mu32 = (float)(S[dec.chosen] / (double)k);
    dec.mu_signed = dec.chosen ? -mu32 : mu32;
    dec.ok = true;
    if (tid == 0) {
        st_t->tau[0] = tau[0]; st_t->tau[1] = tau[1];
        st_t->itau[0] = itau[0]; st_t->itau[1] = itau[1];
        st_t->kc[0] = k; st_t->kc[1] = k;
        st_t->S[0] = S[0]; st_t->S[1] = S[1];
        st_t->side = dec.chosen ? -1 : 1;
        st_t->mu_signed = dec.mu_signed;
        if (carry) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                st_t->lo_key[s] = short_list[s] ? extrapolated_key(tau[s], lo_cur[s], k, r_next, d.n, cnt[s]) : next_key[s];
                st_t->expect[s] = 0u;
            }
        }
    }
    return dec;
}

// Alg. 3 over kk ascending kept indices in LDS (`sorted`): code lengths, bit offsets, the bits
// into zeroed LDS words (`words`, any LDS array but `sorted`), then the stream to the tensor's
// staging words and the indices to the kept-index scratch.  Returns false (in every thread) if
// the stream would exceed max_words.  Contains barriers.
__device__ __forceinline__ bool encode_sorted(StepShared& sh, const uint32_t* sorted, uint32_t* words, uint32_t kk,
                                              int b, uint32_t max_words, uint32_t* __restrict__ stage_out,
                                              uint32_t* __restrict__ kept_out, TensorState* __restrict__ st_t) {
    const int tid = threadIdx.x;
    const uint32_t E = (kk + kStepThreads - 1) / kStepThreads;
    const uint32_t i0 = tid * E < kk ? tid * E : kk;
    const uint32_t i1 = i0 + E < kk ? i0 + E : kk;
    unsigned long long bits = 0ull;
    {
        uint32_t pe = i0 ? sorted[i0 - 1] + 1u : 0u;
        for (uint32_t i = i0; i < i1; ++i) {
            const uint32_t x = sorted[i];
            bits += golomb_len(x - pe, b);
            pe = x + 1u;
        }
    }
    unsigned long long total_bits;
    unsigned long long pos = block_excl_sum<unsigned long long, kStepThreads>(bits, &total_bits, sh.scratch64);
    const unsigned long long n_words64 = (total_bits + 31ull) >> 5;
    if (n_words64 > (unsigned long long)max_words) return false;       // uniform
    const uint32_t n_words = (uint32_t)n_words64;
    for (uint32_t w = tid; w < n_words + 1u; w += kStepThreads) words[w] = 0u;
    __syncthreads();
    {
        uint32_t pe = i0 ? sorted[i0 - 1] + 1u : 0u;
        for (uint32_t i = i0; i < i1; ++i) {
            const uint32_t x = sorted[i];
            const uint32_t gap = x - pe;
            const uint32_t q = gap >> b;
            put_ones(words, pos, q);
            pos += q;
            put_bits(words, pos, gap & ((1u << b) - 1u), b + 1);       // the zero and the remainder
            pos += (unsigned)b + 1u;
            pe = x + 1u;
        }
    }
    __syncthreads();
    for (uint32_t w = tid; w < n_words; w += kStepThreads) stage_out[w] = words[w];
    for (uint32_t i = tid; i < kk; i += kStepThreads) kept_out[i] = sorted[i];
    if (tid == 0) { st_t->bit_len = total_bits; st_t->nnz = kk; }
    return true;
}

// --------------------------------------------------------------------------
// A tensor of one chunk, all of it in this workgroup's registers.
// --------------------------------------------------------------------------
__device__ __forceinline__ void finish_small(StepShared& sh, const LdsChunk& src, const TensorDesc& d,
                                             TensorState* __restrict__ st_t, uint32_t* __restrict__ stage,
                                             uint32_t* __restrict__ kept_idx, int b, ResultBlock* __restrict__ result) {
    const int tid = threadIdx.x;
    int parity = 0;
    const uint32_t k = d.k;
    const uint32_t cnt[2] = {d.n, d.n}, lo_cur[2] = {0u, 0u};
    uint32_t tau[2], itau[2];
    const Decision dec = select_tensor<LdsChunk, true>(sh, parity, src, d, st_t, cnt, lo_cur, false, tau, itau, result);
    if (!dec.ok) return;                                  // uniform
    const uint32_t ktau = tau[dec.chosen], kitau = itau[dec.chosen];
    // kept positions as a bitmap in LDS; the residual update of the kept entries goes out right
    // away (this workgroup stored A at these positions before the barriers above, and stores of
    // one workgroup to one address stay in order across a barrier)
    uint32_t* const bitmap = sh.lds;                      // region A: the histogram is no longer needed
    uint32_t* const words = sh.lds + kChunkWords;
    if (tid < kChunkWords) bitmap[tid] = 0u;
    __syncthreads();
    const gfloat_ptr R = as_global(d.R);
    auto keep = [&](uint32_t key, uint32_t pos) {
        if (cand_kept(key, pos, ktau, kitau)) {
            atomicOr(&bitmap[pos >> 5], 1u << (pos & 31u));
            const float a = __uint_as_float(bits_of_key(dec.chosen ? ~key : key));
            R[pos] = a - dec.mu_signed;                   // Alg. 1: R <- dW - dW*
        }
    };
    if (dec.chosen) src.for_each<1>(keep); else src.for_each<0>(keep);
    __syncthreads();
    // Alg. 3 from the bitmap: one word per thread (of the first 256)
    const uint32_t word = tid < kChunkWords ? bitmap[tid] : 0u;
    const uint32_t end_w = word ? (uint32_t)(tid * 32 + 32 - __clz(word)) : 0u;
    uint32_t last_end;
    uint32_t pe = block_excl_max<uint32_t, kStepThreads>(end_w, &last_end, sh.scratch32);
    unsigned long long bits = 0ull;
    {
        uint32_t m = word, p = pe;
        while (m) {
            const uint32_t x = (uint32_t)(tid * 32 + __ffs(m) - 1);
            m &= m - 1u;
            bits += golomb_len(x - p, b);
            p = x + 1u;
        }
    }
    const unsigned long long packed = bits | ((unsigned long long)__popc(word) << 40);
    unsigned long long total;
    const unsigned long long ex = block_excl_sum<unsigned long long, kStepThreads>(packed, &total, sh.scratch64);
    const unsigned long long total_bits = total & ((1ull << 40) - 1ull);
    const uint32_t kk = (uint32_t)(total >> 40);
    const unsigned long long n_words = (total_bits + 31ull) >> 5;
    if (kk != k || n_words > d.bound_words || n_words > kSmallMaxWords) {   // uniform; cannot happen
        if (tid == 0) atomicOr(&result->err, kErrInternal);
        return;
    }
    for (uint32_t w = tid; w < (uint32_t)n_words + 1u; w += kStepThreads) words[w] = 0u;
    __syncthreads();
    {
        unsigned long long pos = ex & ((1ull << 40) - 1ull);
        uint32_t rank = (uint32_t)(ex >> 40);
        uint32_t* __restrict__ ki = kept_idx + d.kept_off;
        uint32_t m = word;
        while (m) {
            const uint32_t x = (uint32_t)(tid * 32 + __ffs(m) - 1);
            m &= m - 1u;
            const uint32_t gap = x - pe;
            const uint32_t q = gap >> b;
            put_ones(words, pos, q);
            pos += q;
            put_bits(words, pos, gap & ((1u << b) - 1u), b + 1);
            pos += (unsigned)b + 1u;
            pe = x + 1u;
            ki[rank++] = x;
        }
    }
    __syncthreads();
    uint32_t* __restrict__ out = stage + d.stage_off;
    for (uint32_t w = tid; w < (uint32_t)n_words; w += kStepThreads) out[w] = words[w];
    if (tid == 0) { st_t->bit_len = total_bits; st_t->nnz = kk; st_t->flags = kStInlineDone | kStResidualDone; }
}

// --------------------------------------------------------------------------
// A tensor of several chunks, finished by the last of its workgroups to arrive, from the
// candidate lists the others have appended; returns true if the tensor is to be left to k_select.
// offs (kInlineBuckets words), grp (k + 2 words) and
// sorted (k words): LDS for the index sort, which may overlay the histogram but not the entries
// `src` reads.
// --------------------------------------------------------------------------
template <typename Src, bool CAN_BISECT>
__device__ __forceinline__ bool finish_from_lists(StepShared& sh, const Src& src, const TensorDesc& d,
                                                  TensorState* __restrict__ st_t, uint32_t cnt_p, uint32_t cnt_n,
                                                  uint32_t lo_p, uint32_t lo_n, uint32_t* offs, uint32_t* grp,
                                                  uint32_t* sorted, uint32_t* __restrict__ stage,
                                                  uint32_t* __restrict__ kept_idx, int b, bool carry,
                                                  ResultBlock* __restrict__ result) {
    const int tid = threadIdx.x;
    int parity = 0;
    const uint32_t k = d.k, n = d.n;
    const uint32_t cnt[2] = {cnt_p, cnt_n}, lo_cur[2] = {lo_p, lo_n};
    uint32_t tau[2], itau[2];
    const Decision dec = select_tensor<Src, CAN_BISECT>(sh, parity, src, d, st_t, cnt, lo_cur, carry, tau, itau, result);
    SBC_STEP_TS(5);
    if (!dec.ok) return dec.defer;                        // uniform
    const uint32_t ktau = tau[dec.chosen], kitau = itau[dec.chosen];

    // ---- the k kept indices, ascending: bucket by leading index bits, rank inside the bucket ----
    int shift = 32 - __clz((int)(n - 1u | 1u)) - 10;      // bucket = idx >> shift, below kInlineBuckets
    if (shift < 0) shift = 0;
    for (int i = tid; i < kInlineBuckets; i += kStepThreads) offs[i] = 0u;
    __syncthreads();
    bool bad = false;
    auto count_kept = [&](uint32_t key, uint32_t idx) {
        if (cand_kept(key, idx, ktau, kitau)) { if (idx < n) atomicAdd(&offs[idx >> shift], 1u); else bad = true; }
    };
    if (dec.chosen) src.template for_each<1>(count_kept); else src.template for_each<0>(count_kept);
    __syncthreads();
    {   // exclusive scan of the bucket counts, in place: consecutive buckets per thread
        constexpr int PB = kInlineBuckets / kStepThreads;
        uint32_t loc[PB], sum = 0u;
#pragma unroll
        for (int j = 0; j < PB; ++j) { loc[j] = offs[tid * PB + j]; sum += loc[j]; }
        uint32_t total;
        uint32_t ex = block_excl_sum<uint32_t, kStepThreads>(sum, &total, sh.scratch32);
#pragma unroll
        for (int j = 0; j < PB; ++j) { offs[tid * PB + j] = ex; ex += loc[j]; }
        if (total != k || __syncthreads_or(bad ? 1 : 0)) {      // uniform; cannot happen
            if (tid == 0) atomicOr(&result->err, kErrInternal);
            return false;
        }
    }
    // scatter: a bucket's slot counter runs from its start to its end (= the next bucket's start)
    auto scatter_kept = [&](uint32_t key, uint32_t idx) {
        if (cand_kept(key, idx, ktau, kitau) && idx < n) grp[atomicAdd(&offs[idx >> shift], 1u)] = idx;
    };
    if (dec.chosen) src.template for_each<1>(scatter_kept); else src.template for_each<0>(scatter_kept);
    __syncthreads();
    for (uint32_t i = tid; i < k; i += kStepThreads) {
        const uint32_t v = grp[i];
        const uint32_t bk = v >> shift;
        const uint32_t lo = bk ? offs[bk - 1u] : 0u, hi = offs[bk];
        uint32_t rank = 0u;
        for (uint32_t j = lo; j < hi; ++j) rank += (grp[j] < v) ? 1u : 0u;
        sorted[lo + rank] = v;
    }
    __syncthreads();
    const uint32_t max_words = min(d.bound_words, kInlineMaxWords);
    if (!encode_sorted(sh, sorted, grp, k, b, max_words, stage + d.stage_off, kept_idx + d.kept_off, st_t)) {
        if (tid == 0) atomicOr(&result->err, kErrInternal);   // the host only inlines tensors whose bound fits
        return false;
    }
    if (tid == 0) st_t->flags = kStInlineDone;
    return false;
}

// --------------------------------------------------------------------------
// The streaming kernel.  sched[blockIdx.x] = (chunk in the call-wide numbering, tensor).
// STREAM: the update is loaded with the nontemporal hint (calls far beyond the last-level cache).
// --------------------------------------------------------------------------
template <bool STREAM>
__global__ __launch_bounds__(kStepThreads, 4) void k_client_step(
        const TensorDesc* __restrict__ desc, const uint2* __restrict__ sched, TensorState* __restrict__ st,
        uint2* __restrict__ cand, uint32_t* __restrict__ bitmap, uint32_t* __restrict__ stage,
        uint32_t* __restrict__ kept_idx, GroupState* __restrict__ groups, int b, int carry,
        ResultBlock* __restrict__ result) {
    __shared__ StepShared sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    SBC_STEP_TS(0);
    const uint2 sc = sched[blockIdx.x];
    const uint32_t c = sc.x;
    const int t = (int)sc.y;
    const TensorDesc d = desc[t];
    const uint32_t lo_p = st[t].lo_key[0], lo_n = st[t].lo_key[1];
    const uint32_t cc = c - d.chunk0;
    const uint32_t e0 = cc * (uint32_t)kChunk;
    const uint32_t cnt = min((uint32_t)kChunk, d.n - e0);
    const bool inline_t = (d.flags & kDescInline) != 0u;
    const bool small = inline_t && d.nchunks == 1u && d.n <= kSmallMaxN;

    if (!(d.flags & kDescFused)) {
        // encoded from the bitmap later: clear this chunk's bitmap words and share of the staging words
        bitmap[(uint64_t)c * kChunkWords + tid] = 0u;
        const uint32_t per = (d.bound_words + d.nchunks - 1u) / d.nchunks;
        const uint32_t lo = per * cc;
        const uint32_t hi = (lo + per < d.bound_words) ? lo + per : d.bound_words;
        for (uint32_t w = lo + tid; w < hi; w += kStepThreads) stage[d.stage_off + w] = 0u;
    }

    // ---- A = R + dW in registers: slot s of a thread is entry local(s) of the chunk ----
    const gcfloat_ptr dw = as_global(d.dW + e0);
    const gfloat_ptr r = as_global(d.R + e0);
    float a[kSlots];
    const bool vec = (cnt == (uint32_t)kChunk) && ((((uintptr_t)(d.dW + e0) | (uintptr_t)(d.R + e0)) & 15u) == 0u);
    if (vec) {
        const gcf32x4_ptr dw4 = (gcf32x4_ptr)dw;
        const gcf32x4_ptr r4 = (gcf32x4_ptr)r;
        constexpr int IT = kSlots / 4;                    // 4
        f32x4 dv[IT], rv[IT];
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            dv[i] = STREAM ? __builtin_nontemporal_load(&dw4[i * kStepThreads + tid]) : dw4[i * kStepThreads + tid];
            rv[i] = r4[i * kStepThreads + tid];
        }
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            a[4 * i + 0] = rv[i].x + dv[i].x;
            a[4 * i + 1] = rv[i].y + dv[i].y;
            a[4 * i + 2] = rv[i].z + dv[i].z;
            a[4 * i + 3] = rv[i].w + dv[i].w;
        }
    } else {
        // a tensor's last, partial chunk, or operands that are only 4-byte aligned: eight entries per
        // thread in flight at a time
        constexpr int IT = 8;
#pragma unroll
        for (int bt = 0; bt < kSlots / IT; ++bt) {
            float dv[IT], rv[IT];
            if ((uint32_t)(bt * IT * kStepThreads) < cnt) {     // uniform
#pragma unroll
                for (int j = 0; j < IT; ++j) {
                    const uint32_t i = (uint32_t)((bt * IT + j) * kStepThreads + tid);
                    const uint32_t ii = i < cnt ? i : 0u;
                    dv[j] = dw[ii];
                    rv[j] = r[ii];
                }
#pragma unroll
                for (int j = 0; j < IT; ++j) a[bt * IT + j] = rv[j] + dv[j];
            } else {
#pragma unroll
                for (int j = 0; j < IT; ++j) a[bt * IT + j] = 0.f;
            }
        }
    }
    // position within the chunk of the thread's slot s, and whether the slot holds an entry
    // (a per-thread base plus a term that is the same for the whole workgroup)
    const uint32_t lane_base = vec ? (uint32_t)tid * 4u : (uint32_t)tid;
    auto local = [&](int s) -> uint32_t {
        return lane_base + (vec ? (uint32_t)((s >> 2) * kStepThreads * 4 + (s & 3)) : (uint32_t)(s * kStepThreads));
    };
    auto used = [&](int s) -> bool { return vec || (uint32_t)(s * kStepThreads + tid) < cnt; };
    // A over R.  Stores of one thread stay in order, and nothing below waits for these.
    auto store_A = [&]() {
        if (vec) {
            const gf32x4_ptr r4 = (gf32x4_ptr)r;
#pragma unroll
            for (int i = 0; i < kSlots / 4; ++i) {
                f32x4 v;
                v.x = a[4 * i + 0]; v.y = a[4 * i + 1]; v.z = a[4 * i + 2]; v.w = a[4 * i + 3];
                r4[i * kStepThreads + tid] = v;
            }
        } else {
#pragma unroll
            for (int s = 0; s < kSlots; ++s) {
                const uint32_t i = (uint32_t)(s * kStepThreads + tid);
                if (i < cnt) r[i] = a[s];
            }
        }
    };
    SBC_STEP_TS(1);
    SBC_STEP_VAL(7, (unsigned long long)t | ((unsigned long long)cc << 32));

    if (small) {
        // ---- the whole tensor is here: its keys go to LDS, and the workgroup finishes it ----
        store_A();
        __builtin_amdgcn_s_setprio(3);
        uint32_t* const keys = sh.region_b();
        uint32_t mxs = 0u;
#pragma unroll
        for (int s = 0; s < kSlots; ++s) {
            if ((uint32_t)(s * kStepThreads + tid) < cnt) {   // (a one-chunk tensor never takes the vector layout)
                const uint32_t u = __float_as_uint(a[s]);
                keys[s * kStepThreads + tid] = key_of_bits(u);
                const uint32_t mag = u & 0x7FFFFFFFu;
                mxs = mag > mxs ? mag : mxs;
            }
        }
        if (__syncthreads_or(mxs >= 0x7F800000u ? 1 : 0)) {   // a NaN or an infinity: the call fails
            if (tid == 0) atomicOr(&result->err, kErrNonFinite);
            return;
        }
        LdsChunk src;
        src.keys = keys; src.n = cnt;
        finish_small(sh, src, d, &st[t], stage, kept_idx, b, result);
        SBC_STEP_TS(6);
        return;
    }

    // ---- filter: per-wavefront queues filled with ballots ----
    uint32_t wc_p = 0u, wc_n = 0u;                        // wave-uniform counts (may exceed the queue: overflow)
    uint32_t mx = 0u;                                     // largest magnitude bits seen (non-finite check)
#pragma unroll
    for (int s = 0; s < kSlots; ++s) {
        const uint32_t u = __float_as_uint(a[s]);
        const uint32_t mag = u & 0x7FFFFFFFu;
        mx = mag > mx ? mag : mx;
        const uint32_t kk = key_of_bits(u);
        const bool in = used(s);
        const bool cp = in && kk >= lo_p, cn = in && ~kk >= lo_n;
        const unsigned long long bp = __ballot(cp), bn = __ballot(cn);
        if (bp) {
            const uint32_t at = wc_p + lane_rank(bp);
            if (cp && at < (uint32_t)kWaveQueue) sh.wq(wave, 0)[at] = make_uint2(kk, e0 + local(s));
            wc_p += (uint32_t)__popcll(bp);
        }
        if (bn) {
            const uint32_t at = wc_n + lane_rank(bn);
            if (cn && at < (uint32_t)kWaveQueue) sh.wq(wave, 1)[at] = make_uint2(~kk, e0 + local(s));
            wc_n += (uint32_t)__popcll(bn);
        }
    }
    if (mx >= 0x7F800000u) atomicOr(&result->err, kErrNonFinite);
    if (lane == 0) { sh.wcnt[wave][0] = wc_p; sh.wcnt[wave][1] = wc_n; }
    __syncthreads();
    uint32_t qp = 0u, qn = 0u, before_p = 0u, before_n = 0u;
    bool overflow = false;
#pragma unroll
    for (int w = 0; w < kStepWaves; ++w) {
        const uint32_t x = sh.wcnt[w][0], y = sh.wcnt[w][1];
        if (w < wave) { before_p += x; before_n += y; }
        qp += x; qn += y;
        overflow = overflow || x > (uint32_t)kWaveQueue || y > (uint32_t)kWaveQueue;
    }
    uint2* __restrict__ lp = cand + d.cand_off;
    uint2* __restrict__ ln = cand + d.cand_off + d.cand_cap;
    unsigned long long* const counter = reinterpret_cast<unsigned long long*>(&st[t].cand_cnt[0]);
    const uint32_t grp = cc / (uint32_t)kGroupChunks;
    const uint32_t n_groups = (d.nchunks + kGroupChunks - 1u) / kGroupChunks;
    // Counts this chunk in (thread 0); true in thread 0 of the tensor's last workgroup.
    auto count_in = [&]() -> bool {
        // two levels, so that the thousands of workgroups of a large tensor do not queue on one address
        const uint32_t g_size = min((uint32_t)kGroupChunks, d.nchunks - grp * kGroupChunks);
        if (atomicAdd(&groups[d.grp0 + grp].done, 1u) + 1u != g_size) return false;
        return n_groups == 1u || atomicAdd(&st[t].done, 1u) + 1u == n_groups;
    };
    bool fatal = false, last = false;
    if (!overflow) {
        if (qp + qn != 0u) {                              // uniform
            if (tid == 0) {
                // both sides' counters advance in one 64-bit atomic
                const unsigned long long old = atomicAdd(counter, (unsigned long long)qp | ((unsigned long long)qn << 32));
                sh.base[0] = (uint32_t)old;
                sh.base[1] = (uint32_t)(old >> 32);
            }
            __syncthreads();
            const uint32_t bp0 = sh.base[0], bn0 = sh.base[1];
            if ((uint64_t)bp0 + qp > d.cand_cap || (uint64_t)bn0 + qn > d.cand_cap) {
                // (beyond a list's capacity nothing is stored: the counters then show that the lists are not usable)
            } else {
                for (uint32_t i = lane; i < wc_p; i += 64u) { const uint2 e = sh.wq(wave, 0)[i]; store_cand(lp + bp0 + before_p + i, e.x, e.y); }
                for (uint32_t i = lane; i < wc_n; i += 64u) { const uint2 e = sh.wq(wave, 1)[i]; store_cand(ln + bn0 + before_n + i, e.x, e.y); }
            }
        }
        if (fatal) atomicOr(&result->err, kErrInternal);
        SBC_STEP_TS(2);
        if (!inline_t) {                                  // finished by the kernels that follow
            store_A();
            return;
        }
        // ---- count this chunk in; the last workgroup of the tensor finishes it ----
        wait_all_memory();                                // this wavefront's candidate stores have completed
        __syncthreads();
        if (tid == 0) last = count_in();
        store_A();                                        // (goes out while the count comes back)
    } else {
        // a queue overflowed (tie-heavy or constant data, or an all-pass key): A is stored now, and
        // the chunk's candidates are appended from a second read of it, 2048 entries at a time with
        // a block scan
        store_A();
        wait_all_memory();
        __syncthreads();
        for (uint32_t base0 = 0; base0 < cnt; base0 += 8u * kStepThreads) {
            uint32_t mp = 0u, mn = 0u, kk8[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t pos = base0 + (uint32_t)j * kStepThreads + tid;
                kk8[j] = key_of_bits(__float_as_uint(r[pos < cnt ? pos : 0u]));
                if (pos < cnt && kk8[j] >= lo_p) mp |= 1u << j;
                if (pos < cnt && ~kk8[j] >= lo_n) mn |= 1u << j;
            }
            const uint32_t packed = __popc(mp) | (__popc(mn) << 16);
            uint32_t total;
            const uint32_t ex = block_excl_sum<uint32_t, kStepThreads>(packed, &total, sh.scratch32);
            if (total == 0u) continue;                    // uniform
            if (tid == 0) {
                const unsigned long long old = atomicAdd(counter, (unsigned long long)(total & 0xFFFFu) | ((unsigned long long)(total >> 16) << 32));
                sh.base[0] = (uint32_t)old;
                sh.base[1] = (uint32_t)(old >> 32);
            }
            __syncthreads();
            uint32_t op = sh.base[0] + (ex & 0xFFFFu), on = sh.base[1] + (ex >> 16);
            __syncthreads();                              // base is rewritten in the next round
            if ((uint64_t)op + __popc(mp) > d.cand_cap || (uint64_t)on + __popc(mn) > d.cand_cap) continue;   // (nothing is stored beyond a list's capacity)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t pos = base0 + (uint32_t)j * kStepThreads + tid;
                if (mp & (1u << j)) store_cand(lp + op++, kk8[j], e0 + pos);
                if (mn & (1u << j)) store_cand(ln + on++, ~kk8[j], e0 + pos);
            }
        }
        if (fatal) atomicOr(&result->err, kErrInternal);
        if (!inline_t) return;
        wait_all_memory();
        __syncthreads();
        if (tid == 0) last = count_in();
    }
    if (tid == 0) sh.flag = last ? 1u : 0u;
    __syncthreads();
    SBC_STEP_TS(3);
    if (sh.flag == 0u) return;
    // the rest is a chain of short dependent steps: let it go ahead of the streaming wavefronts
    // it shares the compute unit with
    __builtin_amdgcn_s_setprio(3);
    const unsigned long long counts = load_shared_u64(counter);
    const uint32_t cnt_p = __builtin_amdgcn_readfirstlane((uint32_t)counts);
    const uint32_t cnt_n = __builtin_amdgcn_readfirstlane((uint32_t)(counts >> 32));
    if (tid == 0) { st[t].cand_seen[0] = cnt_p; st[t].cand_seen[1] = cnt_n; }
    if (cnt_p > d.n || cnt_n > d.n) {
        if (tid == 0) atomicOr(&result->err, kErrInternal);
        return;
    }
    if (cnt_p > d.cand_cap || cnt_n > d.cand_cap) {
        // compact context: more candidates than a list holds; the histogram route extracts a tighter set
        if (tid == 0) { st[t].flags = kStFailed; atomicOr(&result->err, kErrPrefilter); }
        return;
    }
    if (cnt_p < d.k || cnt_n < d.k) {
        // the filter kept too few entries on a side: the histogram route redoes this tensor
        if (tid == 0) { st[t].flags = kStFailed; atomicOr(&result->err, kErrPrefilter); }
        return;
    }
    bool defer = false;
    // Lists that fit region B beside the sort arrays of a tensor that keeps few entries (in region
    // A) are staged in LDS, every load in flight at once; longer ones are read from memory in
    // every sweep, and the sort arrays take both regions.
    const bool staged = 2u * (cnt_p + cnt_n) <= kLdsB && kInlineBuckets + 2u * d.k + 2u <= kLdsA;
    if (staged) {
        uint2* const ep = reinterpret_cast<uint2*>(sh.region_b());
        uint2* const en = ep + cnt_p;
        for (uint32_t i0 = tid; i0 < cnt_p + cnt_n; i0 += 8u * kStepThreads) {
            uint2 e[8];
#pragma unroll
            for (uint32_t u = 0; u < 8u; ++u) {
                const uint32_t i = i0 + u * kStepThreads;
                e[u] = load_cand(i < cnt_p ? lp + i : ln + (i < cnt_p + cnt_n ? i - cnt_p : 0u));
            }
#pragma unroll
            for (uint32_t u = 0; u < 8u; ++u) { const uint32_t i = i0 + u * kStepThreads; if (i < cnt_p + cnt_n) ep[i] = e[u]; }
        }
        __syncthreads();
        LdsLists src;
        src.e[0] = ep; src.e[1] = en; src.cnt[0] = cnt_p; src.cnt[1] = cnt_n;
        SBC_STEP_TS(4);
        defer = finish_from_lists<LdsLists, true>(sh, src, d, &st[t], cnt_p, cnt_n, lo_p, lo_n, sh.lds, sh.lds + kInlineBuckets,
                                                  sh.lds + kInlineBuckets + d.k + 2u, stage, kept_idx, b, carry != 0, result);
    } else if (cnt_p <= kInlineMaxCand && cnt_n <= kInlineMaxCand) {
        MemLists src;
        src.g[0] = lp; src.g[1] = ln; src.cnt[0] = cnt_p; src.cnt[1] = cnt_n;
        SBC_STEP_TS(4);
        defer = finish_from_lists<MemLists, false>(sh, src, d, &st[t], cnt_p, cnt_n, lo_p, lo_n, sh.lds, sh.lds + kInlineBuckets,
                                                   sh.lds + kInlineBuckets + d.k + 2u, stage, kept_idx, b, carry != 0, result);
    } else {
        defer = true;
    }
    if (defer && tid == 0) {                              // left to k_select
        st[t].flags = kStDeferred;
        atomicOr(&result->err, kErrDeferred);
    }
    SBC_STEP_TS(6);
}

// --------------------------------------------------------------------------
// Message assembly and the end of the call.  grid (T, P): workgroup (t, y) copies every P-th
// 256-word slice of tensor t's stream to its place in the payload (streams in tensor order, each
// starting on a word boundary); the lead workgroup of a tensor writes its table entry, applies
// the residual update R[j] = A[j] - mu at the kept entries of a tensor finished inside
// k_client_step (Alg. 1: R <- dW - dW*), and leaves the tensor's counters clean for the next
// call; workgroup (0, 0) writes the header and the call's result block, also to pinned host
// memory.  If some tensor still has to be redone by the kernels of the other routes, nothing but
// the result block is written: the host launches those kernels and this one again.
// --------------------------------------------------------------------------
// The call's result block in pinned host memory is complete: its sequence number goes out last, so
// that a host that polls for the number finds size and error word in place.
__device__ __forceinline__ void publish_result(ResultBlock* host_result, uint32_t seq) {
    __threadfence_system();
    __hip_atomic_store(&host_result->pad, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ __launch_bounds__(256) void k_finish_message(const TensorDesc* __restrict__ desc,
                                                        TensorState* __restrict__ st, int T, int b,
                                                        const uint32_t* __restrict__ stage,
                                                        const uint32_t* __restrict__ kept_idx,
                                                        GroupState* __restrict__ groups,
                                                        uint8_t* __restrict__ msg, uint64_t msg_capacity,
                                                        ResultBlock* __restrict__ result,
                                                        ResultBlock* __restrict__ next_result,
                                                        ResultBlock* __restrict__ host_result, uint32_t seq) {
    __shared__ unsigned long long part[2][4];
    const int t = blockIdx.x, tid = threadIdx.x;
    const bool lead = (blockIdx.y == 0);
    const uint32_t err_in = result->err;
    if (err_in & (kErrPrefilter | kErrDeferred | kErrInternal | kErrNonFinite | kErrOverflow)) {
        if (t == 0 && lead && tid == 0) { host_result->msg_bytes = 0ull; host_result->err = err_in; publish_result(host_result, seq); }
        return;
    }
    const TensorDesc d = desc[t];
    const uint32_t my_flags = st[t].flags;
    const unsigned long long bit_len = st[t].bit_len;
    const uint32_t nnz = st[t].nnz;
    const float mu_signed = st[t].mu_signed;
    // word offset of this tensor's stream: streams are packed in tensor order
    unsigned long long mine = 0ull, all = 0ull;
    const int upto = (t == 0 && lead) ? T : t;          // workgroup (0, 0) also needs the grand total
    for (int i = tid; i < upto; i += 256) {
        const unsigned long long words = (st[i].bit_len + 31ull) >> 5;
        all += words;
        if (i < t) mine += words;
    }
    mine = wave_incl_sum(mine);                         // (the scan's last lane holds the wavefront's total)
    all = wave_incl_sum(all);
    if ((tid & 63) == 63) { part[0][tid >> 6] = mine; part[1][tid >> 6] = all; }
    __syncthreads();
    const unsigned long long word_off = part[0][0] + part[0][1] + part[0][2] + part[0][3];
    const unsigned long long tot_all = part[1][0] + part[1][1] + part[1][2] + part[1][3];
    const unsigned long long n_words = (bit_len + 31ull) >> 5;
    const unsigned long long table_end = 32ull + 24ull * (unsigned)T;
    if (n_words > d.bound_words || table_end + 4ull * (word_off + n_words) > msg_capacity || nnz > d.kcap) {
        if (tid == 0) { atomicOr(&result->err, kErrInternal); if (lead) atomicOr(&host_result->err, kErrInternal); }
        return;
    }
    if (lead) {
        if ((my_flags & kStInlineDone) && !(my_flags & kStResidualDone)) {
            const gfloat_ptr R = as_global(d.R);
            const uint32_t* __restrict__ ki = kept_idx + d.kept_off;
            for (uint32_t i0 = tid; i0 < nnz; i0 += 256u * 4u) {
                uint32_t j[4]; float a[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) { const uint32_t i = i0 + 256u * u; j[u] = i < nnz ? ki[i] : 0xFFFFFFFFu; }
#pragma unroll
                for (int u = 0; u < 4; ++u) a[u] = j[u] < d.n ? R[j[u]] : 0.f;
#pragma unroll
                for (int u = 0; u < 4; ++u) if (j[u] < d.n) R[j[u]] = a[u] - mu_signed;
            }
        }
        // the counters of this tensor's chunk groups, for the next call
        if (d.flags & kDescInline) {
            const uint32_t n_groups = (d.nchunks + kGroupChunks - 1u) / kGroupChunks;
            GroupState z;
            z.done = 0u; z.pad[0] = z.pad[1] = z.pad[2] = 0u;
            for (uint32_t g = tid; g < n_groups; g += 256u) groups[d.grp0 + g] = z;
        }
        if (tid == 0) {
            uint8_t* e = msg + 32 + 24ull * (unsigned)t;
            *reinterpret_cast<float*>(e) = mu_signed;
            *reinterpret_cast<uint32_t*>(e + 4) = nnz;
            *reinterpret_cast<uint64_t*>(e + 8) = bit_len;
            *reinterpret_cast<uint64_t*>(e + 16) = word_off;
            st[t].cand_cnt[0] = 0u; st[t].cand_cnt[1] = 0u; st[t].flags = 0u; st[t].done = 0u;
            if (t == 0) {
                uint32_t* h = reinterpret_cast<uint32_t*>(msg);
                h[0] = 0x31434253u; h[1] = 1u; h[2] = (uint32_t)T; h[3] = (uint32_t)b;
                *reinterpret_cast<uint64_t*>(msg + 16) = tot_all;
                *reinterpret_cast<uint64_t*>(msg + 24) = 0ull;
                const unsigned long long bytes = table_end + 4ull * tot_all;
                result->msg_bytes = bytes;
                host_result->msg_bytes = bytes; host_result->err = err_in;
                publish_result(host_result, seq);
                // the result block of the next call starts out clean
                next_result->err = 0u; next_result->pad = 0u; next_result->msg_bytes = 0ull;
            }
        }
    }
    const uint32_t* __restrict__ src = stage + d.stage_off;
    uint32_t* __restrict__ dst = reinterpret_cast<uint32_t*>(msg + table_end) + word_off;
    for (unsigned long long w = (unsigned long long)blockIdx.y * 256ull + tid; w < n_words;
         w += 256ull * gridDim.y)
        dst[w] = src[w];
}

}  // namespace sbc
