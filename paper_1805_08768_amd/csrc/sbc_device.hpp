// Device-side building blocks shared by the SBC kernels: the order-preserving
// key of an fp32 value, wavefront/block scans for 64-wide wavefronts, and the
// "find the digit that holds the need-th largest entry" step of a radix select.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sbc {

// ---------------------------------------------------------------- layout ----

constexpr int kChunk = 8192;            // entries of one tensor handled by one workgroup
constexpr int kChunkWords = kChunk / 32; // bitmap words per chunk (= threads of a chunk kernel)
constexpr int kStreamThreads = 256;     // workgroup size of the streaming kernels
constexpr int kL1Bits = 10;             // first radix digit: sign, exponent, top mantissa bit
constexpr int kL1Bins = 1 << kL1Bits;
constexpr int kL1Shift = 32 - kL1Bits;
constexpr int kSelThreads = 1024;       // workgroup size of the per-tensor select kernel
constexpr int kDigBits = 11;            // later digits
constexpr int kDigBins = 1 << kDigBits;

// error bits raised by kernels (word 0 of the result block)
constexpr uint32_t kErrNonFinite = 1u;
constexpr uint32_t kErrInternal = 2u;
constexpr uint32_t kErrCorrupt = 4u;

// One tensor of the call, built on the host.
struct TensorDesc {
    const float* dW;
    float* R;           // residual in/out (compress) or accumulator (decode)
    uint32_t n;         // entries
    uint32_t k;         // entries kept per side
    uint32_t chunk0;    // first chunk of this tensor in the call-wide chunk numbering
    uint32_t nchunks;
    uint64_t cand_off;  // candidate list of the positive side starts here; negative side at +n
};

// Per-tensor results of the select stages, written on the device.
struct TensorState {
    uint32_t cand_cnt[2];  // candidates appended per side
    uint32_t bin[2];       // first-digit bin holding the k-th entry of each side (side key space)
    uint32_t above[2];     // entries in bins strictly above it
    uint32_t tau[2];       // full 32-bit threshold key per side
    uint32_t itau[2];      // ties at tau are kept up to this index
    double S[2];           // sum of the k kept values per side (negated on the negative side)
    int32_t side;          // +1 / -1
    float mu_signed;
    uint32_t nnz;
    uint32_t pad;
    uint64_t bit_len;
};

// Per-chunk summary of the kept-position bitmap.
struct ChunkSummary {
    uint32_t cnt;        // kept entries in the chunk
    uint32_t first;      // chunk-local position of the first one (undefined if cnt == 0)
    uint32_t last_end;   // chunk-local position of the last one plus 1 (0 if none)
    uint32_t inner_bits; // Golomb bits of all kept entries whose predecessor is in the chunk
};

// Result block copied back to the host after each call.
struct ResultBlock {
    uint32_t err;
    uint32_t pad;
    uint64_t msg_bytes;
};

// ------------------------------------------------------------------ keys ----

// Unsigned key with the same order as the fp32 value; -0.0 and +0.0 share a key.
__device__ __forceinline__ uint32_t key_of_bits(uint32_t u) {
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ uint32_t bits_of_key(uint32_t key) {
    return (key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key;
}

// ----------------------------------------------------------------- scans ----

template <typename T>
__device__ __forceinline__ T wave_incl_sum(T v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        T o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}

template <typename T>
__device__ __forceinline__ T wave_incl_max(T v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        T o = __shfl_up(v, d, 64);
        if (lane >= d && o > v) v = o;
    }
    return v;
}

// Exclusive prefix sum over the NT threads of a workgroup; *total receives the sum.
// smem: NT/64 elements of T.  Contains two barriers; every thread must call it.
template <typename T, int NT>
__device__ __forceinline__ T block_excl_sum(T v, T* total, T* smem) {
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    T inc = wave_incl_sum(v);
    if (lane == 63) smem[w] = inc;
    __syncthreads();
    T base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NT / 64; ++i) {
        T s = smem[i];
        if (i < w) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

// Exclusive prefix maximum (identity 0) over the NT threads of a workgroup.
template <typename T, int NT>
__device__ __forceinline__ T block_excl_max(T v, T* total, T* smem) {
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    T inc = wave_incl_max(v);
    T prev = __shfl_up(inc, 1, 64);
    if (lane == 0) prev = 0;
    if (lane == 63) smem[w] = inc;
    __syncthreads();
    T base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NT / 64; ++i) {
        T s = smem[i];
        if (i < w && s > base) base = s;
        if (s > tot) tot = s;
    }
    __syncthreads();
    *total = tot;
    return prev > base ? prev : base;
}

// Radix-select step.  hist (LDS, NB bins) counts entries per digit value; walking the digits
// from the top (REV = false) or from the bottom (REV = true), find the digit at which the
// running count first reaches `need` (1 <= need <= sum of hist).  res[0] receives that digit
// expressed in "top is largest" order (NB-1-digit when REV), res[1] the count strictly
// before it in walking order.  res[0] stays 0xFFFFFFFF if need exceeds the total.
// scratch: NT/64 words.  Contains barriers; every thread must call it.
template <int NB, int NT, bool REV>
__device__ __forceinline__ void find_from_top(const uint32_t* hist, uint32_t need, uint32_t* res,
                                              uint32_t* scratch) {
    constexpr int PER = (NB + NT - 1) / NT;
    const int t = threadIdx.x;
    if (t == 0) { res[0] = 0xFFFFFFFFu; res[1] = 0u; }
    uint32_t local = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int rb = t * PER + j;
        if (rb < NB) local += hist[REV ? rb : NB - 1 - rb];
    }
    uint32_t total;
    const uint32_t ex = block_excl_sum<uint32_t, NT>(local, &total, scratch);
    if (ex < need && need <= ex + local) {
        uint32_t cum = ex;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int rb = t * PER + j;
            if (rb < NB) {
                const uint32_t h = hist[REV ? rb : NB - 1 - rb];
                if (cum < need && cum + h >= need) { res[0] = NB - 1 - rb; res[1] = cum; }
                cum += h;
            }
        }
    }
    __syncthreads();
}

// Which tensor does call-wide chunk c belong to?  chunk_start has T+1 ascending entries.
__device__ __forceinline__ int tensor_of_chunk(const uint32_t* __restrict__ chunk_start, int T, uint32_t c) {
    int lo = 0, hi = T;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (chunk_start[mid] <= c) lo = mid; else hi = mid;
    }
    return lo;
}

}  // namespace sbc
