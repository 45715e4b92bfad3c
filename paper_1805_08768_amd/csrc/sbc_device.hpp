// Device-side building blocks shared by the SBC kernels: the order-preserving key of an
// fp32 value, wavefront/block scans for 64-wide wavefronts, and the byte-wise radix-select
// step that serves two independent selections (the two sign sides) at once.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sbc {

// Optional phase timestamps for tuning (build with -DSBC_PHASE_TIMING): thread 0 of the first
// 1024 workgroups of a kernel stores the 100 MHz wall clock into slot `i` of table `k`.
#ifdef SBC_PHASE_TIMING
__device__ unsigned long long g_phase_clock[3][1024][16];
#define SBC_TS(k, i) do { if (threadIdx.x == 0 && blockIdx.x < 1024) g_phase_clock[k][blockIdx.x][i] = wall_clock64(); } while (0)
#define SBC_TS_VAL(k, i, v) do { if (threadIdx.x == 0 && blockIdx.x < 1024) g_phase_clock[k][blockIdx.x][i] = (v); } while (0)
// the streaming kernel: every workgroup (up to 16384), eight stamps each
__device__ unsigned long long g_step_clock[16384][8];
#define SBC_STEP_TS(i) do { if (threadIdx.x == 0 && blockIdx.x < 16384) g_step_clock[blockIdx.x][i] = wall_clock64(); } while (0)
#define SBC_STEP_VAL(i, v) do { if (threadIdx.x == 0 && blockIdx.x < 16384) g_step_clock[blockIdx.x][i] = (v); } while (0)
#else
#define SBC_STEP_TS(i) do {} while (0)
#define SBC_STEP_VAL(i, v) do {} while (0)
#define SBC_TS(k, i) do {} while (0)
#define SBC_TS_VAL(k, i, v) do {} while (0)
#endif

// Pointers that a kernel reads out of a descriptor table reach the compiler as generic
// pointers, and it would use flat memory instructions for them: those are counted against the
// LDS counter as well, so the first use of any loaded value waits for every outstanding load
// and LDS operation.  Naming the global address space gives global_load / global_store.
#ifndef SBC_GLOBAL_AS
#define SBC_GLOBAL_AS __attribute__((address_space(1)))
typedef float f32x4 __attribute__((ext_vector_type(4)));
#endif
typedef SBC_GLOBAL_AS float* gfloat_ptr;
typedef const SBC_GLOBAL_AS float* gcfloat_ptr;
typedef SBC_GLOBAL_AS f32x4* gf32x4_ptr;
typedef const SBC_GLOBAL_AS f32x4* gcf32x4_ptr;
__device__ __forceinline__ gfloat_ptr as_global(float* p) { return (gfloat_ptr)p; }
__device__ __forceinline__ gcfloat_ptr as_global(const float* p) { return (gcfloat_ptr)p; }

// ---------------------------------------------------------------- layout ----

constexpr int kChunk = 8192;             // entries of one tensor handled by one workgroup
constexpr int kChunkWords = kChunk / 32; // bitmap words per chunk (= threads of a chunk kernel)
constexpr int kStreamThreads = 256;      // workgroup size of the streaming kernels
constexpr int kSampleThreads = 512;      // workgroup size of the sample kernel
constexpr int kSelThreads = 1024;        // workgroup size of the select kernel
constexpr int kSampleMax = 16384;        // entries sampled per tensor for the prefilter threshold
constexpr int kSampleWindow = 2048;      // leading-16-bit key values counted below the sample's extreme

// first digit of the histogram path: sign, exponent, top three mantissa bits
constexpr int kL1Bits = 12;
constexpr int kL1Bins = 1 << kL1Bits;
constexpr int kL1Shift = 32 - kL1Bits;

constexpr int kBucketBits = 11;          // index sort of the fused encoder: buckets by leading index bits
constexpr int kBuckets = 1 << kBucketBits;
constexpr uint32_t kFusedMaxK = 6144;    // a tensor with k up to this, and a stream bound of up to
constexpr uint32_t kFusedMaxWords = 4096; // this many words, is sorted and encoded inside the select kernel
// ... and so is one that keeps up to kFusedBigK entries, if that is below the threshold of the
// grid-wide kernels: beyond kSelLds kept entries the candidate lists cannot be staged in LDS,
// which leaves their space to the sort.  (One workgroup reads such lists from memory in every
// sweep; by default the grid-wide kernels take over from 8192 kept entries.)
constexpr uint32_t kFusedBigK = 16384;
constexpr int kFilterQueue = 1024;       // candidates per side a workgroup of the streaming kernel can queue in LDS
constexpr uint32_t kMaxChunksPerWorkgroup = 8;   // consecutive chunks of one very long tensor per such workgroup

// error bits raised by kernels (word 0 of the result block)
constexpr uint32_t kErrNonFinite = 1u;
constexpr uint32_t kErrInternal = 2u;
constexpr uint32_t kErrCorrupt = 4u;
constexpr uint32_t kErrOverflow = 128u;  // a candidate list of a compact context cannot hold what the histogram route extracts
constexpr uint32_t kErrPrefilter = 8u;   // not an error: some tensor needs the histogram path
constexpr uint32_t kErrWide = 32u;       // not an error: the grid-wide selection kernels completed some tensor
constexpr uint32_t kErrLoose = 16u;      // not an error: a carried-over filter key let far too many entries pass
constexpr uint32_t kErrStaleKeys = 256u; // not an error: the filter keys the previous call left would have let far too many entries pass now
constexpr uint32_t kErrDeferred = 64u;   // not an error: a tensor the streaming kernel could not finish itself is left to k_select

// Candidates per side beyond which a list counts as a flood (the next call then estimates its keys
// afresh): 16 k + 8192, but at most one entry in 16 of the tensor if that is above 8 k + 4096 (a
// workgroup of the streaming kernel queues up to 1024 candidates per side of its 8192 entries in
// LDS; beyond that it reads its chunk a second time).  Lists of a few times k are the normal
// state while a residual still builds up and cost a selection a few microseconds; a key that has
// fallen behind the data lets 30 to 60 times k pass.
__host__ __device__ inline unsigned long long loose_limit(uint32_t k, uint32_t n) {
    const unsigned long long lo = 8ull * k + 4096ull, hi = 16ull * k + 8192ull, dense = (unsigned long long)n / 16ull;
    const unsigned long long cap = dense > lo ? dense : lo;
    return hi < cap ? hi : cap;
}

// TensorDesc::flags
constexpr int kWindow = 2048;             // bins of the leading-bits histograms (k_select, grid-wide selection)
// Grid-wide selection, first histogram: the leading 19 key bits (1024 steps per octave) counted in a window of two octaves
// above the filter key.  Wider than k_select's half octave on purpose: a filter key carried over
// from the previous call may lie far below this call's k-th entry while the data still grows, and
// a tensor whose k-th entry lies beyond the window falls to one workgroup.
constexpr int kWideShift = 13;

// The window bin of a side key, given the side's filter key.
__device__ __forceinline__ uint32_t wide_window_bin(uint32_t key, uint32_t lo_key) {
    const uint32_t v = key >> kWideShift, base = lo_key >> kWideShift;
    const uint32_t o = v >= base ? v - base : 0u;       // (no candidate lies below its filter key)
    return o < (uint32_t)(kWindow - 1) ? o : (uint32_t)(kWindow - 1);
}

constexpr uint32_t kDescFused = 1u;      // sorted and encoded inside the select kernel
constexpr uint32_t kDescWide = 2u;       // keeps so many entries that the grid-wide selection kernels take it
constexpr uint32_t kDescSampled = 4u;    // subsampled variant: the sampled threshold decides what is kept
constexpr uint32_t kDescInline = 8u;     // finished inside the streaming kernel by the last of its workgroups
// TensorState::flags
constexpr uint32_t kStFailed = 1u;       // prefilter kept fewer than k candidates on a side
constexpr uint32_t kStExact = 2u;        // taken over by the histogram path
constexpr uint32_t kStWideDone = 4u;     // selected and applied by the grid-wide kernels
constexpr uint32_t kStInlineDone = 8u;   // selected and encoded inside the streaming kernel
constexpr uint32_t kStResidualDone = 16u; // ... which also applied the residual update (one-chunk tensors)
constexpr uint32_t kStDeferred = 32u;    // the streaming kernel left this tensor to k_select

// One tensor of the call, built on the host.
struct TensorDesc {
    const float* dW;
    float* R;             // residual, in/out
    uint32_t n;           // entries
    uint32_t k;           // entries kept per side
    uint32_t chunk0;      // first chunk of this tensor in the call-wide chunk numbering
    uint32_t nchunks;
    uint64_t cand_off;    // candidate list of the positive side starts here; negative side at +cand_cap
    uint64_t stage_off;   // first word of this tensor's stream in the staging area
    uint32_t bound_words; // worst-case stream length in words
    uint32_t kept_off;    // first entry of this tensor in the kept-index scratch
    uint32_t flags;
    uint32_t kcap;        // most entries a side may keep: k, or min(n, 2k + 64) in the subsampled variant
    uint32_t grp0;        // first of this tensor's chunk groups
    uint32_t cand_cap;    // entries each side's candidate list holds: n, or fewer in a compact context
};

// Per-tensor results, written on the device.
struct alignas(8) TensorState {
    uint32_t lo_key[2];    // prefilter: side keys at or above these become candidates
    uint32_t cand_cnt[2];  // candidates appended per side (8-byte aligned: advanced together as one u64)
    uint32_t bin[2];       // histogram path: first-digit bin holding the k-th entry of each side
    uint32_t tau[2];       // full 32-bit threshold key per side (side key space)
    uint32_t itau[2];      // ties at tau are kept up to this index
    uint32_t kc[2];        // entries kept per side: k, or the count the sampled threshold gave
    double S[2];           // sum of the kept values per side (negated on the negative side)
    int32_t side;          // +1 / -1
    float mu_signed;
    uint32_t nnz;
    uint32_t flags;
    uint64_t bit_len;
    uint32_t done;         // chunks (or groups of chunks) of this tensor that the streaming kernel has completed
    uint32_t pad;
    uint32_t cand_seen[2]; // candidates per side the finishing workgroup found (inspection)
    uint32_t expect[2];    // carried keys: entries per side known to lie at or beyond lo_key before the next update
                           // is added (0: not known)
};

// Per group of kGroupChunks consecutive chunks of a tensor that the streaming kernel finishes
// itself: how many of the group's chunks have been counted in (a first level, so that the
// workgroups of a large tensor do not all queue on one counter).
constexpr int kGroupChunks = 32;
constexpr int kMaxGroups = 64;           // groups of a tensor the streaming kernel finishes itself
struct alignas(16) GroupState {
    uint32_t done;
    uint32_t pad[3];
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

// Filter keys a following call may start from instead of sampling: this call's exact threshold,
// lowered by a margin that shrinks with k (the k-th order statistic of similar data moves by
// about 1/sqrt(k) of the tail's scale from round to round).  Only a filter: a tensor it
// misleads is noticed and redone through the histogram route.
__device__ __forceinline__ uint32_t carried_key(uint32_t tau_side_key, uint32_t k) {
    const float margin = fminf(0.25f, fmaxf(0.04f, 3.0f * rsqrtf((float)k)));
    const float x = __uint_as_float(bits_of_key(tau_side_key));       // how extreme the k-th entry is
    const float lo_x = x - margin * fabsf(x) - 1.17549435e-38f;
    const uint32_t lo = key_of_bits(__float_as_uint(lo_x));
    return lo > tau_side_key ? tau_side_key : lo;
}

// Rank of the entry whose key a following call starts from (see k_select): the k entries kept now
// are gone from above that key in the next call (on the side that is sent), and k more must
// remain even if the next update moves nothing across the key.
__device__ __forceinline__ uint32_t carried_rank(uint32_t k) {
    return 2u * k + 4u * (uint32_t)sqrtf((float)k) + 16u;
}
// The same when this call could see how many entries the update moved across the key it started
// from: `net` more than were known to lie beyond it (net < 0: fewer).  Half of that gain is
// counted on again; at least k / 8 entries beside the k-th stay in reserve.
__device__ __forceinline__ uint32_t carried_rank(uint32_t k, long long net) {
    long long spare = (long long)k - net / 2;
    const long long lo = (long long)(k / 8u), hi = 2ll * (long long)k;
    spare = spare < lo ? lo : (spare > hi ? hi : spare);
    return k + (uint32_t)spare + 4u * (uint32_t)sqrtf((float)k) + 16u;
}

// A side key moved towards less extreme values by the fraction `margin` of its value.
__device__ __forceinline__ uint32_t lowered_key(uint32_t side_key, float margin) {
    const float x = __uint_as_float(bits_of_key(side_key));
    const float lo_x = x - margin * fabsf(x) - 1.17549435e-38f;
    const uint32_t lo = key_of_bits(__float_as_uint(lo_x));
    return lo > side_key ? side_key : lo;
}

// Filter key for a following call when this call's candidate list (cnt entries at or beyond
// cur_side_key, the k-th of them at tau_side_key) is too short to hold the entry of rank r > k
// that the key should sit at.  The list says nothing about what lies below its own key, so the
// count above a value x is extrapolated as exp(-x / s).  If the list is clearly longer than k,
// s comes from the list itself (k entries above tau, cnt above the current key): the slope just
// below the k-th entry, where entries that were never sent pile up from round to round.
// Otherwise the whole side is taken as exponential (n / 2 entries in all), which gives
// s = tau / ln(n / 2k).  Only a filter: if the guess is too tight the histogram route redoes the
// tensor, if it is too loose the list is longer than it had to be.
__device__ __forceinline__ uint32_t extrapolated_key(uint32_t tau_side_key, uint32_t cur_side_key, uint32_t k,
                                                     uint32_t r, uint32_t n, uint32_t cnt) {
    const uint32_t zero_key = key_of_bits(0u);                          // every entry of the side's sign
    const float xt = __uint_as_float(bits_of_key(tau_side_key));        // how extreme the k-th entry is
    const float xc = __uint_as_float(bits_of_key(cur_side_key));        // and the current key
    if (!(xt > 0.f) || n <= 2u * r) return cur_side_key < zero_key ? cur_side_key : zero_key;
    float x;
    if (cnt >= k + k / 8u + 2u && cnt < r && xc > 0.f && xt > xc)
        x = xc - (xt - xc) * logf((float)r / (float)cnt) / logf((float)cnt / (float)k);
    else
        x = xt * (1.f - logf((float)r / (float)k) / logf((float)n / (float)(2u * k)));
    const uint32_t guess = x > 0.f ? key_of_bits(__float_as_uint(x)) : zero_key;
    return guess < cur_side_key ? guess : cur_side_key;
}

// ----------------------------------------------------------------- scans ----

// Wavefront scans through the data-parallel primitives of the vector ALU (a lane reads the
// register of another lane of its row of 16, or a row's last lane is broadcast to the rows after
// it) instead of the LDS crossbar: six steps of a few cycles each.  A lane without a source lane
// in a step receives the identity (0).
//   row_shr:d (d = 1, 2, 4, 8): lane i of a row reads lane i - d of the same row
//   row_bcast:15 to rows 1 and 3, row_bcast:31 to rows 2 and 3
template <int CTRL, int ROW_MASK, typename T>
__device__ __forceinline__ T dpp_fetch(T v) {
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "32- or 64-bit values");
    if constexpr (sizeof(T) == 4) {
        return (T)(uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, CTRL, ROW_MASK, 0xf, false);
    } else {
        const unsigned long long x = (unsigned long long)v;
        const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)x, CTRL, ROW_MASK, 0xf, false);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(x >> 32), CTRL, ROW_MASK, 0xf, false);
        return (T)(((unsigned long long)hi << 32) | lo);
    }
}

template <typename T>
__device__ __forceinline__ T wave_incl_sum(T v) {
    v += dpp_fetch<0x111, 0xf>(v);
    v += dpp_fetch<0x112, 0xf>(v);
    v += dpp_fetch<0x114, 0xf>(v);
    v += dpp_fetch<0x118, 0xf>(v);
    v += dpp_fetch<0x142, 0xa>(v);
    v += dpp_fetch<0x143, 0xc>(v);
    return v;
}

// (unsigned values: the identity 0 never wins)
template <typename T>
__device__ __forceinline__ T wave_incl_max(T v) {
    T o;
    o = dpp_fetch<0x111, 0xf>(v); v = o > v ? o : v;
    o = dpp_fetch<0x112, 0xf>(v); v = o > v ? o : v;
    o = dpp_fetch<0x114, 0xf>(v); v = o > v ? o : v;
    o = dpp_fetch<0x118, 0xf>(v); v = o > v ? o : v;
    o = dpp_fetch<0x142, 0xa>(v); v = o > v ? o : v;
    o = dpp_fetch<0x143, 0xc>(v); v = o > v ? o : v;
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

// Radix-select step over a wide digit (histogram path).  hist (LDS, NB bins) counts entries
// per digit value; walking the digits from the top (REV = false) or from the bottom
// (REV = true), find the digit at which the running count first reaches `need`
// (1 <= need <= sum of hist).  res[0] receives that digit expressed in "top is largest" order
// (NB-1-digit when REV), res[1] the count strictly before it in walking order.  res[0] stays
// 0xFFFFFFFF if need exceeds the total.  scratch: NT/64 words.  Contains barriers.
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

// Histogram update that first adds up runs of equal bins in a register: the leading bytes of
// floating-point keys take very few distinct values, and same-address LDS atomics serialize.
struct RunCounter {
    uint32_t bin = 0xFFFFFFFFu;
    uint32_t cnt = 0u;
    __device__ __forceinline__ void add(uint32_t* hist, uint32_t b) {
        if (b != bin) {
            if (cnt) atomicAdd(&hist[bin], cnt);
            bin = b; cnt = 0u;
        }
        ++cnt;
    }
    __device__ __forceinline__ void flush(uint32_t* hist) {
        if (cnt) atomicAdd(&hist[bin], cnt);
        cnt = 0u; bin = 0xFFFFFFFFu;
    }
};

// ------------------------------------------- byte-wise select, two at once ----
//
// The select and sample kernels look for the need-th largest 32-bit value of two independent
// collections (one per sign side) by fixing one byte per pass, most significant first.  For
// each pass the caller has filled hist[s][0..255] (LDS) with the counts of byte values among
// the entries of collection s that match the bytes fixed so far.  pick_byte_both finds, for
// both collections in one block scan, the byte value at which the count from the top reaches
// need[s]; it lowers need[s] by the count strictly above that byte and returns the byte and
// the number of entries holding it.  A collection that is not `active` is left alone.  If a
// need exceeds the total, found[s] stays false.  res: 8 words of LDS that nothing else touches
// until the caller's next barrier, scratch: NT/64 u64 (LDS).  Contains barriers; every thread
// must call it.
// Same for a wide digit: hist[s][0..NB-1], PER = NB/NT consecutive bins per thread.  If rank2
// is given, the same scan also finds the digit at which the count from the top reaches
// rank2[s] (digit2[s]; 0xFFFFFFFF if the total is smaller) if want2 is set; res2: two more words
// of LDS.  (Values and references, no pointers to the caller's arrays: those would live in memory.)
template <int NB, int NT>
__device__ __forceinline__ void pick_wide_both(const uint32_t (*hist)[NB], uint32_t (&need)[2],
                                               const bool (&active)[2], uint32_t* res,
                                               unsigned long long* scratch, uint32_t (&digit)[2], bool (&found)[2],
                                               bool want2, const uint32_t (&rank2)[2], uint32_t* res2,
                                               uint32_t (&digit2)[2]) {
    constexpr int PER = NB / NT;
    static_assert(PER >= 1 && PER * NT == NB, "bins divide evenly over the threads");
    const int t = threadIdx.x;
    if (t < 8) res[t] = (t & 3) == 0 ? 0xFFFFFFFFu : 0u;       // res[4*s + {0: digit, 1: above}]
    if (want2 && t < 2) res2[t] = 0xFFFFFFFFu;
    uint32_t h[2][PER], loc0 = 0u, loc1 = 0u;
#pragma unroll
    for (int j = 0; j < PER; ++j) {                            // walking from the top digit down
        h[0][j] = active[0] ? hist[0][NB - 1 - (t * PER + j)] : 0u;
        h[1][j] = active[1] ? hist[1][NB - 1 - (t * PER + j)] : 0u;
        loc0 += h[0][j]; loc1 += h[1][j];
    }
    unsigned long long total;
    const unsigned long long ex =
        block_excl_sum<unsigned long long, NT>((unsigned long long)loc0 | ((unsigned long long)loc1 << 32), &total, scratch);
    uint32_t cum[2] = {(uint32_t)ex, (uint32_t)(ex >> 32)};
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            if (active[s] && cum[s] < need[s] && need[s] <= cum[s] + h[s][j]) {
                res[4 * s] = (uint32_t)(NB - 1 - (t * PER + j)); res[4 * s + 1] = cum[s];
            }
            if (want2 && active[s] && cum[s] < rank2[s] && rank2[s] <= cum[s] + h[s][j])
                res2[s] = (uint32_t)(NB - 1 - (t * PER + j));
            cum[s] += h[s][j];
        }
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        digit[s] = res[4 * s];
        found[s] = active[s] && digit[s] != 0xFFFFFFFFu;
        if (found[s]) need[s] -= res[4 * s + 1];
        if (want2) digit2[s] = res2[s];
    }
}

template <int NB, int NT>
__device__ __forceinline__ void pick_wide_both(const uint32_t (*hist)[NB], uint32_t (&need)[2],
                                               const bool (&active)[2], uint32_t* res,
                                               unsigned long long* scratch, uint32_t (&digit)[2], bool (&found)[2]) {
    const uint32_t no_rank[2] = {0u, 0u};
    uint32_t no_digit[2];
    pick_wide_both<NB, NT>(hist, need, active, res, scratch, digit, found, false, no_rank, res, no_digit);
}

struct BytePick {
    uint32_t byte[2];
    uint32_t count[2];
    bool found[2];
};

template <int NT>
__device__ __forceinline__ BytePick pick_byte_both(const uint32_t (*hist)[256], uint32_t (&need)[2],
                                                   const bool (&active)[2], uint32_t* res,
                                                   unsigned long long* scratch) {
    static_assert(NT >= 256, "one thread per byte value");
    const int t = threadIdx.x;
    if (t < 8) res[t] = (t & 3) == 0 ? 0xFFFFFFFFu : 0u;       // res[4*s + {0: byte, 1: above, 2: count}]
    // (the finder threads write res only after the barriers of the scan below)
    uint32_t h0 = 0u, h1 = 0u;
    if (t < 256) { h0 = active[0] ? hist[0][255 - t] : 0u; h1 = active[1] ? hist[1][255 - t] : 0u; }
    unsigned long long total;
    const unsigned long long ex =
        block_excl_sum<unsigned long long, NT>((unsigned long long)h0 | ((unsigned long long)h1 << 32), &total, scratch);
    const uint32_t ex0 = (uint32_t)ex, ex1 = (uint32_t)(ex >> 32);
    if (t < 256) {
        if (active[0] && ex0 < need[0] && need[0] <= ex0 + h0) { res[0] = 255u - t; res[1] = ex0; res[2] = h0; }
        if (active[1] && ex1 < need[1] && need[1] <= ex1 + h1) { res[4] = 255u - t; res[5] = ex1; res[6] = h1; }
    }
    __syncthreads();
    BytePick p;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        p.byte[s] = res[4 * s]; p.count[s] = res[4 * s + 2];
        p.found[s] = active[s] && p.byte[s] != 0xFFFFFFFFu;
        if (p.found[s]) need[s] -= res[4 * s + 1];
        p.byte[s] &= 255u;
    }
    return p;
}

}  // namespace sbc
