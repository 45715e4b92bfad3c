// Alg. 2 in full, Alg. 1's residual line, and (for tensors of ordinary size) Alg. 3.
//
// k_select runs one workgroup per tensor and works on both sign sides together:
//   * a histogram of the leading key bits over a window above the filter key finds the bucket of
//     the k-th most extreme entry of each side; the few entries of that bucket are ranked
//     against each other by (key descending, index ascending), which yields the threshold key
//     tau and the highest index kept among entries equal to tau (equal values go to the lowest
//     index).  Tie-heavy data falls back to a byte-wise radix select (four passes) for tau and
//     a second one over the tied indices;
//   * S, the sum of the k kept values of a side, is accumulated as exact integers (mantissas
//     shifted to the threshold's scale in one 64-bit integer, or one integer per fp32 exponent
//     where that does not apply), so it does not depend on the order of the list, and is
//     rounded to fp64 in a fixed order.
// It then decides the side (positive iff mu+ >= mu-) and applies it:
//   * residual update R[j] = A[j] - mu_signed at the k kept entries;
//   * tensors flagged kDescFused: the kept indices are sorted in LDS (bucket by leading
//     index bits, rank inside the bucket), their gaps Golomb-coded into LDS words and the
//     stream written to the tensor's staging words;
//   * other tensors: bit j of the kept-position bitmap is set, and the bitmap kernels encode.
// Lists of up to kSelLds candidates per side are staged in LDS for all sweeps.
#pragma once

#include "sbc_device.hpp"

namespace sbc {

__device__ __forceinline__ uint32_t golomb_len(uint32_t gap, int b) { return (gap >> b) + 1u + (uint32_t)b; }

// val (< 2^nb, 1 <= nb <= 32) written MSB-first at bit `pos` of a zero-initialised word array.
__device__ __forceinline__ void put_bits(uint32_t* words, unsigned long long pos, uint32_t val, int nb) {
    const unsigned long long w = pos >> 5;
    const int off = (int)(pos & 31ull);
    const unsigned long long v = (unsigned long long)val << (64 - off - nb);
    const uint32_t hi = (uint32_t)(v >> 32), lo = (uint32_t)v;
    if (hi) atomicOr(&words[w], hi);
    if (lo) atomicOr(&words[w + 1], lo);
}

// q one-bits starting at bit `pos`.
__device__ __forceinline__ void put_ones(uint32_t* words, unsigned long long pos, unsigned long long q) {
    while (q) {
        const unsigned long long w = pos >> 5;
        const uint32_t room = 32u - (uint32_t)(pos & 31ull);
        const uint32_t take = q < room ? (uint32_t)q : room;
        if (take == 32u) words[w] = 0xFFFFFFFFu;        // the whole word belongs to this run
        else atomicOr(&words[w], ((1u << take) - 1u) << (room - take));
        pos += take;
        q -= take;
    }
}

constexpr uint32_t kSelLds = 8192;                       // candidates per side staged in LDS
constexpr int kWinShift = 11;                            // it counts key >> kWinShift: 2^12 steps per octave, half an octave
constexpr uint32_t kRankMax = 512;                       // threshold buckets up to this size are ranked directly
static_assert(2 * kFusedMaxK * 4 <= kSelLds * 8, "sort arrays reuse one side's candidate space");
static_assert(kFusedMaxWords <= kFusedMaxK, "stream words reuse the grouping array");
static_assert(kFusedBigK == 2 * kSelLds, "a large tensor's sort arrays take one side's candidate space each");

// Capacity (entries, and stream words + 1) of each of the two sort arrays of the fused encoder for
// a tensor that keeps k entries per side: lists that keep more than kSelLds entries are never
// staged in LDS, so both sides' space is free.
__host__ __device__ inline uint32_t fused_sort_capacity(uint32_t k) { return k > kSelLds ? 2u * kSelLds : kSelLds; }

struct SelectShared {
    uint2 cand[2][kSelLds];                              // both sides' lists when they fit
    union {
        uint32_t whist[2][kWindow];                     // leading 21 key bits, as an offset from the filter key
        struct {
            uint32_t hist[4][2][256];                    // byte histograms: [pass][side][byte]
            long long acc[2][256];                       // per-exponent integer sums
        };
        struct {                                         // the entries sharing the threshold's leading 16 bits,
            uint2 bucket[2][kRankMax];                   // and how many of them rank ahead of each
            uint32_t ahead[2][kRankMax];
        };
        struct {                                         // index sort, after the side is decided
            uint32_t bucket_cnt[kBuckets];               // entries per bucket, then offsets
            uint32_t bucket_fill[kBuckets];
        };
    };
    uint32_t res[4][8];
    uint32_t scratch[kSelThreads / 64];
    unsigned long long scratch64[kSelThreads / 64];
    long long fast_sum[2][kSelThreads / 64];             // per-wavefront partial sums of the common-scale path
    uint32_t any_slow;                                   // some kept entry does not fit the common-scale sum
    double S[2];
};

// The candidate lists of a tensor: (side key, index) pairs, staged in LDS when both sides fit,
// else read from global memory in every sweep.  Sweeps are loops with a small unroll factor on
// purpose: every workgroup executes this kernel's code only once, so the code must stay small
// enough to stream through the instruction cache, while a few loads in flight hide latency.
struct CandLists {
    const uint2* g[2];
    uint32_t cnt[2];
    bool staged;
};

template <int S, typename F>
__device__ __forceinline__ void sweep(const SelectShared& sh, const CandLists& l, F f) {
    if (l.staged) {
        const uint2* p = sh.cand[S];                    // LDS
#pragma unroll 4
        for (uint32_t i = threadIdx.x; i < l.cnt[S]; i += kSelThreads) f(p[i]);
    } else {
        const uint2* __restrict__ p = l.g[S];           // global
#pragma unroll 8
        for (uint32_t i = threadIdx.x; i < l.cnt[S]; i += kSelThreads) f(p[i]);
    }
}

__device__ __forceinline__ bool cand_kept(uint32_t key, uint32_t idx, uint32_t tau, uint32_t itau) {
    return key > tau || (key == tau && idx <= itau);
}

// The need[s]-th largest value over the entries of side s, for both sides at once, one byte per
// pass.  mode 0 ranks side keys over all entries; mode 1 ranks complemented indices over the
// entries whose key equals tie_key[s] (the lowest indices among ties).  Returns the values in
// out[s]; last[s] is the number of entries equal to out[s]; need[s] ends as the rank of the
// wanted entry among those equals.  A side that is not active is skipped.  Returns false if a
// need exceeded a side's population.  Contains barriers; every thread must call it.
template <int S>
__device__ __forceinline__ void byte_histogram(SelectShared& sh, const CandLists& l, int pass, int mode,
                                               uint32_t pfx, uint32_t tk) {
    const int shift = 24 - 8 * pass;
    RunCounter rc;
    uint32_t* h = sh.hist[pass][S];
    sweep<S>(sh, l, [&](const uint2& e) {
        const uint32_t v = mode ? ~e.y : e.x;
        if ((!mode || e.x == tk) && (pass == 0 || (v >> (shift + 8)) == pfx)) rc.add(h, (v >> shift) & 255u);
    });
    rc.flush(h);
}

// Side s takes part in byte passes first_pass[s]..3; prefix[s] holds the bytes fixed before.
__device__ __forceinline__ bool select_both(SelectShared& sh, const CandLists& l, uint32_t (&need)[2],
                                            const bool (&active)[2], int mode, const uint32_t (&tie_key)[2],
                                            const int (&first_pass)[2], uint32_t (&prefix)[2],
                                            uint32_t (&out)[2], uint32_t (&last)[2]) {
    bool ok = true;
    for (int i = threadIdx.x; i < 4 * 2 * 256; i += kSelThreads) (&sh.hist[0][0][0])[i] = 0u;
    __syncthreads();
#pragma nounroll
    for (int pass = 0; pass < 4; ++pass) {
        const bool act[2] = {active[0] && pass >= first_pass[0], active[1] && pass >= first_pass[1]};
        if (!act[0] && !act[1]) continue;
        if (act[0]) byte_histogram<0>(sh, l, pass, mode, prefix[0], tie_key[0]);
        if (act[1]) byte_histogram<1>(sh, l, pass, mode, prefix[1], tie_key[1]);
        __syncthreads();
        const BytePick pk = pick_byte_both<kSelThreads>(sh.hist[pass], need, act, sh.res[pass], sh.scratch64);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (!act[s]) continue;
            if (!pk.found[s]) ok = false;
            prefix[s] = (prefix[s] << 8) | pk.byte[s];
            last[s] = pk.count[s];
        }
    }
    __syncthreads();                                  // hist and res may be reused by the next selection
    out[0] = prefix[0]; out[1] = prefix[1];
    return ok;
}

// Exact sum of the kept values of side S (of -A on the negative side), in two parts.  If
// `common` is set, every kept entry has the sign of its side and a biased exponent of at least
// e_ref, and there are at most 2^15 of them: an entry whose exponent exceeds e_ref by at most
// 24 is added, shifted to the scale of e_ref, to a 64-bit integer the thread keeps in a
// register (24 + 24 + 15 bits at most).  Every other entry goes to acc[S][exponent], exact
// integers per fp32 exponent in LDS; a thread first adds up runs of equal exponent in a
// register.  SLOW = false: only the first part; returns the integer and raises sh.any_slow if
// an entry belongs to the second part.  SLOW = true: only the second part.
template <int S, bool SLOW>
__device__ __forceinline__ long long exponent_sums(SelectShared& sh, const CandLists& l, uint32_t tk, uint32_t ti,
                                                   bool common, uint32_t e_ref) {
    uint32_t cur_ex = 0u;
    long long cur = 0ll, scaled = 0ll;
    sweep<S>(sh, l, [&](const uint2& e) {
        if (cand_kept(e.x, e.y, tk, ti)) {
            const uint32_t u = bits_of_key(S ? ~e.x : e.x);
            uint32_t ex = (u >> 23) & 0xFFu;
            long long m = (long long)(ex ? ((u & 0x7FFFFFu) | 0x800000u) : (u & 0x7FFFFFu));
            if (ex == 0u) ex = 1u;
            const bool fits = common && ex >= e_ref && ex - e_ref <= 24u;
            if (!SLOW) {
                if (fits) scaled += m << (ex - e_ref);
                else sh.any_slow = 1u;
                return;
            }
            if (fits) return;
            if (((u >> 31) != 0u) != (S != 0)) m = -m;           // the negative side sums -A
            if (ex != cur_ex) {
                if (cur != 0ll) atomicAdd(reinterpret_cast<unsigned long long*>(&sh.acc[S][cur_ex]), (unsigned long long)cur);
                cur_ex = ex; cur = 0ll;
            }
            cur += m;
        }
    });
    if (cur != 0ll) atomicAdd(reinterpret_cast<unsigned long long*>(&sh.acc[S][cur_ex]), (unsigned long long)cur);
    return scaled;
}

// What a tensor's candidate counts rule out before any selection: true if the tensor cannot be
// selected from its lists (the thread with `lead` set has then flagged it, for the histogram route
// or as an error).
__device__ __forceinline__ bool lists_unusable(const TensorDesc& d, TensorState* __restrict__ st, int t, uint32_t cnt_p,
                                               uint32_t cnt_n, int pass, bool lead, ResultBlock* __restrict__ result) {
    const bool sampled = (d.flags & kDescSampled) != 0u;
    if (cnt_p > d.n || cnt_n > d.n || (sampled && (cnt_p == 0u || cnt_n == 0u))) {
        // (a sampled threshold is the key of an entry of the tensor, so that entry is a candidate)
        if (lead) atomicOr(&result->err, kErrInternal);
        return true;
    }
    if (cnt_p > d.cand_cap || cnt_n > d.cand_cap) {
        // compact context: more candidates than a list holds (nothing was stored beyond its end).  The
        // histogram route extracts a tighter set; if that does not fit either, the call fails.
        if (lead) {
            st[t].flags = kStFailed;
            st[t].bit_len = 0ull; st[t].nnz = 0u;
            atomicOr(&result->err, pass == 0 && !sampled ? kErrPrefilter : kErrOverflow);
        }
        return true;
    }
    if (!sampled && (cnt_p < d.k || cnt_n < d.k)) {
        // the filter kept too few entries on a side: the histogram path redoes this tensor
        if (lead) {
            st[t].flags = kStFailed;
            st[t].bit_len = 0ull; st[t].nnz = 0u;
            atomicOr(&result->err, pass == 0 ? kErrPrefilter : kErrInternal);
        }
        return true;
    }
    return false;
}

// One workgroup per tensor; `order` lists the tensors by decreasing size so that the
// long-running workgroups start first.  pass 0: every tensor; pass 1: only tensors handed to
// the histogram path (kStExact).
__global__ __launch_bounds__(kSelThreads) void k_select(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ order,
        TensorState* __restrict__ st, const uint2* __restrict__ cand, uint32_t* __restrict__ bitmap,
        uint32_t* __restrict__ stage, uint32_t* __restrict__ kept_idx, int b, int pass, int carry,
        ResultBlock* __restrict__ result) {
    __shared__ SelectShared sh;
    SBC_TS(1, 0);
    const int t = (int)order[blockIdx.x], tid = threadIdx.x;
    if (tid == 0) sh.any_slow = 0u;
    // (the descriptor and the state words go out together: one round trip instead of three)
    const TensorDesc d = desc[t];
    const uint32_t st_flags = st[t].flags;
    const uint32_t cnt_p = __builtin_amdgcn_readfirstlane(st[t].cand_cnt[0]);
    const uint32_t cnt_n = __builtin_amdgcn_readfirstlane(st[t].cand_cnt[1]);
    const uint32_t lo_key_p = st[t].lo_key[0], lo_key_n = st[t].lo_key[1];
    const uint32_t expect_p = st[t].expect[0], expect_n = st[t].expect[1];
    if (pass == 1 && !(st_flags & (kStExact | kStDeferred))) return;
    if (pass == 0 && (d.flags & kDescWide) && (st_flags & kStWideDone)) return;   // done by the grid-wide kernels
    if (pass == 0 && (st_flags & kStInlineDone)) return;                          // done by the streaming kernel
    const uint32_t k = d.k, n = d.n;
    const bool sampled = (d.flags & kDescSampled) != 0u;
    if (lists_unusable(d, st, t, cnt_p, cnt_n, pass, tid == 0, result)) return;
    if (tid == 0) { st[t].cand_seen[0] = cnt_p; st[t].cand_seen[1] = cnt_n; }    // (inspection only)
    SBC_TS(1, 1);                                     // descriptor and counts read
    SBC_TS_VAL(1, 13, cnt_p); SBC_TS_VAL(1, 14, cnt_n); SBC_TS_VAL(1, 15, (unsigned)t);
    CandLists list;
    list.g[0] = cand + d.cand_off; list.cnt[0] = cnt_p;
    list.g[1] = cand + d.cand_off + d.cand_cap; list.cnt[1] = cnt_n;
    list.staged = cnt_p <= kSelLds && cnt_n <= kSelLds;

    // Leading 21 key bits of the k-th most extreme entry of each side.  Every candidate's key is at
    // or above the side's filter key, and the k-th lies close above it, so a window of kWindow
    // values of (key >> kWinShift) starting at the filter key's is histogrammed in the same sweep
    // that stages the lists in LDS; the top bin collects everything beyond the window.
    // Entries kept per side: k; in the subsampled variant every candidate (all entries at or beyond
    // the sampled threshold), up to the cap.  If no side exceeds the cap there is nothing to select.
    const uint32_t kc[2] = {sampled ? min(cnt_p, d.kcap) : k, sampled ? min(cnt_n, d.kcap) : k};
    const bool pick = !sampled || cnt_p > d.kcap || cnt_n > d.kcap;
    uint32_t need[2] = {kc[0], kc[1]}, tau[2] = {0u, 0u};
    const bool both[2] = {true, true};
    const uint32_t wbase[2] = {lo_key_p >> kWinShift, lo_key_n >> kWinShift};
    bool ok = true;
    for (int i = tid; i < 2 * kWindow; i += kSelThreads) (&sh.whist[0][0])[i] = 0u;
    __syncthreads();
    auto count = [&](int s, const uint2& e) {
        const uint32_t v = e.x >> kWinShift;
        const uint32_t o = v >= wbase[s] ? v - wbase[s] : 0u;   // (no candidate lies below its filter key)
        atomicAdd(&sh.whist[s][o < (uint32_t)(kWindow - 1) ? o : (uint32_t)(kWindow - 1)], 1u);
    };
    if (list.staged) {
        // every load of both lists is issued before the first entry is used: the lists were written
        // by other compute units a moment ago, and each dependent round trip costs a microsecond
        constexpr int PER = kSelLds / kSelThreads;      // 8
        uint2 e[2][PER];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const uint2* __restrict__ g = list.g[s];
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                const uint32_t i = (uint32_t)j * kSelThreads + tid;
                e[s][j] = g[i < list.cnt[s] ? i : 0u];
            }
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                const uint32_t i = (uint32_t)j * kSelThreads + tid;
                if (i < list.cnt[s]) { sh.cand[s][i] = e[s][j]; if (pick) count(s, e[s][j]); }
            }
        }
    } else if (pick) {
        sweep<0>(sh, list, [&](const uint2& e) { count(0, e); });
        sweep<1>(sh, list, [&](const uint2& e) { count(1, e); });
    }
    __syncthreads();
    SBC_TS(1, 2);                                     // staged, leading bits counted
    uint32_t digit[2] = {0u, 0u};
    bool found[2] = {false, false};
    uint32_t bsize[2] = {0u, 0u};
    // Filter keys a following call may start from instead of sampling.  With the residual carried
    // over, the k-th entry sits at the edge of a cliff (everything above it has just been cut down
    // to about mu), so a margin in value below it lets a flood of entries pass, while a margin in
    // rank does not: the key is the lower edge of the window bin of this call's r-th most extreme
    // entry, r = 2 k + 4 sqrt(k) + 16 (if the next update is small beside the residual, the k
    // entries kept now are gone from above that key, and k more must remain).  A list shorter
    // than r says nothing about that entry: its place is extrapolated from the k-th.
    // (a call that started from carried keys sees how many entries its update moved across them,
    // and counts on half as many again: see carried_rank)
    const bool net_known = pass == 0 && carry && expect_p != 0u && expect_n != 0u;
    const uint32_t rank2[2] = {net_known ? carried_rank(k, (long long)cnt_p - (long long)expect_p) : carried_rank(k),
                               net_known ? carried_rank(k, (long long)cnt_n - (long long)expect_n) : carried_rank(k)};
    uint32_t digit2[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
    if (pick) {
        pick_wide_both<kWindow, kSelThreads>(sh.whist, need, both, sh.res[0], sh.scratch64, digit, found,
                                             carry != 0, rank2, sh.res[1], digit2);
        // entries in each side's threshold bucket (same leading key bits as the k-th entry)
#pragma unroll
        for (int s = 0; s < 2; ++s) bsize[s] = found[s] ? sh.whist[s][digit[s]] : 0u;
    }
    __syncthreads();                                  // whist shares its space with what follows
    if (pick && !list.staged && found[0] && found[1] && digit[0] != (uint32_t)(kWindow - 1) &&
        digit[1] != (uint32_t)(kWindow - 1)) {
        // Lists too long for LDS: nothing below the threshold's bucket matters any more, and what
        // lies in or above it usually fits.  One more sweep over global memory copies that part,
        // and every later sweep runs in LDS.
        const uint32_t keep[2] = {kc[0] - need[0] + bsize[0], kc[1] - need[1] + bsize[1]};
        if (keep[0] <= kSelLds && keep[1] <= kSelLds) {        // uniform
            if (tid < 2) sh.res[3][tid] = 0u;
            __syncthreads();
            auto copy_in = [&](int sd, const uint2& e) {
                if ((e.x >> kWinShift) >= wbase[sd] + digit[sd]) {
                    const uint32_t q = atomicAdd(&sh.res[3][sd], 1u);
                    if (q < kSelLds) sh.cand[sd][q] = e;
                }
            };
            sweep<0>(sh, list, [&](const uint2& e) { copy_in(0, e); });
            sweep<1>(sh, list, [&](const uint2& e) { copy_in(1, e); });
            __syncthreads();
            if (sh.res[3][0] != keep[0] || sh.res[3][1] != keep[1]) ok = false;   // cannot happen
            list.cnt[0] = keep[0]; list.cnt[1] = keep[1];
            list.staged = true;
        }
    }
    SBC_TS(1, 3);
    uint32_t itau[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
    const bool rankable = found[0] && found[1] && digit[0] != (uint32_t)(kWindow - 1) &&
                          digit[1] != (uint32_t)(kWindow - 1) && bsize[0] <= kRankMax && bsize[1] <= kRankMax;
    if (!pick) {
        // every candidate is kept: the filter key serves as the threshold (no candidate lies below it)
        tau[0] = lo_key_p; tau[1] = lo_key_n;
    } else if (rankable) {
        // The usual case: few entries share the threshold's leading bits.  They are copied out,
        // and every thread ranks one of them against the others by (key descending, index
        // ascending); the entry of rank need - 1 is the k-th of its side, ties included.
        if (tid < 4) { sh.res[1][tid] = 0u; sh.res[2][tid] = 0u; }
        for (int i = tid; i < 2 * (int)kRankMax; i += kSelThreads) (&sh.ahead[0][0])[i] = 0u;
        __syncthreads();
        auto copy_out = [&](int sd, const uint2& e) {
            if ((e.x >> kWinShift) == wbase[sd] + digit[sd]) {
                const uint32_t q = atomicAdd(&sh.res[1][sd], 1u);
                if (q < kRankMax) sh.bucket[sd][q] = e;
            }
        };
        sweep<0>(sh, list, [&](const uint2& e) { copy_out(0, e); });
        sweep<1>(sh, list, [&](const uint2& e) { copy_out(1, e); });
        __syncthreads();
        SBC_TS_VAL(1, 13, cnt_p | ((unsigned long long)sh.res[1][0] << 32)); SBC_TS_VAL(1, 14, cnt_n | ((unsigned long long)sh.res[1][1] << 32));
#pragma unroll
        for (int sd = 0; sd < 2; ++sd) {
            const uint32_t m = sh.res[1][sd];
            if (m != bsize[sd] || m == 0u || m > kRankMax) { ok = false; continue; }   // uniform; cannot happen
            // M = m rounded up to a power of two; kSelThreads / M threads share the work on one entry
            const uint32_t M = m > 1u ? 1u << (32 - __clz((int)(m - 1u))) : 1u;
            const uint32_t parts = (uint32_t)kSelThreads / M, i = (uint32_t)tid & (M - 1u), part = (uint32_t)tid / M;
            if (i < m) {
                // one 64-bit comparison per pair: key descending, then index ascending
                const uint2 me2 = sh.bucket[sd][i];
                const unsigned long long me = ((unsigned long long)me2.x << 32) | (uint32_t)~me2.y;
                uint32_t ahead = 0u;
                // this thread's share of the others: a contiguous range, eight LDS reads in flight
                const uint32_t len = (m + parts - 1u) / parts;
                const uint32_t j_end = min(m, (part + 1u) * len);
                for (uint32_t j0 = part * len; j0 < j_end; j0 += 8u) {
                    uint2 o[8];
#pragma unroll
                    for (uint32_t u = 0; u < 8u; ++u) o[u] = sh.bucket[sd][min(j0 + u, kRankMax - 1u)];
#pragma unroll
                    for (uint32_t u = 0; u < 8u; ++u)
                        ahead += (j0 + u < j_end && (((unsigned long long)o[u].x << 32) | (uint32_t)~o[u].y) > me) ? 1u : 0u;
                }
                if (ahead) atomicAdd(&sh.ahead[sd][i], ahead);
            }
        }
        __syncthreads();
#pragma unroll
        for (int sd = 0; sd < 2; ++sd) {
            if (ok && (uint32_t)tid < bsize[sd] && sh.ahead[sd][tid] + 1u == need[sd]) {
                const uint2 me = sh.bucket[sd][tid];
                sh.res[2][2 * sd] = me.x; sh.res[2][2 * sd + 1] = me.y; sh.res[1][2 + sd] = 1u;
            }
        }
        __syncthreads();
#pragma unroll
        for (int sd = 0; sd < 2; ++sd) {
            tau[sd] = sh.res[2][2 * sd]; itau[sd] = sh.res[2][2 * sd + 1];
            if (sh.res[1][2 + sd] != 1u) ok = false;
        }
        __syncthreads();                              // the bucket space is reused below
    } else {
        // Tie-heavy data, or a k-th entry beyond the window: tau byte by byte from the top, then
        // (second round, only if some ties must be dropped) the r lowest indices among the
        // entries equal to tau.
        bool active[2] = {true, true};
        int first_pass[2];
        uint32_t prefix[2], tie_key[2] = {0u, 0u};
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            first_pass[s] = 0; prefix[s] = 0u; need[s] = kc[s];
        }
#pragma nounroll
        for (int mode = 0; mode < 2; ++mode) {
            uint32_t out[2], last[2] = {0u, 0u};
            ok = select_both(sh, list, need, active, mode, tie_key, first_pass, prefix, out, last) && ok;
            if (mode == 0) {
                // need[s] is now the number r of entries equal to tau[s] that are kept (1 <= r <= ties)
                bool any = false;
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    tau[s] = out[s];
                    active[s] = ok && need[s] < last[s];      // fewer than all ties are kept
                    any = any || active[s];
                    tie_key[s] = tau[s]; first_pass[s] = 0; prefix[s] = 0u;
                }
                if (!any) break;
            } else {
                // the r-th largest complemented index among the ties
#pragma unroll
                for (int s = 0; s < 2; ++s) if (active[s]) itau[s] = ~out[s];
            }
        }
    }

    SBC_TS(1, 4);                                     // tau and tie index known
    // S+ and S-.  Usual case: every kept entry of a side fits one common-scale 64-bit integer sum;
    // the per-exponent accumulators are brought in only for what does not.
    // common-scale path: the k-th entry of a side has the side's sign (so have all kept ones)
    const bool common[2] = {kc[0] <= 32768u && tau[0] > 0x80000000u, kc[1] <= 32768u && tau[1] >= 0x80000000u};
    uint32_t e_ref[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint32_t ex = (bits_of_key(s ? ~tau[s] : tau[s]) >> 23) & 0xFFu;
        e_ref[s] = ex ? ex : 1u;
    }
    {
        long long part[2];
        part[0] = common[0] ? exponent_sums<0, false>(sh, list, tau[0], itau[0], true, e_ref[0]) : 0ll;
        part[1] = common[1] ? exponent_sums<1, false>(sh, list, tau[1], itau[1], true, e_ref[1]) : 0ll;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            // (integer sums wrap consistently: the scan's last lane holds the wavefront's total)
            const long long total = (long long)wave_incl_sum<unsigned long long>((unsigned long long)part[s]);
            if ((tid & 63) == 63) sh.fast_sum[s][tid >> 6] = total;
        }
    }
    __syncthreads();
    double Ssum[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        long long total = 0ll;
#pragma unroll
        for (int w = 0; w < kSelThreads / 64; ++w) total += sh.fast_sum[s][w];
        Ssum[s] = ldexp((double)total, (int)e_ref[s] - 150);
    }
    if (!common[0] || !common[1] || sh.any_slow) {       // uniform
        for (int i = tid; i < 512; i += kSelThreads) (&sh.acc[0][0])[i] = 0ll;
        __syncthreads();
        (void)exponent_sums<0, true>(sh, list, tau[0], itau[0], common[0], e_ref[0]);
        (void)exponent_sums<1, true>(sh, list, tau[1], itau[1], common[1], e_ref[1]);
        __syncthreads();
        if (tid < 128) {
            // fixed order: lane l of wavefront s adds exponents 4l..4l+3 ascending, then a fixed
            // shuffle tree; the common-scale integer is added last
            const int s = tid >> 6, lane = tid & 63;
            double v = 0.0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int ex = 4 * lane + j;
                v += ldexp((double)sh.acc[s][ex], ex - 150);
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
            if (lane == 0) sh.S[s] = v;
        }
        __syncthreads();
        Ssum[0] = sh.S[0] + Ssum[0];
        Ssum[1] = sh.S[1] + Ssum[1];
    }
    SBC_TS(1, 5);                                     // sums done
    const double Sp = Ssum[0], Sn = Ssum[1];
    // Alg. 2 compares the means (sums that differ may still give equal means: the positive side then)
    const int chosen = (Sp / (double)kc[0] >= Sn / (double)kc[1]) ? 0 : 1;
    const uint32_t kk = chosen ? kc[1] : kc[0];       // entries this tensor sends
    const float mu32 = (float)((chosen ? Sn : Sp) / (double)kk);
    const float mu_signed = chosen ? -mu32 : mu32;
    if (tid == 0) {
        st[t].tau[0] = tau[0]; st[t].tau[1] = tau[1];
        st[t].itau[0] = itau[0]; st[t].itau[1] = itau[1];
        st[t].kc[0] = kc[0]; st[t].kc[1] = kc[1];
        st[t].S[0] = Sp; st[t].S[1] = Sn;
        st[t].side = chosen ? -1 : 1;
        st[t].mu_signed = mu_signed;
        if (!ok) atomicOr(&result->err, kErrInternal);
        // filter keys a following round may start from instead of sampling
        if (carry) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const bool ranked = digit2[s] != 0xFFFFFFFFu;
                st[t].lo_key[s] = ranked ? (wbase[s] + digit2[s]) << kWinShift
                                         : extrapolated_key(tau[s], s ? lo_key_n : lo_key_p, k, rank2[s], n, s ? cnt_n : cnt_p);
                // at least rank2[s] entries lie at or beyond that key now; the side that is sent loses k of them
                st[t].expect[s] = ranked ? rank2[s] - (s == chosen ? kk : 0u) : 0u;
            }
        }
        // many times more candidates than needed: the next call should estimate its keys afresh
        // (lists somewhat too long for LDS only cost one more sweep here)
        const unsigned long long many = loose_limit(k, n);
        if (cnt_p > many || cnt_n > many) atomicOr(&result->err, kErrLoose);
    }
    if (!ok) return;

    const uint32_t ktau = chosen ? tau[1] : tau[0], kitau = chosen ? itau[1] : itau[0];
    // one sweep over the chosen side's list
    auto sweep_kept = [&](auto f) {
        if (chosen) sweep<1>(sh, list, [&](const uint2& e) { if (cand_kept(e.x, e.y, ktau, kitau)) f(e); });
        else sweep<0>(sh, list, [&](const uint2& e) { if (cand_kept(e.x, e.y, ktau, kitau)) f(e); });
    };
    const gfloat_ptr R = as_global(d.R);

    if (!(d.flags & kDescFused)) {
        // residual update; positions go to the bitmap
        uint32_t* __restrict__ bm = bitmap + (uint64_t)d.chunk0 * kChunkWords;
        sweep_kept([&](const uint2& e) {
            if (e.y >= n) { atomicOr(&result->err, kErrInternal); return; }
            const float a = __uint_as_float(bits_of_key(chosen ? ~e.x : e.x));
            R[e.y] = a - mu_signed;
            atomicOr(&bm[e.y >> 5], 1u << (e.y & 31u));
        });
        return;
    }

    SBC_TS(1, 6);
    // ---- fused: sort the k kept indices, encode their gaps (Alg. 3), write the stream ----
    // the LDS space of the side that was not chosen holds the sort arrays
    // (both sides' space if the lists are read from memory: see fused_sort_capacity)
    const uint32_t sort_cap = list.staged ? kSelLds : 2u * kSelLds;
    uint32_t* grp = reinterpret_cast<uint32_t*>(list.staged ? sh.cand[chosen ^ 1] : sh.cand[0]);   // kept indices grouped by bucket
    uint32_t* sorted = grp + sort_cap;                                  // kept indices ascending
    if (kk > sort_cap) {                              // uniform; cannot happen: staged lists hold at most kSelLds entries
        if (tid == 0) atomicOr(&result->err, kErrInternal);
        return;
    }
    int shift = 32 - __clz((int)(n - 1u | 1u)) - kBucketBits;           // bucket = idx >> shift, below kBuckets
    if (shift < 0) shift = 0;
    for (int i = tid; i < kBuckets; i += kSelThreads) { sh.bucket_cnt[i] = 0u; sh.bucket_fill[i] = 0u; }
    __syncthreads();
    sweep_kept([&](const uint2& e) {
        if (e.y < n) atomicAdd(&sh.bucket_cnt[e.y >> shift], 1u);
    });
    __syncthreads();
    SBC_TS(1, 7);                                     // buckets counted
    {   // exclusive scan of the bucket counts, in place: consecutive buckets per thread
        constexpr int PB = kBuckets / kSelThreads;
        uint32_t loc[PB], sum = 0u;
#pragma unroll
        for (int j = 0; j < PB; ++j) { loc[j] = sh.bucket_cnt[tid * PB + j]; sum += loc[j]; }
        uint32_t total;
        uint32_t ex = block_excl_sum<uint32_t, kSelThreads>(sum, &total, sh.scratch);
#pragma unroll
        for (int j = 0; j < PB; ++j) { sh.bucket_cnt[tid * PB + j] = ex; ex += loc[j]; }
        if (total != kk) {                            // uniform: every thread sees the same total
            if (tid == 0) atomicOr(&result->err, kErrInternal);
            return;
        }
    }
    __syncthreads();
    sweep_kept([&](const uint2& e) {
        if (e.y < n) {
            const uint32_t bk = e.y >> shift;
            grp[sh.bucket_cnt[bk] + atomicAdd(&sh.bucket_fill[bk], 1u)] = e.y;
            const float a = __uint_as_float(bits_of_key(chosen ? ~e.x : e.x));
            R[e.y] = a - mu_signed;                   // Alg. 1: R <- dW - dW*
        }
    });
    __syncthreads();
    SBC_TS(1, 8);                                     // grouped, residual updated
    for (uint32_t i = tid; i < kk; i += kSelThreads) {
        const uint32_t v = grp[i];
        const uint32_t bk = v >> shift;
        const uint32_t lo = sh.bucket_cnt[bk], hi = lo + sh.bucket_fill[bk];
        uint32_t rank = 0u;
        for (uint32_t j = lo; j < hi; ++j) rank += (grp[j] < v) ? 1u : 0u;
        sorted[lo + rank] = v;
    }
    __syncthreads();

    SBC_TS(1, 9);                                     // sorted
    // Golomb code lengths of E consecutive entries per thread, then their bit offsets
    const uint32_t E = (kk + kSelThreads - 1) / kSelThreads;
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
    unsigned long long pos = block_excl_sum<unsigned long long, kSelThreads>(bits, &total_bits, sh.scratch64);
    const uint32_t n_words = (uint32_t)((total_bits + 31ull) >> 5);
    if (n_words > d.bound_words || n_words + 1u > sort_cap) {    // uniform; cannot happen
        if (tid == 0) atomicOr(&result->err, kErrInternal);
        return;
    }
    SBC_TS(1, 10);
    uint32_t* words = grp;                            // the grouping array is free again
    for (uint32_t w = tid; w < n_words + 1u; w += kSelThreads) words[w] = 0u;
    __syncthreads();
    {
        uint32_t pe = i0 ? sorted[i0 - 1] + 1u : 0u;
        for (uint32_t i = i0; i < i1; ++i) {
            const uint32_t x = sorted[i];
            const uint32_t gap = x - pe;
            const uint32_t q = gap >> b;
            put_ones(words, pos, q);
            pos += q;
            put_bits(words, pos, gap & ((1u << b) - 1u), b + 1);   // the zero and the remainder
            pos += (unsigned)b + 1u;
            pe = x + 1u;
        }
    }
    __syncthreads();
    SBC_TS(1, 11);                                    // encoded
    uint32_t* __restrict__ out = stage + d.stage_off;
    for (uint32_t w = tid; w < n_words; w += kSelThreads) out[w] = words[w];
    uint32_t* __restrict__ ki = kept_idx + d.kept_off;
    for (uint32_t i = tid; i < kk; i += kSelThreads) ki[i] = sorted[i];
    if (tid == 0) { st[t].bit_len = total_bits; st[t].nnz = kk; }
    SBC_TS(1, 12);
}

}  // namespace sbc
