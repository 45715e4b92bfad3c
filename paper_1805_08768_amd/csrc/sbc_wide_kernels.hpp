// Alg. 2 for tensors that keep so many entries that one workgroup would take too long: the same
// steps as k_select (threshold key by radix selection over the candidate lists, ties to the
// lowest index, exact integer sums, side decision, residual update), each as a grid-wide sweep
// over the tensor's two candidate lists with a one-workgroup step in between.
//
//   k_wide_count    histogram of the 19 leading key bits of every candidate, in a window above
//                   the filter key
//   k_wide_refine   the window bin that holds the k-th entry of each side; histogram of the other
//                   13 key bits over the entries of that bin
//   k_wide_sums     the threshold key tau, the number of entries equal to it and how many of
//                   those are kept; exact per-exponent integer sums of the entries beyond tau;
//                   if some ties must be dropped, the indices of the entries equal to tau
//   k_wide_apply    the highest index kept among the ties (by rank); S+, S-, side, mu and the
//                   per-tensor results; residual update and bitmap bits at the kept positions
//
// A tensor for which any step does not apply (k-th entry beyond the window, more ties than the
// tie list holds) is left to k_select, which runs afterwards and skips the tensors done here.
#pragma once

#include "sbc_device.hpp"
#include "sbc_select_kernels.hpp"

namespace sbc {

constexpr int kWideThreads = 256;        // sweep kernels
constexpr uint32_t kWideTieMax = 1024;   // tied entries whose indices can be ranked
constexpr uint32_t kWideRefine = 1u << kWideShift;   // bins of the second histogram: the remaining key bits
constexpr int kWideSweepThreads = 1024;              // sweeps that carry that histogram in LDS (64 KiB)
constexpr int kWideQuads = 2 * (int)kWideRefine / 4 / kWideSweepThreads;   // 16-byte pieces of it per thread
static_assert(kWideQuads * 4 * kWideSweepThreads == 2 * (int)kWideRefine, "the histogram divides evenly over the threads");

// The call's wide tensors, passed to the kernels by value: a workgroup learns its tensor from the
// kernel arguments instead of from a load that everything else would have to wait for.
constexpr int kMaxWide = 64;              // tensors per call that the grid-wide selection kernels can take
struct WideIds { uint32_t id[kMaxWide]; };

struct WideState {
    uint32_t ok;          // k_wide_refine: 1 if its step applied
    uint32_t ok2;         // k_wide_sums: 1 if every step so far applied
    uint32_t prefix[2];   // leading key bits of the k-th entry (k_wide_refine)
    uint32_t need[2];     // rank of the k-th entry among the entries with those leading bits
    uint32_t tau[2];      // threshold key per side (side key space; k_wide_sums)
    uint32_t keep[2];     // entries equal to tau that are kept (those of lowest index)
    uint32_t ties[2];     // entries equal to tau
    uint32_t kc[2];       // entries kept per side: k, or (subsampled variant) the candidates up to the cap
    uint32_t all;         // 1: every candidate is kept (subsampled variant), tau is the filter key
    uint32_t next_key[2]; // filter keys a following call may start from (see k_select)
};

// Entries kept per side of a tensor, from its candidate counts.
__device__ __forceinline__ void wide_kept(const TensorDesc& d, const TensorState& s, uint32_t (&kc)[2], bool& enough, bool& all) {
    const uint32_t cp = s.cand_cnt[0], cn = s.cand_cnt[1];
    if (d.flags & kDescSampled) {
        kc[0] = min(cp, d.kcap); kc[1] = min(cn, d.kcap);
        enough = cp >= 1u && cn >= 1u && cp <= d.cand_cap && cn <= d.cand_cap;
        all = cp <= d.kcap && cn <= d.kcap;
    } else {
        kc[0] = kc[1] = d.k;
        enough = cp >= d.k && cn >= d.k && cp <= d.cand_cap && cn <= d.cand_cap;
        all = false;
    }
}

// The tensor-wide steps between the sweeps (which bin holds the k-th entry, which tie is the last
// one kept, which side wins) are taken by every workgroup of the sweep that needs the answer, all
// of them at once from the same counts, instead of by a one-workgroup launch in between: four
// launches in a row instead of eleven.  The first workgroup of a tensor records what later
// kernels and the rest of the call need; it also clears the counts that the kernel before it
// has read, so that every array is clean again when the call ends (the sums: in the next call's
// k_wide_refine).

// k_wide_count: histogram of the leading key bits of both lists, in the window above the filter keys.
// (Counting them where the streaming kernel stores the candidates would save this sweep, but every
// count would be an atomic on memory that all compute-unit groups share, and those on one bin queue
// up for about half a microsecond each: four times the streaming kernel's time on Gaussian data.)
__global__ __launch_bounds__(kWideThreads) void k_wide_count(
        const TensorDesc* __restrict__ desc, const WideIds wide_ids,
        const TensorState* __restrict__ st, const uint2* __restrict__ cand,
        uint32_t* __restrict__ whist) {
    __shared__ uint32_t hist[2][kWindow];
    const int w = blockIdx.y, tid = threadIdx.x;
    const int t = (int)wide_ids.id[w];
    const TensorDesc d = desc[t];
    const uint32_t cnt[2] = {min(st[t].cand_cnt[0], d.cand_cap), min(st[t].cand_cnt[1], d.cand_cap)};
    {
        uint32_t kc[2];
        bool enough, all;
        wide_kept(d, st[t], kc, enough, all);
        if (!enough || all) return;                    // k_wide_refine reports it / nothing to select
    }
    for (int i = tid; i < 2 * kWindow; i += kWideThreads) (&hist[0][0])[i] = 0u;
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint2* __restrict__ list = cand + d.cand_off + (s ? d.cand_cap : 0u);
        const uint32_t lo_key = st[t].lo_key[s];
        const uint64_t stride = (uint64_t)gridDim.x * kWideThreads;
#pragma unroll 4
        for (uint64_t i = (uint64_t)blockIdx.x * kWideThreads + tid; i < cnt[s]; i += stride)
            atomicAdd(&hist[s][wide_window_bin(list[i].x, lo_key)], 1u);
    }
    __syncthreads();
    uint32_t* __restrict__ g = whist + (size_t)w * 2 * kWindow;
    for (int i = tid; i < 2 * kWindow; i += kWideThreads) {
        const uint32_t v = (&hist[0][0])[i];
        if (v) atomicAdd(&g[i], v);
    }
}

// k_wide_refine: the window bin of each side's k-th entry from the first histogram, then the
// counts of the remaining kWideShift key bits over the entries in that bin.
__global__ __launch_bounds__(kWideSweepThreads) void k_wide_refine(
        const TensorDesc* __restrict__ desc, const WideIds wide_ids,
        const TensorState* __restrict__ st, const uint2* __restrict__ cand,
        WideState* __restrict__ ws, const uint32_t* __restrict__ whist, uint32_t* __restrict__ whist2,
        long long* __restrict__ wacc, uint32_t* __restrict__ wtie_cnt) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[2 * kWideRefine];   // the window's counts first, the refinement's afterwards
    __shared__ uint32_t res[8], res2[2];
    __shared__ unsigned long long scratch64[kWideSweepThreads / 64];
    static_assert(kWindow <= kWideRefine, "the window histogram fits");
    uint32_t (*const win)[kWindow] = reinterpret_cast<uint32_t (*)[kWindow]>(lds);
    uint32_t (*const fine)[kWideRefine] = reinterpret_cast<uint32_t (*)[kWideRefine]>(lds);
    const int w = blockIdx.y, tid = threadIdx.x;
    const int t = (int)wide_ids.id[w];
    const bool lead = blockIdx.x == 0 && tid == 0;     // the one thread that records the tensor's state
    // (the window's counts are asked for together with the descriptor and the state, before those say
    // whether they are needed: one round trip to memory less)
    static_assert(2 * kWindow == 4 * kWideSweepThreads, "one 16-byte piece of the window's counts per thread");
    const uint4 win_mine = reinterpret_cast<const uint4*>(whist + (size_t)w * 2 * kWindow)[tid];
    if (blockIdx.x == 0) {                             // the sums of the call before this one have been read
        long long* __restrict__ a = wacc + (size_t)w * 512;
        for (int i = tid; i < 512; i += kWideSweepThreads) a[i] = 0ll;
    }
    const TensorDesc d = desc[t];
    const uint32_t lo_key[2] = {st[t].lo_key[0], st[t].lo_key[1]};
    uint32_t kc[2];
    bool enough, all;
    wide_kept(d, st[t], kc, enough, all);
    if (lead) {
        WideState z;
        z.ok = enough ? 1u : 0u; z.ok2 = 0u;
        z.prefix[0] = z.prefix[1] = 0u; z.need[0] = kc[0]; z.need[1] = kc[1];
        z.tau[0] = lo_key[0]; z.tau[1] = lo_key[1];
        z.keep[0] = z.keep[1] = 0u; z.ties[0] = z.ties[1] = 0u;
        z.kc[0] = kc[0]; z.kc[1] = kc[1]; z.all = all ? 1u : 0u;
        z.next_key[0] = lo_key[0]; z.next_key[1] = lo_key[1];
        ws[w] = z;
        wtie_cnt[2 * w] = 0u; wtie_cnt[2 * w + 1] = 0u;
    }
    if (!enough || all) return;                        // k_select flags the tensor / nothing to select
    reinterpret_cast<uint4*>(lds)[tid] = win_mine;
    __syncthreads();
    uint32_t need[2] = {kc[0], kc[1]};
    const bool both[2] = {true, true};
    uint32_t digit[2];
    bool found[2];
    // (the same scan also finds the bin of the entry a following call's key sits at)
    const uint32_t r_next = carried_rank(kc[0] > kc[1] ? kc[0] : kc[1]);
    const uint32_t rank2[2] = {r_next, r_next};
    uint32_t digit2[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
    pick_wide_both<kWindow, kWideSweepThreads>(win, need, both, res, scratch64, digit, found, true, rank2, res2, digit2);
    // (the k-th entry beyond the window: the tensor falls to k_select)
    const bool ok = found[0] && found[1] && digit[0] != (uint32_t)(kWindow - 1) && digit[1] != (uint32_t)(kWindow - 1);
    const uint32_t prefix[2] = {(lo_key[0] >> kWideShift) + digit[0], (lo_key[1] >> kWideShift) + digit[1]};
    if (lead) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            ws[w].next_key[s] = digit2[s] != 0xFFFFFFFFu ? ((lo_key[s] >> kWideShift) + digit2[s]) << kWideShift
                                                          : lowered_key(lo_key[s], 0.1f);
            if (ok) { ws[w].prefix[s] = prefix[s]; ws[w].need[s] = need[s]; }
        }
        ws[w].ok = ok ? 1u : 0u;
    }
    if (!ok) return;
    __syncthreads();                                   // the window's counts have been read
    uint4* const lds4 = reinterpret_cast<uint4*>(lds);
#pragma unroll
    for (int i = 0; i < kWideQuads; ++i) lds4[i * kWideSweepThreads + tid] = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint32_t cnt = min(st[t].cand_cnt[s], d.cand_cap);
        const uint2* __restrict__ list = cand + d.cand_off + (s ? d.cand_cap : 0u);
        const uint64_t stride = (uint64_t)gridDim.x * kWideSweepThreads;
#pragma unroll 4
        for (uint64_t i = (uint64_t)blockIdx.x * kWideSweepThreads + tid; i < cnt; i += stride) {
            const uint32_t key = list[i].x;
            if ((key >> kWideShift) == prefix[s]) atomicAdd(&fine[s][key & (kWideRefine - 1u)], 1u);
        }
    }
    __syncthreads();
    uint32_t* __restrict__ g2 = whist2 + (size_t)w * 2 * kWideRefine;
#pragma unroll
    for (int i = 0; i < kWideQuads; ++i) {            // (nearly all of it is zero)
        const int q = i * kWideSweepThreads + tid;
        const uint4 v = lds4[q];
        if (v.x | v.y | v.z | v.w) {
            if (v.x) atomicAdd(&g2[4 * q + 0], v.x);
            if (v.y) atomicAdd(&g2[4 * q + 1], v.y);
            if (v.z) atomicAdd(&g2[4 * q + 2], v.z);
            if (v.w) atomicAdd(&g2[4 * q + 3], v.w);
        }
    }
}

// Mantissa (signed the way the side sums it) and exponent slot of the value a side key stands for.
__device__ __forceinline__ long long wide_mantissa(uint32_t key, int s, uint32_t& ex) {
    const uint32_t u = bits_of_key(s ? ~key : key);
    ex = (u >> 23) & 0xFFu;
    long long m = (long long)(ex ? ((u & 0x7FFFFFu) | 0x800000u) : (u & 0x7FFFFFu));
    if (ex == 0u) ex = 1u;
    if (((u >> 31) != 0u) != (s != 0)) m = -m;         // the negative side sums -A
    return m;
}

// k_wide_sums: the threshold key tau of each side from the second histogram; then the exact
// per-exponent integer sums of the entries beyond tau (the kept entries equal to tau all have
// tau's value: k_wide_apply adds them as a product), and, for a side that keeps only some of
// its ties, the indices of the entries equal to tau.
__global__ __launch_bounds__(kWideSweepThreads) void k_wide_sums(
        const TensorDesc* __restrict__ desc, const WideIds wide_ids,
        const TensorState* __restrict__ st, const uint2* __restrict__ cand,
        WideState* __restrict__ ws, uint32_t* __restrict__ whist, const uint32_t* __restrict__ whist2,
        long long* __restrict__ wacc, uint32_t* __restrict__ wtie, uint32_t* __restrict__ wtie_cnt) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[2 * kWideRefine];
    __shared__ long long acc[2][256];
    __shared__ uint32_t res[8];
    __shared__ unsigned long long scratch64[kWideSweepThreads / 64];
    uint32_t (*const fine)[kWideRefine] = reinterpret_cast<uint32_t (*)[kWideRefine]>(lds);
    const int w = blockIdx.y, tid = threadIdx.x;
    const int t = (int)wide_ids.id[w];
    const bool lead = blockIdx.x == 0 && tid == 0;
    // (the second histogram is asked for at once, all 64 KiB of it, before the state says whether it
    // is needed: one round trip to memory less)
    uint4 fine_mine[kWideQuads];
    {
        const uint4* __restrict__ g4 = reinterpret_cast<const uint4*>(whist2 + (size_t)w * 2 * kWideRefine);
#pragma unroll
        for (int i = 0; i < kWideQuads; ++i) fine_mine[i] = g4[i * kWideSweepThreads + tid];
    }
    if (blockIdx.x == 0)                               // every workgroup of k_wide_refine has read the window's counts
        reinterpret_cast<uint4*>(whist + (size_t)w * 2 * kWindow)[tid] = make_uint4(0u, 0u, 0u, 0u);
    if (!ws[w].ok) return;
    const TensorDesc d = desc[t];
    const bool all = ws[w].all != 0u;
    uint32_t tau[2] = {st[t].lo_key[0], st[t].lo_key[1]};      // (if every candidate is kept)
    uint32_t keep[2] = {0u, 0u}, ties[2] = {0u, 0u};
    bool some_ties[2] = {false, false};
    bool ok = true;
    if (!all) {
#pragma unroll
        for (int i = 0; i < kWideQuads; ++i) reinterpret_cast<uint4*>(lds)[i * kWideSweepThreads + tid] = fine_mine[i];
        __syncthreads();
        uint32_t need[2] = {ws[w].need[0], ws[w].need[1]};
        const bool both[2] = {true, true};
        uint32_t digit[2];
        bool found[2];
        pick_wide_both<kWideRefine, kWideSweepThreads>(fine, need, both, res, scratch64, digit, found);
        ok = found[0] && found[1];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (!ok) break;
            tau[s] = (ws[w].prefix[s] << kWideShift) | digit[s];
            keep[s] = need[s];
            ties[s] = fine[s][digit[s]];
            some_ties[s] = keep[s] < ties[s];
        }
    }
    if (lead) {                                        // (fields that no workgroup of this kernel reads)
#pragma unroll
        for (int s = 0; s < 2; ++s) { ws[w].tau[s] = tau[s]; ws[w].keep[s] = keep[s]; ws[w].ties[s] = ties[s]; }
        ws[w].ok2 = ok ? 1u : 0u;
    }
    if (!ok) return;
    __syncthreads();                                   // the second histogram has been read: its space is free
    for (int i = tid; i < 512; i += kWideSweepThreads) (&acc[0][0])[i] = 0ll;
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint32_t cnt = min(st[t].cand_cnt[s], d.cand_cap);
        const uint2* __restrict__ list = cand + d.cand_off + (s ? d.cand_cap : 0u);
        uint32_t* __restrict__ out = wtie + ((size_t)w * 2 + s) * kWideTieMax;
        const uint64_t stride = (uint64_t)gridDim.x * kWideSweepThreads;
        uint32_t cur_ex = 0u;
        long long cur = 0ll;
#pragma unroll 4
        for (uint64_t i = (uint64_t)blockIdx.x * kWideSweepThreads + tid; i < cnt; i += stride) {
            const uint2 e = list[i];
            if (e.x > tau[s] || all) {                 // (every candidate, in the subsampled variant below the cap)
                uint32_t ex;
                const long long m = wide_mantissa(e.x, s, ex);
                if (ex != cur_ex) {
                    if (cur != 0ll) atomicAdd(reinterpret_cast<unsigned long long*>(&acc[s][cur_ex]), (unsigned long long)cur);
                    cur_ex = ex; cur = 0ll;
                }
                cur += m;
            } else if (e.x == tau[s] && some_ties[s]) {
                const uint32_t q = atomicAdd(&wtie_cnt[2 * w + s], 1u);
                if (q < kWideTieMax) out[q] = e.y;
            }
        }
        if (cur != 0ll) atomicAdd(reinterpret_cast<unsigned long long*>(&acc[s][cur_ex]), (unsigned long long)cur);
    }
    __syncthreads();
    long long* __restrict__ g = wacc + (size_t)w * 512;
    for (int i = tid; i < 512; i += kWideSweepThreads) {
        const long long v = (&acc[0][0])[i];
        if (v != 0ll) atomicAdd(reinterpret_cast<unsigned long long*>(&g[i]), (unsigned long long)v);
    }
}

// k_wide_apply: the last tie kept (by rank among the collected indices), S+, S-, side and mu,
// in every workgroup; then the residual update and the bitmap bits at the kept positions.  The
// first workgroup records the tensor's results.  handback: 0 if k_select runs after this kernel
// and takes the tensors no step applied to by itself, 1 if the call must be told to run it.
__global__ __launch_bounds__(kWideThreads) void k_wide_apply(
        const TensorDesc* __restrict__ desc, const WideIds wide_ids,
        TensorState* __restrict__ st, const uint2* __restrict__ cand,
        const WideState* __restrict__ ws, uint32_t* __restrict__ whist2, const long long* __restrict__ wacc,
        const uint32_t* __restrict__ wtie, const uint32_t* __restrict__ wtie_cnt, uint32_t* __restrict__ bitmap, int handback,
        ResultBlock* __restrict__ result) {
    __shared__ uint32_t idx[kWideTieMax];
    __shared__ uint32_t hit[2], itau_sh[2];
    __shared__ double S[2];
    const int w = blockIdx.y, tid = threadIdx.x;
    const int t = (int)wide_ids.id[w];
    const bool lead = blockIdx.x == 0 && tid == 0;
    if (blockIdx.x == 0) {                             // every workgroup of k_wide_sums has read the second histogram
        uint4* __restrict__ g4 = reinterpret_cast<uint4*>(whist2 + (size_t)w * 2 * kWideRefine);
        for (int i = tid; i < 2 * (int)kWideRefine / 4; i += kWideThreads) g4[i] = make_uint4(0u, 0u, 0u, 0u);
    }
    bool ok = ws[w].ok != 0u && ws[w].ok2 != 0u;
    const bool all = ws[w].all != 0u;
    const uint32_t tau[2] = {ws[w].tau[0], ws[w].tau[1]};
    const uint32_t need[2] = {ws[w].keep[0], ws[w].keep[1]};
    uint32_t itau[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
    if (ok && !all) {
        // the need-th lowest index among the collected ties of a side that drops some
        for (int s = 0; s < 2; ++s) {
            const uint32_t ties = ws[w].ties[s];
            if (need[s] >= ties) continue;             // uniform: all ties are kept
            const uint32_t m = wtie_cnt[2 * w + s];
            if (m != ties || m > kWideTieMax) { ok = false; continue; }
            __syncthreads();
            if (tid == 0) hit[s] = 0u;
            for (uint32_t i = tid; i < m; i += kWideThreads) idx[i] = wtie[((size_t)w * 2 + s) * kWideTieMax + i];
            __syncthreads();
            for (uint32_t i = tid; i < m; i += kWideThreads) {
                const uint32_t me = idx[i];
                uint32_t below = 0u;
#pragma unroll 8
                for (uint32_t j = 0; j < m; ++j) below += idx[j] < me ? 1u : 0u;
                if (below + 1u == need[s]) { itau_sh[s] = me; hit[s] = 1u; }
            }
            __syncthreads();
            if (hit[s] != 1u) ok = false; else itau[s] = itau_sh[s];
        }
    }
    const TensorDesc d = desc[t];
    if (!ok) {
        // (what k_select would do with the tensor in this pass, if it ran)
        if (handback && !lists_unusable(d, st, t, st[t].cand_cnt[0], st[t].cand_cnt[1], 0, lead, result) && lead) {
            st[t].flags |= kStDeferred;
            atomicOr(&result->err, kErrDeferred);
        }
        return;
    }
    const uint32_t kc[2] = {ws[w].kc[0], ws[w].kc[1]};
    {
        // fixed order: lane l of wavefront s adds exponents 4l..4l+3 ascending, then a fixed shuffle tree
        const long long* __restrict__ g = wacc + (size_t)w * 512;
        const int s = (tid >> 6) & 1, lane = tid & 63;
        uint32_t ex_tau;
        const long long m_tau = all ? 0ll : wide_mantissa(tau[s], s, ex_tau) * (long long)need[s];
        if (all) ex_tau = 0u;
        double v = 0.0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int ex = 4 * lane + j;
            v += ldexp((double)(g[s * 256 + ex] + ((uint32_t)ex == ex_tau ? m_tau : 0ll)), ex - 150);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
        if (lane == 0 && tid < 128) S[s] = v;
    }
    __syncthreads();
    const double Sp = S[0], Sn = S[1];
    // Alg. 2 compares the means
    const int chosen = (Sp / (double)kc[0] >= Sn / (double)kc[1]) ? 0 : 1;
    const float mu32 = (float)((chosen ? Sn : Sp) / (double)kc[chosen]);
    const float mu_signed = chosen ? -mu32 : mu32;
    if (lead) {
        st[t].kc[0] = kc[0]; st[t].kc[1] = kc[1];
        st[t].tau[0] = tau[0]; st[t].tau[1] = tau[1];
        st[t].itau[0] = itau[0]; st[t].itau[1] = itau[1];
        st[t].S[0] = Sp; st[t].S[1] = Sn;
        st[t].side = chosen ? -1 : 1;
        st[t].mu_signed = mu_signed;
        st[t].flags |= kStWideDone;
        atomicOr(&result->err, kErrWide);
        // filter keys a following call may start from (same rule as in k_select)
        st[t].lo_key[0] = ws[w].next_key[0];
        st[t].lo_key[1] = ws[w].next_key[1];
        st[t].expect[0] = 0u; st[t].expect[1] = 0u;
        // many times more candidates than needed: the next call should estimate its keys afresh
        const unsigned long long many = loose_limit(d.k, d.n);
        if (st[t].cand_cnt[0] > many || st[t].cand_cnt[1] > many) atomicOr(&result->err, kErrLoose);
    }
    const int s = chosen;
    const uint32_t cnt = min(st[t].cand_cnt[s], d.cand_cap);
    const uint2* __restrict__ list = cand + d.cand_off + (s ? d.cand_cap : 0u);
    const gfloat_ptr R = as_global(d.R);
    uint32_t* __restrict__ bm = bitmap + (uint64_t)d.chunk0 * kChunkWords;
    const uint64_t stride = (uint64_t)gridDim.x * kWideThreads;
#pragma unroll 4
    for (uint64_t i = (uint64_t)blockIdx.x * kWideThreads + tid; i < cnt; i += stride) {
        const uint2 e = list[i];
        if (cand_kept(e.x, e.y, tau[s], itau[s])) {
            if (e.y >= d.n) { atomicOr(&result->err, kErrInternal); continue; }
            const float a = __uint_as_float(bits_of_key(s ? ~e.x : e.x));
            R[e.y] = a - mu_signed;                   // Alg. 1: R <- dW - dW*
            atomicOr(&bm[e.y >> 5], 1u << (e.y & 31u));
        }
    }
}

}  // namespace sbc
