// Alg. 2 for tensors that keep so many entries that one workgroup would take too long: the same
// steps as k_select (threshold key by radix selection over the candidate lists, ties to the
// lowest index, exact integer sums, side decision, residual update), each as a grid-wide sweep
// over the tensor's two candidate lists with a one-workgroup step in between.
//
//   k_wide_count (pass 0,1,2)  histogram of the next key digit over the entries that match the
//                              digits fixed so far: 19 leading bits in a window above the filter
//                              key, then 8 bits, then the last 5
//   k_wide_pick  (pass 0,1,2)  the digit that holds the k-th entry of each side; after pass 2 the
//                              threshold key tau, the number of entries equal to it and how many
//                              of those are kept
//   k_wide_ties, k_wide_rank   only if some ties must be dropped: the indices of the entries equal
//                              to tau are collected, and the highest index kept is found by rank
//   k_wide_sums                exact per-exponent integer sums of the kept values of both sides
//   k_wide_decide              S+, S-, side, mu; per-tensor results
//   k_wide_apply               residual update and bitmap bits at the kept positions
//
// A tensor for which any step does not apply (k-th entry beyond the window, more ties than the
// tie list holds) is left to k_select, which runs afterwards and skips the tensors done here.
#pragma once

#include "sbc_device.hpp"
#include "sbc_select_kernels.hpp"

namespace sbc {

constexpr int kWideThreads = 256;        // sweep kernels
constexpr uint32_t kWideTieMax = 1024;   // tied entries whose indices can be ranked
// First pass: the leading 19 key bits (1024 steps per octave) counted in a window of two octaves
// above the filter key.  Wider than k_select's half octave on purpose: a filter key carried over
// from the previous call may lie far below this call's k-th entry while the data still grows, and
// a tensor whose k-th entry lies beyond the window falls to one workgroup.
constexpr int kWideShift = 13;
constexpr int kWideLastBits = kWideShift - 8;   // key bits left for the third pass (the second takes 8)
static_assert(kWideLastBits >= 1 && kWideLastBits <= 11, "the last two digits fit the histogram");

struct WideState {
    uint32_t ok;          // 1 while every step so far applied
    uint32_t prefix[2];   // key digits fixed so far, as the leading bits of the key
    uint32_t need[2];     // rank of the wanted entry among the entries matching the prefix
    uint32_t tau[2];      // threshold key per side (side key space)
    uint32_t itau[2];     // ties at tau are kept up to this index
    uint32_t ties[2];     // entries equal to tau
    uint32_t tie_cnt[2];  // indices collected by k_wide_ties
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

__global__ __launch_bounds__(kWideThreads) void k_wide_count(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ wide_ids,
        const TensorState* __restrict__ st, const uint2* __restrict__ cand,
        const WideState* __restrict__ ws, uint32_t* __restrict__ whist, int pass) {
    __shared__ uint32_t hist[2][kWindow];
    const int w = blockIdx.y, tid = threadIdx.x;
    const int t = (int)wide_ids[w];
    if (pass > 0 && !ws[w].ok) return;
    const TensorDesc d = desc[t];
    const uint32_t cnt[2] = {min(st[t].cand_cnt[0], d.cand_cap), min(st[t].cand_cnt[1], d.cand_cap)};
    {
        uint32_t kc[2];
        bool enough, all;
        wide_kept(d, st[t], kc, enough, all);
        if (!enough || all) return;                    // k_wide_pick reports it / nothing to select
    }
    for (int i = tid; i < 2 * kWindow; i += kWideThreads) (&hist[0][0])[i] = 0u;
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint2* __restrict__ list = cand + d.cand_off + (s ? d.cand_cap : 0u);
        const uint32_t base = st[t].lo_key[s] >> kWideShift;
        const uint32_t prefix = ws[w].prefix[s];
        const uint64_t stride = (uint64_t)gridDim.x * kWideThreads;
#pragma unroll 4
        for (uint64_t i = (uint64_t)blockIdx.x * kWideThreads + tid; i < cnt[s]; i += stride) {
            const uint32_t key = list[i].x;
            if (pass == 0) {
                const uint32_t v = key >> kWideShift;
                const uint32_t o = v >= base ? v - base : 0u;
                atomicAdd(&hist[s][o < (uint32_t)(kWindow - 1) ? o : (uint32_t)(kWindow - 1)], 1u);
            } else if (pass == 1) {
                if ((key >> kWideShift) == prefix) atomicAdd(&hist[s][(key >> kWideLastBits) & 255u], 1u);
            } else {
                if ((key >> kWideLastBits) == prefix) atomicAdd(&hist[s][key & ((1u << kWideLastBits) - 1u)], 1u);
            }
        }
    }
    __syncthreads();
    uint32_t* __restrict__ g = whist + (size_t)w * 2 * kWindow;
    for (int i = tid; i < 2 * kWindow; i += kWideThreads) {
        const uint32_t v = (&hist[0][0])[i];
        if (v) atomicAdd(&g[i], v);
    }
}

__global__ __launch_bounds__(kSelThreads) void k_wide_pick(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ wide_ids,
        const TensorState* __restrict__ st, WideState* __restrict__ ws, uint32_t* __restrict__ whist, int pass) {
    __shared__ uint32_t hist[2][kWindow];
    __shared__ uint32_t res[8], res2[2];
    __shared__ unsigned long long scratch64[kSelThreads / 64];
    const int w = blockIdx.x, tid = threadIdx.x;
    const int t = (int)wide_ids[w];
    const TensorDesc d = desc[t];
    uint32_t* __restrict__ g = whist + (size_t)w * 2 * kWindow;
    uint32_t kc[2];
    bool enough, all;
    wide_kept(d, st[t], kc, enough, all);
    if (pass == 0) {
        if (tid == 0) {
            WideState z;
            z.ok = enough ? 1u : 0u;
            z.prefix[0] = z.prefix[1] = 0u; z.need[0] = kc[0]; z.need[1] = kc[1];
            z.tau[0] = all ? st[t].lo_key[0] : 0u; z.tau[1] = all ? st[t].lo_key[1] : 0u;
            z.itau[0] = z.itau[1] = 0xFFFFFFFFu;
            z.ties[0] = z.ties[1] = 0u; z.tie_cnt[0] = z.tie_cnt[1] = 0u;
            z.kc[0] = kc[0]; z.kc[1] = kc[1]; z.all = all ? 1u : 0u;
            z.next_key[0] = st[t].lo_key[0]; z.next_key[1] = st[t].lo_key[1];
            ws[w] = z;
        }
        if (!enough) return;                           // k_select flags the tensor for the histogram path
    } else if (!ws[w].ok) {
        return;
    }
    if (all) return;                                   // nothing to select: no histogram was counted
    for (int i = tid; i < 2 * kWindow; i += kSelThreads) { (&hist[0][0])[i] = g[i]; g[i] = 0u; }
    __syncthreads();
    uint32_t need[2] = {kc[0], kc[1]};
    if (pass > 0) { need[0] = ws[w].need[0]; need[1] = ws[w].need[1]; }
    const bool both[2] = {true, true};
    uint32_t digit[2];
    bool found[2];
    // (first pass: the same scan also finds the bin of the entry a following call's key sits at)
    const uint32_t r_next = carried_rank(kc[0] > kc[1] ? kc[0] : kc[1]);
    const uint32_t rank2[2] = {r_next, r_next};
    uint32_t digit2[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
    pick_wide_both<kWindow, kSelThreads>(hist, need, both, res, scratch64, digit, found, pass == 0, rank2, res2, digit2);
    if (tid == 0) {
        bool ok = found[0] && found[1];
        if (pass == 0) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
                ws[w].next_key[s] = digit2[s] != 0xFFFFFFFFu ? ((st[t].lo_key[s] >> kWideShift) + digit2[s]) << kWideShift
                                                              : lowered_key(st[t].lo_key[s], 0.1f);
            ok = ok && digit[0] != (uint32_t)(kWindow - 1) && digit[1] != (uint32_t)(kWindow - 1);
            if (ok) {
#pragma unroll
                for (int s = 0; s < 2; ++s) ws[w].prefix[s] = (st[t].lo_key[s] >> kWideShift) + digit[s];
            }
        } else if (ok) {
            const int bits = pass == 1 ? 8 : kWideLastBits;
#pragma unroll
            for (int s = 0; s < 2; ++s) ws[w].prefix[s] = (ws[w].prefix[s] << bits) | digit[s];
        }
        if (ok) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                ws[w].need[s] = need[s];
                if (pass == 2) {
                    ws[w].tau[s] = ws[w].prefix[s];
                    ws[w].ties[s] = hist[s][digit[s]];
                }
            }
        }
        ws[w].ok = ok ? 1u : 0u;
    }
}

// Entries equal to tau on a side that keeps only some of its ties: their indices.
__global__ __launch_bounds__(kWideThreads) void k_wide_ties(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ wide_ids,
        const TensorState* __restrict__ st, const uint2* __restrict__ cand,
        WideState* __restrict__ ws, uint32_t* __restrict__ wtie) {
    const int w = blockIdx.y, tid = threadIdx.x;
    const int t = (int)wide_ids[w];
    if (!ws[w].ok || ws[w].all) return;
    const TensorDesc d = desc[t];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        if (ws[w].need[s] >= ws[w].ties[s]) continue;          // all ties are kept
        const uint32_t cnt = min(st[t].cand_cnt[s], d.cand_cap);
        const uint32_t tau = ws[w].tau[s];
        const uint2* __restrict__ list = cand + d.cand_off + (s ? d.cand_cap : 0u);
        uint32_t* __restrict__ out = wtie + ((size_t)w * 2 + s) * kWideTieMax;
        const uint64_t stride = (uint64_t)gridDim.x * kWideThreads;
#pragma unroll 4
        for (uint64_t i = (uint64_t)blockIdx.x * kWideThreads + tid; i < cnt; i += stride) {
            const uint2 e = list[i];
            if (e.x == tau) {
                const uint32_t q = atomicAdd(&ws[w].tie_cnt[s], 1u);
                if (q < kWideTieMax) out[q] = e.y;
            }
        }
    }
}

// The need-th lowest index among the collected ties of each side.
__global__ __launch_bounds__(kSelThreads) void k_wide_rank(const uint32_t* __restrict__ wide_ids,
                                                           WideState* __restrict__ ws,
                                                           const uint32_t* __restrict__ wtie) {
    __shared__ uint32_t idx[kWideTieMax];
    __shared__ uint32_t hit[2];
    const int w = blockIdx.x, tid = threadIdx.x;
    (void)wide_ids;
    if (!ws[w].ok || ws[w].all) return;
    bool ok = true;
    for (int s = 0; s < 2; ++s) {
        const uint32_t need = ws[w].need[s], ties = ws[w].ties[s];
        if (need >= ties) continue;                            // uniform
        const uint32_t m = ws[w].tie_cnt[s];
        if (m != ties || m > kWideTieMax) { ok = false; continue; }
        __syncthreads();
        if (tid < 2) hit[tid] = 0u;
        for (uint32_t i = tid; i < m; i += kSelThreads) idx[i] = wtie[((size_t)w * 2 + s) * kWideTieMax + i];
        __syncthreads();
        if ((uint32_t)tid < m) {
            const uint32_t me = idx[tid];
            uint32_t below = 0u;
#pragma unroll 8
            for (uint32_t j = 0; j < m; ++j) below += idx[j] < me ? 1u : 0u;
            if (below + 1u == need) { ws[w].itau[s] = me; hit[0] = 1u; }
        }
        __syncthreads();
        if (hit[0] != 1u) ok = false;
    }
    if (!ok && tid == 0) ws[w].ok = 0u;
}

// Per-exponent exact integer sums of the kept values, both sides.
__global__ __launch_bounds__(kWideThreads) void k_wide_sums(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ wide_ids,
        const TensorState* __restrict__ st, const uint2* __restrict__ cand,
        const WideState* __restrict__ ws, long long* __restrict__ wacc) {
    __shared__ long long acc[2][256];
    const int w = blockIdx.y, tid = threadIdx.x;
    const int t = (int)wide_ids[w];
    if (!ws[w].ok) return;
    const TensorDesc d = desc[t];
    for (int i = tid; i < 512; i += kWideThreads) (&acc[0][0])[i] = 0ll;
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint32_t cnt = min(st[t].cand_cnt[s], d.cand_cap);
        const uint32_t tau = ws[w].tau[s], itau = ws[w].itau[s];
        const uint2* __restrict__ list = cand + d.cand_off + (s ? d.cand_cap : 0u);
        const uint64_t stride = (uint64_t)gridDim.x * kWideThreads;
        uint32_t cur_ex = 0u;
        long long cur = 0ll;
#pragma unroll 4
        for (uint64_t i = (uint64_t)blockIdx.x * kWideThreads + tid; i < cnt; i += stride) {
            const uint2 e = list[i];
            if (cand_kept(e.x, e.y, tau, itau)) {
                const uint32_t u = bits_of_key(s ? ~e.x : e.x);
                uint32_t ex = (u >> 23) & 0xFFu;
                long long m = (long long)(ex ? ((u & 0x7FFFFFu) | 0x800000u) : (u & 0x7FFFFFu));
                if (ex == 0u) ex = 1u;
                if (((u >> 31) != 0u) != (s != 0)) m = -m;         // the negative side sums -A
                if (ex != cur_ex) {
                    if (cur != 0ll) atomicAdd(reinterpret_cast<unsigned long long*>(&acc[s][cur_ex]), (unsigned long long)cur);
                    cur_ex = ex; cur = 0ll;
                }
                cur += m;
            }
        }
        if (cur != 0ll) atomicAdd(reinterpret_cast<unsigned long long*>(&acc[s][cur_ex]), (unsigned long long)cur);
    }
    __syncthreads();
    long long* __restrict__ g = wacc + (size_t)w * 512;
    for (int i = tid; i < 512; i += kWideThreads) {
        const long long v = (&acc[0][0])[i];
        if (v != 0ll) atomicAdd(reinterpret_cast<unsigned long long*>(&g[i]), (unsigned long long)v);
    }
}

__global__ __launch_bounds__(128) void k_wide_decide(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ wide_ids,
        TensorState* __restrict__ st, const WideState* __restrict__ ws, long long* __restrict__ wacc,
        ResultBlock* __restrict__ result) {
    __shared__ double S[2];
    const int w = blockIdx.x, tid = threadIdx.x;
    const int t = (int)wide_ids[w];
    long long* __restrict__ g = wacc + (size_t)w * 512;
    const bool ok = ws[w].ok != 0u;
    {
        // fixed order: lane l of wavefront s adds exponents 4l..4l+3 ascending, then a fixed shuffle tree
        const int s = tid >> 6, lane = tid & 63;
        double v = 0.0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int ex = 4 * lane + j;
            v += ldexp((double)g[s * 256 + ex], ex - 150);
            g[s * 256 + ex] = 0ll;                              // clean for the next call
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
        if (lane == 0) S[s] = v;
    }
    __syncthreads();
    if (!ok || tid != 0) return;
    const uint32_t k = desc[t].k;
    const double Sp = S[0], Sn = S[1];
    const uint32_t kc[2] = {ws[w].kc[0], ws[w].kc[1]};
    // Alg. 2 compares the means
    const int chosen = (Sp / (double)kc[0] >= Sn / (double)kc[1]) ? 0 : 1;
    const float mu32 = (float)((chosen ? Sn : Sp) / (double)kc[chosen]);
    st[t].kc[0] = kc[0]; st[t].kc[1] = kc[1];
    st[t].tau[0] = ws[w].tau[0]; st[t].tau[1] = ws[w].tau[1];
    st[t].itau[0] = ws[w].itau[0]; st[t].itau[1] = ws[w].itau[1];
    st[t].S[0] = Sp; st[t].S[1] = Sn;
    st[t].side = chosen ? -1 : 1;
    st[t].mu_signed = chosen ? -mu32 : mu32;
    st[t].flags |= kStWideDone;
    atomicOr(&result->err, kErrWide);
    // filter keys a following call may start from (same rule as in k_select)
    st[t].lo_key[0] = ws[w].next_key[0];
    st[t].lo_key[1] = ws[w].next_key[1];
    st[t].expect[0] = 0u; st[t].expect[1] = 0u;
    // many times more candidates than needed: the next call should estimate its keys afresh
    const uint32_t many = 8u * k + 4096u;
    if (st[t].cand_cnt[0] > many || st[t].cand_cnt[1] > many) atomicOr(&result->err, kErrLoose);
}

__global__ __launch_bounds__(kWideThreads) void k_wide_apply(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ wide_ids,
        const TensorState* __restrict__ st, const uint2* __restrict__ cand,
        const WideState* __restrict__ ws, uint32_t* __restrict__ bitmap, ResultBlock* __restrict__ result) {
    const int w = blockIdx.y, tid = threadIdx.x;
    const int t = (int)wide_ids[w];
    if (!ws[w].ok) return;
    const TensorDesc d = desc[t];
    const int s = st[t].side < 0 ? 1 : 0;
    const float mu_signed = st[t].mu_signed;
    const uint32_t cnt = min(st[t].cand_cnt[s], d.cand_cap);
    const uint32_t tau = ws[w].tau[s], itau = ws[w].itau[s];
    const uint2* __restrict__ list = cand + d.cand_off + (s ? d.cand_cap : 0u);
    const gfloat_ptr R = as_global(d.R);
    uint32_t* __restrict__ bm = bitmap + (uint64_t)d.chunk0 * kChunkWords;
    const uint64_t stride = (uint64_t)gridDim.x * kWideThreads;
#pragma unroll 4
    for (uint64_t i = (uint64_t)blockIdx.x * kWideThreads + tid; i < cnt; i += stride) {
        const uint2 e = list[i];
        if (cand_kept(e.x, e.y, tau, itau)) {
            if (e.y >= d.n) { atomicOr(&result->err, kErrInternal); continue; }
            const float a = __uint_as_float(bits_of_key(s ? ~e.x : e.x));
            R[e.y] = a - mu_signed;                   // Alg. 1: R <- dW - dW*
            atomicOr(&bm[e.y >> 5], 1u << (e.y & 31u));
        }
    }
}

}  // namespace sbc
