// Stage 1 of the client step and the candidate search around it.
//
// Fast path (two launches):
//   k_sample_thresholds  per tensor: a stratified sample of A = R + dW gives, for each sign
//                        side, a key that is with overwhelming probability at or below the
//                        k-th most extreme entry of the whole tensor (conservative: only a
//                        filter, never the answer)
//   k_accumulate_filter  per chunk: A = R + dW written over R (Alg. 1, client line
//                        dW_i <- R_i + local update); every entry at or beyond a side's
//                        filter key is appended to that side's candidate list
// If a side ends up with fewer than k candidates the filter was too tight for that tensor;
// the histogram path below then finds its candidates exactly from a second read of A:
//   k_hist_flagged, k_pick_bins, k_extract
// Either way the select kernel receives, per tensor and side, a list that contains the k most
// extreme entries, and the result is exact.
#pragma once

#include "sbc_device.hpp"

namespace sbc {

// --------------------------------------------------------------------------
// Plain streaming copy of 16-byte units: the yardstick the streaming kernels are measured
// against (same workgroup shape and loads in flight as the accumulation kernel).
// --------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_copy_baseline(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                       uint64_t n16) {
    const uint64_t base = (uint64_t)blockIdx.x * 2048ull + threadIdx.x;
    if (base - threadIdx.x + 2048ull <= n16) {
        uint4 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = src[base + 256ull * i];
#pragma unroll
        for (int i = 0; i < 8; ++i) dst[base + 256ull * i] = v[i];
    } else {
        for (uint64_t j = base; j < n16; j += 256ull) dst[j] = src[j];
    }
}

__global__ __launch_bounds__(256) void k_zero_words(uint32_t* __restrict__ p, uint64_t n) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0u;
}

// The result block of a server call, copied to pinned host memory by a dispatch of its own behind
// the decode kernels (the runtime's own device-to-host copy of 16 bytes and its wait for the
// stream take longer); the sequence number goes out last, so that a host that looks for it finds
// the status in place.
__global__ void k_publish(ResultBlock* __restrict__ host_dst, const ResultBlock* __restrict__ src, uint32_t seq) {
    if (threadIdx.x == 0) {
        host_dst->msg_bytes = src->msg_bytes;
        host_dst->err = src->err;
        __threadfence_system();
        __hip_atomic_store(&host_dst->pad, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
    return x;
}

// --------------------------------------------------------------------------
// Prefilter thresholds from a sample.  One workgroup (512 threads) per tensor.  Tensors of up to
// kSampleMax entries are read completely (the threshold is then the exact k-th key to 16
// bits); larger ones contribute 256 runs of 64 consecutive entries, one run at a pseudo-random
// place in each of 256 equal strata.  With m sampled entries out of n, lambda = k*m/n of them
// are expected among the tensor's k most extreme; the filter key is the lower edge of the
// 16-bit key bucket holding the sample's r-th most extreme entry, r = lambda + 4*sqrt(lambda)
// + 3, so that the chance of cutting into the true top k is negligible (and harmless: the
// histogram path then redoes the tensor).  Both sides are selected together, the negative side
// on complemented keys.  The kernel also clears the per-tensor state, and
// it tells whether the keys the previous call left for this one (they are still in the state when
// the kernel starts) would have held: if the sample says that far more entries than a selection
// wants lie at or above them, kErrStaleKeys is raised, and the host goes on sampling.
// For tensors flagged kDescSampled ("Sparse Binarization": the threshold is estimated from a
// random subsample, which makes the amount of sparsity noisy) the key is instead the full 32-bit
// key of the sample's r-th most extreme entry, r = max(1, floor(p*m)): the threshold itself.
// --------------------------------------------------------------------------
__global__ __launch_bounds__(kSampleThreads) void k_sample_thresholds(
        const TensorDesc* __restrict__ desc, TensorState* __restrict__ st,
        ResultBlock* __restrict__ result, int force_exact, double sampled_p) {
    constexpr int RUNS = kSampleMax / 64;             // 256
    constexpr int COPIES = 16;
    __shared__ uint32_t skey[kSampleMax];             // the sample, as keys (loops stay rolled: small code)
    __shared__ uint32_t hist0[2][256][COPIES];        // first byte: lane-private copies, one bank each
    __shared__ uint32_t hist[4][2][256];
    __shared__ uint32_t whist[2][kSampleWindow];      // leading 16 key bits, counted down from the extreme
    __shared__ uint32_t wave_ext[2][kSampleThreads / 64];
    __shared__ uint32_t wave_above[kSampleThreads / 64];
    __shared__ uint32_t blist[2][kSampleThreads];     // subsampled variant: the sampled keys of the threshold's bucket
    __shared__ uint32_t bcnt[2], btau[2];
    __shared__ uint32_t res[4][8];
    __shared__ unsigned long long scratch[kSampleThreads / 64];
    SBC_TS(0, 0);
    const int t = blockIdx.x, tid = threadIdx.x;
    const TensorDesc d = desc[t];
    const uint32_t old_p = st[t].lo_key[0], old_n = st[t].lo_key[1];      // what the previous call left
    __syncthreads();                                  // (every thread has them before the state is cleared)
    if (tid == 0) {
        // (the call's result block is clean already: the previous call's last kernel, or the host
        // after an error, cleared it.  A plain store to it here would sit in this compute-unit group's
        // L2 until the kernel ends and then overwrite the bits other groups' workgroups raise below.)
        TensorState z;
        z.lo_key[0] = z.lo_key[1] = force_exact ? 0xFFFFFFFFu : 0u;
        z.cand_cnt[0] = z.cand_cnt[1] = 0u;
        z.bin[0] = z.bin[1] = 0u;
        z.tau[0] = z.tau[1] = 0u;
        z.itau[0] = z.itau[1] = 0u;
        z.kc[0] = z.kc[1] = 0u;
        z.S[0] = z.S[1] = 0.0;
        z.side = 0; z.mu_signed = 0.f; z.nnz = 0u; z.flags = 0u; z.bit_len = 0ull;
        z.done = 0u; z.pad = 0u; z.cand_seen[0] = z.cand_seen[1] = 0u; z.expect[0] = z.expect[1] = 0u;
        st[t] = z;
    }
    if (force_exact) return;
    // a one-chunk tensor that the streaming kernel finishes by itself needs no filter key
    if ((d.flags & kDescInline) && d.nchunks == 1u && d.n <= 6144u) return;       // (kSmallMaxN of the streaming kernel)

    const uint32_t n = d.n;
    const uint32_t m = n < (uint32_t)kSampleMax ? n : (uint32_t)kSampleMax;
    const bool sampled = (d.flags & kDescSampled) != 0u;
    uint32_t rs = d.k;
    if (sampled) {
        // "Sparse Binarization", subsampled variant: the r-th most extreme sampled value itself is
        // the threshold, r = max(1, floor(p * m))
        const double r = floor(sampled_p * (double)m);
        rs = r < 1.0 ? 1u : (uint32_t)r;
    } else if (n > (uint32_t)kSampleMax) {
        const double lambda = (double)d.k * (double)m / (double)n;
        rs = (uint32_t)ceil(lambda + 4.0 * sqrt(lambda) + 3.0);
    }
    if (rs >= m) return;                              // keep the all-pass keys (0, 0)
    const int passes = sampled ? 4 : 2;               // all 32 key bits, or the leading 16

    for (int i = tid; i < 3 * 2 * 256; i += kSampleThreads) (&hist[1][0][0])[i] = 0u;
    for (int i = tid; i < 2 * 256 * COPIES; i += kSampleThreads) (&hist0[0][0][0])[i] = 0u;
    for (int i = tid; i < 2 * kSampleWindow; i += kSampleThreads) (&whist[0][0])[i] = 0u;
    __syncthreads();
    uint32_t need[2] = {rs, rs};
    const bool active[2] = {true, true};
    uint32_t prefix[2] = {0u, 0u};
    int first_pass = 0;
    // The sample: all of a thread's loads are issued before the first key is formed, so that the
    // kernel pays the memory latency once.
    const gcfloat_ptr R = as_global(d.R);
    const gcfloat_ptr dW = as_global(d.dW);
    {
        constexpr int PER = kSampleMax / kSampleThreads;      // 32
        float a[PER], w[PER];
        if (n <= (uint32_t)kSampleMax) {
#pragma unroll
            for (int s = 0; s < PER; ++s) {
                const uint32_t i = s * kSampleThreads + tid;
                const uint32_t j = i < m ? i : 0u;
                a[s] = R[j]; w[s] = dW[j];
            }
        } else {
            const unsigned long long slots = n / 64u;     // >= RUNS
            const uint32_t lane = tid & 63u;
#pragma unroll
            for (int s = 0; s < PER; ++s) {
                const uint32_t run = s * (kSampleThreads / 64) + (tid >> 6);             // 0..RUNS-1
                const uint32_t h = mix32(run * 0x9E3779B9u + (uint32_t)t * 0x85EBCA6Bu + 1u);
                const uint32_t s_lo = (uint32_t)(run * slots / RUNS), s_hi = (uint32_t)((run + 1u) * slots / RUNS);
                const uint32_t i = (s_lo + __umulhi(h, s_hi - s_lo)) * 64u + lane;       // a slot of the run's stratum
                a[s] = R[i]; w[s] = dW[i];
            }
        }
        // Keys, and the most extreme key of each side (this thread's, then the workgroup's).
        uint32_t key[PER], ext_p = 0u, ext_n = 0u, above = 0u;       // above: sampled entries at or beyond the old keys, 16 bits per side
#pragma unroll
        for (int s = 0; s < PER; ++s) {
            key[s] = key_of_bits(__float_as_uint(a[s] + w[s]));
            skey[s * kSampleThreads + tid] = key[s];
            if ((uint32_t)(s * kSampleThreads + tid) < m) {
                ext_p = key[s] > ext_p ? key[s] : ext_p;
                ext_n = ~key[s] > ext_n ? ~key[s] : ext_n;
                above += (key[s] >= old_p ? 1u : 0u) + (~key[s] >= old_n ? 0x10000u : 0u);
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const uint32_t op = __shfl_xor(ext_p, off, 64), on = __shfl_xor(ext_n, off, 64);
            ext_p = op > ext_p ? op : ext_p;
            ext_n = on > ext_n ? on : ext_n;
            above += __shfl_xor(above, off, 64);      // (at most 2048 per side and wavefront)
        }
        if ((tid & 63) == 0) { wave_ext[0][tid >> 6] = ext_p; wave_ext[1][tid >> 6] = ext_n; wave_above[tid >> 6] = above; }
        __syncthreads();
        SBC_TS(0, 1);                                 // sample loaded
        if (tid == 0) {
            uint32_t ap = 0u, an = 0u;
            for (int wv = 0; wv < kSampleThreads / 64; ++wv) { ap += wave_above[wv] & 0xFFFFu; an += wave_above[wv] >> 16; }
            // scaled to the tensor; the limit is the one beyond which k_select calls a list loose
            const double scale = (double)n / (double)m, many = (double)loose_limit(d.k, n);
            if ((double)ap * scale > many || (double)an * scale > many) atomicOr(&result->err, kErrStaleKeys);
        }
#pragma unroll
        for (int wv = 0; wv < kSampleThreads / 64; ++wv) {
            ext_p = wave_ext[0][wv] > ext_p ? wave_ext[0][wv] : ext_p;
            ext_n = wave_ext[1][wv] > ext_n ? wave_ext[1][wv] : ext_n;
        }
        // The r-th most extreme key lies within a few octaves of the most extreme one: the leading
        // 16 key bits are counted in a window of kSampleWindow values (16 octaves) below it, straight
        // from the registers; the bulk of the sample spreads over hundreds of bins there, where the
        // leading byte alone takes a handful of values.  Keys below the window are not counted.
        const uint32_t top[2] = {ext_p >> 16, ext_n >> 16};
#pragma unroll
        for (int s = 0; s < PER; ++s) {
            if ((uint32_t)(s * kSampleThreads + tid) < m) {
                const uint32_t dp = top[0] - (key[s] >> 16), dn = top[1] - (~key[s] >> 16);
                if (dp < (uint32_t)(kSampleWindow - 1)) atomicAdd(&whist[0][(uint32_t)(kSampleWindow - 1) - dp], 1u);
                if (dn < (uint32_t)(kSampleWindow - 1)) atomicAdd(&whist[1][(uint32_t)(kSampleWindow - 1) - dn], 1u);
            }
        }
        __syncthreads();
        SBC_TS(0, 2);                                 // window histogram done
        uint32_t digit[2];
        bool found[2];
        pick_wide_both<kSampleWindow, kSampleThreads>(whist, need, active, res[0], scratch, digit, found);
        SBC_TS(0, 3);
        if (found[0] && found[1]) {                   // uniform
            prefix[0] = top[0] - ((uint32_t)(kSampleWindow - 1) - digit[0]);
            prefix[1] = top[1] - ((uint32_t)(kSampleWindow - 1) - digit[1]);
            first_pass = 2;
        } else {
            need[0] = need[1] = rs;                   // (a found side's need was lowered)
        }
        if (sampled && first_pass == 2) {
            // All 32 bits of the r-th key are wanted: the sampled keys of its bucket (a handful) are
            // collected and each is ranked against the others; the one that need[s] - 1 others
            // exceed is the key.  A crowded bucket is left to the byte passes below.
            if (tid < 2) bcnt[tid] = 0u;
            __syncthreads();
#pragma unroll
            for (int s = 0; s < PER; ++s) {
                if ((uint32_t)(s * kSampleThreads + tid) < m) {
                    if ((key[s] >> 16) == prefix[0]) {
                        const uint32_t q = atomicAdd(&bcnt[0], 1u);
                        if (q < (uint32_t)kSampleThreads) blist[0][q] = key[s];
                    }
                    if ((~key[s] >> 16) == prefix[1]) {
                        const uint32_t q = atomicAdd(&bcnt[1], 1u);
                        if (q < (uint32_t)kSampleThreads) blist[1][q] = ~key[s];
                    }
                }
            }
            __syncthreads();
            const uint32_t c0 = bcnt[0], c1 = bcnt[1];
            if (c0 <= (uint32_t)kSampleThreads && c1 <= (uint32_t)kSampleThreads) {      // uniform
#pragma unroll
                for (int sd = 0; sd < 2; ++sd) {
                    const uint32_t cn = sd ? c1 : c0;
                    if ((uint32_t)tid < cn) {
                        const uint32_t me = blist[sd][tid];
                        uint32_t above = 0u, at_least = 0u;
                        for (uint32_t j = 0; j < cn; ++j) {
                            const uint32_t o = blist[sd][j];
                            above += o > me ? 1u : 0u;
                            at_least += o >= me ? 1u : 0u;
                        }
                        if (above < need[sd] && need[sd] <= at_least) btau[sd] = me;   // equal keys write the same value
                    }
                }
                __syncthreads();
                prefix[0] = btau[0]; prefix[1] = btau[1];
                first_pass = 4;
            }
        }
    }
    __syncthreads();
    if (first_pass == 0) {
        // The r-th entry lies below the window (mostly-zero tensors): byte by byte from the top.
        // First byte: floating-point keys take only a handful of values here, so every lane group
        // counts into its own copy and the copies are added up afterwards.
        const int copy = ((tid >> 6) & 1) * 8 + (tid & 7);
#pragma unroll 8
        for (uint32_t i = tid; i < m; i += kSampleThreads) {
            const uint32_t kp = skey[i];
            atomicAdd(&hist0[0][kp >> 24][copy], 1u);
            atomicAdd(&hist0[1][(~kp) >> 24][copy], 1u);
        }
        __syncthreads();
        if (tid < 2 * 256) {
            uint32_t sum = 0u;
#pragma unroll
            for (int c = 0; c < COPIES; ++c) sum += (&hist0[0][0][0])[tid * COPIES + c];   // tid = side*256 + byte
            (&hist[0][0][0])[tid] = sum;
        }
        __syncthreads();
    }
    SBC_TS(0, 2);                                     // first-byte histogram done
    // the remaining bytes of the r-th largest key (positive side) and of the r-th largest
    // complemented key (negative side), one byte per pass
#pragma nounroll
    for (int pass = first_pass; pass < passes; ++pass) {
        if (pass > 0) {
            const int shift = 24 - 8 * pass;
#pragma unroll 8
            for (uint32_t i = tid; i < m; i += kSampleThreads) {
                const uint32_t kp = skey[i], kn = ~kp;
                if ((kp >> (shift + 8)) == prefix[0]) atomicAdd(&hist[pass][0][(kp >> shift) & 255u], 1u);
                if ((kn >> (shift + 8)) == prefix[1]) atomicAdd(&hist[pass][1][(kn >> shift) & 255u], 1u);
            }
            __syncthreads();
        }
        SBC_TS(0, 3 + 2 * pass);
        const BytePick pk = pick_byte_both<kSampleThreads>(hist[pass], need, active, res[pass], scratch);
        SBC_TS(0, 4 + 2 * pass);
        if (!pk.found[0] || !pk.found[1]) return;     // uniform; cannot happen; all-pass keys stay
        prefix[0] = (prefix[0] << 8) | pk.byte[0];
        prefix[1] = (prefix[1] << 8) | pk.byte[1];
    }
    SBC_TS(0, 11);
    if (tid == 0) {
        const int left = 32 - 8 * passes;             // 16: lower edge of the 16-bit bucket; 0: the key itself
        st[t].lo_key[0] = prefix[0] << left;
        st[t].lo_key[1] = prefix[1] << left;          // same, in the complemented key space
    }
}

// --------------------------------------------------------------------------
// Appends flagged entries of one chunk to the two candidate lists of its tensor with a block
// scan: used by the histogram path and as the second try of a chunk whose LDS queue
// overflowed.  key[s] is the plain key of the thread's s-th entry (entry s*NT + tid of the
// chunk); bit s of mp / mn flags it for the positive / negative list; the negative list stores
// complemented keys.  Contains barriers; every thread of the workgroup must call it.
// --------------------------------------------------------------------------
template <int PER>
__device__ __forceinline__ void append_candidates(const uint32_t (&key)[PER], uint32_t mp, uint32_t mn,
                                                  uint32_t e_first, const TensorDesc& d, TensorState* __restrict__ st_t,
                                                  uint2* __restrict__ cand, ResultBlock* __restrict__ result,
                                                  uint32_t* scratch, uint32_t* base) {
    const int tid = threadIdx.x;
    const uint32_t packed = __popc(mp) | (__popc(mn) << 16);
    uint32_t total;
    const uint32_t ex = block_excl_sum<uint32_t, kStreamThreads>(packed, &total, scratch);
    if (total == 0u) return;                          // uniform
    if (tid == 0) {
        const uint32_t tp = total & 0xFFFFu, tn = total >> 16;
        const unsigned long long old = atomicAdd(reinterpret_cast<unsigned long long*>(&st_t->cand_cnt[0]),
                                                 (unsigned long long)tp | ((unsigned long long)tn << 32));
        base[0] = (uint32_t)old;
        base[1] = (uint32_t)(old >> 32);
    }
    __syncthreads();
    uint32_t op = base[0] + (ex & 0xFFFFu);
    uint32_t on = base[1] + (ex >> 16);
    __syncthreads();                                  // base may be rewritten by the next call
    // (beyond a list's capacity nothing is stored: the counters then show that the tensor's lists
    // are not usable, see k_select; a list of a full context holds every entry)
    if (op + __popc(mp) > d.cand_cap || on + __popc(mn) > d.cand_cap) return;
    uint2* __restrict__ cp = cand + d.cand_off;
    uint2* __restrict__ cn = cand + d.cand_off + d.cand_cap;
#pragma unroll
    for (int s = 0; s < PER; ++s) {
        const uint32_t idx = e_first + s * kStreamThreads + tid;
        if (mp & (1u << s)) cp[op++] = make_uint2(key[s], idx);
        if (mn & (1u << s)) cn[on++] = make_uint2(~key[s], idx);
    }
}

// --------------------------------------------------------------------------
// Residual accumulation fused with the prefilter.  One workgroup per chunk of 8192 entries:
// 8 x 16-byte loads of each operand in flight per thread, A stored over R, and the few
// entries at or beyond a side's filter key queued in LDS, then appended to the tensor's
// candidate list with one atomic per side.  A chunk with more candidates than the queue
// holds (tie-heavy or constant data) appends them again from a second read of its entries.
// Chunks of tensors that are encoded from the bitmap also clear their bitmap words and their
// share of the tensor's staging words.
// --------------------------------------------------------------------------
struct FilterShared {
    uint2 queue[2][kFilterQueue];
    uint32_t qcnt[2];
    uint32_t base[2];
    uint32_t scratch[kStreamThreads / 64];
};

__device__ __forceinline__ void filter_entry(float a, uint32_t idx, uint32_t lo_p, uint32_t lo_n,
                                             FilterShared& sh, uint32_t& bad) {
    const uint32_t u = __float_as_uint(a);
    if ((u & 0x7F800000u) == 0x7F800000u) bad = 1u;
    const uint32_t kk = key_of_bits(u);
    if (kk >= lo_p) {
        const uint32_t s = atomicAdd(&sh.qcnt[0], 1u);
        if (s < (uint32_t)kFilterQueue) sh.queue[0][s] = make_uint2(kk, idx);
    }
    if (~kk >= lo_n) {
        const uint32_t s = atomicAdd(&sh.qcnt[1], 1u);
        if (s < (uint32_t)kFilterQueue) sh.queue[1][s] = make_uint2(~kk, idx);
    }
}

// STREAM: the update is loaded with the nontemporal hint.  It is read exactly once, and when a
// call's footprint is well beyond the last-level cache, keeping it out of that cache leaves more
// of it to the residual, which is read and written.
template <bool STREAM>
__global__ __launch_bounds__(kStreamThreads) void k_accumulate_filter(
        const TensorDesc* __restrict__ desc, const uint2* __restrict__ sched,
        TensorState* __restrict__ st, uint2* __restrict__ cand, uint32_t* __restrict__ bitmap,
        uint32_t* __restrict__ stage, ResultBlock* __restrict__ result) {
    __shared__ FilterShared sh;
    const int tid = threadIdx.x;
    // sched[workgroup] = (first chunk in the call-wide numbering, tensor | consecutive chunks of it << 24)
    const uint2 sc = sched[blockIdx.x];
    const int t = (int)(sc.y & 0xFFFFFFu);
    const uint32_t n_sub = sc.y >> 24;
    const TensorDesc d = desc[t];
    const uint32_t lo_p = st[t].lo_key[0], lo_n = st[t].lo_key[1];
    if (tid < 2) sh.qcnt[tid] = 0u;
    __syncthreads();
    uint32_t bad = 0u;

#pragma unroll 1
    for (uint32_t sub = 0; sub < n_sub; ++sub) {
        const uint32_t c = sc.x + sub;
        const uint32_t cc = c - d.chunk0;
        const uint32_t e0 = cc * (uint32_t)kChunk;
        const uint32_t cnt = min((uint32_t)kChunk, d.n - e0);
        if (!(d.flags & kDescFused)) {
            bitmap[(uint64_t)c * kChunkWords + tid] = 0u;
            const uint32_t per = (d.bound_words + d.nchunks - 1u) / d.nchunks;
            const uint32_t lo = per * cc;
            const uint32_t hi = (lo + per < d.bound_words) ? lo + per : d.bound_words;
            for (uint32_t w = lo + tid; w < hi; w += kStreamThreads) stage[d.stage_off + w] = 0u;
        }
        const gcfloat_ptr dw = as_global(d.dW + e0);
        const gfloat_ptr r = as_global(d.R + e0);
        const bool vec = (cnt == (uint32_t)kChunk) && ((((uintptr_t)(d.dW + e0) | (uintptr_t)(d.R + e0)) & 15u) == 0u);
        if (vec) {
            const gcf32x4_ptr dw4 = (gcf32x4_ptr)dw;
            const gf32x4_ptr r4 = (gf32x4_ptr)r;
            constexpr int IT = kChunk / 4 / kStreamThreads;   // 8
            f32x4 dv[IT], rv[IT];
#pragma unroll
            for (int i = 0; i < IT; ++i) {
                dv[i] = STREAM ? __builtin_nontemporal_load(&dw4[i * kStreamThreads + tid]) : dw4[i * kStreamThreads + tid];
                rv[i] = r4[i * kStreamThreads + tid];
            }
#pragma unroll
            for (int i = 0; i < IT; ++i) {
                f32x4 a;
                a.x = rv[i].x + dv[i].x;
                a.y = rv[i].y + dv[i].y;
                a.z = rv[i].z + dv[i].z;
                a.w = rv[i].w + dv[i].w;
                r4[i * kStreamThreads + tid] = a;
                const uint32_t idx = e0 + (i * kStreamThreads + tid) * 4;
                filter_entry(a.x, idx + 0, lo_p, lo_n, sh, bad);
                filter_entry(a.y, idx + 1, lo_p, lo_n, sh, bad);
                filter_entry(a.z, idx + 2, lo_p, lo_n, sh, bad);
                filter_entry(a.w, idx + 3, lo_p, lo_n, sh, bad);
            }
        } else {
            // a tensor's last, partial chunk, or operands that are only 4-byte aligned: eight entries per
            // thread in flight at a time (later loads may not pass earlier stores to the same array,
            // so a plain loop would pay the memory latency once per entry)
            constexpr int IT = 8;
            for (uint32_t base = 0; base < cnt; base += IT * kStreamThreads) {
                float dv[IT], rv[IT];
#pragma unroll
                for (int j = 0; j < IT; ++j) {
                    const uint32_t i = base + j * kStreamThreads + tid;
                    const uint32_t ii = i < cnt ? i : 0u;
                    dv[j] = dw[ii];
                    rv[j] = r[ii];
                }
#pragma unroll
                for (int j = 0; j < IT; ++j) {
                    const uint32_t i = base + j * kStreamThreads + tid;
                    if (i < cnt) {
                        const float a = rv[j] + dv[j];
                        r[i] = a;
                        filter_entry(a, e0 + i, lo_p, lo_n, sh, bad);
                    }
                }
            }
        }
    }
    if (bad) atomicOr(&result->err, kErrNonFinite);
    __syncthreads();
    const uint32_t qp = sh.qcnt[0], qn = sh.qcnt[1];
    if (qp <= (uint32_t)kFilterQueue && qn <= (uint32_t)kFilterQueue) {
        if (qp + qn == 0u) return;
        if (tid == 0) {
            // both sides' counters advance in one 64-bit atomic: workgroups of one tensor queue up
            // on this address, and the wait grows with the number of atomics
            const unsigned long long old = atomicAdd(reinterpret_cast<unsigned long long*>(&st[t].cand_cnt[0]),
                                                     (unsigned long long)qp | ((unsigned long long)qn << 32));
            sh.base[0] = (uint32_t)old;
            sh.base[1] = (uint32_t)(old >> 32);
        }
        __syncthreads();
        // (beyond a list's capacity nothing is stored: see append_candidates)
        if ((uint64_t)sh.base[0] + qp > d.cand_cap || (uint64_t)sh.base[1] + qn > d.cand_cap) return;
        uint2* __restrict__ cp = cand + d.cand_off + sh.base[0];
        uint2* __restrict__ cn = cand + d.cand_off + d.cand_cap + sh.base[1];
        for (uint32_t i = tid; i < qp; i += kStreamThreads) cp[i] = sh.queue[0][i];
        for (uint32_t i = tid; i < qn; i += kStreamThreads) cn[i] = sh.queue[1][i];
        return;
    }
    // queue overflow: append the candidates of this workgroup's chunks from a second read of A,
    // 4096 entries at a time (the barrier above ordered the workgroup's stores of A before these
    // loads).  Filter keys that let a flood pass send most workgroups of a call this way, so a step
    // takes as many entries as the scan's 16-bit counts per side allow.
    constexpr int kRedo = 16;
    static_assert(kRedo * kStreamThreads <= 65535, "the per-side counts of one step fit their 16-bit fields");
    for (uint32_t sub = 0; sub < n_sub; ++sub) {
        const uint32_t e0 = (sc.x + sub - d.chunk0) * (uint32_t)kChunk;
        const uint32_t cnt = min((uint32_t)kChunk, d.n - e0);
        const gcfloat_ptr r = as_global(d.R + e0);
        for (uint32_t off = 0; off < cnt; off += kRedo * kStreamThreads) {
            uint32_t key[kRedo];
            uint32_t mp = 0u, mn = 0u;
#pragma unroll
            for (int s = 0; s < kRedo; ++s) {
                const uint32_t i = off + s * kStreamThreads + tid;
                key[s] = __float_as_uint(r[i < cnt ? i : 0u]);
            }
#pragma unroll
            for (int s = 0; s < kRedo; ++s) {
                const uint32_t i = off + s * kStreamThreads + tid;
                const bool in = i < cnt;
                key[s] = key_of_bits(key[s]);
                if (in && key[s] >= lo_p) mp |= 1u << s;
                if (in && ~key[s] >= lo_n) mn |= 1u << s;
            }
            append_candidates<kRedo>(key, mp, mn, e0 + off, d, &st[t], cand, result, sh.scratch, sh.base);
        }
    }
}

// --------------------------------------------------------------------------
// Histogram path, used only for tensors whose prefilter failed (kStFailed).
// k_hist_flagged: per chunk, first-digit histogram of A (already stored in R).
// --------------------------------------------------------------------------
__global__ __launch_bounds__(kStreamThreads) void k_hist_flagged(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ chunk_tensor,
        const TensorState* __restrict__ st, uint32_t* __restrict__ hist) {
    __shared__ uint32_t lh[kL1Bins];
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    const int t = (int)chunk_tensor[c];
    if (!(st[t].flags & kStFailed)) return;
    const TensorDesc d = desc[t];
    const uint32_t e0 = (c - d.chunk0) * (uint32_t)kChunk;
    const uint32_t cnt = min((uint32_t)kChunk, d.n - e0);
    for (int i = tid; i < kL1Bins; i += kStreamThreads) lh[i] = 0u;
    __syncthreads();
    const gcfloat_ptr a = as_global(d.R + e0);
    uint32_t zeros = 0u;
    for (uint32_t i = tid; i < cnt; i += kStreamThreads) {
        const uint32_t u = __float_as_uint(a[i]);
        if ((u << 1) == 0u) ++zeros;
        else atomicAdd(&lh[key_of_bits(u) >> kL1Shift], 1u);
    }
    if (zeros) atomicAdd(&lh[0x80000000u >> kL1Shift], zeros);
    __syncthreads();
    uint32_t* __restrict__ gh = hist + (size_t)t * kL1Bins;
    for (int i = tid; i < kL1Bins; i += kStreamThreads) {
        const uint32_t v = lh[i];
        if (v) atomicAdd(&gh[i], v);
    }
}

// k_pick_bins: per flagged tensor, the bins that hold the k-th largest and k-th smallest
// entry; the tensor's candidate lists restart empty and it is handed to the exact pass.
__global__ __launch_bounds__(256) void k_pick_bins(const TensorDesc* __restrict__ desc,
                                                   const uint32_t* __restrict__ hist,
                                                   TensorState* __restrict__ st,
                                                   ResultBlock* __restrict__ result) {
    __shared__ uint32_t h[kL1Bins];
    __shared__ uint32_t res[2];
    __shared__ uint32_t scratch[4];
    const int t = blockIdx.x, tid = threadIdx.x;
    if (!(st[t].flags & kStFailed)) return;
    const uint32_t k = desc[t].k;
    for (int i = tid; i < kL1Bins; i += 256) h[i] = hist[(size_t)t * kL1Bins + i];
    __syncthreads();
    find_from_top<kL1Bins, 256, false>(h, k, res, scratch);
    const uint32_t bp = res[0];
    __syncthreads();
    find_from_top<kL1Bins, 256, true>(h, k, res, scratch);
    const uint32_t bn = res[0];
    if (tid == 0) {
        if (bp == 0xFFFFFFFFu || bn == 0xFFFFFFFFu) atomicOr(&result->err, kErrInternal);
        st[t].bin[0] = bp;
        st[t].bin[1] = bn;                            // complemented-key numbering
        st[t].lo_key[0] = bp << kL1Shift;             // every candidate's side key is at or above these
        st[t].lo_key[1] = bn << kL1Shift;
        st[t].cand_cnt[0] = 0u; st[t].cand_cnt[1] = 0u;
        st[t].flags = kStExact;
    }
}

// k_extract: per chunk of a tensor in the exact pass, every entry whose first digit lies in or
// beyond a side's threshold bin becomes a candidate of that side.
__global__ __launch_bounds__(kStreamThreads) void k_extract(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ chunk_tensor,
        TensorState* __restrict__ st, uint2* __restrict__ cand, ResultBlock* __restrict__ result) {
    constexpr int PER = kChunk / kStreamThreads;
    __shared__ uint32_t scratch[kStreamThreads / 64];
    __shared__ uint32_t base[2];
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    const int t = (int)chunk_tensor[c];
    if (!(st[t].flags & kStExact)) return;
    const TensorDesc d = desc[t];
    const uint32_t e0 = (c - d.chunk0) * (uint32_t)kChunk;
    const uint32_t cnt = min((uint32_t)kChunk, d.n - e0);
    const uint32_t bin_p = st[t].bin[0];
    const uint32_t bin_n = (uint32_t)(kL1Bins - 1) - st[t].bin[1];  // in the plain key space
    const gcfloat_ptr a = as_global(d.R + e0);
    uint32_t key[PER];
    uint32_t mp = 0u, mn = 0u;
#pragma unroll
    for (int s = 0; s < PER; ++s) {
        const uint32_t i = s * kStreamThreads + tid;
        const bool in = i < cnt;
        key[s] = key_of_bits(__float_as_uint(a[in ? i : 0u]));
        const uint32_t bin = key[s] >> kL1Shift;
        if (in && bin >= bin_p) mp |= 1u << s;
        if (in && bin <= bin_n) mn |= 1u << s;
    }
    append_candidates<PER>(key, mp, mn, e0, d, &st[t], cand, result, scratch, base);
}

}  // namespace sbc
