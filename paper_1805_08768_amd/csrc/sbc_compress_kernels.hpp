// Kernels of the client step: residual accumulation with a first-digit histogram,
// threshold-bin choice, candidate extraction, exact per-tensor selection on both sign
// sides with means, binarization and residual update, and Golomb encoding of the kept
// positions from a bitmap.
#pragma once

#include "sbc_device.hpp"

namespace sbc {

// --------------------------------------------------------------------------
// Reset of per-call scratch: histograms, per-tensor state, result block.
// --------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_reset(uint32_t* __restrict__ hist, uint32_t hist_words,
                                               uint32_t* __restrict__ state_words, uint32_t n_state_words,
                                               ResultBlock* __restrict__ result) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t stride = gridDim.x * blockDim.x;
    for (uint32_t j = i; j < hist_words; j += stride) hist[j] = 0u;
    for (uint32_t j = i; j < n_state_words; j += stride) state_words[j] = 0u;
    if (i == 0) { result->err = 0u; result->pad = 0u; result->msg_bytes = 0ull; }
}

// --------------------------------------------------------------------------
// Plain streaming copy of 16-byte units, the yardstick the streaming kernels are measured
// against (same workgroup shape and loads in flight as the accumulation kernel).
// --------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_copy_baseline(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                       uint64_t n16) {
    const uint64_t base = (uint64_t)blockIdx.x * 2048ull + threadIdx.x;
    uint4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) if (base + 256ull * i < n16) v[i] = src[base + 256ull * i];
#pragma unroll
    for (int i = 0; i < 8; ++i) if (base + 256ull * i < n16) dst[base + 256ull * i] = v[i];
}

// --------------------------------------------------------------------------
// Stage 1 (Alg. 1, client: dW_i <- R_i + local update): A = R + dW written over R, plus
// the per-tensor histogram of the first key digit.  One workgroup per chunk.  The same
// pass clears the chunk's slice of the kept-position bitmap and a slice of the message
// payload.
// --------------------------------------------------------------------------
struct Tally {
    uint32_t zeros = 0;
    uint32_t bad = 0;
    __device__ __forceinline__ void add(float a, uint32_t* lh) {
        const uint32_t u = __float_as_uint(a);
        if ((u & 0x7F800000u) == 0x7F800000u) bad = 1u;
        if ((u << 1) == 0u) ++zeros;
        else atomicAdd(&lh[key_of_bits(u) >> kL1Shift], 1u);
    }
};

__global__ __launch_bounds__(kStreamThreads) void k_accumulate_hist(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ chunk_start, int T,
        uint32_t* __restrict__ hist, uint32_t* __restrict__ bitmap,
        uint32_t* __restrict__ payload, uint64_t zero_words, ResultBlock* __restrict__ result) {
    __shared__ uint32_t lh[kL1Bins];
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    const int t = tensor_of_chunk(chunk_start, T, c);
    const TensorDesc d = desc[t];
    const uint32_t e0 = (c - d.chunk0) * (uint32_t)kChunk;
    const uint32_t cnt = min((uint32_t)kChunk, d.n - e0);

#pragma unroll
    for (int j = 0; j < kL1Bins / kStreamThreads; ++j) lh[j * kStreamThreads + tid] = 0u;
    bitmap[(uint64_t)c * kChunkWords + tid] = 0u;
    {   // this workgroup's share of the payload words that must start out zero
        const uint64_t per = (zero_words + gridDim.x - 1) / gridDim.x;
        const uint64_t lo = per * c;
        const uint64_t hi = (lo + per < zero_words) ? lo + per : zero_words;
        for (uint64_t w = lo + tid; w < hi; w += kStreamThreads) payload[w] = 0u;
    }
    __syncthreads();

    Tally tally;
    const float* __restrict__ dw = d.dW + e0;
    float* __restrict__ r = d.R + e0;
    const bool vec = (cnt == (uint32_t)kChunk) &&
                     ((((uintptr_t)dw | (uintptr_t)r) & 15u) == 0u);
    if (vec) {
        const float4* __restrict__ dw4 = reinterpret_cast<const float4*>(dw);
        float4* __restrict__ r4 = reinterpret_cast<float4*>(r);
        constexpr int IT = kChunk / 4 / kStreamThreads;  // 8
        float4 dv[IT], rv[IT];
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            dv[i] = dw4[i * kStreamThreads + tid];
            rv[i] = r4[i * kStreamThreads + tid];
        }
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            float4 a;
            a.x = rv[i].x + dv[i].x;
            a.y = rv[i].y + dv[i].y;
            a.z = rv[i].z + dv[i].z;
            a.w = rv[i].w + dv[i].w;
            r4[i * kStreamThreads + tid] = a;
            tally.add(a.x, lh); tally.add(a.y, lh); tally.add(a.z, lh); tally.add(a.w, lh);
        }
    } else {
        for (uint32_t i = tid; i < cnt; i += kStreamThreads) {
            const float a = r[i] + dw[i];
            r[i] = a;
            tally.add(a, lh);
        }
    }
    if (tally.zeros) atomicAdd(&lh[0x80000000u >> kL1Shift], tally.zeros);
    if (tally.bad) atomicOr(&result->err, kErrNonFinite);
    __syncthreads();
    uint32_t* __restrict__ gh = hist + (size_t)t * kL1Bins;
#pragma unroll
    for (int j = 0; j < kL1Bins / kStreamThreads; ++j) {
        const uint32_t v = lh[j * kStreamThreads + tid];
        if (v) atomicAdd(&gh[j * kStreamThreads + tid], v);
    }
}

// --------------------------------------------------------------------------
// Stage 2a (Alg. 2, top_p% on both sides): from the first-digit histogram choose, per
// tensor, the bin that holds the k-th largest entry (positive side) and the k-th smallest
// (negative side, expressed in the complemented key space).  One workgroup per tensor.
// --------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_pick_bins(const TensorDesc* __restrict__ desc,
                                                   const uint32_t* __restrict__ hist,
                                                   TensorState* __restrict__ st,
                                                   ResultBlock* __restrict__ result) {
    __shared__ uint32_t h[kL1Bins];
    __shared__ uint32_t res[2];
    __shared__ uint32_t scratch[4];
    const int t = blockIdx.x, tid = threadIdx.x;
    const uint32_t k = desc[t].k;
#pragma unroll
    for (int j = 0; j < kL1Bins / 256; ++j) h[j * 256 + tid] = hist[(size_t)t * kL1Bins + j * 256 + tid];
    __syncthreads();
    find_from_top<kL1Bins, 256, false>(h, k, res, scratch);
    const uint32_t bp = res[0], ap = res[1];
    __syncthreads();
    find_from_top<kL1Bins, 256, true>(h, k, res, scratch);
    const uint32_t bn = res[0], an = res[1];
    if (tid == 0) {
        if (bp == 0xFFFFFFFFu || bn == 0xFFFFFFFFu) atomicOr(&result->err, kErrInternal);
        st[t].bin[0] = bp; st[t].above[0] = ap;
        st[t].bin[1] = bn; st[t].above[1] = an;
        st[t].cand_cnt[0] = 0u; st[t].cand_cnt[1] = 0u;
    }
}

// --------------------------------------------------------------------------
// Stage 2b: second read of A.  Every entry whose first digit lies in or beyond the
// threshold bin of a side is appended, as (side key, index), to that side's candidate
// list; the negative side stores the complemented key, so that "largest key" means "most
// extreme value" on both sides.  One workgroup per chunk, one atomic per side per
// workgroup; the order of candidates in a list is arbitrary.
// --------------------------------------------------------------------------
__global__ __launch_bounds__(kStreamThreads) void k_extract(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ chunk_start, int T,
        TensorState* __restrict__ st, uint2* __restrict__ cand, int reverse,
        ResultBlock* __restrict__ result) {
    constexpr int PER = kChunk / kStreamThreads;  // 32 entries per thread
    __shared__ uint32_t scratch[kStreamThreads / 64];
    __shared__ uint32_t base[2];
    const int tid = threadIdx.x;
    const uint32_t c = reverse ? (gridDim.x - 1 - blockIdx.x) : blockIdx.x;
    const int t = tensor_of_chunk(chunk_start, T, c);
    const TensorDesc d = desc[t];
    const uint32_t e0 = (c - d.chunk0) * (uint32_t)kChunk;
    const uint32_t cnt = min((uint32_t)kChunk, d.n - e0);
    const uint32_t bin_p = st[t].bin[0];
    const uint32_t bin_n = (uint32_t)(kL1Bins - 1) - st[t].bin[1];  // in the plain key space

    const float* __restrict__ a = d.R + e0;
    uint32_t key[PER];
    const bool vec = (cnt == (uint32_t)kChunk) && (((uintptr_t)a & 15u) == 0u);
    if (vec) {
        const uint4* __restrict__ a4 = reinterpret_cast<const uint4*>(a);
#pragma unroll
        for (int i = 0; i < PER / 4; ++i) {
            const uint4 v = a4[i * kStreamThreads + tid];
            key[4 * i + 0] = key_of_bits(v.x); key[4 * i + 1] = key_of_bits(v.y);
            key[4 * i + 2] = key_of_bits(v.z); key[4 * i + 3] = key_of_bits(v.w);
        }
    } else {
#pragma unroll
        for (int s = 0; s < PER; ++s) {
            const uint32_t i = s * kStreamThreads + tid;
            // entries past the end get the key of zero and are masked out below
            key[s] = (i < cnt) ? key_of_bits(__float_as_uint(a[i])) : 0x80000000u;
        }
    }
    uint32_t mp = 0u, mn = 0u;
#pragma unroll
    for (int s = 0; s < PER; ++s) {
        const uint32_t local = vec ? ((s >> 2) * kStreamThreads + tid) * 4 + (s & 3)
                                   : s * kStreamThreads + tid;
        const uint32_t bin = key[s] >> kL1Shift;
        const bool in = local < cnt;
        if (in && bin >= bin_p) mp |= 1u << s;
        if (in && bin <= bin_n) mn |= 1u << s;
    }
    const uint32_t packed = __popc(mp) | (__popc(mn) << 16);
    uint32_t total;
    const uint32_t ex = block_excl_sum<uint32_t, kStreamThreads>(packed, &total, scratch);
    if (tid == 0) {
        const uint32_t tp = total & 0xFFFFu, tn = total >> 16;
        base[0] = tp ? atomicAdd(&st[t].cand_cnt[0], tp) : 0u;
        base[1] = tn ? atomicAdd(&st[t].cand_cnt[1], tn) : 0u;
    }
    __syncthreads();
    uint32_t op = base[0] + (ex & 0xFFFFu);
    uint32_t on = base[1] + (ex >> 16);
    if (op + __popc(mp) > d.n || on + __popc(mn) > d.n) {  // cannot happen: a list holds at most n
        atomicOr(&result->err, kErrInternal);
        return;
    }
    uint2* __restrict__ cp = cand + d.cand_off;
    uint2* __restrict__ cn = cand + d.cand_off + d.n;
#pragma unroll
    for (int s = 0; s < PER; ++s) {
        const uint32_t local = vec ? ((s >> 2) * kStreamThreads + tid) * 4 + (s & 3)
                                   : s * kStreamThreads + tid;
        if (mp & (1u << s)) cp[op++] = make_uint2(key[s], e0 + local);
        if (mn & (1u << s)) cn[on++] = make_uint2(~key[s], e0 + local);
    }
}

// --------------------------------------------------------------------------
// Stages 2c-5 (Alg. 2 in full, then Alg. 1's residual line), one workgroup per tensor:
//   * radix select on the candidates of each side for the exact k-th key tau and the
//     number r of entries equal to tau that are kept; if fewer than all ties are kept,
//     a second radix select over the tied indices finds the r lowest (ties go to the
//     lowest index);
//   * S+ and S-: sums of the k kept values per side, accumulated as exact integers per
//     fp32 exponent (order independent), combined in a fixed order in fp64;
//   * side: positive iff mu+ >= mu-, which for equal counts is S+ >= S-;
//   * R[j] = A[j] - mu_signed and bitmap bit j set for the kept entries of that side.
// --------------------------------------------------------------------------
struct SelectShared {
    uint32_t hist[kDigBins];
    long long acc[256];
    uint32_t res[2];
    uint32_t scratch[kSelThreads / 64];
    double S[2];
};

__device__ __forceinline__ bool cand_kept(uint32_t key, uint32_t idx, uint32_t tau, uint32_t itau) {
    return key > tau || (key == tau && idx <= itau);
}

template <int NB>
__device__ __forceinline__ void zero_hist(uint32_t* h) {
    for (int i = threadIdx.x; i < NB; i += kSelThreads) h[i] = 0u;
    __syncthreads();
}

// Exact selection on one side's candidate list.  Returns tau (the k-th largest side key) and
// itau (entries equal to tau are kept while their index is <= itau), and leaves the sum of
// the kept values in sh.S[side].  Every thread of the workgroup must call it.
__device__ __forceinline__ void select_side(SelectShared& sh, const uint2* __restrict__ cl, uint32_t cnt,
                                            uint32_t B, uint32_t need0, int side,
                                            uint32_t& tau_out, uint32_t& itau_out, bool& failed) {
    const int tid = threadIdx.x;

    // second digit among candidates of the threshold bin
    zero_hist<kDigBins>(sh.hist);
    for (uint32_t i = tid; i < cnt; i += kSelThreads) {
        const uint32_t kp = cl[i].x;
        if ((kp >> kL1Shift) == B) atomicAdd(&sh.hist[(kp >> kDigBits) & (kDigBins - 1)], 1u);
    }
    __syncthreads();
    find_from_top<kDigBins, kSelThreads, false>(sh.hist, need0, sh.res, sh.scratch);
    const uint32_t d2 = sh.res[0];
    const uint32_t need1 = need0 - sh.res[1];
    if (d2 == 0xFFFFFFFFu) failed = true;
    const uint32_t prefix = (B << kDigBits) | (d2 & (kDigBins - 1));

    // third digit
    zero_hist<kDigBins>(sh.hist);
    for (uint32_t i = tid; i < cnt; i += kSelThreads) {
        const uint32_t kp = cl[i].x;
        if ((kp >> kDigBits) == prefix) atomicAdd(&sh.hist[kp & (kDigBins - 1)], 1u);
    }
    __syncthreads();
    find_from_top<kDigBins, kSelThreads, false>(sh.hist, need1, sh.res, sh.scratch);
    const uint32_t d3 = sh.res[0];
    if (d3 == 0xFFFFFFFFu) failed = true;
    const uint32_t r = need1 - sh.res[1];                 // ties to keep (>= 1)
    const uint32_t ties = sh.hist[d3 & (kDigBins - 1)];   // entries equal to tau
    const uint32_t tau = (prefix << kDigBits) | (d3 & (kDigBins - 1));
    uint32_t itau = 0xFFFFFFFFu;
    __syncthreads();                                      // everyone has read hist and res

    if (!failed && r < ties) {
        // the r lowest indices among the ties: select the r-th largest of ~idx
        zero_hist<kDigBins>(sh.hist);
        for (uint32_t i = tid; i < cnt; i += kSelThreads) {
            const uint2 e = cl[i];
            if (e.x == tau) atomicAdd(&sh.hist[(~e.y) >> 22], 1u);
        }
        __syncthreads();
        find_from_top<kL1Bins, kSelThreads, false>(sh.hist, r, sh.res, sh.scratch);
        const uint32_t dA = sh.res[0];
        const uint32_t needB = r - sh.res[1];
        if (dA == 0xFFFFFFFFu) failed = true;
        zero_hist<kDigBins>(sh.hist);
        for (uint32_t i = tid; i < cnt; i += kSelThreads) {
            const uint2 e = cl[i];
            const uint32_t ri = ~e.y;
            if (e.x == tau && (ri >> 22) == dA) atomicAdd(&sh.hist[(ri >> kDigBits) & (kDigBins - 1)], 1u);
        }
        __syncthreads();
        find_from_top<kDigBins, kSelThreads, false>(sh.hist, needB, sh.res, sh.scratch);
        const uint32_t dB = sh.res[0];
        const uint32_t needC = needB - sh.res[1];
        if (dB == 0xFFFFFFFFu) failed = true;
        const uint32_t pfx = ((dA & (kL1Bins - 1)) << kDigBits) | (dB & (kDigBins - 1));
        zero_hist<kDigBins>(sh.hist);
        for (uint32_t i = tid; i < cnt; i += kSelThreads) {
            const uint2 e = cl[i];
            const uint32_t ri = ~e.y;
            if (e.x == tau && (ri >> kDigBits) == pfx) atomicAdd(&sh.hist[ri & (kDigBins - 1)], 1u);
        }
        __syncthreads();
        find_from_top<kDigBins, kSelThreads, false>(sh.hist, needC, sh.res, sh.scratch);
        const uint32_t dC = sh.res[0];
        if (dC == 0xFFFFFFFFu) failed = true;
        itau = ~((pfx << kDigBits) | (dC & (kDigBins - 1)));
        __syncthreads();
    }
    tau_out = tau;
    itau_out = itau;

    // sum of the kept values: exact integer accumulation per exponent
    for (int i = tid; i < 256; i += kSelThreads) sh.acc[i] = 0ll;
    __syncthreads();
    for (uint32_t i = tid; i < cnt; i += kSelThreads) {
        const uint2 e = cl[i];
        if (cand_kept(e.x, e.y, tau, itau)) {
            const uint32_t u = bits_of_key(side ? ~e.x : e.x);
            const uint32_t ex = (u >> 23) & 0xFFu;
            long long m = (long long)(ex ? ((u & 0x7FFFFFu) | 0x800000u) : (u & 0x7FFFFFu));
            const bool neg = ((u >> 31) != 0u) != (side != 0);   // the negative side sums -A
            if (neg) m = -m;
            atomicAdd(reinterpret_cast<unsigned long long*>(&sh.acc[ex ? ex : 1u]),
                      (unsigned long long)m);
        }
    }
    __syncthreads();
    if (tid < 64) {
        // fixed order: lane l adds exponents 4l..4l+3 ascending, then a fixed shuffle tree
        double s = 0.0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int ex = 4 * tid + j;
            s += ldexp((double)sh.acc[ex], ex - 150);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_down(s, off, 64);
        if (tid == 0) sh.S[side] = s;
    }
    __syncthreads();
}

__global__ __launch_bounds__(kSelThreads) void k_select_apply(
        const TensorDesc* __restrict__ desc, TensorState* __restrict__ st,
        const uint2* __restrict__ cand, uint32_t* __restrict__ bitmap,
        ResultBlock* __restrict__ result) {
    __shared__ SelectShared sh;
    const int t = blockIdx.x, tid = threadIdx.x;
    const TensorDesc d = desc[t];
    bool failed = false;
    uint32_t tau_p, itau_p, tau_n, itau_n;
    const uint32_t cnt_p = st[t].cand_cnt[0], cnt_n = st[t].cand_cnt[1];
    if (cnt_p > d.n || cnt_n > d.n) failed = true;
    const uint2* __restrict__ cl_p = cand + d.cand_off;
    const uint2* __restrict__ cl_n = cand + d.cand_off + d.n;
    select_side(sh, cl_p, failed ? 0u : cnt_p, st[t].bin[0], d.k - st[t].above[0], 0, tau_p, itau_p, failed);
    select_side(sh, cl_n, failed ? 0u : cnt_n, st[t].bin[1], d.k - st[t].above[1], 1, tau_n, itau_n, failed);

    const double Sp = sh.S[0], Sn = sh.S[1];
    const int side = (Sp >= Sn) ? 0 : 1;              // mu+ >= mu-  <=>  S+ >= S-  (equal counts)
    const float mu32 = (float)((side ? Sn : Sp) / (double)d.k);
    const float mu_signed = side ? -mu32 : mu32;
    if (tid == 0) {
        st[t].tau[0] = tau_p; st[t].tau[1] = tau_n;
        st[t].itau[0] = itau_p; st[t].itau[1] = itau_n;
        st[t].S[0] = Sp; st[t].S[1] = Sn;
        st[t].side = side ? -1 : 1;
        st[t].mu_signed = mu_signed;
        if (failed) atomicOr(&result->err, kErrInternal);
    }
    if (failed) return;

    // binarization and residual update on the chosen side
    const uint2* __restrict__ cl = side ? cl_n : cl_p;
    const uint32_t cnt = side ? cnt_n : cnt_p;
    const uint32_t tau = side ? tau_n : tau_p, itau = side ? itau_n : itau_p;
    uint32_t* __restrict__ bm = bitmap + (uint64_t)d.chunk0 * kChunkWords;
    for (uint32_t i = tid; i < cnt; i += kSelThreads) {
        const uint2 e = cl[i];
        if (cand_kept(e.x, e.y, tau, itau)) {
            if (e.y >= d.n) { atomicOr(&result->err, kErrInternal); continue; }
            const float a = __uint_as_float(bits_of_key(side ? ~e.x : e.x));
            d.R[e.y] = a - mu_signed;
            atomicOr(&bm[e.y >> 5], 1u << (e.y & 31u));
        }
    }
}

// --------------------------------------------------------------------------
// Stage 6 (Alg. 3): Golomb encoding of the gaps between kept positions, from the bitmap.
//   k_chunk_summary : per chunk, count / first / last kept position and the code bits of
//                     every kept entry whose predecessor lies in the same chunk
//   k_tensor_scan   : per tensor, scan over its chunks: predecessor of each chunk's first
//                     kept entry, bit offset of each chunk, total bit length
//   k_pack          : per chunk, writes q ones, a zero and the b-bit remainder of every
//                     kept entry at its bit offset; also the header and table
// --------------------------------------------------------------------------
__device__ __forceinline__ uint32_t golomb_len(uint32_t gap, int b) { return (gap >> b) + 1u + (uint32_t)b; }

__global__ __launch_bounds__(kChunkWords) void k_chunk_summary(const uint32_t* __restrict__ bitmap,
                                                               ChunkSummary* __restrict__ sum, int b) {
    __shared__ uint32_t scratch[kChunkWords / 64];
    __shared__ uint32_t s_cnt, s_first, s_bits;
    const int w = threadIdx.x;
    const uint32_t c = blockIdx.x;
    if (w == 0) { s_cnt = 0u; s_first = 0xFFFFFFFFu; s_bits = 0u; }
    const uint32_t word = bitmap[(uint64_t)c * kChunkWords + w];
    const uint32_t end_w = word ? (uint32_t)(w * 32 + 32 - __clz(word)) : 0u;
    uint32_t last_end;
    uint32_t pe = block_excl_max<uint32_t, kChunkWords>(end_w, &last_end, scratch);  // barriers inside
    if (word) {
        uint32_t m = word, bits = 0u;
        while (m) {
            const uint32_t x = (uint32_t)(w * 32 + __ffs(m) - 1);
            m &= m - 1u;
            if (pe) bits += golomb_len(x - pe, b);
            else s_first = x;                       // the only entry of the chunk without predecessor
            pe = x + 1u;
        }
        atomicAdd(&s_cnt, (uint32_t)__popc(word));
        if (bits) atomicAdd(&s_bits, bits);
    }
    __syncthreads();
    if (w == 0) {
        ChunkSummary s;
        s.cnt = s_cnt; s.first = s_first; s.last_end = last_end; s.inner_bits = s_bits;
        sum[c] = s;
    }
}

__global__ __launch_bounds__(256) void k_tensor_scan(const TensorDesc* __restrict__ desc,
                                                     const ChunkSummary* __restrict__ sum,
                                                     uint32_t* __restrict__ chunk_prev_end,
                                                     uint64_t* __restrict__ chunk_bitoff,
                                                     TensorState* __restrict__ st, int b) {
    __shared__ uint32_t scratch32[4];
    __shared__ unsigned long long scratch64[4];
    const int t = blockIdx.x, tid = threadIdx.x;
    const TensorDesc d = desc[t];
    uint32_t carry_end = 0u;             // position+1 of the last kept entry so far (0: none)
    unsigned long long carry_bits = 0ull;
    uint32_t carry_cnt = 0u;
    for (uint32_t base = 0; base < d.nchunks; base += 256) {
        const uint32_t cc = base + tid;
        ChunkSummary s; s.cnt = 0u; s.first = 0u; s.last_end = 0u; s.inner_bits = 0u;
        if (cc < d.nchunks) s = sum[d.chunk0 + cc];
        const uint32_t gend = s.cnt ? cc * (uint32_t)kChunk + s.last_end : 0u;
        uint32_t tile_end;
        uint32_t pe = block_excl_max<uint32_t, 256>(gend, &tile_end, scratch32);
        if (carry_end > pe) pe = carry_end;
        unsigned long long bits = 0ull;
        if (s.cnt) {
            const uint32_t gap = cc * (uint32_t)kChunk + s.first - pe;
            bits = (unsigned long long)s.inner_bits + (unsigned long long)(gap >> b) + 1ull + (unsigned long long)b;
        }
        unsigned long long tile_bits;
        const unsigned long long off = block_excl_sum<unsigned long long, 256>(bits, &tile_bits, scratch64);
        uint32_t tile_cnt;
        (void)block_excl_sum<uint32_t, 256>(s.cnt, &tile_cnt, scratch32);
        if (cc < d.nchunks) {
            chunk_prev_end[d.chunk0 + cc] = pe;
            chunk_bitoff[d.chunk0 + cc] = carry_bits + off;
        }
        if (tile_end > carry_end) carry_end = tile_end;
        carry_bits += tile_bits;
        carry_cnt += tile_cnt;
    }
    if (tid == 0) { st[t].bit_len = carry_bits; st[t].nnz = carry_cnt; }
}

__device__ __forceinline__ void put_bits(uint32_t* __restrict__ payload, unsigned long long pos,
                                         uint32_t val, int nb) {   // 1 <= nb <= 32, val < 2^nb
    const unsigned long long w = pos >> 5;
    const int off = (int)(pos & 31ull);
    const unsigned long long v = (unsigned long long)val << (64 - off - nb);
    const uint32_t hi = (uint32_t)(v >> 32), lo = (uint32_t)v;
    if (hi) atomicOr(&payload[w], hi);
    if (lo) atomicOr(&payload[w + 1], lo);
}

__device__ __forceinline__ void put_ones(uint32_t* __restrict__ payload, unsigned long long pos,
                                         unsigned long long q) {
    while (q) {
        const unsigned long long w = pos >> 5;
        const uint32_t room = 32u - (uint32_t)(pos & 31ull);
        const uint32_t take = q < room ? (uint32_t)q : room;
        if (take == 32u) payload[w] = 0xFFFFFFFFu;      // whole word belongs to this run
        else atomicOr(&payload[w], ((1u << take) - 1u) << (room - take));
        pos += take;
        q -= take;
    }
}

__global__ __launch_bounds__(kChunkWords) void k_pack(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ chunk_start, int T,
        const uint32_t* __restrict__ bitmap, const ChunkSummary* __restrict__ sum,
        const uint32_t* __restrict__ chunk_prev_end, const uint64_t* __restrict__ chunk_bitoff,
        const TensorState* __restrict__ st, int b, uint8_t* __restrict__ msg,
        uint64_t zero_words, ResultBlock* __restrict__ result) {
    __shared__ uint32_t scratch32[kChunkWords / 64];
    __shared__ unsigned long long scratch64[kChunkWords / 64];
    const int w = threadIdx.x;
    const uint32_t c = blockIdx.x;
    const int t = tensor_of_chunk(chunk_start, T, c);
    const TensorDesc d = desc[t];
    const bool first_chunk = (c == d.chunk0);
    const ChunkSummary s = sum[c];
    if (s.cnt == 0u && !first_chunk) return;           // uniform for the workgroup

    // word offset of this tensor's stream: streams are packed in tensor order
    unsigned long long mine = 0ull, all = 0ull;
    const int upto = (c == 0u) ? T : t;                 // chunk 0 also needs the grand total
    for (int i = w; i < upto; i += kChunkWords) {
        const unsigned long long words = (st[i].bit_len + 31ull) >> 5;
        all += words;
        if (i < t) mine += words;
    }
    unsigned long long tot_mine, tot_all;
    (void)block_excl_sum<unsigned long long, kChunkWords>(mine, &tot_mine, scratch64);
    (void)block_excl_sum<unsigned long long, kChunkWords>(all, &tot_all, scratch64);
    const unsigned long long word_off = tot_mine;
    uint32_t* __restrict__ payload = reinterpret_cast<uint32_t*>(msg + 32 + 24ull * (unsigned)T);

    if (w == 0) {
        if (first_chunk) {
            uint8_t* e = msg + 32 + 24ull * (unsigned)t;
            *reinterpret_cast<float*>(e) = st[t].mu_signed;
            *reinterpret_cast<uint32_t*>(e + 4) = st[t].nnz;
            *reinterpret_cast<uint64_t*>(e + 8) = st[t].bit_len;
            *reinterpret_cast<uint64_t*>(e + 16) = word_off;
            if (st[t].nnz != d.k) atomicOr(&result->err, kErrInternal);
        }
        if (c == 0u) {
            uint32_t* h = reinterpret_cast<uint32_t*>(msg);
            h[0] = 0x31434253u; h[1] = 1u; h[2] = (uint32_t)T; h[3] = (uint32_t)b;
            *reinterpret_cast<uint64_t*>(msg + 16) = tot_all;
            *reinterpret_cast<uint64_t*>(msg + 24) = 0ull;
            result->msg_bytes = 32ull + 24ull * (unsigned)T + 4ull * tot_all;
            if (tot_all > zero_words) atomicOr(&result->err, kErrInternal);
        }
    }
    if (s.cnt == 0u) return;

    const uint32_t word = bitmap[(uint64_t)c * kChunkWords + w];
    const uint32_t end_w = word ? (uint32_t)(w * 32 + 32 - __clz(word)) : 0u;
    uint32_t last_end;
    const uint32_t pe_local = block_excl_max<uint32_t, kChunkWords>(end_w, &last_end, scratch32);
    const uint32_t e0 = (c - d.chunk0) * (uint32_t)kChunk;
    uint32_t pe = pe_local ? e0 + pe_local : chunk_prev_end[c];   // global position+1 of the predecessor
    unsigned long long bits = 0ull;
    {
        uint32_t m = word, p = pe;
        while (m) {
            const uint32_t x = e0 + (uint32_t)(w * 32 + __ffs(m) - 1);
            m &= m - 1u;
            bits += (unsigned long long)((x - p) >> b) + 1ull + (unsigned long long)b;
            p = x + 1u;
        }
    }
    unsigned long long chunk_bits;
    const unsigned long long ex = block_excl_sum<unsigned long long, kChunkWords>(bits, &chunk_bits, scratch64);
    unsigned long long pos = word_off * 32ull + chunk_bitoff[c] + ex;
    if (word && ((pos + bits + 31ull) >> 5) > zero_words) {       // would leave the cleared region
        atomicOr(&result->err, kErrInternal);
        return;
    }
    uint32_t m = word;
    while (m) {
        const uint32_t x = e0 + (uint32_t)(w * 32 + __ffs(m) - 1);
        m &= m - 1u;
        const uint32_t gap = x - pe;
        const uint32_t q = gap >> b;
        put_ones(payload, pos, q);
        pos += q;
        put_bits(payload, pos, gap & ((1u << b) - 1u), b + 1);    // the zero and the remainder
        pos += (unsigned)b + 1u;
        pe = x + 1u;
    }
}

}  // namespace sbc
