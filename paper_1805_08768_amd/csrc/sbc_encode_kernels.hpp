// Alg. 3 for tensors whose kept positions are in the bitmap (k or the stream too large for the
// fused path), and the final assembly of the message.
//   k_chunk_summary : per chunk, count / first / last kept position and the code bits of
//                     every kept entry whose predecessor lies in the same chunk
//   k_tensor_scan   : per tensor, scan over its chunks: predecessor of each chunk's first
//                     kept entry, bit offset of each chunk, total bit length
//   k_pack          : per chunk, writes q ones, a zero and the b-bit remainder of every
//                     kept entry at its bit offset in the tensor's staging words
//   k_gather        : copies every tensor's stream from staging to its place in the payload
//                     (streams in tensor order, each starting on a word boundary) and writes
//                     the header and the table
#pragma once

#include "sbc_device.hpp"
#include "sbc_select_kernels.hpp"

namespace sbc {

__global__ __launch_bounds__(kChunkWords) void k_chunk_summary(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ chunk_tensor,
        const uint32_t* __restrict__ bitmap, ChunkSummary* __restrict__ sum, int b) {
    __shared__ uint32_t scratch[kChunkWords / 64];
    __shared__ uint32_t s_cnt, s_first, s_bits;
    const int w = threadIdx.x;
    const uint32_t c = blockIdx.x;
    if (desc[chunk_tensor[c]].flags & kDescFused) return;
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

constexpr int kScanThreads = 1024;
constexpr int kScanPer = 4;              // consecutive chunks per thread and round

__global__ __launch_bounds__(kScanThreads) void k_tensor_scan(const TensorDesc* __restrict__ desc,
                                                              const ChunkSummary* __restrict__ sum,
                                                              uint32_t* __restrict__ chunk_prev_end,
                                                              uint64_t* __restrict__ chunk_bitoff,
                                                              TensorState* __restrict__ st, int b) {
    __shared__ uint32_t scratch32[kScanThreads / 64];
    __shared__ unsigned long long scratch64[kScanThreads / 64];
    const int t = blockIdx.x, tid = threadIdx.x;
    const TensorDesc d = desc[t];
    if (d.flags & kDescFused) return;
    uint32_t carry_end = 0u;             // position+1 of the last kept entry so far (0: none)
    unsigned long long carry_bits = 0ull;
    uint32_t carry_cnt = 0u;
    for (uint32_t base = 0; base < d.nchunks; base += kScanThreads * kScanPer) {
        const uint32_t c0 = base + (uint32_t)tid * kScanPer;
        ChunkSummary s[kScanPer];
        uint32_t gend[kScanPer], my_end = 0u, my_cnt = 0u;
#pragma unroll
        for (int j = 0; j < kScanPer; ++j) {
            s[j].cnt = 0u; s[j].first = 0u; s[j].last_end = 0u; s[j].inner_bits = 0u;
            if (c0 + j < d.nchunks) s[j] = sum[d.chunk0 + c0 + j];
            gend[j] = s[j].cnt ? (c0 + j) * (uint32_t)kChunk + s[j].last_end : 0u;
            if (gend[j] > my_end) my_end = gend[j];
            my_cnt += s[j].cnt;
        }
        uint32_t tile_end;
        uint32_t pe = block_excl_max<uint32_t, kScanThreads>(my_end, &tile_end, scratch32);
        if (carry_end > pe) pe = carry_end;
        // predecessor end and code bits of every chunk's first kept entry
        uint32_t pes[kScanPer];
        unsigned long long bits[kScanPer], my_bits = 0ull;
#pragma unroll
        for (int j = 0; j < kScanPer; ++j) {
            pes[j] = pe;
            bits[j] = 0ull;
            if (s[j].cnt) {
                const uint32_t gap = (c0 + j) * (uint32_t)kChunk + s[j].first - pe;
                bits[j] = (unsigned long long)s[j].inner_bits + (unsigned long long)(gap >> b) + 1ull + (unsigned long long)b;
                pe = gend[j];
            }
            my_bits += bits[j];
        }
        unsigned long long tile_bits;
        unsigned long long off = carry_bits + block_excl_sum<unsigned long long, kScanThreads>(my_bits, &tile_bits, scratch64);
        uint32_t tile_cnt;
        (void)block_excl_sum<uint32_t, kScanThreads>(my_cnt, &tile_cnt, scratch32);
#pragma unroll
        for (int j = 0; j < kScanPer; ++j) {
            if (c0 + j < d.nchunks) {
                chunk_prev_end[d.chunk0 + c0 + j] = pes[j];
                chunk_bitoff[d.chunk0 + c0 + j] = off;
            }
            off += bits[j];
        }
        if (tile_end > carry_end) carry_end = tile_end;
        carry_bits += tile_bits;
        carry_cnt += tile_cnt;
    }
    if (tid == 0) { st[t].bit_len = carry_bits; st[t].nnz = carry_cnt; }
}

__global__ __launch_bounds__(kChunkWords) void k_pack(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ chunk_tensor,
        const uint32_t* __restrict__ bitmap, const ChunkSummary* __restrict__ sum,
        const uint32_t* __restrict__ chunk_prev_end, const uint64_t* __restrict__ chunk_bitoff,
        int b, uint32_t* __restrict__ stage, ResultBlock* __restrict__ result) {
    __shared__ uint32_t scratch32[kChunkWords / 64];
    __shared__ unsigned long long scratch64[kChunkWords / 64];
    const int w = threadIdx.x;
    const uint32_t c = blockIdx.x;
    const int t = (int)chunk_tensor[c];
    const TensorDesc d = desc[t];
    if (d.flags & kDescFused) return;
    if (sum[c].cnt == 0u) return;                       // uniform for the workgroup

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
    unsigned long long pos = chunk_bitoff[c] + ex;
    if (word && ((pos + bits + 31ull) >> 5) > d.bound_words) {    // would leave the tensor's staging words
        atomicOr(&result->err, kErrInternal);
        return;
    }
    uint32_t* __restrict__ words = stage + d.stage_off;
    uint32_t m = word;
    while (m) {
        const uint32_t x = e0 + (uint32_t)(w * 32 + __ffs(m) - 1);
        m &= m - 1u;
        const uint32_t gap = x - pe;
        const uint32_t q = gap >> b;
        put_ones(words, pos, q);
        pos += q;
        put_bits(words, pos, gap & ((1u << b) - 1u), b + 1);      // the zero and the remainder
        pos += (unsigned)b + 1u;
        pe = x + 1u;
    }
}

// grid (T, P): workgroup (t, y) copies every P-th 256-word slice of tensor t's stream.  The
// lead workgroup of a tensor also leaves the tensor's candidate counters and flags clean for the
// next call (which may skip the sampling kernel that otherwise resets them).
__global__ __launch_bounds__(256) void k_gather(const TensorDesc* __restrict__ desc,
                                                TensorState* __restrict__ st, int T, int b,
                                                const uint32_t* __restrict__ stage, uint8_t* __restrict__ msg,
                                                uint64_t msg_capacity, ResultBlock* __restrict__ result,
                                                ResultBlock* __restrict__ next_result) {
    __shared__ unsigned long long part[2][4];
    const int t = blockIdx.x, tid = threadIdx.x;
    const bool lead = (blockIdx.y == 0);
    // (loaded up front: nothing below depends on the sums until the offsets are needed)
    const TensorDesc d = desc[t];
    const uint32_t my_flags = st[t].flags;
    const unsigned long long bit_len = st[t].bit_len;
    // word offset of this tensor's stream: streams are packed in tensor order
    unsigned long long mine = 0ull, all = 0ull;
    const int upto = (t == 0 && lead) ? T : t;          // workgroup (0, 0) also needs the grand total
    for (int i = tid; i < upto; i += 256) {
        const unsigned long long words = (st[i].bit_len + 31ull) >> 5;
        all += words;
        if (i < t) mine += words;
    }
    // both sums in one reduction
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        mine += __shfl_down(mine, off, 64);
        all += __shfl_down(all, off, 64);
    }
    if ((tid & 63) == 0) { part[0][tid >> 6] = mine; part[1][tid >> 6] = all; }
    __syncthreads();
    const unsigned long long word_off = part[0][0] + part[0][1] + part[0][2] + part[0][3];
    const unsigned long long tot_all = part[1][0] + part[1][1] + part[1][2] + part[1][3];
    if (my_flags & kStFailed) return;                 // this tensor is redone by the histogram path
    const unsigned long long n_words = (bit_len + 31ull) >> 5;
    const unsigned long long table_end = 32ull + 24ull * (unsigned)T;
    if (n_words > d.bound_words || table_end + 4ull * (word_off + n_words) > msg_capacity) {
        if (tid == 0) atomicOr(&result->err, kErrInternal);
        return;
    }
    if (tid == 0 && lead) {
        uint8_t* e = msg + 32 + 24ull * (unsigned)t;
        *reinterpret_cast<float*>(e) = st[t].mu_signed;
        *reinterpret_cast<uint32_t*>(e + 4) = st[t].nnz;
        *reinterpret_cast<uint64_t*>(e + 8) = bit_len;
        *reinterpret_cast<uint64_t*>(e + 16) = word_off;
        if (st[t].nnz != st[t].kc[st[t].side < 0 ? 1 : 0] || st[t].nnz > d.kcap) atomicOr(&result->err, kErrInternal);
        st[t].cand_cnt[0] = 0u; st[t].cand_cnt[1] = 0u; st[t].flags = 0u;
        if (t == 0) {
            uint32_t* h = reinterpret_cast<uint32_t*>(msg);
            h[0] = 0x31434253u; h[1] = 1u; h[2] = (uint32_t)T; h[3] = (uint32_t)b;
            *reinterpret_cast<uint64_t*>(msg + 16) = tot_all;
            *reinterpret_cast<uint64_t*>(msg + 24) = 0ull;
            result->msg_bytes = table_end + 4ull * tot_all;
            // the result block of the next call starts out clean
            next_result->err = 0u; next_result->pad = 0u; next_result->msg_bytes = 0ull;
        }
    }
    const uint32_t* __restrict__ src = stage + d.stage_off;
    uint32_t* __restrict__ dst = reinterpret_cast<uint32_t*>(msg + table_end) + word_off;
    for (unsigned long long w = (unsigned long long)blockIdx.y * 256ull + tid; w < n_words;
         w += 256ull * gridDim.y)
        dst[w] = src[w];
}


}  // namespace sbc
