// Alg. 3 for tensors whose kept positions are in the bitmap (k or the stream too large for the
// fused path), and the final assembly of the message.
//   k_chunk_summary : per chunk, count / first / last kept position and the code bits of
//                     every kept entry whose predecessor lies in the same chunk
//   k_tile_summary, k_tensor_scan : per tensor, scan over its chunks in tiles of 4096:
//                     predecessor of each chunk's first kept entry, bit offset of each chunk,
//                     total bit length
//   k_pack          : per chunk, writes q ones, a zero and the b-bit remainder of every
//                     kept entry at its bit offset in the tensor's staging words
//                     (SELF: for tensors of few chunks it also does the scan's work for its own
//                     chunk, from the summaries of the chunks before it, and no scan is launched)
// (the message is then assembled by k_finish_message)
#pragma once

#include "sbc_device.hpp"
#include "sbc_select_kernels.hpp"

namespace sbc {

// B: chunks per workgroup.  A workgroup's life is mostly the wait for its loads; with very many
// chunks, B of them share that wait (all loads are issued before the first chunk is worked on).
template <int B>
__global__ __launch_bounds__(kChunkWords) void k_chunk_summary(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ chunk_tensor,
        const uint32_t* __restrict__ bitmap, ChunkSummary* __restrict__ sum, int b, uint32_t n_chunks) {
    __shared__ uint32_t scratch[kChunkWords / 64];
    __shared__ uint32_t s_cnt, s_first, s_bits;
    const int w = threadIdx.x;
    // (the bitmap words are asked for before the descriptors say whether they are needed: one round
    // trip to memory less in a kernel that consists of little else; the words exist for every chunk)
    uint32_t words[B], tensor[B];
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const uint32_t c = blockIdx.x * (uint32_t)B + (uint32_t)j;
        const uint32_t cs = c < n_chunks ? c : n_chunks - 1u;
        words[j] = bitmap[(uint64_t)cs * kChunkWords + w];
        tensor[j] = chunk_tensor[cs];
    }
    uint32_t flags[B];
#pragma unroll
    for (int j = 0; j < B; ++j) flags[j] = desc[tensor[j]].flags;
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const uint32_t c = blockIdx.x * (uint32_t)B + (uint32_t)j;
        if (c >= n_chunks || (flags[j] & kDescFused)) continue;     // uniform for the workgroup
        const uint32_t word = words[j];
        if (w == 0) { s_cnt = 0u; s_first = 0xFFFFFFFFu; s_bits = 0u; }
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
        if (B > 1) __syncthreads();                     // the shared counters start over for the next chunk
    }
}

constexpr int kScanThreads = 1024;
constexpr int kScanPer = 4;              // consecutive chunks per thread
constexpr uint32_t kScanTile = kScanThreads * kScanPer;   // chunks per workgroup of the scan

// What a tile of kScanTile consecutive chunks of a tensor contributes to the scan over all of
// the tensor's chunks.  The code of the tile's first kept entry depends on where the previous
// kept entry lies, which the tile does not know: its bits are left out and its position kept.
struct TileSummary {
    uint32_t cnt;              // kept entries in the tile
    uint32_t end;              // position + 1 of the last one (0: none)
    uint32_t first;            // position of the first one (if cnt != 0)
    uint32_t pad;
    unsigned long long bits;   // code bits of all of them but the first
    unsigned long long pad2;
};

// Tiles of tensor t live at tiles[chunk0 / kScanTile + t ...]: tensors never overlap there
// (floor((a + n) / T) + 1 >= floor(a / T) + ceil(n / T)).
__device__ __forceinline__ uint32_t tile_base(const TensorDesc& d, int t) { return d.chunk0 / kScanTile + (uint32_t)t; }

// One tile's share of the scan, given what precedes the tile: predecessor of each chunk's first
// kept entry, bit offset of each chunk.  WRITE = false only adds up the tile (first pass of a
// tensor of several tiles, carries unknown: pe == 0 marks the tile's first kept entry).
template <bool WRITE>
__device__ __forceinline__ void scan_tile(const TensorDesc& d, uint32_t tile, const ChunkSummary* __restrict__ sum,
                                          uint32_t carry_end, unsigned long long carry_bits, int b,
                                          uint32_t* __restrict__ chunk_prev_end, uint64_t* __restrict__ chunk_bitoff,
                                          uint32_t* scratch32, unsigned long long* scratch64,
                                          uint32_t& tile_end, unsigned long long& tile_bits, uint32_t& tile_cnt,
                                          uint32_t& first_pos, bool& has_first) {
    const int tid = threadIdx.x;
    const uint32_t c0 = tile * kScanTile + (uint32_t)tid * kScanPer;
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
    uint32_t pe = block_excl_max<uint32_t, kScanThreads>(my_end, &tile_end, scratch32);
    if (carry_end > pe) pe = carry_end;
    // predecessor end and code bits of every chunk's first kept entry
    uint32_t pes[kScanPer];
    unsigned long long bits[kScanPer], my_bits = 0ull;
    has_first = false; first_pos = 0u;
#pragma unroll
    for (int j = 0; j < kScanPer; ++j) {
        pes[j] = pe;
        bits[j] = 0ull;
        if (s[j].cnt) {
            const uint32_t pos = (c0 + j) * (uint32_t)kChunk + s[j].first;
            bits[j] = (unsigned long long)s[j].inner_bits;
            if (!WRITE && pe == 0u) { has_first = true; first_pos = pos; }      // (a kept entry's end is at least 1)
            else bits[j] += (unsigned long long)((pos - pe) >> b) + 1ull + (unsigned long long)b;
            pe = gend[j];
        }
        my_bits += bits[j];
    }
    unsigned long long off = carry_bits + block_excl_sum<unsigned long long, kScanThreads>(my_bits, &tile_bits, scratch64);
    (void)block_excl_sum<uint32_t, kScanThreads>(my_cnt, &tile_cnt, scratch32);
    if (WRITE) {
#pragma unroll
        for (int j = 0; j < kScanPer; ++j) {
            if (c0 + j < d.nchunks) {
                chunk_prev_end[d.chunk0 + c0 + j] = pes[j];
                chunk_bitoff[d.chunk0 + c0 + j] = off;
            }
            off += bits[j];
        }
    }
}

// grid (T, tiles): first pass over a tensor of several tiles (tensors of one tile need none)
__global__ __launch_bounds__(kScanThreads) void k_tile_summary(const TensorDesc* __restrict__ desc,
                                                               const ChunkSummary* __restrict__ sum,
                                                               TileSummary* __restrict__ tiles, int b) {
    __shared__ uint32_t scratch32[kScanThreads / 64];
    __shared__ unsigned long long scratch64[kScanThreads / 64];
    const int t = blockIdx.x, tid = threadIdx.x;
    const TensorDesc d = desc[t];
    if (d.flags & kDescFused) return;
    const uint32_t n_tiles = (d.nchunks + kScanTile - 1u) / kScanTile;
    if (n_tiles < 2u || blockIdx.y >= n_tiles) return;
    uint32_t tile_end, tile_cnt, first_pos;
    unsigned long long tile_bits;
    bool has_first;
    scan_tile<false>(d, blockIdx.y, sum, 0u, 0ull, b, nullptr, nullptr, scratch32, scratch64, tile_end, tile_bits, tile_cnt,
                     first_pos, has_first);
    TileSummary* const out = tiles + tile_base(d, t) + blockIdx.y;
    if (has_first) out->first = first_pos;              // exactly one thread of a tile that holds entries
    if (tid == 0) { out->cnt = tile_cnt; out->end = tile_end; out->bits = tile_bits; }
}

// grid (T, tiles): per tensor, scan over its chunks: every tile folds the summaries of the
// tiles before it, then scans its own chunks.
__global__ __launch_bounds__(kScanThreads) void k_tensor_scan(const TensorDesc* __restrict__ desc,
                                                              const ChunkSummary* __restrict__ sum,
                                                              const TileSummary* __restrict__ tiles,
                                                              uint32_t* __restrict__ chunk_prev_end,
                                                              uint64_t* __restrict__ chunk_bitoff,
                                                              TensorState* __restrict__ st, int b) {
    __shared__ uint32_t scratch32[kScanThreads / 64];
    __shared__ unsigned long long scratch64[kScanThreads / 64];
    const int t = blockIdx.x, tid = threadIdx.x;
    const TensorDesc d = desc[t];
    if (d.flags & kDescFused) return;
    const uint32_t n_tiles = (d.nchunks + kScanTile - 1u) / kScanTile;
    if (blockIdx.y >= n_tiles) return;
    uint32_t carry_end = 0u, carry_cnt = 0u;            // position+1 of the last kept entry so far (0: none)
    unsigned long long carry_bits = 0ull;
    const TileSummary* __restrict__ ts = tiles + tile_base(d, t);
    for (uint32_t j = 0; j < blockIdx.y; ++j) {         // (every thread: the same few loads)
        const TileSummary s = ts[j];
        if (s.cnt) {
            carry_bits += s.bits + (unsigned long long)((s.first - carry_end) >> b) + 1ull + (unsigned long long)b;
            carry_end = s.end;                           // positions grow from tile to tile
            carry_cnt += s.cnt;
        }
    }
    uint32_t tile_end, tile_cnt, first_pos;
    unsigned long long tile_bits;
    bool has_first;
    scan_tile<true>(d, blockIdx.y, sum, carry_end, carry_bits, b, chunk_prev_end, chunk_bitoff, scratch32, scratch64,
                    tile_end, tile_bits, tile_cnt, first_pos, has_first);
    if (tid == 0 && blockIdx.y == n_tiles - 1u) { st[t].bit_len = carry_bits + tile_bits; st[t].nnz = carry_cnt + tile_cnt; }
}

// Most chunks a tensor may have for the workgroups of k_pack to do the scan's work themselves
// (each reads the summaries of all chunks before its own: two per thread).
constexpr uint32_t kSelfScanChunks = 2 * kChunkWords;

// What precedes chunk cc of a tensor, from the summaries of its chunks 0 .. cc-1: position + 1 of
// the last kept entry before the chunk (0: none), the code bits and the kept entries before it.
// Contains barriers; every thread of the workgroup must call it.
__device__ __forceinline__ void scan_before_chunk(const TensorDesc& d, uint32_t cc, const ChunkSummary* __restrict__ sum,
                                                  int b, uint32_t* scratch32, unsigned long long* scratch64,
                                                  uint32_t& prev_end, unsigned long long& bit_off, uint32_t& cnt_before) {
    const int w = threadIdx.x;
    ChunkSummary s[2];
    uint32_t gend[2], my_end = 0u, my_cnt = 0u;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint32_t i = (uint32_t)w * 2u + (uint32_t)j;
        s[j].cnt = 0u; s[j].first = 0u; s[j].last_end = 0u; s[j].inner_bits = 0u;
        if (i < cc) s[j] = sum[d.chunk0 + i];
        gend[j] = s[j].cnt ? i * (uint32_t)kChunk + s[j].last_end : 0u;
        if (gend[j] > my_end) my_end = gend[j];
        my_cnt += s[j].cnt;
    }
    uint32_t pe = block_excl_max<uint32_t, kChunkWords>(my_end, &prev_end, scratch32);
    unsigned long long my_bits = 0ull;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        if (s[j].cnt) {
            const uint32_t pos = ((uint32_t)w * 2u + (uint32_t)j) * (uint32_t)kChunk + s[j].first;
            my_bits += (unsigned long long)s[j].inner_bits + (unsigned long long)golomb_len(pos - pe, b);
            pe = gend[j];
        }
    }
    (void)block_excl_sum<unsigned long long, kChunkWords>(my_bits, &bit_off, scratch64);
    (void)block_excl_sum<uint32_t, kChunkWords>(my_cnt, &cnt_before, scratch32);
}

template <int B, bool SELF>
__global__ __launch_bounds__(kChunkWords) void k_pack(
        const TensorDesc* __restrict__ desc, const uint32_t* __restrict__ chunk_tensor,
        const uint32_t* __restrict__ bitmap, const ChunkSummary* __restrict__ sum,
        const uint32_t* __restrict__ chunk_prev_end, const uint64_t* __restrict__ chunk_bitoff,
        TensorState* __restrict__ st, int b, uint32_t* __restrict__ stage, ResultBlock* __restrict__ result,
        uint32_t n_chunks) {
    static_assert(!SELF || B == 1, "a workgroup that scans for itself takes one chunk");
    __shared__ uint32_t scratch32[kChunkWords / 64];
    __shared__ unsigned long long scratch64[kChunkWords / 64];
    const int w = threadIdx.x;
    // (everything the chunks may need is asked for at once, before the descriptors say whether it is
    // needed: the arrays hold an element for every chunk)
    uint32_t words[B], tensor[B], chunk_cnt[B], prev_end[B];
    unsigned long long bit_off[B];
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const uint32_t c = blockIdx.x * (uint32_t)B + (uint32_t)j;
        const uint32_t cs = c < n_chunks ? c : n_chunks - 1u;
        tensor[j] = chunk_tensor[cs];
        words[j] = bitmap[(uint64_t)cs * kChunkWords + w];
        chunk_cnt[j] = sum[cs].cnt;
        prev_end[j] = SELF ? 0u : chunk_prev_end[cs];
        bit_off[j] = SELF ? 0ull : chunk_bitoff[cs];
    }
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const uint32_t c = blockIdx.x * (uint32_t)B + (uint32_t)j;
        if (c >= n_chunks) continue;
        const TensorDesc d = desc[tensor[j]];           // (consecutive chunks mostly share it)
        if (d.flags & kDescFused) continue;             // uniform for the workgroup
        const bool last_chunk = SELF && c - d.chunk0 == d.nchunks - 1u;
        uint32_t cnt_before = 0u;
        if (SELF) {
            if (chunk_cnt[j] == 0u && !last_chunk) continue;
            scan_before_chunk(d, c - d.chunk0, sum, b, scratch32, scratch64, prev_end[j], bit_off[j], cnt_before);
        }
        if (chunk_cnt[j] == 0u) {
            if (last_chunk && w == 0) { st[tensor[j]].bit_len = bit_off[j]; st[tensor[j]].nnz = cnt_before; }
            continue;
        }
        const uint32_t word = words[j];
        const uint32_t end_w = word ? (uint32_t)(w * 32 + 32 - __clz(word)) : 0u;
        uint32_t last_end;
        const uint32_t pe_local = block_excl_max<uint32_t, kChunkWords>(end_w, &last_end, scratch32);
        const uint32_t e0 = (c - d.chunk0) * (uint32_t)kChunk;
        uint32_t pe = pe_local ? e0 + pe_local : prev_end[j];         // global position+1 of the predecessor
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
        if (last_chunk && w == 0) { st[tensor[j]].bit_len = bit_off[j] + chunk_bits; st[tensor[j]].nnz = cnt_before + chunk_cnt[j]; }
        unsigned long long pos = bit_off[j] + ex;
        if (word && ((pos + bits + 31ull) >> 5) > d.bound_words) {    // would leave the tensor's staging words
            atomicOr(&result->err, kErrInternal);
            continue;
        }
        uint32_t* __restrict__ out = stage + d.stage_off;
        uint32_t m = word;
        while (m) {
            const uint32_t x = e0 + (uint32_t)(w * 32 + __ffs(m) - 1);
            m &= m - 1u;
            const uint32_t gap = x - pe;
            const uint32_t q = gap >> b;
            put_ones(out, pos, q);
            pos += q;
            put_bits(out, pos, gap & ((1u << b) - 1u), b + 1);        // the zero and the remainder
            pos += (unsigned)b + 1u;
            pe = x + 1u;
        }
    }
}

}  // namespace sbc
