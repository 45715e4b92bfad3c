// Server step: parallel Golomb position decoding (the supplement's Alg. 4) fused with the
// scaled accumulation of Alg. 1's averaging line.
//
// Alg. 4 is a bit-serial state machine.  At a bit boundary its state is either "reading
// the unary part" (state 0) or "j remainder bits still to read" (state j, 1 <= j <= b).
// One workgroup per tensor stream cuts the stream into 64-bit segments, one per thread and
// tile.  For every segment and every one of the b+1 entry states it computes the exit
// state; an inclusive scan under function composition over the segments of a tile gives
// each segment its true entry state.  A position is then a linear function of what
// precedes its terminating zero:
//     position_i = 2^b * (#unary ones before the zero) + (sum of remainders up to code i) + i
// so three prefix sums over segments (unary ones, zeros that end a unary part, remainders)
// place every code without any sequential dependence.
#pragma once

#include "sbc_device.hpp"

namespace sbc {

constexpr int kDecThreads = 512;
constexpr int kMaxB = 30;
constexpr int kStates = kMaxB + 1;
constexpr int kPackedMaxB = 15;               // up to 16 states fit one 64-bit word of 4-bit fields

struct DecDesc {
    float* out;
    uint32_t n;
    uint32_t wide;        // 1: decoded by the tile kernels below, not by k_decode_accumulate
};

constexpr int kTileWords = 2 * kDecThreads;   // stream words covered by one tile of segments
constexpr int kTileSlack = 2;                 // a remainder may reach this many words past the tile

// b bits (MSB first, 0 <= b <= 30) starting at bit `pos` of the tile staged in LDS.
__device__ __forceinline__ uint32_t read_bits(const uint32_t* tile, uint32_t pos, int b) {
    if (b == 0) return 0u;
    const uint32_t w = pos >> 5;
    const int off = (int)(pos & 31u);
    const unsigned long long v = ((unsigned long long)tile[w] << 32) | tile[w + 1];
    return (uint32_t)((v >> (64 - off - b)) & ((1ull << b) - 1ull));
}

// First zero bit of `w` (bit 0 = most significant) at or after offset x (< 64); 64 if none.
__device__ __forceinline__ int first_zero_from(unsigned long long w, int x) {
    const unsigned long long zz = (~w) & (~0ull >> x);
    return zz ? __clzll((long long)zz) : 64;
}

// State in which Alg. 4 leaves a 64-bit segment that it enters in state s (the first s bits
// finish a remainder).
__device__ __forceinline__ int exit_state_of(unsigned long long w64, int s, int b) {
    int x = s;
    while (true) {
        if (x >= 64) return x - 64;
        const int z = first_zero_from(w64, x);
        if (z == 64) return 0;
        x = z + b + 1;
    }
}

// Exit states of a 64-bit segment for all entry states 0..b at once (b <= 15), as 4-bit fields:
// field s holds exit_state_of(w64, s, b).  With g(x) the exit state when Alg. 4 is in its unary
// state at bit x (bit 0 = most significant): g(x) = x - 64 for 64 <= x <= 64 + b, and for x < 64
// g(x) = g(x + 1) if bit x is a one (one more unary bit), g(x + b + 1) if it is a zero (the code
// ends b bits later).  The last b + 1 values are kept as the fields of one word while x runs from
// 63 down to 0: 64 steps without a branch, where walking every entry state separately takes up to
// b + 1 walks of several steps each.
__device__ __forceinline__ unsigned long long packed_exits(unsigned long long w64, int b) {
    unsigned long long g = 0xFEDCBA9876543210ull;           // field j = g(64 + j) = j
    const int top = 4 * b;
#pragma unroll
    for (int i = 0; i < 64; ++i) {                          // x = 63 - i
        const unsigned long long one = g & 15ull;           // g(x + 1)
        const unsigned long long zero = (g >> top) & 15ull; // g(x + b + 1)
        g = (g << 4) | (((w64 >> i) & 1ull) ? one : zero);
    }
    return b == 15 ? g : (g & ((1ull << (4 * (b + 1))) - 1ull));
}

// Transition functions over at most 16 states as 4-bit fields of one word: field s holds f(s).
__device__ __forceinline__ int apply_packed(unsigned long long f, int s) { return (int)((f >> (4 * s)) & 15ull); }
// later o earlier
__device__ __forceinline__ unsigned long long compose_packed(unsigned long long later, unsigned long long earlier, int S) {
    unsigned long long r = 0ull;
    for (int s = 0; s < S; ++s) r |= ((later >> (4 * apply_packed(earlier, s))) & 15ull) << (4 * s);
    return r;
}

__global__ __launch_bounds__(kDecThreads) void k_decode_accumulate(
        const uint8_t* __restrict__ msg, unsigned long long msg_bytes,
        const DecDesc* __restrict__ dd, const uint2* __restrict__ blocks, int T, int b, float scale,
        ResultBlock* __restrict__ result, ResultBlock* __restrict__ next_result) {
    __shared__ uint8_t fn[2][kStates][kDecThreads];       // transition functions, [state][segment] (b > kPackedMaxB)
    __shared__ unsigned long long wave_fn[kDecThreads / 64];
    __shared__ unsigned long long scratch64[kDecThreads / 64];
    __shared__ uint32_t s_state;
    __shared__ uint32_t tile[kTileWords + kTileSlack];   // words past the stream read as ones

    const int tid = threadIdx.x;
    // Workgroup -> (stream, share): every workgroup of a stream decodes all of it, and applies the
    // updates of the threads whose number is congruent to its share.
    const uint2 bk = blocks[blockIdx.x];
    const int t = (int)bk.x;
    const uint32_t share = bk.y & 0xFFFFu, shares = bk.y >> 16;
    const bool mine = ((uint32_t)tid % shares) == share;
    SBC_TS(2, 0);
    if (blockIdx.x == 0 && tid == 0) { next_result->err = 0u; next_result->pad = 0u; next_result->msg_bytes = 0ull; }
    if (dd[t].wide) return;

    // ---- header and table entry (validated by every workgroup; all threads agree).  The host has
    // checked that the message holds the header and T table entries, so all loads go out together.
    const uint32_t* h = reinterpret_cast<const uint32_t*>(msg);
    const unsigned long long table_end = 32ull + 24ull * (unsigned)T;
    const uint8_t* e = msg + 32 + 24ull * (unsigned)t;
    const uint32_t h0 = h[0], h1 = h[1], h2 = h[2], h3 = h[3];
    const unsigned long long payload_words = *reinterpret_cast<const unsigned long long*>(msg + 16);
    const float mu = *reinterpret_cast<const float*>(e);
    const uint32_t nnz = *reinterpret_cast<const uint32_t*>(e + 4);
    const unsigned long long bit_len = *reinterpret_cast<const unsigned long long*>(e + 8);
    const unsigned long long word_off = *reinterpret_cast<const unsigned long long*>(e + 16);
    const uint32_t n = dd[t].n;
    const gfloat_ptr out = as_global(dd[t].out);
    bool ok = msg_bytes >= table_end && h0 == 0x31434253u && h1 == 1u && h2 == (uint32_t)T && h3 == (uint32_t)b;
    if (ok) {
        const unsigned long long max_words = (msg_bytes - table_end) >> 2;
        const unsigned long long n_words_t = (bit_len + 31ull) >> 5;
        ok = payload_words <= max_words && bit_len <= (max_words << 5) &&
             word_off <= payload_words && n_words_t <= payload_words - word_off &&
             nnz <= n && (unsigned long long)nnz * (unsigned)(b + 1) <= bit_len &&
             (nnz != 0u || bit_len == 0ull);
    }
    if (!ok) {
        if (tid == 0) atomicOr(&result->err, kErrCorrupt);
        return;
    }
    if (nnz == 0u) return;
    SBC_TS(2, 1);                                     // header read
    SBC_TS_VAL(2, 15, nnz);

    const float addend = scale * mu;
    const uint32_t* __restrict__ words =
        reinterpret_cast<const uint32_t*>(msg + table_end) + word_off;
    const unsigned long long n_words = (bit_len + 31ull) >> 5;
    const unsigned long long n_seg = (bit_len + 63ull) >> 6;
    const int S = b + 1;                                  // number of states
    const bool packed = b <= kPackedMaxB;
    const int lane = tid & 63, wave = tid >> 6;

    int carry_state = 0;
    unsigned long long carry_U = 0ull;   // unary ones so far
    unsigned long long carry_T = 0ull;   // codes so far
    unsigned long long carry_R = 0ull;   // sum of remainders so far
    bool bad = false;

    for (unsigned long long seg0 = 0; seg0 < n_seg; seg0 += kDecThreads) {
        const unsigned long long seg = seg0 + tid;
        // stage the tile's words in LDS; bits at or past bit_len read as ones (never a terminator)
        __syncthreads();
        for (int i = tid; i < kTileWords + kTileSlack; i += kDecThreads) {
            const unsigned long long w = 2ull * seg0 + (unsigned)i;
            uint32_t v = 0xFFFFFFFFu;
            if (w < n_words) {
                v = words[w];
                const unsigned long long valid = bit_len - 32ull * w;
                if (valid < 32ull) v |= (0xFFFFFFFFu >> valid);
            }
            tile[i] = v;
        }
        __syncthreads();
        const unsigned long long w64 = ((unsigned long long)tile[2 * tid] << 32) | tile[2 * tid + 1];
        SBC_TS(2, 2);                                 // tile staged

        int entry;
        if (packed) {
            // ---- exit state per entry state in one word; scan under composition with shuffles
            // inside a wavefront, then the state is walked through the wavefronts' totals ----
            unsigned long long f = packed_exits(w64, b);
            SBC_TS(2, 3);                             // exit states
#pragma unroll
            for (int dlt = 1; dlt < 64; dlt <<= 1) {
                const unsigned long long o = __shfl_up(f, dlt, 64);
                if (lane >= dlt) f = compose_packed(f, o, S);
            }
            if (lane == 63) wave_fn[wave] = f;
            const unsigned long long before = __shfl_up(f, 1, 64);   // lanes 0..lane-1 of this wavefront
            __syncthreads();
            int st = carry_state, st_mine = carry_state;
#pragma unroll
            for (int w = 0; w < kDecThreads / 64; ++w) {
                if (w == wave) st_mine = st;
                st = apply_packed(wave_fn[w], st);
            }
            entry = lane == 0 ? st_mine : apply_packed(before, st_mine);
            carry_state = st;                              // the same in every thread
        } else {
            // ---- exit state for every entry state, one byte each ----
            int ex = exit_state_of(w64, 0, b);
            fn[0][0][tid] = (uint8_t)ex;
            for (int s = 1; s < S; ++s) {
                if (!((w64 >> (64 - s)) & 1ull)) ex = exit_state_of(w64, s, b);
                fn[0][s][tid] = (uint8_t)ex;
            }
            __syncthreads();
            // ---- inclusive scan under composition: fn[cur][.][i] = f_i o ... o f_0 ----
            int cur = 0;
            for (int dlt = 1; dlt < kDecThreads; dlt <<= 1) {
                for (int s = 0; s < S; ++s) {
                    uint8_t v;
                    if (tid >= dlt) v = fn[cur][fn[cur][s][tid - dlt]][tid];
                    else v = fn[cur][s][tid];
                    fn[cur ^ 1][s][tid] = v;
                }
                __syncthreads();
                cur ^= 1;
            }
            entry = (tid == 0) ? carry_state : (int)fn[cur][carry_state][tid - 1];
            if (tid == kDecThreads - 1) s_state = fn[cur][carry_state][tid];
            __syncthreads();
            carry_state = (int)s_state;
        }

        SBC_TS(2, 4);                                 // entry states known
        // ---- first walk: unary ones, terminators and remainder sum of this segment.  For the first
        // eight codes the running counts are kept, so that their positions follow from the scan
        // below by arithmetic alone and all their loads go out together ----
        uint32_t nU = 0u, nT = 0u;
        unsigned long long sR = 0ull;
        uint32_t lu[8], lr[8];                        // unary ones / remainder sum up to and including code i
        unsigned long long last_end = 0ull;           // bit after the segment's last code
        int x = entry;
        bool open = seg < n_seg;
        auto walk_code = [&](int& xx) -> bool {       // one step of Alg. 4's outer loop; false: no code ended
            const int z = first_zero_from(w64, xx);
            nU += (uint32_t)(z - xx);
            if (z == 64) { xx = 64; return false; }
            const unsigned long long zpos = seg * 64ull + (unsigned)z;
            if (zpos + 1ull + (unsigned)b > bit_len) { bad = true; open = false; return false; }
            sR += read_bits(tile, (uint32_t)(tid * 64 + z + 1), b);
            ++nT;
            last_end = zpos + 1ull + (unsigned)b;
            xx = z + b + 1;
            return true;
        };
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            lu[i] = 0u; lr[i] = 0u;
            if (open && x < 64 && walk_code(x)) { lu[i] = nU; lr[i] = (uint32_t)sR; }
        }
        // where the second walk resumes in a segment with more than eight codes (b < 7 only)
        const int x8 = x;
        const uint32_t nU8 = nU, nT8 = nT;
        const unsigned long long sR8 = sR;
        while (open && x < 64) (void)walk_code(x);
        SBC_TS(2, 5);                                 // first walk
        unsigned long long exU, exT, exR, tile_U, tile_T, tile_R;
        if (packed) {
            // a tile holds at most 2^15 ones and codes, and remainders below 2^32 in total
            unsigned long long tot;
            const unsigned long long ex = block_excl_sum<unsigned long long, kDecThreads>(
                (unsigned long long)nU | ((unsigned long long)nT << 16) | (sR << 32), &tot, scratch64);
            exU = ex & 0xFFFFull; exT = (ex >> 16) & 0xFFFFull; exR = ex >> 32;
            tile_U = tot & 0xFFFFull; tile_T = (tot >> 16) & 0xFFFFull; tile_R = tot >> 32;
        } else {
            exU = block_excl_sum<unsigned long long, kDecThreads>(nU, &tile_U, scratch64);
            exT = block_excl_sum<unsigned long long, kDecThreads>(nT, &tile_T, scratch64);
            exR = block_excl_sum<unsigned long long, kDecThreads>(sR, &tile_R, scratch64);
        }

        SBC_TS(2, 6);                                 // offsets known
        // ---- place every code whose terminating zero lies in this segment:
        //      position = 2^b * (unary ones before its zero) + (remainders up to it) + (codes before it) ----
        if (seg < n_seg && !bad) {
            const unsigned long long U0 = carry_U + exU, T0 = carry_T + exT, R0 = carry_R + exR;
            // the stream's last code ends the stream exactly
            if (nT > 0u && T0 + nT == (unsigned long long)nnz && last_end != bit_len) bad = true;
            const uint32_t m = nT < 8u ? nT : 8u;
            uint32_t pend[8];                         // positions are distinct: update them eight at a time
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const unsigned long long pos = ((U0 + lu[i]) << b) + R0 + lr[i] + T0 + (unsigned)i;
                if ((uint32_t)i < m && (pos >= n || T0 + (unsigned)i >= nnz)) bad = true;
                pend[i] = (uint32_t)pos;
            }
            if (!bad && mine) {
                float v[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = (uint32_t)i < m ? out[pend[i]] : 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) if ((uint32_t)i < m) out[pend[i]] = v[i] + addend;
            }
            SBC_TS(2, 8);
            if (nT > 8u && !bad && mine) {
                // the remaining codes of a segment with more than eight: walked again from the ninth
                unsigned long long U = U0 + nU8, Tn = T0 + nT8, R = R0 + sR8;
                int xx = x8;
                int np = 0;
                while (xx < 64) {
                    const int z = first_zero_from(w64, xx);
                    U += (unsigned)(z - xx);
                    if (z == 64) break;
                    R += read_bits(tile, (uint32_t)(tid * 64 + z + 1), b);
                    const unsigned long long pos = (U << b) + R + Tn;
                    if (pos >= n || Tn >= nnz) { bad = true; break; }
                    pend[np++] = (uint32_t)pos;
                    if (np == 8) {
                        float v[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) v[i] = out[pend[i]];
#pragma unroll
                        for (int i = 0; i < 8; ++i) out[pend[i]] = v[i] + addend;
                        np = 0;
                    }
                    ++Tn;
                    xx = z + b + 1;
                }
                if (np) {
                    float v[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[i] = i < np ? out[pend[i]] : 0.f;
#pragma unroll
                    for (int i = 0; i < 8; ++i) if (i < np) out[pend[i]] = v[i] + addend;
                }
            }
            SBC_TS(2, 9);
        }
        carry_U += tile_U; carry_T += tile_T; carry_R += tile_R;
        SBC_TS(2, 7);                                 // placed
    }
    if (carry_T != nnz) bad = true;           // identical in every thread
    if (bad) atomicOr(&result->err, kErrCorrupt);
}

// --------------------------------------------------------------------------
// One long stream decoded by many workgroups, a tile of kDecThreads segments each (streams of
// tensors that keep very many entries; needs b <= kPackedMaxB).  The dependence between tiles is
// what k_decode_accumulate carries from tile to tile in registers; here it goes through memory:
//   k_dec_tile_fn      per tile: every segment's transition function composed with those before
//                      it in the tile (seg_fn), and the tile's total (tile_fn)
//   k_dec_tile_sums    per tile: the state in which the tile is entered, from the totals of the
//                      tiles before it (tile_entry); then the unary ones, codes and remainder
//                      sum before each segment within the tile (seg_pack) and the tile's totals
//                      (tile_sum)
//   k_dec_tile_place   per tile: the sums of the tiles before it; positions, checks,
//                      out[j] += fl32(scale * mu); the last tile checks the code count against nnz
// Every tile folds what precedes it by itself (a few hundred small values), which costs less
// than a launch per stream in between.
// --------------------------------------------------------------------------
struct DecWide {
    uint32_t t;           // tensor
    uint32_t tile0;       // first tile of this stream in the tile arrays
    uint32_t max_tiles;   // tiles reserved for it (from the worst-case stream length)
    uint32_t pad;
    uint64_t seg0;        // first segment of this stream in the segment arrays
};

struct StreamInfo {
    bool ok;
    float mu;
    uint32_t nnz, n;
    unsigned long long bit_len, word_off, n_words, n_seg;
    const uint32_t* words;
};

// Header and table entry of tensor t, validated as in k_decode_accumulate.
__device__ __forceinline__ StreamInfo stream_info(const uint8_t* __restrict__ msg, unsigned long long msg_bytes,
                                                  const DecDesc* __restrict__ dd, int T, int b, int t) {
    StreamInfo si;
    const uint32_t* h = reinterpret_cast<const uint32_t*>(msg);
    const unsigned long long table_end = 32ull + 24ull * (unsigned)T;
    const uint8_t* e = msg + 32 + 24ull * (unsigned)t;
    const uint32_t h0 = h[0], h1 = h[1], h2 = h[2], h3 = h[3];
    const unsigned long long payload_words = *reinterpret_cast<const unsigned long long*>(msg + 16);
    si.mu = *reinterpret_cast<const float*>(e);
    si.nnz = *reinterpret_cast<const uint32_t*>(e + 4);
    si.bit_len = *reinterpret_cast<const unsigned long long*>(e + 8);
    si.word_off = *reinterpret_cast<const unsigned long long*>(e + 16);
    si.n = dd[t].n;
    si.ok = msg_bytes >= table_end && h0 == 0x31434253u && h1 == 1u && h2 == (uint32_t)T && h3 == (uint32_t)b;
    si.n_words = (si.bit_len + 31ull) >> 5;
    si.n_seg = (si.bit_len + 63ull) >> 6;
    if (si.ok) {
        const unsigned long long max_words = (msg_bytes - table_end) >> 2;
        si.ok = payload_words <= max_words && si.bit_len <= (max_words << 5) &&
                si.word_off <= payload_words && si.n_words <= payload_words - si.word_off &&
                si.nnz <= si.n && (unsigned long long)si.nnz * (unsigned)(b + 1) <= si.bit_len &&
                (si.nnz != 0u || si.bit_len == 0ull);
    }
    si.words = reinterpret_cast<const uint32_t*>(msg + table_end) + si.word_off;
    return si;
}

// Which stream and tile a workgroup of a tile kernel works on; false if it has nothing to do.
__device__ __forceinline__ bool tile_of_block(const DecWide* __restrict__ dw, int n_wide, uint32_t blk,
                                              int* which, uint32_t* tile) {
    for (int i = 0; i < n_wide; ++i) {
        if (blk >= dw[i].tile0 && blk < dw[i].tile0 + dw[i].max_tiles) { *which = i; *tile = blk - dw[i].tile0; return true; }
    }
    return false;
}

// Stages the words of tile `tile` in LDS (bits at or past bit_len read as ones) and returns the
// calling thread's 64-bit segment.  Contains barriers.
__device__ __forceinline__ unsigned long long stage_tile(const StreamInfo& si, uint32_t tile, uint32_t* lds_tile) {
    const int tid = threadIdx.x;
    const unsigned long long w0 = 2ull * kDecThreads * tile;
    __syncthreads();
    for (int i = tid; i < kTileWords + kTileSlack; i += kDecThreads) {
        const unsigned long long w = w0 + (unsigned)i;
        uint32_t v = 0xFFFFFFFFu;
        if (w < si.n_words) {
            v = si.words[w];
            const unsigned long long valid = si.bit_len - 32ull * w;
            if (valid < 32ull) v |= (0xFFFFFFFFu >> valid);
        }
        lds_tile[i] = v;
    }
    __syncthreads();
    return ((unsigned long long)lds_tile[2 * tid] << 32) | lds_tile[2 * tid + 1];
}

__global__ __launch_bounds__(kDecThreads) void k_dec_tile_fn(
        const uint8_t* __restrict__ msg, unsigned long long msg_bytes, const DecDesc* __restrict__ dd,
        const DecWide* __restrict__ dw, int n_wide, int T, int b,
        unsigned long long* __restrict__ seg_fn, unsigned long long* __restrict__ tile_fn,
        ResultBlock* __restrict__ result) {
    __shared__ uint32_t tile_words[kTileWords + kTileSlack];
    __shared__ unsigned long long wave_fn[kDecThreads / 64];
    int which; uint32_t tile;
    if (!tile_of_block(dw, n_wide, blockIdx.x, &which, &tile)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const StreamInfo si = stream_info(msg, msg_bytes, dd, T, b, (int)dw[which].t);
    const unsigned long long n_tiles = (si.n_seg + kDecThreads - 1) / kDecThreads;
    if (!si.ok || n_tiles > dw[which].max_tiles) {        // a valid stream never exceeds its worst case
        if (tile == 0 && tid == 0) atomicOr(&result->err, kErrCorrupt);
        return;
    }
    if (tile >= n_tiles) return;
    const int S = b + 1;
    const unsigned long long w64 = stage_tile(si, tile, tile_words);
    unsigned long long f = packed_exits(w64, b);
#pragma unroll
    for (int dlt = 1; dlt < 64; dlt <<= 1) {
        const unsigned long long o = __shfl_up(f, dlt, 64);
        if (lane >= dlt) f = compose_packed(f, o, S);
    }
    if (lane == 63) wave_fn[wave] = f;
    __syncthreads();
    // everything before this wavefront, as one function
    unsigned long long before = 0ull;
    for (int s = 0; s < S; ++s) before |= (unsigned long long)s << (4 * s);      // identity
    for (int w = 0; w < wave; ++w) before = compose_packed(wave_fn[w], before, S);
    f = compose_packed(f, before, S);
    seg_fn[dw[which].seg0 + (unsigned long long)tile * kDecThreads + tid] = f;
    if (tid == kDecThreads - 1) tile_fn[dw[which].tile0 + tile] = f;
}

// State in which tile `tile` of a stream is entered: the total functions of tiles 0 .. tile-1
// applied in order to state 0.  Thread i folds a run of consecutive tiles, the wavefronts scan
// under composition, and the wavefront totals are walked.  wave_fn: kDecThreads / 64 words of
// LDS.  Contains a barrier; every thread must call it.  The result is the same in every thread.
__device__ __forceinline__ int tile_entry_state(const unsigned long long* __restrict__ fn_of_stream, uint32_t tile,
                                                int S, unsigned long long* wave_fn) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unsigned long long f = 0ull;
    for (int s = 0; s < S; ++s) f |= (unsigned long long)s << (4 * s);           // identity
    const uint32_t per = (tile + kDecThreads - 1) / kDecThreads;
    for (uint32_t j = 0; j < per; ++j) {
        const uint32_t i = (uint32_t)tid * per + j;
        if (i < tile) f = compose_packed(fn_of_stream[i], f, S);
    }
#pragma unroll
    for (int dlt = 1; dlt < 64; dlt <<= 1) {
        const unsigned long long o = __shfl_up(f, dlt, 64);
        if (lane >= dlt) f = compose_packed(f, o, S);
    }
    if (lane == 63) wave_fn[wave] = f;
    __syncthreads();
    int st = 0;
#pragma unroll
    for (int w = 0; w < kDecThreads / 64; ++w) st = apply_packed(wave_fn[w], st);
    return st;
}

__global__ __launch_bounds__(kDecThreads) void k_dec_tile_sums(
        const uint8_t* __restrict__ msg, unsigned long long msg_bytes, const DecDesc* __restrict__ dd,
        const DecWide* __restrict__ dw, int n_wide, int T, int b,
        const unsigned long long* __restrict__ seg_fn, const unsigned long long* __restrict__ tile_fn,
        uint32_t* __restrict__ tile_entry, unsigned long long* __restrict__ seg_pack,
        unsigned long long* __restrict__ tile_sum, ResultBlock* __restrict__ result) {
    __shared__ uint32_t tile_words[kTileWords + kTileSlack];
    __shared__ unsigned long long scratch64[kDecThreads / 64];
    __shared__ unsigned long long wave_fn[kDecThreads / 64];
    int which; uint32_t tile;
    if (!tile_of_block(dw, n_wide, blockIdx.x, &which, &tile)) return;
    const int tid = threadIdx.x;
    const StreamInfo si = stream_info(msg, msg_bytes, dd, T, b, (int)dw[which].t);
    const unsigned long long n_tiles = (si.n_seg + kDecThreads - 1) / kDecThreads;
    if (!si.ok || n_tiles > dw[which].max_tiles || tile >= n_tiles) return;
    const unsigned long long w64 = stage_tile(si, tile, tile_words);
    const unsigned long long seg = (unsigned long long)tile * kDecThreads + tid;
    const int tile_in = tile_entry_state(tile_fn + dw[which].tile0, tile, b + 1, wave_fn);
    if (tid == 0) tile_entry[dw[which].tile0 + tile] = (uint32_t)tile_in;
    const int entry = tid == 0 ? tile_in : apply_packed(seg_fn[dw[which].seg0 + seg - 1], tile_in);
    uint32_t nU = 0u, nT = 0u;
    unsigned long long sR = 0ull;
    bool bad = false;
    if (seg < si.n_seg) {
        int x = entry;
        while (x < 64) {
            const int z = first_zero_from(w64, x);
            nU += (uint32_t)(z - x);
            if (z == 64) break;
            const unsigned long long zpos = seg * 64ull + (unsigned)z;
            if (zpos + 1ull + (unsigned)b > si.bit_len) { bad = true; break; }
            ++nT;
            sR += read_bits(tile_words, (uint32_t)(tid * 64 + z + 1), b);
            x = z + b + 1;
        }
    }
    if (bad) atomicOr(&result->err, kErrCorrupt);
    unsigned long long tot;
    const unsigned long long ex = block_excl_sum<unsigned long long, kDecThreads>(
        (unsigned long long)nU | ((unsigned long long)nT << 16) | (sR << 32), &tot, scratch64);
    seg_pack[dw[which].seg0 + seg] = ex;
    if (tid == 0) tile_sum[dw[which].tile0 + tile] = tot;
}

__global__ __launch_bounds__(kDecThreads) void k_dec_tile_place(
        const uint8_t* __restrict__ msg, unsigned long long msg_bytes, const DecDesc* __restrict__ dd,
        const DecWide* __restrict__ dw, int n_wide, int T, int b, float scale,
        const unsigned long long* __restrict__ seg_fn, const uint32_t* __restrict__ tile_entry,
        const unsigned long long* __restrict__ seg_pack, const unsigned long long* __restrict__ tile_sum,
        ResultBlock* __restrict__ result) {
    __shared__ uint32_t tile_words[kTileWords + kTileSlack];
    __shared__ unsigned long long scratch64[kDecThreads / 64];
    int which; uint32_t tile;
    if (!tile_of_block(dw, n_wide, blockIdx.x, &which, &tile)) return;
    const int tid = threadIdx.x;
    const int t = (int)dw[which].t;
    const StreamInfo si = stream_info(msg, msg_bytes, dd, T, b, t);
    const unsigned long long n_tiles = (si.n_seg + kDecThreads - 1) / kDecThreads;
    if (!si.ok || n_tiles > dw[which].max_tiles || tile >= n_tiles) return;
    const unsigned long long w64 = stage_tile(si, tile, tile_words);
    const unsigned long long seg = (unsigned long long)tile * kDecThreads + tid;
    // unary ones, codes and remainders of the tiles before this one
    unsigned long long off[3];
    {
        unsigned long long part[3] = {0ull, 0ull, 0ull};
        for (uint32_t i = (uint32_t)tid; i < tile; i += kDecThreads) {
            const unsigned long long v = tile_sum[dw[which].tile0 + i];
            part[0] += v & 0xFFFFull; part[1] += (v >> 16) & 0xFFFFull; part[2] += v >> 32;
        }
#pragma unroll
        for (int j = 0; j < 3; ++j) (void)block_excl_sum<unsigned long long, kDecThreads>(part[j], &off[j], scratch64);
    }
    if (tile + 1 == n_tiles && tid == 0) {            // the stream's code count must equal nnz
        const unsigned long long v = tile_sum[dw[which].tile0 + tile];
        if (off[1] + ((v >> 16) & 0xFFFFull) != si.nnz) atomicOr(&result->err, kErrCorrupt);
    }
    if (seg >= si.n_seg) return;
    const int tile_in = (int)tile_entry[dw[which].tile0 + tile];
    const int entry = tid == 0 ? tile_in : apply_packed(seg_fn[dw[which].seg0 + seg - 1], tile_in);
    const unsigned long long pk = seg_pack[dw[which].seg0 + seg];
    unsigned long long U = off[0] + (pk & 0xFFFFull), Tn = off[1] + ((pk >> 16) & 0xFFFFull), R = off[2] + (pk >> 32);
    const gfloat_ptr out = as_global(dd[t].out);
    const float addend = scale * si.mu;
    const uint32_t n = si.n, nnz = si.nnz;
    bool bad = false;
    int x = entry;
    uint32_t pend[8];
    int np = 0;
    while (x < 64) {
        const int z = first_zero_from(w64, x);
        U += (unsigned)(z - x);
        if (z == 64) break;
        const unsigned long long zpos = seg * 64ull + (unsigned)z;
        if (zpos + 1ull + (unsigned)b > si.bit_len) { bad = true; break; }
        R += read_bits(tile_words, (uint32_t)(tid * 64 + z + 1), b);
        const unsigned long long pos = (U << b) + R + Tn;
        if (pos >= n || Tn >= nnz) { bad = true; break; }
        if (Tn == (unsigned long long)nnz - 1ull && zpos + 1ull + (unsigned)b != si.bit_len) bad = true;
        pend[np++] = (uint32_t)pos;
        if (np == 8) {
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = out[pend[i]];
#pragma unroll
            for (int i = 0; i < 8; ++i) out[pend[i]] = v[i] + addend;
            np = 0;
        }
        ++Tn;
        x = z + b + 1;
    }
    if (np) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = i < np ? out[pend[i]] : 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) if (i < np) out[pend[i]] = v[i] + addend;
    }
    if (bad) atomicOr(&result->err, kErrCorrupt);
}

}  // namespace sbc
