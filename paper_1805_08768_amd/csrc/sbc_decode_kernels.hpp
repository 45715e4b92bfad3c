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

constexpr int kDecThreads = 256;
constexpr int kMaxB = 30;
constexpr int kStates = kMaxB + 1;

struct DecDesc {
    float* out;
    uint32_t n;
    uint32_t pad;
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

__global__ __launch_bounds__(kDecThreads) void k_decode_accumulate(
        const uint8_t* __restrict__ msg, unsigned long long msg_bytes,
        const DecDesc* __restrict__ dd, int T, int b, float scale, ResultBlock* __restrict__ result) {
    __shared__ uint8_t fn[2][kStates][kDecThreads];       // transition functions, [state][segment]
    __shared__ unsigned long long scratch64[kDecThreads / 64];
    __shared__ uint32_t s_state;
    __shared__ uint32_t tile[kTileWords + kTileSlack];   // words past the stream read as ones

    const int tid = threadIdx.x;
    const int t = blockIdx.x;

    // ---- header and table entry (validated by every workgroup; all threads agree) ----
    const uint32_t* h = reinterpret_cast<const uint32_t*>(msg);
    const unsigned long long table_end = 32ull + 24ull * (unsigned)T;
    bool ok = msg_bytes >= table_end && h[0] == 0x31434253u && h[1] == 1u &&
              h[2] == (uint32_t)T && h[3] == (uint32_t)b;
    unsigned long long payload_words = 0ull, bit_len = 0ull, word_off = 0ull;
    uint32_t nnz = 0u;
    float mu = 0.f;
    if (ok) {
        payload_words = *reinterpret_cast<const unsigned long long*>(msg + 16);
        const uint8_t* e = msg + 32 + 24ull * (unsigned)t;
        mu = *reinterpret_cast<const float*>(e);
        nnz = *reinterpret_cast<const uint32_t*>(e + 4);
        bit_len = *reinterpret_cast<const unsigned long long*>(e + 8);
        word_off = *reinterpret_cast<const unsigned long long*>(e + 16);
        const unsigned long long max_words = (msg_bytes - table_end) >> 2;
        const unsigned long long n_words_t = (bit_len + 31ull) >> 5;
        ok = payload_words <= max_words && bit_len <= (max_words << 5) &&
             word_off <= payload_words && n_words_t <= payload_words - word_off &&
             nnz <= dd[t].n && (unsigned long long)nnz * (unsigned)(b + 1) <= bit_len &&
             (nnz != 0u || bit_len == 0ull);
    }
    if (!ok) {
        if (tid == 0) atomicOr(&result->err, kErrCorrupt);
        return;
    }
    if (nnz == 0u) return;

    const uint32_t n = dd[t].n;
    const gfloat_ptr out = as_global(dd[t].out);
    const float addend = scale * mu;
    const uint32_t* __restrict__ words =
        reinterpret_cast<const uint32_t*>(msg + table_end) + word_off;
    const unsigned long long n_words = (bit_len + 31ull) >> 5;
    const unsigned long long n_seg = (bit_len + 63ull) >> 6;
    const int S = b + 1;                                  // number of states

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

        // ---- exit state for every entry state ----
        for (int s = 0; s < S; ++s) {
            int x = s;                       // entry state j: the first j bits finish a remainder
            int exit_state = 0;
            while (true) {
                if (x >= 64) { exit_state = x - 64; break; }
                const int z = first_zero_from(w64, x);
                if (z == 64) { exit_state = 0; break; }
                x = z + b + 1;
            }
            fn[0][s][tid] = (uint8_t)exit_state;
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
        const int entry = (tid == 0) ? carry_state : (int)fn[cur][carry_state][tid - 1];
        if (tid == kDecThreads - 1) s_state = fn[cur][carry_state][tid];
        __syncthreads();
        carry_state = (int)s_state;

        // ---- first walk: unary ones, terminators and remainder sum of this segment ----
        uint32_t nU = 0u, nT = 0u;
        unsigned long long sR = 0ull;
        if (seg < n_seg) {
            int x = entry;
            while (x < 64) {
                const int z = first_zero_from(w64, x);
                nU += (uint32_t)(z - x);
                if (z == 64) break;
                const unsigned long long zpos = seg * 64ull + (unsigned)z;
                if (zpos + 1ull + (unsigned)b > bit_len) { bad = true; break; }
                ++nT;
                sR += read_bits(tile, (uint32_t)(tid * 64 + z + 1), b);
                x = z + b + 1;
            }
        }
        unsigned long long tile_U, tile_T, tile_R;
        const unsigned long long exU = block_excl_sum<unsigned long long, kDecThreads>(nU, &tile_U, scratch64);
        const unsigned long long exT = block_excl_sum<unsigned long long, kDecThreads>(nT, &tile_T, scratch64);
        const unsigned long long exR = block_excl_sum<unsigned long long, kDecThreads>(sR, &tile_R, scratch64);

        // ---- second walk: place every code whose terminating zero lies in this segment ----
        if (seg < n_seg && !bad) {
            unsigned long long U = carry_U + exU, Tn = carry_T + exT, R = carry_R + exR;
            int x = entry;
            uint32_t pend[4];                // positions are distinct: update them four at a time
            int np = 0;
            while (x < 64) {
                const int z = first_zero_from(w64, x);
                U += (unsigned)(z - x);
                if (z == 64) break;
                const unsigned long long zpos = seg * 64ull + (unsigned)z;
                R += read_bits(tile, (uint32_t)(tid * 64 + z + 1), b);
                const unsigned long long pos = (U << b) + R + Tn;
                if (pos >= n || Tn >= nnz) { bad = true; break; }
                if (Tn == (unsigned long long)nnz - 1ull && zpos + 1ull + (unsigned)b != bit_len) bad = true;
                pend[np++] = (uint32_t)pos;
                if (np == 4) {
                    const float v0 = out[pend[0]], v1 = out[pend[1]], v2 = out[pend[2]], v3 = out[pend[3]];
                    out[pend[0]] = v0 + addend; out[pend[1]] = v1 + addend;
                    out[pend[2]] = v2 + addend; out[pend[3]] = v3 + addend;
                    np = 0;
                }
                ++Tn;
                x = z + b + 1;
            }
            for (int i = 0; i < np; ++i) out[pend[i]] += addend;
        }
        carry_U += tile_U; carry_T += tile_T; carry_R += tile_R;
    }
    if (carry_T != nnz) bad = true;           // identical in every thread
    if (bad) atomicOr(&result->err, kErrCorrupt);
}

}  // namespace sbc
