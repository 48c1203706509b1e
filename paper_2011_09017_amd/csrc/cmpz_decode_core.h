// Huffman decode core shared by the decompression kernels: table layout and the
// per-lane decode loop.  Internal to libcmpz.
//
// Two lookup levels.  Level 1 is indexed by the next kLB bits and resolves every
// codeword of at most kLB bits.  Canonical codes grow with their length when
// left-aligned, so all longer codewords sit above a threshold t32 in the
// left-aligned code space; level 2 is indexed by (next 32 bits - t32) >> sh and
// resolves codewords of up to 32 - sh bits.  Whatever is longer still (rare, and
// impossible unless counts are extremely skewed) is found by the textbook
// canonical search over first[]/count[].
#pragma once
#include "cmpz_internal.h"

namespace cmpz {

constexpr uint32_t kT1Size = 1u << kLB;
constexpr uint32_t kT2Bits = 10;
constexpr uint32_t kT2Size = 1u << kT2Bits;

// Table entries: symbol in bits 0..9, code length in bits 10..15; 0 = not resolved here.
struct DecodeTables {
    uint16_t t1[kT1Size];
    uint16_t t2[kT2Size];
    uint16_t sorted[kMaxSym];     // symbols ordered by (length, symbol)
    uint64_t first[64];           // first canonical code of each length
    uint32_t count[64];           // codes of each length
    uint32_t offs[64];            // index into sorted[] of the first symbol of each length
    uint32_t t32;                 // left-aligned threshold above which codes are longer than kLB
    uint32_t sh;                  // level-2 shift
    uint32_t has_long;            // any code longer than kLB bits
    uint32_t max_len;
    uint32_t payload_units;
    uint32_t n_outliers;
};

// Cooperative copy global -> LDS (both are the same struct).
__device__ __forceinline__ void load_tables(DecodeTables &dst, const DecodeTables *__restrict__ src, int tid,
                                            int nthreads)
{
    static_assert(sizeof(DecodeTables) % 4 == 0, "copied as words");
    const uint32_t *s = reinterpret_cast<const uint32_t *>(src);
    uint32_t *d = reinterpret_cast<uint32_t *>(&dst);
    for (uint32_t k = tid; k < sizeof(DecodeTables) / 4; k += nthreads) d[k] = s[k];
}

// Decode `count` codewords that start at bit `start` of a chunk stream whose 32-bit words
// are read through rd(word index); rd must be safe for any index (clamp) -- words past the
// stream only ever reach bits that a well-formed stream does not consume.  put(k, symbol) is
// called for k >= klo.  Returns the bit position after the last codeword; sets bad when a
// bit pattern matches no codeword.
//
// The bit window is refilled from a word fetched one refill ahead, so the only memory
// latency on the per-symbol dependency chain is the table lookup.
template <bool EAGER, class RD, class PUT>
__device__ __forceinline__ uint32_t decode_run(const DecodeTables &T, RD rd, uint32_t start, uint32_t count,
                                               uint32_t klo, uint32_t fallback_sym, PUT put, bool &bad,
                                               long long *dbg_t0 = nullptr)
{
    uint32_t wi = start >> 5;
    uint64_t win = ((((uint64_t)rd(wi)) << 32) | rd(wi + 1)) << (start & 31);
    int avail = 64 - (int)(start & 31);
    wi += 2;
    uint32_t nxt = rd(wi);
    const uint32_t t32 = T.t32, sh = T.sh, has_long = T.has_long;
#ifdef CMPZ_PHASE_CLOCKS
    if (dbg_t0) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); *dbg_t0 = clock64(); }
#endif
    for (uint32_t k = 0; k < count; ++k) {
        if (EAGER) {
            // cheap reads (LDS): branch-free refill, the next word is refetched every step
            const bool need = avail <= 32;
            const uint64_t add = ((uint64_t)nxt) << ((32 - avail) & 31);
            win |= need ? add : 0ull;
            avail += need ? 32 : 0;
            wi += need ? 1u : 0u;
            nxt = rd(wi);
        } else if (avail <= 32) {
            // global memory: touch the prefetched word only here, so that its latency is waited
            // for once per consumed word and not on every step
            win |= ((uint64_t)nxt) << (32 - avail);
            avail += 32;
            ++wi;
            nxt = rd(wi);
        }
        const uint32_t hi = (uint32_t)(win >> 32);
        uint32_t e = T.t1[hi >> (32 - kLB)];
        if (e == 0) {
            if (has_long) {
                uint32_t i2 = (hi - t32) >> sh;
                i2 = i2 < kT2Size ? i2 : kT2Size - 1;
                e = T.t2[i2];
            }
            if (e == 0) {
                // canonical search on a fresh 64-bit window (codes longer than level 2 resolves)
                uint32_t pos = 32u * wi - (uint32_t)avail;
                const uint32_t w0 = pos >> 5, off = pos & 31;
                uint64_t w64 = ((((uint64_t)rd(w0)) << 32) | rd(w0 + 1)) << off;
                if (off) w64 |= (uint64_t)(rd(w0 + 2) >> (32 - off));
                uint32_t len = 0, sy = fallback_sym;
                for (uint32_t L = kLB + 1; L <= T.max_len; ++L) {
                    const uint64_t code = w64 >> (64 - L);
                    if (code >= T.first[L] && code - T.first[L] < T.count[L]) {
                        sy = T.sorted[T.offs[L] + (uint32_t)(code - T.first[L])];
                        len = L;
                        break;
                    }
                }
                if (len == 0) { bad = true; len = 1; }
                pos += len;
                wi = pos >> 5;
                win = ((((uint64_t)rd(wi)) << 32) | rd(wi + 1)) << (pos & 31);
                avail = 64 - (int)(pos & 31);
                wi += 2;
                nxt = rd(wi);
                e = sy | (64u << 10);            // length already consumed: marker above any real length
            }
        }
        const uint32_t len = e >> 10;
        if (len < 64u) { win <<= len; avail -= (int)len; }
        if (k >= klo) put(k, e & 1023u);
    }
    return 32u * wi - (uint32_t)avail;
}

// Variant of decode_run for short runs (at most 32 codewords): the first eight 32-bit words of
// the run are fetched up front, back to back, and consumed from registers, so that no memory
// latency sits inside the per-symbol loop -- in a wave the lanes refill at different steps, and
// a load issued by some lanes one step ago would otherwise be waited for by all.  A run that
// needs a ninth word (more than about 7 bits per codeword) fetches the rest on demand.
// words[k] must be valid for k <= last; larger indices are clamped to `last`.
template <class PUT>
__device__ __forceinline__ uint32_t decode_run_regs(const DecodeTables &T, const uint32_t *__restrict__ words,
                                                    uint32_t last, uint32_t start, uint32_t count, uint32_t klo,
                                                    uint32_t fallback_sym, PUT put, bool &bad)
{
    const uint32_t w0 = start >> 5;
    uint32_t q[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { const uint32_t k = w0 + j; q[j] = words[k < last ? k : last]; }
    auto rd = [&](uint32_t k) -> uint32_t { return words[k < last ? k : last]; };
    uint64_t win = ((((uint64_t)q[0]) << 32) | q[1]) << (start & 31);
    int avail = 64 - (int)(start & 31);
    uint32_t wi = w0 + 2;                     // index of the word held in nxt
    uint32_t nxt = q[2];
    uint32_t q3 = q[3], q4 = q[4], q5 = q[5], q6 = q[6], q7 = q[7];
    const uint32_t t32 = T.t32, sh = T.sh, has_long = T.has_long;
    for (uint32_t k = 0; k < count; ++k) {
        if (avail <= 32) {
            win |= ((uint64_t)nxt) << (32 - avail);
            avail += 32;
            ++wi;
            nxt = q3; q3 = q4; q4 = q5; q5 = q6; q6 = q7;
            if (wi >= w0 + 8) nxt = rd(wi);   // past the prefetched words
        }
        const uint32_t hi = (uint32_t)(win >> 32);
        uint32_t e = T.t1[hi >> (32 - kLB)];
        if (e == 0) {
            if (has_long) {
                uint32_t i2 = (hi - t32) >> sh;
                i2 = i2 < kT2Size ? i2 : kT2Size - 1;
                e = T.t2[i2];
            }
            if (e == 0) {
                // canonical search on a fresh 64-bit window (codes longer than level 2 resolves)
                uint32_t pos = 32u * wi - (uint32_t)avail;
                const uint32_t p0 = pos >> 5, off = pos & 31;
                uint64_t w64 = ((((uint64_t)rd(p0)) << 32) | rd(p0 + 1)) << off;
                if (off) w64 |= (uint64_t)(rd(p0 + 2) >> (32 - off));
                uint32_t len = 0, sy = fallback_sym;
                for (uint32_t L = kLB + 1; L <= T.max_len; ++L) {
                    const uint64_t code = w64 >> (64 - L);
                    if (code >= T.first[L] && code - T.first[L] < T.count[L]) {
                        sy = T.sorted[T.offs[L] + (uint32_t)(code - T.first[L])];
                        len = L;
                        break;
                    }
                }
                if (len == 0) { bad = true; len = 1; }
                pos += len;
                wi = pos >> 5;
                win = ((((uint64_t)rd(wi)) << 32) | rd(wi + 1)) << (pos & 31);
                avail = 64 - (int)(pos & 31);
                wi += 2;
                nxt = rd(wi);
                // the register queue must line up with wi again: words wi+1 .. wi+5.  (If wi is already
                // past the prefetched range the on-demand fetch above keeps overriding it: still right.)
                q3 = rd(wi + 1); q4 = rd(wi + 2); q5 = rd(wi + 3); q6 = rd(wi + 4); q7 = rd(wi + 5);
                e = sy | (64u << 10);            // length already consumed: marker above any real length
            }
        }
        const uint32_t len = e >> 10;
        if (len < 64u) { win <<= len; avail -= (int)len; }
        if (k >= klo) put(k, e & 1023u);
    }
    return 32u * wi - (uint32_t)avail;
}

// Decoder for one complete sub-block of 32 codewords (the hot loop of the fused
// kernel).  The eight first words of the run are fetched up front and consumed from a register
// queue; the 64-bit window is topped up once per two codewords (it then holds more than 32 valid
// bits, enough for two first-level codewords of at most kLB bits or one longer codeword).
// ROWSUM: instead of the residual d[k] the running row sum is stored, restarted wherever bit k
// of reset_mask is set.  out[k] is written for every k in 0..31.
// Returns the bit position after the 32nd codeword.
template <bool ROWSUM>
__device__ __forceinline__ uint32_t decode32(const DecodeTables &T, const uint32_t *__restrict__ words, uint32_t last,
                                             uint32_t start, uint32_t reset_mask, int32_t radius, int32_t *out,
                                             bool &bad)
{
    const uint32_t w0 = start >> 5;
    uint32_t q[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { const uint32_t k = w0 + j; q[j] = words[k < last ? k : last]; }
    auto rd = [&](uint32_t k) -> uint32_t { return words[k < last ? k : last]; };
    uint64_t win = ((((uint64_t)q[0]) << 32) | q[1]) << (start & 31);
    int avail = 64 - (int)(start & 31);
    uint32_t wi = w0 + 2;                     // index of the word held in nxt
    uint32_t nxt = q[2];
    uint32_t q3 = q[3], q4 = q[4], q5 = q[5], q6 = q[6], q7 = q[7];
    const uint32_t t32 = T.t32, sh = T.sh, has_long = T.has_long;
    int32_t run = 0;

    auto refill = [&]() {
        if (avail <= 32) {
            win |= ((uint64_t)nxt) << (32 - avail);
            avail += 32;
            ++wi;
            nxt = q3; q3 = q4; q4 = q5; q5 = q6; q6 = q7;
            if (wi >= w0 + 8) nxt = rd(wi);   // past the prefetched words
        }
    };
    // first-level miss: second level, then the canonical search; consumes the codeword itself
    auto slow = [&]() -> uint32_t {
        refill();                              // second level looks at up to 32 bits
        const uint32_t hi = (uint32_t)(win >> 32);
        uint32_t e = 0;
        if (has_long) {
            uint32_t i2 = (hi - t32) >> sh;
            i2 = i2 < kT2Size ? i2 : kT2Size - 1;
            e = T.t2[i2];
        }
        if (e != 0) {
            const uint32_t len = e >> 10;
            win <<= len; avail -= (int)len;
            refill();                          // a long codeword may have used up the margin
            return e & 1023u;
        }
        uint32_t pos = 32u * wi - (uint32_t)avail;
        const uint32_t p0 = pos >> 5, off = pos & 31;
        uint64_t w64 = ((((uint64_t)rd(p0)) << 32) | rd(p0 + 1)) << off;
        if (off) w64 |= (uint64_t)(rd(p0 + 2) >> (32 - off));
        uint32_t len = 0, sy = (uint32_t)radius;
        for (uint32_t L = kLB + 1; L <= T.max_len; ++L) {
            const uint64_t code = w64 >> (64 - L);
            if (code >= T.first[L] && code - T.first[L] < T.count[L]) {
                sy = T.sorted[T.offs[L] + (uint32_t)(code - T.first[L])];
                len = L;
                break;
            }
        }
        if (len == 0) { bad = true; len = 1; }
        pos += len;
        wi = pos >> 5;
        win = ((((uint64_t)rd(wi)) << 32) | rd(wi + 1)) << (pos & 31);
        avail = 64 - (int)(pos & 31);
        wi += 2;
        nxt = rd(wi);
        q3 = rd(wi + 1); q4 = rd(wi + 2); q5 = rd(wi + 3); q6 = rd(wi + 4); q7 = rd(wi + 5);
        return sy;
    };
    auto one = [&](int k) {
        const uint32_t hi = (uint32_t)(win >> 32);
        const uint32_t e = T.t1[hi >> (32 - kLB)];
        uint32_t sy;
        if (e != 0) {
            const uint32_t len = e >> 10;
            sy = e & 1023u;
            win <<= len; avail -= (int)len;
        } else {
            sy = slow();
        }
        const int32_t d = (int32_t)sy - radius;
        if (ROWSUM) {
            const int32_t keep = ~__builtin_amdgcn_sbfe((int)reset_mask, k, 1);     // 0 where the row restarts
            run = (run & keep) + d;
            out[k] = run;
        } else {
            out[k] = d;
        }
    };
    // not unrolled further: the rare paths are inlined in every copy of the body, and the loop
    // has to stay well inside the instruction cache
#pragma unroll 1
    for (int k = 0; k < 32; k += 2) {
        refill();
        one(k);
        one(k + 1);
    }
    return 32u * wi - (uint32_t)avail;
}

}  // namespace cmpz
