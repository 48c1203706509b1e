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
// The bit window is refilled without a branch, from a word fetched one refill ahead, so the
// only memory latency on the per-symbol dependency chain is the table lookup.
template <class RD, class PUT>
__device__ __forceinline__ uint32_t decode_run(const DecodeTables &T, RD rd, uint32_t start, uint32_t count,
                                               uint32_t klo, uint32_t fallback_sym, PUT put, bool &bad)
{
    uint32_t wi = start >> 5;
    uint64_t win = ((((uint64_t)rd(wi)) << 32) | rd(wi + 1)) << (start & 31);
    int avail = 64 - (int)(start & 31);
    wi += 2;
    uint32_t nxt = rd(wi);
    const uint32_t t32 = T.t32, sh = T.sh, has_long = T.has_long;
    for (uint32_t k = 0; k < count; ++k) {
        const bool need = avail <= 32;
        const uint64_t add = ((uint64_t)nxt) << ((32 - avail) & 31);
        win |= need ? add : 0ull;
        avail += need ? 32 : 0;
        wi += need ? 1u : 0u;
        nxt = rd(wi);
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

}  // namespace cmpz
