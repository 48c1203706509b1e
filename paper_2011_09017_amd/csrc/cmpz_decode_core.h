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
constexpr uint32_t kT2Bits = 8;
constexpr uint32_t kT2Size = 1u << kT2Bits;

// Table entries: symbol in bits 0..9, code length in bits 10..15; 0 = not resolved here.
struct DecodeTables {
    uint16_t t1[kT1Size];
    uint16_t t2[kT2Size];
    uint32_t sorted3[(kMaxSym + 2) / 3];   // symbols ordered by (length, symbol), each as its residual
                                  // (symbol - radius) in 10 bits, two's complement, three to a word
                                  // (read only for codewords that neither table level resolves)
    uint64_t first[kMaxCodeLen + 2];   // first canonical code of each length (indexed by the length)
    uint32_t count[kMaxCodeLen + 2];   // codes of each length
    uint32_t offs[kMaxCodeLen + 2];    // index into sorted[] of the first symbol of each length
    uint32_t t32;                 // left-aligned threshold above which codes are longer than kLB
    uint32_t sh;                  // level-2 shift
    uint32_t has_long;            // any code longer than kLB bits
    uint32_t max_len;
    uint32_t payload_units;
    uint32_t n_outliers;
};

// Entry i of the symbols ordered by (length, symbol).
__device__ __forceinline__ uint32_t sorted_at(const DecodeTables &T, uint32_t i)
{
    const uint32_t w = i / 3u;
    return (T.sorted3[w] >> (10u * (i - 3u * w))) & 1023u;
}

// Cooperative copy global -> LDS (both are the same struct).
__device__ __forceinline__ void load_tables(DecodeTables &dst, const DecodeTables *__restrict__ src, int tid,
                                            int nthreads)
{
    static_assert(sizeof(DecodeTables) % 4 == 0, "copied as words");
    const uint32_t *s = reinterpret_cast<const uint32_t *>(src);
    uint32_t *d = reinterpret_cast<uint32_t *>(&dst);
    for (uint32_t k = tid; k < sizeof(DecodeTables) / 4; k += nthreads) d[k] = s[k];
}

// Validation of the container header and code lengths, and construction of the decode tables
// in LDS, by one workgroup of NT >= 256 threads (every workgroup of the fused decode kernel does
// this for itself: about a microsecond, and no separate kernel or round trip through memory).
// The first 256 threads do the work (four symbols each); the others only help to fill level 1.
// `scratch` is LDS the caller does not need yet (at least 12 KB; the ordered symbols are laid out
// there as 16-bit values while the tables are filled).  Returns 0 or the status bits
// of the defect found; contains barriers, so all NT threads must call it.
//
// Canonical codes are ascending in (length, symbol) when left-aligned, so with
//   s[l] = count[l] << (48 - l)  and  P[l] = sum of s[j] over 1 <= j < l
// the first code of length l is P[l] >> (48 - l), the code is complete iff the total is 2^48,
// and a left-aligned value v belongs to the shortest length l with v < P[l+1].
template <int NT>
__device__ __forceinline__ uint32_t build_tables(DecodeTables &T, const DecompressArgs &a, uint32_t *scratch)
{
    static_assert(NT >= 256 && NT % 64 == 0, "whole waves, at least four");
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const bool worker = tid < 256;                                    // uniform in a wave
    Header *hd = reinterpret_cast<Header *>(scratch);                 // 64 words
    uint32_t *ends = scratch + 64;                                    // 4 words
    uint32_t *bad_s = scratch + 68, *bad2_s = scratch + 69;       // defects found before / after the second barrier
    uint64_t *lim = reinterpret_cast<uint64_t *>(scratch + 72);       // 64 x u64: P[l+1], units of 2^-48
    uint32_t (*wave_cnt)[64] = reinterpret_cast<uint32_t (*)[64]>(scratch + 200);   // 16 x 64: [pass*4 + wave][length]
    uint16_t *sorted = reinterpret_cast<uint16_t *>(scratch + 1224);  // kMaxSym x u16
    uint32_t *used_s = scratch + 70;
    const uint32_t nsym = 2 * a.radius;

    if (tid < (int)(kHeaderBytes / 4)) {
        const uint32_t v = reinterpret_cast<const uint32_t *>(a.buf)[tid];
        scratch[tid] = v;
    }
    if (tid >= 64 && tid < 68) {
        const uint32_t *chunk_off = reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_chunk_off);
        const uint32_t *outl_off = reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_outl_off);
        const int k = tid - 64;
        ends[k] = (k == 0) ? chunk_off[0] : (k == 1) ? chunk_off[a.lay.nchunks] : (k == 2) ? outl_off[0] : outl_off[a.lay.nchunks];
    }
    if (tid == 68) { *bad_s = 0; *bad2_s = 0; }
    for (int k = tid; k < 16 * 64; k += NT) (&wave_cnt[0][0])[k] = 0;
    // code lengths, 4 symbols per thread (symbol q*256 + tid), fetched while the header arrives
    const uint32_t padded = (nsym + 15u) & ~15u;
    uint32_t L[4];
    bool bad_len = false;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t k = q * 256u + tid;
        uint32_t v = 0;
        if (worker && k < padded) v = a.buf[a.lay.off_lens + k];
        if ((k >= nsym && v) || v > kMaxCodeLen) { bad_len = true; v = 0; }
        L[q] = v;
    }
    __syncthreads();
    {
        // the reserved tail of the header must be zero
        constexpr int kFirstZero = (int)(offsetof(Header, zero) / 4);
        bool nz = false;
        if (tid >= kFirstZero && tid < (int)(kHeaderBytes / 4)) nz = scratch[tid] != 0;
        if (nz || bad_len) atomicOr(bad_s, kStFormat);
    }
    if (tid == 0) {
        uint32_t bad = 0;
        const Layout &l = a.lay;
        if (hd->magic != kMagic || (hd->version != kVersion && hd->version != kVersionZB) || hd->status != 0) bad = kStFormat;
        if (!bad) {
            if (hd->eb_bits != a.eb_bits) bad = kStMismatch;
            if (hd->version != (a.zero_blocks ? kVersionZB : kVersion)) bad = kStMismatch;
            for (int k = 0; k < 4; ++k) if (hd->shape[k] != a.shape[k]) bad = kStMismatch;
            if (hd->radius != a.radius || hd->chunk != kChunk || hd->sub != a.sub ||
                hd->guard_shift != a.guard_shift) bad = kStMismatch;
        }
        if (!bad) {
            const uint64_t n_out = hd->n_outliers;
            const uint64_t sect = (4 * n_out + 15) & ~15ull;
            if (hd->numel != a.numel || hd->nchunks != l.nchunks) bad = kStFormat;
            else if (hd->off_lens != l.off_lens || hd->off_chunk_off != l.off_chunk_off ||
                     hd->off_outl_off != l.off_outl_off || hd->off_sub_bits != l.off_sub_bits ||
                     hd->off_payload != l.off_payload) bad = kStFormat;
            else if (hd->total_size > a.size || n_out > a.numel || hd->range_events > a.numel) bad = kStFormat;
            else if (hd->off_outl_idx < l.off_payload || ((hd->off_outl_idx - l.off_payload) & 15)) bad = kStFormat;
            else if (hd->off_outl_val != hd->off_outl_idx + sect || hd->total_size != hd->off_outl_val + sect)
                bad = kStFormat;
            else if (((hd->off_outl_idx - l.off_payload) >> 4) >= (1ull << 32)) bad = kStFormat;
            if (!bad) {
                const uint32_t units = (uint32_t)((hd->off_outl_idx - l.off_payload) >> 4);
                if (ends[0] != 0 || ends[1] != units) bad = kStFormat;
                if (ends[2] != 0 || ends[3] != (uint32_t)n_out) bad = kStFormat;
                T.payload_units = units;
                T.n_outliers = (uint32_t)n_out;
            }
        }
        if (bad) atomicOr(bad_s, bad);
    }
    // rank of every symbol among the symbols of its length in its wave and pass
    uint32_t in_wave[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t Lq = L[q];
        uint32_t r = 0;
        unsigned long long remaining = __ballot(Lq != 0);
        while (remaining) {                                   // wave-uniform
            const int leader = __ffsll((long long)remaining) - 1;
            const uint32_t Lx = (uint32_t)__builtin_amdgcn_readlane((int)Lq, leader);
            const unsigned long long m = __ballot(Lq == Lx);
            if (Lq == Lx) r = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            if (lane == leader) wave_cnt[q * 4 + wv][Lx] = (uint32_t)__popcll(m);
            remaining &= ~m;
        }
        in_wave[q] = r;
    }
    __syncthreads();
    if (*bad_s) return *bad_s;

    // wave 0, lane = length: totals per length, start of every (pass, wave) group, first codes
    if (wv == 0) {
        uint32_t cnt = 0;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const uint32_t c = wave_cnt[k][lane];
            wave_cnt[k][lane] = cnt;                          // symbols of this length in earlier groups
            cnt += c;
        }
        if (lane == 0) cnt = 0;
        const uint32_t used = (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_sum(cnt), 63);
        const uint32_t offs = wave_inclusive_sum(cnt) - cnt;
        const unsigned long long present = __ballot(cnt != 0);
        const uint32_t max_len = present ? 63u - (uint32_t)__builtin_clzll(present) : 0u;
        // s < 2^58: three limbs of 24 bits, each scanned in 32 bits without overflow
        const uint64_t sl = (lane >= 1 && lane <= (int)kMaxCodeLen) ? ((uint64_t)cnt << (kMaxCodeLen - lane)) : 0ull;
        const uint32_t i0 = wave_inclusive_sum((uint32_t)(sl & 0xffffffu));
        const uint32_t i1 = wave_inclusive_sum((uint32_t)((sl >> 24) & 0xffffffu));
        const uint32_t i2 = wave_inclusive_sum((uint32_t)(sl >> 48));
        const uint64_t incl = (uint64_t)i0 + ((uint64_t)i1 << 24) + ((uint64_t)i2 << 48);
        const uint64_t excl = incl - sl;
        const uint64_t first = (lane >= 1 && lane <= (int)kMaxCodeLen) ? (excl >> (kMaxCodeLen - lane)) : 0ull;
        if (lane <= (int)kMaxCodeLen) { T.first[lane] = first; T.count[lane] = cnt; T.offs[lane] = offs; }
        lim[lane] = incl;
        if (lane == 63) {
            uint32_t bad = 0;
            const uint64_t one = 1ull << kMaxCodeLen;
            if (used >= 2 && incl != one) bad = kStFormat;
            if (used == 1 && max_len != 1) bad = kStFormat;
            // no codeword at all: an empty tensor, or (version 2) nothing but sub-blocks of zero residuals
            if (used == 0 && a.numel != 0 && !(a.zero_blocks && hd->total_bits == 0)) bad = kStFormat;
            if (hd->max_len != max_len) bad = kStFormat;
            if (bad) *bad2_s = bad;
            *used_s = used;
            T.max_len = max_len;
        }
        if (lane == (int)kLB) {
            // codes longer than kLB bits occupy left-aligned 32-bit values [t32, 2^32)
            const uint64_t t = incl >> (kMaxCodeLen - 32);
            const uint64_t span = (1ull << 32) - (t < (1ull << 32) ? t : (1ull << 32));
            uint32_t sh = 0;
            while ((span >> sh) > kT2Size) ++sh;
            T.t32 = (uint32_t)t; T.sh = sh; T.has_long = (max_len > kLB && span > 0) ? 1u : 0u;
        }
    }
    __syncthreads();
    if (*bad2_s) return *bad2_s;

    // symbols ordered by (length, symbol)
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (L[q]) sorted[T.offs[L[q]] + wave_cnt[q * 4 + wv][L[q]] + in_wave[q]] = (uint16_t)((q * 256 + tid - a.radius) & 1023u);
    __syncthreads();

    // level 1: entry idx is the codeword (if any, of at most kLB bits) that prefixes idx
    {
        uint32_t l1[kLB + 1];
#pragma unroll
        for (uint32_t l = 1; l <= kLB; ++l) {
            const uint64_t v = lim[l] >> (kMaxCodeLen - kLB);
            l1[l] = v > kT1Size ? kT1Size : (uint32_t)v;
        }
#pragma unroll 2
        for (uint32_t idx = tid; idx < kT1Size; idx += NT) {
            uint32_t l = 1;
#pragma unroll
            for (uint32_t k = 1; k <= kLB; ++k) l += (idx >= l1[k]) ? 1u : 0u;
            uint32_t e = 0;
            if (l <= kLB) e = sorted[T.offs[l] + (idx >> (kLB - l)) - (uint32_t)T.first[l]] | (l << 10);
            T.t1[idx] = (uint16_t)e;
        }
    }
    // level 2: entry i covers left-aligned 32-bit values t32 + [i << sh, (i+1) << sh); it holds a
    // codeword only if the whole entry lies inside it (length at most 32 - sh)
    if (worker) {
        const uint32_t sh = T.sh, t32 = T.t32, has_long = T.has_long;
        const uint32_t lmax = (32 - sh < T.max_len) ? 32 - sh : T.max_len;
        constexpr int kPer = (int)kT2Size / 256;            // entries per thread
        static_assert(kPer * 256 == (int)kT2Size, "level 2 is filled by 256 threads");
        uint64_t v[kPer];
        uint32_t l[kPer];
#pragma unroll
        for (int k = 0; k < kPer; ++k) { v[k] = (uint64_t)t32 + ((uint64_t)(tid + 256 * k) << sh); l[k] = kLB + 1; }
        for (uint32_t j = kLB + 1; j <= lmax; ++j) {          // uniform
            const uint64_t lj = lim[j] >> (kMaxCodeLen - 32);
#pragma unroll
            for (int k = 0; k < kPer; ++k) l[k] += (v[k] >= lj) ? 1u : 0u;
        }
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            uint32_t e = 0;
            if (has_long && v[k] < (1ull << 32) && l[k] <= lmax)
                e = sorted[T.offs[l[k]] + (uint32_t)((v[k] >> (32 - l[k])) - T.first[l[k]])] | (l[k] << 10);
            T.t2[tid + 256 * k] = (uint16_t)e;
        }
    }
    // the ordered symbols in their packed form, for the codewords the two levels leave
    {
        const uint32_t used = *used_s;
        for (uint32_t w = tid; w < (kMaxSym + 2) / 3; w += NT) {
            uint32_t v = 0;
#pragma unroll
            for (uint32_t j = 0; j < 3; ++j)
                if (3 * w + j < used) v |= (uint32_t)sorted[3 * w + j] << (10 * j);
            T.sorted3[w] = v;
        }
    }
    __syncthreads();
    return 0;
}

// Table entries are length << 10 | residual, the residual (symbol - radius) in 10 bits.
__device__ __forceinline__ int32_t entry_residual(uint32_t e)
{
    return __builtin_amdgcn_sbfe((int)e, 0, 10);
}

// Level 2 resolves every codeword of at most 32 - sh bits (its entries start at t32, a multiple
// of 2^sh whenever such a codeword exists, so each one covers whole entries): the search over
// the lengths starts behind them.
__device__ __forceinline__ uint32_t first_unresolved_length(uint32_t sh)
{
    const uint32_t l = 33u - sh;
    return l > kLB + 1 ? l : kLB + 1;
}

// Decode `count` codewords that start at bit `start` of a chunk stream whose 32-bit words
// are read through rd(word index); rd must be safe for any index (clamp) -- words past the
// stream only ever reach bits that a well-formed stream does not consume.  put(k, symbol) is
// called for k >= klo, where the second argument is the residual symbol - radius (the outlier
// marker, symbol 0, arrives as -radius).  Returns the bit position after the last codeword; sets bad when a
// bit pattern matches no codeword.
//
// The bit window is refilled from a word fetched one refill ahead, so the only memory
// latency on the per-symbol dependency chain is the table lookup.
template <bool EAGER, class RD, class PUT>
__device__ __forceinline__ uint32_t decode_run(const DecodeTables &T, RD rd, uint32_t start, uint32_t count,
                                               uint32_t klo, PUT put, bool &bad)
{
    uint32_t wi = start >> 5;
    uint64_t win = ((((uint64_t)rd(wi)) << 32) | rd(wi + 1)) << (start & 31);
    int avail = 64 - (int)(start & 31);
    wi += 2;
    uint32_t nxt = rd(wi);
    const uint32_t t32 = T.t32, sh = T.sh, has_long = T.has_long;
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
                uint32_t len = 0, sy = 0;                    // no match: residual 0
                for (uint32_t L = has_long ? first_unresolved_length(sh) : kLB + 1; L <= T.max_len; ++L) {
                    const uint64_t code = w64 >> (64 - L);
                    if (code >= T.first[L] && code - T.first[L] < T.count[L]) {
                        sy = sorted_at(T, T.offs[L] + (uint32_t)(code - T.first[L]));
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
        if (k >= klo) put(k, entry_residual(e));
    }
    return 32u * wi - (uint32_t)avail;
}

// Decoder for a bit stream staged in LDS.  Word k of the stream is S[kStagePad + k].  Decodes
// `count` codewords from bit `pos` on and calls put(k, residual) for k >= skip; returns the bit
// position after the last codeword.
//
// The 32 bits from position p on are alignbit(S[j], S[j+1], -p mod 32) with j = (p + 31) / 32 - 1
// (stream words): counted this way the shift stays below 32 also when p is a multiple of 32.
// Word indices are not clamped: a codeword has at most kMaxCodeLen bits, so `count` codewords
// starting inside the staged words read at most count * kMaxCodeLen / 32 + 3 words past them,
// whatever the stream holds; the caller's buffer has that many words behind the staged ones
// (stage_tail_words).
constexpr uint32_t stage_tail_words(uint32_t count) { return count * kMaxCodeLen / 32 + 4; }
constexpr int kStagePad = 4;
template <class PUT>
__device__ __forceinline__ uint32_t decode_lds(const DecodeTables &T, const uint32_t *S, uint32_t pos,
                                               uint32_t count, uint32_t skip, PUT put, bool &bad)
{
    const uint32_t t32 = T.t32, sh = T.sh;
    const char *t1 = reinterpret_cast<const char *>(T.t1);
    // The three stream words around the position live in registers: wa, wb are the window of the
    // current codeword, wc the word after them.  A codeword of the first two table levels is at
    // most 27 bits long, so the window moves on by one word at most, and the word that then
    // becomes wc is fetched a whole step before it can be needed: the only LDS access a step
    // has to wait for is the table look-up.
    uint32_t npos = 0u - pos;                                 // alignbit takes its shift from -pos mod 32
    // stream word J-1 holds bit pos (or ends just before it), J = ceil(pos / 32); kept as N = -J, which is
    // one arithmetic shift of npos
    int32_t N = (int32_t)npos >> 5;
    const uint32_t *Sw = S + kStagePad;
    // LDS byte address of stream word 1: word 1 - Nn is then one multiply-add away
    typedef const uint32_t __attribute__((address_space(3))) *lds_word_ptr;
    const uint32_t sw1 = (uint32_t)(uintptr_t)(lds_word_ptr)(Sw + 1);
    uint32_t wa = Sw[-1 - N], wb = Sw[-N], wc = Sw[1 - N];
#pragma unroll 4
    for (uint32_t k = 0; k < count; ++k) {
        const uint32_t hi = __builtin_amdgcn_alignbit(wa, wb, npos);
        uint32_t e = *reinterpret_cast<const uint16_t *>(t1 + ((hi >> (31 - kLB)) & (2u * kT1Size - 2u)));
        if (__builtin_expect(e == 0, 0)) {
            {
                // (a codebook without long codes has a second table of zeros: no test for that case)
                uint32_t i2 = (hi - t32) >> sh;
                i2 = i2 < kT2Size ? i2 : kT2Size - 1;
                e = T.t2[i2];
            }
            if (__builtin_expect(e == 0, 0)) {
                // canonical search over the lengths the second level does not resolve: up to 31 bits
                // in 32-bit arithmetic (a code below the first one of its length wraps to a difference
                // of at least 2^31, far above any count), beyond that on a 64-bit window
                uint32_t len = 0, sy = 0;                     // no match: residual 0
                const uint32_t max_len = T.max_len;
                uint32_t L = first_unresolved_length(sh);
                for (; L <= max_len && L < 32u; ++L) {
                    const uint32_t rel = (hi >> (32u - L)) - (uint32_t)T.first[L];
                    if (rel < T.count[L]) {
                        sy = sorted_at(T, T.offs[L] + rel);
                        len = L;
                        break;
                    }
                }
                if (len == 0 && max_len >= 32u) {
                    const uint32_t lo = __builtin_amdgcn_alignbit(wb, wc, npos);
                    const uint64_t v = (((uint64_t)hi) << 32) | lo;
                    for (L = L < 32u ? 32u : L; L <= max_len; ++L) {
                        const uint64_t code = v >> (64 - L);
                        if (code >= T.first[L] && code - T.first[L] < T.count[L]) {
                            sy = sorted_at(T, T.offs[L] + (uint32_t)(code - T.first[L]));
                            len = L;
                            break;
                        }
                    }
                }
                if (len == 0) { bad = true; len = 1; }
                e = sy | (len << 10);
                // such a codeword may end two words further on: take the first of the two moves here
                const int32_t Nf = (int32_t)(npos - len) >> 5;
                if (Nf < N - 1) { wa = wb; wb = wc; wc = Sw[2 - N]; --N; }
            }
        }
        npos -= e >> 10;
        const int32_t Nn = (int32_t)npos >> 5;
        const bool moved = Nn != N;
        wa = moved ? wb : wa;
        wb = moved ? wc : wb;
        {
            uint32_t at;                                     // sw1 - 4 * Nn (|Nn| is a word index: far inside 24 bits)
            asm("v_mad_i32_i24 %0, %1, -4, %2" : "=v"(at) : "v"(Nn), "s"(sw1));
            wc = *(lds_word_ptr)(uintptr_t)at;
        }
        N = Nn;
        if (k >= skip) put(k, entry_residual(e));
    }
    return 0u - npos;
}

}  // namespace cmpz
