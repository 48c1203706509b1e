// Sweep 2 of compression: chunked Huffman bit-packing (the entropy-coding stage of Section 3.1)
// for all tensors of a call, in three launches with no ordering between workgroups:
//
//   k_lengths  one streaming pass over the symbols (8 or 16 bits each, as the first sweep left
//              them): the bit count of every sub-block (written straight into the container),
//              of every chunk and of every range of kPackChunks chunks;
//   k_scan     one workgroup per tensor: exclusive prefix sums of the ranges' payload units
//              and outlier counts, the container header, the decision whether it fits;
//   k_pack     the same ranges again: chunk offsets from the range's prefix, the codewords of
//              a chunk (four neighbours merged in registers) OR-ed into a per-wave LDS image at
//              their own bit positions, 128-bit stores; outlier records of the chunks that hold
//              any.
//
// Reading the symbols twice costs 1 to 2 bytes per element of extra traffic and buys packing
// workgroups that never wait for one another: every wave walks its own chunks with no
// workgroup barrier after the offsets are known.
#include "cmpz_internal.h"

#include <type_traits>

namespace cmpz {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves   = kThreads / kWave;
static_assert(kPackChunks <= (uint32_t)kWave, "one lane per chunk of a range");

constexpr uint32_t kPastEnd  = kMaxSym;      // symbol value of elements past the end of the tensor (codes to nothing)
constexpr uint32_t kShortMax = 27;           // longest codeword the 32-bit table entries can hold

// LDS written by some lanes of a wave is read by others: the hardware keeps a wave's LDS
// operations in order, this keeps the compiler from moving them across.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// The tensor a chunk range belongs to (uniform: scalar loads from the kernel arguments).
__device__ __forceinline__ uint32_t tensor_of_range(const BatchC &b, uint32_t range)
{
    uint32_t ti = 0;
    for (uint32_t k = 1; k < b.n; ++k) if (range >= b.t[k].pack_base) ti = k;
    return ti;
}

__device__ __forceinline__ void unpack8(const uint4 &v, uint32_t s[8])
{
    s[0] = v.x & 0xffffu; s[1] = v.x >> 16; s[2] = v.y & 0xffffu; s[3] = v.y >> 16;
    s[4] = v.z & 0xffffu; s[5] = v.z >> 16; s[6] = v.w & 0xffffu; s[7] = v.w >> 16;
}

// ---------------------------------------------------------------------------
// Bit counts.  A wave takes whole chunks; per step every lane holds 8 consecutive 16-bit symbols
// or 16 consecutive bytes (one 128-bit load, consecutive lanes consecutive addresses), so a
// sub-block of 32, 64 or 128 codes is a few neighbouring lanes of one DPP row.
// ---------------------------------------------------------------------------
// ZB: container version 2 (sub-blocks of zero residuals have no bits)
template <bool ZB>
__global__ __launch_bounds__(kThreads) void k_lengths(BatchC b)
{
    __shared__ uint32_t lens_s[kMaxSym / 4 + 1];     // code length per symbol, one byte each; symbol kPastEnd: 0
    __shared__ uint32_t bits_s[kPackChunks];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    // The ranges are taken last first: the first sweep wrote the symbols in ascending order, so what
    // it wrote last is what the memory-side cache still holds; and what this pass reads last (the
    // first ranges) is what the packing pass, which runs forwards, reads first.
    const uint32_t range = b.pack_wgs - 1u - blockIdx.x;
    const uint32_t ti = tensor_of_range(b, range);
    const TensorC &tc = b.t[ti];
    const uint32_t c0 = (range - tc.pack_base) * kPackChunks;
    const uint32_t nq = (tc.nchunks - c0 < kPackChunks) ? tc.nchunks - c0 : kPackChunks;
    const uint32_t numel = tc.numel;
    static_assert(kMaxSym / 4 == kThreads, "one word of the length table per thread");
    lens_s[tid] = reinterpret_cast<const uint32_t *>(b.lens + (uint64_t)ti * kMaxSym)[tid];
    if (tid == 0) lens_s[kMaxSym / 4] = 0;
    __syncthreads();
    const uint8_t *L = reinterpret_cast<const uint8_t *>(lens_s);
    const uint16_t *__restrict__ sym = b.sym + (uint64_t)tc.chunk_base * kChunk;
    const Layout lay = make_layout(numel, b.radius, b.sub);
    const OutRef oref = resolve_out(tc);
    const bool fixed_fit = oref.cap >= lay.off_payload;              // room for the sections of fixed size (uniform)
    uint16_t *__restrict__ sub_bits = reinterpret_cast<uint16_t *>(oref.out + lay.off_sub_bits);

    for (uint32_t q = wv; q < nq; q += kWaves) {
        const uint32_t c = c0 + q;
        const uint32_t e0 = c * kChunk;              // first element of the chunk
        const bool full = numel - e0 >= kChunk;
        uint32_t chunk_bits = 0;
        // sub-block bit counts from the lanes' bit counts
        auto emit = [&](uint32_t bits, uint32_t first_sub, uint32_t group) {
            const uint32_t inc = wave_inclusive_sum(bits);
            const uint32_t exc = inc - bits;
            // the first lane of a sub-block sits group-1 lanes below its last lane, in the same DPP row
            const uint32_t first_exc = (group == 16) ? dpp_u32<0x11F, 0xf>(exc) : (group == 8) ? dpp_u32<0x117, 0xf>(exc)
                                     : (group == 4)  ? dpp_u32<0x113, 0xf>(exc) : dpp_u32<0x111, 0xf>(exc);
            if (fixed_fit && ((uint32_t)lane & (group - 1)) == group - 1)
                sub_bits[(uint64_t)c * lay.nsub + first_sub + (uint32_t)lane / group] = (uint16_t)(inc - first_exc);
            chunk_bits += (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
        };
        // the four quarters of the chunk, each with 16-bit symbols (8 per lane and step, two steps, a
        // sub-block is 4, 8 or 16 lanes) or with bytes (16 per lane, one step, a sub-block is 2, 4 or 8
        // lanes); all loads first (the scratch holds whole chunks: always in bounds)
        const uint4 wq = *reinterpret_cast<const uint4 *>(b.wide + (uint64_t)(tc.chunk_base + c) * 4);
        const bool wide[4] = {__builtin_amdgcn_readfirstlane(wq.x) != 0, __builtin_amdgcn_readfirstlane(wq.y) != 0,
                              __builtin_amdgcn_readfirstlane(wq.z) != 0, __builtin_amdgcn_readfirstlane(wq.w) != 0};
        uint4 v[4][2];
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
            const uint16_t *slot = sym + e0 + 1024u * qt;
            if (wide[qt]) {
                v[qt][0] = *reinterpret_cast<const uint4 *>(slot + (uint32_t)lane * 8u);
                v[qt][1] = *reinterpret_cast<const uint4 *>(slot + 512u + (uint32_t)lane * 8u);
            } else {
                v[qt][0] = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint8_t *>(slot) + (uint32_t)lane * 16u);
                v[qt][1] = v[qt][0];
            }
        }
        const uint8_t *Lo = L + b.sym_off;
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
            if (wide[qt]) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    uint32_t s[8];
                    unpack8(v[qt][j], s);
                    if (!full) {
                        const uint32_t i0 = e0 + 1024u * qt + 512u * j + (uint32_t)lane * 8u;
#pragma unroll
                        for (int k = 0; k < 8; ++k) if (i0 + k >= numel) s[k] = kPastEnd;
                    }
                    uint32_t bits = 0;
#pragma unroll
                    for (int k = 0; k < 8; ++k) bits += L[s[k]];
                    if (ZB) {
                        bool az = true;          // nothing but the zero residual (or nothing at all) in this lane
#pragma unroll
                        for (int k = 0; k < 8; ++k) az = az && (s[k] == b.radius || s[k] == kPastEnd);
                        if (group_all(az, (uint32_t)lane, b.sub / 8)) bits = 0;
                    }
                    emit(bits, (1024u * qt + 512u * j) / b.sub, b.sub / 8);
                }
            } else {
                const uint32_t w[4] = {v[qt][0].x, v[qt][0].y, v[qt][0].z, v[qt][0].w};
                const uint32_t i0 = e0 + 1024u * qt + (uint32_t)lane * 16u;
                uint32_t bits = 0;
                bool az = true;
                if (full) {                                  // uniform; every chunk of a tensor but its last
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        const uint32_t byte = (w[k >> 2] >> (8 * (k & 3))) & 0xffu;
                        bits += Lo[byte];
                        if (ZB) az = az && (byte + b.sym_off == b.radius);
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        const uint32_t byte = (w[k >> 2] >> (8 * (k & 3))) & 0xffu;
                        const uint32_t len = Lo[byte];
                        const bool there = i0 + k < numel;
                        bits += there ? len : 0u;
                        az = az && (!there || byte + b.sym_off == b.radius);
                    }
                }
                if (ZB && group_all(az, (uint32_t)lane, b.sub / 16)) bits = 0;
                emit(bits, (1024u * qt) / b.sub, b.sub / 16);
            }
        }
        if (lane == 0) { bits_s[q] = chunk_bits; b.chunk_bits[tc.chunk_base + c] = chunk_bits; }
    }
    __syncthreads();
    if (wv == 0) {
        const uint32_t bits = (lane < (int)nq) ? bits_s[lane] : 0u;
        const uint32_t oc = (lane < (int)nq) ? b.outl_cnt[tc.chunk_base + c0 + lane] : 0u;
        const uint32_t tu = wave_inclusive_sum((bits + 127u) >> 7);
        const uint32_t to = wave_inclusive_sum(oc);
        const uint32_t tb = wave_inclusive_sum(bits);
        if (lane == 63) { b.range_units[range] = tu; b.range_outl[range] = to; b.range_bits[range] = tb; }
    }
}

// ---------------------------------------------------------------------------
// Offsets and header.  One workgroup per tensor turns the ranges' payload units and outlier
// counts into exclusive prefixes (in place), writes the end markers of the two offset tables,
// the zero padding of the outlier sections and the header, and decides whether the container
// fits before any payload is written.
// ---------------------------------------------------------------------------
constexpr int kScanThreads = 1024;

__global__ __launch_bounds__(kScanThreads) void k_scan(BatchC b)
{
    __shared__ uint32_t wave_u[kScanThreads / kWave], wave_o[kScanThreads / kWave];
    __shared__ unsigned long long bits_s;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const uint32_t ti = blockIdx.x;
    const TensorC &tc = b.t[ti];
    const uint32_t nr = (tc.nchunks + kPackChunks - 1) / kPackChunks;
    uint32_t *__restrict__ ru = b.range_units + tc.pack_base;
    uint32_t *__restrict__ ro = b.range_outl + tc.pack_base;
    const uint32_t *__restrict__ rb = b.range_bits + tc.pack_base;
    if (tid == 0) bits_s = 0;
    uint32_t base_u = 0, base_o = 0;
    unsigned long long my_bits = 0;
    for (uint32_t k0 = 0; k0 < nr; k0 += kScanThreads) {            // uniform
        const uint32_t k = k0 + tid;
        const uint32_t u = (k < nr) ? ru[k] : 0u, o = (k < nr) ? ro[k] : 0u;
        if (k < nr) my_bits += rb[k];
        const uint32_t iu = wave_inclusive_sum(u), io = wave_inclusive_sum(o);
        __syncthreads();                                             // the previous round's totals have been read
        if (lane == 63) { wave_u[wv] = iu; wave_o[wv] = io; }
        __syncthreads();
        uint32_t pu = 0, po = 0, tu = 0, to = 0;
#pragma unroll
        for (int w = 0; w < kScanThreads / kWave; ++w) {
            const uint32_t a = wave_u[w], c = wave_o[w];
            if (w < wv) { pu += a; po += c; }
            tu += a; to += c;
        }
        if (k < nr) { ru[k] = base_u + pu + iu - u; ro[k] = base_o + po + io - o; }
        base_u += tu; base_o += to;
    }
    {
        // sum of the ranges' bit counts: 64-bit, one atomic per wave
        const uint32_t lo = wave_inclusive_sum((uint32_t)(my_bits & 0xffffffu));
        const uint32_t mid = wave_inclusive_sum((uint32_t)((my_bits >> 24) & 0xffffffu));
        const uint32_t hi = wave_inclusive_sum((uint32_t)(my_bits >> 48));
        __syncthreads();                                             // bits_s is initialised
        if (lane == 63) atomicAdd(&bits_s, (unsigned long long)lo + ((unsigned long long)mid << 24) + ((unsigned long long)hi << 48));
    }
    __syncthreads();
    if (tid != 0) return;

    const Layout lay = make_layout(tc.numel, b.radius, b.sub);
    TensorMeta &tm = b.tmeta[ti];
    const uint64_t total_units = base_u, n_out = base_o;
    const uint64_t off_outl_idx = lay.off_payload + total_units * 16;
    const uint64_t sect = (4 * n_out + 15) & ~15ull;
    const uint64_t off_outl_val = off_outl_idx + sect;
    const uint64_t total = off_outl_val + sect;
    const OutRef oref = resolve_out(tc);
    const bool fixed_fit = oref.cap >= lay.off_payload;
    const bool fits = total <= oref.cap;
    const uint32_t range_events = tm.range_events;

    // end markers and zero padding of the two offset tables (the fixed sections always fit)
    uint32_t *chunk_off = reinterpret_cast<uint32_t *>(oref.out + lay.off_chunk_off);
    uint32_t *outl_off = reinterpret_cast<uint32_t *>(oref.out + lay.off_outl_off);
    const uint32_t padded = (tc.nchunks + 1 + 3) & ~3u;
    if (fixed_fit) {
        chunk_off[tc.nchunks] = (uint32_t)total_units;
        outl_off[tc.nchunks] = (uint32_t)n_out;
        for (uint32_t k = tc.nchunks + 1; k < padded; ++k) { chunk_off[k] = 0; outl_off[k] = 0; }
    }
    if (fits) {
        // zero padding of both outlier sections
        uint32_t *oidx = reinterpret_cast<uint32_t *>(oref.out + off_outl_idx);
        uint32_t *oval = reinterpret_cast<uint32_t *>(oref.out + off_outl_val);
        for (uint64_t k = n_out; k < ((n_out + 3) & ~3ull); ++k) { oidx[k] = 0; oval[k] = 0; }
    }

    Header hd;
    uint32_t *raw = reinterpret_cast<uint32_t *>(&hd);
    for (uint32_t k = 0; k < kHeaderBytes / 4; ++k) raw[k] = 0;
    hd.magic = kMagic; hd.version = b.zero_blocks ? kVersionZB : kVersion; hd.status = fits ? 0u : kStNoSpace;
    hd.eb_bits = tc.eb_bits;
    for (int k = 0; k < 4; ++k) hd.shape[k] = tc.shape[k];
    hd.numel = tc.numel;
    hd.radius = b.radius; hd.chunk = kChunk; hd.sub = b.sub; hd.guard_shift = b.guard_shift;
    hd.nchunks = tc.nchunks; hd.n_outliers = (uint32_t)n_out;
    hd.range_events = range_events; hd.max_len = tc.numel ? tm.max_len : 0u;
    hd.total_bits = bits_s;
    hd.off_lens = lay.off_lens; hd.off_chunk_off = lay.off_chunk_off;
    hd.off_outl_off = lay.off_outl_off; hd.off_sub_bits = lay.off_sub_bits;
    hd.off_payload = lay.off_payload; hd.off_outl_idx = off_outl_idx;
    hd.off_outl_val = off_outl_val; hd.total_size = total;
    uint32_t *dst = reinterpret_cast<uint32_t *>(oref.out);
    if (fixed_fit) for (uint32_t k = 0; k < kHeaderBytes / 4; ++k) dst[k] = raw[k];

    uint32_t st = 0;
    if (!fits) st |= kStNoSpace;
    if (range_events) st |= kStRange;
    if (st) atomicOr(b.status, st);
    tm.skip = fits ? 0u : 1u;
    tm.n_outliers = (uint32_t)n_out;
    tm.total_units = (uint32_t)total_units;
    tm.total_bits = bits_s;
    tm.total_size = total;
    tm.range_events = 0;                             // ready for the next call
}

// ---------------------------------------------------------------------------
// Packing.  A wave packs a chunk in steps of 1024 codes (16 per lane; 512 and 8 when codewords
// may exceed 27 bits): the lanes' bit offsets come from a wave scan of their code lengths, every
// codeword is OR-ed into the wave's zeroed LDS image at its own position (bit k of the chunk is bit
// 31-(k%32) of little-endian word k/32), the 16-byte units that are complete go out with 128-bit
// stores, and the unit that is still open moves to the front of the image for the next step.
// ---------------------------------------------------------------------------
constexpr uint32_t kStepBitsMax = 1024 * kShortMax;                    // = 27648 >= 512 * kMaxCodeLen
static_assert(512 * kMaxCodeLen <= kStepBitsMax, "image size");
constexpr uint32_t kImageUnits = kStepBitsMax / 128 + 2;               // the open unit in front, one of slack behind
constexpr uint32_t kImageWords = kImageUnits * 4;

template <bool ZB>
__global__ __launch_bounds__(kThreads, ZB ? 5 : 6) void k_pack(BatchC b)
{
    __shared__ uint64_t table[kMaxSym + 1];          // length << 56 | code; or, as 32-bit words, code << (32 - length) | length
    __shared__ __align__(16) uint32_t images[kWaves][kImageWords];
    __shared__ uint32_t coff_s[kPackChunks], ooff_s[kPackChunks + 1], bits_s[kPackChunks];
    __shared__ uint16_t olists[kWaves][kWave];       // per wave: where in a step the outliers of one pass sit
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t ti = tensor_of_range(b, blockIdx.x);
    const TensorC &tc = b.t[ti];
    const TensorMeta &tm = b.tmeta[ti];
    if (tm.skip) return;                             // uniform: the container does not fit, its header says so
    const uint32_t c0 = (blockIdx.x - tc.pack_base) * kPackChunks;
    const uint32_t nq = (tc.nchunks - c0 < kPackChunks) ? tc.nchunks - c0 : kPackChunks;
    const uint32_t numel = tc.numel;
    const bool short_codes = tm.max_len <= kShortMax;                // uniform
    const Layout lay = make_layout(numel, b.radius, b.sub);
    uint8_t *const out = resolve_out(tc).out;

    uint32_t *table32 = reinterpret_cast<uint32_t *>(table);
    if (short_codes) {
        const uint32_t *src = b.enc32 + (uint64_t)ti * kMaxSym;
        for (int k = tid; k <= (int)kMaxSym; k += kThreads) table32[k] = (k < (int)kMaxSym) ? src[k] : 0u;
    } else {
        const uint64_t *src = b.codes + (uint64_t)ti * kMaxSym;
        for (int k = tid; k <= (int)kMaxSym; k += kThreads) table[k] = (k < (int)kMaxSym) ? src[k] : 0ull;
    }
    uint32_t *img = images[wv];
    uint16_t *olist = olists[wv];
    for (uint32_t k = lane; k < kImageUnits; k += kWave) reinterpret_cast<uint4 *>(img)[k] = make_uint4(0, 0, 0, 0);

    // where the range's chunks and their outlier records start
    if (wv == 0) {
        const uint32_t g = tc.chunk_base + c0 + lane;
        const uint32_t bits = (lane < (int)nq) ? b.chunk_bits[g] : 0u;
        const uint32_t oc = (lane < (int)nq) ? b.outl_cnt[g] : 0u;
        const uint32_t units = (bits + 127u) >> 7;
        const uint32_t cu = b.range_units[blockIdx.x] + wave_inclusive_sum(units) - units;
        const uint32_t co = b.range_outl[blockIdx.x] + wave_inclusive_sum(oc) - oc;
        if (lane < (int)nq) {
            reinterpret_cast<uint32_t *>(out + lay.off_chunk_off)[c0 + lane] = cu;
            reinterpret_cast<uint32_t *>(out + lay.off_outl_off)[c0 + lane] = co;
            coff_s[lane] = cu; bits_s[lane] = bits;
        }
        if (lane <= (int)nq && lane <= (int)kPackChunks) ooff_s[lane] = co;      // lane nq: the end of the last chunk's records
    }
    __syncthreads();
    // ---- from here on the waves are on their own ----

    const uint16_t *__restrict__ sym = b.sym + (uint64_t)tc.chunk_base * kChunk;
    const float *__restrict__ x = tc.x;
    const uint32_t W = tc.shape[3], HW = tc.shape[2] * W;
    uint4 *__restrict__ payload = reinterpret_cast<uint4 *>(out + lay.off_payload);
    const uint64_t off_outl_idx = lay.off_payload + (uint64_t)tm.total_units * 16;
    uint32_t *__restrict__ oidx = reinterpret_cast<uint32_t *>(out + off_outl_idx);
    int32_t *__restrict__ oval = reinterpret_cast<int32_t *>(out + off_outl_idx + ((4ull * tm.n_outliers + 15) & ~15ull));
    bool failed = false;

    for (uint32_t q = wv; q < nq; q += kWaves) {
        const uint32_t c = c0 + q;
        const uint32_t e0 = c * kChunk;
        const bool full = numel - e0 >= kChunk;
        const uint32_t chunk_units = (bits_s[q] + 127u) >> 7;
        uint4 *__restrict__ dst = payload + coff_s[q];
        uint32_t orank = ooff_s[q];
        const bool has_outl = ooff_s[q + 1] != orank;                // uniform
        uint32_t bitpos = 0;                         // bits of the chunk packed so far
        uint32_t ubase = 0;                          // units of the chunk stored so far: image unit 0 is stream unit ubase

        // one step: the lane's n consecutive symbols s[] starting at element i0.  narrow: s[] holds the
        // bytes of a quarter stored with 8 bits per symbol, i.e. symbol - sym_off (no outlier among them)
        auto step = [&](const uint32_t *s, auto n_c, auto narrow_c, uint32_t i0, bool last) {
            constexpr int n = decltype(n_c)::value;
            constexpr bool narrow = decltype(narrow_c)::value;
            const uint32_t zero_sym = narrow ? b.radius - b.sym_off : b.radius;    // the zero residual, as s[] has it
            const uint32_t past_sym = narrow ? kPastEnd - b.sym_off : kPastEnd;    // elements past the end of the tensor
            const uint32_t *tab = narrow ? table32 + b.sym_off : table32;
            // outlier records: rank the zero symbols of the step; then one lane per outlier recomputes
            // its residual from x, so that the loads of all of them are in flight together
            if (!narrow && has_outl) {
                uint32_t mine = 0;
                _Pragma("unroll") for (int k = 0; k < n; ++k) mine += (s[k] == 0u) ? 1u : 0u;
                const uint32_t inc = wave_inclusive_sum(mine);
                const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
                const uint32_t step0 = i0 - (uint32_t)lane * (uint32_t)n;          // first element of the step
                for (uint32_t r0 = 0; r0 < total; r0 += kWave) {                 // uniform; one pass unless outliers crowd
                    uint32_t rk = inc - mine - r0;                               // place of the lane's next outlier in this pass
                    _Pragma("unroll") for (int k = 0; k < n; ++k) {
                        if (s[k] == 0u) {
                            if (rk < (uint32_t)kWave) olist[rk] = (uint16_t)(lane * n + k);
                            ++rk;
                        }
                    }
                    wave_sync();
                    const uint32_t me = r0 + (uint32_t)lane;
                    if (me < total) {
                        const uint32_t i = step0 + olist[lane];
                        const uint32_t p = tc.divHW.div(i);
                        const uint32_t rem = i - p * HW;
                        const uint32_t h = tc.divW.div(rem), w = rem - h * W;
                        const uint32_t at = orank + me;
                        if (at < tm.n_outliers) {
                            oidx[at] = i;
                            oval[at] = delta_from_x(x, i, h, w, W, tc.r);
                        }
                    }
                    wave_sync();
                }
                orank += total;
            }
            // version 2: a sub-block of zero residuals (n symbols per lane: sub / n lanes) has no bits
            bool coded = true;
            if (ZB) {
                bool az = true;
                _Pragma("unroll") for (int k = 0; k < n; ++k) az = az && (s[k] == zero_sym || s[k] == past_sym);
                coded = !group_all(az, (uint32_t)lane, b.sub / (uint32_t)n);
            }
            // bit offsets of the lanes; in the short-code case the table entries stay in registers for the packing
            uint32_t bits = 0;
            uint32_t e[n];
            if (short_codes) { _Pragma("unroll") for (int k = 0; k < n; ++k) { e[k] = coded ? tab[s[k]] : 0u; bits += e[k] & 31u; } }
            else             { _Pragma("unroll") for (int k = 0; k < n; ++k) bits += coded ? (uint32_t)(table[s[k]] >> 56) : 0u; }
            const uint32_t inc = wave_inclusive_sum(bits);
            uint32_t pos = bitpos - ubase * 128u + inc - bits;        // bit position in the image
            if (short_codes) {
                // Codewords go into the image in groups: two of them (at most 54 bits together) merged
                // in registers cost three LDS atomics, and so do four when they fit 64 bits, which they
                // nearly always do (uniform test over the wave; otherwise two by two).
                uint32_t longest = 0;
                _Pragma("unroll") for (int k = 0; k < n; k += 4) {
                    const uint32_t tot = (e[k] & 31u) + (e[k + 1] & 31u) + (e[k + 2] & 31u) + (e[k + 3] & 31u);
                    longest = tot > longest ? tot : longest;
                }
                auto pair_of = [](uint32_t ea, uint32_t eb, uint32_t &hi, uint32_t &lo, uint32_t &len) {
                    const uint32_t ca = ea & ~31u, la = ea & 31u;                   // left-aligned codes
                    const uint64_t second = (((uint64_t)(eb & ~31u)) << 32) >> la;
                    hi = ca | (uint32_t)(second >> 32); lo = (uint32_t)second; len = la + (eb & 31u);
                };
                auto put = [&](uint32_t hi, uint32_t lo) {
                    const uint32_t o = pos & 31u;
                    uint32_t *w = img + (pos >> 5);
                    atomicOr(w, hi >> o);
                    atomicOr(w + 1, __builtin_amdgcn_alignbit(hi, lo, o));
                    atomicOr(w + 2, __builtin_amdgcn_alignbit(lo, 0u, o));           // the part that spills over
                };
                if (!__any(longest > 64u)) {
                    _Pragma("unroll") for (int k = 0; k < n; k += 4) {
                        uint32_t h0, l0, n0, h1, l1, n1;
                        pair_of(e[k], e[k + 1], h0, l0, n0);
                        pair_of(e[k + 2], e[k + 3], h1, l1, n1);
                        const uint64_t quad = (((uint64_t)h0 << 32) | l0) | ((((uint64_t)h1 << 32) | l1) >> n0);   // n0 <= 54
                        put((uint32_t)(quad >> 32), (uint32_t)quad);
                        pos += n0 + n1;
                    }
                } else {
                    _Pragma("unroll") for (int k = 0; k < n; k += 2) {
                        uint32_t h0, l0, n0;
                        pair_of(e[k], e[k + 1], h0, l0, n0);
                        put(h0, l0);
                        pos += n0;
                    }
                }
            } else {
                _Pragma("unroll") for (int k = 0; k < n; ++k) {
                    const uint64_t cw = coded ? table[s[k]] : 0ull;
                    const uint32_t len = (uint32_t)(cw >> 56);
                    if (len) {
                        const uint64_t place = (cw & 0x00ffffffffffffffull) << (64u - len);   // left-aligned in 64 bits
                        const uint32_t hi = (uint32_t)(place >> 32), lo = (uint32_t)place, o = pos & 31u;
                        uint32_t *w = img + (pos >> 5);
                        atomicOr(w, hi >> o);
                        atomicOr(w + 1, __builtin_amdgcn_alignbit(hi, lo, o));
                        atomicOr(w + 2, __builtin_amdgcn_alignbit(lo, 0u, o));
                        pos += len;
                    }
                }
            }
            bitpos += (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
            wave_sync();
            // complete units go out; at the end of the chunk also the open one (zero padded)
            uint32_t done = last ? chunk_units : (bitpos >> 7);
            if (done > chunk_units) { done = chunk_units; failed = true; }   // never past the chunk's own units
            const uint32_t nu = done - ubase;
            const bool carry = !last && (bitpos & 127u) != 0;        // uniform
            uint4 open = make_uint4(0, 0, 0, 0);
            if (nu < kImageUnits) {
                for (uint32_t k = lane; k < nu; k += kWave) dst[ubase + k] = reinterpret_cast<const uint4 *>(img)[k];
                if (carry && lane == 0) open = reinterpret_cast<const uint4 *>(img)[nu];
            } else {
                failed = true;                       // cannot happen: a step never holds more than the image
            }
            wave_sync();
            const uint32_t dirty = (nu + 1 < kImageUnits) ? nu + 1 : kImageUnits;
            for (uint32_t k = lane; k < dirty; k += kWave) reinterpret_cast<uint4 *>(img)[k] = make_uint4(0, 0, 0, 0);
            wave_sync();
            if (carry && lane == 0) reinterpret_cast<uint4 *>(img)[0] = open;
            wave_sync();
            ubase = done;
        };

        // per quarter of the chunk: 16-bit symbols, else bytes (uniform)
        const uint4 wq = *reinterpret_cast<const uint4 *>(b.wide + (uint64_t)(tc.chunk_base + c) * 4);
        const uint32_t wide_mask = (__builtin_amdgcn_readfirstlane(wq.x) ? 1u : 0u) | (__builtin_amdgcn_readfirstlane(wq.y) ? 2u : 0u) |
                                   (__builtin_amdgcn_readfirstlane(wq.z) ? 4u : 0u) | (__builtin_amdgcn_readfirstlane(wq.w) ? 8u : 0u);
        const uint8_t *__restrict__ sb = reinterpret_cast<const uint8_t *>(sym + e0);
        auto unpack_bytes = [&](uint32_t w, uint32_t *s4) {
            s4[0] = (w & 0xffu) + b.sym_off; s4[1] = ((w >> 8) & 0xffu) + b.sym_off;
            s4[2] = ((w >> 16) & 0xffu) + b.sym_off; s4[3] = (w >> 24) + b.sym_off;
        };
        if (short_codes) {
            // 16 symbols per lane and step, the next step's symbols in flight.  A step is a quarter of the
            // chunk (2048 bytes apart): a lane's 16 symbols are 32 bytes of a wide quarter, 16 of a narrow
            // one (the second load then repeats the first)
            auto fetch = [&](uint32_t qt, uint4 &a, uint4 &c2) {
                const bool wd = (wide_mask >> qt) & 1u;
                const uint8_t *p = sb + 2048u * qt + (((uint32_t)lane * 16u) << (wd ? 1 : 0));
                a = *reinterpret_cast<const uint4 *>(p);
                c2 = *reinterpret_cast<const uint4 *>(p + (wd ? 16u : 0u));
            };
            uint4 lo, hi;
            fetch(0, lo, hi);
#pragma unroll 1
            for (uint32_t it = 0; it < 4; ++it) {
                const uint32_t i0 = e0 + it * 1024u + (uint32_t)lane * 16u;
                const bool wide = (wide_mask >> it) & 1u;
                uint4 nlo, nhi;
                fetch(it < 3 ? it + 1 : it, nlo, nhi);                    // the last step fetches its own symbols again
                uint32_t s[16];
                if (wide) {
                    unpack8(lo, s); unpack8(hi, s + 8);
                    if (!full) {
#pragma unroll
                        for (int k = 0; k < 16; ++k) if (i0 + k >= numel) s[k] = kPastEnd;
                    }
                    step(s, std::integral_constant<int, 16>{}, std::false_type{}, i0, it == 3);
                } else {
                    const uint32_t w4[4] = {lo.x, lo.y, lo.z, lo.w};
#pragma unroll
                    for (int k = 0; k < 16; ++k) s[k] = (w4[k >> 2] >> (8 * (k & 3))) & 0xffu;
                    if (!full) {
#pragma unroll
                        for (int k = 0; k < 16; ++k) if (i0 + k >= numel) s[k] = kPastEnd - b.sym_off;
                    }
                    step(s, std::integral_constant<int, 16>{}, std::true_type{}, i0, it == 3);
                }
                lo = nlo; hi = nhi;
            }
        } else {
#pragma unroll 1
            for (uint32_t it = 0; it < 8; ++it) {
                const uint32_t i0 = e0 + it * 512u + (uint32_t)lane * 8u;
                uint32_t s[8];
                if ((wide_mask >> (it >> 1)) & 1u) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(sym + i0);
                    unpack8(v, s);
                } else {
                    // quarter it/2, its first or second 512 bytes
                    const uint2 v = *reinterpret_cast<const uint2 *>(sb + 2048u * (it >> 1) + 512u * (it & 1u) + (uint32_t)lane * 8u);
                    unpack_bytes(v.x, s); unpack_bytes(v.y, s + 4);
                }
                if (!full) {
#pragma unroll
                    for (int k = 0; k < 8; ++k) if (i0 + k >= numel) s[k] = kPastEnd;
                }
                step(s, std::integral_constant<int, 8>{}, std::false_type{}, i0, it == 7);
            }
        }
        if (bitpos != bits_s[q]) failed = true;      // the two passes disagree: cannot happen
    }
    if (failed && lane == 0) atomicOr(b.status, kStInternal);
}

// What the first sweep accumulates for the tensors of a group, back to zero (a compress that was
// begun and cannot be finished, or scratch of unknown content).
__global__ __launch_bounds__(kThreads) void k_clear(BatchC b)
{
    const uint32_t ti = blockIdx.x;
    uint32_t *h = b.hist + (uint64_t)ti * kHistCopies * kMaxSym;
    for (uint32_t k = threadIdx.x; k < kHistCopies * kMaxSym; k += kThreads) h[k] = 0;
    if (threadIdx.x == 0) b.tmeta[ti].range_events = 0;
}

// Quarter chunks stored with 8 bits per symbol, rewritten in place with 16 (for inspection of the
// symbols).  One workgroup of 64 threads per quarter.
__global__ __launch_bounds__(64) void k_widen(uint16_t *sym, uint32_t *wide, uint32_t sym_off)
{
    const uint32_t qd = blockIdx.x, lane = threadIdx.x;
    if (wide[qd]) return;                            // uniform
    uint16_t *slot = sym + (uint64_t)qd * 1024u;
    const uint4 v = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint8_t *>(slot) + 16u * lane);
    __syncthreads();                                 // every byte is read before the slot is overwritten
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const uint32_t a = ((w[k >> 1] >> (16 * (k & 1))) & 0xffu) + sym_off;
        const uint32_t b2 = ((w[k >> 1] >> (16 * (k & 1) + 8)) & 0xffu) + sym_off;
        o[k] = a | (b2 << 16);
    }
    *reinterpret_cast<uint4 *>(slot + 16u * lane) = make_uint4(o[0], o[1], o[2], o[3]);
    *reinterpret_cast<uint4 *>(slot + 16u * lane + 8u) = make_uint4(o[4], o[5], o[6], o[7]);
    __syncthreads();
    if (lane == 0) wide[qd] = 1;
}

// ---- the stack of containers (one thread each: a few words of bookkeeping) ----
__global__ void k_arena_init(ArenaState *st, uint32_t slots)
{
    st->top = 0; st->peak = 0; st->nslots = 0; st->failed = 0; st->slots_cap = slots; st->pad = 0;
    for (uint32_t k = 0; k < slots; ++k) { st->slot[k].offset = 0; st->slot[k].size = 0; }
}

// After the kernels of a push: the container is complete, record it and move the top past it.
__global__ void k_arena_pushed(BatchC b, ArenaState *st, uint32_t slot)
{
    const TensorMeta &tm = b.tmeta[0];
    if (slot >= st->slots_cap) { st->failed += 1; return; }
    if (tm.skip) {                                   // it did not fit: the slot stays empty
        st->slot[slot].offset = st->top; st->slot[slot].size = 0;
        st->failed += 1;
    } else {
        st->slot[slot].offset = st->top; st->slot[slot].size = tm.total_size;
        st->top += (tm.total_size + kArenaAlign - 1) / kArenaAlign * kArenaAlign;
        if (st->top > st->peak) st->peak = st->top;
    }
    if (slot + 1 > st->nslots) st->nslots = slot + 1;
}

// A container is no longer needed.  Space comes back when the slots above it are free too.
__global__ void k_arena_release(ArenaState *st, uint32_t slot)
{
    if (slot >= st->slots_cap) return;
    st->slot[slot].size = 0;
    uint32_t n = st->nslots;
    while (n > 0 && st->slot[n - 1].size == 0) { --n; st->top = st->slot[n].offset; }
    st->nslots = n;
}

}  // namespace

void launch_arena_init(ArenaState *st_dev, uint32_t slots, hipStream_t st)
{
    hipLaunchKernelGGL(k_arena_init, dim3(1), dim3(1), 0, st, st_dev, slots);
}
void launch_arena_pushed(const BatchC &b, ArenaState *st_dev, uint32_t slot, hipStream_t st)
{
    hipLaunchKernelGGL(k_arena_pushed, dim3(1), dim3(1), 0, st, b, st_dev, slot);
}
void launch_arena_release(ArenaState *st_dev, uint32_t slot, hipStream_t st)
{
    hipLaunchKernelGGL(k_arena_release, dim3(1), dim3(1), 0, st, st_dev, slot);
}

void launch_widen(uint16_t *sym, uint32_t *wide, uint32_t sym_off, uint32_t nchunks, hipStream_t st)
{
    if (nchunks) hipLaunchKernelGGL(k_widen, dim3(4 * nchunks), dim3(64), 0, st, sym, wide, sym_off);
}

void launch_clear(const BatchC &b, Profiler *prof, hipStream_t st)
{
    if (b.n) launch(prof, kKClear, k_clear, dim3(b.n), dim3(kThreads), st, b);
}

// Bit counts, offsets and header, packing: three launches over all tensors of the group.
void launch_pack(const BatchC &b, Profiler *prof, hipStream_t st)
{
    if (b.pack_wgs) {
        if (b.zero_blocks) launch(prof, kKLengths, k_lengths<true>, dim3(b.pack_wgs), dim3(kThreads), st, b);
        else launch(prof, kKLengths, k_lengths<false>, dim3(b.pack_wgs), dim3(kThreads), st, b);
    }
    launch(prof, kKScan, k_scan, dim3(b.n), dim3(kScanThreads), st, b);
    if (b.pack_wgs) {
        if (b.zero_blocks) launch(prof, kKPack, k_pack<true>, dim3(b.pack_wgs), dim3(kThreads), st, b);
        else launch(prof, kKPack, k_pack<false>, dim3(b.pack_wgs), dim3(kThreads), st, b);
    }
}

}  // namespace cmpz
