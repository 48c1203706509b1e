// Fused decompression: chunked Huffman decode -> outlier patch -> reverse Lorenzo
// (row and column prefix sums) -> de-quantisation, one pass, residuals never
// leave the CU.  HBM traffic is the container read plus the 4-byte result write.
//
// The unit of work is a band: whole rows of one plane, or several whole small
// planes, at most 2048 elements.  Every WAVE owns its bands and its own slice
// of LDS and walks through them on its own: after the decode tables are built
// there is no workgroup barrier, so while one wave of a CU decodes (LDS and
// ALU latency), another runs its column pass (stores) and a third waits for
// its next payload.  The four waves of a workgroup share only the tables.
// Planes larger than a band are walked band by band with running column sums
// (needs W <= 256); where a tensor has few such planes, a variant of the kernel
// gives a plane to a workgroup, whose waves decode four bands side by side and
// share the column pass by columns.  Shapes that fit neither case take the
// unfused kernels of cmpz_decompress.hip.
//
// A band is decoded by one lane per sub-block (the container stores each
// sub-block's bit count, so every lane knows where its codes start) into an LDS
// array of int16 (all sums are taken modulo 2^16: the final integers lie within
// +-16384, so the low 16 bits, sign-extended, are the result whatever the
// intermediate sums and the outlier residuals reach).  The band's stretch of the payload is contiguous in the
// container; it is copied into LDS with 128-bit loads first, and the lanes read
// their codewords from there at arbitrary bit positions (a band whose payload
// exceeds the staging buffer, more than 8 bits per code on average, is decoded
// straight from memory instead).  In a band without outliers a lane adds up its
// residuals along the row while it decodes them, so what it stores is already the
// row prefix sum up to a per-lane carry; one segmented scan over the lanes'
// totals yields the carries, and the column pass (one lane per column, four
// rows in flight) adds them on the fly, de-quantises and stores.  A band with
// outliers stores plain residuals and patches the outliers in; then its lanes
// sum their rows in LDS, and the rest is the same.
// Software pipeline: the bit counts of the next band are fetched during the
// decode of the current one, and its payload during the column pass.
#include "cmpz_decode_core.h"

#include <type_traits>

namespace cmpz {
namespace {

constexpr int kThreads    = 256;
constexpr int kWaves      = kThreads / kWave;
constexpr int kBandMax    = 2048;                 // elements decoded per band at most
constexpr int kStageWords = 512;                  // staged payload per band: 2 KB, i.e. 8 bits per code of a full band
constexpr int kColGroups  = 4;                    // 64-column groups of a big plane (W <= 256)

template <int SUB> struct Cfg;
template <> struct Cfg<128> { static constexpr int kLog = 7; };
template <> struct Cfg<64>  { static constexpr int kLog = 6; };
template <> struct Cfg<32>  { static constexpr int kLog = 5; };

struct FusedPlan {
    uint32_t big;          // 0: groups of whole planes; 1: one plane per item, bands of rows; 2: the same,
                           // the four waves of a workgroup on four consecutive bands of one plane
    uint32_t G;            // planes per group (big == 0)
    uint32_t Rb;           // rows per band (big == 1)
    uint32_t nitems;
    FastDiv  divW;
};

// LDS written by some lanes of a wave is read by others: the hardware keeps a wave's LDS
// operations in order, this keeps the compiler from moving them across.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

struct Band {
    uint32_t e0, n, rows, plane0, npl, row0;
    bool valid;
};

// The stretch of the payload a band's lanes read.
struct Stage {
    uint32_t q0;           // first 16-byte unit staged
    uint32_t nq;           // units staged; 0 = not staged (the band decodes from memory)
};

// One launch decodes all tensors of a call: a workgroup belongs to one tensor (it validates that
// container and builds that codebook's decode tables for itself, about a microsecond), its waves
// take every item_stride-th item of the tensor.
// COOP: the variant for few large planes (plan value big == 2), a launch of its own.
template <int SUB, bool COOP>
__global__ __launch_bounds__(kThreads, 5) void k_decode_fused(BatchD b)
{
    using RT = int16_t;
    constexpr int kRows = 4;                              // rows of the column pass in flight together
    constexpr int kLog  = Cfg<SUB>::kLog;
    constexpr int kND   = kBandMax / SUB;                 // decode lanes per band
    constexpr int kNSub = (int)kChunk / SUB;              // sub-blocks per chunk
    constexpr int kPre  = kNSub + kND;                    // bit-count entries looked at per band
    constexpr int kE    = (kPre + kWave - 1) / kWave;     // of which each lane fetches kE consecutive ones
    static_assert(2 * kND <= kStageWords, "the lane records live in the staging buffer");
    static_assert(kStageWords / 4 == 2 * kWave, "two units per lane");

    // One struct, so that the order in LDS is fixed: the words a damaged stream may read past a
    // wave's staged payload (stage_tail_words) are the next wave's, and behind the last wave's
    // lie the tables.  32 KB at most: five workgroups share a compute unit's LDS.
    struct Lds {
        RT Rs[kWaves][kBandMax + kND];                    // one pad slot per sub-block: lane-conflict free
        alignas(16) uint32_t Ss[kStagePad + kWaves * kStageWords];   // per wave: staged payload; after the decode, the lane records
        DecodeTables T;
    };
    __shared__ Lds lds;
    static_assert(sizeof(Lds) <= 32 * 1024, "five workgroups per compute unit");
    static_assert(sizeof(lds.Rs) >= 13 * 1024, "the table build borrows Rs as scratch");
    static_assert(sizeof(DecodeTables) >= 4 * stage_tail_words(SUB), "reads past the last wave's payload stay inside the tables");
    DecodeTables &T = lds.T;
    // the exclusive prefix of a band's sub-block bit counts lives in the staging buffer too, behind
    // the lane records: it is written after a band's decode and read (into registers) before the
    // next band's payload is stored over it; a wave's LDS operations stay in order
    constexpr int kPOff = kStagePad + 2 * kND;
    static_assert(kPOff + kE * kWave + 2 <= kStagePad + kStageWords, "lane records and prefix fit the staging buffer");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);     // tells the compiler that it is uniform in the wave
    // the tensor of this workgroup (uniform: scalar loads from the kernel arguments)
    uint32_t ti = 0;
    for (uint32_t k = 1; k < b.n; ++k) if (blockIdx.x >= b.t[k].wg_base) ti = k;
    const TensorD &td = b.t[ti];
    const DecompressArgs a = decompress_args(b, td);
    FusedPlan pl;
    pl.big = td.big; pl.G = td.G; pl.Rb = td.Rb; pl.nitems = td.nitems; pl.divW = td.divW;
    // a container on the device-side stack: an empty slot, or one too short for the sections of fixed
    // size, is not looked at (the host has checked this for containers it knows the size of)
    if (td.slot && a.size < a.lay.off_payload) {
        if (blockIdx.x == td.wg_base && tid == 0) atomicOr(a.status, kStFormat);
        return;
    }
    // every workgroup validates the container and builds the decode tables for itself
    {
        const uint32_t defect = build_tables<kThreads>(T, a, reinterpret_cast<uint32_t *>(&lds.Rs[0][0]));
        if (defect) {
            if (blockIdx.x == td.wg_base && tid == 0) atomicOr(a.status, defect);
            return;
        }
    }
    // ---- from here on the waves are on their own ----
    RT       *R = lds.Rs[wv];
    uint32_t *S = lds.Ss + wv * kStageWords;             // the wave's payload starts at S + kStagePad
    uint32_t *P = S + kPOff;
    // per decode lane, after the decode: .x = offset of the lane's first row start (elements before
    // it lack the carry), .y = the carry
    uint2 *RC = reinterpret_cast<uint2 *>(S + kStagePad);
    const uint32_t payload_units = T.payload_units, n_outl = T.n_outliers;

    const uint32_t W = a.W, H = a.H, HW = a.HW;
    const uint32_t *__restrict__ chunk_off = reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_chunk_off);
    const uint32_t *__restrict__ outl_off = reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_outl_off);
    const uint16_t *__restrict__ sub_bits = reinterpret_cast<const uint16_t *>(a.buf + a.lay.off_sub_bits);
    const Header *hd = reinterpret_cast<const Header *>(a.buf);
    const uint32_t *__restrict__ oidx = reinterpret_cast<const uint32_t *>(a.buf + hd->off_outl_idx);
    const int32_t *__restrict__ oval = reinterpret_cast<const int32_t *>(a.buf + hd->off_outl_val);
    const uint4 *__restrict__ payload4 = reinterpret_cast<const uint4 *>(a.buf + a.lay.off_payload);
    const float s = a.s;
    bool bad = false;

    // What a lane fetches ahead for a band: its bit-count entries, its sub-block's chunk bounds
    // (those of the first and the last lane are the payload bounds of the band's chunks), and, in
    // lanes 0 and 1, the two ends of the band's range in the outlier list.
    struct Ahead {
        uint32_t v[kE], uu0, uu1, oo;
    };

    auto band_of = [&](uint32_t item, uint32_t b) -> Band {
        Band g;
        g.valid = item < pl.nitems && (!pl.big || b * pl.Rb < H);
        if (!g.valid) { g.e0 = g.n = g.rows = g.plane0 = g.npl = g.row0 = 0; return g; }
        if (pl.big) {
            g.plane0 = item; g.npl = 1; g.row0 = b * pl.Rb;
            g.rows = (H - g.row0 < pl.Rb) ? H - g.row0 : pl.Rb;
        } else {
            g.plane0 = item * pl.G; g.row0 = 0;
            g.npl = (a.planes - g.plane0 < pl.G) ? a.planes - g.plane0 : pl.G;
            g.rows = g.npl * H;
        }
        g.e0 = g.plane0 * HW + g.row0 * W;
        g.n = g.rows * W;
        return g;
    };
    auto fetch = [&](const Band &g) -> Ahead {
        Ahead f;
#pragma unroll
        for (int i = 0; i < kE; ++i) f.v[i] = 0;
        f.uu0 = f.uu1 = f.oo = 0;
        if (!g.valid) return f;
        const uint32_t sb0 = g.e0 >> kLog, sb1 = (g.e0 + g.n - 1) >> kLog;
        const uint32_t j0 = sb0 & (kNSub - 1), ent0 = sb0 - j0, nent = j0 + (sb1 - sb0 + 1);
#pragma unroll
        for (int i = 0; i < kE; ++i) {
            const uint32_t e = (uint32_t)kE * lane + i;
            if (e < nent) f.v[i] = sub_bits[(uint64_t)ent0 + e];
        }
        if (sb0 + lane <= sb1) {
            const uint32_t c = (sb0 + lane) / kNSub;
            f.uu0 = chunk_off[c]; f.uu1 = chunk_off[c + 1];
        }
        // uniform values, but fetched with a vector load: scalar loads share their counter with LDS
        // traffic and return out of order, so waiting for one would drain every LDS access in flight
        if (lane < 2) f.oo = outl_off[lane == 0 ? g.e0 / kChunk : (g.e0 + g.n - 1) / kChunk + 1];
        return f;
    };
    // exclusive prefix of a band's bit counts from the start of its first chunk
    auto prefix_bits = [&](const Ahead &f) {
        uint32_t loc = 0;
#pragma unroll
        for (int i = 0; i < kE; ++i) loc += f.v[i];
        const uint32_t inc = wave_inclusive_sum(loc);
        uint32_t ex = inc - loc;
#pragma unroll
        for (int i = 0; i < kE; ++i) { P[kE * lane + i] = ex; ex += f.v[i]; }
        if (lane == 63) P[kE * kWave] = inc;
        wave_sync();
    };
    // the band's stretch of the payload (uniform; needs P): from the word where its first
    // sub-block starts, rounded down to a unit, to the word where its last sub-block ends
    auto stage_of = [&](const Band &g, const Ahead &f) -> Stage {
        Stage st = {0, 0};
        if (!g.valid) return st;
        const uint32_t sb0 = g.e0 >> kLog, sb1 = (g.e0 + g.n - 1) >> kLog;
        const uint32_t j0 = sb0 & (kNSub - 1), jl = sb1 & (kNSub - 1), idxl = j0 + (sb1 - sb0);
        const uint32_t first_bit = P[j0] - P[0];                 // in the first chunk's stream
        const uint32_t end_bit = P[idxl + 1] - P[idxl - jl];     // in the last chunk's stream
        // the band's first sub-block is lane 0's, its last one lane (sb1 - sb0)'s
        const uint32_t cf = __builtin_amdgcn_readfirstlane(f.uu0);
        const uint32_t cl = (uint32_t)__builtin_amdgcn_readlane((int)f.uu0, (int)(sb1 - sb0)),
                       cl1 = (uint32_t)__builtin_amdgcn_readlane((int)f.uu1, (int)(sb1 - sb0));
        if (!(cf <= cl && cl <= cl1 && cl1 <= payload_units)) return st;
        const uint64_t w_lo = (uint64_t)cf * 4 + (first_bit >> 5);
        const uint64_t w_hi = (uint64_t)cl * 4 + ((uint64_t)end_bit + 31) / 32;
        if (w_hi > (uint64_t)cl1 * 4 || w_hi <= w_lo) return st;
        const uint64_t q0 = w_lo >> 2, q1 = (w_hi + 3) >> 2;
        if (q1 - q0 > (uint64_t)(kStageWords / 4)) return st;
        st.q0 = (uint32_t)q0; st.nq = (uint32_t)(q1 - q0);
        return st;
    };
    auto stage_load = [&](const Stage &st, uint4 &s0, uint4 &s1) {
        if ((uint32_t)lane < st.nq) s0 = payload4[(uint64_t)st.q0 + lane];
        if ((uint32_t)lane + kWave < st.nq) s1 = payload4[(uint64_t)st.q0 + lane + kWave];
    };

    // Few large planes (fewer than the chip has room for waves): the four waves of a workgroup take
    // four consecutive bands of the same plane, decode them side by side, and then share the column
    // pass by columns, each wave running its quarter of the columns down all four bands, with two
    // workgroup barriers per round.  `bi` then counts rounds of four bands.
    constexpr bool coop = COOP;
    const uint32_t nbands_big = pl.big ? (H + pl.Rb - 1) / pl.Rb : 1u;
    const uint32_t nsteps = coop ? (nbands_big + kWaves - 1) / kWaves : nbands_big;
    const uint32_t item_stride = coop ? td.nwg : td.nwg * kWaves;
    uint32_t item = coop ? blockIdx.x - td.wg_base : (blockIdx.x - td.wg_base) * kWaves + wv, bi = 0;
    auto band_at = [&](uint32_t it, uint32_t step) -> Band { return band_of(it, coop ? step * kWaves + wv : step); };
    Band cur = band_at(item, bi);
    Ahead fa = fetch(cur);
    int32_t colacc[kColGroups] = {0, 0, 0, 0};               // running column sums (big planes)
    uint4 s0 = make_uint4(0, 0, 0, 0), s1 = s0;
    Stage sg = {0, 0};
    if (cur.valid) {
        prefix_bits(fa);
        sg = stage_of(cur, fa);
        stage_load(sg, s0, s1);
    }

    while (item < pl.nitems) {                       // uniform in the wave; with shared planes, in the workgroup
        // ---- next band: geometry now, bit counts in flight while this band is decoded ----
        uint32_t nitem = item, nb = bi + 1;
        if (nb >= nsteps) { nitem = item + item_stride; nb = 0; }
        const Band nxt = band_at(nitem, nb);
        const Ahead fn = fetch(nxt);

        const uint32_t e0 = cur.e0, n = cur.n, rows = cur.rows, npl = cur.npl;
        const uint32_t sb0 = e0 >> kLog;
        // (a wave without a band in this round of a shared plane: no sub-blocks, no rows)
        const uint32_t sb1 = cur.valid ? (e0 + n - 1) >> kLog : sb0;
        const uint32_t nsb = cur.valid ? sb1 - sb0 + 1 : 0u;   // <= kND by construction of the plan
        const uint32_t base = sb0 << kLog;
        const uint32_t u0 = e0 - base;
        const uint32_t j0 = sb0 & (kNSub - 1);           // position of sb0 in its chunk
        if (bi == 0) {
#pragma unroll
            for (int c = 0; c < kColGroups; ++c) colacc[c] = 0;
        }

        // this lane's sub-block in its chunk's stream (P is rewritten for the next band below)
        uint32_t start = 0, sbits = 0;
        if (lane < (int)nsb) {
            const uint32_t j = (sb0 + lane) & (kNSub - 1);
            const uint32_t idx = j0 + lane;
            start = P[idx] - P[idx - j];
            sbits = P[idx + 1] - P[idx];
        }
        const bool staged = sg.nq != 0;                  // uniform
        if (staged) {
            if ((uint32_t)lane < sg.nq) reinterpret_cast<uint4 *>(S + kStagePad)[lane] = s0;
            if ((uint32_t)lane + kWave < sg.nq) reinterpret_cast<uint4 *>(S + kStagePad)[lane + kWave] = s1;
        }
        wave_sync();

        // outliers of the band: a range of the outlier list (filtered by index below)
        uint32_t olo = __builtin_amdgcn_readfirstlane(fa.oo), ohi = (uint32_t)__builtin_amdgcn_readlane((int)fa.oo, 1);
        if (olo > ohi || ohi > n_outl) { bad = true; olo = ohi = 0; }
        // uniform: no outliers, rows are summed while decoding
        const bool folded = olo == ohi;

        // ---- decode: one lane per sub-block ----
        int32_t my_tail = 0;
        uint32_t my_reset = 0;
        // (a band with outliers: what the lane needs to sum its rows once the outliers are patched in)
        uint32_t late_klo = 0, late_khi = 0, late_w = 0;
        if (lane < (int)nsb) {
            const uint32_t g = sb0 + lane;
            const uint32_t uu0 = fa.uu0, uu1 = fa.uu1;
            bool lbad = !(uu0 <= uu1 && uu1 <= payload_units);
            const uint32_t nw = lbad ? 0u : (uu1 - uu0) * 4;
            // version 2: a stored bit count of 0 stands for a sub-block of zero residuals
            const bool zeros_only = a.zero_blocks && sbits == 0;
            // otherwise a sub-block holds at least one codeword of at least one bit: an empty chunk stream is damage
            if ((nw == 0 && !zeros_only) || (uint64_t)start + sbits > (uint64_t)nw * 32) lbad = true;
            const uint32_t el0 = g << kLog;              // first element of the sub-block
            const uint32_t n_here = (a.numel - el0 >= (uint32_t)SUB) ? (uint32_t)SUB : a.numel - el0;
            // elements of this sub-block that belong to the band: k in [klo, khi)
            const uint32_t klo = (el0 < e0) ? e0 - el0 : 0u;
            const uint32_t khi = (el0 + n_here > e0 + n) ? e0 + n - el0 : n_here;
            RT *my = R + lane * (SUB + 1);
            my_reset = klo;
            // position of the sub-block in the staging buffer (its chunk must lie in the staged stretch)
            uint32_t spos = 0;
            if (staged && !lbad) {
                const int64_t rel = ((int64_t)uu0 - (int64_t)sg.q0) * 128 + (int64_t)start;
                if (rel < 0 || rel + (int64_t)sbits > (int64_t)sg.nq * 128) lbad = true;
                else spos = (uint32_t)rel;
            }
            uint32_t end = 0;
            if (!lbad) {
                // row starts among the lane's elements from klo on (the band begins at one)
                const uint32_t l_first = el0 + klo - e0;                 // band-local index of the first element
                uint32_t w_first = 0;
                if (folded) w_first = l_first - pl.divW.div(l_first) * W;
                const uint32_t last = nw - 1;
                const uint32_t *__restrict__ gw =
                    reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_payload + (uint64_t)uu0 * 16);
                auto run_decode = [&](uint32_t count, uint32_t skip, auto put) -> uint32_t {
                    if (zeros_only) {
                        for (uint32_t k = skip; k < count; ++k) put(k, 0);
                        return start;
                    }
                    if (staged)
                        return decode_lds(T, S, spos, count, skip, put, lbad) - spos + start;
                    return decode_run<false>(T, [&](uint32_t k) -> uint32_t { return gw[k < last ? k : last]; }, start,
                                             count, skip, put, lbad);
                };
                if (SUB == 32 && n_here == 32u && folded) {
                    // complete 32-codeword sub-block: the row starts as a bit mask; all 32 slots of
                    // the lane are written (those outside the band are never read)
                    uint32_t mask = 0;
                    uint32_t k0 = klo + (w_first ? W - w_first : 0u);
                    my_reset = k0 < 32u ? k0 : (uint32_t)SUB;
                    for (; k0 < 32u; k0 += W) mask |= 1u << k0;
                    int32_t run = 0;
                    const uint32_t keep_mask = ~mask;
                    end = run_decode(32u, 0u, [&](uint32_t k, int32_t d) {
                        // run * (0 where the row restarts, else 1) + d in one multiply-add: the sums of a
                        // lane's 32 in-range residuals stay far inside 24 bits
                        const uint32_t keep01 = __builtin_amdgcn_ubfe(keep_mask, k, 1);
                        asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(run) : "v"(run), "v"(keep01), "v"(d));
                        my[k] = run;
                    });
                    my_tail = my[khi - 1];
                } else if (folded) {
                    // running sum along the row, restarted at every row start
                    uint32_t w = w_first;
                    int32_t run = 0;
                    uint32_t first_reset = (uint32_t)SUB;
                    end = run_decode(khi, klo, [&](uint32_t k, int32_t d) {
                        if (w == 0) { run = 0; first_reset = first_reset < k ? first_reset : k; }
                        run += d;
                        my[k] = run;
                        w = (w + 1 == W) ? 0u : w + 1;
                    });
                    my_tail = run;
                    my_reset = first_reset;
                } else {
                    const bool whole = (SUB == 32 && n_here == 32u);
                    end = run_decode(whole ? 32u : khi, whole ? 0u : klo,
                                     [&](uint32_t k, int32_t d) { my[k] = d; });
                    late_klo = klo; late_khi = khi; late_w = l_first;
                }
            }
            // a sub-block decoded to its end must land exactly on its stored bit count
            if (!lbad && (khi == n_here || (SUB == 32 && n_here == 32u)) && end != start + sbits) lbad = true;
            bad |= lbad;
        }
        wave_sync();                                     // S is free: the lane records take its place

        if (!folded) {
            // ---- outliers overwrite their residuals; then every lane sums its rows as the other
            //      bands' lanes do while they decode ----
            for (uint32_t k = olo + lane; k < ohi; k += kWave) {
                const uint32_t i = oidx[k];
                if (i >= e0 && i - e0 < n) {
                    const uint32_t u = i - base;
                    R[u + (u >> kLog)] = oval[k];
                }
            }
            wave_sync();
            if (late_klo < late_khi) {
                RT *my = R + lane * (SUB + 1);
                uint32_t w = late_w - pl.divW.div(late_w) * W;           // place in its row of the lane's first element
                int32_t run = 0;
                uint32_t first_reset = (uint32_t)SUB;
                for (uint32_t k = late_klo; k < late_khi; ++k) {
                    if (w == 0) { run = 0; first_reset = first_reset < k ? first_reset : k; }
                    run += my[k];
                    my[k] = run;
                    w = (w + 1 == W) ? 0u : w + 1;
                }
                my_tail = run;
                my_reset = first_reset;
            }
        }
        {
            // ---- carries: what each lane's leading elements (before its first row start) lack ----
            int32_t v = my_tail;                                        // 0 in lanes without a sub-block
            uint32_t f = (lane < (int)nsb && my_reset != (uint32_t)SUB) ? 1u : 0u;   // the lane's run contains a row start
            wave_segmented_sum(v, f);                                   // v: row-sum at the end of the lane's run
            // what flows into a lane is the inclusive value of the lane before it; a band begins a row
            int32_t into = (int32_t)dpp_u32<0x138, 0xf>((uint32_t)v);   // wave_shr:1
            if (lane == 0) into = 0;
            if (lane < kND) RC[lane] = make_uint2(lane < (int)nsb ? my_reset : 0u, (uint32_t)into);
        }
        wave_sync();

        // ---- next band: bit positions now, its payload in flight during the column pass ----
        Stage sgn = {0, 0};
        if (nxt.valid) {                                 // uniform
            prefix_bits(fn);
            sgn = stage_of(nxt, fn);
            stage_load(sgn, s0, s1);
        }

        // ---- column prefix sums (adding the lanes' carries), de-quantisation, stores: one lane per column ----
        const uint32_t nrow = pl.big ? rows : H;
        // One column of a band (Rj: its sums along the rows, RCj: its lane records, first element
        // uj0 slots into Rj, nrowj rows, output from outj on), continuing the column sum acc.
        // Byte offsets from the band's first output element: the stores then take a uniform base
        // and a 32-bit offset per lane.
        auto walk_band = [&](const RT *Rj, const uint2 *RCj, uint32_t uj0, uint32_t nrowj, char *__restrict__ band_out,
                             uint32_t col, int32_t acc) -> int32_t {
            const RT *R = Rj;
            const uint2 *RC = RCj;
            const uint32_t nrow = nrowj;
            const uint32_t p = pl.big ? 0u : pl.divW.div(col);
            const uint32_t w = col - p * W;
            uint32_t u = p * HW + w + uj0;
            uint32_t off = (p * HW + w) * 4u;
            // kRows rows at a time, their loads in flight together; then the short batch that may remain
            auto batch = [&](auto full_c, uint32_t nr) {
                constexpr bool kFull = decltype(full_c)::value;
                int32_t t8[kRows];
                uint32_t kk[kRows];
                uint2 rc[kRows];
#pragma unroll
                for (int q = 0; q < kRows; ++q) {
                    if (kFull || (uint32_t)q < nr) {
                        const uint32_t uq = u + q * W;
                        uint32_t t = uq >> kLog;
                        asm("" : "+v"(t));           // one shift serves both addresses below (else the compiler derives each from uq anew)
                        kk[q] = uq & (uint32_t)(SUB - 1);
                        t8[q] = R[uq + t]; rc[q] = RC[t];
                    }
                }
#pragma unroll
                for (int q = 0; q < kRows; ++q) {
                    if (kFull || (uint32_t)q < nr) {
                        acc += t8[q] + ((kk[q] < rc[q].x) ? (int32_t)rc[q].y : 0);
                        // the row's offset is uniform: it goes to the scalar base, the lane keeps one offset
                        *reinterpret_cast<float *>((band_out + (size_t)(q * 4u * W)) + off) = (float)(int16_t)acc * s;
                    }
                }
            };
            uint32_t h = 0;
            for (; h + kRows <= nrow; h += kRows) {
                batch(std::true_type{}, (uint32_t)kRows);
                u += kRows * W;
                off += 4u * kRows * W;
            }
            if (h < nrow) batch(std::false_type{}, nrow - h);        // uniform
            return acc;
        };
        auto walk = [&](uint32_t col, int32_t acc) -> int32_t {
            return walk_band(R, RC, u0, nrow, reinterpret_cast<char *>(a.xout + e0), col, acc);
        };
        if (coop) {
            // every wave has decoded its band of this round: now a quarter of the columns each,
            // down the round's bands in their order
            __syncthreads();
            const uint32_t cw = (W + kWaves - 1) / kWaves;           // <= 64: W <= kColGroups * 64
            const uint32_t col = (uint32_t)wv * cw + (uint32_t)lane;
            if ((uint32_t)lane < cw && col < W) {
                int32_t acc = colacc[0];
                for (uint32_t j = 0; j < (uint32_t)kWaves; ++j) {
                    const uint32_t row0 = (bi * kWaves + j) * pl.Rb;
                    if (row0 >= H) break;                            // uniform
                    const uint32_t rowsj = (H - row0 < pl.Rb) ? H - row0 : pl.Rb;
                    const uint32_t ej0 = item * HW + row0 * W;
                    acc = walk_band(lds.Rs[j], reinterpret_cast<const uint2 *>(lds.Ss + j * kStageWords + kStagePad),
                                    ej0 - ((ej0 >> kLog) << kLog), rowsj, reinterpret_cast<char *>(a.xout + ej0), col, acc);
                }
                colacc[0] = acc;
            }
            __syncthreads();                              // R and the staging buffers are reused by the next round
        } else {
            if (pl.big) {
#pragma unroll
                for (int c = 0; c < kColGroups; ++c) {
                    const uint32_t col = c * kWave + lane;
                    if (col < W) colacc[c] = walk(col, colacc[c]);
                }
            } else {
                const uint32_t ncols = npl * W;
                for (uint32_t col = lane; col < ncols; col += kWave) (void)walk(col, 0);
            }
            wave_sync();                                      // R and the staging buffer are reused by the next band
        }
        cur = nxt; fa = fn; sg = sgn; item = nitem; bi = nb;
    }
    if (bad) atomicOr(a.status, kStFormat);
}

}  // namespace

// The fused kernel's plan for one tensor.  Returns false when the shape does not fit it (planes
// larger than one band with rows wider than kColGroups waves): such tensors take the unfused
// kernels.
bool plan_decode_fused(TensorD *t, uint32_t sub)
{
    const uint32_t H = t->shape[2], W = t->shape[3], HW = H * W, planes = t->shape[0] * t->shape[1];
    const uint32_t ndec = kBandMax / sub;
    const uint64_t cap = (uint64_t)(ndec - 1) * sub + 1;       // a band then spans at most ndec sub-blocks
    t->divW = FastDiv::make(W);
    t->nwg = 0;
    if (t->numel == 0) return false;
    if (HW <= cap) {
        t->big = 0; t->G = (uint32_t)(cap / HW); t->Rb = 0;
        t->nitems = (planes + t->G - 1) / t->G;
    } else if (W <= (uint32_t)(kColGroups * kWave) && W <= cap) {
        t->big = 1; t->G = 1; t->Rb = (uint32_t)(cap / W);
        t->nitems = planes;
    } else {
        return false;
    }
    return true;
}

// One launch over the tensors of the group that have a plan (and a second one, of the variant
// that shares planes between waves, over those with few large planes).  Five workgroups are
// resident per compute unit.  A small call gets one round of them (a second round would build its
// decode tables for little work); a large one up to six rounds, dealt to the tensors in proportion
// to their elements, so that workgroups of different cost (small planes cost more per element than
// large ones) even out and the chip does not idle while the last round's slowest workgroup
// finishes.  Measured on the ResNet-18-shaped stream (17 tensors, 591 M elements): 1.00 / 0.96 /
// 0.93 / 0.94 / 0.94 / 0.94 ms for 3 / 4 / 5 / 6 / 8 / 12 rounds.  No more than a tensor has items
// for, at least one.
void launch_decode_fused(BatchD &b, uint32_t cus, Profiler *prof, hipStream_t st)
{
    uint64_t total = 0;
    for (uint32_t k = 0; k < b.n; ++k) if (b.t[k].nitems) total += b.t[k].numel;
    const uint64_t slots = 5ull * cus;
    uint64_t rounds = total / (slots * 16384ull * kWaves);   // at least 16 K elements per wave and round
    rounds = rounds < 1 ? 1 : rounds > 6 ? 6 : rounds;
    const uint64_t deal = slots * rounds;
    for (uint32_t k = 0; k < b.n; ++k) {
        TensorD &t = b.t[k];
        // Large planes, fewer of them than the chip holds waves (one wave per plane would leave it
        // half empty): a workgroup per plane, its waves side by side on the plane's bands.
        if (t.nitems && t.big) t.big = (t.nitems < slots * kWaves && t.shape[2] > t.Rb) ? 2u : 1u;
    }
    for (uint32_t shared = 0; shared < 2; ++shared) {
        uint32_t grid = 0;
        for (uint32_t k = 0; k < b.n; ++k) {
            TensorD &t = b.t[k];
            t.wg_base = grid;
            t.nwg = 0;
            if (!t.nitems || (t.big == 2) != (shared == 1)) continue;    // not in this launch: no workgroups
            const uint64_t share = ((uint64_t)t.numel * deal + total - 1) / total;
            const uint64_t most = shared ? t.nitems : (t.nitems + kWaves - 1) / kWaves;
            t.nwg = (uint32_t)(share < most ? share : most);
            if (t.nwg < 1) t.nwg = 1;
            grid += t.nwg;
        }
        if (!grid) continue;
        if (shared) {
            switch (b.sub) {
            case 32:  launch(prof, kKDecodeFused, k_decode_fused<32, true>, dim3(grid), dim3(kThreads), st, b); break;
            case 64:  launch(prof, kKDecodeFused, k_decode_fused<64, true>, dim3(grid), dim3(kThreads), st, b); break;
            default:  launch(prof, kKDecodeFused, k_decode_fused<128, true>, dim3(grid), dim3(kThreads), st, b); break;
            }
        } else {
            switch (b.sub) {
            case 32:  launch(prof, kKDecodeFused, k_decode_fused<32, false>, dim3(grid), dim3(kThreads), st, b); break;
            case 64:  launch(prof, kKDecodeFused, k_decode_fused<64, false>, dim3(grid), dim3(kThreads), st, b); break;
            default:  launch(prof, kKDecodeFused, k_decode_fused<128, false>, dim3(grid), dim3(kThreads), st, b); break;
            }
        }
    }
}

}  // namespace cmpz
