// Fused decompression: chunked Huffman decode -> outlier patch -> reverse Lorenzo
// (row and column prefix sums) -> de-quantisation, one pass, residuals never
// leave the CU.  HBM traffic is the container read plus the 4-byte result write.
//
// A workgroup owns whole planes.  Planes no larger than the band capacity are
// processed several at a time; a larger plane is walked in bands of whole rows
// with one running column sum per thread (needs W <= 256).  Shapes that fit
// neither case take the unfused kernels of cmpz_decompress.hip.
//
// A band is decoded by one lane per sub-block (the container stores each
// sub-block's bit count, so every lane knows where its codes start) into an LDS
// array of int32.  In a band without outliers a lane adds up its residuals along
// the row while it decodes them, so what it stores is already the row prefix sum
// up to a per-lane carry; a short segmented scan over the lanes' totals yields the
// carries and the column pass adds them on the fly.  A band with outliers stores
// plain residuals, patches the outliers in and runs an explicit row scan.
// The bit counts and offsets of the next band are fetched while the current one
// is processed.
#include "cmpz_decode_core.h"

namespace cmpz {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves   = kThreads / kWave;
constexpr int kBandMax = 8192;                    // elements decoded per band at most

template <int SUB> struct Cfg;
template <> struct Cfg<128> { static constexpr int kLog = 7; };
template <> struct Cfg<64>  { static constexpr int kLog = 6; };
template <> struct Cfg<32>  { static constexpr int kLog = 5; };

struct FusedPlan {
    uint32_t big;          // 0: groups of whole planes; 1: one plane per item, bands of rows
    uint32_t G;            // planes per group (big == 0)
    uint32_t Rb;           // rows per band (big == 1)
    uint32_t nitems;
    FastDiv  divW;
};

#ifdef CMPZ_PHASE_CLOCKS
#define PHASE(k) if (tid == 0) { const long long now_ = clock64(); clk[k] += now_ - last_; last_ = now_; }
#else
#define PHASE(k)
#endif

struct Band {
    uint32_t e0, n, rows, plane0, npl, row0;
    bool valid;
};

// What a thread fetches ahead for a band: its two bit-count entries, its lane's chunk bounds,
// and (uniform) the band's range in the outlier list.
struct Ahead {
    uint32_t v0, v1, uu0, uu1, olo, ohi;
};

template <int SUB>
__global__ __launch_bounds__(kThreads) void k_decode_fused(DecompressArgs a, FusedPlan pl)
{
    constexpr int kLog  = Cfg<SUB>::kLog;
    constexpr int kNDec = kBandMax / SUB;                 // decode lanes per band
    constexpr int kNSub = (int)kChunk / SUB;              // sub-blocks per chunk
    constexpr int kPre  = kNSub + kNDec;                  // bit-count entries looked at per band

    __shared__ int32_t  R[kBandMax + kNDec];              // one pad word per sub-block: lane-conflict free
    __shared__ DecodeTables T;
    __shared__ uint32_t P[kPre + 1];                      // exclusive prefix of sub-block bit counts
    __shared__ uint32_t wave_tot[kWaves];
    __shared__ int32_t  lane_tail[kNDec];                 // row-sum at the end of each decode lane's run
    __shared__ uint32_t lane_reset[kNDec];                // offset of the lane's first row start (SUB = none)
    __shared__ int32_t  lane_carry[kNDec];                // what the lane's elements before that offset lack

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
#ifdef CMPZ_PHASE_CLOCKS
    long long clk[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    long long last_ = clock64();
#endif
    // every workgroup validates the container and builds the decode tables for itself
    {
        const uint32_t defect = build_tables_256(T, a, reinterpret_cast<uint32_t *>(R));
        if (defect) {
            if (blockIdx.x == 0 && tid == 0) atomicOr(a.status, defect);
            return;
        }
    }
    PHASE(0)
    const uint32_t payload_units = T.payload_units, n_outl = T.n_outliers;

    const uint32_t W = a.W, H = a.H, HW = a.HW, R0 = a.radius;
    const uint32_t *__restrict__ chunk_off = reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_chunk_off);
    const uint32_t *__restrict__ outl_off = reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_outl_off);
    const uint16_t *__restrict__ sub_bits = reinterpret_cast<const uint16_t *>(a.buf + a.lay.off_sub_bits);
    const Header *hd = reinterpret_cast<const Header *>(a.buf);
    const uint32_t *__restrict__ oidx = reinterpret_cast<const uint32_t *>(a.buf + hd->off_outl_idx);
    const int32_t *__restrict__ oval = reinterpret_cast<const int32_t *>(a.buf + hd->off_outl_val);
    const float s = a.s;
    bool bad = false;

    auto band_of = [&](uint32_t item, uint32_t b) -> Band {
        Band g;
        g.valid = item < pl.nitems;
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
        Ahead f = {0, 0, 0, 0, 0, 0};
        if (!g.valid) return f;
        const uint32_t sb0 = g.e0 >> kLog, sb1 = (g.e0 + g.n - 1) >> kLog;
        const uint32_t j0 = sb0 & (kNSub - 1), ent0 = sb0 - j0, nent = j0 + (sb1 - sb0 + 1);
        if (2u * tid < nent) f.v0 = sub_bits[(uint64_t)ent0 + 2u * tid];
        if (2u * tid + 1 < nent) f.v1 = sub_bits[(uint64_t)ent0 + 2u * tid + 1];
        if (sb0 + tid <= sb1) {
            const uint32_t c = (sb0 + tid) / kNSub;
            f.uu0 = chunk_off[c]; f.uu1 = chunk_off[c + 1];
        }
        f.olo = outl_off[g.e0 / kChunk];
        f.ohi = outl_off[(g.e0 + g.n - 1) / kChunk + 1];
        return f;
    };

    const uint32_t nbands_big = pl.big ? (H + pl.Rb - 1) / pl.Rb : 1u;
    uint32_t item = blockIdx.x, b = 0;
    Band cur = band_of(item, b);
    Ahead fa = fetch(cur);
    int32_t colacc = 0;                                      // running column sum (big planes)

    while (cur.valid) {
        // ---- next band: geometry now, loads in flight while this band is processed ----
        uint32_t nitem = item, nb = b + 1;
        if (nb >= nbands_big) { nitem = item + gridDim.x; nb = 0; }
        const Band nxt = band_of(nitem, nb);
        const Ahead fn = fetch(nxt);

        const uint32_t e0 = cur.e0, n = cur.n, rows = cur.rows, npl = cur.npl;
        const uint32_t sb0 = e0 >> kLog;
        const uint32_t sb1 = (e0 + n - 1) >> kLog;
        const uint32_t nsb = sb1 - sb0 + 1;              // <= kNDec by construction of the plan
        const uint32_t base = sb0 << kLog;
        const uint32_t u0 = e0 - base;
        const uint32_t j0 = sb0 & (kNSub - 1);           // position of sb0 in its chunk
        if (b == 0) colacc = 0;

        // ---- exclusive prefix of the bit counts from the start of the first chunk ----
        {
            const uint32_t inc = wave_inclusive_sum(fa.v0 + fa.v1);
            if (lane == 63) wave_tot[wv] = inc;
            __syncthreads();
            uint32_t wbase = 0;
            for (int k = 0; k < wv; ++k) wbase += wave_tot[k];
            const uint32_t ex = wbase + inc - (fa.v0 + fa.v1);
            if (2 * tid < kPre + 1) P[2 * tid] = ex;
            if (2 * tid + 1 < kPre + 1) P[2 * tid + 1] = ex + fa.v0;
            __syncthreads();
        }
        PHASE(1)

        // outliers of the band: a range of the outlier list (filtered by index below)
        uint32_t olo = fa.olo, ohi = fa.ohi;
        if (olo > ohi || ohi > n_outl) { bad = true; olo = ohi = 0; }
        const bool folded = (olo == ohi);                // uniform: no outliers, rows are summed while decoding

        // ---- decode: one lane per sub-block ----
        if (tid < (int)nsb) {
            const uint32_t g = sb0 + tid;
            const uint32_t j = g & (kNSub - 1);
            const uint32_t idx = j0 + tid;
            const uint32_t start = P[idx] - P[idx - j];
            const uint32_t sbits = P[idx + 1] - P[idx];
            const uint32_t uu0 = fa.uu0, uu1 = fa.uu1;
            bool lbad = !(uu0 <= uu1 && uu1 <= payload_units);
            const uint32_t nw = lbad ? 0u : (uu1 - uu0) * 4;
            if ((uint64_t)start + sbits > (uint64_t)nw * 32) lbad = true;
            const uint32_t el0 = g << kLog;              // first element of the sub-block
            const uint32_t n_here = (a.numel - el0 >= (uint32_t)SUB) ? (uint32_t)SUB : a.numel - el0;
            // elements of this sub-block that belong to the band: k in [klo, khi)
            const uint32_t klo = (el0 < e0) ? e0 - el0 : 0u;
            const uint32_t khi = (el0 + n_here > e0 + n) ? e0 + n - el0 : n_here;
            int32_t *my = R + tid * (SUB + 1);
            uint32_t end = 0;
            if (!lbad) {
                const uint32_t last = nw - 1;
                const uint32_t *__restrict__ gw =
                    reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_payload + (uint64_t)uu0 * 16);
                auto rd = [&](uint32_t k) -> uint32_t { return gw[k < last ? k : last]; };
                // runs of 32 codewords are decoded from a register queue, longer ones straight from memory
                auto run_decode = [&](auto put) -> uint32_t {
                    if constexpr (SUB == 32) return decode_run_regs(T, gw, last, start, khi, klo, R0, put, lbad);
                    else return decode_run<false>(T, rd, start, khi, klo, R0, put, lbad);
                };
                if (SUB == 32 && n_here == 32u) {
                    // complete 32-codeword sub-block: unrolled decoder, all 32 slots of the lane are
                    // written (those outside the band are never read)
                    uint32_t mask = 0, first_reset = (uint32_t)SUB;
                    if (folded) {
                        // row starts among the lane's elements from klo on (the band begins at one)
                        const uint32_t l_first = el0 + klo - e0;
                        const uint32_t w_first = l_first - pl.divW.div(l_first) * W;
                        uint32_t k0 = klo + (w_first ? W - w_first : 0u);
                        first_reset = k0 < 32u ? k0 : (uint32_t)SUB;
                        for (; k0 < 32u; k0 += W) mask |= 1u << k0;
                        end = decode32<true>(T, gw, last, start, mask, (int32_t)R0, my, lbad);
                        lane_tail[tid] = my[khi - 1];
                        lane_reset[tid] = first_reset;
                    } else {
                        end = decode32<false>(T, gw, last, start, 0u, (int32_t)R0, my, lbad);
                    }
                } else if (folded) {
                    // running sum along the row, restarted at every row start
                    const uint32_t l_first = el0 + klo - e0;             // band-local index of the first element
                    uint32_t w = l_first - pl.divW.div(l_first) * W;
                    int32_t run = 0;
                    uint32_t first_reset = (uint32_t)SUB;
                    end = run_decode([&](uint32_t k, uint32_t sy) {
                        const int32_t d = (int32_t)sy - (int32_t)R0;
                        if (w == 0) { run = 0; first_reset = first_reset < k ? first_reset : k; }
                        run += d;
                        my[k] = run;
                        w = (w + 1 == W) ? 0u : w + 1;
                    });
                    lane_tail[tid] = run;
                    lane_reset[tid] = first_reset;
                } else {
                    end = run_decode([&](uint32_t k, uint32_t sy) { my[k] = (int32_t)sy - (int32_t)R0; });
                }
            } else {
                lane_tail[tid] = 0; lane_reset[tid] = klo;
            }
            // a sub-block decoded to its end must land exactly on its stored bit count
            if ((khi == n_here || (SUB == 32 && n_here == 32u)) && end != start + sbits) lbad = true;
            bad |= lbad;
#ifdef CMPZ_PHASE_CLOCKS
            if (tid == 0) { const long long now_ = clock64(); clk[6] += now_ - last_; last_ = now_; }
#endif
        }
        __syncthreads();
        PHASE(3)

        if (folded) {
            // ---- carries: what each lane's leading elements (before its first row start) lack ----
            if (wv == 0) {
                int32_t chain = 0;                                   // row-sum flowing out of the previous 64 lanes
                for (uint32_t t0 = 0; t0 < nsb; t0 += 64) {
                    const uint32_t t = t0 + lane;
                    const bool in = t < nsb;
                    int32_t v = in ? lane_tail[t] : 0;
                    uint32_t f = (in && lane_reset[t] != (uint32_t)SUB) ? 1u : 0u;   // the lane's run contains a row start
                    wave_segmented_sum(v, f);                        // v: row-sum at the end of lane t, within this group
                    if (!f) v += chain;
                    // exclusive: what flows into lane t is the inclusive value of lane t-1
                    int32_t into = (int32_t)dpp_u32<0x138, 0xf>((uint32_t)v);        // wave_shr:1
                    if (lane == 0) into = chain;
                    if (in) lane_carry[t] = into;
                    chain = __builtin_amdgcn_readlane(v, 63);
                }
            }
            __syncthreads();
            // every decode lane adds its carry to the elements before its first row start
            if (tid < (int)nsb) {
                const int32_t cy = lane_carry[tid];
                const uint32_t el0 = (sb0 + tid) << kLog;
                const uint32_t n_here = (a.numel - el0 >= (uint32_t)SUB) ? (uint32_t)SUB : a.numel - el0;
                const uint32_t klo = (el0 < e0) ? e0 - el0 : 0u;
                uint32_t khi = (el0 + n_here > e0 + n) ? e0 + n - el0 : n_here;
                const uint32_t fr = lane_reset[tid];
                khi = khi < fr ? khi : fr;
                int32_t *my = R + tid * (SUB + 1);
                if (cy != 0) for (uint32_t k = klo; k < khi; ++k) my[k] += cy;
            }
        } else {
            // ---- outliers overwrite their residuals, then an explicit row scan ----
            for (uint32_t k = olo + tid; k < ohi; k += kThreads) {
                const uint32_t i = oidx[k];
                if (i >= e0 && i - e0 < n) {
                    const uint32_t u = i - base;
                    R[u + (u >> kLog)] = oval[k];
                }
            }
            __syncthreads();
            const uint32_t r_lo = (uint32_t)(((uint64_t)rows * wv) / kWaves);
            const uint32_t r_hi = (uint32_t)(((uint64_t)rows * (wv + 1)) / kWaves);
            const uint32_t l_lo = r_lo * W, l_hi = r_hi * W;
            int32_t carry = 0;
            for (uint32_t l0 = l_lo; l0 < l_hi; l0 += 64) {
                const uint32_t l = l0 + lane;
                const bool in = l < l_hi;
                const uint32_t u = l + u0;
                const uint32_t ph = u + (u >> kLog);
                int32_t v = in ? R[ph] : 0;
                uint32_t f = (l - pl.divW.div(l) * W == 0) ? 1u : 0u;      // row start
                wave_segmented_sum(v, f);
                if (!f) v += carry;
                if (in) R[ph] = v;
                carry = __builtin_amdgcn_readlane(v, 63);
            }
        }
        __syncthreads();
        PHASE(4)

        // ---- column prefix sums; wide rows are de-quantised and stored from here ----
        const bool direct = W >= 32;                     // a wave then stores runs of >= 128 bytes
        {
            const uint32_t ncols = pl.big ? W : npl * W;
            const uint32_t nrow = pl.big ? rows : H;
            for (uint32_t col = tid; col < ncols; col += kThreads) {
                const uint32_t p = pl.big ? 0u : pl.divW.div(col);
                const uint32_t w = col - p * W;
                int32_t acc = pl.big ? colacc : 0;
                uint32_t u = p * HW + w + u0;
                float *__restrict__ dst = a.xout + e0 + p * HW + w;
                uint32_t h = 0;
                for (; h + 8 <= nrow; h += 8) {          // 8 rows at a time: loads in flight together
                    int32_t t8[8];
                    uint32_t ph[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) { const uint32_t uq = u + q * W; ph[q] = uq + (uq >> kLog); t8[q] = R[ph[q]]; }
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        acc += t8[q];
                        if (direct) dst[(h + q) * W] = (float)acc * s; else R[ph[q]] = acc;
                    }
                    u += 8 * W;
                }
                for (; h < nrow; ++h, u += W) {
                    const uint32_t ph = u + (u >> kLog);
                    acc += R[ph];
                    if (direct) dst[h * W] = (float)acc * s; else R[ph] = acc;
                }
                if (pl.big) colacc = acc;
            }
        }

        // ---- narrow rows: de-quantise and store from LDS, 128 bits at a time ----
        if (!direct) {
            __syncthreads();
            const uint32_t q_lo = e0 >> 2, q_hi = (e0 + n + 3) >> 2;       // global quads touched
            for (uint32_t qd = q_lo + tid; qd < q_hi; qd += kThreads) {
                const uint32_t i = qd << 2;
                float o[4];
                bool ok[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const uint32_t e = i + t;
                    ok[t] = e >= e0 && e - e0 < n;
                    const uint32_t u = e - base;
                    o[t] = ok[t] ? (float)R[u + (u >> kLog)] * s : 0.0f;
                }
                if (ok[0] && ok[3]) {
                    *reinterpret_cast<float4 *>(a.xout + i) = make_float4(o[0], o[1], o[2], o[3]);
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t) if (ok[t]) a.xout[i + t] = o[t];
                }
            }
        }
        __syncthreads();                                  // R and the lane arrays are reused by the next band
        PHASE(5)
        cur = nxt; fa = fn; item = nitem; b = nb;
    }
    if (bad) atomicOr(a.status, kStFormat);
#ifdef CMPZ_PHASE_CLOCKS
    if (tid == 0)
        for (int k = 0; k < 8; ++k)
            atomicAdd(reinterpret_cast<unsigned long long *>(a.meta + kMetaClocks) + k, (unsigned long long)clk[k]);
#endif
}

}  // namespace

// Returns false when the shape does not fit the fused kernel (caller falls back).
bool launch_decode_fused(const DecompressArgs &a, Profiler *prof, hipStream_t st)
{
    const uint32_t ndec = kBandMax / a.sub;
    const uint64_t cap = (uint64_t)(ndec - 1) * a.sub + 1;     // a band then spans at most ndec sub-blocks
    FusedPlan pl;
    pl.divW = FastDiv::make(a.W);
    if (a.HW <= cap) {
        pl.big = 0; pl.G = (uint32_t)(cap / a.HW); pl.Rb = 0;
        pl.nitems = (a.planes + pl.G - 1) / pl.G;
    } else if (a.W <= (uint32_t)kThreads) {
        pl.big = 1; pl.G = 1; pl.Rb = (uint32_t)(cap / a.W);
        pl.nitems = a.planes;
    } else {
        return false;
    }
    const uint32_t grid = pl.nitems < 256u * 8u ? pl.nitems : 256u * 8u;
    switch (a.sub) {
    case 32:  launch(prof, kKDecodeFused, k_decode_fused<32>, dim3(grid), dim3(kThreads), st, a, pl); break;
    case 64:  launch(prof, kKDecodeFused, k_decode_fused<64>, dim3(grid), dim3(kThreads), st, a, pl); break;
    default:  launch(prof, kKDecodeFused, k_decode_fused<128>, dim3(grid), dim3(kThreads), st, a, pl); break;
    }
    return true;
}

}  // namespace cmpz
