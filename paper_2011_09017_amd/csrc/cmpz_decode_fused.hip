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
// sub-block's bit count, so every lane knows where its codes start), into an LDS
// array of int32 residuals that the whole workgroup then scans in place.
#include "cmpz_decode_core.h"

namespace cmpz {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves   = kThreads / kWave;
constexpr int kBandMax = 8192;                    // elements decoded per band at most
constexpr int kStageWords = 2560;                 // LDS copy of the band's bit stream (10 bits per code)
constexpr int kMaxSlots = 4;                      // chunks a band can touch

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

template <int SUB>
__global__ __launch_bounds__(kThreads) void k_decode_fused(DecompressArgs a, const DecodeTables *__restrict__ tb,
                                                           FusedPlan pl)
{
    constexpr int kLog  = Cfg<SUB>::kLog;
    constexpr int kNDec = kBandMax / SUB;                 // decode lanes per band
    constexpr int kNSub = (int)kChunk / SUB;              // sub-blocks per chunk
    constexpr int kPre  = kNSub + kNDec;                  // bit-count entries looked at per band

    __shared__ int32_t  R[kBandMax + kNDec];              // one pad word per sub-block: lane-conflict free
    __shared__ DecodeTables T;
    __shared__ uint32_t P[kPre + 1];                      // exclusive prefix of sub-block bit counts
    __shared__ uint32_t wave_tot[kWaves];
    __shared__ uint32_t stage[kStageWords];
    __shared__ uint32_t slot_w0[kMaxSlots], slot_nw[kMaxSlots], slot_base[kMaxSlots], slot_unit0[kMaxSlots];
    __shared__ uint32_t slot_bad, staged;

    if (a.meta[kMetaBad]) return;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
#ifdef CMPZ_PHASE_CLOCKS
    long long clk[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    long long last_ = clock64();
#endif
    load_tables(T, tb, tid, kThreads);
    __syncthreads();
    PHASE(0)
    const uint32_t payload_units = T.payload_units, n_outl = T.n_outliers;

    if (tid == 0) slot_bad = 0;
    const uint32_t W = a.W, H = a.H, HW = a.HW, R0 = a.radius;
    const uint32_t *__restrict__ chunk_off = reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_chunk_off);
    const uint32_t *__restrict__ outl_off = reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_outl_off);
    const uint16_t *__restrict__ sub_bits = reinterpret_cast<const uint16_t *>(a.buf + a.lay.off_sub_bits);
    const Header *hd = reinterpret_cast<const Header *>(a.buf);
    const uint32_t *__restrict__ oidx = reinterpret_cast<const uint32_t *>(a.buf + hd->off_outl_idx);
    const int32_t *__restrict__ oval = reinterpret_cast<const int32_t *>(a.buf + hd->off_outl_val);
    const float s = a.s;
    bool bad = false;

    for (uint32_t item = blockIdx.x; item < pl.nitems; item += gridDim.x) {
        uint32_t plane0, npl, nbands;
        if (pl.big) { plane0 = item; npl = 1; nbands = (H + pl.Rb - 1) / pl.Rb; }
        else { plane0 = item * pl.G; npl = (a.planes - plane0 < pl.G) ? a.planes - plane0 : pl.G; nbands = 1; }
        int32_t colacc = 0;                                  // running column sum (big planes)

        for (uint32_t b = 0; b < nbands; ++b) {
            const uint32_t row0 = pl.big ? b * pl.Rb : 0;
            const uint32_t rows = pl.big ? ((H - row0 < pl.Rb) ? H - row0 : pl.Rb) : npl * H;
            const uint32_t e0 = plane0 * HW + row0 * W;      // first element of the band
            const uint32_t n = rows * W;                     // elements in the band (<= kBandMax)
            const uint32_t sb0 = e0 >> kLog;
            const uint32_t sb1 = (e0 + n - 1) >> kLog;
            const uint32_t nsb = sb1 - sb0 + 1;              // <= kNDec by construction of the plan
            const uint32_t base = sb0 << kLog;
            const uint32_t u0 = e0 - base;
            const uint32_t j0 = sb0 & (kNSub - 1);           // position of sb0 in its chunk
            const uint32_t ent0 = sb0 - j0;                  // first sub-block of that chunk

            // ---- exclusive prefix of the bit counts from the start of the first chunk ----
            {
                const uint32_t nent = j0 + nsb;              // <= kPre
                uint32_t v[2];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const uint32_t k = 2 * tid + q;
                    v[q] = (k < nent) ? sub_bits[(uint64_t)ent0 + k] : 0u;
                }
                // block exclusive scan of v[0] + v[1]
                const uint32_t inc = wave_inclusive_sum(v[0] + v[1]);
                if (lane == 63) wave_tot[wv] = inc;
                __syncthreads();
                uint32_t wbase = 0;
                for (int k = 0; k < wv; ++k) wbase += wave_tot[k];
                const uint32_t ex = wbase + inc - (v[0] + v[1]);
                if (2 * tid < kPre + 1) P[2 * tid] = ex;
                if (2 * tid + 1 < kPre + 1) P[2 * tid + 1] = ex + v[0];
                __syncthreads();
            }

            PHASE(1)
            // ---- where each touched chunk's needed words live; copy them into LDS if they fit ----
            const uint32_t c_first = sb0 / kNSub, c_last = sb1 / kNSub;    // at most kMaxSlots chunks
            if (tid <= (int)(c_last - c_first) && tid < kMaxSlots) {
                const uint32_t c = c_first + tid;
                const uint32_t ja = (c == c_first) ? j0 : 0u;                       // first needed sub-block
                const uint32_t jb = (c == c_last) ? (sb1 & (kNSub - 1)) : kNSub - 1;  // last needed
                const uint32_t ia = (c - c_first) * kNSub;                          // entry of the chunk start in P
                const uint32_t bit_a = P[ia + ja] - P[ia], bit_b = P[ia + jb + 1] - P[ia];
                const uint32_t uu0 = chunk_off[c], uu1 = chunk_off[c + 1];
                uint32_t w0 = bit_a >> 5, nw = ((bit_b + 31) >> 5) - w0 + 1;
                bool ok = uu0 <= uu1 && uu1 <= payload_units && (uint64_t)bit_b <= (uint64_t)(uu1 - uu0) * 128;
                if (ok && w0 + nw > (uu1 - uu0) * 4) nw = (uu1 - uu0) * 4 - w0;
                if (!ok) { nw = 0; atomicOr(&slot_bad, 1u); }
                slot_w0[tid] = w0; slot_nw[tid] = nw; slot_unit0[tid] = ok ? uu0 : 0u;
            }
            if (tid == 0) staged = 0;
            __syncthreads();
            if (tid == 0) {
                uint32_t acc = 0;
                for (uint32_t k = 0; k <= c_last - c_first && k < (uint32_t)kMaxSlots; ++k) { slot_base[k] = acc; acc += slot_nw[k]; }
                staged = (acc <= (uint32_t)kStageWords) ? 1u : 0u;
            }
            __syncthreads();
            const bool use_lds = staged != 0;
            if (use_lds) {
                for (uint32_t k = 0; k <= c_last - c_first; ++k) {
                    const uint32_t *__restrict__ src = reinterpret_cast<const uint32_t *>(
                        a.buf + a.lay.off_payload + (uint64_t)slot_unit0[k] * 16) + slot_w0[k];
                    for (uint32_t q = tid; q < slot_nw[k]; q += kThreads) stage[slot_base[k] + q] = src[q];
                }
                __syncthreads();
            }

            PHASE(2)
            // ---- decode: one lane per sub-block ----
            if (tid < (int)nsb) {
                const uint32_t g = sb0 + tid;
                const uint32_t c = g / kNSub, j = g & (kNSub - 1);
                const uint32_t idx = j0 + tid;
                const uint32_t start = P[idx] - P[idx - j];
                const uint32_t sbits = P[idx + 1] - P[idx];
                const uint32_t slot = c - c_first;
                const uint32_t w0 = slot_w0[slot], nw = slot_nw[slot], sbase = slot_base[slot];
                const uint32_t *__restrict__ words = reinterpret_cast<const uint32_t *>(
                    a.buf + a.lay.off_payload + (uint64_t)slot_unit0[slot] * 16);
                bool lbad = false;
                if (nw == 0 || (start >> 5) < w0 || ((start + sbits + 31) >> 5) > w0 + nw) lbad = true;
                const uint32_t el0 = g << kLog;              // first element of the sub-block
                const uint32_t n_here = (a.numel - el0 >= (uint32_t)SUB) ? (uint32_t)SUB : a.numel - el0;
                // elements of this sub-block that belong to the band: k in [klo, khi)
                const uint32_t klo = (el0 < e0) ? e0 - el0 : 0u;
                const uint32_t khi = (el0 + n_here > e0 + n) ? e0 + n - el0 : n_here;
                int32_t *my = R + tid * (SUB + 1);
                auto put = [&](uint32_t k, uint32_t sy) { my[k] = (int32_t)sy - (int32_t)R0; };
                uint32_t end = 0;
                if (!lbad) {
                    const uint32_t last = nw - 1;
                    if (use_lds) {
                        const uint32_t *sw = stage + sbase;
                        end = decode_run(T, [&](uint32_t k) -> uint32_t { const uint32_t r = k - w0; return sw[r < last ? r : last]; },
                                         start, khi, klo, R0, put, lbad);
                    } else {
                        const uint32_t *__restrict__ gw = words + w0;
                        end = decode_run(T, [&](uint32_t k) -> uint32_t { const uint32_t r = k - w0; return gw[r < last ? r : last]; },
                                         start, khi, klo, R0, put, lbad);
                    }
                }
                // a sub-block decoded to its end must land exactly on its stored bit count
                if (khi == n_here && end != start + sbits) lbad = true;
                bad |= lbad;
            }
            __syncthreads();

            PHASE(3)
            // ---- outliers of the band overwrite their residuals ----
            {
                const uint32_t c_lo = e0 / kChunk, c_hi = (e0 + n - 1) / kChunk;
                uint32_t lo = outl_off[c_lo], hi = outl_off[c_hi + 1];
                if (lo > hi || hi > n_outl) { bad = true; hi = lo = 0; }
                for (uint32_t k = lo + tid; k < hi; k += kThreads) {
                    const uint32_t i = oidx[k];
                    if (i >= e0 && i - e0 < n) {
                        const uint32_t u = i - base;
                        R[u + (u >> kLog)] = oval[k];
                    }
                }
                if (lo != hi) __syncthreads();               // uniform: lo, hi are the same for all threads
            }

            PHASE(4)
            // ---- row prefix sums: every wave takes a contiguous range of whole rows ----
            {
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

            PHASE(5)
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
                        int32_t t[8];
                        uint32_t ph[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q) { const uint32_t uq = u + q * W; ph[q] = uq + (uq >> kLog); t[q] = R[ph[q]]; }
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            acc += t[q];
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
            __syncthreads();                                  // R is reused by the next band
            PHASE(6)
        }
    }
    if (bad || slot_bad) atomicOr(a.status, kStFormat);
#ifdef CMPZ_PHASE_CLOCKS
    if (tid == 0)
        for (int k = 0; k < 8; ++k)
            atomicAdd(reinterpret_cast<unsigned long long *>(a.meta + kMetaClocks) + k, (unsigned long long)clk[k]);
#endif
}

}  // namespace

// Returns false when the shape does not fit the fused kernel (caller falls back).
bool launch_decode_fused(const DecompressArgs &a, const DecodeTables *tb, Profiler *prof, hipStream_t st)
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
    case 32:  launch(prof, kKDecodeFused, k_decode_fused<32>, dim3(grid), dim3(kThreads), st, a, tb, pl); break;
    case 64:  launch(prof, kKDecodeFused, k_decode_fused<64>, dim3(grid), dim3(kThreads), st, a, tb, pl); break;
    default:  launch(prof, kKDecodeFused, k_decode_fused<128>, dim3(grid), dim3(kThreads), st, a, tb, pl); break;
    }
    return true;
}

}  // namespace cmpz
