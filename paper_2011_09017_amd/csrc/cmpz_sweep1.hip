// Sweep 1 of compression, LDS-tiled: pre-quantisation, 2D Lorenzo prediction,
// quantisation-code / outlier split, histogram -- one read of x, one write of
// the 16-bit symbols.
//
// The tensor is one linear array (element i has its neighbours at i-1, i-W and
// i-W-1 of the same plane).  A workgroup takes chunks of 4096 consecutive
// elements.  Phase A quantises the chunk and the W+1 elements before it once
// each, with 128-bit loads, into an LDS array of int16 (|q| <= 16384).  Phase B
// gives every thread 16 consecutive elements: residuals from the LDS values,
// symbols, histogram (LDS-private, the zero residual counted per wave).  A wave's
// 1024 symbols (a quarter of the chunk) are stored with 8 bits each if they all
// lie within 127 of the zero residual (the usual case), one 128-bit store per
// thread, otherwise with 16 bits, two stores: the second sweep reads that scratch
// twice.  Rows wider than the halo capacity take the untiled kernel in
// cmpz_compress.hip.
#include "cmpz_internal.h"

namespace cmpz {
namespace {

constexpr int kThreads = 256;
constexpr int kHalo    = 1040;                    // LDS slots in front of the chunk; needs W + 4 <= kHalo
constexpr int kQWords  = kHalo + (int)kChunk + 16;

// Bit k of m as a mask of all ones or all zeros.  The empty asm keeps the compiler from turning
// the AND with it into a compare and a select (three instructions and a wait state for two).
__device__ __forceinline__ int mask_of_bit(int m, int k)
{
    int r = __builtin_amdgcn_sbfe(m, k, 1);
    asm("" : "+v"(r));
    return r;
}

__global__ __launch_bounds__(kThreads) void k_quant_lorenzo_split_hist_tiled(BatchC b)
{
    __shared__ __align__(16) int16_t Q[kQWords];
    __shared__ uint32_t hist[kMaxSym];
    __shared__ uint32_t ocnt;
    const int tid = threadIdx.x, lane = tid & 63;
    for (int k = tid; k < (int)kMaxSym; k += kThreads) hist[k] = 0;

    // the tensor this workgroup works on (uniform: scalar loads from the kernel arguments)
    uint32_t ti = 0;
    for (uint32_t k = 1; k < b.n; ++k) if (blockIdx.x >= b.t[k].sweep_base) ti = k;
    const TensorC &tc = b.t[ti];
    const uint32_t wg = blockIdx.x - tc.sweep_base;
    const float *__restrict__ x = tc.x;
    const uint32_t numel = tc.numel, H = tc.shape[2], W = tc.shape[3], HW = H * W, nchunks = tc.nchunks;
    const FastDiv divW = tc.divW, divHW = tc.divHW;
    uint16_t *__restrict__ sym = b.sym + (uint64_t)tc.chunk_base * kChunk;
    const int R = (int)b.radius;
    const float r = tc.r;
    uint32_t events = 0, zero_run = 0;            // clamped elements; symbols equal to R seen by this thread

    for (uint32_t t = 0; t < b.sweep_chunks; ++t) {
        const uint32_t c = wg * b.sweep_chunks + t;
        if (c >= nchunks) break;
        const uint32_t t0 = c * kChunk;                              // first element of the chunk
        const uint32_t t1 = (numel - t0 < kChunk) ? numel : t0 + kChunk;
        __syncthreads();                                             // previous chunk's phase B is done with Q
        if (tid == 0) ocnt = 0;

        // ---- phase A: quantise [t0 - (W+1) rounded down to 4, t1) into Q ----
        const uint32_t want = W + 1;
        const uint32_t hs = (t0 >= want ? t0 - want : 0u) & ~3u;     // first element loaded
        for (uint32_t g = hs + 4u * tid; g < t1; g += 4u * kThreads) {
            float v[4];
            if (g + 4 <= numel) {
                const float4 f = *reinterpret_cast<const float4 *>(x + g);
                v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = (g + j < numel) ? x[g + j] : 0.0f;
            }
            // Four values at once: while the largest magnitude of x*r (as a bit pattern: a NaN or an
            // infinity compares above every finite value) stays within the quantiser's range, the
            // clamp has nothing to do and no event to count.
            float tt[4];
            uint32_t mag = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                tt[j] = v[j] * r;
                const uint32_t a = __float_as_uint(tt[j]) & 0x7fffffffu;
                mag = a > mag ? a : mag;
            }
            int q[4];
            if (mag <= 0x46800000u) {                                // 16384.0f
#pragma unroll
                for (int j = 0; j < 4; ++j) q[j] = (int)__builtin_rintf(tt[j]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) q[j] = quant(v[j], r);
                if (g >= t0) {                                       // (g and t0 are multiples of 4: no straddling)
#pragma unroll
                    for (int j = 0; j < 4; ++j) events += (g + j < numel) ? clamps(v[j], r) : 0u;
                }
            }
            uint2 pk;
            pk.x = ((uint32_t)q[0] & 0xffffu) | ((uint32_t)q[1] << 16);
            pk.y = ((uint32_t)q[2] & 0xffffu) | ((uint32_t)q[3] << 16);
            // slot of element g: kHalo + (g - t0); g - t0 is a multiple of 4 (t0 and g are)
            *reinterpret_cast<uint2 *>(&Q[(int)kHalo + (int)g - (int)t0]) = pk;
        }
        __syncthreads();

        // ---- phase B: 16 consecutive elements per thread ----
        const uint32_t i0 = 16u * tid;                               // chunk-local index of the first element
        const uint32_t g0 = t0 + i0;
        uint32_t s[16];
        uint32_t nout = 0;
        uint32_t bytes_or = 0;                                       // above 0xff: some symbol of the thread has no byte form
        uint32_t zeros = 0, nhere = 0;                               // zero residuals among the thread's elements; how many it has
        if (g0 < t1) {
            // plane coordinates of the first element, then bit masks over the 16 elements:
            // mw bit j = element j starts a row, mh bit j = element j lies in row 0 of its plane
            const uint32_t p = divHW.div(g0);
            const uint32_t rem = g0 - p * HW;
            uint32_t h = divW.div(rem);
            const uint32_t w = rem - h * W;
            uint32_t mw = 0, mh = 0;
            uint32_t j = w ? W - w : 0u;                             // first row start at or after element 0
            if (h == 0 && j) mh |= (j >= 16u) ? 0xffffu : ((1u << j) - 1u);
            if (w) h = (h + 1 == H) ? 0u : h + 1;                    // row index of that row start
            for (; j < 16u; j += W) {
                mw |= 1u << j;
                if (h == 0) {
                    const uint32_t e = j + W;
                    mh |= ((e >= 16u) ? 0xffffu : ((1u << e) - 1u)) & ~((1u << j) - 1u);
                }
                h = (h + 1 == H) ? 0u : h + 1;
            }
            const int li = (int)kHalo + (int)i0;
            int cur[17], up[17];                                     // index k holds element k-1
            {
                const uint4 a0 = *reinterpret_cast<const uint4 *>(&Q[li]);
                const uint4 a1 = *reinterpret_cast<const uint4 *>(&Q[li + 8]);
                const uint32_t wd[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    cur[1 + 2 * k] = (int)(int16_t)(wd[k] & 0xffffu);
                    cur[2 + 2 * k] = (int)(int16_t)(wd[k] >> 16);
                }
                cur[0] = Q[li - 1];
            }
#pragma unroll
            for (int k = 0; k < 17; ++k) up[k] = Q[li - (int)W - 1 + k];

            const uint32_t nval = (t1 - g0 >= 16u) ? 16u : t1 - g0;
            nhere = nval;
            if (nval == 16u) {
                // all 16 elements exist.  With v = q - (q of the row above, 0 in the first row) the
                // residual is v[k] - v[k-1], the second term 0 at a row start (an element that does not
                // start a row lies in the row of its left neighbour, so the neighbour's v may be taken
                // with this element's first-row mask).  Symbols first; the in-range test and the test
                // for the byte form on the smallest and the largest of them.
                const int nmw = (int)~mw, nmh = (int)~mh;                        // bit k set: keep the term
                int vprev = cur[0] - (up[0] & mask_of_bit(nmh, 0));
                int smax = -0x7fffffff, smin = 0x7fffffff;
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const int vk = cur[k + 1] - (up[k + 1] & mask_of_bit(nmh, k));
                    const int sk = (vk + R) - (vprev & mask_of_bit(nmw, k));
                    vprev = vk;
                    s[k] = (uint32_t)sk;
                    smax = sk > smax ? sk : smax;
                    smin = sk < smin ? sk : smin;
                }
                if (smin < 1 || smax > 2 * R - 1) {                              // rare: some residual is an outlier
#pragma unroll
                    for (int k = 0; k < 16; ++k)
                        if (s[k] - 1u >= (uint32_t)(2 * R - 1)) { s[k] = 0u; ++nout; }
                    bytes_or = 0x100u;                                           // the outlier symbol has no byte form
                } else if (smin < (int)b.sym_off || smax > (int)b.sym_off + 255) {
                    bytes_or = 0x100u;
                }
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    if (s[k] == (uint32_t)R) ++zeros;
                    else atomicAdd(&hist[s[k]], 1u);
                }
            } else {
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const int keepw = ~__builtin_amdgcn_sbfe((int)mw, k, 1);
                    const int keeph = ~__builtin_amdgcn_sbfe((int)mh, k, 1);
                    const int d = (cur[k + 1] - (cur[k] & keepw)) - ((up[k + 1] - (up[k] & keepw)) & keeph);
                    const uint32_t sy = (uint32_t)(d + R);
                    const bool in = (sy - 1u) < (uint32_t)(2 * R - 1);           // 1 <= d+R <= 2R-1
                    s[k] = in ? sy : 0u;
                    if ((uint32_t)k < nval) {
                        bytes_or |= in ? sy - b.sym_off : 0x100u;
                        nout += in ? 0u : 1u;
                        if (s[k] == (uint32_t)R) ++zeros;
                        else atomicAdd(&hist[s[k]], 1u);
                    }
                }
            }
        }
        // Version 2: the zero residuals of a sub-block that holds nothing else are not counted (a thread
        // that found only zeros has touched no other bin).  A sub-block is sub/16 neighbouring threads.
        if (!(b.zero_blocks && group_all(zeros == nhere, (uint32_t)lane, b.sub / 16u))) zero_run += zeros;
        {
            // the wave's quarter of the chunk: bytes if every symbol has a byte form.  The scratch holds
            // whole chunks: the stores past the end of the tensor stay inside the chunk's slot.
            const bool wide_q = __ballot(bytes_or > 0xffu) != 0;         // uniform in the wave
            const uint32_t quarter = (uint32_t)tid >> 6;
            if (lane == 0) b.wide[(uint64_t)(tc.chunk_base + c) * 4 + quarter] = wide_q ? 1u : 0u;
            if (g0 < t1) {
                if (wide_q) {
                    uint4 o0, o1;
                    o0.x = s[0] | (s[1] << 16); o0.y = s[2] | (s[3] << 16); o0.z = s[4] | (s[5] << 16); o0.w = s[6] | (s[7] << 16);
                    o1.x = s[8] | (s[9] << 16); o1.y = s[10] | (s[11] << 16); o1.z = s[12] | (s[13] << 16); o1.w = s[14] | (s[15] << 16);
                    *reinterpret_cast<uint4 *>(sym + g0) = o0;
                    *reinterpret_cast<uint4 *>(sym + g0 + 8) = o1;
                } else {
                    // (symbols past the end of the tensor may not fit a byte: whatever they leave is never read)
                    uint32_t o[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const uint32_t b0 = s[4 * k] - b.sym_off, b1 = s[4 * k + 1] - b.sym_off;
                        const uint32_t b2 = s[4 * k + 2] - b.sym_off, b3 = s[4 * k + 3] - b.sym_off;
                        o[k] = b0 | (b1 << 8) | (b2 << 16) | (b3 << 24);       // no masks: only positions past the end
                                                                                // can exceed a byte, and they spill upward
                    }
                    // the quarter's slot starts where its 16-bit symbols would; the wave's bytes fill its first half
                    *reinterpret_cast<uint4 *>(reinterpret_cast<uint8_t *>(sym + t0 + 1024u * quarter) + 16u * lane) =
                        make_uint4(o[0], o[1], o[2], o[3]);
                }
            }
        }
        if (nout) atomicAdd(&ocnt, nout);
        __syncthreads();
        if (tid == 0) b.outl_cnt[tc.chunk_base + c] = ocnt;
    }

    // zero residuals: one LDS atomic per wave
    {
        const uint32_t tot = wave_inclusive_sum(zero_run);
        if (lane == 63 && tot) atomicAdd(&hist[R], tot);
    }
    __syncthreads();
    for (int k = tid; k < (int)kMaxSym; k += kThreads) {
        const uint32_t n = hist[k];
        if (n) atomicAdd(&b.hist[((uint64_t)ti * kHistCopies + wg % kHistCopies) * kMaxSym + k], n);
    }
    {
        const uint32_t tot = wave_inclusive_sum(events);
        if (lane == 63 && tot) atomicAdd(&b.tmeta[ti].range_events, tot);
    }
}

}  // namespace

// Rows this wide do not fit the halo: such tensors take the untiled kernel.
bool sweep1_tiled_fits(uint32_t W) { return W + 4 <= (uint32_t)kHalo; }

// One launch over the tensors of the group whose rows fit (their sweep_base ranges).
void launch_sweep1(const BatchC &b, Profiler *prof, hipStream_t st)
{
    if (b.sweep_wgs == 0) return;
    launch(prof, kKQuantLorenzoHist, k_quant_lorenzo_split_hist_tiled, dim3(b.sweep_wgs), dim3(kThreads), st, b);
}

}  // namespace cmpz
