// The first sweep of compression for tensors whose rows are too wide for the LDS-tiled
// kernel of cmpz_sweep1.hip: pre-quantisation + 2D Lorenzo + split + histogram straight from
// global memory (the neighbours above and to the left are quantised again).
//
// The tensor is treated as one linear array: element i of plane p = i / (H*W)
// has neighbours i-1, i-W and i-W-1 in the same plane, so a workgroup can own a
// chunk-aligned linear range whatever H and W are.
#include "cmpz_internal.h"

namespace cmpz {
namespace {

constexpr int kThreads    = 256;
constexpr int kTileChunks = 4;                       // chunks per workgroup
constexpr int kTile       = kTileChunks * kChunk;    // 16384 elements

// ---------------------------------------------------------------------------
// Sweep 1: x -> symbols (u16 scratch), histogram, outliers per chunk, range events.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_quant_lorenzo_split_hist(BatchC b, uint32_t ti)
{
    const TensorC &tc = b.t[ti];
    __shared__ uint32_t hist[kMaxSym];
    __shared__ uint32_t ocnt[kTileChunks];
    const int tid = threadIdx.x;
    for (int k = tid; k < (int)kMaxSym; k += kThreads) hist[k] = 0;
    if (tid < kTileChunks) ocnt[tid] = 0;
    __syncthreads();

    const float *__restrict__ x = tc.x;
    const uint32_t numel = tc.numel, H = tc.shape[2], W = tc.shape[3], HW = H * W;
    uint16_t *__restrict__ sym = b.sym + (uint64_t)tc.chunk_base * kChunk;
    const int R = (int)b.radius;
    const float r = tc.r;
    const uint64_t tile0 = (uint64_t)blockIdx.x * kTile;
    uint32_t events = 0;

    for (int it = 0; it < kTile / (kThreads * 4); ++it) {
        const uint64_t i64 = tile0 + (uint64_t)it * (kThreads * 4) + (uint64_t)tid * 4;
        if (i64 >= numel) continue;
        const uint32_t i0 = (uint32_t)i64;
        const uint32_t nval = (numel - i0 >= 4) ? 4u : (numel - i0);

        float xv[4];
        if (nval == 4) {
            const float4 v = *reinterpret_cast<const float4 *>(x + i0);
            xv[0] = v.x; xv[1] = v.y; xv[2] = v.z; xv[3] = v.w;
        } else {
            for (uint32_t j = 0; j < 4; ++j) xv[j] = (j < nval) ? x[i0 + j] : 0.0f;
        }
        uint32_t rem = i0 % HW;
        uint32_t h = rem / W, w = rem - h * W;

        int q[4], up[4];
        uint32_t s[4];
        uint32_t nout = 0;
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) {
            if (j < nval) {
                const uint32_t i = i0 + j;
                q[j] = quant(xv[j], r);
                events += clamps(xv[j], r) ? 1u : 0u;
                up[j] = (h > 0) ? quant(x[i - W], r) : 0;
                int left = 0, diag = 0;
                if (w > 0) {
                    left = (j > 0) ? q[j - 1] : quant(x[i - 1], r);
                    if (h > 0) diag = (j > 0) ? up[j - 1] : quant(x[i - W - 1], r);
                }
                const int d = q[j] - left - up[j] + diag;
                const bool in = (d > -R) && (d < R);
                s[j] = in ? (uint32_t)(d + R) : 0u;
                nout += in ? 0u : 1u;
                // advance plane coordinates
                if (++w == W) { w = 0; if (++h == H) h = 0; }
            } else {
                q[j] = 0; up[j] = 0; s[j] = 0xffffffffu;
            }
        }
        if (nval == 4) {
            uint2 pk;
            pk.x = s[0] | (s[1] << 16);
            pk.y = s[2] | (s[3] << 16);
            *reinterpret_cast<uint2 *>(sym + i0) = pk;
        } else {
            for (uint32_t j = 0; j < nval; ++j) sym[i0 + j] = (uint16_t)s[j];
        }
        // Histogram in LDS.  Post-ReLU tensors are mostly runs of the zero residual, so
        // lanes whose four symbols are all R are counted with one ballot per wave.
        const bool all_mode = (s[0] == (uint32_t)R) && (s[1] == (uint32_t)R) &&
                              (s[2] == (uint32_t)R) && (s[3] == (uint32_t)R);
        const unsigned long long m = __ballot(all_mode);
        // Version 2: the zero residuals of a sub-block that holds nothing else are not counted.  A
        // sub-block is sub/4 neighbouring lanes; lanes past the end of the tensor are not here and
        // count as empty.
        bool counted = true;
        if (b.zero_blocks) {
            bool az = true;
#pragma unroll
            for (uint32_t j = 0; j < 4; ++j) az = az && (s[j] == (uint32_t)R || s[j] == 0xffffffffu);
            const unsigned long long zm = __ballot(az) | ~__ballot(true);
            const uint32_t g = b.sub / 4u, ln = (uint32_t)__lane_id();
            const unsigned long long grp = ((1ull << g) - 1ull) << (ln & ~(g - 1u));
            counted = (zm & grp) != grp;
        }
        if (!counted) {
            // nothing to count
        } else if (all_mode) {
            if (b.zero_blocks) atomicAdd(&hist[R], 4u);          // (the lanes counted together may not all be counted)
            else if ((int)(__lane_id()) == __ffsll((long long)m) - 1) atomicAdd(&hist[R], 4u * (uint32_t)__popcll(m));
        } else {
            uint32_t run = 1;
#pragma unroll
            for (uint32_t j = 1; j < 4; ++j) {
                if (s[j] == s[j - 1]) { ++run; }
                else {
                    if (s[j - 1] != 0xffffffffu) atomicAdd(&hist[s[j - 1]], run);
                    run = 1;
                }
            }
            if (s[3] != 0xffffffffu) atomicAdd(&hist[s[3]], run);
        }
        if (nout) atomicAdd(&ocnt[it / 4], nout);
    }
    __syncthreads();
    for (int k = tid; k < (int)kMaxSym; k += kThreads) {
        const uint32_t c = hist[k];
        if (c) atomicAdd(&b.hist[((uint64_t)ti * kHistCopies + blockIdx.x % kHistCopies) * kMaxSym + k], c);
    }
    if (tid < kTileChunks) {
        const uint64_t c = (uint64_t)blockIdx.x * kTileChunks + tid;
        if (c < tc.nchunks) {
            b.outl_cnt[tc.chunk_base + c] = ocnt[tid];
            for (int k = 0; k < 4; ++k) b.wide[(tc.chunk_base + c) * 4 + k] = 1;      // always 16-bit symbols
        }
    }
    // range events: one atomic per wave
    for (int o = 32; o > 0; o >>= 1) events += __shfl_down(events, o);
    if ((tid & 63) == 0 && events) atomicAdd(&b.tmeta[ti].range_events, events);
}

}  // namespace

void launch_sweep1_untiled(const BatchC &b, uint32_t t, Profiler *prof, hipStream_t st)
{
    const uint32_t tiles = (b.t[t].nchunks + kTileChunks - 1) / kTileChunks;
    if (tiles) launch(prof, kKQuantLorenzoHist, k_quant_lorenzo_split_hist, dim3(tiles), dim3(kThreads), st, b, t);
}

}  // namespace cmpz
