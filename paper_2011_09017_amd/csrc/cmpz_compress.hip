// Compression kernels: pre-quantisation + 2D Lorenzo + split + histogram (one
// sweep over x), per-chunk bit counts, offset scan + header, chunked Huffman
// bit-packing, outlier records.  The codebook kernel lives in cmpz_codebook.hip.
//
// The tensor is treated as one linear array: element i of plane p = i / (H*W)
// has neighbours i-1, i-W and i-W-1 in the same plane, so a workgroup can own a
// chunk-aligned linear range whatever H and W are.
#include "cmpz_internal.h"

namespace cmpz {
namespace {

constexpr int kThreads    = 256;
constexpr int kTileChunks = 4;                       // chunks per workgroup in the first sweep
constexpr int kTile       = kTileChunks * kChunk;    // 16384 elements

// Pre-quantisation of one value (Section 3.1, first stage): one fp32 multiply,
// clamp to +-16384 (NaN -> 0), round half to even (v_rndne_f32).
__device__ __forceinline__ int quant(float x, float r)
{
    float t = x * r;
    if (!(fabsf(t) <= (float)kQMax)) t = (t != t) ? 0.0f : copysignf((float)kQMax, t);
    return (int)__builtin_rintf(t);
}
__device__ __forceinline__ bool clamps(float x, float r)
{
    float t = x * r;
    return !(fabsf(t) <= (float)kQMax);
}

// Lorenzo residual of element i at plane coordinates (h, w), from x alone.
__device__ __forceinline__ int delta_from_x(const float *__restrict__ x, uint32_t i, uint32_t h,
                                            uint32_t w, uint32_t W, float r)
{
    int q = quant(x[i], r);
    int left = (w > 0) ? quant(x[i - 1], r) : 0;
    int up = (h > 0) ? quant(x[i - W], r) : 0;
    int diag = (h > 0 && w > 0) ? quant(x[i - W - 1], r) : 0;
    return q - left - up + diag;
}

// ---------------------------------------------------------------------------
// Sweep 1: x -> symbols (u16 scratch), histogram, outliers per chunk, range events.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_quant_lorenzo_split_hist(CompressArgs a)
{
    __shared__ uint32_t hist[kMaxSym];
    __shared__ uint32_t ocnt[kTileChunks];
    const int tid = threadIdx.x;
    for (int k = tid; k < (int)kMaxSym; k += kThreads) hist[k] = 0;
    if (tid < kTileChunks) ocnt[tid] = 0;
    __syncthreads();

    const float *__restrict__ x = a.x;
    const uint32_t numel = a.numel, W = a.W, H = a.H, HW = a.HW;
    const int R = (int)a.radius;
    const float r = a.r;
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
            *reinterpret_cast<uint2 *>(a.sym + i0) = pk;
        } else {
            for (uint32_t j = 0; j < nval; ++j) a.sym[i0 + j] = (uint16_t)s[j];
        }
        // Histogram in LDS.  Post-ReLU tensors are mostly runs of the zero residual, so
        // lanes whose four symbols are all R are counted with one ballot per wave.
        const bool all_mode = (s[0] == (uint32_t)R) && (s[1] == (uint32_t)R) &&
                              (s[2] == (uint32_t)R) && (s[3] == (uint32_t)R);
        const unsigned long long m = __ballot(all_mode);
        if (all_mode) {
            if ((int)(__lane_id()) == __ffsll((long long)m) - 1) atomicAdd(&hist[R], 4u * (uint32_t)__popcll(m));
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
        if (c) atomicAdd(&a.hist[k], c);
    }
    if (tid < kTileChunks) {
        const uint64_t c = (uint64_t)blockIdx.x * kTileChunks + tid;
        if (c < a.lay.nchunks) a.outl_cnt[c] = ocnt[tid];
    }
    // range events: one atomic per wave
    for (int o = 32; o > 0; o >>= 1) events += __shfl_down(events, o);
    if ((tid & 63) == 0 && events) atomicAdd(&a.meta[kMetaRangeEvents], events);
}

// ---------------------------------------------------------------------------
// Per-chunk bit counts: sub_bits (into the container) and the chunk's payload
// size in 16-byte units (scratch).  One workgroup per chunk, 16 symbols a thread.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void load16(const uint16_t *__restrict__ sym, uint64_t i0, uint32_t numel,
                                       uint32_t s[16])
{
    if (i0 + 16 <= numel) {
        const uint4 a = *reinterpret_cast<const uint4 *>(sym + i0);
        const uint4 b = *reinterpret_cast<const uint4 *>(sym + i0 + 8);
        const uint32_t wds[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) { s[2 * j] = wds[j] & 0xffffu; s[2 * j + 1] = wds[j] >> 16; }
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) s[j] = (i0 + j < numel) ? sym[i0 + j] : 0xffffffffu;
    }
}

__global__ __launch_bounds__(kThreads) void k_chunk_bits(CompressArgs a)
{
    __shared__ __align__(16) uint8_t lens[kMaxSym];
    __shared__ uint32_t wave_sum[kThreads / kWave];
    const int tid = threadIdx.x;
    for (int k = tid; k < (int)kMaxSym / 4; k += kThreads)
        reinterpret_cast<uint32_t *>(lens)[k] = reinterpret_cast<const uint32_t *>(a.lens)[k];
    __syncthreads();

    const uint32_t c = blockIdx.x;
    const uint64_t i0 = (uint64_t)c * kChunk + (uint64_t)tid * 16;
    uint32_t s[16];
    load16(a.sym, i0, a.numel, s);
    uint32_t bits = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) bits += (s[j] != 0xffffffffu) ? lens[s[j]] : 0u;

    // sub-block totals: `sub/16` consecutive lanes form one sub-block
    const uint32_t group = a.sub / 16;              // 2, 4, 8 or 16
    uint32_t g = bits;
    for (uint32_t o = 1; o < group; o <<= 1) g += __shfl_xor(g, o);
    if ((tid & (group - 1)) == 0) {
        uint16_t *sub_bits = reinterpret_cast<uint16_t *>(a.out + a.lay.off_sub_bits);
        sub_bits[(uint64_t)c * a.lay.nsub + tid / group] = (uint16_t)g;
    }
    uint32_t t = bits;
    for (int o = 32; o > 0; o >>= 1) t += __shfl_down(t, o);
    if ((tid & 63) == 0) wave_sum[tid >> 6] = t;
    __syncthreads();
    if (tid == 0) {
        const uint32_t total = wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
        a.chunk_units[c] = (total + 127u) / 128u;
    }
}

// ---------------------------------------------------------------------------
// Exclusive scans of chunk sizes and outlier counts into the container, then the
// header.  One workgroup of 1024 threads walks the chunks in slabs.
// ---------------------------------------------------------------------------
constexpr int kScanThreads = 1024;

__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_tot, uint32_t &total)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    uint32_t inc = v;
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t n = __shfl_up(inc, o);
        if (lane >= o) inc += n;
    }
    __syncthreads();                      // wave_tot may still be read from the previous call
    if (lane == 63) wave_tot[wv] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
    for (int k = 0; k < (int)(blockDim.x >> 6); ++k) {
        const uint32_t t = wave_tot[k];
        if (k < wv) base += t;
        tot += t;
    }
    total = tot;
    return base + inc - v;
}

__global__ __launch_bounds__(kScanThreads) void k_scan_header(CompressArgs a)
{
    __shared__ uint32_t wave_tot[kScanThreads / kWave];
    const int tid = threadIdx.x;
    const uint32_t nchunks = a.lay.nchunks;
    uint32_t *chunk_off = reinterpret_cast<uint32_t *>(a.out + a.lay.off_chunk_off);
    uint32_t *outl_off = reinterpret_cast<uint32_t *>(a.out + a.lay.off_outl_off);

    uint64_t carry_units = 0;
    uint32_t carry_outl = 0;
    uint64_t bits_total = 0;
    // entries nchunks .. pad4(nchunks+1)-1: the end marker and zero padding
    const uint32_t padded = (nchunks + 1 + 3) & ~3u;
    for (uint32_t base = 0; base < padded; base += kScanThreads) {
        const uint32_t c = base + tid;
        const uint32_t u = (c < nchunks) ? a.chunk_units[c] : 0u;
        const uint32_t o = (c < nchunks) ? a.outl_cnt[c] : 0u;
        uint32_t tu, to;
        const uint32_t eu = block_exclusive_scan(u, wave_tot, tu);
        const uint32_t eo = block_exclusive_scan(o, wave_tot, to);
        if (c < padded) {
            // offsets are u32 in the format; a payload of 2^32 units cannot occur below 2^32 codes
            chunk_off[c] = (c <= nchunks) ? (uint32_t)(carry_units + eu) : 0u;
            outl_off[c] = (c <= nchunks) ? carry_outl + eo : 0u;
        }
        carry_units += tu;
        carry_outl += to;
    }
    // total_bits = sum of sub_bits (read back from the container section just written by k_chunk_bits)
    {
        const uint16_t *sub_bits = reinterpret_cast<const uint16_t *>(a.out + a.lay.off_sub_bits);
        const uint64_t n = (uint64_t)nchunks * a.lay.nsub;
        uint64_t acc = 0;
        for (uint64_t k = tid; k < n; k += kScanThreads) acc += sub_bits[k];
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o);
        __shared__ uint64_t wave_bits[kScanThreads / kWave];
        if ((tid & 63) == 0) wave_bits[tid >> 6] = acc;
        __syncthreads();
        if (tid == 0) for (int k = 0; k < kScanThreads / kWave; ++k) bits_total += wave_bits[k];
    }
    if (tid == 0) {
        const uint64_t n_out = carry_outl;
        const uint64_t off_outl_idx = a.lay.off_payload + carry_units * 16;
        const uint64_t sect = (4 * n_out + 15) & ~15ull;
        const uint64_t off_outl_val = off_outl_idx + sect;
        const uint64_t total = off_outl_val + sect;
        const bool fits = total <= a.out_cap;
        Header hd;
        uint32_t *raw = reinterpret_cast<uint32_t *>(&hd);
        for (uint32_t k = 0; k < kHeaderBytes / 4; ++k) raw[k] = 0;
        hd.magic = kMagic; hd.version = kVersion; hd.status = fits ? 0u : kStNoSpace;
        hd.eb_bits = a.eb_bits;
        for (int k = 0; k < 4; ++k) hd.shape[k] = a.shape[k];
        hd.numel = a.numel;
        hd.radius = a.radius; hd.chunk = kChunk; hd.sub = a.sub; hd.guard_shift = a.guard_shift;
        hd.nchunks = nchunks; hd.n_outliers = (uint32_t)n_out;
        hd.range_events = a.meta[kMetaRangeEvents]; hd.max_len = a.meta[kMetaMaxLen];
        hd.total_bits = bits_total;
        hd.off_lens = a.lay.off_lens; hd.off_chunk_off = a.lay.off_chunk_off;
        hd.off_outl_off = a.lay.off_outl_off; hd.off_sub_bits = a.lay.off_sub_bits;
        hd.off_payload = a.lay.off_payload; hd.off_outl_idx = off_outl_idx;
        hd.off_outl_val = off_outl_val; hd.total_size = total;
        uint32_t *dst = reinterpret_cast<uint32_t *>(a.out);
        for (uint32_t k = 0; k < kHeaderBytes / 4; ++k) dst[k] = raw[k];
        uint32_t st = 0;
        if (!fits) st |= kStNoSpace;
        if (hd.range_events) st |= kStRange;
        if (st) atomicOr(a.status, st);
        a.meta[kMetaSkip] = fits ? 0u : 1u;
        a.meta[kMetaNOutliers] = (uint32_t)n_out;
        a.meta[kMetaRangeEvents] = 0;          // ready for the next call
    }
}

// ---------------------------------------------------------------------------
// Chunked Huffman bit-packing.  One workgroup per chunk: every thread packs its
// 16 codewords at its bit offset into a zeroed LDS image of the chunk, which is
// then copied out with 128-bit stores.  Bit k of the chunk is bit 31-(k%32) of
// little-endian word k/32.
// ---------------------------------------------------------------------------
constexpr uint32_t kChunkImageWords = kChunk * kMaxCodeLen / 32;   // 6144 words = 24 KB

__global__ __launch_bounds__(kThreads) void k_encode(CompressArgs a)
{
    __shared__ uint64_t codes[kMaxSym];
    __shared__ __align__(16) uint32_t image[kChunkImageWords];
    __shared__ uint32_t wave_tot[kThreads / kWave];
    if (a.meta[kMetaSkip]) return;
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    const uint32_t *chunk_off = reinterpret_cast<const uint32_t *>(a.out + a.lay.off_chunk_off);
    const uint32_t u0 = chunk_off[c], u1 = chunk_off[c + 1];
    const uint32_t nwords = (u1 - u0) * 4;
    if (u1 < u0 || nwords > kChunkImageWords) return;   // cannot happen for counts below 2^32

    for (int k = tid; k < (int)kMaxSym; k += kThreads) codes[k] = a.codes[k];
    for (uint32_t k = tid; k < nwords; k += kThreads) image[k] = 0;

    const uint64_t i0 = (uint64_t)c * kChunk + (uint64_t)tid * 16;
    uint32_t s[16];
    load16(a.sym, i0, a.numel, s);
    __syncthreads();

    uint64_t cw[16];
    uint32_t bits = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        cw[j] = (s[j] != 0xffffffffu) ? codes[s[j]] : 0ull;
        bits += (uint32_t)(cw[j] >> 56);
    }
    uint32_t total;
    uint32_t pos = block_exclusive_scan(bits, wave_tot, total);

    // Append codewords MSB-first.  `acc` holds the bits of word `wi` and the next one,
    // left-aligned; `fill` counts the valid bits in it.
    uint32_t wi = pos >> 5;
    uint32_t fill = pos & 31;
    uint64_t acc = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        uint32_t len = (uint32_t)(cw[j] >> 56);
        const uint64_t code = cw[j] & 0x00ffffffffffffffull;
        if (len > 32) {                                     // rare: split off the high part
            const uint32_t hl = len - 32;
            acc |= (code >> 32) << (64 - fill - hl);
            fill += hl;
            if (fill >= 32) { atomicOr(&image[wi], (uint32_t)(acc >> 32)); acc <<= 32; fill -= 32; ++wi; }
            len = 32;
        }
        if (len) {
            acc |= (code & 0xffffffffull) << (64 - fill - len);
            fill += len;
            if (fill >= 32) { atomicOr(&image[wi], (uint32_t)(acc >> 32)); acc <<= 32; fill -= 32; ++wi; }
        }
    }
    if (fill && (uint32_t)(acc >> 32)) atomicOr(&image[wi], (uint32_t)(acc >> 32));
    __syncthreads();

    uint4 *dst = reinterpret_cast<uint4 *>(a.out + a.lay.off_payload + (uint64_t)u0 * 16);
    const uint4 *src = reinterpret_cast<const uint4 *>(image);
    for (uint32_t k = tid; k < u1 - u0; k += kThreads) dst[k] = src[k];
}

// ---------------------------------------------------------------------------
// Outlier records (index, residual), ascending by index.  One workgroup per
// chunk that holds outliers: rank the zero symbols, recompute their residual
// from x, store at outl_off[c] + rank.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_outliers(CompressArgs a)
{
    __shared__ uint32_t wave_tot[kThreads / kWave];
    if (a.meta[kMetaSkip]) return;
    const int tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    const uint32_t *outl_off = reinterpret_cast<const uint32_t *>(a.out + a.lay.off_outl_off);
    const uint32_t n_out = a.meta[kMetaNOutliers];
    const Header *hd = reinterpret_cast<const Header *>(a.out);
    uint32_t *oidx = reinterpret_cast<uint32_t *>(a.out + hd->off_outl_idx);
    int32_t *oval = reinterpret_cast<int32_t *>(a.out + hd->off_outl_val);
    if (c == 0 && tid < 4) {                       // zero padding of both sections
        const uint32_t k = n_out + tid;
        if (k < ((n_out + 3) & ~3u)) { oidx[k] = 0; oval[k] = 0; }
    }
    const uint32_t o0 = outl_off[c], o1 = outl_off[c + 1];
    if (o0 == o1) return;

    const uint64_t i0 = (uint64_t)c * kChunk + (uint64_t)tid * 16;
    uint32_t s[16];
    load16(a.sym, i0, a.numel, s);
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) mine += (s[j] == 0u) ? 1u : 0u;
    uint32_t total;
    uint32_t rank = block_exclusive_scan(mine, wave_tot, total);
    if (!mine) return;
    for (int j = 0; j < 16; ++j) {
        if (s[j] != 0u) continue;
        const uint32_t i = (uint32_t)i0 + j;
        const uint32_t rem = i % a.HW;
        const uint32_t h = rem / a.W, w = rem - h * a.W;
        oidx[o0 + rank] = i;
        oval[o0 + rank] = delta_from_x(a.x, i, h, w, a.W, a.r);
        ++rank;
    }
}

// Empty tensor: the container is header + zero lens + two one-entry offset tables.
__global__ void k_empty_container(CompressArgs a)
{
    const uint32_t tid = threadIdx.x;
    const uint64_t total = a.lay.off_payload;
    uint32_t *dst = reinterpret_cast<uint32_t *>(a.out);
    for (uint64_t k = tid; k < total / 4; k += blockDim.x) dst[k] = 0;
    __syncthreads();
    if (tid == 0) {
        Header *hd = reinterpret_cast<Header *>(a.out);
        hd->magic = kMagic; hd->version = kVersion; hd->eb_bits = a.eb_bits;
        for (int k = 0; k < 4; ++k) hd->shape[k] = a.shape[k];
        hd->radius = a.radius; hd->chunk = kChunk; hd->sub = a.sub; hd->guard_shift = a.guard_shift;
        hd->off_lens = a.lay.off_lens; hd->off_chunk_off = a.lay.off_chunk_off;
        hd->off_outl_off = a.lay.off_outl_off; hd->off_sub_bits = a.lay.off_sub_bits;
        hd->off_payload = total; hd->off_outl_idx = total; hd->off_outl_val = total;
        hd->total_size = total;
    }
}

}  // namespace

void launch_compress(const CompressArgs &a, Profiler *prof, hipStream_t st)
{
    if (a.numel == 0) {
        launch(prof, kKEmpty, k_empty_container, dim3(1), dim3(256), st, a);
        return;
    }
    const uint32_t nchunks = a.lay.nchunks;
    const uint32_t tiles = (nchunks + kTileChunks - 1) / kTileChunks;
    launch(prof, kKQuantLorenzoHist, k_quant_lorenzo_split_hist, dim3(tiles), dim3(kThreads), st, a);
    launch_codebook(a, prof, st);
    launch(prof, kKChunkBits, k_chunk_bits, dim3(nchunks), dim3(kThreads), st, a);
    launch(prof, kKScanHeader, k_scan_header, dim3(1), dim3(kScanThreads), st, a);
    launch(prof, kKEncode, k_encode, dim3(nchunks), dim3(kThreads), st, a);
    launch(prof, kKOutliers, k_outliers, dim3(nchunks), dim3(kThreads), st, a);
}

}  // namespace cmpz
