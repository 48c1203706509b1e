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
        if (c) atomicAdd(&a.hist[(blockIdx.x % kHistCopies) * kMaxSym + k], c);
    }
    if (tid < kTileChunks) {
        const uint64_t c = (uint64_t)blockIdx.x * kTileChunks + tid;
        if (c < a.lay.nchunks) {
            a.outl_cnt[c] = ocnt[tid];
            if (c % a.tile_chunks == 0) a.desc[c / a.tile_chunks] = 0;     // re-arm the encode sweep's scan
        }
    }
    // range events: one atomic per wave
    for (int o = 32; o > 0; o >>= 1) events += __shfl_down(events, o);
    if ((tid & 63) == 0 && events) atomicAdd(&a.meta[kMetaRangeEvents], events);
}

// 16 consecutive symbols of a chunk; positions past the tensor end read as "no symbol".
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

// exclusive prefix sum over the 256 threads of a workgroup (contains two barriers)
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_tot, uint32_t &total)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const uint32_t inc = wave_inclusive_sum(v);
    __syncthreads();                      // wave_tot may still be read from the previous call
    if (lane == 63) wave_tot[wv] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int k = 0; k < kThreads / kWave; ++k) {
        const uint32_t t = wave_tot[k];
        if (k < wv) base += t;
        tot += t;
    }
    total = tot;
    return base + inc - v;
}

__device__ __forceinline__ uint64_t desc_load(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void desc_store(uint64_t *p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Sum of a 62-bit descriptor value over the lanes selected by `take` (two 32-bit fields that
// cannot carry into each other: units stay below 2^30, outliers below 2^32).
__device__ __forceinline__ uint64_t wave_desc_sum(uint64_t d, bool take)
{
    const uint32_t lo = take ? (uint32_t)d : 0u, hi = take ? (uint32_t)((d & kDescMask) >> 32) : 0u;
    const uint32_t slo = (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_sum(lo), 63);
    const uint32_t shi = (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_sum(hi), 63);
    return ((uint64_t)shi << 32) | slo;
}

constexpr uint32_t kSpinLimit = 1u << 22;          // polls before a look-back gives up

// Exclusive prefix (units, outliers) of tile c from the descriptors of its predecessors;
// one wave, every lane inspects one predecessor per round (single-pass scan with look-back).
// Tiles are handed out in index order, so every predecessor is owned by a workgroup that
// is already running and publishes without waiting on anyone: the wait always ends.  The
// poll limit only guards against a defect; on expiry *failed is set and 0 returned.
// Starts at predecessor j with `excl` already summed over the tiles above j.
__device__ __forceinline__ uint64_t look_back_from(const uint64_t *desc, int64_t j, uint64_t excl, int lane, bool *failed)
{
    uint32_t spins = 0;
    while (j >= 0) {
        const int64_t idx = j - lane;
        const uint64_t d = (idx >= 0) ? desc_load(desc + idx) : kDescPrefix;   // before tile 0: prefix 0
        const uint32_t state = (uint32_t)(d >> 62);
        const unsigned long long inv = __ballot(state == 0);
        const unsigned long long pre = __ballot(state == 2);
        const int first_inv = inv ? __ffsll((long long)inv) - 1 : 64;
        const int first_pre = pre ? __ffsll((long long)pre) - 1 : 64;
        if (first_pre < first_inv) {               // aggregates up to a published prefix: done
            excl += wave_desc_sum(d, lane <= first_pre);
            break;
        }
        if (first_inv > 0) {                       // a run of aggregates: take them, look further back
            excl += wave_desc_sum(d, lane < first_inv);
            j -= first_inv;
            continue;
        }
        if (++spins > kSpinLimit) { *failed = true; return 0; }
        __builtin_amdgcn_s_sleep(2);
    }
    return excl;
}

// The descriptors of the kSnapRounds * 64 nearest predecessors of tile c, fetched in one go.  The
// loads are issued where the snapshot is taken and their latency passes while the workgroup
// packs; what the snapshot cannot settle (a predecessor that had not published yet, or no
// prefix that near) is looked up again when the offset is needed.
constexpr int kSnapRounds = 2;
struct DescSnapshot {
    uint64_t d[kSnapRounds];
};
__device__ __forceinline__ DescSnapshot look_back_snapshot(const uint64_t *desc, uint32_t c, int lane)
{
    DescSnapshot sn;
#pragma unroll
    for (int r = 0; r < kSnapRounds; ++r) {
        const int64_t idx = (int64_t)c - 1 - r * kWave - lane;
        sn.d[r] = (idx >= 0) ? desc_load(desc + idx) : kDescPrefix;
    }
    return sn;
}
__device__ __forceinline__ uint64_t look_back_finish(const uint64_t *desc, uint32_t c, const DescSnapshot &sn, int lane,
                                                     bool *failed)
{
    uint64_t excl = 0;
    int64_t j = (int64_t)c - 1;
#pragma unroll
    for (int r = 0; r < kSnapRounds; ++r) {
        if (j < 0) return excl;
        const uint64_t d = sn.d[r];
        const uint32_t state = (uint32_t)(d >> 62);
        const unsigned long long inv = __ballot(state == 0);
        const unsigned long long pre = __ballot(state == 2);
        const int first_inv = inv ? __ffsll((long long)inv) - 1 : 64;
        const int first_pre = pre ? __ffsll((long long)pre) - 1 : 64;
        if (first_pre < first_inv) return excl + wave_desc_sum(d, lane <= first_pre);
        excl += wave_desc_sum(d, lane < first_inv);
        j -= first_inv;
        if (first_inv < 64) break;                 // not published when the snapshot was taken
    }
    return look_back_from(desc, j, excl, lane, failed);
}

// ---------------------------------------------------------------------------
// Sweep 2: chunked Huffman bit-packing with the bit offsets found on the fly.
// Workgroups take tiles of up to 8 consecutive chunks in index order from a
// ticket counter.  First the code lengths of a tile's symbols are summed
// (sub_bits, chunk sizes, the tile's size, which is published at once), then
// each chunk is packed into a zeroed LDS image (bit k of the chunk is bit
// 31-(k%32) of little-endian word k/32), which is copied out with 128-bit stores
// at the offset that wave 0 finds meanwhile by look-back.  While no codeword is
// longer than 27 bits (the usual case) the tile's symbols stay in registers
// between the two passes, a table entry is the left-aligned code with its length
// in the low bits, and a codeword is OR-ed into the image at its own bit position
// with two LDS atomics; longer codes take a slower path (symbols read twice, a
// 64-bit accumulator).  The workgroup that finishes last writes the header.
// ---------------------------------------------------------------------------
constexpr uint32_t kChunkImageWords = kChunk * kMaxCodeLen / 32;   // 6144 words = 24 KB
constexpr int kTileMax = 8;

template <int CTRL>
__device__ __forceinline__ uint32_t row_shr(uint32_t x) { return dpp_u32<CTRL, 0xf>(x); }

__device__ __forceinline__ uint32_t sym_at(const uint4 &lo, const uint4 &hi, int j)
{
    const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    const uint32_t v = w[j >> 1];
    return (j & 1) ? (v >> 16) : (v & 0xffffu);
}

// Append one codeword (len <= 32) to the thread's bit accumulator and flush full 32-bit
// words.  `acc` holds the bits of image word `wi` and the next one, left-aligned; `fill` < 32
// counts the valid bits.
__device__ __forceinline__ void append_bits(uint32_t *img, uint64_t &acc, uint32_t &fill, uint32_t &wi,
                                            uint32_t code, uint32_t len)
{
    acc |= ((uint64_t)code) << ((64u - fill - len) & 63u);        // len == 0 adds nothing (code == 0)
    fill += len;
    if (fill >= 32) {
        atomicOr(&img[wi], (uint32_t)(acc >> 32));
        acc <<= 32; fill -= 32; ++wi;
    }
}

// Per-chunk state of a tile lives in registers, chunk q in slot q.  The per-chunk loops below run
// un-unrolled over slot 0 and rotate the slots after each chunk, so the loop body exists once.
struct TileRegs {
    uint32_t pos[kTileMax];          // this thread's bit offset inside each chunk
    __device__ __forceinline__ void rotate()
    {
        const uint32_t p = pos[0];
#pragma unroll
        for (int q = 0; q + 1 < kTileMax; ++q) pos[q] = pos[q + 1];
        pos[kTileMax - 1] = p;
    }
};

constexpr uint32_t kPastEnd  = kMaxSym;      // symbol value of elements past the end of the tensor (codes to nothing)
constexpr uint32_t kShortMax = 27;           // longest codeword the 32-bit table entries can hold

#ifdef CMPZ_PHASE_CLOCKS
#define PHASE(k) if (tid == 0) { const long long now_ = clock64(); clk[k] += now_ - last_; last_ = now_; }
#else
#define PHASE(k)
#endif

__global__ __launch_bounds__(kThreads) void k_encode(CompressArgs a)
{
#ifdef CMPZ_PHASE_CLOCKS
    long long clk[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    long long last_ = clock64();
#endif
    __shared__ uint64_t table[kMaxSym + 1];          // length << 56 | code; or, as 32-bit words, code << (32 - length) | length
    __shared__ __align__(16) uint32_t image[kChunkImageWords + 4];
    __shared__ uint32_t wave_bits[kThreads / kWave][kTileMax];
    __shared__ uint32_t s_units[kTileMax];
    __shared__ uint32_t s_tile;
    __shared__ uint64_t s_excl;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const uint32_t nchunks = a.lay.nchunks, tc = a.tile_chunks;
    const uint32_t ntiles = (nchunks + tc - 1) / tc;
    uint32_t *chunk_off = reinterpret_cast<uint32_t *>(a.out + a.lay.off_chunk_off);
    uint32_t *outl_off = reinterpret_cast<uint32_t *>(a.out + a.lay.off_outl_off);
    uint16_t *sub_bits = reinterpret_cast<uint16_t *>(a.out + a.lay.off_sub_bits);
    const uint32_t group = a.sub / 16;               // lanes per sub-block: 2, 4 or 8
    const uint32_t *len_word = reinterpret_cast<const uint32_t *>(table) + 1;   // high words: length << 24 | ...

    uint32_t *table32 = reinterpret_cast<uint32_t *>(table);
    const bool short_codes = a.meta[kMetaMaxLen] <= kShortMax;       // uniform; written by the codebook kernel
    for (int k = tid; k <= (int)kMaxSym; k += kThreads) {
        const uint64_t e = (k < (int)kMaxSym) ? a.codes[k] : 0ull;
        const uint32_t len = (uint32_t)(e >> 56);
        if (short_codes) table32[k] = len ? (((uint32_t)e << (32u - len)) | len) : 0u;
        else table[k] = e;
    }
    uint64_t my_bits = 0;                            // thread 0: bits of the chunks this workgroup packed
    bool failed = false;
    TileRegs r;

    for (;;) {
        __syncthreads();                             // previous round is done with the LDS state
        if (tid == 0) s_tile = atomicAdd(&a.meta[kMetaTicket], 1u);
        __syncthreads();
        const uint32_t t = s_tile;
        PHASE(0)
        if (t >= ntiles) break;
        const uint32_t c0 = t * tc;
        const uint32_t nq = (nchunks - c0 < tc) ? nchunks - c0 : tc;     // chunks in this tile

        // 16 symbols of chunk c for this thread; elements past the end read as kPastEnd (the
        // symbol buffer holds whole chunks, so the loads themselves are always in bounds)
        auto load_syms = [&](uint32_t c, uint4 &lo, uint4 &hi) {
            const uint64_t i0 = (uint64_t)c * kChunk + (uint64_t)tid * 16;
            lo = *reinterpret_cast<const uint4 *>(a.sym + i0);
            hi = *reinterpret_cast<const uint4 *>(a.sym + i0 + 8);
            if (i0 + 16 > a.numel) {
                const uint32_t valid = (i0 < a.numel) ? (uint32_t)(a.numel - i0) : 0u;   // < 16
                auto fix = [&](uint32_t w, uint32_t j) -> uint32_t {                      // word j holds elements 2j, 2j+1
                    if (2 * j >= valid) return kPastEnd | (kPastEnd << 16);
                    if (2 * j + 1 >= valid) return (w & 0xffffu) | (kPastEnd << 16);
                    return w;
                };
                lo = make_uint4(fix(lo.x, 0), fix(lo.y, 1), fix(lo.z, 2), fix(lo.w, 3));
                hi = make_uint4(fix(hi.x, 4), fix(hi.y, 5), fix(hi.z, 6), fix(hi.w, 7));
            }
        };
#pragma unroll
        for (int q = 0; q < kTileMax; ++q) r.pos[q] = 0;
        // sums the code lengths of this thread's 16 symbols of chunk c0+q: sub-block bit counts,
        // the thread's bit offset within its wave, the wave's total
        auto lens_chunk = [&](int q, const uint4 &lo, const uint4 &hi, uint32_t &pos_out) {
            uint32_t bits = 0;
            if (short_codes) {
#pragma unroll
                for (int j = 0; j < 16; ++j) bits += table32[sym_at(lo, hi, j)] & 31u;
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j) bits += len_word[2 * sym_at(lo, hi, j)] >> 24;
            }
            const uint32_t inc = wave_inclusive_sum(bits);
            const uint32_t exc = inc - bits;
            // the first lane of a sub-block sits group-1 lanes below its last lane, in the same DPP row
            const uint32_t first_exc = (group == 8) ? row_shr<0x117>(exc) : (group == 4) ? row_shr<0x113>(exc)
                                                                                          : row_shr<0x111>(exc);
            if ((tid & (group - 1)) == group - 1)
                sub_bits[(uint64_t)(c0 + q) * a.lay.nsub + tid / group] = (uint16_t)(inc - first_exc);
            pos_out = exc;                           // completed below with the lower waves' bits
            if (lane == 63) wave_bits[wv][q] = inc;
        };
        uint4 sv[kTileMax][2];                       // short codes: the tile's symbols stay in registers
        uint4 lo, hi, nlo, nhi;                      // long codes: one chunk at a time, read again for the packing
        if (short_codes) {
#pragma unroll
            for (int q = 0; q < kTileMax; ++q)
                if (q < (int)nq) load_syms(c0 + q, sv[q][0], sv[q][1]);      // all in flight together
            PHASE(1)
#pragma unroll
            for (int q = 0; q < kTileMax; ++q)
                if (q < (int)nq) lens_chunk(q, sv[q][0], sv[q][1], r.pos[q]);
        } else {
            load_syms(c0, lo, hi);
            nlo = lo; nhi = hi;
#pragma unroll 1
            for (int q = 0; q < kTileMax; ++q) {
                if (q < (int)nq) {
                    if (q + 1 < (int)nq) load_syms(c0 + q + 1, nlo, nhi);    // in flight during this chunk
                    lens_chunk(q, lo, hi, r.pos[0]);
                    lo = nlo; hi = nhi;
                }
                r.rotate();
            }
            load_syms(c0, lo, hi);                   // second read of the tile, for the packing below
            nlo = lo; nhi = hi;
        }
        __syncthreads();
        uint32_t tile_units = 0;
#pragma unroll
        for (int q = 0; q < kTileMax; ++q) {
            if (q < (int)nq) {
                uint32_t base = 0, tot = 0;
#pragma unroll
                for (int k = 0; k < kThreads / kWave; ++k) {
                    const uint32_t w = wave_bits[k][q];
                    if (k < wv) base += w;
                    tot += w;
                }
                r.pos[q] += base;
                const uint32_t u = (tot + 127u) / 128u;
                tile_units += u;
                if (tid == 0) { my_bits += tot; s_units[q] = u; }
            }
        }
        PHASE(2)
        // ---- publish the tile's size and fetch the predecessors' descriptors; the tile's offset is
        //      settled from them later, by wave 0, while the workgroup is packing ----
        DescSnapshot snap;
        uint32_t oc = 0, oinc = 0, tile_outl = 0;
        bool settled = false;                        // wave 0: s_excl and the offset tables are written
        if (wv == 0) {
            oc = (lane < (int)nq) ? a.outl_cnt[c0 + lane] : 0u;
            oinc = wave_inclusive_sum(oc);
            tile_outl = (uint32_t)__builtin_amdgcn_readlane((int)oinc, 63);
            const uint64_t own = ((uint64_t)tile_units << 32) | tile_outl;
            if (lane == 0) desc_store(a.desc + t, kDescAgg | own);
            snap = look_back_snapshot(a.desc, t, lane);
        }
        auto settle = [&]() {                        // wave 0 only
            if (settled) return;
            settled = true;
            const uint64_t own = ((uint64_t)tile_units << 32) | tile_outl;
            const uint64_t excl = look_back_finish(a.desc, t, snap, lane, &failed);
            if (lane == 0) {
                s_excl = excl;
                // publish the inclusive prefix even after a failure so that successors do not wait
                desc_store(a.desc + t, kDescPrefix | ((excl + own) & kDescMask));
            }
            // where the tile's chunks and their outlier records start
            const uint32_t uq = (lane < (int)nq) ? s_units[lane] : 0u;
            const uint32_t uinc = wave_inclusive_sum(uq);
            if (lane < (int)nq) {
                outl_off[c0 + lane] = (uint32_t)excl + oinc - oc;
                chunk_off[c0 + lane] = (uint32_t)(excl >> 32) + uinc - uq;
            }
            if (c0 + nq == nchunks && lane == 0) {
                // end markers, zero padding of both tables, and the totals for the header
                const uint32_t padded = (nchunks + 1 + 3) & ~3u;
                const uint32_t tot_u = (uint32_t)(excl >> 32) + tile_units, tot_o = (uint32_t)excl + tile_outl;
                chunk_off[nchunks] = tot_u;
                outl_off[nchunks] = tot_o;
                for (uint32_t k = nchunks + 1; k < padded; ++k) { chunk_off[k] = 0; outl_off[k] = 0; }
                a.meta[kMetaTotalUnits] = tot_u;
                a.meta[kMetaNOutliers] = tot_o;
            }
        };

        PHASE(3)
        // ---- pack and store: consecutive chunks share the LDS image while they fit ----
        constexpr uint32_t kImageUnits = kChunkImageWords / 4;
        uint32_t u_img = 0;                          // units packed into the image and not yet stored
        uint32_t u_done = 0;                         // units of the tile already stored
        uint32_t left = tile_units;                  // units of the tile not yet packed
        auto zero_image = [&]() {
            const uint32_t nw = (left < kImageUnits ? left : kImageUnits) * 4;
            for (uint32_t k = tid; k < nw; k += kThreads) image[k] = 0;
        };
        auto store_image = [&]() {                   // between two barriers issued by the caller
            const uint32_t u0 = (uint32_t)(s_excl >> 32) + u_done;
            const uint64_t end = a.lay.off_payload + ((uint64_t)u0 + u_img) * 16;
            if (end <= a.out_cap) {
                uint4 *dst = reinterpret_cast<uint4 *>(a.out + a.lay.off_payload + (uint64_t)u0 * 16);
                const uint4 *src = reinterpret_cast<const uint4 *>(image);
                for (uint32_t k = tid; k < u_img; k += kThreads) dst[k] = src[k];
            }
            u_done += u_img;
            u_img = 0;
        };
        zero_image();
        __syncthreads();                             // also makes s_units visible
        // packs chunk c0+q into the image at this thread's bit offset pos_q
        auto pack_chunk = [&](int q, const uint4 &lo, const uint4 &hi, uint32_t pos_q) {
            const uint32_t uq = s_units[q];
            if (uq > kImageUnits) { failed = true; return; }          // cannot happen for counts below 2^32
            if (u_img + uq > kImageUnits) {          // image full: store it and start afresh
                if (wv == 0) settle();
                __syncthreads();
                store_image();
                __syncthreads();
                zero_image();
                __syncthreads();
            }
            const uint32_t p0 = u_img * 128u + pos_q;                 // bit position in the image
            if (short_codes) {
                uint32_t pos = p0;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const uint32_t e = table32[sym_at(lo, hi, j)];
                    const uint32_t code = e & ~31u, o = pos & 31u;    // left-aligned code
                    uint32_t *w = image + (pos >> 5);
                    atomicOr(w, code >> o);
                    atomicOr(w + 1, __builtin_amdgcn_alignbit(code, 0u, o));   // the part that spills over
                    pos += e & 31u;
                }
            } else {
                uint32_t wi = p0 >> 5, fill = p0 & 31;
                uint64_t acc = 0;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const uint64_t cw = table[sym_at(lo, hi, j)];
                    uint32_t len = (uint32_t)(cw >> 56);
                    if (len > 32) {                                   // rare: split off the high part
                        append_bits(image, acc, fill, wi, (uint32_t)((cw & 0x00ffffffffffffffull) >> 32), len - 32);
                        len = 32;
                    }
                    append_bits(image, acc, fill, wi, (uint32_t)cw, len);
                }
                if (fill && (uint32_t)(acc >> 32)) atomicOr(&image[wi], (uint32_t)(acc >> 32));
            }
            u_img += uq;
            left -= uq;
        };
        if (short_codes) {
#pragma unroll
            for (int q = 0; q < kTileMax; ++q) {
                if (q < (int)nq) pack_chunk(q, sv[q][0], sv[q][1], r.pos[q]);     // uniform
                if (q == 1 && wv == 0) settle();     // the descriptors have arrived by now; successors want the prefix
            }
        } else {
#pragma unroll 1
            for (int q = 0; q < kTileMax; ++q) {
                if (q < (int)nq) {
                    if (q + 1 < (int)nq) load_syms(c0 + q + 1, nlo, nhi);
                    pack_chunk(q, lo, hi, r.pos[0]);
                    lo = nlo; hi = nhi;
                }
                r.rotate();
            }
        }
        if (wv == 0) settle();
        PHASE(4)
        __syncthreads();                             // image complete, s_excl visible
        store_image();
        PHASE(5)
    }
#ifdef CMPZ_PHASE_CLOCKS
    if (tid == 0)
        for (int k = 0; k < 8; ++k)
            atomicAdd(reinterpret_cast<unsigned long long *>(a.meta + kMetaClocks) + 8 + k, (unsigned long long)clk[k]);
#endif

    // ---- the last workgroup to finish writes the header and re-arms the counters ----
    if (tid == 0) {
        unsigned long long *bits_acc = reinterpret_cast<unsigned long long *>(a.meta + kMetaBitsLo);
        if (my_bits) atomicAdd(bits_acc, (unsigned long long)my_bits);
        if (failed) atomicOr(a.status, kStInternal);
        __threadfence();
        const uint32_t done = atomicAdd(&a.meta[kMetaDone], 1u);
        if (done == gridDim.x - 1) {
            __threadfence();
            const uint64_t total_units = __hip_atomic_load(&a.meta[kMetaTotalUnits], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint64_t n_out = __hip_atomic_load(&a.meta[kMetaNOutliers], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint64_t bits_total = __hip_atomic_load(bits_acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t range_events = __hip_atomic_load(&a.meta[kMetaRangeEvents], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint64_t off_outl_idx = a.lay.off_payload + total_units * 16;
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
            hd.range_events = range_events; hd.max_len = a.meta[kMetaMaxLen];
            hd.total_bits = bits_total;
            hd.off_lens = a.lay.off_lens; hd.off_chunk_off = a.lay.off_chunk_off;
            hd.off_outl_off = a.lay.off_outl_off; hd.off_sub_bits = a.lay.off_sub_bits;
            hd.off_payload = a.lay.off_payload; hd.off_outl_idx = off_outl_idx;
            hd.off_outl_val = off_outl_val; hd.total_size = total;
            uint32_t *dst = reinterpret_cast<uint32_t *>(a.out);
            for (uint32_t k = 0; k < kHeaderBytes / 4; ++k) dst[k] = raw[k];
            uint32_t st = 0;
            if (!fits) st |= kStNoSpace;
            if (range_events) st |= kStRange;
            if (st) atomicOr(a.status, st);
            a.meta[kMetaSkip] = fits ? 0u : 1u;
            a.meta[kMetaRangeEvents] = 0;          // ready for the next call
            a.meta[kMetaTicket] = 0;
            a.meta[kMetaDone] = 0;
            *bits_acc = 0;
        }
    }
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

// Sweep 1 alone (nothing for an empty tensor).
void launch_compress_begin(const CompressArgs &a, Profiler *prof, hipStream_t st)
{
    if (a.numel == 0) return;
    const uint32_t tiles = (a.lay.nchunks + kTileChunks - 1) / kTileChunks;
    if (!launch_sweep1_tiled(a, prof, st))
        launch(prof, kKQuantLorenzoHist, k_quant_lorenzo_split_hist, dim3(tiles), dim3(kThreads), st, a);
}

// Codebook, sweep 2 and the outlier records, from what sweep 1 left in the scratch.
void launch_compress_finish(const CompressArgs &a, Profiler *prof, hipStream_t st)
{
    if (a.numel == 0) {
        launch(prof, kKEmpty, k_empty_container, dim3(1), dim3(256), st, a);
        return;
    }
    const uint32_t nchunks = a.lay.nchunks;
    launch_codebook(a, prof, st);
    const uint32_t ntiles = (nchunks + a.tile_chunks - 1) / a.tile_chunks;
    // every workgroup costs a ticket, a look-back over the tiles in flight and a code table load:
    // about one workgroup per 16 chunks, between one and two per CU.  Three would fit and are a
    // little faster when the kernel has the chip to itself; two leave registers for the first
    // sweep of another stream's tensor beside it, which is worth more.
    uint32_t egrid = nchunks / 16;
    egrid = egrid < 256u ? 256u : egrid > 512u ? 512u : egrid;
    egrid = egrid < ntiles ? egrid : ntiles;
    launch(prof, kKEncode, k_encode, dim3(egrid), dim3(kThreads), st, a);
    launch(prof, kKOutliers, k_outliers, dim3(nchunks), dim3(kThreads), st, a);
}

}  // namespace cmpz
