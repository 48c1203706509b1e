// Internal declarations shared by the HIP translation units of libcmpz.
// Nothing here is visible through the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

namespace cmpz {

constexpr int      kWave        = 64;       // CDNA wavefront
constexpr uint32_t kChunk       = 4096;     // codes per Huffman chunk (fixed on the GPU path)
constexpr uint32_t kMaxSym      = 1024;     // 2 * largest radius
constexpr int      kQMax        = 16384;    // clamp of the pre-quantised integer
constexpr uint32_t kHeaderBytes = 256;
// Largest array the kernels index with 32 bits: their loop counters step by up to 4096 past the
// last element before they compare, so the bound stays two such steps below 2^32.
constexpr uint64_t kMaxNumel    = (1ull << 32) - 8192;
constexpr uint32_t kMaxCodeLen  = 48;       // counts below 2^32 bound a Huffman depth by 45
constexpr uint32_t kVersion     = 1;        // every code is in the bit stream
constexpr uint32_t kVersionZB   = 2;        // sub-blocks of zero residuals are left out of it
constexpr uint32_t kHistCopies  = 8;        // global histogram replicas that workgroups flush into (less contention)

// Container header, little-endian, 256 bytes; bytes 144..255 are zero.
struct Header {
    uint32_t magic;            // "CMPZ"
    uint32_t version;
    uint32_t status;           // 0 = complete; 2 = ran out of room (total_size = bytes needed)
    uint32_t eb_bits;          // bit pattern of the user's fp32 error bound
    uint32_t shape[4];         // N, C, H, W
    uint64_t numel;
    uint32_t radius, chunk, sub, guard_shift;
    uint32_t nchunks, n_outliers, range_events, max_len;
    uint64_t total_bits;       // sum of codeword lengths, padding excluded
    uint64_t off_lens, off_chunk_off, off_outl_off, off_sub_bits, off_payload;
    uint64_t off_outl_idx, off_outl_val;
    uint64_t total_size;
    uint8_t  zero[112];
};
static_assert(sizeof(Header) == kHeaderBytes, "header layout");
constexpr uint32_t kMagic = 0x5A504D43u;    // 'C','M','P','Z' in memory order

// Section offsets that depend on shape and configuration only.
struct Layout {
    uint32_t nchunks, nsub;
    uint64_t off_lens, off_chunk_off, off_outl_off, off_sub_bits, off_payload;
};

// Device-side status bits (ctx->d_status), most severe wins on the host.
constexpr uint32_t kStRange    = 1u;
constexpr uint32_t kStNoSpace  = 2u;
constexpr uint32_t kStFormat   = 4u;
constexpr uint32_t kStMismatch = 8u;
constexpr uint32_t kStInternal = 16u;       // a bounded wait ran out (reported as CMP_E_HIP)

// Exact n / d for 32-bit n and d via one 64x32 high multiply (M = ceil(2^64 / d)).
struct FastDiv {
    uint32_t d, mhi, mlo;
    __host__ static FastDiv make(uint32_t d)
    {
        FastDiv f;
        f.d = d ? d : 1;
        const uint64_t m = f.d > 1 ? (~0ull / f.d) + 1 : 0;
        f.mhi = (uint32_t)(m >> 32);
        f.mlo = (uint32_t)m;
        return f;
    }
    __device__ __forceinline__ uint32_t div(uint32_t n) const
    {
        if (d == 1) return n;
        const uint64_t t = (uint64_t)mhi * n + __umulhi(mlo, n);
        return (uint32_t)(t >> 32);
    }
};

// Section offsets of a container that depend on the element count and the configuration only.
__host__ __device__ inline Layout make_layout(uint64_t numel, uint32_t radius, uint32_t sub)
{
    auto up16 = [](uint64_t v) { return (v + 15) & ~15ull; };
    Layout l;
    l.nchunks = (uint32_t)((numel + kChunk - 1) / kChunk);
    l.nsub = kChunk / sub;
    l.off_lens = kHeaderBytes;
    l.off_chunk_off = l.off_lens + up16(2ull * radius);
    l.off_outl_off = l.off_chunk_off + up16(4ull * ((uint64_t)l.nchunks + 1));
    l.off_sub_bits = l.off_outl_off + up16(4ull * ((uint64_t)l.nchunks + 1));
    l.off_payload = l.off_sub_bits + up16(2ull * (uint64_t)l.nchunks * l.nsub);
    return l;
}

// Scratch words in ctx->d_meta (decompression side).
enum MetaWord : int {
    kMetaBad         = 4,   // decompress: nonzero when the container failed validation
    kMetaWords       = 64
};

// ---- compression: one call handles a batch of tensors, every stage is one launch ----
//
// Chunks of all tensors of a call are numbered consecutively (tensor t owns the global chunks
// chunk_base .. chunk_base + nchunks - 1); the symbol scratch holds whole chunks, so tensor t's
// symbols start at element chunk_base * 4096.  The bit-count and packing kernels give a workgroup
// a range of kPackChunks consecutive chunks of one tensor; those ranges are numbered
// consecutively too (tensor t owns pack_base .. ).
constexpr int      kBatchMax   = 24;        // tensors per launch group (kernel arguments hold their descriptors)
constexpr uint32_t kPackChunks = 16;        // chunks per workgroup of the bit-count and packing kernels

// A stack of containers in one device buffer whose bookkeeping lives on the device: where the
// next container goes is known to the GPU only (it depends on the sizes of the containers before
// it), so the host can push tensor after tensor without ever waiting (cmp_arena_* in cmpz.h).
struct ArenaSlot { uint64_t offset, size; };   // size 0: not held (never pushed, failed, or popped)
struct ArenaState {
    uint64_t top;          // bytes in use: where the next container starts
    uint64_t peak;         // largest `top` so far
    uint32_t nslots;       // slots pushed and not yet given back (slots are numbered in push order)
    uint32_t failed;       // pushes that did not fit
    uint32_t slots_cap, pad;
    ArenaSlot slot[1];     // [slots_cap]
};
constexpr uint64_t kArenaAlign = 256;          // containers start at multiples of this

struct TensorC {
    const float *x;
    uint8_t     *out;
    uint64_t     out_cap;
    const ArenaState *arena;    // not NULL: the container goes to out + arena->top (out_cap counts from out)
    uint32_t     shape[4];
    uint32_t     numel, nchunks, chunk_base, eb_bits;
    float        r;
    uint32_t     sweep_base;    // first workgroup of this tensor in the first sweep
    uint32_t     pack_base;     // first chunk range of this tensor
    FastDiv      divW, divHW;
};

// Per tensor slot, written by the kernels of a call; range_events is zero between calls.
struct TensorMeta {
    uint32_t range_events;      // elements clamped by the pre-quantisation
    uint32_t max_len;           // longest codeword
    uint32_t skip;              // the container does not fit: nothing but the header is written
    uint32_t n_outliers;
    uint32_t total_units;       // payload size in 16-byte units
    uint32_t pad;
    uint64_t total_bits;
    uint64_t total_size;        // container bytes
};

// Where the container of a tensor goes and how much room there is.
struct OutRef { uint8_t *out; uint64_t cap; };
__device__ __forceinline__ OutRef resolve_out(const TensorC &tc)
{
    uint64_t at = tc.arena ? tc.arena->top : 0;
    if (at > tc.out_cap) at = tc.out_cap;
    OutRef o = {tc.out + at, tc.out_cap - at};
    return o;
}

struct BatchC {
    uint32_t n;                 // tensors of this launch group
    uint32_t radius, sub, guard_shift;
    uint32_t zero_blocks;       // 1: sub-blocks of zero residuals are not coded (container version 2)
    uint32_t sweep_chunks;      // chunks per workgroup in the first sweep
    uint32_t sweep_wgs, pack_wgs, total_chunks;
    // context scratch
    uint16_t   *sym;            // whole chunks of 4096 symbols, 8192 bytes apart.  Every quarter of a chunk (1024
                                // symbols, 2048 bytes apart) holds 16 bits per symbol or, if not marked wide,
                                // 8 bits (symbol - sym_off) in its first 1024 bytes
    uint32_t   *wide;           // [global chunk][quarter]: nonzero = 16-bit symbols
    uint32_t    sym_off;        // radius - 128 (0 for radii up to 128): byte b stands for symbol b + sym_off
    uint32_t   *hist;           // [slot][kHistCopies][kMaxSym], zero between calls
    uint32_t   *hist_copy;      // [slot][kMaxSym]
    uint8_t    *lens;           // [slot][kMaxSym]
    uint64_t   *codes;          // [slot][kMaxSym]: len << 56 | code
    uint32_t   *enc32;          // [slot][kMaxSym]: code << (32 - len) | len, valid while max_len <= 27
    uint32_t   *outl_cnt;       // [global chunk]: outliers
    uint32_t   *chunk_bits;     // [global chunk]: sum of codeword lengths
    uint32_t   *range_units;    // [chunk range]: payload units, later their exclusive prefix within the tensor
    uint32_t   *range_outl;     // [chunk range]: outliers, later their exclusive prefix within the tensor
    uint32_t   *range_bits;     // [chunk range]: sum of codeword lengths
    TensorMeta *tmeta;          // [slot]
    uint32_t   *status;
    TensorC     t[kBatchMax];
};

struct DecompressArgs {
    const uint8_t *buf;
    uint64_t       size;
    float         *xout;
    uint32_t       numel, planes, H, W, HW;
    uint32_t       shape[4];
    uint32_t       radius, sub, guard_shift, eb_bits;
    uint32_t       zero_blocks;
    float          s;
    Layout         lay;
    uint32_t *meta;
    uint32_t *status;
};

// ---- decompression: one call handles a batch of containers ----
struct TensorD {
    const uint8_t *buf;
    uint64_t       size;
    const ArenaSlot *slot;                  // not NULL (fused kernel only): the container is at buf + slot->offset,
                                            // slot->size bytes
    float         *xout;
    uint32_t       shape[4];
    uint32_t       numel, eb_bits;
    float          s;
    // plan of the fused kernel (nitems == 0: the tensor takes the unfused kernels)
    uint32_t       wg_base, nwg;            // its workgroups in the launch
    uint32_t       big, G, Rb, nitems;
    FastDiv        divW;
};

struct BatchD {
    uint32_t  n;
    uint32_t  radius, sub, guard_shift, zero_blocks;
    uint32_t *meta;
    uint32_t *status;
    TensorD   t[kBatchMax];
};

__host__ __device__ inline DecompressArgs decompress_args(const BatchD &b, const TensorD &t)
{
    DecompressArgs a;
    a.buf = t.buf; a.size = t.size; a.xout = t.xout;
#if defined(__HIP_DEVICE_COMPILE__)
    if (t.slot) { a.buf = t.buf + t.slot->offset; a.size = t.slot->size; }
#endif
    a.numel = t.numel; a.planes = t.shape[0] * t.shape[1];
    a.H = t.shape[2]; a.W = t.shape[3]; a.HW = a.H * a.W;
    for (int i = 0; i < 4; ++i) a.shape[i] = t.shape[i];
    a.radius = b.radius; a.sub = b.sub; a.guard_shift = b.guard_shift; a.eb_bits = t.eb_bits;
    a.zero_blocks = b.zero_blocks;
    a.s = t.s;
    a.lay = make_layout(t.numel, b.radius, b.sub);
    a.meta = b.meta; a.status = b.status;
    return a;
}

constexpr uint32_t kLB = 11;                      // bits resolved by the first decode table (4 KB of LDS; with the
                                                  // fused decoder's other arrays five workgroups just fit a CU)
struct DecodeTables;                              // cmpz_decode_core.h

// Pre-quantisation of one value (Section 3.1, first stage): one fp32 multiply, clamp to +-16384
// (NaN -> 0), round half to even (v_rndne_f32).
__device__ __forceinline__ int quant(float x, float r)
{
    float t = x * r;
    if (!(fabsf(t) <= (float)kQMax)) t = (t != t) ? 0.0f : copysignf((float)kQMax, t);
    return (int)__builtin_rintf(t);
}
// 1 if the pre-quantisation clamps this value (it lies outside the quantiser's range or is not finite)
__device__ __forceinline__ uint32_t clamps(float x, float r)
{
    const float t = x * r;
    return (fabsf(t) <= (float)kQMax) ? 0u : 1u;
}
// Lorenzo residual of element i at plane coordinates (h, w), from x alone.
__device__ __forceinline__ int delta_from_x(const float *__restrict__ x, uint32_t i, uint32_t h, uint32_t w,
                                            uint32_t W, float r)
{
    const int q = quant(x[i], r);
    const int left = (w > 0) ? quant(x[i - 1], r) : 0;
    const int up = (h > 0) ? quant(x[i - W], r) : 0;
    const int diag = (h > 0 && w > 0) ? quant(x[i - W - 1], r) : 0;
    return q - left - up + diag;
}

// True in every lane of an aligned group of g lanes (g a power of two) iff `flag` holds in all of them.
__device__ __forceinline__ bool group_all(bool flag, uint32_t lane, uint32_t g)
{
    const unsigned long long m = __ballot(flag);
    const unsigned long long grp = (g >= 64u ? ~0ull : ((1ull << g) - 1ull)) << (lane & ~(g - 1u));
    return (m & grp) == grp;
}

// --- wave-level scans on the DPP network (row shifts inside 16-lane rows, then the two
// row broadcasts that CDNA keeps from GCN); no LDS traffic, unlike __shfl_up ---------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t src)
{
    // lanes without a valid source lane, and rows outside ROW_MASK, read 0
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)src, CTRL, ROW_MASK, 0xf, false);
}

// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t x)
{
    x += dpp_u32<0x111, 0xf>(x);     // row_shr:1
    x += dpp_u32<0x112, 0xf>(x);     // row_shr:2
    x += dpp_u32<0x114, 0xf>(x);     // row_shr:4
    x += dpp_u32<0x118, 0xf>(x);     // row_shr:8
    x += dpp_u32<0x142, 0xa>(x);     // row_bcast:15 into rows 1 and 3
    x += dpp_u32<0x143, 0xc>(x);     // row_bcast:31 into rows 2 and 3
    return x;
}

// inclusive segmented prefix sum: f != 0 marks the first lane of a segment; on return f is
// nonzero for every lane at or after the first segment start of the wave
#define CMPZ_SEG_STEP(CTRL, MASK)                                   \
    {                                                               \
        const uint32_t pv = dpp_u32<CTRL, MASK>((uint32_t)v);       \
        const uint32_t pf = dpp_u32<CTRL, MASK>(f);                 \
        v = f ? v : v + (int32_t)pv;                                \
        f |= pf;                                                    \
    }
__device__ __forceinline__ void wave_segmented_sum(int32_t &v, uint32_t &f)
{
    CMPZ_SEG_STEP(0x111, 0xf)
    CMPZ_SEG_STEP(0x112, 0xf)
    CMPZ_SEG_STEP(0x114, 0xf)
    CMPZ_SEG_STEP(0x118, 0xf)
    CMPZ_SEG_STEP(0x142, 0xa)
    CMPZ_SEG_STEP(0x143, 0xc)
}
#undef CMPZ_SEG_STEP

// For each of 1024 symbols (one per thread, 16 waves): how many symbols with a smaller index
// have the same nonzero code length L.  wave_cnt is LDS scratch; contains a barrier.
__device__ __forceinline__ uint32_t rank_within_length(uint32_t L, uint32_t (*wave_cnt)[64], int tid)
{
    const int lane = tid & 63, wv = tid >> 6;
    for (int k = tid; k < 16 * 64; k += 1024) (&wave_cnt[0][0])[k] = 0;
    __syncthreads();
    uint32_t in_wave = 0;
    unsigned long long remaining = __ballot(L != 0);
    while (remaining) {                                   // wave-uniform
        const int leader = __ffsll((long long)remaining) - 1;
        const uint32_t Lx = __shfl(L, leader);
        const unsigned long long m = __ballot(L == Lx);
        if (L == Lx) in_wave = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
        if (lane == leader) wave_cnt[wv][Lx & 63u] = (uint32_t)__popcll(m);
        remaining &= ~m;
    }
    __syncthreads();
    uint32_t base = 0;
    if (L) for (int k = 0; k < wv; ++k) base += wave_cnt[k][L & 63u];
    return base + in_wave;
}

// Kernel identifiers for the optional per-kernel timing (cmp_profile).
enum KernelId : int {
    kKQuantLorenzoHist = 0, kKCodebook, kKLengths, kKScan, kKPack, kKClear,
    kKDecodeTables, kKDecode, kKPatchOutliers, kKRowScan, kKColScanDequant, kKDecodeFused, kKControllerStats,
    kKernelCount
};
extern const char *const kKernelNames[kKernelCount];

// When enabled, every launch is bracketed by two events on its stream.
struct Profiler {
    struct Rec { int id; hipEvent_t beg, end; };
    bool enabled = false;
    std::vector<Rec> recs;
    std::vector<hipEvent_t> pool;
    size_t used = 0;
    hipEvent_t get()
    {
        if (used == pool.size()) { hipEvent_t e; (void)hipEventCreate(&e); pool.push_back(e); }
        return pool[used++];
    }
};

template <class K, class... A>
inline void launch(Profiler *p, int id, K kernel, dim3 grid, dim3 block, hipStream_t st, A... args)
{
    if (p && p->enabled) {
        Profiler::Rec r{id, p->get(), p->get()};
        (void)hipEventRecord(r.beg, st);
        hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
        (void)hipEventRecord(r.end, st);
        p->recs.push_back(r);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
    }
}

// Compression stages, each one launch over all tensors of the group (cmpz_sweep1.hip,
// cmpz_compress.hip, cmpz_codebook.hip, cmpz_pack.hip).
void launch_sweep1(const BatchC &b, Profiler *prof, hipStream_t st);
void launch_sweep1_untiled(const BatchC &b, uint32_t t, Profiler *prof, hipStream_t st);
bool sweep1_tiled_fits(uint32_t W);
void launch_codebook(const BatchC &b, Profiler *prof, hipStream_t st);
void launch_pack(const BatchC &b, Profiler *prof, hipStream_t st);
void launch_clear(const BatchC &b, Profiler *prof, hipStream_t st);
void launch_arena_init(ArenaState *st_dev, uint32_t slots, hipStream_t st);
void launch_arena_pushed(const BatchC &b, ArenaState *st_dev, uint32_t slot, hipStream_t st);
void launch_arena_release(ArenaState *st_dev, uint32_t slot, hipStream_t st);
void launch_widen(uint16_t *sym, uint32_t *wide, uint32_t sym_off, uint32_t nchunks, hipStream_t st);
size_t decode_tables_bytes();
bool plan_decode_fused(TensorD *t, uint32_t sub);
void launch_decode_fused(BatchD &b, uint32_t cus, Profiler *prof, hipStream_t st);
void launch_decompress_unfused(const DecompressArgs &a, void *tables, Profiler *prof, hipStream_t st);

// Error-bound estimator: device scratch (zero between calls) and result record.
constexpr uint32_t kMaxBatch = 65536;
struct ControllerScratch {
    unsigned long long nonzero;     // activation elements != 0
    double             msum;        // sum of |momentum|
    uint32_t           done;        // workgroups finished
    uint32_t           pad;
    uint32_t           maxbits[kMaxBatch];   // per sample: bit pattern of the largest |loss| (a NaN pattern wins)
};
struct ControllerResult {
    float    eb;
    int32_t  rc;                    // 0 or 1 (nothing to estimate from)
    double   stats[3];              // R, Lbar, Mavg
};
struct ControllerArgs {
    const float *act, *loss, *mom;
    uint32_t n_act, n_loss, n_mom, batch_n, per_sample;
    float sigma_frac, a, eb_min, eb_max;
    ControllerScratch *scratch;
    ControllerResult  *result;
};
void launch_controller(const ControllerArgs &a, Profiler *prof, hipStream_t st);

}  // namespace cmpz
