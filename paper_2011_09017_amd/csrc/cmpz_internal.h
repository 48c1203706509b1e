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
constexpr uint32_t kMaxCodeLen  = 48;       // counts below 2^32 bound a Huffman depth by 45
constexpr uint32_t kVersion     = 1;
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

// Tile descriptors of the encode sweep's single-pass scan: bits 63..62 state,
// bits 61..32 payload units, bits 31..0 outlier count.  The first sweep leaves 0.
constexpr uint64_t kDescAgg    = 1ull << 62;   // value = this tile alone
constexpr uint64_t kDescPrefix = 2ull << 62;   // value = all tiles up to and including this one
constexpr uint64_t kDescMask   = (1ull << 62) - 1;

// Scratch words in ctx->d_meta.
enum MetaWord : int {
    kMetaRangeEvents = 0,   // elements clamped by the current compress
    kMetaMaxLen      = 1,   // longest codeword of the current codebook
    kMetaSkip        = 2,   // nonzero: container does not fit, later kernels write nothing
    kMetaNOutliers   = 3,
    kMetaBad         = 4,   // decompress: nonzero when the container failed validation
    kMetaTicket      = 5,   // next chunk to hand out in the encode sweep (zero between calls)
    kMetaDone        = 6,   // workgroups of the encode sweep that have finished (zero between calls)
    kMetaTotalUnits  = 7,   // payload size in 16-byte units
    kMetaBitsLo      = 8,   // uint64 sum of codeword lengths (words 8 and 9; zero between calls)
    kMetaClocks      = 16,  // 24 uint64 phase-clock accumulators (only in CMPZ_PHASE_CLOCKS builds)
    kMetaWords       = 64
};

struct CompressArgs {
    const float *x;
    uint8_t     *out;
    uint64_t     out_cap;
    uint32_t     numel, H, W, HW;
    uint32_t     shape[4];
    uint32_t     radius, sub, guard_shift, eb_bits;
    float        r;
    Layout       lay;
    // context scratch
    uint16_t *sym;
    uint32_t *hist;         // zero between calls
    uint32_t *hist_copy;
    uint8_t  *lens;
    uint64_t *codes;        // len << 56 | code
    uint64_t *desc;         // one descriptor per encode tile, see kDescAgg
    uint32_t *outl_cnt;     // outliers in each chunk
    uint32_t  tile_chunks;  // chunks per encode tile: 1, 2, 4 or 8
    uint32_t *meta;
    uint32_t *status;
};

struct DecompressArgs {
    const uint8_t *buf;
    uint64_t       size;
    float         *xout;
    uint32_t       numel, planes, H, W, HW;
    uint32_t       shape[4];
    uint32_t       radius, sub, guard_shift, eb_bits;
    float          s;
    Layout         lay;
    uint32_t *meta;
    uint32_t *status;
};

constexpr uint32_t kLB = 11;                      // bits resolved by the first decode table
struct DecodeTables;                              // cmpz_decode_core.h

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
    kKQuantLorenzoHist = 0, kKCodebook, kKEncode, kKOutliers, kKEmpty,
    kKDecodeTables, kKDecode, kKPatchOutliers, kKRowScan, kKColScanDequant, kKDecodeFused, kKDecodeFusedRest, kKControllerStats,
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

void launch_compress_begin(const CompressArgs &a, Profiler *prof, hipStream_t st);
void launch_compress_finish(const CompressArgs &a, Profiler *prof, hipStream_t st);
void launch_codebook(const CompressArgs &a, Profiler *prof, hipStream_t st);
bool launch_sweep1_tiled(const CompressArgs &a, Profiler *prof, hipStream_t st);
size_t decode_tables_bytes();
void launch_decompress(const DecompressArgs &a, void *tables, uint32_t *items, const volatile uint32_t *hint_host,
                       uint32_t *hint_dev, Profiler *prof, hipStream_t st);
bool launch_decode_fused(const DecompressArgs &a, uint32_t *items, const volatile uint32_t *hint_host,
                         uint32_t *hint_dev, Profiler *prof, hipStream_t st);
uint64_t fused_item_words(uint64_t numel);

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
