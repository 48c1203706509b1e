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

// Scratch words in ctx->d_meta.
enum MetaWord : int {
    kMetaRangeEvents = 0,   // elements clamped by the current compress
    kMetaMaxLen      = 1,   // longest codeword of the current codebook
    kMetaSkip        = 2,   // nonzero: container does not fit, later kernels write nothing
    kMetaNOutliers   = 3,
    kMetaBad         = 4,   // decompress: nonzero when the container failed validation
    kMetaWords       = 16
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
    uint32_t *chunk_units;  // payload size of each chunk in 16-byte units
    uint32_t *outl_cnt;     // outliers in each chunk
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

// Kernel identifiers for the optional per-kernel timing (cmp_profile).
enum KernelId : int {
    kKQuantLorenzoHist = 0, kKCodebook, kKChunkBits, kKScanHeader, kKEncode, kKOutliers, kKEmpty,
    kKDecodeTables, kKDecode, kKPatchOutliers, kKRowScan, kKColScanDequant, kKernelCount
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

void launch_compress(const CompressArgs &a, Profiler *prof, hipStream_t st);
void launch_codebook(const CompressArgs &a, Profiler *prof, hipStream_t st);
size_t decode_tables_bytes();
void launch_decompress(const DecompressArgs &a, void *tables, Profiler *prof, hipStream_t st);

}  // namespace cmpz
