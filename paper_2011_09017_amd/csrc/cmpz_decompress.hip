// Decompression kernels: container validation + decode tables, chunked Huffman
// decode (one lane per sub-block), outlier patch, reverse Lorenzo as row and
// column prefix sums, de-quantisation.
//
// This first path stages the residuals as int32 in the output buffer itself and
// turns them into fp32 in place: decode -> patch -> row scan -> column scan with
// de-quantisation.  It needs no scratch and works for any H and W.
#include "cmpz_decode_core.h"

namespace cmpz {
namespace {

constexpr int      kThreads  = 256;
constexpr int      kDecThreads = 128;              // sub-blocks (lanes) per decode workgroup

// ---------------------------------------------------------------------------
// Validation of the header and the code lengths, and the decode tables, for the
// kernels below: the same routine the fused kernel runs in every workgroup, here
// in a workgroup of its own that leaves the tables in global memory.  On failure
// meta[kMetaBad] = 1 and every later kernel of the call returns at once.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_decode_tables(DecompressArgs a, DecodeTables *tb)
{
    __shared__ DecodeTables T;
    __shared__ uint32_t scratch[3584];               // 14 KB, what build_tables asks for
    const int tid = threadIdx.x;
    const uint32_t defect = build_tables<256>(T, a, scratch);
    if (defect) {
        if (tid == 0) { a.meta[kMetaBad] = 1; atomicOr(a.status, defect); }
        return;
    }
    const uint32_t *src = reinterpret_cast<const uint32_t *>(&T);
    uint32_t *dst = reinterpret_cast<uint32_t *>(tb);
    for (uint32_t k = tid; k < sizeof(DecodeTables) / 4; k += 256) dst[k] = src[k];
    if (tid == 0) a.meta[kMetaBad] = 0;
}

// ---------------------------------------------------------------------------
// Unfused path, for shapes the fused kernel does not take.  Chunked Huffman
// decode: one lane per sub-block, 128 sub-blocks per workgroup.  Symbols go to an
// LDS stage (odd word stride per lane, conflict free) and leave as int32
// residuals with coalesced stores.  Outliers (symbol 0) are patched by the next
// kernel.
// ---------------------------------------------------------------------------
template <int SUB>
__global__ __launch_bounds__(kDecThreads) void k_decode(DecompressArgs a, const DecodeTables *__restrict__ tb)
{
    constexpr int kStride = SUB + 2;                       // u16 units; (SUB+2)/2 words is odd
    __shared__ DecodeTables T;
    __shared__ int16_t stage[kDecThreads * kStride];
    if (a.meta[kMetaBad]) return;
    const int tid = threadIdx.x;
    load_tables(T, tb, tid, kDecThreads);
    __syncthreads();

    constexpr uint32_t nsub = kChunk / SUB;
    const uint64_t g = (uint64_t)blockIdx.x * kDecThreads + tid;      // global sub-block index
    const uint32_t c = (uint32_t)(g / nsub), j = (uint32_t)(g % nsub);
    const uint64_t e0 = g * SUB;                                    // first element of the sub-block
    uint32_t n_here = 0;
    if (e0 < a.numel) n_here = (a.numel - e0 >= (uint64_t)SUB) ? (uint32_t)SUB : (uint32_t)(a.numel - e0);
    bool bad = false;

    if (n_here) {
        const uint32_t *chunk_off = reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_chunk_off);
        const uint16_t *sub_bits = reinterpret_cast<const uint16_t *>(a.buf + a.lay.off_sub_bits) + (uint64_t)c * nsub;
        const uint32_t u0 = chunk_off[c], u1 = chunk_off[c + 1];
        uint32_t nwords = 0;
        if (u0 <= u1 && u1 <= T.payload_units) nwords = (u1 - u0) * 4; else bad = true;
        const uint32_t *__restrict__ words =
            reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_payload + (uint64_t)(bad ? 0u : u0) * 16);
        uint32_t start = 0;
        for (uint32_t k = 0; k < j; ++k) start += sub_bits[k];
        const uint32_t sb = sub_bits[j];
        if ((uint64_t)start + sb > (uint64_t)nwords * 32) { bad = true; nwords = 0; }
        int16_t *my = stage + tid * kStride;
        uint32_t end = 0;
        if (a.zero_blocks && sb == 0 && !bad) {
            // version 2: a stored bit count of 0 stands for a sub-block of zero residuals
            for (uint32_t k = 0; k < n_here; ++k) my[k] = 0;
            end = start;
        } else if (nwords) {
            const uint32_t last = nwords - 1;
            end = decode_run<false>(T, [&](uint32_t k) -> uint32_t { return words[k < last ? k : last]; }, start, n_here, 0u,
                             [&](uint32_t k, int32_t d) { my[k] = (int16_t)d; }, bad);
        }
        if (end != start + sb) bad = true;
    }
    if (bad) atomicOr(a.status, kStFormat);
    __syncthreads();

    // coalesced write-out of the tile as int32 residuals
    int32_t *out = reinterpret_cast<int32_t *>(a.xout);
    const uint64_t tile0 = (uint64_t)blockIdx.x * kDecThreads * SUB;
    for (uint32_t e = tid; e < (uint32_t)(kDecThreads * SUB); e += kDecThreads) {
        const uint64_t i = tile0 + e;
        if (i >= a.numel) break;
        out[i] = stage[(e / SUB) * kStride + (e % SUB)];
    }
}

// Outlier patch: residual[idx] = value.
__global__ __launch_bounds__(kThreads) void k_patch_outliers(DecompressArgs a, const DecodeTables *__restrict__ tb)
{
    if (a.meta[kMetaBad]) return;
    const Header *hd = reinterpret_cast<const Header *>(a.buf);
    const uint32_t n = tb->n_outliers;
    const uint32_t *oidx = reinterpret_cast<const uint32_t *>(a.buf + hd->off_outl_idx);
    const int32_t *oval = reinterpret_cast<const int32_t *>(a.buf + hd->off_outl_val);
    int32_t *out = reinterpret_cast<int32_t *>(a.xout);
    for (uint64_t k = (uint64_t)blockIdx.x * kThreads + threadIdx.x; k < n; k += (uint64_t)gridDim.x * kThreads) {
        const uint32_t i = oidx[k];
        if (i < a.numel) out[i] = oval[k]; else atomicOr(a.status, kStFormat);
    }
}

// Row-wise inclusive prefix sum in place: one wave per row.
__global__ __launch_bounds__(kThreads) void k_row_scan(DecompressArgs a)
{
    if (a.meta[kMetaBad]) return;
    const int lane = threadIdx.x & 63;
    const uint64_t rows = (uint64_t)a.planes * a.H;
    int32_t *out = reinterpret_cast<int32_t *>(a.xout);
    for (uint64_t row = (uint64_t)blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6); row < rows;
         row += (uint64_t)gridDim.x * (kThreads / kWave)) {
        int32_t *p = out + row * a.W;
        int32_t carry = 0;
        for (uint32_t w0 = 0; w0 < a.W; w0 += 64) {
            const uint32_t w = w0 + lane;
            int32_t v = (w < a.W) ? p[w] : 0;
            for (int o = 1; o < 64; o <<= 1) {
                const int32_t n = __shfl_up(v, o);
                if (lane >= o) v += n;
            }
            v += carry;
            if (w < a.W) p[w] = v;
            carry = __shfl(v, 63);
        }
    }
}

// Column-wise inclusive prefix sum and de-quantisation in place: one thread per column.
__global__ __launch_bounds__(kThreads) void k_col_scan_dequant(DecompressArgs a)
{
    if (a.meta[kMetaBad]) return;
    const uint64_t cols = (uint64_t)a.planes * a.W;
    for (uint64_t g = (uint64_t)blockIdx.x * kThreads + threadIdx.x; g < cols; g += (uint64_t)gridDim.x * kThreads) {
        const uint64_t p = g / a.W;
        const uint32_t w = (uint32_t)(g - p * a.W);
        int32_t *col = reinterpret_cast<int32_t *>(a.xout) + p * a.HW + w;
        float *fcol = a.xout + p * a.HW + w;
        int32_t acc = 0;
        for (uint32_t h = 0; h < a.H; ++h) {
            acc += col[(uint64_t)h * a.W];
            fcol[(uint64_t)h * a.W] = (float)acc * a.s;
        }
    }
}

}  // namespace

size_t decode_tables_bytes() { return sizeof(DecodeTables); }

// Shapes the fused kernel does not take, and empty tensors (validation only): residuals staged in
// the output buffer.
void launch_decompress_unfused(const DecompressArgs &a, void *tables, Profiler *prof, hipStream_t st)
{
    DecodeTables *tb = static_cast<DecodeTables *>(tables);
    launch(prof, kKDecodeTables, k_decode_tables, dim3(1), dim3(256), st, a, tb);
    if (a.numel == 0) return;
    const DecodeTables *ctb = tb;
    const uint64_t nsubs = (uint64_t)a.lay.nchunks * a.lay.nsub;
    const uint32_t blocks = (uint32_t)((nsubs + kDecThreads - 1) / kDecThreads);
    switch (a.sub) {
    case 32:  launch(prof, kKDecode, k_decode<32>, dim3(blocks), dim3(kDecThreads), st, a, ctb); break;
    case 64:  launch(prof, kKDecode, k_decode<64>, dim3(blocks), dim3(kDecThreads), st, a, ctb); break;
    default:  launch(prof, kKDecode, k_decode<128>, dim3(blocks), dim3(kDecThreads), st, a, ctb); break;
    }
    launch(prof, kKPatchOutliers, k_patch_outliers, dim3(256), dim3(kThreads), st, a, ctb);
    const uint64_t cap = 65536ull * 8;
    const uint64_t rows = (uint64_t)a.planes * a.H;
    const uint64_t rblocks = (rows + 3) / 4 < cap ? (rows + 3) / 4 : cap;
    launch(prof, kKRowScan, k_row_scan, dim3((uint32_t)rblocks), dim3(kThreads), st, a);
    const uint64_t cols = (uint64_t)a.planes * a.W;
    const uint64_t cblocks = (cols + kThreads - 1) / kThreads < cap ? (cols + kThreads - 1) / kThreads : cap;
    launch(prof, kKColScanDequant, k_col_scan_dequant, dim3((uint32_t)cblocks), dim3(kThreads), st, a);
}

}  // namespace cmpz
