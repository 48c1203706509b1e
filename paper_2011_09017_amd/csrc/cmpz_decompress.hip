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
__device__ __forceinline__ uint64_t align16(uint64_t v) { return (v + 15) & ~15ull; }

// ---------------------------------------------------------------------------
// Validation of the header and the code lengths, and the decode tables.
// One workgroup of 1024 threads.  On failure meta[kMetaBad] = 1 and every later
// kernel of the call returns at once.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_decode_tables(DecompressArgs a, DecodeTables *tb)
{
    __shared__ DecodeTables T;
    __shared__ uint32_t wave_cnt[16][64];
    __shared__ uint32_t bl_count[64];
    __shared__ uint64_t first_code[64];
    __shared__ uint32_t offs[64];
    __shared__ uint32_t bad_s, used_s, max_len_s;
    __shared__ unsigned long long kraft_s;      // in units of 2^-56
    const int tid = threadIdx.x;
    const uint32_t nsym = 2 * a.radius;
    // the header and the four table ends are fetched by separate lanes in one round trip
    __shared__ Header hd_s;
    __shared__ uint32_t ends_s[4];
    if (tid < (int)(kHeaderBytes / 4)) reinterpret_cast<uint32_t *>(&hd_s)[tid] = reinterpret_cast<const uint32_t *>(a.buf)[tid];
    if (tid >= 64 && tid < 68) {
        const uint32_t *chunk_off = reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_chunk_off);
        const uint32_t *outl_off = reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_outl_off);
        const int k = tid - 64;
        ends_s[k] = (k == 0) ? chunk_off[0] : (k == 1) ? chunk_off[a.lay.nchunks] : (k == 2) ? outl_off[0] : outl_off[a.lay.nchunks];
    }
    __syncthreads();
    const Header *hd = &hd_s;

    if (tid == 0) {
        uint32_t bad = 0;
        const Layout &l = a.lay;
        if (hd->magic != kMagic || hd->version != kVersion || hd->status != 0) bad = kStFormat;
        for (int k = 0; k < 112 && !bad; ++k) if (hd->zero[k]) bad = kStFormat;
        if (!bad) {
            if (hd->eb_bits != a.eb_bits) bad = kStMismatch;
            for (int k = 0; k < 4; ++k) if (hd->shape[k] != a.shape[k]) bad = kStMismatch;
            if (hd->radius != a.radius || hd->chunk != kChunk || hd->sub != a.sub ||
                hd->guard_shift != a.guard_shift) bad = kStMismatch;
        }
        if (!bad) {
            const uint64_t n_out = hd->n_outliers;
            const uint64_t sect = align16(4 * n_out);
            if (hd->numel != a.numel || hd->nchunks != l.nchunks) bad = kStFormat;
            else if (hd->off_lens != l.off_lens || hd->off_chunk_off != l.off_chunk_off ||
                     hd->off_outl_off != l.off_outl_off || hd->off_sub_bits != l.off_sub_bits ||
                     hd->off_payload != l.off_payload) bad = kStFormat;
            else if (hd->total_size > a.size || n_out > a.numel || hd->range_events > a.numel) bad = kStFormat;
            else if (hd->off_outl_idx < l.off_payload || ((hd->off_outl_idx - l.off_payload) & 15)) bad = kStFormat;
            else if (hd->off_outl_val != hd->off_outl_idx + sect || hd->total_size != hd->off_outl_val + sect)
                bad = kStFormat;
            else if (((hd->off_outl_idx - l.off_payload) >> 4) >= (1ull << 32)) bad = kStFormat;
            if (!bad) {
                const uint32_t units = (uint32_t)((hd->off_outl_idx - l.off_payload) >> 4);
                if (ends_s[0] != 0 || ends_s[1] != units) bad = kStFormat;
                if (ends_s[2] != 0 || ends_s[3] != (uint32_t)n_out) bad = kStFormat;
                T.payload_units = units;
                T.n_outliers = (uint32_t)n_out;
            }
        }
        bad_s = bad; used_s = 0; max_len_s = 0; kraft_s = 0;
    }
    if (tid < 64) { bl_count[tid] = 0; first_code[tid] = 0; offs[tid] = 0; }
    __syncthreads();
    if (bad_s) {
        if (tid == 0) { a.meta[kMetaBad] = 1; atomicOr(a.status, bad_s); }
        return;
    }

    // code lengths: range, Kraft sum, maximum
    uint32_t L = 0;
    if ((uint32_t)tid < nsym) L = a.buf[a.lay.off_lens + tid];
    else if ((uint32_t)tid < ((nsym + 15u) & ~15u)) { if (a.buf[a.lay.off_lens + tid]) atomicOr(&bad_s, kStFormat); }
    if (L > kMaxCodeLen) { atomicOr(&bad_s, kStFormat); L = 0; }
    if (L) {
        atomicAdd(&used_s, 1u);
        atomicAdd(&kraft_s, 1ull << (56 - L));
        atomicMax(&max_len_s, L);
        atomicAdd(&bl_count[L], 1u);
    }
    __syncthreads();
    if (tid == 0) {
        const unsigned long long one = 1ull << 56;
        if (used_s >= 2 && kraft_s != one) bad_s |= kStFormat;
        if (used_s == 1 && max_len_s != 1) bad_s |= kStFormat;
        if (used_s == 0 && a.numel != 0) bad_s |= kStFormat;
        if (hd->max_len != max_len_s) bad_s |= kStFormat;
        uint64_t code = 0;
        uint32_t o = 0;
        for (int k = 1; k < 64; ++k) {
            code = (code + (uint64_t)(k > 1 ? bl_count[k - 1] : 0u)) << 1;
            first_code[k] = code;
            offs[k] = o;
            o += bl_count[k];
        }
        // left-aligned end of the codes of at most kLB bits, and the level-2 geometry
        const uint64_t t = (first_code[kLB] + bl_count[kLB]) << (32 - kLB);
        const uint64_t span = (1ull << 32) - t;              // code space of the longer codes
        uint32_t sh = 0;
        while ((span >> sh) > kT2Size) ++sh;
        T.t32 = (uint32_t)t; T.sh = sh; T.has_long = (max_len_s > kLB && span > 0) ? 1u : 0u;
        T.max_len = max_len_s;
    }
    __syncthreads();
    if (bad_s) {
        if (tid == 0) { a.meta[kMetaBad] = 1; atomicOr(a.status, bad_s); }
        return;
    }

    // symbols ordered by (length, symbol)
    const uint32_t rank = rank_within_length(L, wave_cnt, tid);
    if (L) T.sorted[offs[L] + rank] = (uint16_t)(((uint32_t)tid - a.radius) & 1023u);   // as a residual
    if (tid < 64) { T.first[tid] = first_code[tid]; T.count[tid] = bl_count[tid]; T.offs[tid] = offs[tid]; }
    __syncthreads();

    // level 1: entry idx is the codeword (if any, of at most kLB bits) that prefixes idx
    for (uint32_t idx = tid; idx < kT1Size; idx += 1024) {
        uint32_t e = 0;
        for (uint32_t l = 1; l <= kLB; ++l) {
            const uint32_t code = idx >> (kLB - l);
            const uint32_t f = (uint32_t)first_code[l];
            if (code >= f && code - f < bl_count[l]) { e = T.sorted[offs[l] + code - f] | (l << 10); break; }
        }
        T.t1[idx] = (uint16_t)e;
    }
    // level 2: entry i covers left-aligned values t32 + [i << sh, (i+1) << sh)
    if ((uint32_t)tid < kT2Size) {
        const uint32_t idx = tid;
        uint32_t e = 0;
        const uint64_t v = (uint64_t)T.t32 + ((uint64_t)idx << T.sh);
        if (T.has_long && v < (1ull << 32)) {
            const uint32_t lmax = (32 - T.sh < T.max_len) ? 32 - T.sh : T.max_len;
            for (uint32_t l = kLB + 1; l <= lmax; ++l) {
                const uint64_t code = v >> (32 - l);
                if (code >= first_code[l] && code - first_code[l] < bl_count[l]) {
                    e = T.sorted[offs[l] + (uint32_t)(code - first_code[l])] | (l << 10);
                    break;
                }
            }
        }
        T.t2[idx] = (uint16_t)e;
    }
    __syncthreads();
    {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(&T);
        uint32_t *dst = reinterpret_cast<uint32_t *>(tb);
        for (uint32_t k = tid; k < sizeof(DecodeTables) / 4; k += 1024) dst[k] = src[k];
    }
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
        if (nwords) {
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
    launch(prof, kKDecodeTables, k_decode_tables, dim3(1), dim3(1024), st, a, tb);
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
