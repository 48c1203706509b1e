// Decompression kernels: container validation + decode tables, chunked Huffman
// decode (one lane per sub-block), outlier patch, reverse Lorenzo as row and
// column prefix sums, de-quantisation.
//
// This first path stages the residuals as int32 in the output buffer itself and
// turns them into fp32 in place: decode -> patch -> row scan -> column scan with
// de-quantisation.  It needs no scratch and works for any H and W.
#include "cmpz_internal.h"

namespace cmpz {
namespace {

constexpr int      kThreads  = 256;
constexpr int      kDecThreads = 128;              // sub-blocks (lanes) per decode workgroup
constexpr uint32_t kLB       = 10;                 // bits resolved by the direct lookup table
constexpr uint32_t kFastSize = 1u << kLB;

// Decode tables kept in context scratch between the table kernel and the decoders.
struct DecodeTables {
    uint32_t fast[kFastSize];     // symbol | length << 16, length 0 = longer than kLB bits
    uint64_t first[64];           // first canonical code of each length
    uint32_t count[64];           // codes of each length
    uint32_t offs[64];            // index into sorted[] of the first symbol of each length
    uint16_t sorted[kMaxSym];     // symbols ordered by (length, symbol)
    uint32_t max_len;
    uint32_t payload_units;
    uint32_t n_outliers;
    uint32_t pad;
};

__device__ __forceinline__ uint64_t align16(uint64_t v) { return (v + 15) & ~15ull; }

// ---------------------------------------------------------------------------
// Validation of the header and the code lengths, and the decode tables.
// One workgroup of 1024 threads.  On failure meta[kMetaBad] = 1 and every later
// kernel of the call returns at once.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_decode_tables(DecompressArgs a, DecodeTables *tb)
{
    __shared__ uint32_t len_of[kMaxSym];
    __shared__ uint32_t bl_count[64];
    __shared__ uint64_t first_code[64];
    __shared__ uint32_t offs[64];
    __shared__ uint32_t bad_s, used_s, max_len_s;
    __shared__ unsigned long long kraft_s;      // in units of 2^-56
    const int tid = threadIdx.x;
    const uint32_t nsym = 2 * a.radius;
    const Header *hd = reinterpret_cast<const Header *>(a.buf);

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
                const uint32_t *chunk_off = reinterpret_cast<const uint32_t *>(a.buf + l.off_chunk_off);
                const uint32_t *outl_off = reinterpret_cast<const uint32_t *>(a.buf + l.off_outl_off);
                if (chunk_off[0] != 0 || chunk_off[l.nchunks] != units) bad = kStFormat;
                if (outl_off[0] != 0 || outl_off[l.nchunks] != (uint32_t)n_out) bad = kStFormat;
                tb->payload_units = units;
                tb->n_outliers = (uint32_t)n_out;
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
    len_of[tid] = L;
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
    }
    __syncthreads();
    if (bad_s) {
        if (tid == 0) { a.meta[kMetaBad] = 1; atomicOr(a.status, bad_s); }
        return;
    }

    __shared__ uint32_t fast_s[kFastSize];
    for (uint32_t k = tid; k < kFastSize; k += 1024) fast_s[k] = 0;
    __syncthreads();
    if (L) {
        uint32_t rank = 0;
        for (int j = 0; j < tid; ++j) rank += (len_of[j] == L) ? 1u : 0u;
        const uint64_t code = first_code[L] + rank;
        tb->sorted[offs[L] + rank] = (uint16_t)tid;
        if (L <= kLB) {
            const uint32_t lo = (uint32_t)code << (kLB - L), n = 1u << (kLB - L);
            const uint32_t e = (uint32_t)tid | (L << 16);
            for (uint32_t k = 0; k < n; ++k) fast_s[lo + k] = e;
        }
    }
    __syncthreads();
    for (uint32_t k = tid; k < kFastSize; k += 1024) tb->fast[k] = fast_s[k];
    if (tid < 64) { tb->first[tid] = first_code[tid]; tb->count[tid] = bl_count[tid]; tb->offs[tid] = offs[tid]; }
    if (tid == 0) { tb->max_len = max_len_s; a.meta[kMetaBad] = 0; }
}

// ---------------------------------------------------------------------------
// Chunked Huffman decode: one lane per sub-block, 128 sub-blocks per workgroup.
// Symbols go to an LDS stage (odd word stride per lane, conflict free) and leave
// as int32 residuals with coalesced stores.  Outliers (symbol 0) are patched by
// the next kernel.
// ---------------------------------------------------------------------------
template <int SUB>
__global__ __launch_bounds__(kDecThreads) void k_decode(DecompressArgs a, const DecodeTables *__restrict__ tb)
{
    constexpr int kStride = SUB + 2;                       // u16 units; (SUB+2)/2 words is odd
    __shared__ uint32_t fast[kFastSize];
    __shared__ uint64_t first[64];
    __shared__ uint32_t count[64], offs[64];
    __shared__ uint16_t sorted[kMaxSym];
    __shared__ uint16_t stage[kDecThreads * kStride];
    if (a.meta[kMetaBad]) return;
    const int tid = threadIdx.x;
    for (int k = tid; k < (int)kFastSize; k += kDecThreads) fast[k] = tb->fast[k];
    for (int k = tid; k < (int)kMaxSym; k += kDecThreads) sorted[k] = tb->sorted[k];
    if (tid < 64) { first[tid] = tb->first[tid]; count[tid] = tb->count[tid]; offs[tid] = tb->offs[tid]; }
    __syncthreads();

    constexpr uint32_t nsub = kChunk / SUB;
    const uint32_t max_len = tb->max_len;
    const uint32_t R = a.radius;
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
        if (u0 <= u1 && u1 <= tb->payload_units) nwords = (u1 - u0) * 4; else bad = true;
        const uint32_t *__restrict__ words =
            reinterpret_cast<const uint32_t *>(a.buf + a.lay.off_payload + (uint64_t)(bad ? 0u : u0) * 16);
        uint32_t start = 0;
        for (uint32_t k = 0; k < j; ++k) start += sub_bits[k];
        const uint32_t sb = sub_bits[j];
        if ((uint64_t)start + sb > (uint64_t)nwords * 32) bad = true;

        auto rd = [&](uint32_t k) -> uint32_t { return k < nwords ? words[k] : 0u; };
        uint32_t pos = start;
        uint32_t wi = pos >> 5;
        uint64_t win = ((((uint64_t)rd(wi)) << 32) | rd(wi + 1)) << (pos & 31);
        int avail = 64 - (int)(pos & 31);
        wi += 2;
        uint16_t *my = stage + tid * kStride;
        for (uint32_t k = 0; k < n_here; ++k) {
            if (avail <= 32) { win |= ((uint64_t)rd(wi++)) << (32 - avail); avail += 32; }
            const uint32_t e = fast[(uint32_t)(win >> (64 - kLB))];
            uint32_t len = e >> 16, s = e & 0xffffu;
            if (len == 0) {
                // codeword longer than the table: canonical search on a fresh 64-bit window
                const uint32_t w0 = pos >> 5, off = pos & 31;
                uint64_t w64 = ((((uint64_t)rd(w0)) << 32) | rd(w0 + 1)) << off;
                if (off) w64 |= (uint64_t)(rd(w0 + 2) >> (32 - off));
                for (uint32_t L = kLB + 1; L <= max_len; ++L) {
                    const uint64_t code = w64 >> (64 - L);
                    if (code >= first[L] && code - first[L] < count[L]) {
                        s = sorted[offs[L] + (uint32_t)(code - first[L])];
                        len = L;
                        break;
                    }
                }
                if (len == 0) { bad = true; len = 1; s = R; }
                pos += len;
                wi = pos >> 5;
                win = ((((uint64_t)rd(wi)) << 32) | rd(wi + 1)) << (pos & 31);
                avail = 64 - (int)(pos & 31);
                wi += 2;
            } else {
                win <<= len; avail -= (int)len; pos += len;
            }
            my[k] = (uint16_t)s;
        }
        if (pos != start + sb) bad = true;
    }
    if (bad) atomicOr(a.status, kStFormat);
    __syncthreads();

    // coalesced write-out of the tile as int32 residuals
    int32_t *out = reinterpret_cast<int32_t *>(a.xout);
    const uint64_t tile0 = (uint64_t)blockIdx.x * kDecThreads * SUB;
    for (uint32_t e = tid; e < (uint32_t)(kDecThreads * SUB); e += kDecThreads) {
        const uint64_t i = tile0 + e;
        if (i >= a.numel) break;
        const uint32_t s = stage[(e / SUB) * kStride + (e % SUB)];
        out[i] = (int32_t)s - (int32_t)R;
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

void launch_decompress(const DecompressArgs &a, void *tables, Profiler *prof, hipStream_t st)
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
