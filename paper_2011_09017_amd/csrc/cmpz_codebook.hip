// Huffman codebook on the GPU: histogram -> code lengths -> canonical codes.
// One workgroup; no host round trip between the two sweeps of a compress.
//
// Rule (fixes one of the equally optimal codebooks): leaves sorted ascending by
// (count, symbol); two FIFO queues, leaves and internal nodes in creation order;
// the lighter head is taken, a leaf before an internal node of equal weight.
// Codes are canonical: ordered by (length, symbol), first code 0, read MSB first.
#include "cmpz_internal.h"

namespace cmpz {
namespace {

constexpr int kCbThreads = 1024;

__global__ __launch_bounds__(kCbThreads) void k_codebook(CompressArgs a)
{
    __shared__ uint64_t key[kMaxSym];            // count << 10 | symbol, unused = all ones
    __shared__ uint64_t weight[2 * kMaxSym];     // node weights: leaves 0..n-1, internal n..2n-2
    __shared__ uint16_t parent[2 * kMaxSym];
    __shared__ uint32_t len_of[kMaxSym];         // code length per symbol
    __shared__ uint32_t bl_count[64];
    __shared__ uint64_t first_code[64];
    __shared__ uint32_t n_used_s, max_len_s;

    const int tid = threadIdx.x;
    const uint32_t nsym = 2 * a.radius;

    // 1. fetch the histogram, leave it zeroed for the next call, keep a copy for inspection
    uint32_t cnt = 0;
    if ((uint32_t)tid < nsym) { cnt = a.hist[tid]; }
    a.hist[tid] = 0;
    a.hist_copy[tid] = cnt;
    key[tid] = cnt ? (((uint64_t)cnt << 10) | (uint64_t)tid) : ~0ull;
    len_of[tid] = 0;
    if (tid < 64) { bl_count[tid] = 0; first_code[tid] = 0; }
    if (tid == 0) { n_used_s = 0; max_len_s = 0; }
    __syncthreads();
    if (cnt) atomicAdd(&n_used_s, 1u);

    // 2. bitonic sort of the 1024 keys, ascending
    for (uint32_t k = 2; k <= kMaxSym; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            __syncthreads();
            const uint32_t ixj = (uint32_t)tid ^ j;
            if (ixj > (uint32_t)tid) {
                const uint64_t x = key[tid], y = key[ixj];
                const bool up = ((uint32_t)tid & k) == 0;
                if ((x > y) == up) { key[tid] = y; key[ixj] = x; }
            }
        }
    }
    __syncthreads();
    const uint32_t n = n_used_s;

    // 3. two-queue merge (serial, one lane)
    if ((uint32_t)tid < n) weight[tid] = key[tid] >> 10;
    __syncthreads();
    if (tid == 0 && n >= 2) {
        uint32_t q1 = 0, q2 = n, next = n;
        while (next < 2 * n - 1) {
            uint32_t pick[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const bool have_leaf = q1 < n, have_int = q2 < next;
                if (have_leaf && (!have_int || weight[q1] <= weight[q2])) pick[t] = q1++;
                else pick[t] = q2++;
            }
            weight[next] = weight[pick[0]] + weight[pick[1]];
            parent[pick[0]] = (uint16_t)next;
            parent[pick[1]] = (uint16_t)next;
            ++next;
        }
    }
    __syncthreads();

    // 4. depth of every leaf = its code length
    if ((uint32_t)tid < n) {
        uint32_t depth = 0;
        if (n == 1) depth = 1;
        else {
            const uint32_t root = 2 * n - 2;
            for (uint32_t v = tid; v != root; v = parent[v]) ++depth;
        }
        const uint32_t symbol = (uint32_t)(key[tid] & 1023u);
        len_of[symbol] = depth;
        atomicAdd(&bl_count[depth & 63u], 1u);
        atomicMax(&max_len_s, depth);
    }
    __syncthreads();

    // 5. canonical codes: first code of each length, then rank within the length
    if (tid == 0) {
        uint64_t code = 0;
        for (int L = 1; L < 64; ++L) {
            code = (code + (uint64_t)(L > 1 ? bl_count[L - 1] : 0u)) << 1;
            first_code[L] = code;
        }
    }
    __syncthreads();
    const uint32_t L = len_of[tid];
    uint64_t entry = 0;
    if (L) {
        uint32_t rank = 0;
        for (int j = 0; j < tid; ++j) rank += (len_of[j] == L) ? 1u : 0u;
        entry = ((uint64_t)L << 56) | (first_code[L] + rank);
    }
    a.codes[tid] = entry;
    a.lens[tid] = (uint8_t)L;
    // container section `lens`: 2*radius bytes, zero padded to a multiple of 16
    const uint32_t padded = (nsym + 15u) & ~15u;
    if ((uint32_t)tid < padded) a.out[a.lay.off_lens + tid] = ((uint32_t)tid < nsym) ? (uint8_t)L : 0;
    if (tid == 0) a.meta[kMetaMaxLen] = max_len_s;
}

}  // namespace

void launch_codebook(const CompressArgs &a, Profiler *prof, hipStream_t st)
{
    launch(prof, kKCodebook, k_codebook, dim3(1), dim3(kCbThreads), st, a);
}

}  // namespace cmpz
