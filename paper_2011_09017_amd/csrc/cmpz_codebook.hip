// Huffman codebook on the GPU: histogram -> code lengths -> canonical codes.
// One workgroup per tensor; no host round trip between the two sweeps of a compress.
//
// Rule (fixes one of the equally optimal codebooks): leaves sorted ascending by
// (count, symbol); two FIFO queues, leaves and internal nodes in creation order;
// the lighter head is taken, a leaf before an internal node of equal weight.
// Codes are canonical: ordered by (length, symbol), first code 0, read MSB first.
//
// The merge runs in rounds that join up to 32 pairs at once (see step 4).  Sorting is by
// counting ranks in blocks of 64 and binary search across blocks, depths by walking parent
// links, ranks within a length by wave ballots.
#include "cmpz_internal.h"

namespace cmpz {
namespace {

constexpr int kCbThreads = 1024;
constexpr uint32_t kInf = 0xffffffffu;       // "no such node"; real weights stay below 2^32 - 8192, the largest tensor

__device__ __forceinline__ uint32_t rdlane(uint32_t v, uint32_t l)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)l);
}

// LDS written by some lanes of a wave is read by others: the hardware keeps a wave's LDS
// operations in order, this keeps the compiler from moving them across.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__global__ __launch_bounds__(kCbThreads) void k_codebook(BatchC b)
{
    // one workgroup per tensor of the group
    const uint32_t ti = blockIdx.x;
    uint32_t *__restrict__ g_hist = b.hist + (uint64_t)ti * kHistCopies * kMaxSym;
    const OutRef oref = resolve_out(b.t[ti]);
    uint8_t *__restrict__ out = oref.out;
    __shared__ uint64_t key[kMaxSym];            // used symbols, compacted: count << 10 | symbol
    __shared__ uint64_t skey[kMaxSym];           // the same, every block of 64 in ascending order
    __shared__ uint32_t leaf_w[kMaxSym + 192];   // leaf weights, ascending, padded with kInf
    __shared__ uint16_t leaf_sym[kMaxSym];
    __shared__ uint32_t node_w[kMaxSym + 192];   // internal node weights in creation order, kInf = not made
    __shared__ uint16_t parent[2 * kMaxSym];     // node ids: leaves 0..n-1, internal n..2n-2
    __shared__ uint32_t pair_w[64];              // weights of a round's nodes in their common order
    __shared__ uint32_t len_of[kMaxSym];         // code length per symbol
    __shared__ uint32_t wave_cnt[16][64];
    __shared__ uint32_t bl_count[64];
    __shared__ uint64_t first_code[64];
    __shared__ uint32_t wave_used[16];
    __shared__ uint32_t max_len_s;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const uint32_t nsym = 2 * b.radius;

    // 1. fetch the histogram, leave it zeroed for the next call, keep a copy for inspection
    uint32_t cnt = 0;
#pragma unroll
    for (uint32_t k = 0; k < kHistCopies; ++k) {
        if ((uint32_t)tid < nsym) cnt += g_hist[k * kMaxSym + tid];
        g_hist[k * kMaxSym + tid] = 0;
    }
    b.hist_copy[ti * kMaxSym + tid] = cnt;
    len_of[tid] = 0;
    if (tid < 64) { bl_count[tid] = 0; first_code[tid] = 0; }
    if (tid == 0) max_len_s = 0;

    // 2. compact the used symbols (ballot + per-wave offsets)
    const unsigned long long used_mask = __ballot(cnt != 0);
    if (lane == 0) wave_used[wv] = (uint32_t)__popcll(used_mask);
    __syncthreads();
    uint32_t n = 0, my_slot = 0;
    for (int k = 0; k < 16; ++k) { if (k < wv) my_slot += wave_used[k]; n += wave_used[k]; }
    my_slot += (uint32_t)__popcll(used_mask & ((1ull << lane) - 1ull));
    if (cnt) key[my_slot] = ((uint64_t)cnt << 10) | (uint64_t)tid;
    __syncthreads();

    // 3. sort (keys are distinct).  Every wave orders its own 64 keys by counting the smaller ones
    //    among them; the rank of a key is then its place in its own block plus, by binary search,
    //    the number of smaller keys in every other block.
    const uint32_t nblocks = (n + 63u) >> 6;                         // uniform
    const uint64_t mine = ((uint32_t)tid < n) ? key[tid] : ~0ull;    // past the end: heavier than any key
    uint32_t in_block = (uint32_t)lane;
    if ((uint32_t)wv < nblocks) {
        if ((uint32_t)tid < n) {
            const uint32_t first = (uint32_t)wv << 6;
            const uint32_t here = (n - first < 64u) ? n - first : 64u;
            in_block = 0;
#pragma unroll 8
            for (uint32_t j = 0; j < here; ++j) in_block += (key[first + j] < mine) ? 1u : 0u;
        }
        skey[((uint32_t)wv << 6) + in_block] = mine;
    }
    __syncthreads();
    if ((uint32_t)tid < n) {
        uint32_t rank = in_block;
        for (uint32_t w = 0; w < nblocks; ++w) {
            if (w == (uint32_t)wv) continue;                         // uniform
            const uint64_t *blk = skey + (w << 6);
            uint32_t pos = 0;
#pragma unroll
            for (uint32_t step = 32; step >= 1; step >>= 1) pos += (blk[pos + step - 1] < mine) ? step : 0u;
            pos += (blk[pos] < mine) ? 1u : 0u;                      // a count of 63 may be 64
            rank += pos;
        }
        leaf_w[rank] = (uint32_t)(mine >> 10);
        leaf_sym[rank] = (uint16_t)(mine & 1023u);
    }
    if ((uint32_t)tid < 192) leaf_w[n + tid] = kInf;
    node_w[tid] = kInf;
    if (tid < 192) node_w[kMaxSym + tid] = kInf;
    __syncthreads();

    // 4. the two-queue merge, by wave 0, in rounds of up to 32 nodes.  The sequential rule takes the
    //    unused nodes of both queues in one fixed order -- by weight, a leaf before an internal node
    //    of the same weight, each queue in its own order -- and joins them two by two.  A node made
    //    now weighs at least t, the sum of the two lightest unused nodes, and queues up behind every
    //    node that exists already; so all unused nodes of weight <= t keep their places in that
    //    order whatever is made from them, and a whole round of them can be joined at once: every
    //    lane looks at one leaf and one internal node of the 64 next of either queue, finds their
    //    places in the common order by binary search in the other queue, and the pairs (0,1), (2,3),
    //    ... become the new nodes, already in order of weight.  Activation histograms need about
    //    twenty rounds where the sequential rule needs hundreds of steps.
    if (__builtin_amdgcn_readfirstlane(wv) == 0 && __builtin_amdgcn_readfirstlane((int)n) >= 2) {
        const uint32_t nu = (uint32_t)__builtin_amdgcn_readfirstlane((int)n);   // n came from LDS: tell the compiler it is uniform
        const uint32_t steps = nu - 1;
        uint32_t ql = 0, qi = 0, m = 0;                      // leaves used, internal nodes used, internal nodes made
        while (m < steps) {
            const uint32_t *lw = leaf_w + ql, *iw = node_w + qi;
            const uint32_t LB = lw[lane];                    // kInf past the last leaf
            const uint32_t IB = iw[lane];                    // kInf at and past node m
            const uint64_t l0 = rdlane(LB, 0), l1 = rdlane(LB, 1), i0 = rdlane(IB, 0), i1 = rdlane(IB, 1);
            uint64_t t = l0 + l1;                            // the two lightest of the four heads
            t = (l0 + i0 < t) ? l0 + i0 : t;
            t = (i0 + i1 < t) ? i0 + i1 : t;
            const uint32_t t32 = (t < (uint64_t)kInf) ? (uint32_t)t : kInf - 1u;
            const bool inL = LB <= t32, inI = IB <= t32;     // a prefix of either window
            // places in the common order: internal nodes lighter than the leaf come before it, leaves
            // no heavier than the internal node before that one.  Counts are exact up to 64, and a
            // node with 64 others in front of it is not part of this round anyway.
            // (searches with three pivots per step: three dependent LDS accesses instead of six)
            uint32_t before_leaf = 0, before_node = 0;
#pragma unroll
            for (uint32_t step = 16; step >= 1; step >>= 2) {
                const uint32_t a1 = iw[before_leaf + step - 1], a2 = iw[before_leaf + 2 * step - 1], a3 = iw[before_leaf + 3 * step - 1];
                const uint32_t c1 = lw[before_node + step - 1], c2 = lw[before_node + 2 * step - 1], c3 = lw[before_node + 3 * step - 1];
                before_leaf += (((a1 < LB) ? 1u : 0u) + ((a2 < LB) ? 1u : 0u) + ((a3 < LB) ? 1u : 0u)) * step;
                before_node += (((c1 <= IB) ? 1u : 0u) + ((c2 <= IB) ? 1u : 0u) + ((c3 <= IB) ? 1u : 0u)) * step;
            }
            {
                const uint32_t a = iw[before_leaf], c = lw[before_node];    // counts of 63 may be 64
                before_leaf += (a < LB) ? 1u : 0u;
                before_node += (c <= IB) ? 1u : 0u;
            }
            const uint32_t rank_leaf = (uint32_t)lane + before_leaf, rank_node = (uint32_t)lane + before_node;
            const uint32_t avail = (uint32_t)__popcll(__ballot(inL)) + (uint32_t)__popcll(__ballot(inI));
            uint32_t npairs = avail >> 1;
            npairs = npairs < 32u ? npairs : 32u;
            npairs = npairs < steps - m ? npairs : steps - m;
            // the two lightest nodes always weigh <= t, so a round joins at least one pair; a histogram
            // whose counts do not add up below 2^32 (damaged scratch memory) could break that: leave
            // rather than spin
            if (npairs == 0) {
                if (lane == 0) atomicOr(b.status, kStInternal);
                break;
            }
            const bool use_leaf = inL && rank_leaf < 2u * npairs, use_node = inI && rank_node < 2u * npairs;
            if (use_leaf) { pair_w[rank_leaf] = LB; parent[ql + lane] = (uint16_t)(nu + m + (rank_leaf >> 1)); }
            if (use_node) { pair_w[rank_node] = IB; parent[nu + qi + lane] = (uint16_t)(nu + m + (rank_node >> 1)); }
            wave_lds_sync();
            if ((uint32_t)lane < npairs) node_w[m + lane] = pair_w[2 * lane] + pair_w[2 * lane + 1];
            wave_lds_sync();
            ql += (uint32_t)__popcll(__ballot(use_leaf));
            qi += (uint32_t)__popcll(__ballot(use_node));
            m += npairs;
        }
    }
    __syncthreads();

    // 5. depth of every leaf = its code length
    if ((uint32_t)tid < n) {
        uint32_t depth = 0;
        if (n == 1) depth = 1;
        else {
            const uint32_t root = 2 * n - 2;
            // (bounded: a walk over a complete tree ends at the root after at most kMaxCodeLen steps)
            for (uint32_t v = tid; v != root && depth < 64u; v = parent[v] & (2 * kMaxSym - 1)) ++depth;
        }
        len_of[leaf_sym[tid]] = depth;
        atomicAdd(&bl_count[depth & 63u], 1u);
        atomicMax(&max_len_s, depth);
    }
    __syncthreads();

    // 6. canonical codes: first code of each length, then rank within the length
    if (tid == 0) {
        uint64_t code = 0;
        for (int L = 1; L < 64; ++L) {
            code = (code + (uint64_t)(L > 1 ? bl_count[L - 1] : 0u)) << 1;
            first_code[L] = code;
        }
    }
    const uint32_t L = len_of[tid];
    const uint32_t rank = rank_within_length(L, wave_cnt, tid);       // contains barriers
    const uint64_t entry = L ? (((uint64_t)L << 56) | (first_code[L] + rank)) : 0ull;
    b.codes[ti * kMaxSym + tid] = entry;
    b.lens[ti * kMaxSym + tid] = (uint8_t)L;
    // what the packing kernel looks up while no codeword is longer than 27 bits: the codeword
    // left-aligned in 32 bits with its length in the low five
    b.enc32[ti * kMaxSym + tid] = (L && L <= 27u) ? (((uint32_t)entry << (32u - L)) | L) : 0u;
    // container section `lens`: 2*radius bytes, zero padded to a multiple of 16
    const uint32_t padded = (nsym + 15u) & ~15u;
    if ((uint32_t)tid < padded && oref.cap >= kHeaderBytes + padded) out[kHeaderBytes + tid] = ((uint32_t)tid < nsym) ? (uint8_t)L : 0;
    if (tid == 0) b.tmeta[ti].max_len = max_len_s;
}

}  // namespace

void launch_codebook(const BatchC &b, Profiler *prof, hipStream_t st)
{
    launch(prof, kKCodebook, k_codebook, dim3(b.n), dim3(kCbThreads), st, b);
}

}  // namespace cmpz
