// Huffman codebook on the GPU: histogram -> code lengths -> canonical codes.
// One workgroup; no host round trip between the two sweeps of a compress.
//
// Rule (fixes one of the equally optimal codebooks): leaves sorted ascending by
// (count, symbol); two FIFO queues, leaves and internal nodes in creation order;
// the lighter head is taken, a leaf before an internal node of equal weight.
// Codes are canonical: ordered by (length, symbol), first code 0, read MSB first.
//
// Only the merge itself is serial (one lane, n-1 steps for n used symbols); it
// keeps the heads of both queues in registers and fetches their successors one
// step ahead, so a step costs ALU time only.  Sorting is by counting ranks,
// depths by walking parent links, ranks within a length by wave ballots.
#include "cmpz_internal.h"

namespace cmpz {
namespace {

constexpr int kCbThreads = 1024;
constexpr uint32_t kInf = 0xffffffffu;       // "queue empty"; a real weight reaches it only at the root

__device__ __forceinline__ uint32_t rdlane(uint32_t v, uint32_t l)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)l);
}

__global__ __launch_bounds__(kCbThreads) void k_codebook(BatchC b)
{
    // one workgroup per tensor of the group
    const uint32_t ti = blockIdx.x;
    uint32_t *__restrict__ g_hist = b.hist + (uint64_t)ti * kHistCopies * kMaxSym;
    const OutRef oref = resolve_out(b.t[ti]);
    uint8_t *__restrict__ out = oref.out;
    __shared__ uint64_t key[kMaxSym];            // used symbols, compacted: count << 10 | symbol
    __shared__ uint32_t leaf_w[kMaxSym + 192];   // leaf weights, ascending, padded with kInf
    __shared__ uint16_t leaf_sym[kMaxSym];
    __shared__ uint32_t node_w[kMaxSym + 192];   // internal node weights in creation order, kInf = not made
    __shared__ uint16_t parent[2 * kMaxSym];     // node ids: leaves 0..n-1, internal n..2n-2
    __shared__ uint32_t merge_log[kMaxSym + 64]; // children of each internal node, two 16-bit ids
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

    // 3. sort by counting: the rank of a key is the number of smaller keys (keys are distinct)
    if ((uint32_t)tid < n) {
        const uint64_t mine = key[tid];
        uint32_t rank = 0;
#pragma unroll 8
        for (uint32_t j = 0; j < n; ++j) rank += (key[j] < mine) ? 1u : 0u;
        leaf_w[rank] = (uint32_t)(mine >> 10);
        leaf_sym[rank] = (uint16_t)(mine & 1023u);
    }
    if ((uint32_t)tid < 192) leaf_w[n + tid] = kInf;
    node_w[tid] = kInf;
    if (tid < 192) node_w[kMaxSym + tid] = kInf;
    __syncthreads();

    // 4. two-queue merge by wave 0.  Lane j of LB holds the weight of leaf lbase+j, lane j of IB
    //    that of internal node ibase+j (kInf = not made yet).  The two lightest unused nodes of
    //    either queue are kept in scalar registers; step m makes internal node m and logs its
    //    weight and its two children in lane m%64 of WLOG / PLOG, which go to LDS once per 64
    //    steps.  A lone wave pays about six cycles per instruction whatever its kind, so the steps
    //    between two window slides run in a hand-written loop of about 25 scalar and lane
    //    instructions (the compiler's version of the same step has about 70).
    if (__builtin_amdgcn_readfirstlane(wv) == 0 && __builtin_amdgcn_readfirstlane((int)n) >= 2) {
        uint32_t LB = leaf_w[lane], IB = kInf, WLOG = kInf, PLOG = 0;
        uint32_t lbase = 0, ibase = 0, ql = 0, qi = 0, m = 0;
        uint32_t l0 = rdlane(LB, 0), l1 = rdlane(LB, 1), i0 = kInf, i1 = kInf;
        const uint32_t nu = (uint32_t)__builtin_amdgcn_readfirstlane((int)n);   // n came from LDS: tell the compiler it is uniform
        const uint32_t steps = nu - 1;
        while (m < steps) {
            // rare: start a new log block, slide a window (heads are re-read from the new window)
            if ((m & 63u) == 0 && m != 0) {
                node_w[m - 64 + lane] = WLOG; merge_log[m - 64 + lane] = PLOG;
                WLOG = kInf;
            }
            if (ql - lbase >= 32) {
                lbase = ql; LB = leaf_w[ql + lane];
                l0 = rdlane(LB, 0); l1 = rdlane(LB, 1);
            }
            if (qi - ibase >= 32) {
                // every node made so far must be readable from LDS: flush the open log block too
                node_w[(m & ~63u) + lane] = WLOG;
                ibase = qi;
                IB = node_w[qi + lane];                     // entries at or past m are still kInf
                i0 = rdlane(IB, 0); i1 = rdlane(IB, 1);
            }
            uint32_t lrel = ql - lbase, irel = qi - ibase, slot = m & 63u, mrel = m - ibase;
            // steps that need no slide and no flush: both windows are read at most one lane past
            // their head, which advances by at most two per step
            uint32_t cnt = steps - m;
            cnt = cnt < 64 - slot ? cnt : 64 - slot;
            cnt = cnt < (62 - lrel) / 2 ? cnt : (62 - lrel) / 2;
            cnt = cnt < (62 - irel) / 2 ? cnt : (62 - irel) / 2;
            m += cnt;
            // every scalar operand of the loop below, made provably uniform (a few moves per ~20 steps)
            auto uni = [](uint32_t &v) { v = (uint32_t)__builtin_amdgcn_readfirstlane((int)v); };
            uni(l0); uni(l1); uni(i0); uni(i1); uni(ql); uni(qi); uni(lrel); uni(irel); uni(slot); uni(mrel); uni(cnt);
            uint32_t t1, t2, ws, kd, m0_saved;
            asm volatile(
                "s_mov_b32 %[sv], m0\n"
                "s_nop 3\n"                                        // lane selects below were written by vector moves
                "1:\n"
                "  s_cmp_le_u32 %[l1], %[i0]\n"                    // a leaf wins ties
                "  s_cbranch_scc0 2f\n"
                "  s_add_u32 %[ws], %[l0], %[l1]\n"               // two leaves
                "  s_add_u32 %[t1], %[ql], 1\n"
                "  s_lshl_b32 %[t1], %[t1], 16\n"
                "  s_or_b32 %[kd], %[t1], %[ql]\n"
                "  s_add_u32 %[ql], %[ql], 2\n"
                "  s_add_u32 %[lrel], %[lrel], 2\n"
                "  s_add_u32 %[t1], %[lrel], 1\n"
                "  v_readlane_b32 %[l0], %[LB], %[lrel]\n"
                "  v_readlane_b32 %[l1], %[LB], %[t1]\n"
                "  s_branch 4f\n"
                "2:\n"
                "  s_cmp_lt_u32 %[i1], %[l0]\n"
                "  s_cbranch_scc0 3f\n"
                "  s_add_u32 %[ws], %[i0], %[i1]\n"               // two internal nodes
                "  s_add_u32 %[t1], %[n], %[qi]\n"
                "  s_add_u32 %[t2], %[t1], 1\n"
                "  s_lshl_b32 %[t2], %[t2], 16\n"
                "  s_or_b32 %[kd], %[t2], %[t1]\n"
                "  s_add_u32 %[qi], %[qi], 2\n"
                "  s_add_u32 %[irel], %[irel], 2\n"
                "  s_branch 4f\n"
                "3:\n"
                "  s_add_u32 %[ws], %[l0], %[i0]\n"               // one of each
                "  s_add_u32 %[t1], %[n], %[qi]\n"
                "  s_lshl_b32 %[t1], %[t1], 16\n"
                "  s_or_b32 %[kd], %[t1], %[ql]\n"
                "  s_add_u32 %[ql], %[ql], 1\n"
                "  s_add_u32 %[qi], %[qi], 1\n"
                "  s_add_u32 %[lrel], %[lrel], 1\n"
                "  s_add_u32 %[irel], %[irel], 1\n"
                "  s_mov_b32 %[l0], %[l1]\n"
                "  s_add_u32 %[t1], %[lrel], 1\n"
                "  v_readlane_b32 %[l1], %[LB], %[t1]\n"
                "4:\n"
                "  s_mov_b32 m0, %[slot]\n"                        // log node m
                "  s_nop 0\n"
                "  v_writelane_b32 %[WL], %[ws], m0\n"
                "  v_writelane_b32 %[PL], %[kd], m0\n"
                "  s_cmp_lt_u32 %[mrel], 64\n"
                "  s_cbranch_scc0 5f\n"
                "  s_mov_b32 m0, %[mrel]\n"                        // and make it visible to the internal queue
                "  s_nop 0\n"
                "  v_writelane_b32 %[IB], %[ws], m0\n"
                "5:\n"
                "  s_add_u32 %[t1], %[irel], 1\n"
                "  v_readlane_b32 %[i0], %[IB], %[irel]\n"
                "  v_readlane_b32 %[i1], %[IB], %[t1]\n"
                "  s_add_u32 %[slot], %[slot], 1\n"
                "  s_add_u32 %[mrel], %[mrel], 1\n"
                "  s_sub_u32 %[cnt], %[cnt], 1\n"
                "  s_cmp_lg_u32 %[cnt], 0\n"
                "  s_cbranch_scc1 1b\n"
                "  s_mov_b32 m0, %[sv]\n"
                : [l0] "+s"(l0), [l1] "+s"(l1), [i0] "+s"(i0), [i1] "+s"(i1), [ql] "+s"(ql), [qi] "+s"(qi),
                  [lrel] "+s"(lrel), [irel] "+s"(irel), [slot] "+s"(slot), [mrel] "+s"(mrel), [cnt] "+s"(cnt),
                  [IB] "+v"(IB), [WL] "+v"(WLOG), [PL] "+v"(PLOG),
                  [t1] "=&s"(t1), [t2] "=&s"(t2), [ws] "=&s"(ws), [kd] "=&s"(kd), [sv] "=&s"(m0_saved)
                : [LB] "v"(LB), [n] "s"(nu)
                : "scc", "memory");
        }
        const uint32_t blk = (steps - 1) & ~63u;             // the open log block
        node_w[blk + lane] = WLOG; merge_log[blk + lane] = PLOG;
    }
    __syncthreads();
    // parents from the log: step m made node n+m out of the two logged children
    if ((uint32_t)tid + 1 < n) {
        const uint32_t kids = merge_log[tid];
        parent[kids & 0xffffu] = (uint16_t)(n + tid);
        parent[kids >> 16] = (uint16_t)(n + tid);
    }
    __syncthreads();

    // 5. depth of every leaf = its code length
    if ((uint32_t)tid < n) {
        uint32_t depth = 0;
        if (n == 1) depth = 1;
        else {
            const uint32_t root = 2 * n - 2;
            for (uint32_t v = tid; v != root; v = parent[v]) ++depth;
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
