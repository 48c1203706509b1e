// Error-bound estimator of the adaptive framework (Sections 4.1-4.3): one pass
// over the activation (non-zero fraction R, Eq. 9), the loss arriving at the
// layer (mean over the samples of the largest magnitude, Lbar of Eq. 5) and the
// momentum (mean magnitude, Eq. 7); the workgroup that finishes last evaluates
// sigma = sigma_frac * Mavg and eb = sigma / (a * Lbar * sqrt(N * R)) (Eq. 8)
// in fp64 and leaves the scratch zeroed for the next call.
//
// Pure streaming reads (4 bytes per value, 128-bit loads): HBM bound.  Every
// workgroup takes one contiguous slice of each array, so a thread stays inside
// one sample for many iterations and touches the per-sample maxima rarely.
// Few, long streams: one workgroup per CU with eight loads in flight per thread
// reads at about 4.5 TB/s, where 2048 workgroups reached 1.7 TB/s.
#include "cmpz_internal.h"

#include <type_traits>

namespace cmpz {
namespace {

constexpr int kThreads = 256;
constexpr uint32_t kSliceAlign = 4 * kThreads;
constexpr int kLdsSamples = 4096;

__device__ __forceinline__ double block_sum(double v, double *lds, int tid)
{
    lds[tid] = v;
    __syncthreads();
    for (int s = kThreads / 2; s > 0; s >>= 1) {
        if (tid < s) lds[tid] += lds[tid + s];
        __syncthreads();
    }
    const double r = lds[0];
    __syncthreads();
    return r;
}

// Calls quad(i, v) for every aligned group of four values [i, i+4) of p[lo, hi) and one(k, x) for the
// values of the ragged tail; lo is a multiple of 4.  Eight 128-bit loads per thread are in flight,
// and the next eight are issued before the current ones are consumed: with one or two waves per
// SIMD nothing else would cover the arithmetic.
template <class QUAD, class ONE>
__device__ __forceinline__ void stream_slice(const float *__restrict__ p, uint32_t lo, uint32_t hi, int tid, QUAD quad,
                                             ONE one)
{
    constexpr uint32_t kBatch = 8, kStep = kBatch * kSliceAlign;
    uint32_t i = lo + 4u * tid;
    auto full = [&](uint32_t at) -> bool { return (uint64_t)at + (kBatch - 1) * kSliceAlign + 4 <= hi; };
    float4 cur[kBatch], nxt[kBatch];
    bool have = full(i);
    if (have) {
#pragma unroll
        for (uint32_t q = 0; q < kBatch; ++q) cur[q] = *reinterpret_cast<const float4 *>(p + i + q * kSliceAlign);
    }
    while (have) {
        const bool more = full(i + kStep) && (uint64_t)i + kStep < hi;
        if (more) {
#pragma unroll
            for (uint32_t q = 0; q < kBatch; ++q)
                nxt[q] = *reinterpret_cast<const float4 *>(p + i + kStep + q * kSliceAlign);
        }
#pragma unroll
        for (uint32_t q = 0; q < kBatch; ++q) quad(i + q * kSliceAlign, cur[q]);
        i += kStep;
        have = more;
#pragma unroll
        for (uint32_t q = 0; q < kBatch; ++q) cur[q] = nxt[q];
    }
    for (; i < hi; i += kSliceAlign) {
        if (i + 4 <= hi) quad(i, *reinterpret_cast<const float4 *>(p + i));
        else for (uint32_t k = i; k < hi; ++k) one(k, p[k]);
    }
}

__global__ __launch_bounds__(kThreads) void k_controller_stats(ControllerArgs a, FastDiv div_sample)
{
    __shared__ double lds[kThreads];
    __shared__ uint32_t smax[kLdsSamples];                                // per-sample maxima of this workgroup's slice
    __shared__ uint32_t s_last;
    const int tid = threadIdx.x;
    const uint32_t G = gridDim.x, b = blockIdx.x;
    auto slice = [&](uint32_t n, uint32_t &lo, uint32_t &hi) {
        uint64_t len = ((uint64_t)n + G - 1) / G;
        // an odd number of 4 KB blocks: the slices' starting points then spread over all memory
        // channels instead of a power-of-two fraction of them
        len = ((len + kSliceAlign - 1) / kSliceAlign) | 1u;
        len *= kSliceAlign;
        const uint64_t l = (uint64_t)b * len, h = l + len;
        lo = (uint32_t)(l < n ? l : n);
        hi = (uint32_t)(h < n ? h : n);
    };

    // ---- activation: elements that are not zero ----
    uint32_t lo, hi;
    slice(a.n_act, lo, hi);
    uint32_t nz = 0;
    stream_slice(a.act, lo, hi, tid,
                 [&](uint32_t, const float4 &v) { nz += (v.x != 0.0f) + (v.y != 0.0f) + (v.z != 0.0f) + (v.w != 0.0f); },
                 [&](uint32_t, float x) { nz += (x != 0.0f); });
    const double nz_block = block_sum((double)nz, lds, tid);             // < 2^53: exact
    if (tid == 0 && nz_block != 0.0) atomicAdd(&a.scratch->nonzero, (unsigned long long)nz_block);

    // ---- momentum: sum of magnitudes ----
    slice(a.n_mom, lo, hi);
    double ms = 0.0;
    stream_slice(a.mom, lo, hi, tid,
                 [&](uint32_t, const float4 &v) {
                     ms += (double)fabsf(v.x) + (double)fabsf(v.y) + (double)fabsf(v.z) + (double)fabsf(v.w);
                 },
                 [&](uint32_t, float x) { ms += (double)fabsf(x); });
    const double ms_block = block_sum(ms, lds, tid);
    if (tid == 0 && hi > lo) atomicAdd(&a.scratch->msum, ms_block);

    // ---- loss: largest magnitude of every sample (bit patterns of non-negative floats order
    //      like the floats; a NaN pattern is larger than all of them and therefore sticks).
    //      A thread's indices ascend, so it recomputes the sample index only when it leaves a
    //      sample, and then hands the finished maximum to a table in LDS (LDS atomics do not
    //      share a counter with the loads in flight, global ones would drain them); slices that
    //      cover more samples than the table holds use global atomics directly. ----
    slice(a.n_loss, lo, hi);
    const uint32_t s_first = hi > lo ? div_sample.div(lo) : 0u;
    const uint32_t s_count = hi > lo ? div_sample.div(hi - 1) - s_first + 1 : 0u;
    const bool in_lds = s_count <= (uint32_t)kLdsSamples;                 // uniform
    for (uint32_t k = tid; k < (uint32_t)kLdsSamples; k += kThreads) smax[k] = 0;
    __syncthreads();
    auto mag = [](float v) -> uint32_t { return __float_as_uint(fabsf(v)); };
    auto scan_loss = [&](auto lds_c) {
        constexpr bool kInLds = decltype(lds_c)::value;
        uint32_t cur = 0xffffffffu, curmax = 0;
        uint64_t cur_end = 0;                                             // first index past sample `cur`
        auto flush = [&]() {
            if (cur == 0xffffffffu || curmax == 0) return;
            if (kInLds) atomicMax(&smax[cur - s_first], curmax);
            else atomicMax(&a.scratch->maxbits[cur], curmax);
        };
        auto take = [&](uint32_t i, uint32_t bits) {
            if (i >= cur_end) {
                flush();
                cur = div_sample.div(i); curmax = 0;
                cur_end = (uint64_t)(cur + 1) * a.per_sample;
            }
            curmax = bits > curmax ? bits : curmax;
        };
        if ((a.per_sample & 3u) == 0) {                                   // a quad never straddles two samples
            stream_slice(a.loss, lo, hi, tid,
                         [&](uint32_t i, const float4 &v) {
                             const uint32_t m01 = mag(v.x) > mag(v.y) ? mag(v.x) : mag(v.y);
                             const uint32_t m23 = mag(v.z) > mag(v.w) ? mag(v.z) : mag(v.w);
                             take(i, m01 > m23 ? m01 : m23);
                         },
                         [&](uint32_t k, float x) { take(k, mag(x)); });
        } else {
            stream_slice(a.loss, lo, hi, tid,
                         [&](uint32_t i, const float4 &v) {
                             take(i, mag(v.x)); take(i + 1, mag(v.y)); take(i + 2, mag(v.z)); take(i + 3, mag(v.w));
                         },
                         [&](uint32_t k, float x) { take(k, mag(x)); });
        }
        flush();
    };
    if (in_lds) scan_loss(std::true_type{}); else scan_loss(std::false_type{});
    __syncthreads();
    if (in_lds) {
        for (uint32_t k = tid; k < s_count; k += kThreads)
            if (smax[k]) atomicMax(&a.scratch->maxbits[s_first + k], smax[k]);
    }

    // ---- the last workgroup evaluates the estimate and re-arms the scratch ----
    __threadfence();
    __syncthreads();
    if (tid == 0) s_last = (atomicAdd(&a.scratch->done, 1u) == G - 1) ? 1u : 0u;
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    double ls = 0.0;
    for (uint32_t n = tid; n < a.batch_n; n += kThreads) {
        const uint32_t bits = __hip_atomic_load(&a.scratch->maxbits[n], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ls += (double)__uint_as_float(bits);
        a.scratch->maxbits[n] = 0;
    }
    const double lsum = block_sum(ls, lds, tid);
    if (tid == 0) {
        const unsigned long long nonzero =
            __hip_atomic_load(&a.scratch->nonzero, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const double msum = __hip_atomic_load(&a.scratch->msum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const double R = (double)nonzero / (double)a.n_act;
        const double Lbar = lsum / (double)a.batch_n;
        const double Mavg = msum / (double)a.n_mom;
        const double sigma = (double)a.sigma_frac * Mavg;
        const double denom = (double)a.a * Lbar * sqrt((double)a.batch_n * R);
        float eb;
        int32_t rc = 0;
        if (!(denom > 0.0) || !isfinite(denom) || !isfinite(sigma)) { eb = a.eb_min; rc = 1; }
        else {
            eb = (float)(sigma / denom);
            if (!(eb >= a.eb_min)) eb = a.eb_min;
            if (eb > a.eb_max) eb = a.eb_max;
        }
        a.result->eb = eb; a.result->rc = rc;
        a.result->stats[0] = R; a.result->stats[1] = Lbar; a.result->stats[2] = Mavg;
        a.scratch->nonzero = 0; a.scratch->msum = 0.0; a.scratch->done = 0;
    }
}

}  // namespace

void launch_controller(const ControllerArgs &a, Profiler *prof, hipStream_t st)
{
    const uint64_t total = (uint64_t)a.n_act + a.n_loss + a.n_mom;
    uint64_t grid = (total + 16 * kSliceAlign - 1) / (16 * kSliceAlign);          // >= 16 quads per thread
    grid = grid < 1 ? 1 : grid > 256 ? 256 : grid;                                // one per CU
    launch(prof, kKControllerStats, k_controller_stats, dim3((uint32_t)grid), dim3(kThreads), st, a,
           FastDiv::make(a.per_sample));
}

}  // namespace cmpz
