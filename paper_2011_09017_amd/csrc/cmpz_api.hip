// Host side of libcmpz: the C ABI of include/cmpz.h.  Argument checks, the fp32
// quantiser constants, the container layout and kernel launches; no arithmetic
// of the method runs on the host beyond those three constants.
#include "../../include/cmpz.h"
#include "cmpz_internal.h"

#include <cmath>
#include <cstring>
#include <new>

namespace cmpz {
const char *const kKernelNames[kKernelCount] = {
    "k_quant_lorenzo_split_hist", "k_codebook", "k_encode", "k_outliers",
    "k_empty_container", "k_decode_tables", "k_decode", "k_patch_outliers", "k_row_scan",
    "k_col_scan_dequant", "k_decode_fused", "k_decode_fused_rest", "k_controller_stats"};
}  // namespace cmpz

using namespace cmpz;

struct cmp_ctx {
    cmp_config cfg;
    int        device;
    uint64_t   max_chunks;
    uint8_t   *d_base;          // one allocation, carved up below
    uint16_t  *d_sym;
    uint32_t  *d_hist, *d_hist_copy, *d_meta, *d_status, *d_outl_cnt;
    uint64_t  *d_desc;
    uint8_t   *d_lens;
    uint64_t  *d_codes;
    void      *d_tables;
    uint32_t  *d_items;      // item list of the fused decode kernels
    uint32_t  *h_hint;       // pinned host word the decode kernels report to (see launch_decode_fused)
    uint32_t  *d_hint;       // its device address
    ControllerScratch *d_ctl;
    ControllerResult  *d_ctl_result;
    uint64_t   last_numel;
    CompressArgs pending;       // what cmp_compress_begin left for cmp_compress_finish
    bool       has_pending;
    Profiler   prof;
};

namespace {

uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

bool config_ok(const cmp_config &c)
{
    if (c.radius < 1 || c.radius > kMaxSym / 2) return false;
    if (c.chunk != kChunk) return false;
    if (c.sub != 32 && c.sub != 64 && c.sub != 128) return false;
    if (c.guard_shift < 1 || c.guard_shift > 23) return false;
    if (c.max_numel >= (1ull << 32)) return false;
    return true;
}

bool shape_numel(const int64_t shape[4], uint64_t *numel)
{
    if (!shape) return false;
    uint64_t n = 1;
    for (int i = 0; i < 4; ++i) {
        if (shape[i] < 0 || shape[i] > 0xffffffffLL) return false;
        n *= (uint64_t)shape[i];
        if (n >= (1ull << 32)) return false;
    }
    *numel = n;
    return true;
}

// eb_in = eb - eb*2^-g, s = 2*eb_in, r = 1/s, each a single fp32 operation.
bool constants(float eb, uint32_t guard_shift, float *s, float *r)
{
    if (!(eb >= 0x1p-60f && eb <= 0x1p60f)) return false;
    volatile float g = std::ldexp(eb, -(int)guard_shift);
    volatile float e = eb - g;
    volatile float step = 2.0f * e;
    volatile float rec = 1.0f / step;
    *s = step;
    *r = rec;
    return true;
}

Layout make_layout(uint64_t numel, const cmp_config &c)
{
    Layout l;
    l.nchunks = (uint32_t)((numel + c.chunk - 1) / c.chunk);
    l.nsub = c.chunk / c.sub;
    l.off_lens = kHeaderBytes;
    l.off_chunk_off = l.off_lens + align_up(2ull * c.radius, 16);
    l.off_outl_off = l.off_chunk_off + align_up(4ull * ((uint64_t)l.nchunks + 1), 16);
    l.off_sub_bits = l.off_outl_off + align_up(4ull * ((uint64_t)l.nchunks + 1), 16);
    l.off_payload = l.off_sub_bits + align_up(2ull * (uint64_t)l.nchunks * l.nsub, 16);
    return l;
}

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
        if (prev == dev) prev = -1;
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

int status_to_code(uint32_t st)
{
    if (st & kStInternal) return CMP_E_HIP;
    if (st & kStFormat) return CMP_E_FORMAT;
    if (st & kStMismatch) return CMP_E_MISMATCH;
    if (st & kStNoSpace) return CMP_E_NOSPACE;
    if (st & kStRange) return CMP_W_RANGE;
    return CMP_OK;
}

}  // namespace

extern "C" {

void cmp_default_config(cmp_config *cfg)
{
    if (!cfg) return;
    cfg->radius = 512; cfg->chunk = kChunk; cfg->sub = 128; cfg->guard_shift = 7;
    cfg->max_numel = 1ull << 28;
}

int cmp_create(cmp_ctx **out, const cmp_config *cfg, int device)
{
    if (!out) return CMP_E_ARG;
    *out = nullptr;
    cmp_config c;
    if (cfg) c = *cfg; else cmp_default_config(&c);
    if (!config_ok(c)) return CMP_E_ARG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess) return CMP_E_HIP;
    if (device < 0 || device >= ndev) return CMP_E_ARG;
    DeviceGuard guard(device);
    if (!guard.ok) return CMP_E_HIP;

    cmp_ctx *ctx = new (std::nothrow) cmp_ctx();
    if (!ctx) return CMP_E_HIP;
    ctx->cfg = c;
    ctx->device = device;
    ctx->max_chunks = (c.max_numel + c.chunk - 1) / c.chunk;
    ctx->last_numel = 0;
    ctx->has_pending = false;

    uint64_t off = 0;
    auto carve = [&](uint64_t bytes) { uint64_t o = off; off = align_up(off + bytes, 256); return o; };
    const uint64_t o_sym = carve(2 * (ctx->max_chunks * c.chunk + 16));   // whole chunks: readable past numel
    const uint64_t o_hist = carve(4 * kMaxSym * kHistCopies);
    const uint64_t o_hist_copy = carve(4 * kMaxSym);
    const uint64_t o_desc = carve(8 * (ctx->max_chunks + 1));
    const uint64_t o_ocnt = carve(4 * (ctx->max_chunks + 1));
    const uint64_t o_meta = carve(4 * kMetaWords);
    const uint64_t o_status = carve(4);
    const uint64_t o_lens = carve(kMaxSym);
    const uint64_t o_codes = carve(8 * kMaxSym);
    const uint64_t o_tables = carve(decode_tables_bytes());
    const uint64_t o_items = carve(4 * fused_item_words(c.max_numel));
    const uint64_t o_ctl = carve(sizeof(ControllerScratch));
    const uint64_t o_ctl_result = carve(sizeof(ControllerResult));
    if (hipMalloc(reinterpret_cast<void **>(&ctx->d_base), off) != hipSuccess) { delete ctx; return CMP_E_HIP; }
    // only the small control words need a defined start value; the symbol scratch does not
    if (hipMemset(ctx->d_base + o_hist, 0, off - o_hist) != hipSuccess) {
        (void)hipFree(ctx->d_base); delete ctx; return CMP_E_HIP;
    }
    ctx->d_sym = reinterpret_cast<uint16_t *>(ctx->d_base + o_sym);
    ctx->d_hist = reinterpret_cast<uint32_t *>(ctx->d_base + o_hist);
    ctx->d_hist_copy = reinterpret_cast<uint32_t *>(ctx->d_base + o_hist_copy);
    ctx->d_desc = reinterpret_cast<uint64_t *>(ctx->d_base + o_desc);
    ctx->d_outl_cnt = reinterpret_cast<uint32_t *>(ctx->d_base + o_ocnt);
    ctx->d_meta = reinterpret_cast<uint32_t *>(ctx->d_base + o_meta);
    ctx->d_status = reinterpret_cast<uint32_t *>(ctx->d_base + o_status);
    ctx->d_lens = ctx->d_base + o_lens;
    ctx->d_codes = reinterpret_cast<uint64_t *>(ctx->d_base + o_codes);
    ctx->d_tables = ctx->d_base + o_tables;
    ctx->d_items = reinterpret_cast<uint32_t *>(ctx->d_base + o_items);
    ctx->h_hint = nullptr; ctx->d_hint = nullptr;
    if (hipHostMalloc(reinterpret_cast<void **>(&ctx->h_hint), 64, hipHostMallocMapped) != hipSuccess ||
        hipHostGetDevicePointer(reinterpret_cast<void **>(&ctx->d_hint), ctx->h_hint, 0) != hipSuccess) {
        if (ctx->h_hint) (void)hipHostFree(ctx->h_hint);
        (void)hipFree(ctx->d_base); delete ctx; return CMP_E_HIP;
    }
    *ctx->h_hint = 1;                                  // nothing known yet: assume listed items
    ctx->d_ctl = reinterpret_cast<ControllerScratch *>(ctx->d_base + o_ctl);
    ctx->d_ctl_result = reinterpret_cast<ControllerResult *>(ctx->d_base + o_ctl_result);
    *out = ctx;
    return CMP_OK;
}

void cmp_destroy(cmp_ctx *ctx)
{
    if (!ctx) return;
    DeviceGuard guard(ctx->device);
    (void)hipDeviceSynchronize();
    for (hipEvent_t e : ctx->prof.pool) (void)hipEventDestroy(e);
    if (ctx->h_hint) (void)hipHostFree(ctx->h_hint);
    (void)hipFree(ctx->d_base);
    delete ctx;
}

size_t cmp_bound(const cmp_ctx *ctx, const int64_t shape[4])
{
    uint64_t numel;
    if (!ctx || !shape_numel(shape, &numel)) return 0;
    const Layout l = make_layout(numel, ctx->cfg);
    uint32_t flat = 1;
    while ((1u << flat) < 2 * ctx->cfg.radius) ++flat;
    // a Huffman code is never longer in total than the flat code; each chunk pads < 16 bytes;
    // every element may be an outlier (two 4-byte records)
    const uint64_t payload = (numel * flat + 7) / 8 + 16ull * l.nchunks;
    return (size_t)(l.off_payload + align_up(payload, 16) + 2 * align_up(4 * numel, 16));
}

namespace {

// Argument checks and everything of CompressArgs that does not depend on the output buffer.
int fill_compress_args(cmp_ctx *ctx, const float *d_x, const int64_t shape[4], float eb, CompressArgs *out)
{
    uint64_t numel;
    float s, r;
    if (!ctx || !shape_numel(shape, &numel)) return CMP_E_ARG;
    if (numel > ctx->cfg.max_numel || (numel > 0 && !d_x)) return CMP_E_ARG;
    if (!constants(eb, ctx->cfg.guard_shift, &s, &r)) return CMP_E_ARG;
    if (reinterpret_cast<uintptr_t>(d_x) & 15) return CMP_E_ARG;

    CompressArgs a;
    std::memset(&a, 0, sizeof(a));
    a.lay = make_layout(numel, ctx->cfg);
    a.x = d_x;
    a.numel = (uint32_t)numel;
    a.H = (uint32_t)shape[2]; a.W = (uint32_t)shape[3]; a.HW = a.H * a.W;
    for (int i = 0; i < 4; ++i) a.shape[i] = (uint32_t)shape[i];
    a.radius = ctx->cfg.radius; a.sub = ctx->cfg.sub; a.guard_shift = ctx->cfg.guard_shift;
    std::memcpy(&a.eb_bits, &eb, 4);
    a.r = r;
    a.sym = ctx->d_sym; a.hist = ctx->d_hist; a.hist_copy = ctx->d_hist_copy;
    a.lens = ctx->d_lens; a.codes = ctx->d_codes;
    a.desc = ctx->d_desc; a.outl_cnt = ctx->d_outl_cnt;
    // encode tiles: every tile costs one ticket (a serialised atomic), so as large as still
    // leaves several hundred of them to spread over the chip
    a.tile_chunks = 8;
    while (a.tile_chunks > 1 && (a.lay.nchunks + a.tile_chunks - 1) / a.tile_chunks < 768) a.tile_chunks >>= 1;
    a.meta = ctx->d_meta; a.status = ctx->d_status;
    *out = a;
    return CMP_OK;
}

}  // namespace

int cmp_compress(cmp_ctx *ctx, const float *d_x, const int64_t shape[4], float eb, void *d_out,
                 size_t out_cap, size_t *h_size, void *stream)
{
    CompressArgs a;
    if (!d_out || (reinterpret_cast<uintptr_t>(d_out) & 15)) return CMP_E_ARG;
    const int rc = fill_compress_args(ctx, d_x, shape, eb, &a);
    if (rc != CMP_OK) return rc;
    if (ctx->has_pending) return CMP_E_ARG;                  // between cmp_compress_begin and _finish
    if (out_cap < a.lay.off_payload) {
        if (h_size) *h_size = (size_t)a.lay.off_payload;
        return CMP_E_NOSPACE;
    }
    a.out = static_cast<uint8_t *>(d_out);
    a.out_cap = out_cap;

    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    launch_compress_begin(a, &ctx->prof, st);
    launch_compress_finish(a, &ctx->prof, st);
    ctx->last_numel = a.numel;
    if (hipGetLastError() != hipSuccess) return CMP_E_HIP;
    if (h_size) return cmp_compressed_size(ctx, d_out, h_size, stream);
    return CMP_OK;
}

int cmp_compress_begin(cmp_ctx *ctx, const float *d_x, const int64_t shape[4], float eb, void *stream)
{
    CompressArgs a;
    const int rc = fill_compress_args(ctx, d_x, shape, eb, &a);
    if (rc != CMP_OK) return rc;
    if (ctx->has_pending) return CMP_E_ARG;                  // the previous begin was never finished
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    launch_compress_begin(a, &ctx->prof, static_cast<hipStream_t>(stream));
    if (hipGetLastError() != hipSuccess) return CMP_E_HIP;
    ctx->pending = a;
    ctx->has_pending = true;
    return CMP_OK;
}

int cmp_compress_finish(cmp_ctx *ctx, void *d_out, size_t out_cap, size_t *h_size, void *stream)
{
    if (!ctx || !ctx->has_pending) return CMP_E_ARG;
    if (!d_out || (reinterpret_cast<uintptr_t>(d_out) & 15)) return CMP_E_ARG;
    CompressArgs a = ctx->pending;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ctx->has_pending = false;
    if (out_cap < a.lay.off_payload) {
        // nothing can be written; drop what the first sweep accumulated so that the context is clean
        if (hipMemsetAsync(ctx->d_hist, 0, 4 * kMaxSym * kHistCopies, st) != hipSuccess) return CMP_E_HIP;
        if (hipMemsetAsync(ctx->d_meta + kMetaRangeEvents, 0, 4, st) != hipSuccess) return CMP_E_HIP;
        if (h_size) *h_size = (size_t)a.lay.off_payload;
        return CMP_E_NOSPACE;
    }
    a.out = static_cast<uint8_t *>(d_out);
    a.out_cap = out_cap;
    launch_compress_finish(a, &ctx->prof, st);
    ctx->last_numel = a.numel;
    if (hipGetLastError() != hipSuccess) return CMP_E_HIP;
    if (h_size) return cmp_compressed_size(ctx, d_out, h_size, stream);
    return CMP_OK;
}

int cmp_compressed_size(cmp_ctx *ctx, const void *d_buf, size_t *h_size, void *stream)
{
    if (!ctx || !d_buf || !h_size) return CMP_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Header hd;
    if (hipMemcpyAsync(&hd, d_buf, sizeof(hd), hipMemcpyDeviceToHost, st) != hipSuccess) return CMP_E_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return CMP_E_HIP;
    if (hd.magic != kMagic || hd.version != kVersion) return CMP_E_FORMAT;
    *h_size = (size_t)hd.total_size;
    if (hd.status != 0) return CMP_E_NOSPACE;
    if (hd.range_events != 0) return CMP_W_RANGE;
    return CMP_OK;
}

int cmp_decompress(cmp_ctx *ctx, const void *d_buf, size_t size, const int64_t shape[4], float eb,
                   float *d_xout, void *stream)
{
    uint64_t numel;
    float s, r;
    if (!ctx || !d_buf || !shape_numel(shape, &numel)) return CMP_E_ARG;
    if (numel > ctx->cfg.max_numel || (numel > 0 && !d_xout)) return CMP_E_ARG;
    if (!constants(eb, ctx->cfg.guard_shift, &s, &r)) return CMP_E_ARG;
    if ((reinterpret_cast<uintptr_t>(d_buf) & 15) || (reinterpret_cast<uintptr_t>(d_xout) & 15)) return CMP_E_ARG;

    DecompressArgs a;
    std::memset(&a, 0, sizeof(a));
    a.lay = make_layout(numel, ctx->cfg);
    if (size < a.lay.off_payload) return CMP_E_FORMAT;       // cannot even hold the fixed sections
    a.buf = static_cast<const uint8_t *>(d_buf);
    a.size = size;
    a.xout = d_xout;
    a.numel = (uint32_t)numel;
    a.planes = (uint32_t)(shape[0] * shape[1]);
    a.H = (uint32_t)shape[2]; a.W = (uint32_t)shape[3]; a.HW = a.H * a.W;
    for (int i = 0; i < 4; ++i) a.shape[i] = (uint32_t)shape[i];
    a.radius = ctx->cfg.radius; a.sub = ctx->cfg.sub; a.guard_shift = ctx->cfg.guard_shift;
    std::memcpy(&a.eb_bits, &eb, 4);
    a.s = s;
    a.meta = ctx->d_meta; a.status = ctx->d_status;

    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    launch_decompress(a, ctx->d_tables, ctx->d_items, ctx->h_hint, ctx->d_hint, &ctx->prof,
                      static_cast<hipStream_t>(stream));
    if (hipGetLastError() != hipSuccess) return CMP_E_HIP;
    return CMP_OK;
}

int cmp_last_status(cmp_ctx *ctx, void *stream)
{
    if (!ctx) return CMP_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t word = 0;
    if (hipMemcpyAsync(&word, ctx->d_status, 4, hipMemcpyDeviceToHost, st) != hipSuccess) return CMP_E_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return CMP_E_HIP;
    if (word) {
        const uint32_t zero = 0;
        if (hipMemcpyAsync(ctx->d_status, &zero, 4, hipMemcpyHostToDevice, st) != hipSuccess) return CMP_E_HIP;
        if (hipStreamSynchronize(st) != hipSuccess) return CMP_E_HIP;
    }
    return status_to_code(word);
}

int cmp_debug_stage(cmp_ctx *ctx, int which, const void **d_ptr, size_t *bytes)
{
    if (!ctx || !d_ptr || !bytes) return CMP_E_ARG;
    const size_t nsym = 2 * (size_t)ctx->cfg.radius;
    switch (which) {
    case CMP_STAGE_QUANT_CODES: *d_ptr = ctx->d_sym; *bytes = 2 * (size_t)ctx->last_numel; return CMP_OK;
    case CMP_STAGE_HIST: *d_ptr = ctx->d_hist_copy; *bytes = 4 * nsym; return CMP_OK;
    case CMP_STAGE_LENS: *d_ptr = ctx->d_lens; *bytes = nsym; return CMP_OK;
    case CMP_STAGE_CODES: *d_ptr = ctx->d_codes; *bytes = 8 * nsym; return CMP_OK;
    case CMP_STAGE_COUNTERS: *d_ptr = ctx->d_meta; *bytes = 4 * kMetaWords; return CMP_OK;
    default: return CMP_E_ARG;
    }
}

int cmp_profile(cmp_ctx *ctx, int enable)
{
    if (!ctx) return CMP_E_ARG;
    ctx->prof.enabled = enable != 0;
    if (enable) { ctx->prof.recs.clear(); ctx->prof.used = 0; }
    return CMP_OK;
}

int cmp_profile_read(cmp_ctx *ctx, void *stream, int cap, const char **names, double *total_ms,
                     uint64_t *launches)
{
    if (!ctx || cap < 0 || (cap > 0 && (!names || !total_ms || !launches))) return CMP_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return CMP_E_HIP;
    double ms[kKernelCount] = {0};
    uint64_t cnt[kKernelCount] = {0};
    for (const Profiler::Rec &r : ctx->prof.recs) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, r.beg, r.end) != hipSuccess) return CMP_E_HIP;
        ms[r.id] += t;
        cnt[r.id] += 1;
    }
    int n = 0;
    for (int k = 0; k < kKernelCount; ++k) {
        if (!cnt[k]) continue;
        if (n < cap) { names[n] = kKernelNames[k]; total_ms[n] = ms[k]; launches[n] = cnt[k]; }
        ++n;
    }
    return n;
}

void cmp_default_controller_config(cmp_controller_config *cfg)
{
    if (!cfg) return;
    cfg->sigma_frac = 0.01f; cfg->a = 0.32f; cfg->eb_min = 1e-6f; cfg->eb_max = 1.0f;
}

int cmp_estimate_eb(cmp_ctx *ctx, const float *d_act, uint64_t act_numel, const float *d_loss, uint64_t batch_n,
                    uint64_t per_sample, const float *d_mom, uint64_t mom_numel, const cmp_controller_config *cfg,
                    float *h_eb, double *h_stats, void *stream)
{
    if (!ctx || !d_act || !d_loss || !d_mom || !h_eb) return CMP_E_ARG;
    cmp_controller_config c;
    if (cfg) c = *cfg; else cmp_default_controller_config(&c);
    if (!(c.eb_min > 0.0f) || !(c.eb_max >= c.eb_min) || !(c.sigma_frac > 0.0f) || !(c.a > 0.0f)) return CMP_E_ARG;
    if (act_numel == 0 || batch_n == 0 || per_sample == 0 || mom_numel == 0) return CMP_E_ARG;
    if (batch_n > kMaxBatch || per_sample >= (1ull << 32) || batch_n * per_sample >= (1ull << 32)) return CMP_E_ARG;
    if (act_numel >= (1ull << 32) || mom_numel >= (1ull << 32)) return CMP_E_ARG;
    if ((reinterpret_cast<uintptr_t>(d_act) | reinterpret_cast<uintptr_t>(d_loss) | reinterpret_cast<uintptr_t>(d_mom)) & 15)
        return CMP_E_ARG;

    ControllerArgs a;
    a.act = d_act; a.loss = d_loss; a.mom = d_mom;
    a.n_act = (uint32_t)act_numel; a.n_loss = (uint32_t)(batch_n * per_sample); a.n_mom = (uint32_t)mom_numel;
    a.batch_n = (uint32_t)batch_n; a.per_sample = (uint32_t)per_sample;
    a.sigma_frac = c.sigma_frac; a.a = c.a; a.eb_min = c.eb_min; a.eb_max = c.eb_max;
    a.scratch = ctx->d_ctl; a.result = ctx->d_ctl_result;

    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    launch_controller(a, &ctx->prof, st);
    ControllerResult res;
    if (hipMemcpyAsync(&res, ctx->d_ctl_result, sizeof(res), hipMemcpyDeviceToHost, st) != hipSuccess) return CMP_E_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return CMP_E_HIP;
    *h_eb = res.eb;
    if (h_stats) { h_stats[0] = res.stats[0]; h_stats[1] = res.stats[1]; h_stats[2] = res.stats[2]; }
    return res.rc ? CMP_W_RANGE : CMP_OK;
}

const char *cmp_strerror(int code)
{
    switch (code) {
    case CMP_OK: return "ok";
    case CMP_E_ARG: return "invalid argument";
    case CMP_E_NOSPACE: return "output capacity too small for the container";
    case CMP_E_FORMAT: return "not a valid container";
    case CMP_E_MISMATCH: return "container does not match shape, error bound or configuration";
    case CMP_E_HIP: return "HIP runtime error";
    case CMP_W_RANGE: return "values outside the quantiser range were clamped";
    default: return "unknown code";
    }
}

}  // extern "C"
