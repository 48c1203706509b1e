// Host side of libcmpz: the C ABI of include/cmpz.h.  Argument checks, the fp32
// quantiser constants, the container layout and kernel launches; no arithmetic
// of the method runs on the host beyond those three constants.
#include "../../include/cmpz.h"
#include "cmpz_internal.h"

#include <cmath>
#include <cstring>
#include <mutex>
#include <new>

namespace cmpz {
const char *const kKernelNames[kKernelCount] = {
    "k_quant_lorenzo_split_hist", "k_codebook", "k_lengths", "k_scan",
    "k_pack", "k_clear", "k_decode_tables", "k_decode", "k_patch_outliers", "k_row_scan",
    "k_col_scan_dequant", "k_decode_fused", "k_controller_stats"};
}  // namespace cmpz

using namespace cmpz;

// Device memory of a context, carved out of one block (from hipMalloc in cmp_create).
struct Scratch {
    // compression (see BatchC)
    uint16_t   *sym;
    uint32_t   *hist, *hist_copy, *enc32, *outl_cnt, *wide, *chunk_bits, *range_units, *range_outl, *range_bits, *status;
    uint8_t    *lens;
    uint64_t   *codes;
    TensorMeta *tmeta;
    // decompression
    uint32_t   *meta;
    void       *tables;
    ControllerScratch *ctl;
    ControllerResult  *ctl_result;
    uint64_t    max_chunks;     // chunks the symbol scratch holds
    uint64_t    max_ranges;
};

struct cmp_ctx {
    cmp_config cfg;
    int        device;
    uint32_t   cus;             // compute units of the device
    uint8_t   *d_base;          // one allocation, carved up into `s`
    Scratch    s;
    uint64_t   last_numel;      // first tensor of the latest compress call (cmp_debug_stage)
    const uint8_t *last_out;
    BatchC     pending;         // what cmp_compress_begin left for cmp_compress_finish
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
    if (c.max_numel > kMaxNumel) return false;
    if ((c.flags & ~CMP_F_ZERO_BLOCKS) || c.reserved) return false;
    return true;
}

bool shape_numel(const int64_t shape[4], uint64_t *numel)
{
    if (!shape) return false;
    uint64_t n = 1;
    for (int i = 0; i < 4; ++i) {
        if (shape[i] < 0 || shape[i] > 0xffffffffLL) return false;
        n *= (uint64_t)shape[i];
        if (n > kMaxNumel) return false;
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

Layout make_layout(uint64_t numel, const cmp_config &c) { return cmpz::make_layout(numel, c.radius, c.sub); }

// Carves the scratch of a context for `max_numel` elements per call out of a block starting at
// `base` (NULL: only the size is wanted).  Returns the bytes needed; *zero_from is the offset
// from which the block must start out as zeros (everything but the symbols).
uint64_t carve_scratch(Scratch *sc, uint8_t *base, uint64_t max_numel, uint64_t *zero_from)
{
    Scratch s;
    s.max_chunks = (max_numel + kChunk - 1) / kChunk + kBatchMax;       // every tensor of a call rounds up
    s.max_ranges = (s.max_chunks + kPackChunks - 1) / kPackChunks + kBatchMax;
    uint64_t off = 0;
    auto carve = [&](uint64_t bytes) { uint64_t o = off; off = align_up(off + bytes, 256); return base + o; };
    s.sym = reinterpret_cast<uint16_t *>(carve(2 * (s.max_chunks * kChunk + 16)));   // whole chunks: readable past numel
    if (zero_from) *zero_from = off;
    s.hist = reinterpret_cast<uint32_t *>(carve(4ull * kMaxSym * kHistCopies * kBatchMax));
    s.hist_copy = reinterpret_cast<uint32_t *>(carve(4ull * kMaxSym * kBatchMax));
    s.lens = carve(1ull * kMaxSym * kBatchMax);
    s.codes = reinterpret_cast<uint64_t *>(carve(8ull * kMaxSym * kBatchMax));
    s.enc32 = reinterpret_cast<uint32_t *>(carve(4ull * kMaxSym * kBatchMax));
    s.outl_cnt = reinterpret_cast<uint32_t *>(carve(4 * s.max_chunks));
    s.wide = reinterpret_cast<uint32_t *>(carve(16 * s.max_chunks));
    s.chunk_bits = reinterpret_cast<uint32_t *>(carve(4 * s.max_chunks));
    s.range_units = reinterpret_cast<uint32_t *>(carve(4 * s.max_ranges));
    s.range_outl = reinterpret_cast<uint32_t *>(carve(4 * s.max_ranges));
    s.range_bits = reinterpret_cast<uint32_t *>(carve(4 * s.max_ranges));
    s.tmeta = reinterpret_cast<TensorMeta *>(carve(sizeof(TensorMeta) * kBatchMax));
    s.status = reinterpret_cast<uint32_t *>(carve(4));
    s.meta = reinterpret_cast<uint32_t *>(carve(4 * kMetaWords));
    s.tables = carve(decode_tables_bytes());
    s.ctl = reinterpret_cast<ControllerScratch *>(carve(sizeof(ControllerScratch)));
    s.ctl_result = reinterpret_cast<ControllerResult *>(carve(sizeof(ControllerResult)));
    if (sc) *sc = s;
    return off;
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
    cfg->flags = 0; cfg->reserved = 0;
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
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus < 1) cus = 256;
    ctx->cus = (uint32_t)cus;
    ctx->last_numel = 0;
    ctx->last_out = nullptr;
    ctx->has_pending = false;

    uint64_t zero_from = 0;
    const uint64_t bytes = carve_scratch(nullptr, nullptr, c.max_numel, &zero_from);
    if (hipMalloc(reinterpret_cast<void **>(&ctx->d_base), bytes) != hipSuccess) { delete ctx; return CMP_E_HIP; }
    // only the small control words need a defined start value; the symbol scratch does not
    if (hipMemset(ctx->d_base + zero_from, 0, bytes - zero_from) != hipSuccess) {
        (void)hipFree(ctx->d_base); delete ctx; return CMP_E_HIP;
    }
    carve_scratch(&ctx->s, ctx->d_base, c.max_numel, nullptr);
    *out = ctx;
    return CMP_OK;
}

void cmp_destroy(cmp_ctx *ctx)
{
    if (!ctx) return;
    DeviceGuard guard(ctx->device);
    (void)hipDeviceSynchronize();
    for (hipEvent_t e : ctx->prof.pool) (void)hipEventDestroy(e);
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

// One tensor of a compress call after the argument checks.
struct CheckedTensor {
    const float *x;
    uint32_t shape[4];
    uint64_t numel;
    uint32_t eb_bits;
    float r;
    Layout lay;
};

int check_tensor(const cmp_config &cfg, const float *d_x, const int64_t shape[4], float eb, CheckedTensor *out)
{
    uint64_t numel;
    float s, r;
    if (!shape_numel(shape, &numel)) return CMP_E_ARG;
    if (numel > cfg.max_numel || (numel > 0 && !d_x)) return CMP_E_ARG;
    if (!constants(eb, cfg.guard_shift, &s, &r)) return CMP_E_ARG;
    if (reinterpret_cast<uintptr_t>(d_x) & 15) return CMP_E_ARG;
    out->x = d_x;
    for (int i = 0; i < 4; ++i) out->shape[i] = (uint32_t)shape[i];
    out->numel = numel;
    std::memcpy(&out->eb_bits, &eb, 4);
    out->r = r;
    out->lay = make_layout(numel, cfg);
    return CMP_OK;
}

// The launch group's common part: configuration and scratch pointers.
void group_begin(BatchC *b, const cmp_config &cfg, const Scratch &s)
{
    std::memset(b, 0, sizeof(*b));
    b->radius = cfg.radius; b->sub = cfg.sub; b->guard_shift = cfg.guard_shift;
    b->zero_blocks = (cfg.flags & CMP_F_ZERO_BLOCKS) ? 1u : 0u;
    b->sym = s.sym; b->hist = s.hist; b->hist_copy = s.hist_copy; b->lens = s.lens; b->codes = s.codes;
    b->enc32 = s.enc32; b->outl_cnt = s.outl_cnt; b->wide = s.wide; b->chunk_bits = s.chunk_bits;
    b->sym_off = cfg.radius > 128 ? cfg.radius - 128 : 0;
    b->range_units = s.range_units; b->range_outl = s.range_outl; b->range_bits = s.range_bits;
    b->tmeta = s.tmeta; b->status = s.status;
}

void group_add(BatchC *b, const CheckedTensor &c, void *d_out, size_t out_cap)
{
    TensorC &t = b->t[b->n++];
    t.x = c.x; t.out = static_cast<uint8_t *>(d_out); t.out_cap = out_cap;
    for (int i = 0; i < 4; ++i) t.shape[i] = c.shape[i];
    t.numel = (uint32_t)c.numel; t.nchunks = c.lay.nchunks; t.eb_bits = c.eb_bits; t.r = c.r;
    t.chunk_base = b->total_chunks;
    t.pack_base = b->pack_wgs;
    b->total_chunks += t.nchunks;
    b->pack_wgs += (t.nchunks + kPackChunks - 1) / kPackChunks;
    t.divW = FastDiv::make(c.shape[3]);
    t.divHW = FastDiv::make(c.shape[2] * c.shape[3]);
}

// Workgroups of the first sweep: few, long-lived ones (every workgroup ends with a flush of its
// histogram, contended atomics), but still several per CU.  Tensors whose rows do not fit the
// tiled kernel get none here and a launch of the untiled kernel each.
// Workgroups of the first sweep: eight are resident per compute unit; a workgroup takes
// sweep_chunks consecutive chunks of one tensor.  One round of them for a small call, up to sixteen
// rounds for a large one, so that the chip does not idle while the slowest workgroup of a single
// round finishes (ResNet-18-shaped stream, 144 256 chunks: 0.89 / 0.68 / 0.67 / 0.66 / 0.64 / 0.63 ms
// for 0.5 / 1 / 2 / 4 / 8 / 16 rounds).
void group_plan_sweep(BatchC *b, uint32_t cus)
{
    const uint32_t slots = 8u * cus;
    uint32_t rounds = b->total_chunks / (slots * 4u);         // at least four chunks per workgroup and round
    rounds = rounds < 1 ? 1 : rounds > 16 ? 16 : rounds;
    const uint32_t want = slots * rounds;
    b->sweep_chunks = (b->total_chunks + want - 1) / want;
    if (b->sweep_chunks < 1) b->sweep_chunks = 1;
    b->sweep_wgs = 0;
    for (uint32_t k = 0; k < b->n; ++k) {
        TensorC &t = b->t[k];
        t.sweep_base = b->sweep_wgs;
        if (sweep1_tiled_fits(t.shape[3])) b->sweep_wgs += (t.nchunks + b->sweep_chunks - 1) / b->sweep_chunks;
    }
}

void group_launch_begin(const BatchC &b, Profiler *prof, hipStream_t st)
{
    launch_sweep1(b, prof, st);
    for (uint32_t k = 0; k < b.n; ++k)
        if (!sweep1_tiled_fits(b.t[k].shape[3])) launch_sweep1_untiled(b, k, prof, st);
}

void group_launch_finish(const BatchC &b, Profiler *prof, hipStream_t st)
{
    launch_codebook(b, prof, st);
    launch_pack(b, prof, st);
}

}  // namespace

int cmp_compress_batch(cmp_ctx *ctx, int n, const float *const *d_x, const int64_t (*shapes)[4], const float *eb,
                       void *const *d_out, const size_t *out_cap, size_t *h_sizes, void *stream)
{
    if (!ctx || n < 0 || (n > 0 && (!d_x || !shapes || !eb || !d_out || !out_cap))) return CMP_E_ARG;
    if (ctx->has_pending) return CMP_E_ARG;                  // between cmp_compress_begin and _finish
    // every argument is checked before anything is launched
    std::vector<CheckedTensor> ck((size_t)n);
    int rc_space = CMP_OK;
    for (int i = 0; i < n; ++i) {
        const int rc = check_tensor(ctx->cfg, d_x[i], shapes[i], eb[i], &ck[i]);
        if (rc != CMP_OK) return rc;
        if (!d_out[i] || (reinterpret_cast<uintptr_t>(d_out[i]) & 15)) return CMP_E_ARG;
        if (out_cap[i] < ck[i].lay.off_payload) {
            if (h_sizes) h_sizes[i] = (size_t)ck[i].lay.off_payload;
            rc_space = CMP_E_NOSPACE;
        }
    }
    if (rc_space != CMP_OK) return rc_space;

    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // launch groups: at most kBatchMax tensors and max_numel elements each; the groups of a call
    // use the same scratch one after the other, in stream order
    int i = 0;
    while (i < n) {
        BatchC b;
        group_begin(&b, ctx->cfg, ctx->s);
        uint64_t elems = 0;
        while (i < n && b.n < (uint32_t)kBatchMax && (b.n == 0 || elems + ck[i].numel <= ctx->cfg.max_numel)) {
            elems += ck[i].numel;
            group_add(&b, ck[i], d_out[i], out_cap[i]);
            ++i;
        }
        group_plan_sweep(&b, ctx->cus);
        group_launch_begin(b, &ctx->prof, st);
        group_launch_finish(b, &ctx->prof, st);
        ctx->last_numel = b.t[0].numel;
        ctx->last_out = b.t[0].out;
    }
    if (hipGetLastError() != hipSuccess) return CMP_E_HIP;
    int worst = CMP_OK;
    if (h_sizes) {
        for (int k = 0; k < n; ++k) {
            const int rc = cmp_compressed_size(ctx, d_out[k], &h_sizes[k], stream);
            if (rc < 0 && (worst >= 0 || rc < worst)) worst = rc;
            else if (rc > 0 && worst == CMP_OK) worst = rc;
        }
    }
    return worst;
}

int cmp_compress(cmp_ctx *ctx, const float *d_x, const int64_t shape[4], float eb, void *d_out,
                 size_t out_cap, size_t *h_size, void *stream)
{
    if (!shape) return CMP_E_ARG;
    const float *xs[1] = {d_x};
    void *outs[1] = {d_out};
    return cmp_compress_batch(ctx, 1, xs, reinterpret_cast<const int64_t (*)[4]>(shape), &eb, outs, &out_cap, h_size,
                              stream);
}

// ---- compression without a context and without any allocation ---------------------------------
// The scratch of this entry point: one array per GPU, in the library's device image, held until
// the process ends.  Host code never uses the array's name as an address: every device has its
// own copy at its own address, looked up once (static_scratch_of) and kept.
constexpr uint64_t kStaticMaxNumel = CMP_STATIC_MAX_NUMEL;
constexpr uint64_t kStaticBytes    = 2 * (kStaticMaxNumel + (uint64_t)(kBatchMax + 1) * kChunk) + (3ull << 20);
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
uint8_t   *g_static_ptr[kMaxDevices];          // per device: address of its copy of `scratch`

// Device `device` must be current.  Returns NULL when the lookup fails.
uint8_t *static_scratch_of(int device)
{
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[device]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_static_ptr[device] = static_cast<uint8_t *>(p);
    }
    return g_static_ptr[device];
}

}  // namespace

int cmp_compress_static(int device, const cmp_config *cfg, const float *d_x, const int64_t shape[4], float eb,
                        void *d_out, size_t out_cap, void *stream)
{
    cmp_config c;
    if (cfg) c = *cfg; else cmp_default_config(&c);
    c.max_numel = kStaticMaxNumel;
    if (!config_ok(c)) return CMP_E_ARG;
    if (!d_out || (reinterpret_cast<uintptr_t>(d_out) & 15)) return CMP_E_ARG;
    CheckedTensor ck;
    const int rc = check_tensor(c, d_x, shape, eb, &ck);     // refuses more than CMP_STATIC_MAX_NUMEL elements
    if (rc != CMP_OK) return rc;
    if (out_cap < ck.lay.off_payload) return CMP_E_NOSPACE;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess) return CMP_E_HIP;
    if (device < 0 || device >= ndev) return CMP_E_ARG;
    DeviceGuard guard(device);
    if (!guard.ok) return CMP_E_HIP;
    uint8_t *base = static_scratch_of(device);
    if (!base) return CMP_E_HIP;
    Scratch sc;
    if (carve_scratch(&sc, base, kStaticMaxNumel, nullptr) > kStaticBytes) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    BatchC b;
    group_begin(&b, c, sc);
    group_add(&b, ck, d_out, out_cap);
    // (at most 2^22 elements: one round of workgroups whatever the device has)
    group_plan_sweep(&b, 256);
    // the array keeps the last call's contents, whatever that call was: what the first sweep adds
    // to must start at zero (a fill kernel, so that the call can be captured into a graph)
    launch_clear(b, nullptr, st);
    group_launch_begin(b, nullptr, st);
    group_launch_finish(b, nullptr, st);
    if (hipGetLastError() != hipSuccess) return CMP_E_HIP;
    return CMP_OK;
}

// ---- a stack of containers whose bookkeeping stays on the device --------------------------------
size_t cmp_arena_state_bytes(uint32_t slots)
{
    return sizeof(ArenaState) + (size_t)(slots ? slots - 1 : 0) * sizeof(ArenaSlot);
}

int cmp_arena_accepts(const cmp_ctx *ctx, const int64_t shape[4])
{
    uint64_t numel;
    if (!ctx || !shape_numel(shape, &numel) || numel == 0 || numel > ctx->cfg.max_numel) return 0;
    TensorD t;
    std::memset(&t, 0, sizeof(t));
    for (int k = 0; k < 4; ++k) t.shape[k] = (uint32_t)shape[k];
    t.numel = (uint32_t)numel;
    return plan_decode_fused(&t, ctx->cfg.sub) ? 1 : 0;
}

int cmp_arena_init(cmp_ctx *ctx, void *d_state, uint32_t slots, void *stream)
{
    if (!ctx || !d_state || slots == 0 || (reinterpret_cast<uintptr_t>(d_state) & 15)) return CMP_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    launch_arena_init(static_cast<ArenaState *>(d_state), slots, static_cast<hipStream_t>(stream));
    return hipGetLastError() == hipSuccess ? CMP_OK : CMP_E_HIP;
}

int cmp_arena_push(cmp_ctx *ctx, void *d_arena, size_t arena_cap, void *d_state, uint32_t slot, const float *d_x,
                   const int64_t shape[4], float eb, void *stream)
{
    if (!ctx || !d_arena || !d_state || (reinterpret_cast<uintptr_t>(d_arena) & (kArenaAlign - 1))) return CMP_E_ARG;
    if (ctx->has_pending) return CMP_E_ARG;
    CheckedTensor ck;
    const int rc = check_tensor(ctx->cfg, d_x, shape, eb, &ck);
    if (rc != CMP_OK) return rc;
    if (!cmp_arena_accepts(ctx, shape)) return CMP_E_ARG;      // what cmp_arena_pop could not take back
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    BatchC b;
    group_begin(&b, ctx->cfg, ctx->s);
    group_add(&b, ck, d_arena, arena_cap);
    b.t[0].arena = static_cast<const ArenaState *>(d_state);
    group_plan_sweep(&b, ctx->cus);
    group_launch_begin(b, &ctx->prof, st);
    group_launch_finish(b, &ctx->prof, st);
    launch_arena_pushed(b, static_cast<ArenaState *>(d_state), slot, st);
    ctx->last_numel = b.t[0].numel;
    ctx->last_out = nullptr;                                   // its place is known to the GPU only
    return hipGetLastError() == hipSuccess ? CMP_OK : CMP_E_HIP;
}

int cmp_arena_pop(cmp_ctx *ctx, const void *d_arena, void *d_state, uint32_t slot, const int64_t shape[4], float eb,
                  float *d_xout, void *stream)
{
    uint64_t numel;
    float s, r;
    if (!ctx || !d_arena || !d_state || !shape_numel(shape, &numel)) return CMP_E_ARG;
    if (numel > ctx->cfg.max_numel || (numel > 0 && !d_xout)) return CMP_E_ARG;
    if (!constants(eb, ctx->cfg.guard_shift, &s, &r)) return CMP_E_ARG;
    if (reinterpret_cast<uintptr_t>(d_xout) & 15) return CMP_E_ARG;
    BatchD b;
    std::memset(&b, 0, sizeof(b));
    b.n = 1;
    b.radius = ctx->cfg.radius; b.sub = ctx->cfg.sub; b.guard_shift = ctx->cfg.guard_shift;
    b.zero_blocks = (ctx->cfg.flags & CMP_F_ZERO_BLOCKS) ? 1u : 0u;
    b.meta = ctx->s.meta; b.status = ctx->s.status;
    TensorD &t = b.t[0];
    t.buf = static_cast<const uint8_t *>(d_arena);
    t.size = 0;
    t.slot = static_cast<const ArenaState *>(d_state)->slot + slot;      // address arithmetic only: a device pointer
    t.xout = d_xout;
    for (int k = 0; k < 4; ++k) t.shape[k] = (uint32_t)shape[k];
    t.numel = (uint32_t)numel;
    std::memcpy(&t.eb_bits, &eb, 4);
    t.s = s;
    // the kernels for shapes outside the fused kernel's plan take their arguments from the host,
    // which does not know where the container lies
    if (!plan_decode_fused(&t, ctx->cfg.sub)) return CMP_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    launch_decode_fused(b, ctx->cus, &ctx->prof, st);
    launch_arena_release(static_cast<ArenaState *>(d_state), slot, st);
    return hipGetLastError() == hipSuccess ? CMP_OK : CMP_E_HIP;
}

int cmp_arena_stats(cmp_ctx *ctx, const void *d_state, uint64_t *h_top, uint64_t *h_peak, uint32_t *h_held,
                    uint32_t *h_failed, void *stream)
{
    if (!ctx || !d_state) return CMP_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ArenaState hd;
    if (hipMemcpyAsync(&hd, d_state, sizeof(hd), hipMemcpyDeviceToHost, st) != hipSuccess) return CMP_E_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return CMP_E_HIP;
    if (h_top) *h_top = hd.top;
    if (h_peak) *h_peak = hd.peak;
    if (h_held) *h_held = hd.nslots;
    if (h_failed) *h_failed = hd.failed;
    return hd.failed ? CMP_E_NOSPACE : CMP_OK;
}

int cmp_compress_begin(cmp_ctx *ctx, const float *d_x, const int64_t shape[4], float eb, void *stream)
{
    if (!ctx) return CMP_E_ARG;
    CheckedTensor c;
    const int rc = check_tensor(ctx->cfg, d_x, shape, eb, &c);
    if (rc != CMP_OK) return rc;
    if (ctx->has_pending) return CMP_E_ARG;                  // the previous begin was never finished
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    BatchC &b = ctx->pending;
    group_begin(&b, ctx->cfg, ctx->s);
    group_add(&b, c, nullptr, 0);
    group_plan_sweep(&b, ctx->cus);
    group_launch_begin(b, &ctx->prof, static_cast<hipStream_t>(stream));
    if (hipGetLastError() != hipSuccess) return CMP_E_HIP;
    ctx->has_pending = true;
    return CMP_OK;
}

int cmp_compress_finish(cmp_ctx *ctx, void *d_out, size_t out_cap, size_t *h_size, void *stream)
{
    if (!ctx || !ctx->has_pending) return CMP_E_ARG;
    if (!d_out || (reinterpret_cast<uintptr_t>(d_out) & 15)) return CMP_E_ARG;
    BatchC &b = ctx->pending;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ctx->has_pending = false;
    const uint64_t fixed = make_layout(b.t[0].numel, ctx->cfg).off_payload;
    if (out_cap < fixed) {
        // nothing can be written; drop what the first sweep accumulated so that the context is clean
        launch_clear(b, &ctx->prof, st);
        if (hipGetLastError() != hipSuccess) return CMP_E_HIP;
        if (h_size) *h_size = (size_t)fixed;
        return CMP_E_NOSPACE;
    }
    b.t[0].out = static_cast<uint8_t *>(d_out);
    b.t[0].out_cap = out_cap;
    group_launch_finish(b, &ctx->prof, st);
    ctx->last_numel = b.t[0].numel;
    ctx->last_out = b.t[0].out;
    if (hipGetLastError() != hipSuccess) return CMP_E_HIP;
    if (h_size) return cmp_compressed_size(ctx, d_out, h_size, stream);
    return CMP_OK;
}

int cmp_compressed_size(cmp_ctx *ctx, const void *d_buf, size_t *h_size, void *stream)
{
    if (!d_buf || !h_size) return CMP_E_ARG;
    int device = 0;
    if (ctx) device = ctx->device;
    else if (hipGetDevice(&device) != hipSuccess) return CMP_E_HIP;
    DeviceGuard guard(device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Header hd;
    if (hipMemcpyAsync(&hd, d_buf, sizeof(hd), hipMemcpyDeviceToHost, st) != hipSuccess) return CMP_E_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return CMP_E_HIP;
    if (hd.magic != kMagic || (hd.version != kVersion && hd.version != kVersionZB)) return CMP_E_FORMAT;
    *h_size = (size_t)hd.total_size;
    if (hd.status != 0) return CMP_E_NOSPACE;
    if (hd.range_events != 0) return CMP_W_RANGE;
    return CMP_OK;
}

int cmp_decompress_batch(cmp_ctx *ctx, int n, const void *const *d_buf, const size_t *size, const int64_t (*shapes)[4],
                         const float *eb, float *const *d_xout, void *stream)
{
    if (!ctx || n < 0 || (n > 0 && (!d_buf || !size || !shapes || !eb || !d_xout))) return CMP_E_ARG;
    // every argument is checked before anything is launched
    std::vector<TensorD> td((size_t)n);
    for (int i = 0; i < n; ++i) {
        uint64_t numel;
        float s, r;
        if (!d_buf[i] || !shape_numel(shapes[i], &numel)) return CMP_E_ARG;
        if (numel > ctx->cfg.max_numel || (numel > 0 && !d_xout[i])) return CMP_E_ARG;
        if (!constants(eb[i], ctx->cfg.guard_shift, &s, &r)) return CMP_E_ARG;
        if ((reinterpret_cast<uintptr_t>(d_buf[i]) & 15) || (reinterpret_cast<uintptr_t>(d_xout[i]) & 15)) return CMP_E_ARG;
        if (size[i] < make_layout(numel, ctx->cfg).off_payload) return CMP_E_FORMAT;   // cannot even hold the fixed sections
        TensorD &t = td[(size_t)i];
        std::memset(&t, 0, sizeof(t));
        t.buf = static_cast<const uint8_t *>(d_buf[i]);
        t.size = size[i];
        t.xout = d_xout[i];
        for (int k = 0; k < 4; ++k) t.shape[k] = (uint32_t)shapes[i][k];
        t.numel = (uint32_t)numel;
        std::memcpy(&t.eb_bits, &eb[i], 4);
        t.s = s;
        if (!plan_decode_fused(&t, ctx->cfg.sub)) t.nitems = 0;
    }
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (int i0 = 0; i0 < n; i0 += kBatchMax) {
        BatchD b;
        std::memset(&b, 0, sizeof(b));
        b.radius = ctx->cfg.radius; b.sub = ctx->cfg.sub; b.guard_shift = ctx->cfg.guard_shift;
        b.zero_blocks = (ctx->cfg.flags & CMP_F_ZERO_BLOCKS) ? 1u : 0u;
        b.meta = ctx->s.meta; b.status = ctx->s.status;
        for (int i = i0; i < n && i < i0 + kBatchMax; ++i) b.t[b.n++] = td[(size_t)i];
        launch_decode_fused(b, ctx->cus, &ctx->prof, st);
        // shapes the fused kernel does not take, and empty tensors: one at a time
        for (uint32_t k = 0; k < b.n; ++k)
            if (!b.t[k].nitems) launch_decompress_unfused(decompress_args(b, b.t[k]), ctx->s.tables, &ctx->prof, st);
    }
    if (hipGetLastError() != hipSuccess) return CMP_E_HIP;
    return CMP_OK;
}

int cmp_decompress(cmp_ctx *ctx, const void *d_buf, size_t size, const int64_t shape[4], float eb,
                   float *d_xout, void *stream)
{
    if (!shape) return CMP_E_ARG;
    const void *bufs[1] = {d_buf};
    float *outs[1] = {d_xout};
    return cmp_decompress_batch(ctx, 1, bufs, &size, reinterpret_cast<const int64_t (*)[4]>(shape), &eb, outs, stream);
}

int cmp_last_status(cmp_ctx *ctx, void *stream)
{
    if (!ctx) return CMP_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t word = 0;
    if (hipMemcpyAsync(&word, ctx->s.status, 4, hipMemcpyDeviceToHost, st) != hipSuccess) return CMP_E_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return CMP_E_HIP;
    if (word) {
        const uint32_t zero = 0;
        if (hipMemcpyAsync(ctx->s.status, &zero, 4, hipMemcpyHostToDevice, st) != hipSuccess) return CMP_E_HIP;
        if (hipStreamSynchronize(st) != hipSuccess) return CMP_E_HIP;
    }
    return status_to_code(word);
}

int cmp_debug_stage(cmp_ctx *ctx, int which, const void **d_ptr, size_t *bytes)
{
    if (!ctx || !d_ptr || !bytes) return CMP_E_ARG;
    const size_t nsym = 2 * (size_t)ctx->cfg.radius;
    switch (which) {
    case CMP_STAGE_QUANT_CODES: {
        // quarter chunks kept with 8 bits per symbol are rewritten with 16 first (waits for the GPU)
        DeviceGuard guard(ctx->device);
        if (!guard.ok) return CMP_E_HIP;
        if (hipDeviceSynchronize() != hipSuccess) return CMP_E_HIP;
        launch_widen(ctx->s.sym, ctx->s.wide, ctx->cfg.radius > 128 ? ctx->cfg.radius - 128 : 0,
                     (uint32_t)((ctx->last_numel + kChunk - 1) / kChunk), nullptr);
        if (hipDeviceSynchronize() != hipSuccess) return CMP_E_HIP;
        *d_ptr = ctx->s.sym; *bytes = 2 * (size_t)ctx->last_numel; return CMP_OK;
    }
    case CMP_STAGE_HIST: *d_ptr = ctx->s.hist_copy; *bytes = 4 * nsym; return CMP_OK;
    case CMP_STAGE_LENS: *d_ptr = ctx->s.lens; *bytes = nsym; return CMP_OK;
    case CMP_STAGE_CODES: *d_ptr = ctx->s.codes; *bytes = 8 * nsym; return CMP_OK;
    case CMP_STAGE_OUTLIER_IDX:
    case CMP_STAGE_OUTLIER_VAL: {
        // the records live in the container: its header says where
        if (!ctx->last_out) return CMP_E_ARG;
        DeviceGuard guard(ctx->device);
        if (!guard.ok) return CMP_E_HIP;
        Header hd;
        if (hipDeviceSynchronize() != hipSuccess) return CMP_E_HIP;
        if (hipMemcpy(&hd, ctx->last_out, sizeof(hd), hipMemcpyDeviceToHost) != hipSuccess) return CMP_E_HIP;
        if (hd.magic != kMagic || hd.status != 0) return CMP_E_FORMAT;
        *d_ptr = ctx->last_out + (which == CMP_STAGE_OUTLIER_IDX ? hd.off_outl_idx : hd.off_outl_val);
        *bytes = 4 * (size_t)hd.n_outliers;
        return CMP_OK;
    }
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
    if (batch_n > kMaxBatch || per_sample > kMaxNumel || batch_n * per_sample > kMaxNumel) return CMP_E_ARG;
    if (act_numel > kMaxNumel || mom_numel > kMaxNumel) return CMP_E_ARG;
    if ((reinterpret_cast<uintptr_t>(d_act) | reinterpret_cast<uintptr_t>(d_loss) | reinterpret_cast<uintptr_t>(d_mom)) & 15)
        return CMP_E_ARG;

    ControllerArgs a;
    a.act = d_act; a.loss = d_loss; a.mom = d_mom;
    a.n_act = (uint32_t)act_numel; a.n_loss = (uint32_t)(batch_n * per_sample); a.n_mom = (uint32_t)mom_numel;
    a.batch_n = (uint32_t)batch_n; a.per_sample = (uint32_t)per_sample;
    a.sigma_frac = c.sigma_frac; a.a = c.a; a.eb_min = c.eb_min; a.eb_max = c.eb_max;
    a.scratch = ctx->s.ctl; a.result = ctx->s.ctl_result;

    DeviceGuard guard(ctx->device);
    if (!guard.ok) return CMP_E_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    launch_controller(a, &ctx->prof, st);
    ControllerResult res;
    if (hipMemcpyAsync(&res, ctx->s.ctl_result, sizeof(res), hipMemcpyDeviceToHost, st) != hipSuccess) return CMP_E_HIP;
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
