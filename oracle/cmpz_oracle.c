/*
 * cmpz_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, single-threaded, deliberately slow CPU implementation of the
 * error-bounded activation compressor the paper places on its training hot
 * path: Section 2.2 lists the three steps of the SZ family (prediction,
 * error-bounded quantisation of the residual, Huffman coding); Section 3.1
 * gives the GPU variant's order (quantise first, then a Lorenzo predictor,
 * then one integer code per value, then Huffman coding of the codes);
 * Section 4.4 places decompression in the backward pass.
 * The paper names the stages and the absolute-error-bound guarantee and leaves
 * every other detail open; the readings taken here are spelled out stage by
 * stage below (labels C0..C9) so that each can be checked by eye.
 *
 * Only the tests, the smoke check and the CPU-baseline leg of the benchmark may
 * use this file.  It shares no code, header, table or constant generator with
 * the HIP library; the numeric values of the return codes and the container
 * layout are the same by specification, each side writing them out on its own.
 *
 * Pins (tests/test_oracle_*.py): exact-rational check of C0, |x-x'|<=eb in
 * fp64 on adversarial inputs, zero/sign preservation, quantiser fixed point,
 * Lorenzo/prefix-sum identity and closed forms vs numpy cumsum, histogram vs
 * bincount, RFC 1951 canonical-code example, Kraft equality, brute-force
 * optimal cost on tiny alphabets, independent heap Huffman cost, hand-packed
 * bitstreams, header-corruption rejection, hand-computed 1x1x2x2 container;
 * for the zero-block variant: the flags against their definition, a worked
 * example, the same symbols and reconstruction as the plain variant, never
 * more payload bits than the plain variant.
 * The tie-break among equally optimal codebooks (C5) is a convention fixed
 * here: apart from its worked examples it is "parity unpinned".
 *
 * Floating point: IEEE-754 binary32, round-to-nearest-even, no contraction
 * (build with -ffp-contract=off, no fast-math).  The only fp operations are the
 * host constants of C0, x*r, rint, (float)q and q*s.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK          0
#define ORC_E_ARG      (-1)
#define ORC_E_NOSPACE  (-2)
#define ORC_E_FORMAT   (-3)
#define ORC_E_MISMATCH (-4)
#define ORC_E_NOMEM    (-6)
#define ORC_W_RANGE     1

#define ORC_QMAX        16384
#define ORC_HEADER      256
#define ORC_VERSION     1   /* every code is in the bit stream                                   */
#define ORC_VERSION_ZB  2   /* sub-blocks of zero residuals are left out of it (C4', C6' below)  */
#define ORC_MAX_RADIUS  512
#define ORC_MAX_NSYM    (2 * ORC_MAX_RADIUS)

typedef struct {
    uint32_t radius;       /* R: deltas with |d| < R are coded, symbol = d + R   */
    uint32_t chunk;        /* codes per Huffman chunk                            */
    uint32_t sub;          /* codes per sub-block (divides chunk)                */
    uint32_t guard_shift;  /* eb_in = eb - eb * 2^-guard_shift                   */
    uint32_t zero_blocks;  /* 1: leave sub-blocks of zero residuals out (version 2) */
} orc_config;

/* Optional stage dumps; any pointer may be NULL.  Buffers are caller-owned and
 * sized numel (q, delta, sym, outl_*), 2R (cnt, lens, codes). */
typedef struct {
    int32_t  *q;
    int32_t  *delta;
    uint16_t *sym;
    uint32_t *outl_idx;
    int32_t  *outl_val;
    uint32_t *cnt;
    uint8_t  *lens;
    uint64_t *codes;
    uint64_t  n_outliers;
    uint64_t  range_events;
    uint64_t  total_bits;
    uint32_t  max_len;
} orc_stages;

/* ------------------------------------------------------------------ C0 ---- */
/* Quantiser constants, all in fp32: the error bound is tightened by a guard
 * band so that the user's bound holds strictly after the two fp32 roundings
 * (Section 2.2 defines the error-bounded mode: no reconstructed value may
 * differ from the original by more than the bound the user set).  s is the
 * quantisation step, r its reciprocal rounded once. */
int orc_constants(float eb, uint32_t guard_shift, float *eb_in, float *s, float *r)
{
    if (!(eb >= 0x1p-60f && eb <= 0x1p60f)) return ORC_E_ARG;   /* also rejects NaN */
    if (guard_shift < 1 || guard_shift > 23) return ORC_E_ARG;
    volatile float g = ldexpf(eb, -(int)guard_shift);   /* exact                 */
    volatile float e = eb - g;                          /* one fp32 subtraction  */
    volatile float step = 2.0f * e;                     /* exact                 */
    volatile float rec = 1.0f / step;                   /* one fp32 division     */
    *eb_in = e; *s = step; *r = rec;
    return ORC_OK;
}

/* ------------------------------------------------------------------ C1 ---- */
/* Pre-quantisation (Section 3.1, first stage of the GPU compressor):
 * q = round(x / (2 eb_in)) evaluated as one multiply, q = rint(x*r), ties to
 * even, clamped to +-QMAX; NaN maps to 0.  Returns how many elements fell
 * outside the representable range (for those the bound is void). */
uint64_t orc_prequant(const float *x, size_t n, float r, int32_t *q)
{
    uint64_t range_events = 0;
    for (size_t i = 0; i < n; ++i) {
        volatile float t = x[i] * r;
        float tt = t;
        if (!(fabsf(tt) <= (float)ORC_QMAX)) {
            ++range_events;
            tt = isnan(tt) ? 0.0f : copysignf((float)ORC_QMAX, tt);
        }
        q[i] = (int32_t)nearbyintf(tt);       /* FE_TONEAREST: half to even     */
    }
    return range_events;
}

/* ------------------------------------------------------------------ C2 ---- */
/* First-order 2D Lorenzo predictor on the integer codes of every plane
 * (Section 3.1: each point is predicted from its already-seen neighbours);
 * neighbours outside the plane count as 0. */
void orc_lorenzo2d(const int32_t *q, size_t planes, size_t H, size_t W, int32_t *delta)
{
    for (size_t p = 0; p < planes; ++p) {
        const int32_t *qp = q + p * H * W;
        int32_t *dp = delta + p * H * W;
        for (size_t h = 0; h < H; ++h)
            for (size_t w = 0; w < W; ++w) {
                int32_t left = (w > 0) ? qp[h * W + (w - 1)] : 0;
                int32_t up = (h > 0) ? qp[(h - 1) * W + w] : 0;
                int32_t diag = (h > 0 && w > 0) ? qp[(h - 1) * W + (w - 1)] : 0;
                dp[h * W + w] = qp[h * W + w] - left - up + diag;
            }
    }
}

/* ------------------------------------------------------------------ C8b --- */
/* Reverse Lorenzo: q[h,w] is the sum of delta over the rectangle [0..h]x[0..w]
 * of the plane, written out as that double sum (no running totals). Slow:
 * O(H*W) per element; the fast variant below is what the codec uses and the
 * tests check the two against each other and against numpy's cumsum. */
void orc_prefix2d_definition(const int32_t *delta, size_t planes, size_t H, size_t W, int32_t *q)
{
    for (size_t p = 0; p < planes; ++p) {
        const int32_t *dp = delta + p * H * W;
        int32_t *qp = q + p * H * W;
        for (size_t h = 0; h < H; ++h)
            for (size_t w = 0; w < W; ++w) {
                int32_t acc = 0;
                for (size_t i = 0; i <= h; ++i)
                    for (size_t j = 0; j <= w; ++j) acc += dp[i * W + j];
                qp[h * W + w] = acc;
            }
    }
}

/* Same result through the recurrence q[h,w] = d[h,w] + q[h,w-1] + q[h-1,w] -
 * q[h-1,w-1], which is C2 solved for q. */
void orc_prefix2d(const int32_t *delta, size_t planes, size_t H, size_t W, int32_t *q)
{
    for (size_t p = 0; p < planes; ++p) {
        const int32_t *dp = delta + p * H * W;
        int32_t *qp = q + p * H * W;
        for (size_t h = 0; h < H; ++h)
            for (size_t w = 0; w < W; ++w) {
                int32_t left = (w > 0) ? qp[h * W + (w - 1)] : 0;
                int32_t up = (h > 0) ? qp[(h - 1) * W + w] : 0;
                int32_t diag = (h > 0 && w > 0) ? qp[(h - 1) * W + (w - 1)] : 0;
                qp[h * W + w] = dp[h * W + w] + left + up - diag;
            }
    }
}

/* ------------------------------------------------------------------ C3 ---- */
/* Quantisation code / unpredictable-data split (Section 2.2 step (2)):
 * |d| < R gives symbol d+R in [1, 2R-1]; anything else gives symbol 0 and an
 * (index, delta) record, records in ascending index order. */
uint64_t orc_split(const int32_t *delta, size_t n, uint32_t radius, uint16_t *sym,
                   uint32_t *outl_idx, int32_t *outl_val)
{
    uint64_t n_out = 0;
    int32_t R = (int32_t)radius;
    for (size_t i = 0; i < n; ++i) {
        int32_t d = delta[i];
        if (d > -R && d < R) {
            sym[i] = (uint16_t)(d + R);
        } else {
            sym[i] = 0;
            if (outl_idx) outl_idx[n_out] = (uint32_t)i;
            if (outl_val) outl_val[n_out] = d;
            ++n_out;
        }
    }
    return n_out;
}

/* ------------------------------------------------------------------ C4 ---- */
void orc_histogram(const uint16_t *sym, size_t n, uint32_t nsym, uint32_t *cnt)
{
    for (uint32_t k = 0; k < nsym; ++k) cnt[k] = 0;
    for (size_t i = 0; i < n; ++i) cnt[sym[i]] += 1;
}

/* ------------------------------------------------------------ C4', C6' ---- */
/* The sparsity-aware front end (format version 2).  Activation data are
 * dominated by zeros (Section 3.2 treats them apart: they carry no error;
 * Section 4.4 restores them exactly): where a whole sub-block of `sub`
 * consecutive codes holds nothing but the zero residual (symbol R), that fact
 * alone is recorded -- the sub-block's stored bit count is 0, a value no coded
 * sub-block can have, since every codeword has at least one bit -- and its
 * codes take no part in the histogram, the codebook or the bit stream.
 * flags[j] = 1 for every such sub-block j (sub-blocks tile the linear NCHW
 * array from element 0; the last one may be short; one without elements is
 * never flagged). */
void orc_zero_blocks(const uint16_t *sym, size_t n, uint32_t radius, uint32_t sub, uint8_t *flags)
{
    size_t nblocks = (n + sub - 1) / sub;
    for (size_t j = 0; j < nblocks; ++j) {
        size_t a = j * sub, b = a + sub < n ? a + sub : n;
        uint8_t all_zero = 1;
        for (size_t i = a; i < b; ++i) if (sym[i] != radius) all_zero = 0;
        flags[j] = all_zero;
    }
}

/* C4 restricted to the codes that are coded: those outside flagged sub-blocks. */
void orc_histogram_coded(const uint16_t *sym, size_t n, uint32_t nsym, uint32_t sub, const uint8_t *flags,
                         uint32_t *cnt)
{
    for (uint32_t k = 0; k < nsym; ++k) cnt[k] = 0;
    for (size_t i = 0; i < n; ++i) if (!flags[i / sub]) cnt[sym[i]] += 1;
}

/* ------------------------------------------------------------------ C5 ---- */
/* Huffman code lengths by the two-queue construction, with the tie-break fixed:
 * leaves sorted ascending by (count, symbol); on equal weight a leaf is taken
 * before an internal node; internal nodes are taken in creation order.
 * One used symbol gets length 1.  Unused symbols get length 0.
 * Returns the largest length, or a negative code. */
typedef struct { uint64_t w; uint32_t sym; } orc_leaf;

static int orc_leaf_cmp(const void *a, const void *b)
{
    const orc_leaf *x = (const orc_leaf *)a, *y = (const orc_leaf *)b;
    if (x->w != y->w) return x->w < y->w ? -1 : 1;
    if (x->sym != y->sym) return x->sym < y->sym ? -1 : 1;
    return 0;
}

int orc_codebook_lengths(const uint32_t *cnt, uint32_t nsym, uint8_t *lens)
{
    if (nsym == 0 || nsym > 65536) return ORC_E_ARG;
    orc_leaf *leaf = (orc_leaf *)malloc(sizeof(orc_leaf) * nsym);
    /* node ids: 0..n-1 leaves (sorted order), n..2n-2 internal (creation order) */
    uint64_t *weight = (uint64_t *)malloc(sizeof(uint64_t) * 2 * nsym);
    uint32_t *parent = (uint32_t *)malloc(sizeof(uint32_t) * 2 * nsym);
    if (!leaf || !weight || !parent) { free(leaf); free(weight); free(parent); return ORC_E_NOMEM; }

    uint32_t n = 0;
    for (uint32_t k = 0; k < nsym; ++k) {
        lens[k] = 0;
        if (cnt[k] > 0) { leaf[n].w = cnt[k]; leaf[n].sym = k; ++n; }
    }
    int max_len = 0;
    if (n == 1) {
        lens[leaf[0].sym] = 1;
        max_len = 1;
    } else if (n >= 2) {
        qsort(leaf, n, sizeof(orc_leaf), orc_leaf_cmp);
        for (uint32_t i = 0; i < n; ++i) weight[i] = leaf[i].w;
        uint32_t q1 = 0;          /* head of the leaf queue                     */
        uint32_t q2 = n;          /* head of the internal-node queue            */
        uint32_t next = n;        /* id of the next internal node to create     */
        while (next < 2 * n - 1) {
            uint32_t pick[2];
            for (int t = 0; t < 2; ++t) {
                int have_leaf = q1 < n, have_int = q2 < next;
                if (have_leaf && (!have_int || weight[q1] <= weight[q2])) pick[t] = q1++;
                else pick[t] = q2++;
            }
            weight[next] = weight[pick[0]] + weight[pick[1]];
            parent[pick[0]] = next;
            parent[pick[1]] = next;
            ++next;
        }
        uint32_t root = 2 * n - 2;
        for (uint32_t i = 0; i < n; ++i) {
            int depth = 0;
            for (uint32_t v = i; v != root; v = parent[v]) ++depth;
            lens[leaf[i].sym] = (uint8_t)depth;
            if (depth > max_len) max_len = depth;
        }
    }
    free(leaf); free(weight); free(parent);
    return max_len;
}

/* Canonical code assignment: used symbols ordered by (length, symbol); the
 * first code is 0; each next code is (previous + 1) shifted left by the growth
 * in length.  Codewords are read most-significant bit first.  This is the
 * assignment of RFC 1951 section 3.2.2. */
int orc_canonical_codes(const uint8_t *lens, uint32_t nsym, uint64_t *codes)
{
    uint64_t code = 0;
    int prev_len = 0, first = 1;
    for (uint32_t k = 0; k < nsym; ++k) codes[k] = 0;
    for (int L = 1; L <= 63; ++L)
        for (uint32_t k = 0; k < nsym; ++k) {
            if (lens[k] != L) continue;
            if (first) { code = 0; first = 0; }
            else code = (code + 1) << (L - prev_len);
            prev_len = L;
            if (L < 64 && (code >> L) != 0) return ORC_E_FORMAT;   /* over-subscribed */
            codes[k] = code;
        }
    for (uint32_t k = 0; k < nsym; ++k) if (lens[k] > 63) return ORC_E_FORMAT;
    return ORC_OK;
}

/* ---------------------------------------------------------- container ---- */
static size_t align16(size_t v) { return (v + 15) & ~(size_t)15; }

static void put_u32(uint8_t *p, uint32_t v)
{ p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); p[2] = (uint8_t)(v >> 16); p[3] = (uint8_t)(v >> 24); }
static void put_u64(uint8_t *p, uint64_t v) { put_u32(p, (uint32_t)v); put_u32(p + 4, (uint32_t)(v >> 32)); }
static void put_u16(uint8_t *p, uint16_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
static uint32_t get_u32(const uint8_t *p)
{ return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24); }
static uint64_t get_u64(const uint8_t *p) { return (uint64_t)get_u32(p) | ((uint64_t)get_u32(p + 4) << 32); }
static uint16_t get_u16(const uint8_t *p) { return (uint16_t)(p[0] | (p[1] << 8)); }

/* header field offsets (bytes) */
enum {
    H_MAGIC = 0, H_VERSION = 4, H_STATUS = 8, H_EB_BITS = 12, H_SHAPE = 16, H_NUMEL = 32,
    H_RADIUS = 40, H_CHUNK = 44, H_SUB = 48, H_GUARD = 52, H_NCHUNKS = 56, H_NOUTL = 60,
    H_RANGE = 64, H_MAXLEN = 68, H_TOTAL_BITS = 72, H_OFF_LENS = 80, H_OFF_CHUNK_OFF = 88,
    H_OFF_OUTL_OFF = 96, H_OFF_SUB_BITS = 104, H_OFF_PAYLOAD = 112, H_OFF_OUTL_IDX = 120,
    H_OFF_OUTL_VAL = 128, H_TOTAL_SIZE = 136
};

static int check_config(const orc_config *cfg)
{
    if (!cfg) return ORC_E_ARG;
    if (cfg->radius < 1 || cfg->radius > ORC_MAX_RADIUS) return ORC_E_ARG;
    if (cfg->sub < 1 || cfg->sub > 1024) return ORC_E_ARG;
    if (cfg->chunk < cfg->sub || cfg->chunk % cfg->sub != 0 || cfg->chunk > (1u << 20)) return ORC_E_ARG;
    if (cfg->guard_shift < 1 || cfg->guard_shift > 23) return ORC_E_ARG;
    if (cfg->zero_blocks > 1) return ORC_E_ARG;
    return ORC_OK;
}

static int check_shape(const int64_t shape[4], uint64_t *numel)
{
    if (!shape) return ORC_E_ARG;
    uint64_t n = 1;
    for (int i = 0; i < 4; ++i) {
        if (shape[i] < 0 || shape[i] > 0xffffffffLL) return ORC_E_ARG;
        n *= (uint64_t)shape[i];
        if (n >= (1ull << 32)) return ORC_E_ARG;
    }
    *numel = n;
    return ORC_OK;
}

/* Sizes of the sections whose length depends only on shape and config. */
static void fixed_layout(uint64_t numel, const orc_config *cfg, uint32_t *nchunks,
                         size_t *off_lens, size_t *off_chunk_off, size_t *off_outl_off,
                         size_t *off_sub_bits, size_t *off_payload)
{
    uint32_t nc = (uint32_t)((numel + cfg->chunk - 1) / cfg->chunk);
    uint32_t nsub = cfg->chunk / cfg->sub;
    *nchunks = nc;
    *off_lens = ORC_HEADER;
    *off_chunk_off = *off_lens + align16(2 * (size_t)cfg->radius);
    *off_outl_off = *off_chunk_off + align16(4 * ((size_t)nc + 1));
    *off_sub_bits = *off_outl_off + align16(4 * ((size_t)nc + 1));
    *off_payload = *off_sub_bits + align16(2 * (size_t)nc * nsub);
}

/* Worst-case container size: a Huffman code never spends more bits than the
 * fixed-length code of ceil(log2(2R)) bits per symbol; every chunk may be
 * padded by up to 15 bytes; every element may be an outlier (8 bytes). */
size_t orc_bound(const int64_t shape[4], const orc_config *cfg)
{
    uint64_t numel;
    if (check_config(cfg) != ORC_OK || check_shape(shape, &numel) != ORC_OK) return 0;
    uint32_t nchunks; size_t o1, o2, o3, o4, o5;
    fixed_layout(numel, cfg, &nchunks, &o1, &o2, &o3, &o4, &o5);
    uint32_t flat = 1;
    while ((1u << flat) < 2 * cfg->radius) ++flat;
    size_t payload = (size_t)((numel * flat + 7) / 8) + 16 * (size_t)nchunks;
    return o5 + align16(payload) + 2 * align16(4 * (size_t)numel);
}

/* ------------------------------------------------------------- C6, C7 ---- */
/* Append the low `len` bits of `code`, most significant first, at bit position
 * *pos of a chunk stream whose bit k lives in little-endian 32-bit word k/32 at
 * bit 31-(k%32). */
static void put_bits(uint8_t *stream, uint64_t *pos, uint64_t code, int len)
{
    for (int b = len - 1; b >= 0; --b) {
        uint64_t k = *pos;
        if ((code >> b) & 1) {
            size_t word = (size_t)(k / 32);
            int bit = 31 - (int)(k % 32);
            stream[word * 4 + (size_t)(bit / 8)] |= (uint8_t)(1u << (bit % 8));
        }
        *pos = k + 1;
    }
}

static int get_bit(const uint8_t *stream, uint64_t k)
{
    size_t word = (size_t)(k / 32);
    int bit = 31 - (int)(k % 32);
    return (stream[word * 4 + (size_t)(bit / 8)] >> (bit % 8)) & 1;
}

int orc_compress(const float *x, const int64_t shape[4], float eb, const orc_config *cfg,
                 uint8_t *out, size_t cap, size_t *size, orc_stages *dump)
{
    uint64_t numel;
    float eb_in, s, r;
    int rc;
    if ((rc = check_config(cfg)) != ORC_OK) return rc;
    if ((rc = check_shape(shape, &numel)) != ORC_OK) return rc;
    if ((rc = orc_constants(eb, cfg->guard_shift, &eb_in, &s, &r)) != ORC_OK) return rc;
    if (!out || !size || (numel > 0 && !x)) return ORC_E_ARG;

    const uint32_t R = cfg->radius, nsym = 2 * R;
    const size_t planes = (size_t)shape[0] * (size_t)shape[1];
    const size_t H = (size_t)shape[2], W = (size_t)shape[3];
    const size_t n = (size_t)numel;

    int32_t *q = (int32_t *)malloc(sizeof(int32_t) * (n + 1));
    int32_t *delta = (int32_t *)malloc(sizeof(int32_t) * (n + 1));
    uint16_t *sym = (uint16_t *)malloc(sizeof(uint16_t) * (n + 1));
    uint32_t *oidx = (uint32_t *)malloc(sizeof(uint32_t) * (n + 1));
    int32_t *oval = (int32_t *)malloc(sizeof(int32_t) * (n + 1));
    uint8_t *zflag = (uint8_t *)calloc(n / cfg->sub + 2, 1);   /* all 0 unless cfg->zero_blocks */
    uint32_t cnt[ORC_MAX_NSYM];
    uint8_t lens[ORC_MAX_NSYM];
    uint64_t codes[ORC_MAX_NSYM];
    if (!q || !delta || !sym || !oidx || !oval || !zflag) { rc = ORC_E_NOMEM; goto done; }

    /* C1..C5 */
    uint64_t range_events = orc_prequant(x, n, r, q);
    orc_lorenzo2d(q, planes, H, W, delta);
    uint64_t n_out = orc_split(delta, n, R, sym, oidx, oval);
    if (cfg->zero_blocks) {
        orc_zero_blocks(sym, n, R, cfg->sub, zflag);
        orc_histogram_coded(sym, n, nsym, cfg->sub, zflag, cnt);
    } else {
        orc_histogram(sym, n, nsym, cnt);
    }
    int max_len = orc_codebook_lengths(cnt, nsym, lens);
    if (max_len < 0) { rc = max_len; goto done; }
    if ((rc = orc_canonical_codes(lens, nsym, codes)) != ORC_OK) goto done;

    /* C6: sizes */
    uint32_t nchunks; size_t off_lens, off_chunk_off, off_outl_off, off_sub_bits, off_payload;
    fixed_layout(numel, cfg, &nchunks, &off_lens, &off_chunk_off, &off_outl_off, &off_sub_bits,
                 &off_payload);
    const uint32_t nsub = cfg->chunk / cfg->sub;
    uint64_t total_bits = 0, payload_units = 0;
    for (uint32_t c = 0; c < nchunks; ++c) {
        size_t lo = (size_t)c * cfg->chunk, hi = lo + cfg->chunk < n ? lo + cfg->chunk : n;
        uint64_t bits = 0;
        for (size_t i = lo; i < hi; ++i) if (!zflag[i / cfg->sub]) bits += lens[sym[i]];
        total_bits += bits;
        payload_units += (bits + 127) / 128;
    }
    if (payload_units >= (1ull << 32)) { rc = ORC_E_ARG; goto done; }
    size_t off_outl_idx = off_payload + (size_t)payload_units * 16;
    size_t off_outl_val = off_outl_idx + align16(4 * (size_t)n_out);
    size_t total = off_outl_val + align16(4 * (size_t)n_out);

    if (dump) {
        if (dump->q) memcpy(dump->q, q, sizeof(int32_t) * n);
        if (dump->delta) memcpy(dump->delta, delta, sizeof(int32_t) * n);
        if (dump->sym) memcpy(dump->sym, sym, sizeof(uint16_t) * n);
        if (dump->outl_idx) memcpy(dump->outl_idx, oidx, sizeof(uint32_t) * (size_t)n_out);
        if (dump->outl_val) memcpy(dump->outl_val, oval, sizeof(int32_t) * (size_t)n_out);
        if (dump->cnt) memcpy(dump->cnt, cnt, sizeof(uint32_t) * nsym);
        if (dump->lens) memcpy(dump->lens, lens, nsym);
        if (dump->codes) memcpy(dump->codes, codes, sizeof(uint64_t) * nsym);
        dump->n_outliers = n_out; dump->range_events = range_events;
        dump->total_bits = total_bits; dump->max_len = (uint32_t)max_len;
    }

    *size = total;
    if (total > cap) { rc = ORC_E_NOSPACE; goto done; }

    /* C7: write the container; everything not written below stays zero */
    memset(out, 0, total);
    memcpy(out + H_MAGIC, "CMPZ", 4);
    put_u32(out + H_VERSION, cfg->zero_blocks ? ORC_VERSION_ZB : ORC_VERSION);
    put_u32(out + H_STATUS, 0);
    { uint32_t ebits; memcpy(&ebits, &eb, 4); put_u32(out + H_EB_BITS, ebits); }
    for (int i = 0; i < 4; ++i) put_u32(out + H_SHAPE + 4 * i, (uint32_t)shape[i]);
    put_u64(out + H_NUMEL, numel);
    put_u32(out + H_RADIUS, cfg->radius);
    put_u32(out + H_CHUNK, cfg->chunk);
    put_u32(out + H_SUB, cfg->sub);
    put_u32(out + H_GUARD, cfg->guard_shift);
    put_u32(out + H_NCHUNKS, nchunks);
    put_u32(out + H_NOUTL, (uint32_t)n_out);
    put_u32(out + H_RANGE, (uint32_t)range_events);
    put_u32(out + H_MAXLEN, (uint32_t)max_len);
    put_u64(out + H_TOTAL_BITS, total_bits);
    put_u64(out + H_OFF_LENS, off_lens);
    put_u64(out + H_OFF_CHUNK_OFF, off_chunk_off);
    put_u64(out + H_OFF_OUTL_OFF, off_outl_off);
    put_u64(out + H_OFF_SUB_BITS, off_sub_bits);
    put_u64(out + H_OFF_PAYLOAD, off_payload);
    put_u64(out + H_OFF_OUTL_IDX, off_outl_idx);
    put_u64(out + H_OFF_OUTL_VAL, off_outl_val);
    put_u64(out + H_TOTAL_SIZE, total);

    memcpy(out + off_lens, lens, nsym);

    {
        uint64_t unit = 0;          /* running payload offset in 16-byte units   */
        size_t next_outlier = 0;    /* outliers with index below the chunk start */
        for (uint32_t c = 0; c < nchunks; ++c) {
            size_t lo = (size_t)c * cfg->chunk, hi = lo + cfg->chunk < n ? lo + cfg->chunk : n;
            put_u32(out + off_chunk_off + 4 * (size_t)c, (uint32_t)unit);
            while (next_outlier < n_out && oidx[next_outlier] < lo) ++next_outlier;
            put_u32(out + off_outl_off + 4 * (size_t)c, (uint32_t)next_outlier);
            uint8_t *stream = out + off_payload + (size_t)unit * 16;
            uint64_t pos = 0;
            for (uint32_t j = 0; j < nsub; ++j) {
                size_t a = lo + (size_t)j * cfg->sub, b = a + cfg->sub;
                if (a > hi) a = hi;
                if (b > hi) b = hi;
                uint64_t before = pos;
                for (size_t i = a; i < b; ++i)
                    if (!zflag[i / cfg->sub]) put_bits(stream, &pos, codes[sym[i]], lens[sym[i]]);
                put_u16(out + off_sub_bits + 2 * ((size_t)c * nsub + j), (uint16_t)(pos - before));
            }
            unit += (pos + 127) / 128;
        }
        put_u32(out + off_chunk_off + 4 * (size_t)nchunks, (uint32_t)unit);
        put_u32(out + off_outl_off + 4 * (size_t)nchunks, (uint32_t)n_out);
    }
    for (size_t k = 0; k < n_out; ++k) {
        put_u32(out + off_outl_idx + 4 * k, oidx[k]);
        put_u32(out + off_outl_val + 4 * k, (uint32_t)oval[k]);
    }
    rc = range_events ? ORC_W_RANGE : ORC_OK;

done:
    free(q); free(delta); free(sym); free(oidx); free(oval); free(zflag);
    return rc;
}

/* ------------------------------------------------------------- C8, C9 ---- */
/* Decode the symbol stream of a container into sym[0..numel). The canonical
 * code is rebuilt from the stored lengths; each sub-block is entered at the bit
 * position given by the sum of the preceding sub_bits of its chunk and decoded
 * one bit at a time (textbook canonical decoding: at length L a code below
 * first[L]+count[L] ends a codeword). */
static int decode_symbols(const uint8_t *buf, size_t n, const orc_config *cfg, uint32_t nchunks,
                          size_t off_lens, size_t off_chunk_off, size_t off_sub_bits,
                          size_t off_payload, uint64_t payload_units, uint16_t *sym,
                          uint64_t *total_bits_seen)
{
    const uint32_t nsym = 2 * cfg->radius, nsub = cfg->chunk / cfg->sub;
    const uint8_t *lens = buf + off_lens;
    uint64_t codes[ORC_MAX_NSYM];
    uint32_t count[64], offset[65];
    uint64_t first[64];
    uint16_t sorted[ORC_MAX_NSYM];
    int rc = orc_canonical_codes(lens, nsym, codes);
    if (rc != ORC_OK) return rc;
    for (int L = 0; L < 64; ++L) { count[L] = 0; first[L] = 0; }
    for (uint32_t k = 0; k < nsym; ++k) count[lens[k]] += 1;
    count[0] = 0;
    offset[0] = 0;
    for (int L = 0; L < 64; ++L) offset[L + 1] = offset[L] + count[L];
    {
        uint32_t fill[64];
        for (int L = 0; L < 64; ++L) fill[L] = 0;
        for (uint32_t k = 0; k < nsym; ++k) {
            int L = lens[k];
            if (L == 0) continue;
            if (fill[L] == 0) first[L] = codes[k];      /* smallest symbol of this length */
            sorted[offset[L] + fill[L]] = (uint16_t)k;
            fill[L] += 1;
        }
    }
    uint64_t seen = 0;
    for (uint32_t c = 0; c < nchunks; ++c) {
        uint64_t u0 = get_u32(buf + off_chunk_off + 4 * (size_t)c);
        uint64_t u1 = get_u32(buf + off_chunk_off + 4 * (size_t)(c + 1));
        if (u0 > u1 || u1 > payload_units) return ORC_E_FORMAT;
        const uint8_t *stream = buf + off_payload + (size_t)u0 * 16;
        uint64_t chunk_bits = (u1 - u0) * 128;
        size_t lo = (size_t)c * cfg->chunk, hi = lo + cfg->chunk < n ? lo + cfg->chunk : n;
        uint64_t start = 0;
        for (uint32_t j = 0; j < nsub; ++j) {
            size_t a = lo + (size_t)j * cfg->sub, b = a + cfg->sub;
            if (a > hi) a = hi;
            if (b > hi) b = hi;
            uint64_t sb = get_u16(buf + off_sub_bits + 2 * ((size_t)c * nsub + j));
            if (start + sb > chunk_bits) return ORC_E_FORMAT;
            if (cfg->zero_blocks && sb == 0 && a < b) {       /* C6': nothing but zero residuals */
                for (size_t i = a; i < b; ++i) sym[i] = (uint16_t)cfg->radius;
                continue;
            }
            uint64_t pos = start;
            for (size_t i = a; i < b; ++i) {
                uint64_t code = 0;
                int L = 0, found = 0;
                while (L < 63 && pos < start + sb) {
                    code = (code << 1) | (uint64_t)get_bit(stream, pos);
                    ++pos; ++L;
                    if (count[L] && code >= first[L] && code - first[L] < count[L]) {
                        sym[i] = sorted[offset[L] + (uint32_t)(code - first[L])];
                        found = 1;
                        break;
                    }
                }
                if (!found) return ORC_E_FORMAT;
            }
            if (pos != start + sb) return ORC_E_FORMAT;
            start += sb;
            seen += sb;
        }
        if ((start + 127) / 128 != u1 - u0) return ORC_E_FORMAT;
    }
    *total_bits_seen = seen;
    return ORC_OK;
}

int orc_decompress(const uint8_t *buf, size_t size, const int64_t shape[4], float eb,
                   const orc_config *cfg, float *xout)
{
    uint64_t numel;
    float eb_in, s, r;
    int rc;
    if ((rc = check_config(cfg)) != ORC_OK) return rc;
    if ((rc = check_shape(shape, &numel)) != ORC_OK) return rc;
    if ((rc = orc_constants(eb, cfg->guard_shift, &eb_in, &s, &r)) != ORC_OK) return rc;
    if (!buf || (numel > 0 && !xout)) return ORC_E_ARG;

    /* header: format first, then agreement with the caller's arguments */
    if (size < ORC_HEADER) return ORC_E_FORMAT;
    if (memcmp(buf + H_MAGIC, "CMPZ", 4) != 0) return ORC_E_FORMAT;
    if (get_u32(buf + H_VERSION) != ORC_VERSION && get_u32(buf + H_VERSION) != ORC_VERSION_ZB) return ORC_E_FORMAT;
    if (get_u32(buf + H_STATUS) != 0) return ORC_E_FORMAT;
    for (size_t i = H_TOTAL_SIZE + 8; i < ORC_HEADER; ++i) if (buf[i] != 0) return ORC_E_FORMAT;
    { uint32_t ebits; memcpy(&ebits, &eb, 4); if (get_u32(buf + H_EB_BITS) != ebits) return ORC_E_MISMATCH; }
    for (int i = 0; i < 4; ++i)
        if (get_u32(buf + H_SHAPE + 4 * i) != (uint32_t)shape[i]) return ORC_E_MISMATCH;
    if (get_u32(buf + H_RADIUS) != cfg->radius || get_u32(buf + H_CHUNK) != cfg->chunk ||
        get_u32(buf + H_SUB) != cfg->sub || get_u32(buf + H_GUARD) != cfg->guard_shift ||
        get_u32(buf + H_VERSION) != (cfg->zero_blocks ? ORC_VERSION_ZB : ORC_VERSION))
        return ORC_E_MISMATCH;
    if (get_u64(buf + H_NUMEL) != numel) return ORC_E_FORMAT;

    uint32_t nchunks; size_t off_lens, off_chunk_off, off_outl_off, off_sub_bits, off_payload;
    fixed_layout(numel, cfg, &nchunks, &off_lens, &off_chunk_off, &off_outl_off, &off_sub_bits,
                 &off_payload);
    if (get_u32(buf + H_NCHUNKS) != nchunks) return ORC_E_FORMAT;
    if (get_u64(buf + H_OFF_LENS) != off_lens || get_u64(buf + H_OFF_CHUNK_OFF) != off_chunk_off ||
        get_u64(buf + H_OFF_OUTL_OFF) != off_outl_off || get_u64(buf + H_OFF_SUB_BITS) != off_sub_bits ||
        get_u64(buf + H_OFF_PAYLOAD) != off_payload)
        return ORC_E_FORMAT;
    uint64_t n_out = get_u32(buf + H_NOUTL);
    uint64_t off_outl_idx = get_u64(buf + H_OFF_OUTL_IDX);
    uint64_t off_outl_val = get_u64(buf + H_OFF_OUTL_VAL);
    uint64_t total = get_u64(buf + H_TOTAL_SIZE);
    if (total > size) return ORC_E_FORMAT;
    if (n_out > numel) return ORC_E_FORMAT;
    if (off_outl_idx < off_payload || (off_outl_idx - off_payload) % 16 != 0) return ORC_E_FORMAT;
    if (off_outl_val != off_outl_idx + align16(4 * (size_t)n_out)) return ORC_E_FORMAT;
    if (total != off_outl_val + align16(4 * (size_t)n_out)) return ORC_E_FORMAT;
    uint64_t payload_units = (off_outl_idx - off_payload) / 16;
    if (payload_units >= (1ull << 32)) return ORC_E_FORMAT;
    if (get_u32(buf + H_RANGE) > numel) return ORC_E_FORMAT;

    const uint32_t R = cfg->radius, nsym = 2 * R;
    {   /* stored lengths must form a complete prefix code (or the 0/1-symbol cases);
         * the Kraft sum is taken in integers, in units of 2^-63 */
        const uint8_t *lens = buf + off_lens;
        uint32_t used = 0, mx = 0;
        uint64_t kraft = 0;
        const uint64_t one = 1ull << 63;
        for (uint32_t k = 0; k < nsym; ++k) {
            if (lens[k] > 63) return ORC_E_FORMAT;
            if (lens[k]) {
                ++used;
                kraft += 1ull << (63 - lens[k]);
                if (kraft > one) return ORC_E_FORMAT;
                if (lens[k] > mx) mx = lens[k];
            }
        }
        if (used >= 2 && kraft != one) return ORC_E_FORMAT;
        if (used == 1 && mx != 1) return ORC_E_FORMAT;
        /* no codeword at all: an empty tensor, or (version 2) nothing but flagged sub-blocks */
        if (used == 0 && numel != 0 && !(cfg->zero_blocks && get_u64(buf + H_TOTAL_BITS) == 0)) return ORC_E_FORMAT;
        if (get_u32(buf + H_MAXLEN) != mx) return ORC_E_FORMAT;
        for (size_t i = off_lens + nsym; i < off_chunk_off; ++i) if (buf[i] != 0) return ORC_E_FORMAT;
    }
    if (get_u32(buf + off_chunk_off) != 0) return ORC_E_FORMAT;
    if (get_u32(buf + off_chunk_off + 4 * (size_t)nchunks) != payload_units) return ORC_E_FORMAT;
    if (get_u32(buf + off_outl_off) != 0) return ORC_E_FORMAT;
    if (get_u32(buf + off_outl_off + 4 * (size_t)nchunks) != n_out) return ORC_E_FORMAT;

    const size_t n = (size_t)numel;
    const size_t planes = (size_t)shape[0] * (size_t)shape[1];
    const size_t H = (size_t)shape[2], W = (size_t)shape[3];
    uint16_t *sym = (uint16_t *)malloc(sizeof(uint16_t) * (n + 1));
    int32_t *delta = (int32_t *)malloc(sizeof(int32_t) * (n + 1));
    int32_t *q = (int32_t *)malloc(sizeof(int32_t) * (n + 1));
    if (!sym || !delta || !q) { rc = ORC_E_NOMEM; goto done; }

    /* C8: symbols -> deltas, then outliers overwrite their positions */
    uint64_t bits_seen = 0;
    rc = decode_symbols(buf, n, cfg, nchunks, off_lens, off_chunk_off, off_sub_bits, off_payload,
                        payload_units, sym, &bits_seen);
    if (rc != ORC_OK) goto done;
    if (bits_seen != get_u64(buf + H_TOTAL_BITS)) { rc = ORC_E_FORMAT; goto done; }
    for (size_t i = 0; i < n; ++i) delta[i] = (int32_t)sym[i] - (int32_t)R;
    {
        uint64_t prev = 0;
        for (uint64_t k = 0; k < n_out; ++k) {
            uint32_t idx = get_u32(buf + off_outl_idx + 4 * (size_t)k);
            if (idx >= numel || (k > 0 && idx <= prev) || sym[idx] != 0) { rc = ORC_E_FORMAT; goto done; }
            delta[idx] = (int32_t)get_u32(buf + off_outl_val + 4 * (size_t)k);
            prev = idx;
        }
        /* every symbol 0 must have its record, and outl_off[c] must count the
         * records that lie below chunk c */
        uint64_t zeros = 0;
        for (uint32_t c = 0; c < nchunks; ++c) {
            if (get_u32(buf + off_outl_off + 4 * (size_t)c) != zeros) { rc = ORC_E_FORMAT; goto done; }
            size_t lo = (size_t)c * cfg->chunk, hi = lo + cfg->chunk < n ? lo + cfg->chunk : n;
            for (size_t i = lo; i < hi; ++i) if (sym[i] == 0) ++zeros;
        }
        if (zeros != n_out) { rc = ORC_E_FORMAT; goto done; }
    }
    /* reverse Lorenzo: per-plane 2D inclusive prefix sum of the deltas */
    orc_prefix2d(delta, planes, H, W, q);
    /* C9: de-quantise, one fp32 multiply; q == 0 gives +0.0f */
    for (size_t i = 0; i < n; ++i) {
        volatile float v = (float)q[i] * s;
        xout[i] = (q[i] == 0) ? 0.0f : v;
    }
    rc = ORC_OK;
done:
    free(sym); free(delta); free(q);
    return rc;
}

/* Decode only the symbols and outlier-patched deltas of a container (used by
 * the parity tests to look inside a container produced elsewhere). */
int orc_decode_deltas(const uint8_t *buf, size_t size, const orc_config *cfg, uint16_t *sym_out,
                      int32_t *delta_out)
{
    if (!buf || size < ORC_HEADER || check_config(cfg) != ORC_OK) return ORC_E_ARG;
    uint64_t numel = get_u64(buf + H_NUMEL);
    uint32_t nchunks; size_t o1, o2, o3, o4, o5;
    fixed_layout(numel, cfg, &nchunks, &o1, &o2, &o3, &o4, &o5);
    uint64_t off_outl_idx = get_u64(buf + H_OFF_OUTL_IDX), off_outl_val = get_u64(buf + H_OFF_OUTL_VAL);
    uint64_t n_out = get_u32(buf + H_NOUTL);
    if (get_u64(buf + H_TOTAL_SIZE) > size || off_outl_idx < o5) return ORC_E_FORMAT;
    uint64_t bits = 0;
    int rc = decode_symbols(buf, (size_t)numel, cfg, nchunks, o1, o2, o4, o5, (off_outl_idx - o5) / 16,
                            sym_out, &bits);
    if (rc != ORC_OK) return rc;
    if (delta_out) {
        for (size_t i = 0; i < (size_t)numel; ++i) delta_out[i] = (int32_t)sym_out[i] - (int32_t)cfg->radius;
        for (uint64_t k = 0; k < n_out; ++k) {
            uint32_t idx = get_u32(buf + off_outl_idx + 4 * (size_t)k);
            if (idx >= numel) return ORC_E_FORMAT;
            delta_out[idx] = (int32_t)get_u32(buf + off_outl_val + 4 * (size_t)k);
        }
    }
    return ORC_OK;
}

/* De-quantise alone (C9), exposed for the stage-level pins. */
void orc_dequant(const int32_t *q, size_t n, float s, float *xout)
{
    for (size_t i = 0; i < n; ++i) {
        volatile float v = (float)q[i] * s;
        xout[i] = (q[i] == 0) ? 0.0f : v;
    }
}

/* ------------------------------------------------------------------------
 * Error-bound estimator of the adaptive framework (Sections 4.1-4.3).
 *
 * Collected every W iterations (Section 4.1):
 *   R      fraction of non-zero elements of the activation tensor (Eq. 9: the
 *          predicted sigma shrinks by sqrt(R) because zeros carry no error);
 *   Lbar   "average value of the current layer's loss" (Eq. 5).  Reading taken
 *          here: the loss arrives as batch_n samples of per_sample values each;
 *          Lbar is the mean over the samples of each sample's largest |value|;
 *   Mavg   "average value of the momentum" (Eq. 7).  Reading: mean of |m|.
 * Then (Eq. 7, Eq. 8 with the sqrt(R) of Eq. 9, a = 0.32 in Section 5.1):
 *   sigma = sigma_frac * Mavg,   eb = sigma / (a * Lbar * sqrt(batch_n * R)).
 * All arithmetic in fp64; the result is rounded once to fp32 and clamped to
 * [eb_min, eb_max].  When the denominator is not a positive finite number
 * (all-zero activation, zero loss, NaN anywhere) or Mavg is not finite, the
 * tightest bound eb_min is returned together with ORC_W_RANGE.
 * stats[0..2] = R, Lbar, Mavg.
 *
 * Pins (tests/test_oracle_controller.py): exact closed forms (all parameters
 * powers of two), the sqrt(2) law of Section 3.2 for a doubled batch, the
 * sqrt(R) law of Eq. 9, independent numpy statistics, clamping and the
 * degenerate cases.  The two readings above (Lbar, Mavg) are conventions:
 * apart from those pins they are "parity unpinned".
 * ------------------------------------------------------------------------ */
typedef struct {
    float sigma_frac;   /* 0.01 in the paper */
    float a;            /* 0.32 in the paper */
    float eb_min, eb_max;
} orc_controller_config;

int orc_estimate_eb(const float *act, size_t act_numel, const float *loss, size_t batch_n, size_t per_sample,
                    const float *mom, size_t mom_numel, const orc_controller_config *cfg, float *eb_out,
                    double stats[3])
{
    if (!cfg || !eb_out || !act || !loss || !mom) return ORC_E_ARG;
    if (act_numel == 0 || batch_n == 0 || per_sample == 0 || mom_numel == 0) return ORC_E_ARG;
    if (!(cfg->eb_min > 0.0f) || !(cfg->eb_max >= cfg->eb_min) || !(cfg->sigma_frac > 0.0f) || !(cfg->a > 0.0f))
        return ORC_E_ARG;

    size_t nonzero = 0;
    for (size_t i = 0; i < act_numel; ++i) nonzero += (act[i] != 0.0f) ? 1u : 0u;      /* NaN counts as non-zero */
    const double R = (double)nonzero / (double)act_numel;

    double lsum = 0.0;
    for (size_t n = 0; n < batch_n; ++n) {
        double m = 0.0;
        int nan_seen = 0;
        for (size_t k = 0; k < per_sample; ++k) {
            const double v = fabs((double)loss[n * per_sample + k]);
            if (isnan(v)) nan_seen = 1;
            else if (v > m) m = v;
        }
        lsum += nan_seen ? (double)NAN : m;                         /* a NaN anywhere in the sample sticks */
    }
    const double Lbar = lsum / (double)batch_n;

    double msum = 0.0;
    for (size_t i = 0; i < mom_numel; ++i) msum += fabs((double)mom[i]);
    const double Mavg = msum / (double)mom_numel;

    if (stats) { stats[0] = R; stats[1] = Lbar; stats[2] = Mavg; }
    const double sigma = (double)cfg->sigma_frac * Mavg;
    const double denom = (double)cfg->a * Lbar * sqrt((double)batch_n * R);
    if (!(denom > 0.0) || !isfinite(denom) || !isfinite(sigma)) { *eb_out = cfg->eb_min; return ORC_W_RANGE; }
    float eb = (float)(sigma / denom);
    if (!(eb >= cfg->eb_min)) eb = cfg->eb_min;
    if (eb > cfg->eb_max) eb = cfg->eb_max;
    *eb_out = eb;
    return ORC_OK;
}

