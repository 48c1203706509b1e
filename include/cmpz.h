/*
 * cmpz.h -- C ABI of the MI355X activation compressor.
 *
 * The library implements, as HIP kernels for gfx950, the compressor the paper
 * runs on every convolutional layer's activation tensor in the forward pass and
 * the decompressor it runs when the backward pass reaches that layer
 * (Section 4.4; data flow of Section 2.1): an SZ-type error-bounded lossy codec
 * in absolute-error-bound mode (Section 2.2) whose stages are, in the order of
 * Section 3.1, pre-quantisation of each fp32 value to an integer, a Lorenzo
 * predictor on the integers, one quantisation code per value (with out-of-range
 * residuals kept verbatim), and Huffman coding of the codes.
 *
 * Conventions
 *  - "d_" pointers are DEVICE pointers on the context's GPU, "h_" pointers are
 *    HOST pointers.  `stream` is a hipStream_t passed as void* (NULL = the
 *    default stream).  No HIP or torch type appears in this interface.
 *  - The caller owns every buffer it passes.  The context owns only its scratch
 *    memory, allocated once in cmp_create and sized by cfg.max_numel; compress
 *    and decompress allocate nothing and do not synchronise unless stated.
 *  - All work of one context must be issued on one stream at a time; calls on
 *    one context are not re-entrant.  Use one context per concurrent stream.
 *  - Tensors are fp32, contiguous NCHW; d_x, d_xout and d_out must be 16-byte
 *    aligned.  numel must not exceed 2^32 - 8192.  A dimension may be 0 (empty tensor).
 *  - Return value: 0 = CMP_OK, negative = error, positive = warning.
 *    Conditions only the GPU can see (container too small, malformed container,
 *    out-of-range input) are recorded on the device and reported by the next
 *    synchronising call (cmp_compress with h_size != NULL, cmp_compressed_size,
 *    cmp_last_status).  The library never aborts and never prints.
 *  - Same input bytes, error bound and configuration give the same container
 *    bytes on every run.
 *
 * Arithmetic (all fp32, IEEE round-to-nearest-even, no fused multiply-add):
 *    eb_in = eb - eb * 2^-guard_shift;  s = 2 * eb_in;  r = 1 / s   (host)
 *    q  = rint(x * r) clamped to [-16384, 16384], NaN -> 0           (compress)
 *    x' = (float)q * s                                               (decompress)
 * so that |x - x'| <= eb for every element whose |x * r| <= 16384.
 *
 * Container (little-endian; every section 16-byte aligned; padding bytes zero):
 *    header, 256 bytes: +0 "CMPZ", +4 version u32 (1; 2 with CMP_F_ZERO_BLOCKS), +8 status u32 (0 = complete,
 *      2 = did not fit), +12 eb bits u32, +16 shape u32[4], +32 numel u64,
 *      +40 radius, +44 chunk, +48 sub, +52 guard_shift, +56 nchunks, +60 n_outliers,
 *      +64 range_events, +68 max_len (all u32), +72 total_bits u64, then u64 offsets of
 *      lens (+80), chunk_off (+88), outl_off (+96), sub_bits (+104), payload (+112),
 *      outl_idx (+120), outl_val (+128), +136 total_size u64, rest zero
 *    lens      u8[2*radius]          code length of each symbol (0 = unused); codes are
 *                                    canonical: ordered by (length, symbol), first code 0,
 *                                    read most significant bit first
 *    chunk_off u32[nchunks+1]        start of each chunk's bit stream in 16-byte units
 *    outl_off  u32[nchunks+1]        number of outliers before each chunk
 *    sub_bits  u16[nchunks*chunk/sub] bits of every sub-block of `sub` consecutive codes (version 2:
 *                                    0 for a sub-block of zero residuals, which has no bits in the payload)
 *    payload   chunk bit streams, each padded with zero bits to a multiple of 128 bits;
 *              bit k of a stream is bit 31-(k%32) of little-endian 32-bit word k/32
 *    outl_idx  u32[n_outliers]       linear NCHW index, ascending
 *    outl_val  i32[n_outliers]       the Lorenzo residual kept verbatim
 */
#ifndef CMPZ_H
#define CMPZ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CMP_OK           0
#define CMP_E_ARG      (-1)  /* NULL pointer, bad shape, numel > 2^32 - 8192 or > max_numel, eb not
                                finite or outside [2^-60, 2^60], unsupported configuration   */
#define CMP_E_NOSPACE  (-2)  /* out_cap smaller than the container; nothing is written past
                                out_cap and header.status is set when the header fits        */
#define CMP_E_FORMAT   (-3)  /* decompress: not a container, damaged, or truncated            */
#define CMP_E_MISMATCH (-4)  /* decompress: shape / eb / configuration differ from the header */
#define CMP_E_HIP      (-5)  /* a HIP runtime call failed                                     */
#define CMP_W_RANGE      1   /* some |x*r| > 16384 or non-finite x: those elements were
                                clamped (NaN -> 0) and the error bound does not hold for them */

typedef struct cmp_ctx cmp_ctx;   /* opaque */

typedef struct {
    uint32_t radius;       /* residuals d with |d| < radius get symbol d+radius; 1..512        */
    uint32_t chunk;        /* codes per independently addressable Huffman chunk; 4096          */
    uint32_t sub;          /* codes per sub-block whose bit count is stored: 32, 64 or 128    */
    uint32_t guard_shift;  /* 1..23, see "Arithmetic" above                                    */
    uint64_t max_numel;    /* most elements one launch group holds: no tensor may be larger, and a
                              batch with more in total is worked off in several groups         */
    uint32_t flags;        /* CMP_F_* below                                                    */
    uint32_t reserved;     /* 0                                                                */
} cmp_config;

/* Sparsity-aware front end (container version 2).  Activation data are dominated by zeros
 * (Section 3.2; Section 4.4 restores them exactly): a sub-block whose residuals are all zero is
 * recorded by a stored bit count of 0 -- a value no coded sub-block can have -- and its codes take
 * no part in the histogram, the codebook or the bit stream.  Compress and decompress must agree
 * on the flag (CMP_E_MISMATCH otherwise). */
#define CMP_F_ZERO_BLOCKS 1u

/* Defaults: radius 512, chunk 4096, sub 128, guard_shift 7, max_numel 2^28, flags 0: the
 * parameters of the compressor stages of Section 3.1 that the paper leaves to the implementation. */
void cmp_default_config(cmp_config *cfg);

/* The framework of Section 4.4 compresses the activation of every convolutional layer in every
 * iteration: what the kernels need between their stages (Section 3.1: symbols between the two
 * sweeps, histograms, code tables) is allocated once, here, and reused by every call.
 * Creates a context on GPU `device` with its scratch (about 2 bytes * max_numel + 9 bytes per chunk
 * + 1.3 MB of device memory, owned by the context).  cfg == NULL means defaults.  Returns CMP_E_ARG
 * for an unsupported configuration or device, CMP_E_HIP if the allocation fails (*out = NULL). */
int cmp_create(cmp_ctx **out, const cmp_config *cfg, int device);
/* Waits for the device and frees the context's scratch; containers and tensors are the caller's
 * and are not touched.  NULL is allowed. */
void cmp_destroy(cmp_ctx *ctx);

/* The compressed activation is held in memory until the backward pass (Section 4.4), in a buffer
 * the caller sizes before the data are seen: worst-case container size in bytes for a tensor of
 * this shape (every element an outlier, every code of flat length; 0 on bad arguments).  A
 * container never exceeds it. */
size_t cmp_bound(const cmp_ctx *ctx, const int64_t shape[4]);

/* Forward pass (Section 4.4): compress d_x (fp32, shape N,C,H,W) under the
 * absolute error bound eb into the container at d_out (capacity out_cap bytes).
 * Stages, each a kernel on `stream`: pre-quantisation, per-(n,c)-plane 2D
 * Lorenzo prediction, quantisation-code / outlier split and histogram
 * (Section 3.1); Huffman codebook; chunked bit-packing.
 * h_size == NULL: fully asynchronous.  h_size != NULL: waits for the stream and
 * stores the container size; the return value then also reports CMP_E_NOSPACE
 * (h_size = bytes needed) and CMP_W_RANGE. */
int cmp_compress(cmp_ctx *ctx, const float *d_x, const int64_t shape[4], float eb,
                 void *d_out, size_t out_cap, size_t *h_size, void *stream);

/* cmp_compress for n tensors at once (the activations of several layers, Section 4.4): every
 * stage is ONE kernel launch over all of them (the codebooks are built side by side, one
 * workgroup each), so that small tensors cost their bytes and not a chain of launches.  All
 * arrays are HOST arrays of n entries: device pointers d_x[i], d_out[i], shapes[i], error bounds
 * eb[i], capacities out_cap[i].  Container i is byte for byte what cmp_compress gives for tensor i.
 * Calls with more than 24 tensors or more than cfg.max_numel elements in total are worked off in
 * several groups, one after the other on `stream`; no single tensor may exceed cfg.max_numel.
 * h_sizes == NULL: fully asynchronous.  Otherwise waits for the stream and stores the n container
 * sizes; the return value is then the most severe per-tensor result (as for cmp_compress).
 * Arguments are checked for all tensors before anything is launched. */
int cmp_compress_batch(cmp_ctx *ctx, int n, const float *const *d_x, const int64_t (*shapes)[4], const float *eb,
                       void *const *d_out, const size_t *out_cap, size_t *h_sizes, void *stream);

/* cmp_compress for callers that cannot allocate device memory and therefore cannot hold a
 * context: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * It runs the same kernels as cmp_compress and gives the same container, with its scratch in an
 * array that is part of the library's device image: about 11.7 MB on every GPU the library is
 * loaded on, held until the process ends.  The call allocates nothing (no hipMalloc, no
 * hipFree, no pinned memory) and does not synchronise.
 *   device   the GPU of d_x and d_out;
 *   cfg      NULL = defaults; max_numel is ignored;
 *   limit    at most CMP_STATIC_MAX_NUMEL elements: larger tensors are refused with CMP_E_ARG.
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (two streams, two
 * threads) race; issue them on one stream, or order them with events.  Conditions only the GPU
 * sees are recorded in the container header and reported by cmp_compressed_size (whose ctx may
 * be NULL: the current device is used).  Capacity below the container's fixed sections:
 * CMP_E_NOSPACE. */
#define CMP_STATIC_MAX_NUMEL (1u << 22)
int cmp_compress_static(int device, const cmp_config *cfg, const float *d_x, const int64_t shape[4], float eb,
                        void *d_out, size_t out_cap, void *stream);

/* Compressed activations of a forward pass, held as a stack in ONE device buffer until the
 * backward pass pops them in reverse order (Section 4.4: compress when a layer's activation is
 * saved, keep it in memory, decompress when the backward pass reaches that layer).  Where a
 * container starts depends on the sizes of all containers before it, which only the GPU knows:
 * the bookkeeping (top of the stack, one record per slot) therefore lives in device memory, and
 * none of these calls makes the host wait, except cmp_arena_stats.
 *   d_state   device memory of cmp_arena_state_bytes(slots) bytes, 16-byte aligned, set up by
 *             cmp_arena_init (a kernel on `stream`);
 *   d_arena   the buffer of the containers, 256-byte aligned, arena_cap bytes;
 *   slot      which record a push fills and a pop reads: the caller numbers its pushes 0, 1, 2, ...
 *             and reuses a number only after the slots at and above it have been popped.
 * cmp_arena_push compresses d_x (as cmp_compress does) to the top of the stack and records the
 * container in `slot`; if it does not fit, the slot stays empty and the state counts a failure
 * (also reported by cmp_last_status as CMP_E_NOSPACE).  cmp_arena_pop decompresses the container of
 * `slot` into d_xout (as cmp_decompress does) and gives the slot back: the space returns to the
 * stack as soon as every slot above it has been popped too, so pops in reverse push order keep the
 * stack compact, and a pop out of order leaves a hole until then.  An empty slot pops as a
 * malformed container (CMP_E_FORMAT from cmp_last_status).  Empty tensors and shapes whose
 * planes are larger than one band of the decoder (about 2000 elements) with rows wider than 256
 * are refused by push and pop (CMP_E_ARG; cmp_arena_accepts tells beforehand, 1 = accepted): keep
 * such tensors outside the arena.  All calls that use one d_state must be issued on one stream.
 * cmp_arena_stats waits for `stream` and stores the bytes in use, their peak, the slots held and
 * the pushes that failed (any pointer may be NULL); it returns CMP_E_NOSPACE if any push failed. */
size_t cmp_arena_state_bytes(uint32_t slots);
int cmp_arena_accepts(const cmp_ctx *ctx, const int64_t shape[4]);
int cmp_arena_init(cmp_ctx *ctx, void *d_state, uint32_t slots, void *stream);
int cmp_arena_push(cmp_ctx *ctx, void *d_arena, size_t arena_cap, void *d_state, uint32_t slot, const float *d_x,
                   const int64_t shape[4], float eb, void *stream);
int cmp_arena_pop(cmp_ctx *ctx, const void *d_arena, void *d_state, uint32_t slot, const int64_t shape[4], float eb,
                  float *d_xout, void *stream);
int cmp_arena_stats(cmp_ctx *ctx, const void *d_state, uint64_t *h_top, uint64_t *h_peak, uint32_t *h_held,
                    uint32_t *h_failed, void *stream);

/* cmp_compress in two calls, for callers that pipeline tensors over several streams: the single
 * workgroup that builds the Huffman codebook leaves the GPU idle, and with begin(i+1) issued on
 * one stream while finish(i) runs on another the first sweep of the next tensor fills that time.
 *   cmp_compress_begin   the first sweep (pre-quantisation, Lorenzo prediction, code / outlier
 *                        split, histogram; Section 3.1) on `stream`;
 *   cmp_compress_finish  codebook, bit-packing and outlier records into d_out, on `stream`, which
 *                        may differ from the first one if the caller orders it after that call's
 *                        work (an event).  d_x of the begin call is read again (outlier records)
 *                        and must stay valid and unchanged until this work is done.
 * A context holds one tensor at a time between the two calls: begin returns CMP_E_ARG while a
 * previous begin has not been finished, finish without begin returns CMP_E_ARG.  The pair gives
 * the same container as cmp_compress; h_size as there. */
int cmp_compress_begin(cmp_ctx *ctx, const float *d_x, const int64_t shape[4], float eb, void *stream);
int cmp_compress_finish(cmp_ctx *ctx, void *d_out, size_t out_cap, size_t *h_size, void *stream);

/* Waits for `stream`, reads the header of a container produced by cmp_compress
 * and stores its size in bytes (the compression-ratio monitor of Section 4.4
 * reads this; ctx may be NULL, the current device is then used).  Returns CMP_E_NOSPACE (h_size = bytes needed) if that compress
 * ran out of room, CMP_W_RANGE if it clamped values, CMP_E_FORMAT if d_buf does
 * not start with a container header. */
int cmp_compressed_size(cmp_ctx *ctx, const void *d_buf, size_t *h_size, void *stream);

/* Backward pass (Section 4.4): decode the container at d_buf (`size` = bytes
 * available there), undo the Lorenzo predictor by per-plane 2D prefix sums and
 * de-quantise into d_xout (fp32, shape N,C,H,W).  shape and eb must be those
 * given to cmp_compress.  Zeros of the original tensor come back as +0.0f and no
 * value changes sign, so the re-zero filter of Section 4.4 is the identity.
 * Asynchronous; a malformed or mismatching container leaves d_xout unspecified
 * (never written out of bounds) and is reported by cmp_last_status. */
int cmp_decompress(cmp_ctx *ctx, const void *d_buf, size_t size, const int64_t shape[4],
                   float eb, float *d_xout, void *stream);

/* cmp_decompress for n containers at once (host arrays of n entries, as for cmp_compress_batch):
 * one kernel launch decodes all of them; tensor i comes out bit for bit as cmp_decompress gives
 * it.  Arguments are checked for all containers before anything is launched.  Asynchronous; the
 * most severe condition over the containers is reported by cmp_last_status. */
int cmp_decompress_batch(cmp_ctx *ctx, int n, const void *const *d_buf, const size_t *size, const int64_t (*shapes)[4],
                         const float *eb, float *const *d_xout, void *stream);

/* The error-bounded mode of Section 2.2 is a guarantee, so a call that could not keep it must be
 * able to say so: waits for `stream` and returns, then clears, the most severe condition the
 * GPU recorded for this context since the last query: a negative error code, else
 * CMP_W_RANGE (values outside the quantiser's range were clamped: the bound does not hold for
 * them), else CMP_OK. */
int cmp_last_status(cmp_ctx *ctx, void *stream);

/* Intermediate results of the LAST cmp_compress on this context, one per stage of Section 3.1
 * (quantisation codes and outliers after prediction, histogram, Huffman code lengths and codes),
 * for parity checks.  Stores a device pointer into the context's scratch (valid until the
 * next call on the context) and its size in bytes.  The caller synchronises.  CMP_E_ARG for an
 * unknown stage, for NULL pointers, and for the outlier stages before the first compress. */
#define CMP_STAGE_QUANT_CODES 0   /* uint16[numel]: symbol per element, 0 = outlier (waits for the GPU) */
#define CMP_STAGE_HIST        1   /* uint32[2*radius]: occurrences of each symbol              */
#define CMP_STAGE_LENS        2   /* uint8[2*radius]: Huffman code length, 0 = unused          */
#define CMP_STAGE_CODES       3   /* uint64[2*radius]: length << 56 | canonical code           */
#define CMP_STAGE_OUTLIER_IDX 4   /* uint32[n_outliers]: linear index of every outlier, ascending; this and the
                                     next stage point into the container and wait for the GPU          */
#define CMP_STAGE_OUTLIER_VAL 5   /* int32[n_outliers]: their Lorenzo residuals                        */
int cmp_debug_stage(cmp_ctx *ctx, int which, const void **d_ptr, size_t *bytes);

/* Per-kernel timing for benchmarks.  cmp_profile(ctx, 1) clears the record and makes
 * every later kernel launch of this context be bracketed by two events on its stream
 * (this costs time: do not enable it inside a region whose wall time is reported);
 * cmp_profile(ctx, 0) stops recording.  cmp_profile_read waits for `stream`, then stores,
 * for up to `cap` kernels, the kernel name (static string), the summed duration in
 * milliseconds and the number of launches; it returns the number of kernels seen
 * (which may exceed cap) or a negative error.  Event creation allocates. */
int cmp_profile(cmp_ctx *ctx, int enable);
int cmp_profile_read(cmp_ctx *ctx, void *stream, int cap, const char **h_names,
                     double *h_total_ms, uint64_t *h_launches);

/* Error-bound estimate of the adaptive framework (Sections 4.1-4.3), to be called every W
 * iterations for a convolutional layer.  One kernel reduces three device arrays:
 *   d_act   the layer's activation tensor, act_numel values: R = fraction of non-zero elements
 *           (Eq. 9);
 *   d_loss  the loss arriving at the layer in the backward pass, batch_n samples of per_sample
 *           consecutive values: Lbar = mean over the samples of each sample's largest |value|
 *           (the "average loss" of Eq. 5, as read by this library);
 *   d_mom   the momentum of the layer's weights, mom_numel values: Mavg = mean of |m| (Eq. 7);
 * and evaluates, in fp64 on the device, sigma = sigma_frac * Mavg (Eq. 7) and
 * eb = sigma / (a * Lbar * sqrt(batch_n * R)) (Eq. 8 with the sqrt(R) of Eq. 9), rounded once to
 * fp32 and clamped to [eb_min, eb_max].  Waits for `stream`, then stores the bound in *h_eb and,
 * if h_stats != NULL, R, Lbar, Mavg in h_stats[0..2].  The pointers must be 16-byte aligned, the
 * arrays non-empty, each of at most 2^32 - 8192 values, batch_n <= 65536.
 * Returns CMP_W_RANGE and eb_min when there is nothing to estimate from (no non-zero activation,
 * zero loss, NaN or infinity in a statistic); CMP_E_ARG on bad arguments. */
typedef struct {
    float sigma_frac;   /* acceptable gradient error as a fraction of the momentum: 0.01 (Eq. 7) */
    float a;            /* empirical coefficient of Eq. 5: 0.32 (Section 5.1)                   */
    float eb_min;       /* > 0                                                                   */
    float eb_max;       /* >= eb_min                                                             */
} cmp_controller_config;

/* Defaults: sigma_frac 0.01, a 0.32, eb_min 1e-6, eb_max 1. */
void cmp_default_controller_config(cmp_controller_config *cfg);

int cmp_estimate_eb(cmp_ctx *ctx, const float *d_act, uint64_t act_numel, const float *d_loss, uint64_t batch_n,
                    uint64_t per_sample, const float *d_mom, uint64_t mom_numel, const cmp_controller_config *cfg,
                    float *h_eb, double *h_stats, void *stream);

/* A static English string for a return code of this library (the conditions listed at the top:
 * what broke the guarantee of Section 2.2 or the container of Section 3.1); never NULL. */
const char *cmp_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CMPZ_H */
