/*
 * nq.h -- C ABI of the NestQuant nested-integer library for AMD MI355X (gfx950).
 *
 * The library implements the data-parallel hot path of "NestQuant: Post-Training
 * Integer-Nesting Quantization for On-Device DNN" (arXiv 2506.17870):
 *   - integer weight decomposition of INT-n weights into a higher-bit part
 *     w_high (h bits) and a lower-bit part w_low (l bits), n = h + l
 *     (Sec. 3.2.1, Eq. 4 and Eq. 5);
 *   - packing of the two parts into two separately stored pages
 *     (Sec. 3.3.4, "Packed-Bit Tensors", "Storing & Scheduling");
 *   - switching: page the lower-bit page out (downgrade) or in (upgrade)
 *     (Sec. 3.2.3, Sec. 3.3);
 *   - inference in full-bit mode, weights recomposed on the fly as
 *     w_high * 2^l + w_low and dequantised with the scale s (Eq. 2, Eq. 4), or in
 *     part-bit mode, w_high alone with the scale s * 2^l (Eq. 8), as a GEMM or an
 *     implicit-GEMM convolution with int8 activations (Sec. 4.2), int32
 *     accumulation and a fused fp32 dequantisation epilogue.
 *
 * Conventions
 *   - Every pointer whose name starts with d_ is DEVICE memory, h_ is HOST memory.
 *     All memory is owned by the caller; the library allocates no device memory.
 *   - Every call that takes a `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) only enqueues work on it and returns; results are ready when
 *     that stream reaches the end of the enqueued work.
 *   - Functions return NQ_OK or an error; on error nothing was enqueued.  Nothing
 *     throws or aborts.  Arguments are checked on the host before any launch.
 *   - Weights are W[N][K] row major, N = output channels, K = reduction length.
 *     For a convolution K = KH*KW*Cin ordered (kh, kw, ci), i.e. the weight tensor
 *     is [Cout][KH][KW][Cin]; activations are NHWC int8.
 *   - Supported nestings: n_bits in {8, 6}, 1 <= l_bits <= n_bits - 2 (so h >= 2),
 *     which covers the paper's INT(8|h), h in 3..7, and INT(6|h), h in 3..5
 *     (Sec. 3.3.1).  INT-n weights arrive as int8 values inside [-2^(n-1), 2^(n-1)-1];
 *     the range is the caller's promise and is not checked on the device.
 *   - K must not exceed NQ_MAX_K, so that |acc| <= K * 2^14 fits an int32.
 */
#ifndef NQ_H
#define NQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NQ_MAX_K 65536

typedef enum {
    NQ_OK = 0,
    NQ_ERR_INVALID_ARG = 1,  /* NULL pointer, negative size, bad enum value           */
    NQ_ERR_UNSUPPORTED = 2,  /* (n_bits, l_bits), format or layout outside the above   */
    NQ_ERR_SHAPE = 3,        /* sizes inconsistent with each other or above the limits */
    NQ_ERR_ALIGN = 4,        /* a packed page is not 16-byte aligned                   */
    NQ_ERR_NOT_RESIDENT = 5, /* full-bit call while the lower-bit page is paged out    */
    NQ_ERR_RANGE = 6,        /* a buffer is smaller than the layout needs              */
    NQ_ERR_HIP = 7           /* the HIP runtime reported an error                      */
} nq_status;

/* How w_low is stored (Sec. 3.2.3 Eq. 9 and Sec. 3.3.3).
 * NQ_LOW_UNSIGNED_L: the bit-wise split of Eq. 4: w_high = w_int >> l (arithmetic),
 *   w_low = the low l bits of the two's-complement code, in [0, 2^l - 1]; recomposition
 *   is exact for every INT-n value.
 * NQ_LOW_SIGNED_L1: the paper's extra-1-bit compensation (Sec. 3.3.3): w_high comes from a rounding
 *   other than the shift, w_low = w_int - w_high * 2^l lies in [-2^l + 1, 2^l - 1] and is stored as a
 *   two's-complement field of l + 1 bits (the lower-bit page then has l + 1 bits per element; pass
 *   l + 1 to nq_packed_bytes); recomposition is shift-ADD, w_high * 2^l + w_low (Eq. 4).
 *   nq_decompose / nq_decompose_pack produce w_high = clip(round-half-to-even(w_int / 2^l)) to h bits;
 *   any other w_high (adaptive rounding) goes through nq_pack with its own residual.  Both modes
 *   run on every GEMM / convolution kernel; the full-bit mode decodes one more bit per weight. */
typedef enum { NQ_LOW_UNSIGNED_L = 0, NQ_LOW_SIGNED_L1 = 1 } nq_low_format;

/* Page layouts.
 * NQ_LAYOUT_DENSE: exactly k bits per element on the shape padded to N%32 == 0,
 *   K%64 == 0 (zero fields in the padding).  Tiles of 32 rows x 64 columns, row-block
 *   major, each k*256 bytes.  Inside a tile, dword (i, slot) is at dword offset
 *   slot*k + i, i in [0,k) (the k dwords of a slot are contiguous, so that a kernel fetches
 *   them with one or two wide loads), slot = 32*g + r with r the row in the tile and g the
 *   half of the 64 columns.  The slot's 32 columns are c = 32*g + 4*j + b (j in [0,8) the
 *   position, b in [0,4) the byte lane); byte b of dword (i, slot) is byte B_i of the
 *   group (slot, b), which stores the fields F_0..F_7 of positions 0..7:
 *     higher-bit page ("carrier"): with s = 8-k, bits [7..s] of B_i hold F_i for i < k;
 *       the low s bits of B_0, B_1, ... in this order, least significant first, form a
 *       string of k*s bits holding F_k, ..., F_7 one after the other, LSB first;
 *     lower-bit page ("bit string"): B_0..B_{k-1} read as one little-endian string of
 *       8k bits hold F_j in bits [j*k, (j+1)*k).
 *   A field is the value modulo 2^k.
 * NQ_LAYOUT_PAPER_U64: the paper's packed-bit tensor (Sec. 3.3.4): 64/k (integer
 *   division) fields per unsigned 64-bit word, field j in bits [j*k, (j+1)*k), spare top
 *   bits zero (readers ignore them), each row starts a new word, the last word of a row
 *   zero padded.  This layout can be packed and unpacked, and nq_gemm_* and nq_conv_* read
 *   it directly (a model stored as the paper packs it needs no repacking; the activations
 *   must then start on a 4-byte boundary and stay below 2^31 - 2^16 bytes).  It is the
 *   slower way in: the dense pages are what the kernels are built around, and the grouped
 *   convolution reads nothing else (NQ_ERR_UNSUPPORTED). */
typedef enum { NQ_LAYOUT_DENSE = 0, NQ_LAYOUT_PAPER_U64 = 1 } nq_layout;

typedef struct {
    int32_t n_bits;     /* n: 8 or 6                                  */
    int32_t l_bits;     /* l: 1 .. n-2; h = n - l                     */
    int32_t low_format; /* nq_low_format                              */
    int32_t layout;     /* nq_layout                                  */
} nq_cfg;

/* One nested weight matrix: two pages plus the per-channel scale (Sec. 3.3.4: the model
 * file keeps w_high and w_low under separate names).  A plain descriptor filled by the
 * caller; the library owns none of the memory it points to, only `low_event`. */
typedef struct {
    nq_cfg cfg;
    int64_t N, K;
    const void *d_high;     /* device, packed higher-bit page, 16-byte aligned            */
    uint64_t high_bytes;    /* >= nq_packed_bytes(N, K, h, layout)                        */
    void *d_low;            /* device slot of the lower-bit page, 16-byte aligned; its    */
                            /* contents count only while low_resident != 0                */
    uint64_t low_bytes;     /* >= nq_packed_bytes(N, K, l, layout)                        */
    const void *h_low;      /* host master copy of the lower-bit page ("storage");        */
                            /* pinned memory makes nq_page_in_low asynchronous            */
    const float *d_scale;   /* device, fp32[N], per-output-channel scale s                */
    int32_t low_resident;   /* set by nq_page_in_low, cleared by nq_page_out_low; a       */
                            /* caller that wrote d_low on the device may set it itself    */
    int32_t low_event_armed;/* internal: low_event has been recorded                      */
    void *low_event;        /* internal: hipEvent_t made by nq_weight_init; "page is in"  */
    void *free_event;       /* internal: hipEvent_t made by nq_weight_init; "readers of   */
                            /* the page enqueued before nq_page_out_low are done"         */
    int32_t free_event_armed;
    int32_t events_borrowed;/* internal: the events belong to the head of a group           */
    int32_t group_head;     /* internal: other descriptors borrow this one's events         */
    int32_t reserved_;      /* keeps the size a multiple of 8                               */
} nq_weight;

/* Fused epilogue of the GEMM / convolution (Eq. 2 and Eq. 8), fp32, in this order with
 * one rounding per step and no fused multiply-add:
 *   c = act_scale * scale[n];  part-bit only: c = c * 2^l  (exact)
 *   y = (float)acc * c
 *   y = y + bias[n]                              if d_bias
 *   y = y + residual_scale * (float)residual[m][n]   if d_residual
 *   y = max(y, 0)                                if relu
 *   out_int8 == 0: Y[m][n] = y (fp32)
 *   out_int8 != 0: Y[m][n] = (int8) clamp(round_half_even(y * inv_out_scale), -128, 127)
 * d_acc_dump, if not NULL, also receives the raw int32 accumulators [M][N] (the sum over
 * k of x * w_full in full-bit mode, of x * w_high in part-bit mode). */
typedef struct {
    float act_scale;
    const float *d_bias;        /* device fp32[N] or NULL          */
    const int8_t *d_residual;   /* device int8[M][N] or NULL       */
    float residual_scale;
    int32_t relu;
    int32_t out_int8;
    float inv_out_scale;
    int32_t *d_acc_dump;        /* device int32[M][N] or NULL      */
} nq_epilogue;

/* NHWC convolution, groups = 1, dilation = 1, zero padding.
 * Ho = (H + 2*pad - KH)/stride + 1, Wo likewise; the GEMM view has M = B*Ho*Wo rows. */
typedef struct {
    int64_t B, H, W, Cin, Cout;
    int32_t KH, KW, stride, pad;
} nq_conv_shape;

/* ---- housekeeping ------------------------------------------------------------------ */
int nq_version(void);
const char *nq_status_string(int status);

/* Bytes of one packed page of `field_bits`-bit fields for an N x K matrix in `layout`
 * (DENSE: ceil(N/32)*32 * ceil(K/64)*64 * field_bits / 8; PAPER_U64: N * ceil(K/(64/k)) * 8).
 * Returns 0 for invalid arguments (field_bits outside 1..8 for PAPER_U64, 1..7 for DENSE). */
size_t nq_packed_bytes(int64_t N, int64_t K, int field_bits, int layout);

/* ---- quantisation ---------------------------------------------------------------- */
/* Eq. 1 (Sec. 3.1), per output channel (row n of the fp32 weights [N][K]): symmetric, no zero
 * point; d_scale[n] = max_k |w[n][k]| / (2^(n_bits-1) - 1), 1.0 for an all-zero row;
 * d_w_int[n][k] = Clip(round-half-to-even(w[n][k] / d_scale[n]), -2^(n_bits-1), 2^(n_bits-1) - 1).
 * The quotient and the rounding are taken in fp32 (IEEE division, not a reciprocal), so the codes
 * are a function of the fp32 inputs alone.  n_bits in 2..8.  Weights must be finite.
 * In: device fp32[N*K].  Out: device int8[N*K], fp32[N]; all caller owned. */
nq_status nq_quantize(const float *d_w, int64_t N, int64_t K, int n_bits, int8_t *d_w_int,
                      float *d_scale, void *stream);

/* The step of Eq. 1 for a whole tensor, as the per-tensor quantisation of the 8-bit activations uses it
 * (Sec. 4.2): d_scale[0] = max_i |d_x[i]| / (2^(n_bits-1) - 1), 1.0 for an all-zero (or empty) tensor; the
 * quotient is taken in fp32.  Calibrating a network's activation steps needs nothing else from the device.
 * In: device fp32[count], finite.  Out: device fp32[1] (also used as the accumulator: three small launches).
 * n_bits in 2..8.  NQ_ERR_ALIGN if a pointer is not 4-byte aligned. */
nq_status nq_tensor_scale(const float *d_x, int64_t count, int n_bits, float *d_scale, void *stream);

/* Eq. 1 for a whole tensor, scale and codes: nq_tensor_scale, then d_codes[i] = Clip(round-half-to-even(d_x[i] /
 * d_scale[0]), -2^(n_bits-1), 2^(n_bits-1) - 1) with the fp32 division of nq_quantize.  This is how a float input
 * batch becomes the 8-bit activations of the first layer (Sec. 4.2).  In: device fp32[count], finite.  Out: device
 * int8[count], fp32[1]; caller owned.  count up to 2^41; NQ_ERR_SHAPE beyond, other errors as nq_tensor_scale. */
nq_status nq_quantize_tensor(const float *d_x, int64_t count, int n_bits, int8_t *d_codes, float *d_scale,
                             void *stream);

/* Eq. 1 followed by the decomposition and packing of nq_decompose_pack (Alg. 1 steps 1-3) without the
 * int8 tensor in between: one pass over the fp32 weights for the channel scales, one that quantises,
 * splits and writes the pages.  Same pages as nq_quantize + nq_decompose_pack.  NQ_LAYOUT_DENSE only
 * (NQ_ERR_UNSUPPORTED otherwise).  d_scale: out, fp32[N].  Either page may be NULL. */
nq_status nq_quantize_decompose_pack(const float *d_w, int64_t N, int64_t K, const nq_cfg *cfg,
                                     float *d_scale, void *d_packed_high, void *d_packed_low,
                                     void *stream);

/* ---- decomposition and packing ----------------------------------------------------- */
/* Eq. 4 / Eq. 5 (BitShift): d_high[i] = d_w_int[i] >> l (arithmetic shift, i.e. floor),
 * d_low[i] = d_w_int[i] - d_high[i] * 2^l in [0, 2^l - 1].  Elementwise over N*K int8.
 * In, out: device int8[N*K], caller owned.  Only NQ_LOW_UNSIGNED_L. */
nq_status nq_decompose(const int8_t *d_w_int, int64_t N, int64_t K, const nq_cfg *cfg,
                       int8_t *d_high, int8_t *d_low, void *stream);

/* Sec. 3.3.4: pack unpacked parts into pages of cfg->layout.  d_high holds values in the
 * INT-h range, d_low values in [0, 2^l - 1], both int8[N][K].  Either input/output pair may
 * be NULL to pack only the other page.  Pages: device, 16-byte aligned, at least
 * nq_packed_bytes(...) bytes; every byte of that size is written (padding as zero). */
nq_status nq_pack(const int8_t *d_high, const int8_t *d_low, int64_t N, int64_t K,
                  const nq_cfg *cfg, void *d_packed_high, void *d_packed_low, void *stream);

/* Alg. 1 step 2 (w_low = w_int - w_high * 2^l) and step 3 (pack and store) in one pass:
 * reads each INT-n weight once, writes the two pages.  Same results as nq_decompose
 * followed by nq_pack. */
nq_status nq_decompose_pack(const int8_t *d_w_int, int64_t N, int64_t K, const nq_cfg *cfg,
                            void *d_packed_high, void *d_packed_low, void *stream);

/* nq_decompose_pack for many tensors (the weights of a whole model) in as few launches as possible:
 * a launch per tensor is launch bound for the small layers of a CNN.  `jobs` is a HOST array of `count`
 * entries, read before the call returns; pointers inside are device memory as in nq_decompose_pack, both
 * pages required.  NQ_LAYOUT_DENSE only.  Same pages as `count` calls of nq_decompose_pack. */
typedef struct {
    const int8_t *d_w_int;   /* device int8[N*K] */
    int64_t N, K;
    void *d_packed_high;     /* device, 16-byte aligned, nq_packed_bytes(N, K, h, DENSE) */
    void *d_packed_low;      /* device, 16-byte aligned, nq_packed_bytes(N, K, l or l + 1, DENSE) */
} nq_pack_job;
nq_status nq_decompose_pack_batch(const nq_pack_job *jobs, int64_t count, const nq_cfg *cfg, void *stream);

/* Inverse of nq_pack: pages -> int8[N][K] parts (w_high sign-extended from h bits, w_low
 * in [0, 2^l - 1]).  Either pair may be NULL. */
nq_status nq_unpack(const void *d_packed_high, const void *d_packed_low, int64_t N, int64_t K,
                    const nq_cfg *cfg, int8_t *d_high, int8_t *d_low, void *stream);

/* ---- switching (Sec. 3.2.3, Sec. 3.3) ---------------------------------------------- */
/* Checks the descriptor, creates the internal event, sets low_resident = 0. */
nq_status nq_weight_init(nq_weight *w);
/* Destroys the internal event.  The caller frees its own buffers. */
nq_status nq_weight_destroy(nq_weight *w);

/* Downgrade full-bit -> part-bit: the lower-bit page is paged out.  The host copy is the
 * master, so nothing is moved: the page is marked non-resident, full-bit calls on `w`
 * now fail with NQ_ERR_NOT_RESIDENT, and the owner may reuse or free d_low once the work
 * already enqueued on `stream` has finished.  An internal event is recorded on `stream` at
 * this point; a later nq_page_in_low waits for it, so the incoming copy never overwrites
 * a page that full-bit kernels enqueued earlier on `stream` are still reading. */
nq_status nq_page_out_low(nq_weight *w, void *stream);

/* Upgrade part-bit -> full-bit: copies low_bytes from h_low to d_low on `copy_stream`
 * (asynchronous with respect to the host when h_low is pinned, so it can overlap part-bit
 * work running on another stream), records the internal event and marks the page
 * resident.  Later full-bit calls make their stream wait for that event. */
nq_status nq_page_in_low(nq_weight *w, void *copy_stream);

/* Switching a whole model (Sec. 3.3: the full-bit MODEL downgrades to the part-bit MODEL and
 * back).  nq_weight_init_group initialises `count` descriptors that share one pair of internal
 * events owned by ws[0] (destroy ws[0] last).  The batch calls do for all of them what the
 * single calls do for one, with one event operation in all; nq_page_in_low_batch merges the
 * copies of pages that follow each other without a gap in both host and device memory (pages
 * carved in the same order out of one pinned arena and one device arena) into single transfers,
 * so a model is paged in with a few large copies instead of one small copy per layer.
 * The members of a group (count > 1) share their events, so they switch together: nq_page_out_low and
 * nq_page_in_low on a single member return NQ_ERR_INVALID_ARG (two members paged in on different streams
 * would overwrite each other's "page is in" point); use the batch calls, on the whole group or on any part
 * of it, one call at a time. */
nq_status nq_weight_init_group(nq_weight *const *ws, int64_t count);
nq_status nq_page_out_low_batch(nq_weight *const *ws, int64_t count, void *stream);
nq_status nq_page_in_low_batch(nq_weight *const *ws, int64_t count, void *copy_stream);

/* ---- inference (Sec. 3.3, Eq. 2, Eq. 4, Eq. 8) -------------------------------------- */
/* Y[M][N] = epilogue( sum_k X[m][k] * (w_high[n][k] * 2^l + w_low[n][k]) ).
 * d_x: device int8[M][K], K = w->K, row major.  d_y: device fp32[M][N] or int8[M][N]
 * (epi->out_int8).  Requires w->low_resident, else NQ_ERR_NOT_RESIDENT (never falls back
 * to part-bit: the caller chooses the mode).  Pages in either layout (NQ_LAYOUT_PAPER_U64: see there
 * for its two extra conditions, NQ_ERR_ALIGN / NQ_ERR_SHAPE).  M == 0 is a no-op. */
nq_status nq_gemm_full(const int8_t *d_x, int64_t M, const nq_weight *w, const nq_epilogue *epi,
                       void *d_y, void *stream);

/* Y[M][N] = epilogue( sum_k X[m][k] * w_high[n][k] ) with the scale s * 2^l (Eq. 8).
 * Never reads w->d_low. */
nq_status nq_gemm_part(const int8_t *d_x, int64_t M, const nq_weight *w, const nq_epilogue *epi,
                       void *d_y, void *stream);

/* Many few-row GEMMs in one launch (Sec. 3.3: a deployed model is a stack of nested layers; at small batch the
 * packed pages are the traffic, and a launch per layer of a few blocks each is bound by the launches, not by
 * the pages).  `jobs` is a HOST array of `count` problems, read before the call returns; each is what one
 * nq_gemm_full (full_bit != 0) or nq_gemm_part call takes, with the epilogue by value.  Same results as `count`
 * single calls.  Built for the few-row regime: every M <= 64, K a multiple of 16, d_x 16-byte aligned, dense
 * pages, one nesting and lower-part format for all problems, and one output kind for all (fp32 without
 * residual, or int8 with N a multiple of 16 and aligned pointers; no accumulator dump): NQ_ERR_UNSUPPORTED /
 * NQ_ERR_ALIGN otherwise, and the caller issues single calls.  The problems are handed to the kernel as a
 * table in device memory: d_workspace (16-byte aligned, at least nq_gemm_batch_workspace_bytes(count), caller
 * owned) receives it by a copy ordered on `stream`, and must not be reused by other work until the launch
 * has finished.  Full-bit: every lower-bit page must be resident (NQ_ERR_NOT_RESIDENT); the stream waits for
 * pages still in flight. */
typedef struct {
    const int8_t *d_x;      /* device int8[M][K], K = w->K      */
    int64_t M;
    const nq_weight *w;
    nq_epilogue epi;
    void *d_y;              /* device fp32[M][N] or int8[M][N]  */
} nq_gemm_job;
size_t nq_gemm_batch_workspace_bytes(int64_t count);
nq_status nq_gemm_batch(const nq_gemm_job *jobs, int64_t count, int full_bit, void *d_workspace,
                        size_t workspace_bytes, void *stream);

/* nq_gemm_batch for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid it): the table goes into an array of the library's own in device memory instead
 * of a workspace, so the call allocates nothing and takes no workspace argument.  At most
 * NQ_GEMM_BATCH_STATIC_MAX problems per call (NQ_ERR_SHAPE beyond that).  Every GPU the process uses holds
 * its own copy of that array (about 0.4 MB) until the process ends.  All calls on one GPU share it: a call
 * overwrites the table of the call before, so two calls whose launches may overlap on one GPU (different
 * streams, or threads) race; calls on one stream are safe. */
#define NQ_GEMM_BATCH_STATIC_MAX 2048
nq_status nq_gemm_batch_static(const nq_gemm_job *jobs, int64_t count, int full_bit, void *stream);

/* The same two modes as an implicit-GEMM convolution: d_x is int8[B][H][W][Cin], the
 * output is [B][Ho][Wo][Cout]; w->N == Cout and w->K == KH*KW*Cin with k = (kh*KW + kw)*Cin + ci; the
 * epilogue's residual and accumulator dump are indexed like the output.  Pages in either layout: from
 * NQ_LAYOUT_PAPER_U64 pages (Sec. 3.3.4) a 1x1 stride-1 filter runs as the GEMM over the pixels and any other
 * filter gathers its rows from the input (d_x 4-byte aligned and smaller than 2 GiB, H, W < 16000:
 * NQ_ERR_ALIGN / NQ_ERR_SHAPE otherwise). */
nq_status nq_conv_full(const int8_t *d_x, const nq_conv_shape *shape, const nq_weight *w,
                       const nq_epilogue *epi, void *d_y, void *stream);
nq_status nq_conv_part(const int8_t *d_x, const nq_conv_shape *shape, const nq_weight *w,
                       const nq_epilogue *epi, void *d_y, void *stream);

/* Depthwise / grouped convolution in the same two modes (the layers of the lightweight CNNs of
 * Sec. 4): Cin and Cout are split into `groups` groups of gs = Cin / groups input and Cout / groups output
 * channels; output channel c sums over the gs input channels of group c / (Cout / groups).
 * d_x int8[B][H][W][Cin], output [B][Ho][Wo][Cout]; w->N == Cout, w->K == KH*KW*gs with k = (kh*KW + kw)*gs + ci.
 * Dense pages only (NQ_ERR_UNSUPPORTED for the word layout); groups must divide both channel counts and d_x be
 * smaller than 2 GiB (NQ_ERR_SHAPE).  Two kernels: depthwise layers and groups of 2 or 4 channels with
 * Cin == Cout a multiple of 16, up to 28 taps and a 16-byte aligned d_x run on the matrix cores; every other
 * shape (wider groups, the grouped 1x1 layers whose channel counts differ, odd channel counts, any alignment)
 * runs as a direct convolution on the vector ALU: same results, about a tenth of the speed. */
nq_status nq_gconv_full(const int8_t *d_x, const nq_conv_shape *shape, int groups, const nq_weight *w,
                        const nq_epilogue *epi, void *d_y, void *stream);
nq_status nq_gconv_part(const int8_t *d_x, const nq_conv_shape *shape, int groups, const nq_weight *w,
                        const nq_epilogue *epi, void *d_y, void *stream);

/* Test and tuning aid, not needed in normal use: process-wide overrides of choices the library otherwise
 * makes from the shape.  value 0 restores the library's own choice.  A forced kernel or tile height that
 * does not apply to a shape is ignored for that call.  Meant to be set while no other thread is inside
 * the library (the parity tests run every case once per kernel that can take it).
 *   NQ_TUNE_KERNEL:   1 generic, 2 windowed, 3 register-stationary, 4 large GEMM, 5 few input channels,
 *                     6 few rows, 9 stationary-weights GEMM (short reductions)
 *   NQ_TUNE_BIG_TM:   2..5, rows per block of the large-GEMM kernel = 32 * value; 6 = 128 rows with one block
 *                     per compute unit (the whole register file: deeper weight pipeline); 7 = blocks of 128 rows
 *                     x 128 columns (the library's choice for up to 128 output channels)
 *   NQ_TUNE_GC_UNITS: work units the patch planner of the depthwise / grouped kernel aims for
 *   NQ_TUNE_STAT_ROWS: 1 gives every block of the stationary-weights GEMM one run of consecutive rows instead of
 *                     dealing the row tiles to the blocks in turn
 * NQ_ERR_INVALID_ARG for an unknown key or a negative value. */
typedef enum { NQ_TUNE_KERNEL = 0, NQ_TUNE_BIG_TM = 1, NQ_TUNE_GC_UNITS = 2, NQ_TUNE_STAT_ROWS = 3, NQ_TUNE_COUNT = 4 } nq_tune_key;
nq_status nq_set_tuning(int key, int value);

/* Profiling aid: the next nq_gemm_* (nq_gemm_batch included) / nq_conv_* / nq_gconv_* call made by this host thread attaches the two
 * hipEvent_t (either may be NULL) to its kernel dispatch, so that hipEventElapsedTime(start,
 * stop) is the execution time of that kernel alone.  One shot; events are the caller's. */
nq_status nq_profile_next_launch(void *start_event, void *stop_event);
/* Profiling aid: which kernel the last nq_gemm_* / nq_conv_* / nq_gconv_* launch of this host thread ran:
 * *family as in NQ_TUNE_KERNEL (7 = depthwise / grouped on the matrix cores, 8 = word pages, 10 = direct grouped
 * convolution; 0 before the first launch), *variant the tile height of the large-GEMM kernel (2..6), the tile shape of the generic kernel, the waves along N
 * of the stationary-weights GEMM, else 0.  Lets a
 * benchmark group its time stamps by kernel instantiation, as a kernel trace does.  Either pointer may be NULL. */
nq_status nq_profile_last_kernel(int *family, int *variant);
/* Timing events for the call above: create / destroy a hipEvent_t, and the milliseconds
 * between two completed events (blocks until stop_event has completed). */
nq_status nq_event_create(void **event);
nq_status nq_event_destroy(void *event);
nq_status nq_event_elapsed_ms(void *start_event, void *stop_event, float *h_ms);

/* ---- glue of a residual CNN on int8 NHWC activations (the paper is silent on these;
 * they only make a whole quantised network runnable between the nested convolutions) --- */
/* Max pooling over the int8 codes; padding never wins.  Out: int8[B][Ho][Wo][C]. */
nq_status nq_maxpool_i8(const int8_t *d_x, int64_t B, int64_t H, int64_t W, int64_t C, int ksize,
                        int stride, int pad, int8_t *d_y, void *stream);
/* Global average pooling: int32 sum over the H*W positions, y = (float)sum * (in_scale /
 * (float)(H*W)), q = clamp(round_half_even(y * inv_out_scale), -128, 127).  Out: int8[B][C]. */
nq_status nq_avgpool_i8(const int8_t *d_x, int64_t B, int64_t HW, int64_t C, float in_scale,
                        float inv_out_scale, int8_t *d_y, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* NQ_H */
