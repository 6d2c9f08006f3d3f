/*
 * hdc.h - C ABI of the MI355X (gfx950) library for the data-parallel hot path of
 * binary hyperdimensional computing as defined in arXiv 2206.04746 (HDTorch):
 * ID-Level encoding (Sec. III, Eq. 1), classical and online class-vector training
 * (Sec. III, Eqs. 2-3) and Hamming-distance inference (Sec. III), on bit-packed
 * hypervectors (Sec. IV-B1).
 *
 * Conventions for every entry point
 *   - All functions return 0 (HDC_OK) or a negative hdc_status; nothing throws.
 *     hdc_strerror() gives a short text; after HDC_EHIP, hdc_last_hip_error() gives the
 *     HIP runtime's own message for the calling thread.
 *   - Names ending in _host are HOST pointers, read during the call only.
 *     Names ending in _dev are DEVICE pointers owned by the caller (for example the
 *     data_ptr() of a PyTorch tensor).  The library never frees or keeps them; they
 *     must stay valid until the work enqueued on `stream` has completed.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work; the caller synchronises.
 *   - A hypervector of D bits is W = ceil(D/32) uint32 words, dimension d at bit
 *     (d & 31) of word (d >> 5) (LSB first); bits D..32W-1 of the last word are zero in
 *     every table the caller passes and in every vector the library writes.  Matrices
 *     are row-major and contiguous: hv[N][W], acc[C][D], dist[N][C].
 *   - N == 0 is a successful no-op.  A context may be used from one host thread at a
 *     time.  Work of one context on different streams may overlap only where it shares no
 *     device scratch of the context:
 *       hdc_search, hdc_pack, hdc_unpack, hdc_hsum, hdc_binarize_classical and
 *       hdc_binarize_online use none and may overlap with anything (so the search of one
 *       chunk of a stream can run beside the encoding of the next);
 *       hdc_encode and hdc_encode_sparse share the encoders' staging buffers: one at a time;
 *       hdc_train_classical and hdc_vsum share the training scratch: one at a time;
 *       hdc_train_online, hdc_train_online_batched and hdc_search_cosine share theirs: one
 *       at a time.
 *     With profiling on (hdc_profile_enable) no two calls may overlap.  A second context of
 *     the same model gives a second set of every buffer.
 */
#ifndef HDC_H
#define HDC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hdc_ctx hdc_ctx; /* opaque; owns DEVICE copies of the tables */

typedef enum {
    HDC_OK = 0,
    HDC_EINVAL = -1, /* null pointer, size out of range, misaligned pointer */
    HDC_ENOMEM = -2, /* host or device allocation failed */
    HDC_EHIP = -3,   /* a HIP runtime call or kernel launch failed */
    HDC_ELIMIT = -4, /* argument is valid but beyond what this build supports */
    HDC_ELABEL = -5  /* a label is outside [0, C) and label checking is on (hdc_set_label_check) */
} hdc_status;

typedef enum { HDC_F32 = 0, HDC_U8 = 1 } hdc_dtype;

/* Limits of this build (checked by hdc_create): */
#define HDC_MAX_D 1048576 /* bits per hypervector */
#define HDC_MAX_F 65535   /* features per sample */
#define HDC_MAX_L 256     /* quantisation levels (bin index is kept in one byte) */
#define HDC_MAX_C 1024    /* classes */

typedef struct {
    int32_t D;            /* hypervector dimension in bits, 1..HDC_MAX_D */
    int32_t F;            /* features per sample, 1..HDC_MAX_F */
    int32_t L;            /* quantisation levels (bins), 1..HDC_MAX_L */
    int32_t C;            /* classes, 1..HDC_MAX_C */
    hdc_dtype feat_dtype; /* element type of the feature matrix */
} hdc_params;

/*
 * Create a context on the CURRENT HIP device and copy the encoding tables to it
 * (synchronous, one time, not part of the timed path).
 *   item_host  [F][W]  ID vector of every feature            (Sec. III, the per-feature identity vectors)
 *   level_host [L][W]  value vector of every bin             (Sec. III, the per-bin value vectors)
 *   tie_host   [W]     bit taken when a majority vote ties exactly (F or a class count
 *                      even); the paper asks for a majority vote without a tie rule, this
 *                      one is the library's: strict majority, exact tie -> tie bit
 *   lo_host, scale_host [F]  bin rule for HDC_F32 features: t = (x - lo[f]) * scale[f]
 *                      in fp32 (two roundings, no fused multiply-add), bin = floor(t)
 *                      clamped to [0, L-1]; t < 0 or NaN -> bin 0.  scale is normally
 *                      float(L / (hi - lo)).  Both must be NULL for HDC_U8, whose rule is
 *                      bin = (x * L) >> 8.  (Sec. III fixes the number of bins, not the
 *                      rule that maps a value to one.)
 * Errors: HDC_EINVAL (null/invalid arguments, nonzero pad bits in a table),
 * HDC_ENOMEM, HDC_EHIP.  On error *out is NULL.
 */
int hdc_create(hdc_ctx **out, const hdc_params *p, const uint32_t *item_host,
               const uint32_t *level_host, const uint32_t *tie_host, const float *lo_host,
               const float *scale_host);

/* Free the context and its device tables.  Synchronises the device.  NULL is a no-op. */
int hdc_destroy(hdc_ctx *ctx);

/*
 * ID-Level encoding, Sec. III Eq. (1):
 *   hv[n][d] = majority over f of ( item[f][d] XOR level[bin(feats[n][f])][d] ),
 * strict majority (2*count > F), an exact tie takes tie[d]; pad bits are written 0.
 *   feats_dev [N][F]  fp32 or uint8 as given by feat_dtype, row-major, 4-byte aligned
 *   hv_dev    [N][W]  out
 * The bits do not depend on how the call is carried out: calls of 1024 samples or more (256 for
 * models of a thousand matrix instructions per 32 samples, e.g. 600 features at D = 10000) on a
 * model in which every dimension changes at most once along the levels, or up to 8 times
 * where enough dimensions change at the same levels (at most 256 levels, 4 to 896 features),
 * run as a contraction over the features on the matrix cores (long streams, 128 samples or
 * more per compute unit, of single-change models of at most about 370 features, or about 630
 * with at most 64 levels, in a form of their own), all others on the vector unit.
 */
int hdc_encode(hdc_ctx *ctx, const void *feats_dev, int64_t N, uint32_t *hv_dev, void *stream);

/*
 * hdc_encode for inputs whose features mostly fall into bin 0 (Sec. III Eq. (1); the result is
 * bit-identical to hdc_encode for every input).  Eq. (1)'s sum is split into the votes of a sample
 * with every feature in bin 0, a constant of the model, and a correction for each feature that is
 * not in bin 0; only the latter are bundled, at about 1.5 times the cost of a feature in
 * hdc_encode, so the call pays off when fewer than about 60 % of a sample's features leave bin 0
 * (80 % of the pixels of a digit image are background) and costs at most about half as much again
 * when they all do.  The first call allocates scratch (4 bytes per feature for 65536 samples) and
 * derives three tables on `stream`.  Arguments and errors as hdc_encode.
 */
int hdc_encode_sparse(hdc_ctx *ctx, const void *feats_dev, int64_t N, uint32_t *hv_dev, void *stream);

/*
 * How many 32-bit words per sample hdc_encode actually bundles.  Where all L level vectors
 * have the same bit, Eq. (1) gives the same bit for every sample; hdc_create finds those
 * dimensions and, when at least a quarter of D is like that, hdc_encode bundles the other
 * dimensions only and fills in the constants (the result is bit-identical).  Returns W when
 * every dimension is bundled, fewer otherwise (0 if all level vectors are equal), -1 for a
 * NULL context.  For reporting: the work of an encode call is this many words times F.
 */
int32_t hdc_encoded_words(const hdc_ctx *ctx);

/*
 * Classical training, Sec. III (one pass that adds every encoded vector into the
 * accumulator of its class):
 *   acc[c][d] += hv[n][d]  and  class_n[c] += 1   for c = labels[n].
 * Both outputs are ADDED TO, so chunks of a stream compose in any order (integer sums:
 * the result does not depend on chunking or sample order); the caller zeroes them
 * before the first chunk.  Samples whose label is outside [0, C) are skipped.
 *   hv_dev [N][W], labels_dev [N] int32, acc_dev [C][D] int32 in/out,
 *   class_n_dev [C] int64 in/out.
 */
int hdc_train_classical(hdc_ctx *ctx, const uint32_t *hv_dev, const int32_t *labels_dev,
                        int64_t N, int32_t *acc_dev, int64_t *class_n_dev, void *stream);

/*
 * Class vectors from classical accumulators by the same majority rule as encoding:
 *   class_hv[c][d] = 1 if 2*acc > class_n[c], 0 if <, tie[d] if equal
 * (so an empty class becomes the tie vector).  class_hv_dev [C][W] out, pad bits 0.
 */
int hdc_binarize_classical(hdc_ctx *ctx, const int32_t *acc_dev, const int64_t *class_n_dev,
                           uint32_t *class_hv_dev, void *stream);

/*
 * Online training, Sec. III Eqs. (2),(3) and the caption of Fig. 1: for each epoch, for
 * each sample n = 0..N-1 IN THIS ORDER, with s = 2*hv[n] - 1 (the +-1 view of the bits):
 *   cos_c = <acc[c], s> / (|acc[c]| * sqrt(D))   for every class, from the accumulators
 *           as they are before this sample (0 for an all-zero row; fp64 sums);
 *   pred  = lowest c with the largest cos_c;
 *   acc[y]    += float(1 - cos_y) * s                       (y = labels[n], always);
 *   acc[pred] -= float(lr * (1 - cos_pred)) * s             (only if pred != y).
 * acc_dev [C][D] fp32 is in/out (zero it for a fresh model); repeated calls continue
 * training.  Samples whose label is outside [0, C) are skipped.  The sequential
 * dependency between samples is the method's; one call is one dependency chain.
 * epochs >= 0; lr is the paper's learning rate gamma.  Beyond D = 32768 the call runs
 * hdc_train_online_batched with batches of one sample (the same method, three launches per sample).
 * Where the fastest kernel applies (C <= 12 with D <= 4096, or C <= 6 with D <= 10240) the first
 * call allocates 64 MB of context-owned scratch unless hdc_reserve has done so (HDC_ENOMEM if
 * that fails); later calls only enqueue on `stream`.  Other shapes allocate nothing.
 */
int hdc_train_online(hdc_ctx *ctx, const uint32_t *hv_dev, const int32_t *labels_dev, int64_t N,
                     int32_t epochs, float lr, float *acc_dev, void *stream);

/*
 * Batched online training, Sec. VI-D2 (class vectors updated only after every `batch`
 * datapoints).  For each epoch the samples are taken in consecutive batches of `batch`
 * (the last one may be shorter).  Within a batch the accumulators are frozen: every sample
 * of the batch is scored as in hdc_train_online (cos_c, pred, the two fp32 weights) against
 * the rows as they were before the batch; then
 *   delta[c] = sum over the batch of  +float(1 - cos_y) * s         for c == y
 *                                     -float(lr*(1 - cos_pred)) * s for c == pred != y
 * (fp64 sums) and acc[c] = float(double(acc[c]) + delta[c]), one rounding per element and
 * batch.  batch >= 1; a batch larger than N is one batch per epoch.  Other arguments, layout
 * and the treatment of out-of-range labels are those of hdc_train_online.  The first call,
 * and a call that needs more scratch than any before it (larger batch), allocates device
 * memory owned by the context (HDC_ENOMEM if that fails) and therefore synchronises the
 * device; later calls only enqueue on `stream`.
 */
int hdc_train_online_batched(hdc_ctx *ctx, const uint32_t *hv_dev, const int32_t *labels_dev,
                             int64_t N, int32_t epochs, float lr, int64_t batch, float *acc_dev,
                             void *stream);

/* class_hv[c][d] = 1 if acc > 0, 0 if acc < 0, tie[d] if acc == 0; [C][W] out, pad 0. */
int hdc_binarize_online(hdc_ctx *ctx, const float *acc_dev, uint32_t *class_hv_dev, void *stream);

/*
 * Hamming-distance inference, Sec. III (a query goes to the class whose vector is
 * nearest to it):
 *   dist[n][c] = number of dimensions in which hv[n] and class_hv[c] differ,
 *   pred[n]    = lowest c with the smallest dist[n][c].
 *   hv_dev [N][W], class_hv_dev [C][W] (pad bits zero), dist_dev [N][C] uint32 out or
 *   NULL when only predictions are wanted, pred_dev [N] int32 out (required).
 * Any D up to HDC_MAX_D; the fast paths hold a query row in the registers of one wave
 * (D <= 32768), longer rows are read again for every class.  Streams of 8192 or more
 * queries against 13 or more classes (20480 or more against 9 to 12) at D <= 32768 run as
 * a matrix-core contraction (dist = |hv| + |class_hv| - 2 <hv, class_hv>, exact), 31
 * classes to a pass (32 without distances); beyond four passes (one where D > 10240) the
 * classes are dealt out over several launches, and between them pred_dev holds
 * intermediate keys, not classes: read it after the call's work on the stream is
 * complete, as ever.  The results are the same bits whichever kernel runs.  The pad bits
 * of both inputs must be zero as stated: the kernels differ in what they would make of
 * set pad bits.
 */
int hdc_search(hdc_ctx *ctx, const uint32_t *hv_dev, int64_t N, const uint32_t *class_hv_dev,
               uint32_t *dist_dev, int32_t *pred_dev, void *stream);

/*
 * Cosine-similarity inference, Sec. III (the second similarity of Table I), against
 * real-valued class rows such as the online accumulators: with s = 2*hv[n] - 1,
 *   cos[n][c] = <acc[c], s> / (|acc[c]| * sqrt(D))   (0 for an all-zero row; fp64 sums),
 *   pred[n]   = lowest c with the largest cos[n][c]  (compared in fp64).
 *   hv_dev [N][W], acc_dev [C][D] fp32 (read only), cos_dev [N][C] fp32 out (the fp64 value
 *   rounded once) or NULL, pred_dev [N] int32 out (required).  Allocates context-owned
 *   scratch like hdc_train_online_batched.
 */
int hdc_search_cosine(hdc_ctx *ctx, const uint32_t *hv_dev, int64_t N, const float *acc_dev,
                      float *cos_dev, int32_t *pred_dev, void *stream);

/*
 * The stand-alone hypervector primitives of Sec. IV-B.  D and W are the context's.
 *   hdc_pack   (IV-B1)  bits_dev [N][D] bytes (any non-zero byte is a 1) -> hv_dev [N][W],
 *                       LSB first, pad bits 0.
 *   hdc_unpack (IV-B1)  hv_dev [N][W] -> bits_dev [N][D] bytes of 0 / 1.
 *   hdc_hsum   (IV-B2, horizontal summation)  sum_dev[n] = set dimensions of row n, int32 [N]
 *                       (pad bits must be zero, as everywhere in this library).
 *   hdc_vsum   (IV-B2, vertical summation)    sum_dev[d] = rows with dimension d set,
 *                       int32 [D], overwritten (zeros for N == 0); N <= INT32_MAX.  Uses the
 *                       context's training scratch: do not overlap with hdc_train_classical
 *                       on another stream.
 * All matrices are device pointers, row-major, rows back to back.
 */
int hdc_pack(hdc_ctx *ctx, const uint8_t *bits_dev, int64_t N, uint32_t *hv_dev, void *stream);
int hdc_unpack(hdc_ctx *ctx, const uint32_t *hv_dev, int64_t N, uint8_t *bits_dev, void *stream);
int hdc_hsum(hdc_ctx *ctx, const uint32_t *hv_dev, int64_t N, int32_t *sum_dev, void *stream);
int hdc_vsum(hdc_ctx *ctx, const uint32_t *hv_dev, int64_t N, int32_t *sum_dev, void *stream);

/*
 * Labels outside [0, C) are a caller's mistake.  By default the training calls skip such samples
 * (defined behaviour, see hdc_train_classical).  With label checking on (a debugging aid, off by
 * default) hdc_train_classical, hdc_train_online and hdc_train_online_batched first count the
 * labels outside the range on `stream`, wait for the count (the call synchronises the stream)
 * and return HDC_ELABEL without training anything if there is one.
 */
int hdc_set_label_check(hdc_ctx *ctx, int enable);

/*
 * Allocate now what entry points otherwise allocate at their first call (and which makes that
 * call synchronise the device): after hdc_reserve has covered the sizes that are used, no entry
 * point allocates, frees or synchronises.  `what` is a mask of
 *   HDC_RESERVE_ONLINE          the 64 MB of hdc_train_online's fast path
 *   HDC_RESERVE_ONLINE_BATCHED  hdc_train_online_batched for batches of up to max_batch samples
 *   HDC_RESERVE_SEARCH_COSINE   hdc_search_cosine for calls of up to max_queries queries
 *   HDC_RESERVE_ENCODE_SPARSE   hdc_encode_sparse (its derived tables are computed on `stream`)
 * max_batch / max_queries are read only with their flag (>= 1 then).  Errors: HDC_EINVAL,
 * HDC_ENOMEM, HDC_EHIP.  Growing a buffer frees the old one, which waits for the device.
 */
#define HDC_RESERVE_ONLINE 1u
#define HDC_RESERVE_ONLINE_BATCHED 2u
#define HDC_RESERVE_SEARCH_COSINE 4u
#define HDC_RESERVE_ENCODE_SPARSE 8u
#define HDC_RESERVE_ALL 15u
int hdc_reserve(hdc_ctx *ctx, unsigned what, int64_t max_batch, int64_t max_queries, void *stream);

/*
 * hdc_vsum for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  No context: D is passed, W = ceil(D / 32).  The call allocates
 * nothing and frees nothing; the scratch of its kernels (a row permutation, a work list, the
 * blocks' partial counts) is a static device array of 7.3 MB that every GPU the library runs on
 * holds until the process ends.  Limits: D <= 16384 (HDC_ELIMIT beyond), N <= INT32_MAX; rows are
 * taken 262144 at a time.  The first call on a device looks up the array's address and the device's
 * properties (no allocation; make it outside a capture).  All calls on one GPU share the array:
 * calls on one stream follow each other and are safe, calls that overlap on one GPU (different
 * streams) race.  Result and argument rules as hdc_vsum: sum_dev [D] int32 is overwritten.
 */
int hdc_vsum_static(int32_t D, const uint32_t *hv_dev, int64_t N, int32_t *sum_dev, void *stream);

/*
 * Measurement aid (not an operation of the paper): per-kernel device time.  While enabled,
 * every launch of a hot kernel is bracketed by a pair of HIP events recorded on the stream
 * the kernel runs on.  hdc_profile_read waits for the recorded events of one kernel, returns
 * the summed elapsed milliseconds and the number of timed launches, and forgets them.  At
 * most HDC_PROFILE_SLOTS launches per kernel are kept between two reads; later ones run
 * untimed.  Disabled by default (no events, no overhead).  total_ms / launches are HOST
 * pointers.
 */
typedef enum {
    HDC_K_ENCODE = 0,     /* bind + bundle + majority kernel of hdc_encode */
    HDC_K_QUANTIZE = 1,   /* bin-index kernel of hdc_encode */
    HDC_K_ACCUMULATE = 2, /* per-class vertical count kernel of hdc_train_classical */
    HDC_K_ONLINE = 3,     /* sequential updater of hdc_train_online */
    HDC_K_SEARCH = 4,     /* Hamming distance + argmin kernel of hdc_search */
    HDC_K_ONLINE_FWD = 5, /* partial dot products of hdc_train_online_batched */
    HDC_K_ONLINE_BWD = 6, /* batch sum + accumulator update of hdc_train_online_batched */
    HDC_K_ENCODE_CONTRACT = 7, /* the contraction form of hdc_encode (quantises, bundles and spreads in one kernel) */
    HDC_K_ENCODE_WIDE = 8,     /* the contraction form of hdc_encode for long streams (jobs of 64 or 128 samples) */
    HDC_K_COUNT = 9
} hdc_kernel_id;
#define HDC_PROFILE_SLOTS 512
int hdc_profile_enable(hdc_ctx *ctx, int enable);
int hdc_profile_read(hdc_ctx *ctx, int kernel_id, double *total_ms, int64_t *launches);

/* Text for a status code (static storage, never NULL). */
const char *hdc_strerror(int code);

/* hipGetErrorString of the last HIP failure seen by the calling thread ("" if none). */
const char *hdc_last_hip_error(void);

/* Library version, "major.minor.patch". */
const char *hdc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HDC_H */
