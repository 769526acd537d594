/*
 * ftattn.h -- C ABI of the fault-tolerant fused attention library for AMD MI355X (gfx950).
 *
 * The library computes O = softmax(scale * Q K^T + causal mask) V for tensors of shape
 * [batch, heads, seq, head_dim] (the operand shape of Section 3.1 of "FT-Transformer: Resilient
 * and Reliable Transformer with End-to-End Fault Tolerant Attention") in one flash-style pass
 * and carries strided tensor checksums through that pass as Algorithm 1 of the paper
 * ("EFTA with unified verification", Section 3.4) prescribes:
 *
 *   - tensor checksums of every K and V tile with stride 8 and weights 1 and l+1
 *     (eq. (13), (14));
 *   - GEMM I with two checksum products (eq. (15), (16)), running max, exp, and ONE
 *     product-form check per key-tile iteration that covers GEMM I, the subtraction of the
 *     maximum and the exponentiation (Section 3.4 case 2); a linear fault is located with the
 *     second checksum and repaired from the first, an exponentiation fault is repaired by
 *     recomputation;
 *   - GEMM II with rescale and two checksum products, and ONE sum-form check after the loop
 *     that covers GEMM II, rescale and normalisation;
 *   - a range check of the final row-sum between the sum of exponentials of the per-tile
 *     maxima and the number of unmasked keys, with substitution of the lower bound
 *     (Section 3.4 case 3 and the "optimized EFTA" paragraph).
 *
 * A deterministic fault injector flips chosen bits of chosen fp32 intermediates inside the
 * kernel (fault model of Section 2.2; one bit flip per attention computation, Section 4.3).
 *
 * Conventions
 *   - All functions return FTATTN_OK (0) or a negative error code and never throw or print.
 *     After a failure ftattn_last_error() returns a message owned by the context.
 *   - q, k, v, o are DEVICE pointers owned by the caller: contiguous [batch, heads, seq,
 *     head_dim], 16-byte aligned.  Everything else passed by pointer is HOST memory.
 *   - The context owns all device scratch (encoded K / V tiles, fault and event buffers).
 *     ftattn_forward allocates nothing and is asynchronous on the stream it is given, except
 *     that a non-empty fault list is uploaded synchronously before the launch.
 *     Without a fault list (and with timing off) the call is kernel launches only: no
 *     allocation, memset or copy, so it may be recorded into a HIP graph by stream capture.
 *   - One context serves one shape; calls on one context must not overlap in time.
 */
#ifndef FTATTN_H
#define FTATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ftattn_ctx ftattn_ctx; /* opaque, library-owned */

enum { FTATTN_F16 = 0, FTATTN_BF16 = 1, FTATTN_F32 = 2 };
/* injection stages: which fp32 intermediate a fault hits */
enum { FTATTN_ST_S = 0, FTATTN_ST_EXP = 1, FTATTN_ST_ROWSUM = 2, FTATTN_ST_OACC = 3 };
/* checks that can raise an event */
enum { FTATTN_CHECK_S = 0, FTATTN_CHECK_EXP = 1, FTATTN_CHECK_L = 2, FTATTN_CHECK_O = 3 };
enum { FTATTN_OK = 0, FTATTN_EINVAL = -1, FTATTN_EUNSUPPORTED = -2, FTATTN_EHIP = -3, FTATTN_ENOMEM = -4 };
/* range_flags of the report: operands that do not survive the conversion of bf16 inputs to fp16 */
enum { FTATTN_RANGE_OPERAND_OVERFLOW = 1,   /* a finite bf16 value of Q, K or V of magnitude >= 65536: Inf in fp16 */
       FTATTN_RANGE_OPERAND_UNDERFLOW = 2,  /* a non-zero bf16 value below 2^-24: no significant bit left in fp16 (values
                                               between 2^-24 and 2^-14 become subnormals, error < 2^-25, not flagged) */
       FTATTN_RANGE_CHECKSUM_OVERFLOW = 4 };/* a tensor checksum of K or V beyond the fp16 range (either input type) */
/* ft_mode */
enum { FTATTN_FT_OFF = 0, FTATTN_FT_CORRECT = 1, FTATTN_FT_DETECT = 2 };

/* tile_flags bits (per [b, h, row tile, key tile]) */
enum { FTATTN_TF_DET_S = 1, FTATTN_TF_COR_S = 2, FTATTN_TF_DET_EXP = 4, FTATTN_TF_COR_EXP = 8 };
/* rowtile_flags bits (per [b, h, row tile]) */
enum { FTATTN_RF_DET_L = 1, FTATTN_RF_COR_L = 2, FTATTN_RF_DET_O = 4, FTATTN_RF_COR_O = 8,
       FTATTN_RF_EVENT_OVERFLOW = 16 };

typedef struct {
  uint32_t struct_size;   /* sizeof(ftattn_config), checked */
  int32_t batch, heads, seq, head_dim; /* head_dim 64 or 128; seq >= 1 (any length) */
  int32_t in_dtype;       /* FTATTN_F16 | FTATTN_BF16.  bf16 operands are converted to fp16 on
                             entry (exact for 2^-14 <= |x| <= 65504): the contractions run on
                             fp16 MFMA with fp32 accumulation for either input type.  Values outside
                             that range are reported in range_flags of the report. */
  int32_t out_dtype;      /* FTATTN_F32, or the input type */
  int32_t causal;         /* 0 | 1: lower-triangular mask including the diagonal */
  float softmax_scale;    /* <= 0 selects 1/sqrt(head_dim) */
  int32_t ft_mode;        /* FTATTN_FT_OFF: same kernel with every check compiled out;
                             FTATTN_FT_CORRECT: detect, locate, correct;
                             FTATTN_FT_DETECT: detect and locate, leave values as they are */
  int32_t stride;         /* checksum stride s of eq. (13): 0 or 8 = the strided tensor checksum (eight
                             classes per tile row); 1 = the traditional checksum the paper compares
                             it with (Sections 3.3, 4.2): one class over the 64 keys of a tile row and
                             one over all features, formed from the same encoded tiles, so that a row
                             has one residual per key tile and can name one element of it.  Needs a
                             protected ft_mode, rowsum_fold 0 and per_step 0.  Other values are
                             rejected */
  int32_t block_m, block_n; /* 0 selects the library's tile sizes (256 queries x 64 keys for
                             head_dim 128, 128 x 64 for head_dim 64); other values are
                             rejected.  Effective values: ftattn_get_config. */
  float eps1;             /* threshold of the per-iteration product-form check on
                             |ln prod P - ln P^c1| (Algorithm 1, first "if"); <= 0 selects 0.03 */
  float tau_o;            /* threshold of the final sum-form check on the normalised output
                             (Algorithm 1, last "if"); <= 0 selects 0.75 * 2^-9 */
  float delta_l;          /* relative slack of the row-sum range check; <= 0 selects 2^-10 */
  int32_t rowsum_fold;    /* 0: the row-sum is protected by the range restriction of Section 3.4 case 3
                             (the paper's method).  1 (an extension): the value-tile checksums of class 0
                             also fold a column of ones at feature index head_dim, so that the first
                             checksum of class 0 carries the row-sum through GEMM II and the rescale; after
                             the loop the row-sum it implies is compared with the accumulated one
                             (relative difference against tau_o), the location rule over the
                             head_dim/8 + 1 folds decides whether the row-sum is the wrong element, and
                             if so it is replaced by the implied one (event FTATTN_CHECK_L).  The range
                             restriction is not applied in this mode. */
  int32_t per_step;       /* 0: unified verification (Algorithm 1, Section 3.4 "optimized EFTA").
                             1: verification after every step, the variant the paper measures as EFTA
                             before that optimisation: in every iteration GEMM I is verified on its own
                             (a class whose linear residual exceeds eps1/2 is located and repaired even
                             when the product-form statistic stays below eps1), the row-sum is checked
                             against its range so far after the reduce-sum, and the unnormalised output
                             accumulator against its checksum after GEMM II (|residual| <= tau_o *
                             row-sum); their events carry the key tile.  The checks after the loop stay.
                             2: as 1, with the softmax protected by duplication (eq. (11), (12)) instead
                             of the product-form check and the range restriction: maximum, exponentials
                             and reduce-sum are evaluated twice and compared bit by bit, a third
                             evaluation settles a difference; every differing exponential is reported
                             (FTATTN_CHECK_EXP) and replaced, a differing row-sum likewise
                             (FTATTN_CHECK_L with its key tile).
                             1 and 2 need ft_mode FTATTN_FT_CORRECT and rowsum_fold 0. */
  float rescale_margin;   /* <= 0: Algorithm 1 as printed (the maximum is renewed in every iteration).
                             > 0 (an extension, at most 8): the subtracted value is a reference maximum
                             that is replaced by the running maximum only when that exceeds it by more
                             than this margin (natural-log units); otherwise the rescale factor is one
                             and the rescale of the output, of its checksums and of the row-sum is
                             skipped.  Exponentials reach e^margin instead of 1; the upper bound of the
                             row-sum range carries exp(running maximum - reference).  Applies to the
                             unprotected variant too.  Needs per_step 0, stride 8, rowsum_fold 0. */
  int32_t max_events;     /* capacity of the event log; <= 0 selects 65536 */
  int32_t device;         /* HIP device ordinal */
} ftattn_config;

/* One injected soft error: invert bit `bit` (0..31) of the fp32 encoding of
 *   S      : the raw GEMM I accumulator at (row, col) = (query, key); kv_tile must equal
 *            col / block_n and the position must not be masked;
 *   EXP    : exp(scale*S - m) at (row, col), same constraints;
 *   ROWSUM : the running row-sum of `row` right after the update of iteration kv_tile (col ignored);
 *   OACC   : the un-normalised output accumulator at (row, col = feature) right after the
 *            update of iteration kv_tile.
 * kv_tile must be an iteration that row takes part in (causal rows stop at their diagonal). */
typedef struct { int32_t b, h, stage, kv_tile, row, col, bit; } ftattn_fault;

typedef struct {
  int32_t b, h, check;    /* FTATTN_CHECK_* */
  int32_t kv_tile;        /* key-tile iteration (S, EXP); -1 for the post-loop checks (L, O) */
  int32_t row;            /* global query index */
  int32_t col;            /* S, EXP: global key index; O: feature index; L: 0; -1 = not locatable */
  float residual;         /* S, EXP: log-ratio statistic; L: the offending row-sum; O: sum residual */
  int32_t action;         /* 1 corrected, 0 detected only */
} ftattn_event;

/* Views into host memory owned by the context; valid until the next forward / destroy. */
typedef struct {
  int32_t n_events;           /* events stored */
  int32_t n_events_dropped;   /* events that did not fit max_events */
  const ftattn_event* events; /* sorted by (b, h, check, kv_tile, row, col) */
  int32_t tiles_m, tiles_n;   /* row tiles and key tiles per head */
  const uint8_t* tile_flags;     /* [batch, heads, tiles_m, tiles_n], FTATTN_TF_* (from stored events) */
  const uint8_t* rowtile_flags;  /* [batch, heads, tiles_m], FTATTN_RF_* */
  const float* residual_max;     /* [batch, heads, tiles_m, 4]: largest fault-free-looking statistic seen:
                                    0: |prod/expected - 1| of the product check, 1: |sum residual| of the
                                    O check, 2: row-sum / upper bound (rowsum_fold: relative row-sum
                                    residual), 3: lower bound / row-sum */
  int64_t recheck_entries;    /* how often a wave left the fast path to re-evaluate a check exactly */
  int32_t range_flags;        /* FTATTN_RANGE_* bits, 0 when every operand and checksum kept its value: the
                                 contractions run on fp16 MFMA for either input type, and a bf16 operand
                                 of magnitude >= 65536 or < 2^-24, or a checksum beyond 65504, does not survive the conversion.
                                 The pass still runs (results follow IEEE arithmetic on the converted values);
                                 the caller decides whether to rescale its inputs.  Each forward call reports
                                 on its own; replays of one captured graph share a flag word, so after
                                 replays the bits are those of any replay since the capture. */
} ftattn_report_view;

/* Validates cfg, allocates all device scratch for this shape on cfg->device. */
int ftattn_create(const ftattn_config* cfg, ftattn_ctx** out);
/* Copies the configuration in effect (defaults resolved: tile sizes, thresholds, scale). */
int ftattn_get_config(const ftattn_ctx* ctx, ftattn_config* effective);
/* One attention pass (Algorithm 1, all steps) on `hip_stream` (a hipStream_t, may be NULL).
 * faults: host array or NULL.  Faults that name a masked / out-of-range position make the call
 * fail with FTATTN_EINVAL before anything is launched.  With ft_mode OFF a fault list is
 * still applied (shows the unprotected damage). */
int ftattn_forward(ftattn_ctx* ctx, const void* q, const void* k, const void* v, void* o,
                   const ftattn_fault* faults, int32_t n_faults, void* hip_stream);
/* Waits for the last forward of this context and exposes its flags, residuals and events. */
int ftattn_report(ftattn_ctx* ctx, ftattn_report_view* out);
/* Kernel timing for benchmarks.  After ftattn_set_timing(ctx, 1) every forward brackets its
 * encode kernel and its fused kernel with HIP events on the stream it launches on;
 * ftattn_get_timing waits for the last forward and returns the two durations in milliseconds:
 * ms[0] = encode (Algorithm 1, "Encode tensor checksum", plus operand conversion / transposition),
 * ms[1] = fused attention kernel (all other steps of Algorithm 1). */
int ftattn_set_timing(ftattn_ctx* ctx, int32_t enabled);
int ftattn_get_timing(ftattn_ctx* ctx, float ms[2]);
int ftattn_destroy(ftattn_ctx* ctx);
/* Message of the last failure on this context ("" if none).  ctx may be NULL: returns the
 * message of the last failed ftattn_create of the calling thread. */
const char* ftattn_last_error(const ftattn_ctx* ctx);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The same pass as ftattn_create + ftattn_forward (same
 * kernels, default verification scheme: per_step 0, stride 8; any ft_mode, rowsum_fold, mask and
 * type), without a context: the encoded key / value tiles, the counters and the event log live in
 * one array of FTATTN_STATIC_SCRATCH_MIB MiB that is part of the library's device code and that
 * every GPU the library runs on holds until the process ends.  The call allocates and frees
 * nothing, on the host or on the device, and is two kernel launches on `hip_stream`.
 *   cfg           host pointer, as for ftattn_create (defaults resolved the same way; max_events is
 *                 capped at 4096).  A shape whose encoded tiles do not fit the array fails with
 *                 FTATTN_EUNSUPPORTED and a message that names both sizes; nothing is launched.
 *   q, k, v, o    device pointers owned by the caller, as for ftattn_forward.
 *   n_events_dev  device pointer to one int32 owned by the caller, or NULL: when the pass has run
 *                 it holds the number of events the checks raised (0 on a fault-free pass).
 * No fault list: the injector needs staging buffers.  All calls on one GPU share that GPU's
 * array, which keeps the previous call's contents; every part a pass reads is rewritten by its
 * own encode launch first, so calls may follow each other on one stream in any order of shapes,
 * but calls that overlap in time on one GPU (different streams, different threads) race.
 * On failure returns a negative code; ftattn_static_last_error() then returns the calling
 * thread's message (a fixed buffer, never allocated). */
#define FTATTN_STATIC_SCRATCH_MIB 64
int ftattn_forward_static(const ftattn_config* cfg, const void* q, const void* k, const void* v, void* o,
                          int32_t* n_events_dev, void* hip_stream);
const char* ftattn_static_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FTATTN_H */
