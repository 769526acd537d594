/*
 * ftgemm.h -- C ABI of the fault-tolerant linear layer for AMD MI355X (gfx950), part of the
 * same shared library as ftattn.h.
 *
 * The paper protects the linear modules of a transformer (projections, feed-forward layers)
 * with the strided ABFT it designs for Q K^T (Section 3.3: "Tensor Checksum Design", eq. (13),
 * (14), and "Strided ABFT with Tensor Checksum", eq. (15), (16); Figure 1 shows the feed-forward
 * module under that protection).  This library computes
 *
 *     Y = X W^T,    X: [m, k] (tokens),  W: [n, k] (weights), fp16 or bf16,  Y: [m, n] fp32 or the input type,
 *
 * in one kernel that carries, for every block of 256 output features, the two stride-8 tensor
 * checksums of the weight rows (weights 1 and l+1) through the contraction as 32 extra MFMA
 * rows (each checksum as a high word and a low word of the input type), and after the last
 * accumulation step compares, per token and checksum class, the fold of the 32 results with the
 * first checksum product.  A mismatch is located with the second checksum (fold = residual
 * ratio - 1) and the element is restored from the first.
 *
 * Conventions
 *   - Every function returns FTGEMM_OK (0) or a negative error code and never throws or prints;
 *     ftgemm_last_error() returns the message of the last failure.
 *   - x, w, y are DEVICE pointers owned by the caller, row-major, contiguous, 16-byte aligned.
 *     Everything else passed by pointer is HOST memory.
 *   - The context owns the device scratch (the encoded checksum rows of W, fault and event
 *     buffers).  ftgemm_forward allocates nothing and is asynchronous on its stream, except
 *     that a non-empty fault list is uploaded synchronously before the launch.
 *     Without a fault list the call is kernel launches only (no allocation, memset or copy),
 *     so it may be recorded into a HIP graph by stream capture.
 *   - One context serves one shape; calls on one context must not overlap in time.
 */
#ifndef FTGEMM_H
#define FTGEMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ftgemm_ctx ftgemm_ctx; /* opaque, library-owned */

enum { FTGEMM_F16 = 0, FTGEMM_BF16 = 1, FTGEMM_F32 = 2 };
enum { FTGEMM_OK = 0, FTGEMM_EINVAL = -1, FTGEMM_EUNSUPPORTED = -2, FTGEMM_EHIP = -3, FTGEMM_ENOMEM = -4,
       FTGEMM_ESTATE = -5 };
enum { FTGEMM_FT_OFF = 0, FTGEMM_FT_CORRECT = 1, FTGEMM_FT_DETECT = 2 };

typedef struct {
  uint32_t struct_size;  /* sizeof(ftgemm_config), checked */
  int32_t m, n, k;       /* m, n >= 1 (any value); k >= 8 and a multiple of 8 (rows are read in 16-byte chunks) */
  int32_t in_dtype;      /* FTGEMM_F16 | FTGEMM_BF16: type of x and w; the contraction runs on the MFMA of
                            that type with fp32 accumulation */
  int32_t out_dtype;     /* FTGEMM_F32, or the input type */
  int32_t ft_mode;       /* OFF: same kernel, checks and checksum rows compiled out;
                            CORRECT: detect, locate, restore; DETECT: detect and locate only */
  int32_t stride;        /* checksum stride s of eq. (13); 0 or 8 */
  int32_t block_n;       /* output features per checksum block; 0 or 256 */
  float tau_rel;         /* a class is flagged when |check1 - fold| > tau_abs + tau_rel * sum |Y_l|, */
  float tau_abs;         /* or when that residual is not finite.  tau_rel <= 0 selects 2^-15;
                            tau_abs < 0 selects 0 */
  int32_t fold_tokens;   /* 0: tensor checksums over the weight rows (blocks of 256 output features), encoded
                            once per weight matrix by ftgemm_encode_weights.  1: the column-checksum
                            counterpart (Section 3.3 names it for attention and rejects its memory cost there):
                            checksums over the token rows of x in blocks of 256 tokens, encoded inside every
                            ftgemm_forward; the same method on Y^T = W X^T.  It repairs several errors of one
                            token (they lie in different features) and cannot repair two errors of one feature
                            whose tokens are a multiple of 8 apart.  ftgemm_encode_weights is not needed. */
  int32_t max_events;    /* capacity of the event log; <= 0 selects 65536 */
  int32_t device;        /* HIP device ordinal */
} ftgemm_config;

/* One injected soft error (fault model of Section 2.2): invert bit `bit` (0..31) of the fp32
 * accumulator of Y[row, col] after the last accumulation step, before verification. */
typedef struct { int32_t row, col, bit; } ftgemm_fault;

typedef struct {
  int32_t row;           /* token index */
  int32_t col;           /* located output feature; -1 = flagged but not locatable (with fold_tokens it is the
                            row that is -1 then: the feature is known, the token is not) */
  float residual;        /* check1 - fold of the flagged class */
  int32_t action;        /* 1 restored, 0 detected only */
} ftgemm_event;

/* Views into host memory owned by the context; valid until the next forward / destroy. */
typedef struct {
  int32_t n_events;           /* events stored */
  int32_t n_events_dropped;   /* events that did not fit max_events */
  const ftgemm_event* events; /* sorted by (row, col) */
  float residual_max;         /* largest |check1 - fold| / threshold among classes that passed */
} ftgemm_report_view;

/* Validates cfg and allocates the device scratch for this shape on cfg->device. */
int ftgemm_create(const ftgemm_config* cfg, ftgemm_ctx** out);
/* Copies the configuration in effect (defaults resolved). */
int ftgemm_get_config(const ftgemm_ctx* ctx, ftgemm_config* effective);
/* Encodes the tensor checksums of the weight matrix (eq. (13), (14)) into the context, on
 * `hip_stream`.  Needed once per weight matrix and before the first forward when ft_mode is
 * not OFF (a forward without it fails with FTGEMM_ESTATE); w must be the matrix later passed to
 * ftgemm_forward. */
int ftgemm_encode_weights(ftgemm_ctx* ctx, const void* w, void* hip_stream);
/* One protected product Y = X W^T (eq. (15), (16), verification and repair) on `hip_stream`
 * (a hipStream_t, may be NULL).  faults: host array or NULL; a fault outside the matrix makes
 * the call fail with FTGEMM_EINVAL before anything is launched.  With ft_mode OFF a fault
 * list is still applied (shows the unprotected damage). */
int ftgemm_forward(ftgemm_ctx* ctx, const void* x, const void* w, void* y,
                   const ftgemm_fault* faults, int32_t n_faults, void* hip_stream);
/* Waits for the last forward of this context and exposes its events and residual statistic. */
int ftgemm_report(ftgemm_ctx* ctx, ftgemm_report_view* out);
/* Kernel timing for benchmarks: after ftgemm_set_timing(ctx, 1) every forward brackets its
 * kernel with HIP events on the stream it launches on; ftgemm_get_timing waits for the last
 * forward and returns the duration in milliseconds. */
int ftgemm_set_timing(ftgemm_ctx* ctx, int32_t enabled);
int ftgemm_get_timing(ftgemm_ctx* ctx, float* ms);
int ftgemm_destroy(ftgemm_ctx* ctx);
/* Message of the last failure on this context ("" if none).  ctx may be NULL: returns the
 * message of the last failed ftgemm_create of the calling thread. */
const char* ftgemm_last_error(const ftgemm_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* FTGEMM_H */
