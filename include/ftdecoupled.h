/*
 * ftdecoupled.h -- C ABI of the decoupled, operation-level fault-tolerant attention: the
 * comparison system of Section 3.1 of "FT-Transformer: Resilient and Reliable Transformer with
 * End-to-End Fault Tolerant Attention" ("Operation-level protection for Attention with decoupled
 * kernels"), which the end-to-end kernel of ftattn.h is measured against (Section 4.1).  Part of
 * the same shared library.
 *
 * One forward call is three protected operations, each a kernel launch per head (GEMMs) or one
 * launch for all heads (softmax), with the score matrix S and the probability matrix P written to
 * and read back from device memory in between:
 *
 *   1. ABFT-GEMM I     S = Q K^T, protected by the library's strided ABFT GEMM (ftgemm.h; tensor
 *                      checksums of the rows of K, eq. (13)-(16)); S is stored in fp32.
 *   2. DMR row-softmax P = softmax(scale * S + causal mask), by dual modular redundancy, eq. (11),
 *                      (12): maximum and exponentials are evaluated twice and compared element by
 *                      element (|e_a - e_b| < eps_dmr), their mean is kept; the normalised row is
 *                      checked by |rowsum(P) - 1| < eps_dmr; a row that fails either test is
 *                      evaluated again (at most 3 attempts).  P is stored in fp16.
 *   3. ABFT-GEMM II    O = P V, protected the same way (tensor checksums of the rows of V^T, which
 *                      a small kernel writes in fp16 first), fp32 out.
 *
 * Memory: S and P are [batch, heads, seq, seq] -- the quadratic footprint that Section 3.2 and
 * Section 4.1 hold against this scheme; ftdec_footprint reports the bytes.
 *
 * Conventions as in ftattn.h: every function returns FTDEC_OK (0) or a negative code, never
 * throws or prints; q, k, v, o are DEVICE pointers owned by the caller ([batch, heads, seq,
 * head_dim], contiguous, 16-byte aligned; o is fp32); everything else passed by pointer is HOST
 * memory; the context owns all device scratch; forward allocates nothing.
 */
#ifndef FTDECOUPLED_H
#define FTDECOUPLED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ftdec_ctx ftdec_ctx; /* opaque, library-owned */

enum { FTDEC_F16 = 0, FTDEC_BF16 = 1 };
enum { FTDEC_OK = 0, FTDEC_EINVAL = -1, FTDEC_EUNSUPPORTED = -2, FTDEC_EHIP = -3, FTDEC_ENOMEM = -4 };
enum { FTDEC_FT_OFF = 0, FTDEC_FT_CORRECT = 1 };
/* where a fault is injected / which check raised an event */
enum { FTDEC_ST_GEMM1 = 0,   /* fp32 accumulator of S[row, col = key] after the last accumulation step */
       FTDEC_ST_EXP = 1,     /* first evaluation of exp(scale*S - max) at [row, col = key], first attempt */
       FTDEC_ST_PNORM = 2,   /* normalised P[row, col = key] before it is rounded and stored, first attempt */
       FTDEC_ST_GEMM2 = 3 }; /* fp32 accumulator of O[row, col = feature] */

typedef struct {
  uint32_t struct_size;   /* sizeof(ftdec_config), checked */
  int32_t batch, heads, seq, head_dim;   /* head_dim a multiple of 8, at most 256 */
  int32_t in_dtype;       /* FTDEC_F16 | FTDEC_BF16; GEMM I runs on the MFMA of that type, GEMM II on fp16
                             (P and V^T are held in fp16: exact for bf16 values in the fp16 normal range) */
  int32_t causal;         /* 0 | 1 */
  float softmax_scale;    /* <= 0 selects 1/sqrt(head_dim) */
  int32_t ft_mode;        /* FTDEC_FT_OFF: the same three kernels with every check compiled out or skipped;
                             FTDEC_FT_CORRECT: detect, locate, correct */
  float tau_rel;          /* threshold of the two ABFT GEMMs (see ftgemm.h); <= 0 selects 2^-15 */
  float eps_dmr;          /* tolerance of eq. (11) and (12); <= 0 selects 2^-12 */
  int32_t max_events;     /* capacity of each event log (one per head and GEMM, one for the softmax); <= 0 selects 4096 */
  int32_t device;
} ftdec_config;

typedef struct { int32_t b, h, stage, row, col, bit; } ftdec_fault;   /* invert `bit` (0..31) of the named fp32 value */

typedef struct {
  int32_t b, h, stage;    /* FTDEC_ST_*: the check that fired (GEMM1 / GEMM2: strided ABFT; EXP: eq. (11); PNORM: eq. (12)) */
  int32_t row;
  int32_t col;            /* located key / feature; -1: the row is flagged, no single element named (PNORM) */
  int32_t action;         /* 1 corrected (restored from the checksum / evaluated again), 0 detected only */
} ftdec_event;

typedef struct {
  int32_t n_events, n_events_dropped;
  const ftdec_event* events;   /* sorted by (b, h, stage, row, col); host memory owned by the context */
  int64_t retried_rows;        /* softmax rows that were evaluated more than once */
} ftdec_report_view;

/* Validates cfg and allocates S, P, V^T, the checksum rows and the event logs on cfg->device. */
int ftdec_create(const ftdec_config* cfg, ftdec_ctx** out);
int ftdec_get_config(const ftdec_ctx* ctx, ftdec_config* effective);
/* Device bytes held by the context: total, and the part that is S and P (Section 4.1, memory of the decoupled scheme). */
int ftdec_footprint(const ftdec_ctx* ctx, int64_t* total_bytes, int64_t* s_and_p_bytes);
/* The three protected operations of Section 3.1 on `hip_stream`.  faults: host array or NULL; a
 * fault outside the tensors (or on a masked position) fails with FTDEC_EINVAL before any launch. */
int ftdec_forward(ftdec_ctx* ctx, const void* q, const void* k, const void* v, void* o,
                  const ftdec_fault* faults, int32_t n_faults, void* hip_stream);
/* Waits for the last forward and exposes its events. */
int ftdec_report(ftdec_ctx* ctx, ftdec_report_view* out);
/* After ftdec_set_timing(ctx, 1) every forward brackets its three stages with HIP events on its
 * stream; ftdec_get_timing returns ms[0] = ABFT-GEMM I (all heads, checksum encoding included),
 * ms[1] = DMR row-softmax, ms[2] = ABFT-GEMM II (V^T and checksum encoding included). */
int ftdec_set_timing(ftdec_ctx* ctx, int32_t enabled);
int ftdec_get_timing(ftdec_ctx* ctx, float ms[3]);
int ftdec_destroy(ftdec_ctx* ctx);
/* ctx may be NULL: message of the calling thread's last failed ftdec_create. */
const char* ftdec_last_error(const ftdec_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* FTDECOUPLED_H */
