// Host side of the fault-tolerant linear layer: the C ABI of include/ftgemm.h.  Validation,
// launches and the report are here; encoding, the contraction, verification and repair run in
// the kernels of ftgemm_main.h.
#include "ftgemm_main.h"

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

using namespace ftgemm;

struct ftgemm_ctx {
  ftgemm_config cfg;          // effective configuration
  int Tm = 0, Tn = 0;
  uint16_t* wc = nullptr;     // [Tn][32][k] checksum rows of the weights (input type)
  const void* encoded_w = nullptr;
  GFault* d_faults = nullptr;
  ftgemm_event* d_events = nullptr;
  int32_t* d_ev_count = nullptr;
  uint32_t* d_resmax = nullptr;
  GFault* h_faults = nullptr; // pinned staging
  int fault_cap = 0;
  std::vector<ftgemm_event> events;
  hipStream_t last_stream = nullptr;
  bool ran = false, timing = false;
  hipEvent_t ev[2] = {nullptr, nullptr};
  std::string err;
};

static thread_local std::string g_gemm_create_err;

static int gfail(ftgemm_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_gemm_create_err = msg;
  return code;
}

#define GHIP_TRY(ctx, expr)                                                                     \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess)                                                                       \
      return gfail(ctx, e_ == hipErrorOutOfMemory ? FTGEMM_ENOMEM : FTGEMM_EHIP,                \
                   std::string(#expr) + ": " + hipGetErrorString(e_));                          \
  } while (0)

static void grelease(ftgemm_ctx* c) {
  if (!c) return;
  (void)hipFree(c->wc); (void)hipFree(c->d_faults); (void)hipFree(c->d_events);
  (void)hipFree(c->d_ev_count); (void)hipFree(c->d_resmax);
  if (c->h_faults) (void)hipHostFree(c->h_faults);
  for (hipEvent_t e : c->ev) if (e) (void)hipEventDestroy(e);
  delete c;
}

typedef void (*gemm_fn)(const GArgs);

template <bool BF, bool RAG> static gemm_fn select_gemm_t(bool ft, bool inject) {
  if (ft) return inject ? ftgemm_main<true, true, BF, RAG> : ftgemm_main<true, false, BF, RAG>;
  return inject ? ftgemm_main<false, true, BF, RAG> : ftgemm_main<false, false, BF, RAG>;
}
// ragged: k is not a multiple of the kernel's K step
static gemm_fn select_gemm(bool ft, bool inject, bool bf, bool ragged) {
  if (ragged) return bf ? select_gemm_t<true, true>(ft, inject) : select_gemm_t<false, true>(ft, inject);
  return bf ? select_gemm_t<true, false>(ft, inject) : select_gemm_t<false, false>(ft, inject);
}
static size_t gemm_lds(bool ft) { return ft ? GStage<true>::LDS_TOTAL : GStage<false>::LDS_TOTAL; }

namespace ftgemm {
hipError_t gemm_allow_lds(int k) {
  for (int v = 0; v < 8; ++v) {
    hipError_t he = hipFuncSetAttribute((const void*)select_gemm((v & 1) != 0, (v & 2) != 0, (v & 4) != 0, k % GBK != 0),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_lds((v & 1) != 0));
    if (he != hipSuccess) return he;
  }
  return hipSuccess;
}
hipError_t gemm_launch_encode_w(const uint16_t* w, uint16_t* wc, int n, int k, bool bf16, hipStream_t st, int batch,
                                long long bs_w, long long bs_wc) {
  dim3 grid((n + GBN - 1) / GBN, (k / 8 + 31) / 32, batch);
  if (bf16) ftgemm_encode_w<true><<<grid, 256, 0, st>>>(w, wc, n, k, bs_w, bs_wc);
  else ftgemm_encode_w<false><<<grid, 256, 0, st>>>(w, wc, n, k, bs_w, bs_wc);
  return hipGetLastError();
}
hipError_t gemm_launch(const GArgs& a, bool ft, bool inject, bool bf16, hipStream_t st, int batch) {
  gemm_fn f = select_gemm(ft, inject, bf16, a.K % GBK != 0);
  hipLaunchKernelGGL(f, dim3(a.Tm * a.Tn, batch), dim3(GWAVES * 64), gemm_lds(ft), st, a);
  return hipGetLastError();
}
}  // namespace ftgemm

extern "C" int ftgemm_create(const ftgemm_config* cfg, ftgemm_ctx** out) {
  if (!cfg || !out) return gfail(nullptr, FTGEMM_EINVAL, "null argument");
  *out = nullptr;
  if (cfg->struct_size != sizeof(ftgemm_config)) return gfail(nullptr, FTGEMM_EINVAL, "struct_size mismatch");
  if (cfg->m < 1 || cfg->n < 1) return gfail(nullptr, FTGEMM_EINVAL, "m and n must be >= 1");
  if (cfg->k < 8 || cfg->k % 8 != 0) return gfail(nullptr, FTGEMM_EUNSUPPORTED, "k must be a positive multiple of 8 (rows of 16-byte chunks)");
  if (cfg->in_dtype != FTGEMM_F16 && cfg->in_dtype != FTGEMM_BF16) return gfail(nullptr, FTGEMM_EINVAL, "in_dtype must be F16 or BF16");
  if (cfg->out_dtype != FTGEMM_F32 && cfg->out_dtype != cfg->in_dtype) return gfail(nullptr, FTGEMM_EINVAL, "out_dtype must be F32 or the input type");
  if (cfg->ft_mode < 0 || cfg->ft_mode > 2) return gfail(nullptr, FTGEMM_EINVAL, "ft_mode out of range");
  if (cfg->stride != 0 && cfg->stride != 8) return gfail(nullptr, FTGEMM_EUNSUPPORTED, "stride must be 8");
  if (cfg->block_n != 0 && cfg->block_n != GBN) return gfail(nullptr, FTGEMM_EUNSUPPORTED, "block_n must be 256");
  if (cfg->fold_tokens != 0 && cfg->fold_tokens != 1) return gfail(nullptr, FTGEMM_EINVAL, "fold_tokens must be 0 or 1");
  // with fold_tokens the kernel runs the transposed problem: its tokens are the weight rows, its features the token rows
  const long long km = cfg->fold_tokens ? cfg->n : cfg->m, kn = cfg->fold_tokens ? cfg->m : cfg->n;
  const long long tm = (km + GBM - 1) / GBM, tn = (kn + GBN - 1) / GBN;
  if (tm * tn > 0x7FFFFFFFll) return gfail(nullptr, FTGEMM_EUNSUPPORTED, "too many output tiles");
  // the per-lane load offsets are 32-bit: 256 rows of k fp16 values must fit
  if ((long long)cfg->k * 2 * 256 > 0x7FFFFFFFll) return gfail(nullptr, FTGEMM_EUNSUPPORTED, "k too large");

  ftgemm_ctx* c = new (std::nothrow) ftgemm_ctx();
  if (!c) return gfail(nullptr, FTGEMM_ENOMEM, "out of host memory");
  c->cfg = *cfg;
  ftgemm_config& e = c->cfg;
  e.stride = 8;
  e.block_n = GBN;
  if (!(e.tau_rel > 0.f)) e.tau_rel = 1.0f / 32768.0f;
  if (!(e.tau_abs >= 0.f)) e.tau_abs = 0.f;
  if (e.max_events <= 0) e.max_events = 65536;
  c->Tm = (int)tm;
  c->Tn = (int)tn;
  c->fault_cap = 1 << 16;

  hipError_t he = hipSetDevice(e.device);
  if (he != hipSuccess) { int rc = gfail(nullptr, FTGEMM_EHIP, std::string("hipSetDevice: ") + hipGetErrorString(he)); delete c; return rc; }
#define GCREATE_TRY(expr)                                                                                 \
  do {                                                                                                    \
    hipError_t e_ = (expr);                                                                               \
    if (e_ != hipSuccess) {                                                                               \
      int rc_ = gfail(nullptr, e_ == hipErrorOutOfMemory ? FTGEMM_ENOMEM : FTGEMM_EHIP,                   \
                      std::string(#expr) + ": " + hipGetErrorString(e_));                                 \
      grelease(c);                                                                                        \
      return rc_;                                                                                         \
    }                                                                                                     \
  } while (0)
  const size_t n_wc = (size_t)c->Tn * GCK * e.k;
  GCREATE_TRY(hipMalloc((void**)&c->wc, n_wc * 2));
  GCREATE_TRY(hipMalloc((void**)&c->d_faults, sizeof(GFault) * c->fault_cap));
  GCREATE_TRY(hipMalloc((void**)&c->d_events, sizeof(ftgemm_event) * (size_t)e.max_events));
  GCREATE_TRY(hipMalloc((void**)&c->d_ev_count, sizeof(int32_t)));
  GCREATE_TRY(hipMalloc((void**)&c->d_resmax, sizeof(uint32_t)));
  GCREATE_TRY(hipHostMalloc((void**)&c->h_faults, sizeof(GFault) * c->fault_cap, hipHostMallocDefault));
  GCREATE_TRY(hipMemset(c->wc, 0, n_wc * 2));
  GCREATE_TRY(hipMemset(c->d_ev_count, 0, sizeof(int32_t)));
  GCREATE_TRY(hipMemset(c->d_resmax, 0, sizeof(uint32_t)));
  GCREATE_TRY(gemm_allow_lds(e.k));
  GCREATE_TRY(hipDeviceSynchronize());
#undef GCREATE_TRY
  *out = c;
  return FTGEMM_OK;
}

extern "C" int ftgemm_get_config(const ftgemm_ctx* ctx, ftgemm_config* effective) {
  if (!ctx || !effective) return FTGEMM_EINVAL;
  *effective = ctx->cfg;
  return FTGEMM_OK;
}

extern "C" int ftgemm_encode_weights(ftgemm_ctx* c, const void* w, void* hip_stream) {
  if (!c) return FTGEMM_EINVAL;
  if (!w || ((uintptr_t)w & 15)) return gfail(c, FTGEMM_EINVAL, "w must be a 16-byte aligned device pointer");
  const ftgemm_config& e = c->cfg;
  if (e.fold_tokens) return FTGEMM_OK;      // the checksums are those of x, taken inside every forward
  GHIP_TRY(c, hipSetDevice(e.device));
  hipStream_t st = (hipStream_t)hip_stream;
  dim3 grid(c->Tn, (e.k / 8 + 31) / 32);
  if (e.in_dtype == FTGEMM_BF16) ftgemm_encode_w<true><<<grid, 256, 0, st>>>(reinterpret_cast<const uint16_t*>(w), c->wc, e.n, e.k);
  else ftgemm_encode_w<false><<<grid, 256, 0, st>>>(reinterpret_cast<const uint16_t*>(w), c->wc, e.n, e.k);
  GHIP_TRY(c, hipGetLastError());
  c->encoded_w = w;
  return FTGEMM_OK;
}

extern "C" int ftgemm_forward(ftgemm_ctx* c, const void* x, const void* w, void* y,
                              const ftgemm_fault* faults, int32_t n_faults, void* hip_stream) {
  if (!c) return FTGEMM_EINVAL;
  if (!x || !w || !y) return gfail(c, FTGEMM_EINVAL, "null matrix pointer");
  if (((uintptr_t)x | (uintptr_t)w | (uintptr_t)y) & 15) return gfail(c, FTGEMM_EINVAL, "matrix pointers must be 16-byte aligned");
  if (n_faults < 0 || (n_faults > 0 && !faults)) return gfail(c, FTGEMM_EINVAL, "bad fault list");
  if (n_faults > c->fault_cap) return gfail(c, FTGEMM_EINVAL, "too many faults (limit 65536)");
  const ftgemm_config& e = c->cfg;
  const bool ft = e.ft_mode != FTGEMM_FT_OFF;
  const bool tr = e.fold_tokens != 0;
  if (ft && !tr && c->encoded_w != w) return gfail(c, FTGEMM_ESTATE, "ftgemm_encode_weights has not been called for this weight matrix");
  hipStream_t st = (hipStream_t)hip_stream;
  GHIP_TRY(c, hipSetDevice(e.device));
  for (int i = 0; i < n_faults; ++i) {
    const ftgemm_fault& f = faults[i];
    if (f.row < 0 || f.row >= e.m || f.col < 0 || f.col >= e.n || f.bit < 0 || f.bit > 31) {
      char msg[128];
      snprintf(msg, sizeof msg, "fault %d (row=%d col=%d bit=%d) is outside the matrix", i, f.row, f.col, f.bit);
      return gfail(c, FTGEMM_EINVAL, msg);
    }
    c->h_faults[i] = tr ? GFault{f.col, f.row, f.bit} : GFault{f.row, f.col, f.bit};
  }
  if (n_faults > 0) {
    GHIP_TRY(c, hipMemcpyAsync(c->d_faults, c->h_faults, sizeof(GFault) * n_faults, hipMemcpyHostToDevice, st));
    GHIP_TRY(c, hipStreamSynchronize(st));   // the staging buffer may be rewritten by the next call
  }
  ftgemm_reset<<<1, 64, 0, st>>>(c->d_ev_count, c->d_resmax);

  if (ft && tr) {
    // tensor checksums of this call's token rows (eq. (13), (14) on x)
    dim3 grid(c->Tn, (e.k / 8 + 31) / 32);
    if (e.in_dtype == FTGEMM_BF16) ftgemm_encode_w<true><<<grid, 256, 0, st>>>(reinterpret_cast<const uint16_t*>(x), c->wc, e.m, e.k);
    else ftgemm_encode_w<false><<<grid, 256, 0, st>>>(reinterpret_cast<const uint16_t*>(x), c->wc, e.m, e.k);
    GHIP_TRY(c, hipGetLastError());
  }
  GArgs a;
  a.x = reinterpret_cast<const uint16_t*>(tr ? w : x);
  a.w = reinterpret_cast<const uint16_t*>(tr ? x : w);
  a.wc = c->wc;
  a.y = y; a.out_dtype = e.out_dtype;
  a.M = tr ? e.n : e.m; a.N = tr ? e.m : e.n; a.K = e.k; a.Tm = c->Tm; a.Tn = c->Tn;
  a.transposed = tr ? 1 : 0;
  a.bs_x = a.bs_w = a.bs_wc = a.bs_y_bytes = a.bs_events = 0;
  a.skip_upper = 0; a.k_lower = 0;
  a.tau_rel = e.tau_rel; a.tau_abs = e.tau_abs;
  a.correct = e.ft_mode == FTGEMM_FT_CORRECT ? 1 : 0;
  a.faults = c->d_faults; a.n_faults = n_faults;
  a.events = c->d_events; a.ev_count = c->d_ev_count; a.max_events = e.max_events;
  a.resmax = c->d_resmax;
  gemm_fn f = select_gemm(ft, n_faults > 0, e.in_dtype == FTGEMM_BF16, e.k % GBK != 0);
  if (c->timing) GHIP_TRY(c, hipEventRecord(c->ev[0], st));
  hipLaunchKernelGGL(f, dim3(c->Tm * c->Tn), dim3(GWAVES * 64), gemm_lds(ft), st, a);
  GHIP_TRY(c, hipGetLastError());
  if (c->timing) GHIP_TRY(c, hipEventRecord(c->ev[1], st));
  c->last_stream = st;
  c->ran = true;
  return FTGEMM_OK;
}

extern "C" int ftgemm_report(ftgemm_ctx* c, ftgemm_report_view* out) {
  if (!c || !out) return FTGEMM_EINVAL;
  if (!c->ran) return gfail(c, FTGEMM_EINVAL, "no forward call to report on");
  const ftgemm_config& e = c->cfg;
  GHIP_TRY(c, hipSetDevice(e.device));
  GHIP_TRY(c, hipStreamSynchronize(c->last_stream));
  int32_t count = 0;
  uint32_t rm = 0;
  GHIP_TRY(c, hipMemcpy(&count, c->d_ev_count, sizeof count, hipMemcpyDeviceToHost));
  GHIP_TRY(c, hipMemcpy(&rm, c->d_resmax, sizeof rm, hipMemcpyDeviceToHost));
  const int stored = std::min(count, e.max_events);
  c->events.resize(stored);
  if (stored) GHIP_TRY(c, hipMemcpy(c->events.data(), c->d_events, sizeof(ftgemm_event) * stored, hipMemcpyDeviceToHost));
  std::sort(c->events.begin(), c->events.end(), [](const ftgemm_event& p, const ftgemm_event& q) {
    if (p.row != q.row) return p.row < q.row;
    return p.col < q.col;
  });
  out->n_events = stored;
  out->n_events_dropped = count - stored;
  out->events = c->events.data();
  float rmf;
  std::memcpy(&rmf, &rm, sizeof rmf);
  out->residual_max = rmf;
  return FTGEMM_OK;
}

extern "C" int ftgemm_set_timing(ftgemm_ctx* c, int32_t enabled) {
  if (!c) return FTGEMM_EINVAL;
  GHIP_TRY(c, hipSetDevice(c->cfg.device));
  if (enabled)
    for (hipEvent_t& e : c->ev)
      if (!e) GHIP_TRY(c, hipEventCreate(&e));
  c->timing = enabled != 0;
  return FTGEMM_OK;
}

extern "C" int ftgemm_get_timing(ftgemm_ctx* c, float* ms) {
  if (!c || !ms) return FTGEMM_EINVAL;
  if (!c->timing || !c->ran) return gfail(c, FTGEMM_EINVAL, "timing is not enabled or no forward has run");
  GHIP_TRY(c, hipSetDevice(c->cfg.device));
  GHIP_TRY(c, hipEventSynchronize(c->ev[1]));
  GHIP_TRY(c, hipEventElapsedTime(ms, c->ev[0], c->ev[1]));
  return FTGEMM_OK;
}

extern "C" int ftgemm_destroy(ftgemm_ctx* c) {
  if (!c) return FTGEMM_EINVAL;
  (void)hipSetDevice(c->cfg.device);
  (void)hipDeviceSynchronize();
  grelease(c);
  return FTGEMM_OK;
}

extern "C" const char* ftgemm_last_error(const ftgemm_ctx* c) {
  return c ? c->err.c_str() : g_gemm_create_err.c_str();
}
