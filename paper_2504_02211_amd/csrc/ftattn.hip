// Host side of the fault-tolerant fused attention library: the C ABI of include/ftattn.h.
// Validation, fault bucketing, launches and the report are here; every arithmetic step of
// the attention pass runs in the kernels of ftattn_device.h.
#include "ftattn_main.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace ftattn;

// Shape-derived sizes of one configuration: tiles per head and the element counts of the encoded
// key / value tiles.
struct Geometry { int BH = 0, Ti = 0, Tj = 0, BM = 0; size_t n_kc = 0, n_vt = 0; };

// Device buffers one pass works on (owned by a context, or carved out of the static scratch array).
struct Buffers {
  _Float16* kc = nullptr;
  _Float16* vt = nullptr;
  const DevFault* faults = nullptr;
  const int32_t* fault_off = nullptr;
  ftattn_event* events = nullptr;
  int32_t* ev_count = nullptr;
  unsigned long long* recheck = nullptr;
  uint32_t* resmax = nullptr;
  uint32_t* range = nullptr;          // the word this call sets
  uint32_t* range_next = nullptr;     // the word the next call sets: cleared by this call
};

struct ftattn_ctx {
  ftattn_config cfg;          // effective configuration
  Geometry geo;
  // device scratch
  _Float16* kc = nullptr;
  _Float16* vt = nullptr;
  DevFault* d_faults = nullptr;
  int32_t* d_fault_off = nullptr;
  ftattn_event* d_events = nullptr;
  int32_t* d_ev_count = nullptr;
  unsigned long long* d_recheck = nullptr;
  uint32_t* d_resmax = nullptr;
  uint32_t* d_range = nullptr;        // two words, used in turn by consecutive calls
  unsigned calls = 0;
  int fault_cap = 0;
  // pinned host staging
  DevFault* h_faults = nullptr;
  int32_t* h_fault_off = nullptr;
  // report storage
  std::vector<ftattn_event> events;
  std::vector<uint8_t> tile_flags, rowtile_flags;
  std::vector<float> resmax;
  hipStream_t last_stream = nullptr;
  bool ran = false;
  bool timing = false;
  hipEvent_t ev[3] = {nullptr, nullptr, nullptr};   // before encode, before fused kernel, after
  std::string err;
};

static thread_local std::string g_create_err;

static int fail(ftattn_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_create_err = msg;
  return code;
}

#define HIP_TRY(ctx, expr)                                                                      \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess)                                                                       \
      return fail(ctx, e_ == hipErrorOutOfMemory ? FTATTN_ENOMEM : FTATTN_EHIP,                 \
                  std::string(#expr) + ": " + hipGetErrorString(e_));                           \
  } while (0)

static void release(ftattn_ctx* c) {
  if (!c) return;
  (void)hipFree(c->kc); (void)hipFree(c->vt); (void)hipFree(c->d_faults);
  (void)hipFree(c->d_fault_off); (void)hipFree(c->d_events); (void)hipFree(c->d_ev_count);
  (void)hipFree(c->d_recheck); (void)hipFree(c->d_resmax); (void)hipFree(c->d_range);
  if (c->h_faults) (void)hipHostFree(c->h_faults);
  if (c->h_fault_off) (void)hipHostFree(c->h_fault_off);
  for (hipEvent_t e : c->ev) if (e) (void)hipEventDestroy(e);
  delete c;
}

typedef void (*main_fn)(const KArgs);

template <int D, bool INJ>
static main_fn pick(bool ft, bool causal) {
  if (ft) return causal ? ftattn_main<D, true, true, INJ> : ftattn_main<D, true, false, INJ>;
  return causal ? ftattn_main<D, false, true, INJ> : ftattn_main<D, false, false, INJ>;
}

// inject: the variant that carries the fault-injection code; calls without a fault list run the
// variant that has none of it
// the ablation modes are instantiated in translation units of their own (ftattn_perstep.hip,
// ftattn_elementwide.hip), so that all of them compile side by side
namespace ftattn {
void (*select_perstep(int D, bool causal, bool inject, int mode))(const KArgs);
void (*select_elementwide(int D, bool causal, bool inject))(const KArgs);
void (*select_lazy(int D, bool ft, bool causal, bool inject))(const KArgs);
}

static main_fn select_kernel(int D, bool ft, bool causal, bool inject) {
  if (D == 128) return inject ? pick<128, true>(ft, causal) : pick<128, false>(ft, causal);
  if (D == 64) return inject ? pick<64, true>(ft, causal) : pick<64, false>(ft, causal);
  return nullptr;
}

static size_t lds_bytes(int D, bool ft) {
  if (D == 128) return ft ? Unit<128, true>::LDS_TOTAL : Unit<128, false>::LDS_TOTAL;
  return ft ? Unit<64, true>::LDS_TOTAL : Unit<64, false>::LDS_TOTAL;
}

// Checks cfg and resolves its defaults into e (tile sizes, thresholds, scale) and g.  Touches no
// device.  On failure returns the error code and points `why` at a constant message.
static int resolve_config(const ftattn_config* cfg, ftattn_config& e, Geometry& g, const char*& why) {
  why = "";
  if (cfg->struct_size != sizeof(ftattn_config)) { why = "struct_size mismatch"; return FTATTN_EINVAL; }
  if (cfg->batch < 1 || cfg->heads < 1 || cfg->seq < 1) { why = "batch, heads, seq must be >= 1"; return FTATTN_EINVAL; }
  if ((long long)cfg->batch * cfg->heads > 65535) { why = "batch*heads > 65535"; return FTATTN_EUNSUPPORTED; }
  if (cfg->head_dim != 64 && cfg->head_dim != 128) { why = "head_dim must be 64 or 128"; return FTATTN_EUNSUPPORTED; }
  if (cfg->in_dtype != FTATTN_F16 && cfg->in_dtype != FTATTN_BF16) { why = "in_dtype must be F16 or BF16"; return FTATTN_EINVAL; }
  if (cfg->out_dtype != FTATTN_F32 && cfg->out_dtype != cfg->in_dtype) { why = "out_dtype must be F32 or the input type"; return FTATTN_EINVAL; }
  if (cfg->ft_mode < 0 || cfg->ft_mode > 2) { why = "ft_mode out of range"; return FTATTN_EINVAL; }
  if (cfg->stride != 0 && cfg->stride != 8 && cfg->stride != 1) { why = "stride must be 8 (or 1: the traditional checksum)"; return FTATTN_EUNSUPPORTED; }
  if (cfg->block_n != 0 && cfg->block_n != BN) { why = "block_n must be 64"; return FTATTN_EUNSUPPORTED; }
  if (cfg->block_m != 0 && cfg->block_m != bm_of(cfg->head_dim)) {
    why = "block_m must be 0 or the library's row tile (256 for head_dim 128, 128 for head_dim 64)";
    return FTATTN_EUNSUPPORTED;
  }
  if (cfg->causal != 0 && cfg->causal != 1) { why = "causal must be 0 or 1"; return FTATTN_EINVAL; }
  if (cfg->rowsum_fold != 0 && cfg->rowsum_fold != 1) { why = "rowsum_fold must be 0 or 1"; return FTATTN_EINVAL; }
  if (cfg->per_step < 0 || cfg->per_step > 2) { why = "per_step must be 0, 1 or 2"; return FTATTN_EINVAL; }
  if (cfg->per_step != 0 && (cfg->ft_mode != FTATTN_FT_CORRECT || cfg->rowsum_fold != 0)) {
    why = "per_step needs ft_mode FTATTN_FT_CORRECT and rowsum_fold 0";
    return FTATTN_EINVAL;
  }
  if (cfg->stride == 1 && (cfg->ft_mode == FTATTN_FT_OFF || cfg->rowsum_fold != 0 || cfg->per_step != 0)) {
    why = "stride 1 needs a protected ft_mode, rowsum_fold 0 and per_step 0";
    return FTATTN_EINVAL;
  }
  if (cfg->rescale_margin > 0.f && (cfg->per_step != 0 || cfg->stride == 1 || cfg->rowsum_fold != 0)) {
    why = "rescale_margin needs per_step 0, stride 8 and rowsum_fold 0";
    return FTATTN_EINVAL;
  }
  if (cfg->rescale_margin > 8.f) { why = "rescale_margin must be at most 8 (the exponentials are held in fp16)"; return FTATTN_EINVAL; }
  e = *cfg;
  if (!(e.rescale_margin > 0.f)) e.rescale_margin = 0.f;
  e.stride = cfg->stride == 1 ? 1 : 8;
  e.block_n = BN;
  if (!(e.softmax_scale > 0.f)) e.softmax_scale = 1.0f / std::sqrt((float)e.head_dim);
  if (!(e.eps1 > 0.f)) e.eps1 = 0.03f;
  if (!(e.tau_o > 0.f)) e.tau_o = 0.75f / 512.0f;
  if (!(e.delta_l > 0.f)) e.delta_l = 1.0f / 1024.0f;
  if (e.max_events <= 0) e.max_events = 65536;
  e.block_m = bm_of(e.head_dim);
  g.BH = e.batch * e.heads;
  g.Tj = (e.seq + BN - 1) / BN;
  g.BM = e.block_m;
  g.Ti = (e.seq + g.BM - 1) / g.BM;
  g.n_kc = (size_t)g.BH * g.Tj * (BN + CKR) * e.head_dim;
  g.n_vt = (size_t)g.BH * g.Tj * (e.head_dim + CKR) * BN;
  return FTATTN_OK;
}

// Lets the kernels of one head size (and mode) use their dynamic LDS.  Needs the device current.
static hipError_t allow_lds(int D, int per_step, int stride, const char*& why, bool lazy = false) {
  why = "no kernel for this tile shape";
  for (int v = 0; v < 8; ++v) {
    const int ft = v & 1, ca = (v >> 1) & 1;
    main_fn f = select_kernel(D, ft != 0, ca != 0, (v >> 2) != 0);
    if (!f) return hipErrorInvalidValue;
    hipError_t he = hipFuncSetAttribute((const void*)f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes(D, ft != 0));
    if (he != hipSuccess) { why = "hipFuncSetAttribute"; return he; }
  }
  for (int v = 0; v < 8 && lazy; ++v) {
    const bool ft = (v & 1) != 0;
    main_fn f = select_lazy(D, ft, (v & 2) != 0, (v & 4) != 0);
    if (!f) return hipErrorInvalidValue;
    hipError_t he = hipFuncSetAttribute((const void*)f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes(D, ft));
    if (he != hipSuccess) { why = "hipFuncSetAttribute"; return he; }
  }
  for (int v = 0; v < 4 && (per_step || stride == 1); ++v) {
    main_fn f = per_step ? select_perstep(D, (v & 1) != 0, (v >> 1) != 0, per_step) : select_elementwide(D, (v & 1) != 0, (v >> 1) != 0);
    if (!f) return hipErrorInvalidValue;
    hipError_t he = hipFuncSetAttribute((const void*)f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes(D, true));
    if (he != hipSuccess) { why = "hipFuncSetAttribute"; return he; }
  }
  return hipSuccess;
}

extern "C" int ftattn_create(const ftattn_config* cfg, ftattn_ctx** out) {
  if (!cfg || !out) return fail(nullptr, FTATTN_EINVAL, "null argument");
  *out = nullptr;
  ftattn_config e;
  Geometry g;
  const char* why;
  if (int rc = resolve_config(cfg, e, g, why)) return fail(nullptr, rc, why);

  ftattn_ctx* c = new (std::nothrow) ftattn_ctx();
  if (!c) return fail(nullptr, FTATTN_ENOMEM, "out of host memory");
  c->cfg = e;
  c->geo = g;

  hipError_t he = hipSetDevice(e.device);
  if (he != hipSuccess) { int rc = fail(nullptr, FTATTN_EHIP, std::string("hipSetDevice: ") + hipGetErrorString(he)); delete c; return rc; }

  c->fault_cap = 1 << 16;
  const size_t n_rt = (size_t)g.BH * g.Ti;
#define CREATE_TRY(expr)                                                                                  \
  do {                                                                                                    \
    hipError_t e_ = (expr);                                                                               \
    if (e_ != hipSuccess) {                                                                               \
      int rc_ = fail(nullptr, e_ == hipErrorOutOfMemory ? FTATTN_ENOMEM : FTATTN_EHIP,                    \
                     std::string(#expr) + ": " + hipGetErrorString(e_));                                  \
      release(c);                                                                                         \
      return rc_;                                                                                         \
    }                                                                                                     \
  } while (0)
  CREATE_TRY(hipMalloc((void**)&c->kc, g.n_kc * 2));
  CREATE_TRY(hipMalloc((void**)&c->vt, g.n_vt * 2));
  CREATE_TRY(hipMalloc((void**)&c->d_faults, sizeof(DevFault) * c->fault_cap));
  CREATE_TRY(hipMalloc((void**)&c->d_fault_off, sizeof(int32_t) * (n_rt + 1)));
  CREATE_TRY(hipMalloc((void**)&c->d_events, sizeof(ftattn_event) * (size_t)e.max_events));
  CREATE_TRY(hipMalloc((void**)&c->d_ev_count, sizeof(int32_t)));
  CREATE_TRY(hipMalloc((void**)&c->d_recheck, sizeof(unsigned long long)));
  CREATE_TRY(hipMalloc((void**)&c->d_resmax, sizeof(uint32_t) * n_rt * 4));
  CREATE_TRY(hipMalloc((void**)&c->d_range, sizeof(uint32_t) * 2));
  CREATE_TRY(hipMemset(c->d_range, 0, sizeof(uint32_t) * 2));
  CREATE_TRY(hipHostMalloc((void**)&c->h_faults, sizeof(DevFault) * c->fault_cap, hipHostMallocDefault));
  CREATE_TRY(hipHostMalloc((void**)&c->h_fault_off, sizeof(int32_t) * (n_rt + 1), hipHostMallocDefault));
  // the checksum rows of the encoded tiles are never written when ft_mode is OFF; keep them defined
  CREATE_TRY(hipMemset(c->kc, 0, g.n_kc * 2));
  CREATE_TRY(hipMemset(c->vt, 0, g.n_vt * 2));
  CREATE_TRY(hipMemset(c->d_ev_count, 0, sizeof(int32_t)));
  CREATE_TRY(hipMemset(c->d_recheck, 0, sizeof(unsigned long long)));
  CREATE_TRY(hipMemset(c->d_resmax, 0, sizeof(uint32_t) * n_rt * 4));
  {
    hipError_t le = allow_lds(e.head_dim, e.per_step, e.stride, why, e.rescale_margin > 0.f);
    if (le != hipSuccess) {
      int rc = fail(nullptr, le == hipErrorInvalidValue ? FTATTN_EUNSUPPORTED : FTATTN_EHIP, std::string(why) + ": " + hipGetErrorString(le));
      release(c);
      return rc;
    }
  }
  CREATE_TRY(hipDeviceSynchronize());
#undef CREATE_TRY
  *out = c;
  return FTATTN_OK;
}

extern "C" int ftattn_get_config(const ftattn_ctx* ctx, ftattn_config* effective) {
  if (!ctx || !effective) return FTATTN_EINVAL;
  *effective = ctx->cfg;
  return FTATTN_OK;
}

// The two launches of one pass on `st`: encode (Algorithm 1: "Encode tensor checksum"), once per key
// tile for all row tiles, which also clears the counters of the report; then the fused pass.
// Allocates nothing.  `timing`: three events recorded before, between and after the launches, or null.
static hipError_t launch_pass(const ftattn_config& e, const Geometry& g, const Buffers& b, const void* q, const void* k,
                              const void* v, void* o, bool inject, hipStream_t st, hipEvent_t* timing) {
  const int D = e.head_dim, N = e.seq;
  const bool ft = e.ft_mode != FTATTN_FT_OFF;
  const int n_resmax = g.BH * g.Ti * 4;
  hipError_t he;
  if (timing && (he = hipEventRecord(timing[0], st)) != hipSuccess) return he;
  dim3 eg(g.Tj, g.BH, 2);
  const int bf = e.in_dtype == FTATTN_BF16 ? 1 : 0;
  const int kchk = ft ? 1 : 0, vchk = ft ? 1 + e.rowsum_fold : 0;
  if (D == 128)
    ftattn_prepare<128><<<eg, 256, 0, st>>>(k, v, bf, b.kc, b.vt, N, g.Tj, kchk, vchk, b.ev_count, b.recheck, b.resmax, n_resmax, b.range, b.range_next);
  else
    ftattn_prepare<64><<<eg, 256, 0, st>>>(k, v, bf, b.kc, b.vt, N, g.Tj, kchk, vchk, b.ev_count, b.recheck, b.resmax, n_resmax, b.range, b.range_next);

  KArgs a;
  a.q = q; a.q_bf16 = bf; a.kc = b.kc; a.vt = b.vt; a.o = o; a.out_dtype = e.out_dtype;
  a.N = N; a.H = e.heads; a.Ti = g.Ti; a.Tj = g.Tj;
  a.scale = e.softmax_scale;
  a.scale_log2 = e.softmax_scale * 1.4426950408889634f;
  a.eps1 = e.eps1;
  a.tau_fast = 0.5f * (1.0f - std::exp(-e.eps1));
  a.tau_o = e.tau_o; a.delta_l = e.delta_l;
  a.correct = e.ft_mode == FTATTN_FT_CORRECT ? 1 : 0;
  a.rowsum_fold = e.rowsum_fold;
  a.rescale_margin = e.rescale_margin;
  a.faults = b.faults;
  a.fault_off = inject ? b.fault_off : nullptr;
  a.events = b.events; a.ev_count = b.ev_count; a.max_events = e.max_events;
  a.resmax = b.resmax; a.recheck = b.recheck; a.range = b.range;
  main_fn f = e.per_step ? select_perstep(D, e.causal != 0, inject, e.per_step)
              : e.stride == 1 ? select_elementwide(D, e.causal != 0, inject)
              : e.rescale_margin > 0.f ? select_lazy(D, ft, e.causal != 0, inject)
                              : select_kernel(D, ft, e.causal != 0, inject);
  if (timing && (he = hipEventRecord(timing[1], st)) != hipSuccess) return he;
  hipLaunchKernelGGL(f, dim3(g.BH * g.Ti), dim3(nwave_of(D) * 64), lds_bytes(D, ft), st, a);
  if ((he = hipGetLastError()) != hipSuccess) return he;
  if (timing && (he = hipEventRecord(timing[2], st)) != hipSuccess) return he;
  return hipSuccess;
}

static int n_tiles_for_row(const ftattn_config& e, int row) {
  int last_key = e.causal ? row : e.seq - 1;
  return last_key / BN + 1;
}

extern "C" int ftattn_forward(ftattn_ctx* c, const void* q, const void* k, const void* v, void* o,
                              const ftattn_fault* faults, int32_t n_faults, void* hip_stream) {
  if (!c) return FTATTN_EINVAL;
  if (!q || !k || !v || !o) return fail(c, FTATTN_EINVAL, "null tensor pointer");
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return fail(c, FTATTN_EINVAL, "tensor pointers must be 16-byte aligned");
  if (n_faults < 0 || (n_faults > 0 && !faults)) return fail(c, FTATTN_EINVAL, "bad fault list");
  if (n_faults > c->fault_cap) return fail(c, FTATTN_EINVAL, "too many faults (limit 65536)");
  const ftattn_config& e = c->cfg;
  const int D = e.head_dim, N = e.seq;
  hipStream_t st = (hipStream_t)hip_stream;
  HIP_TRY(c, hipSetDevice(e.device));

  // ---- validate and bucket the fault list by (head, row tile), ordered by key tile
  if (n_faults > 0) {
    struct Keyed { long long key; DevFault f; };
    std::vector<Keyed> ks(n_faults);
    for (int i = 0; i < n_faults; ++i) {
      const ftattn_fault& f = faults[i];
      char msg[160];
      bool ok = f.b >= 0 && f.b < e.batch && f.h >= 0 && f.h < e.heads && f.row >= 0 && f.row < N && f.bit >= 0 && f.bit <= 31 &&
                f.stage >= FTATTN_ST_S && f.stage <= FTATTN_ST_OACC && f.kv_tile >= 0 && f.kv_tile < n_tiles_for_row(e, f.row);
      if (ok && (f.stage == FTATTN_ST_S || f.stage == FTATTN_ST_EXP))
        ok = f.col >= 0 && f.col < N && (!e.causal || f.col <= f.row) && f.kv_tile == f.col / BN;
      if (ok && f.stage == FTATTN_ST_OACC) ok = f.col >= 0 && f.col < D;
      if (!ok) {
        snprintf(msg, sizeof msg, "fault %d (b=%d h=%d stage=%d kv_tile=%d row=%d col=%d bit=%d) names a masked or out-of-range position",
                 i, f.b, f.h, f.stage, f.kv_tile, f.row, f.col, f.bit);
        return fail(c, FTATTN_EINVAL, msg);
      }
      long long bucket = (long long)(f.b * e.heads + f.h) * c->geo.Ti + f.row / c->geo.BM;
      ks[i].key = (bucket << 32) | ((long long)f.kv_tile << 8) | f.stage;
      ks[i].f = DevFault{f.stage, f.kv_tile, f.row, f.col, f.bit};
    }
    std::stable_sort(ks.begin(), ks.end(), [](const Keyed& a, const Keyed& b) { return a.key < b.key; });
    size_t nb = (size_t)c->geo.BH * c->geo.Ti;
    std::fill(c->h_fault_off, c->h_fault_off + nb + 1, 0);
    for (int i = 0; i < n_faults; ++i) { c->h_faults[i] = ks[i].f; c->h_fault_off[(ks[i].key >> 32) + 1]++; }
    for (size_t i = 0; i < nb; ++i) c->h_fault_off[i + 1] += c->h_fault_off[i];
    HIP_TRY(c, hipMemcpyAsync(c->d_faults, c->h_faults, sizeof(DevFault) * n_faults, hipMemcpyHostToDevice, st));
    HIP_TRY(c, hipMemcpyAsync(c->d_fault_off, c->h_fault_off, sizeof(int32_t) * (nb + 1), hipMemcpyHostToDevice, st));
    HIP_TRY(c, hipStreamSynchronize(st));   // the staging buffers may be rewritten by the next call
  }

  Buffers bufs;
  bufs.kc = c->kc; bufs.vt = c->vt; bufs.faults = c->d_faults; bufs.fault_off = n_faults > 0 ? c->d_fault_off : nullptr;
  bufs.events = c->d_events; bufs.ev_count = c->d_ev_count; bufs.recheck = c->d_recheck; bufs.resmax = c->d_resmax;
  bufs.range = c->d_range + (c->calls & 1u); bufs.range_next = c->d_range + ((c->calls + 1u) & 1u);
  hipError_t le = launch_pass(e, c->geo, bufs, q, k, v, o, n_faults > 0, st, c->timing ? c->ev : nullptr);
  if (le != hipSuccess) return fail(c, FTATTN_EHIP, std::string("launch: ") + hipGetErrorString(le));
  c->last_stream = st;
  c->ran = true;
  ++c->calls;
  return FTATTN_OK;
}

extern "C" int ftattn_report(ftattn_ctx* c, ftattn_report_view* out) {
  if (!c || !out) return FTATTN_EINVAL;
  if (!c->ran) return fail(c, FTATTN_EINVAL, "no forward call to report on");
  const ftattn_config& e = c->cfg;
  HIP_TRY(c, hipSetDevice(e.device));
  HIP_TRY(c, hipStreamSynchronize(c->last_stream));
  int32_t count = 0;
  unsigned long long recheck = 0;
  HIP_TRY(c, hipMemcpy(&count, c->d_ev_count, sizeof count, hipMemcpyDeviceToHost));
  HIP_TRY(c, hipMemcpy(&recheck, c->d_recheck, sizeof recheck, hipMemcpyDeviceToHost));
  int stored = std::min(count, e.max_events);
  c->events.resize(stored);
  if (stored) HIP_TRY(c, hipMemcpy(c->events.data(), c->d_events, sizeof(ftattn_event) * stored, hipMemcpyDeviceToHost));
  std::sort(c->events.begin(), c->events.end(), [](const ftattn_event& x, const ftattn_event& y) {
    if (x.b != y.b) return x.b < y.b;
    if (x.h != y.h) return x.h < y.h;
    if (x.check != y.check) return x.check < y.check;
    if (x.kv_tile != y.kv_tile) return x.kv_tile < y.kv_tile;
    if (x.row != y.row) return x.row < y.row;
    return x.col < y.col;
  });
  size_t n_rt = (size_t)c->geo.BH * c->geo.Ti;
  c->tile_flags.assign(n_rt * c->geo.Tj, 0);
  c->rowtile_flags.assign(n_rt, 0);
  for (const ftattn_event& ev : c->events) {
    size_t rt = (size_t)(ev.b * e.heads + ev.h) * c->geo.Ti + ev.row / c->geo.BM;
    if (ev.check == FTATTN_CHECK_S) c->tile_flags[rt * c->geo.Tj + ev.kv_tile] |= FTATTN_TF_DET_S | (ev.action ? FTATTN_TF_COR_S : 0);
    else if (ev.check == FTATTN_CHECK_EXP) c->tile_flags[rt * c->geo.Tj + ev.kv_tile] |= FTATTN_TF_DET_EXP | (ev.action ? FTATTN_TF_COR_EXP : 0);
    else if (ev.check == FTATTN_CHECK_L) c->rowtile_flags[rt] |= FTATTN_RF_DET_L | (ev.action ? FTATTN_RF_COR_L : 0);
    else c->rowtile_flags[rt] |= FTATTN_RF_DET_O | (ev.action ? FTATTN_RF_COR_O : 0);
  }
  if (count > stored)
    for (auto& f : c->rowtile_flags) f |= FTATTN_RF_EVENT_OVERFLOW;
  c->resmax.resize(n_rt * 4);
  HIP_TRY(c, hipMemcpy(c->resmax.data(), c->d_resmax, sizeof(float) * n_rt * 4, hipMemcpyDeviceToHost));
  out->n_events = stored;
  out->n_events_dropped = count - stored;
  out->events = c->events.data();
  out->tiles_m = c->geo.Ti;
  out->tiles_n = c->geo.Tj;
  out->tile_flags = c->tile_flags.data();
  out->rowtile_flags = c->rowtile_flags.data();
  out->residual_max = c->resmax.data();
  out->recheck_entries = (int64_t)recheck;
  uint32_t range = 0;
  HIP_TRY(c, hipMemcpy(&range, c->d_range + ((c->calls - 1u) & 1u), sizeof range, hipMemcpyDeviceToHost));
  out->range_flags = (int32_t)range;
  return FTATTN_OK;
}

extern "C" int ftattn_set_timing(ftattn_ctx* c, int32_t enabled) {
  if (!c) return FTATTN_EINVAL;
  HIP_TRY(c, hipSetDevice(c->cfg.device));
  if (enabled)
    for (hipEvent_t& e : c->ev)
      if (!e) HIP_TRY(c, hipEventCreate(&e));
  c->timing = enabled != 0;
  return FTATTN_OK;
}

extern "C" int ftattn_get_timing(ftattn_ctx* c, float ms[2]) {
  if (!c || !ms) return FTATTN_EINVAL;
  if (!c->timing || !c->ran) return fail(c, FTATTN_EINVAL, "timing is not enabled or no forward has run");
  HIP_TRY(c, hipSetDevice(c->cfg.device));
  HIP_TRY(c, hipEventSynchronize(c->ev[2]));
  HIP_TRY(c, hipEventElapsedTime(&ms[0], c->ev[0], c->ev[1]));
  HIP_TRY(c, hipEventElapsedTime(&ms[1], c->ev[1], c->ev[2]));
  return FTATTN_OK;
}

extern "C" int ftattn_destroy(ftattn_ctx* c) {
  if (!c) return FTATTN_EINVAL;
  (void)hipSetDevice(c->cfg.device);
  (void)hipDeviceSynchronize();
  release(c);
  return FTATTN_OK;
}

extern "C" const char* ftattn_last_error(const ftattn_ctx* c) {
  return c ? c->err.c_str() : g_create_err.c_str();
}

// ------------------------------------------------------------------ the entry point that allocates nothing
//
// Same pass, same kernels, with every device buffer carved out of one file-scope device array
// instead of a context's allocations.  The array exists once per GPU for the life of the process;
// the address a kernel may use is the one hipGetSymbolAddress returns for the current device (the
// array's name is only a host-side handle).

constexpr size_t STATIC_SCRATCH_BYTES = (size_t)FTATTN_STATIC_SCRATCH_MIB << 20;
constexpr int STATIC_MAX_EVENTS = 4096;
constexpr int STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

static std::mutex g_static_mu;
static unsigned char* g_static_ptr[STATIC_MAX_DEVICES];      // per device, null until set up
static bool g_static_lds[STATIC_MAX_DEVICES][2];             // kernels of head_dim 64 / 128 prepared
static unsigned g_static_calls[STATIC_MAX_DEVICES];          // parity picks the range word of a call
static thread_local char g_static_err[256];

static int static_fail(int code, const char* what, hipError_t he = hipSuccess) {
  if (he != hipSuccess) snprintf(g_static_err, sizeof g_static_err, "%s: %s", what, hipGetErrorString(he));
  else snprintf(g_static_err, sizeof g_static_err, "%s", what);
  return code;
}

extern "C" const char* ftattn_static_last_error(void) { return g_static_err; }

extern "C" int ftattn_forward_static(const ftattn_config* cfg, const void* q, const void* k, const void* v, void* o,
                                     int32_t* n_events_dev, void* hip_stream) {
  g_static_err[0] = 0;
  if (!cfg) return static_fail(FTATTN_EINVAL, "null configuration");
  ftattn_config e;
  Geometry g;
  const char* why;
  if (int rc = resolve_config(cfg, e, g, why)) return static_fail(rc, why);
  if (e.per_step != 0 || e.stride != 8 || e.rescale_margin > 0.f)
    return static_fail(FTATTN_EUNSUPPORTED, "the static entry point runs the default verification scheme (per_step 0, stride 8, rescale_margin 0)");
  if (e.device < 0 || e.device >= STATIC_MAX_DEVICES) return static_fail(FTATTN_EINVAL, "device ordinal out of range");
  if (!q || !k || !v || !o) return static_fail(FTATTN_EINVAL, "null tensor pointer");
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return static_fail(FTATTN_EINVAL, "tensor pointers must be 16-byte aligned");
  if ((uintptr_t)n_events_dev & 3) return static_fail(FTATTN_EINVAL, "n_events_dev must be 4-byte aligned");
  if (e.max_events > STATIC_MAX_EVENTS) e.max_events = STATIC_MAX_EVENTS;

  // layout of the array: counters | residual maxima | event log | encoded key tiles | encoded value tiles
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  const size_t off_resmax = 256;
  const size_t off_events = off_resmax + up(sizeof(uint32_t) * (size_t)g.BH * g.Ti * 4);
  const size_t off_kc = off_events + up(sizeof(ftattn_event) * (size_t)e.max_events);
  const size_t off_vt = off_kc + up(g.n_kc * 2);
  const size_t need = off_vt + up(g.n_vt * 2);
  if (need > STATIC_SCRATCH_BYTES) {
    snprintf(g_static_err, sizeof g_static_err, "this shape needs %zu bytes of scratch, the static array holds %zu", need, STATIC_SCRATCH_BYTES);
    return FTATTN_EUNSUPPORTED;
  }

  hipError_t he = hipSetDevice(e.device);
  if (he != hipSuccess) return static_fail(FTATTN_EHIP, "hipSetDevice", he);
  unsigned char* base;
  unsigned calls;
  {
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[e.device]) {
      void* ptr = nullptr;
      he = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (he != hipSuccess || !ptr) return static_fail(FTATTN_EHIP, "hipGetSymbolAddress(scratch)", he);
      g_static_ptr[e.device] = (unsigned char*)ptr;
    }
    const int di = e.head_dim == 128 ? 1 : 0;
    if (!g_static_lds[e.device][di]) {
      he = allow_lds(e.head_dim, 0, 8, why);
      if (he != hipSuccess) return static_fail(FTATTN_EHIP, why, he);
      g_static_lds[e.device][di] = true;
    }
    base = g_static_ptr[e.device];
    calls = g_static_calls[e.device]++;
  }

  Buffers bufs;
  bufs.ev_count = n_events_dev ? n_events_dev : (int32_t*)base;
  bufs.recheck = (unsigned long long*)(base + 8);
  bufs.range = (uint32_t*)(base + 16) + (calls & 1u);
  bufs.range_next = (uint32_t*)(base + 16) + ((calls + 1u) & 1u);
  bufs.resmax = (uint32_t*)(base + off_resmax);
  bufs.events = (ftattn_event*)(base + off_events);
  bufs.kc = (_Float16*)(base + off_kc);
  bufs.vt = (_Float16*)(base + off_vt);
  he = launch_pass(e, g, bufs, q, k, v, o, false, (hipStream_t)hip_stream, nullptr);
  if (he != hipSuccess) return static_fail(FTATTN_EHIP, "launch", he);
  return FTATTN_OK;
}
