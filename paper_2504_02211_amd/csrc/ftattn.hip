// Host side of the fault-tolerant fused attention library: the C ABI of include/ftattn.h.
// Validation, fault bucketing, launches and the report are here; every arithmetic step of
// the attention pass runs in the kernels of ftattn_device.h.
#include "ftattn_main.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

using namespace ftattn;

struct ftattn_ctx {
  ftattn_config cfg;          // effective configuration
  int BH, Ti, Tj, BM;
  // device scratch
  _Float16* kc = nullptr;
  _Float16* vt = nullptr;
  DevFault* d_faults = nullptr;
  int32_t* d_fault_off = nullptr;
  ftattn_event* d_events = nullptr;
  int32_t* d_ev_count = nullptr;
  unsigned long long* d_recheck = nullptr;
  uint32_t* d_resmax = nullptr;
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
  (void)hipFree(c->d_recheck); (void)hipFree(c->d_resmax);
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

extern "C" int ftattn_create(const ftattn_config* cfg, ftattn_ctx** out) {
  if (!cfg || !out) return fail(nullptr, FTATTN_EINVAL, "null argument");
  *out = nullptr;
  if (cfg->struct_size != sizeof(ftattn_config)) return fail(nullptr, FTATTN_EINVAL, "struct_size mismatch");
  if (cfg->batch < 1 || cfg->heads < 1 || cfg->seq < 1) return fail(nullptr, FTATTN_EINVAL, "batch, heads, seq must be >= 1");
  if ((long long)cfg->batch * cfg->heads > 65535) return fail(nullptr, FTATTN_EUNSUPPORTED, "batch*heads > 65535");
  if (cfg->head_dim != 64 && cfg->head_dim != 128) return fail(nullptr, FTATTN_EUNSUPPORTED, "head_dim must be 64 or 128");
  if (cfg->in_dtype != FTATTN_F16 && cfg->in_dtype != FTATTN_BF16) return fail(nullptr, FTATTN_EINVAL, "in_dtype must be F16 or BF16");
  if (cfg->out_dtype != FTATTN_F32 && cfg->out_dtype != cfg->in_dtype) return fail(nullptr, FTATTN_EINVAL, "out_dtype must be F32 or the input type");
  if (cfg->ft_mode < 0 || cfg->ft_mode > 2) return fail(nullptr, FTATTN_EINVAL, "ft_mode out of range");
  if (cfg->stride != 0 && cfg->stride != 8 && cfg->stride != 1) return fail(nullptr, FTATTN_EUNSUPPORTED, "stride must be 8 (or 1: the traditional checksum)");
  if (cfg->block_n != 0 && cfg->block_n != BN) return fail(nullptr, FTATTN_EUNSUPPORTED, "block_n must be 64");
  if (cfg->block_m != 0 && cfg->block_m != bm_of(cfg->head_dim))
    return fail(nullptr, FTATTN_EUNSUPPORTED, "block_m must be 0 or the library's row tile (256 for head_dim 128, 128 for head_dim 64)");
  if (cfg->causal != 0 && cfg->causal != 1) return fail(nullptr, FTATTN_EINVAL, "causal must be 0 or 1");
  if (cfg->rowsum_fold != 0 && cfg->rowsum_fold != 1) return fail(nullptr, FTATTN_EINVAL, "rowsum_fold must be 0 or 1");
  if (cfg->per_step < 0 || cfg->per_step > 2) return fail(nullptr, FTATTN_EINVAL, "per_step must be 0, 1 or 2");
  if (cfg->per_step != 0 && (cfg->ft_mode != FTATTN_FT_CORRECT || cfg->rowsum_fold != 0))
    return fail(nullptr, FTATTN_EINVAL, "per_step needs ft_mode FTATTN_FT_CORRECT and rowsum_fold 0");
  if (cfg->stride == 1 && (cfg->ft_mode == FTATTN_FT_OFF || cfg->rowsum_fold != 0 || cfg->per_step != 0))
    return fail(nullptr, FTATTN_EINVAL, "stride 1 needs a protected ft_mode, rowsum_fold 0 and per_step 0");

  ftattn_ctx* c = new (std::nothrow) ftattn_ctx();
  if (!c) return fail(nullptr, FTATTN_ENOMEM, "out of host memory");
  c->cfg = *cfg;
  ftattn_config& e = c->cfg;
  e.stride = cfg->stride == 1 ? 1 : 8;
  e.block_n = BN;
  if (!(e.softmax_scale > 0.f)) e.softmax_scale = 1.0f / std::sqrt((float)e.head_dim);
  if (!(e.eps1 > 0.f)) e.eps1 = 0.03f;
  if (!(e.tau_o > 0.f)) e.tau_o = 0.75f / 512.0f;
  if (!(e.delta_l > 0.f)) e.delta_l = 1.0f / 1024.0f;
  if (e.max_events <= 0) e.max_events = 65536;
  c->BH = e.batch * e.heads;
  c->Tj = (e.seq + BN - 1) / BN;
  e.block_m = bm_of(e.head_dim);
  c->BM = e.block_m;
  c->Ti = (e.seq + c->BM - 1) / c->BM;

  hipError_t he = hipSetDevice(e.device);
  if (he != hipSuccess) { int rc = fail(nullptr, FTATTN_EHIP, std::string("hipSetDevice: ") + hipGetErrorString(he)); delete c; return rc; }

  const int D = e.head_dim;
  size_t n_kc = (size_t)c->BH * c->Tj * (BN + CKR) * D;
  size_t n_vt = (size_t)c->BH * c->Tj * (D + CKR) * BN;
  c->fault_cap = 1 << 16;
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
  CREATE_TRY(hipMalloc((void**)&c->kc, n_kc * 2));
  CREATE_TRY(hipMalloc((void**)&c->vt, n_vt * 2));
  CREATE_TRY(hipMalloc((void**)&c->d_faults, sizeof(DevFault) * c->fault_cap));
  CREATE_TRY(hipMalloc((void**)&c->d_fault_off, sizeof(int32_t) * ((size_t)c->BH * c->Ti + 1)));
  CREATE_TRY(hipMalloc((void**)&c->d_events, sizeof(ftattn_event) * (size_t)e.max_events));
  CREATE_TRY(hipMalloc((void**)&c->d_ev_count, sizeof(int32_t)));
  CREATE_TRY(hipMalloc((void**)&c->d_recheck, sizeof(unsigned long long)));
  CREATE_TRY(hipMalloc((void**)&c->d_resmax, sizeof(uint32_t) * (size_t)c->BH * c->Ti * 4));
  CREATE_TRY(hipHostMalloc((void**)&c->h_faults, sizeof(DevFault) * c->fault_cap, hipHostMallocDefault));
  CREATE_TRY(hipHostMalloc((void**)&c->h_fault_off, sizeof(int32_t) * ((size_t)c->BH * c->Ti + 1), hipHostMallocDefault));
  // the checksum rows of the encoded tiles are never written when ft_mode is OFF; keep them defined
  CREATE_TRY(hipMemset(c->kc, 0, n_kc * 2));
  CREATE_TRY(hipMemset(c->vt, 0, n_vt * 2));
  CREATE_TRY(hipMemset(c->d_ev_count, 0, sizeof(int32_t)));
  CREATE_TRY(hipMemset(c->d_recheck, 0, sizeof(unsigned long long)));
  CREATE_TRY(hipMemset(c->d_resmax, 0, sizeof(uint32_t) * (size_t)c->BH * c->Ti * 4));
  for (int v = 0; v < 8; ++v) {
      const int ft = v & 1, ca = (v >> 1) & 1;
      main_fn f = select_kernel(D, ft != 0, ca != 0, (v >> 2) != 0);
      if (!f) { release(c); return fail(nullptr, FTATTN_EUNSUPPORTED, "no kernel for this tile shape"); }
      CREATE_TRY(hipFuncSetAttribute((const void*)f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes(D, ft != 0)));
    }
  if (e.per_step)
    for (int v = 0; v < 4; ++v) {
      main_fn f = select_perstep(D, (v & 1) != 0, (v >> 1) != 0, e.per_step);
      if (!f) { release(c); return fail(nullptr, FTATTN_EUNSUPPORTED, "no kernel for this tile shape"); }
      CREATE_TRY(hipFuncSetAttribute((const void*)f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes(D, true)));
    }
  if (e.stride == 1)
    for (int v = 0; v < 4; ++v) {
      main_fn f = select_elementwide(D, (v & 1) != 0, (v >> 1) != 0);
      if (!f) { release(c); return fail(nullptr, FTATTN_EUNSUPPORTED, "no kernel for this tile shape"); }
      CREATE_TRY(hipFuncSetAttribute((const void*)f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes(D, true)));
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
      long long bucket = (long long)(f.b * e.heads + f.h) * c->Ti + f.row / c->BM;
      ks[i].key = (bucket << 32) | ((long long)f.kv_tile << 8) | f.stage;
      ks[i].f = DevFault{f.stage, f.kv_tile, f.row, f.col, f.bit};
    }
    std::stable_sort(ks.begin(), ks.end(), [](const Keyed& a, const Keyed& b) { return a.key < b.key; });
    size_t nb = (size_t)c->BH * c->Ti;
    std::fill(c->h_fault_off, c->h_fault_off + nb + 1, 0);
    for (int i = 0; i < n_faults; ++i) { c->h_faults[i] = ks[i].f; c->h_fault_off[(ks[i].key >> 32) + 1]++; }
    for (size_t i = 0; i < nb; ++i) c->h_fault_off[i + 1] += c->h_fault_off[i];
    HIP_TRY(c, hipMemcpyAsync(c->d_faults, c->h_faults, sizeof(DevFault) * n_faults, hipMemcpyHostToDevice, st));
    HIP_TRY(c, hipMemcpyAsync(c->d_fault_off, c->h_fault_off, sizeof(int32_t) * (nb + 1), hipMemcpyHostToDevice, st));
    HIP_TRY(c, hipStreamSynchronize(st));   // the staging buffers may be rewritten by the next call
  }

  const bool ft = e.ft_mode != FTATTN_FT_OFF;
  int n_resmax = c->BH * c->Ti * 4;
  if (c->timing) HIP_TRY(c, hipEventRecord(c->ev[0], st));
  // ---- encode (Algorithm 1: "Encode tensor checksum"), once per key tile for all row tiles; the same
  // launch clears the counters of the report
  dim3 eg(c->Tj, c->BH, 2);
  const int bf = e.in_dtype == FTATTN_BF16 ? 1 : 0;
  const int kchk = ft ? 1 : 0, vchk = ft ? 1 + e.rowsum_fold : 0;
  if (D == 128)
    ftattn_prepare<128><<<eg, 256, 0, st>>>(k, v, bf, c->kc, c->vt, N, c->Tj, kchk, vchk, c->d_ev_count, c->d_recheck, c->d_resmax, n_resmax);
  else
    ftattn_prepare<64><<<eg, 256, 0, st>>>(k, v, bf, c->kc, c->vt, N, c->Tj, kchk, vchk, c->d_ev_count, c->d_recheck, c->d_resmax, n_resmax);

  // ---- the fused pass
  KArgs a;
  a.q = q; a.q_bf16 = bf; a.kc = c->kc; a.vt = c->vt; a.o = o; a.out_dtype = e.out_dtype;
  a.N = N; a.H = e.heads; a.Ti = c->Ti; a.Tj = c->Tj;
  a.scale = e.softmax_scale;
  a.scale_log2 = e.softmax_scale * 1.4426950408889634f;
  a.eps1 = e.eps1;
  a.tau_fast = 0.5f * (1.0f - std::exp(-e.eps1));
  a.tau_o = e.tau_o; a.delta_l = e.delta_l;
  a.correct = e.ft_mode == FTATTN_FT_CORRECT ? 1 : 0;
  a.rowsum_fold = e.rowsum_fold;
  a.faults = c->d_faults;
  a.fault_off = n_faults > 0 ? c->d_fault_off : nullptr;
  a.events = c->d_events; a.ev_count = c->d_ev_count; a.max_events = e.max_events;
  a.resmax = c->d_resmax; a.recheck = c->d_recheck;
  main_fn f = e.per_step ? select_perstep(D, e.causal != 0, n_faults > 0, e.per_step)
              : e.stride == 1 ? select_elementwide(D, e.causal != 0, n_faults > 0)
                              : select_kernel(D, ft, e.causal != 0, n_faults > 0);
  if (c->timing) HIP_TRY(c, hipEventRecord(c->ev[1], st));
  hipLaunchKernelGGL(f, dim3(c->BH * c->Ti), dim3(nwave_of(D) * 64), lds_bytes(D, ft), st, a);
  HIP_TRY(c, hipGetLastError());
  if (c->timing) HIP_TRY(c, hipEventRecord(c->ev[2], st));
  c->last_stream = st;
  c->ran = true;
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
  size_t n_rt = (size_t)c->BH * c->Ti;
  c->tile_flags.assign(n_rt * c->Tj, 0);
  c->rowtile_flags.assign(n_rt, 0);
  for (const ftattn_event& ev : c->events) {
    size_t rt = (size_t)(ev.b * e.heads + ev.h) * c->Ti + ev.row / c->BM;
    if (ev.check == FTATTN_CHECK_S) c->tile_flags[rt * c->Tj + ev.kv_tile] |= FTATTN_TF_DET_S | (ev.action ? FTATTN_TF_COR_S : 0);
    else if (ev.check == FTATTN_CHECK_EXP) c->tile_flags[rt * c->Tj + ev.kv_tile] |= FTATTN_TF_DET_EXP | (ev.action ? FTATTN_TF_COR_EXP : 0);
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
  out->tiles_m = c->Ti;
  out->tiles_n = c->Tj;
  out->tile_flags = c->tile_flags.data();
  out->rowtile_flags = c->rowtile_flags.data();
  out->residual_max = c->resmax.data();
  out->recheck_entries = (int64_t)recheck;
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
