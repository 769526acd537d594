// The decoupled, operation-level fault-tolerant attention of Section 3.1 (the comparison system of
// Section 4.1): ABFT-GEMM I -> DMR row-softmax -> ABFT-GEMM II, with S and P in device memory between
// the kernels.  The C ABI of include/ftdecoupled.h.  The two GEMMs are the library's strided-ABFT
// GEMM kernel (ftgemm_main.h) launched once per head on buffers of this context; the softmax kernel
// and the V^T kernel are here.
#include "ftdecoupled.h"
#include "ftgemm_main.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

namespace ftdec {

struct SFault { int32_t key, col, bit, stage; };   // key = bh * seq + row; sorted by key

struct SArgs {
  const float* S;          // [BH][N][N]
  _Float16* P;             // [BH][N][Np]
  int32_t N, Np, H, causal;
  float scale_log2, eps;
  int32_t use_lds;         // the row is staged in LDS (it fits), else re-read from memory
  const SFault* faults;
  int32_t n_faults;
  ftdec_event* events;
  int32_t* ev_count;
  int32_t max_events;
  unsigned long long* retried;
};

__device__ __forceinline__ float opaque(float x) { asm volatile("" : "+v"(x)); return x; }
__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float flip(float x, int bit) { return __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, x) ^ (1u << bit)); }

__device__ __forceinline__ void log_softmax_event(const SArgs& a, int bh, int stage, int row, int col) {
  const int idx = atomicAdd(a.ev_count, 1);
  if (idx < a.max_events) {
    ftdec_event e;
    e.b = bh / a.H; e.h = bh % a.H; e.stage = stage; e.row = row; e.col = col; e.action = 1;
    a.events[idx] = e;
  }
}

// block-wide reductions over 256 threads (4 waves); every thread gets the result
__device__ __forceinline__ float block_max(float v, float* red) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = __builtin_fmaxf(v, __shfl_xor(v, off));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return __builtin_fmaxf(__builtin_fmaxf(red[0], red[1]), __builtin_fmaxf(red[2], red[3]));
}
__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}
__device__ __forceinline__ int block_or(int v, int* red) {
  v = __builtin_amdgcn_ballot_w64(v != 0) != 0ull ? 1 : 0;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] | red[1] | red[2] | red[3];
}

// Row softmax by dual modular redundancy (eq. (11), (12)).  One workgroup per (row, head).
//   evaluation a, evaluation b: maximum and exponentials, the second on values the compiler cannot
//   merge with the first; |e_a - e_b| < eps element by element, DMR(e) = (e_a + e_b) / 2;
//   P = DMR(e) / rowsum(DMR(e)); |rowsum(P) - 1| < eps.
// A row that fails either test is evaluated again; injected faults hit the first attempt only (a
// soft error does not repeat).  FT == false: one evaluation, no test.
template <bool FT, bool INJ>
__global__ __launch_bounds__(256) void ftdec_softmax(const SArgs a) {
  extern __shared__ __attribute__((aligned(16))) float rowbuf[];
  __shared__ float red[4];
  __shared__ int redi[4];
  const int row = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
  const int N = a.N, nvalid = a.causal ? row + 1 : N;
  const float* src = a.S + ((size_t)bh * N + row) * N;
  _Float16* dst = a.P + ((size_t)bh * N + row) * a.Np;
  if (a.use_lds) {
    for (int j = tid; j < nvalid; j += 256) rowbuf[j] = src[j];
    __syncthreads();
    src = rowbuf;
  }
  // faults of this row: [f0, f1)
  int f0 = 0, f1 = 0;
  if (INJ) {
    const int key = bh * N + row;
    int lo = 0, hi = a.n_faults;
    while (lo < hi) { const int mid = (lo + hi) >> 1; if (a.faults[mid].key < key) lo = mid + 1; else hi = mid; }
    f0 = lo;
    while (lo < a.n_faults && a.faults[lo].key == key) ++lo;
    f1 = lo;
  }
  const float sl2 = a.scale_log2;
  for (int attempt = 0; attempt < 3; ++attempt) {
    // ---- maximum, twice
    float ma = -__builtin_inff(), mb = -__builtin_inff();
    for (int j = tid; j < nvalid; j += 256) {
      const float s = src[j];
      ma = __builtin_fmaxf(ma, s);
      if (FT) mb = __builtin_fmaxf(mb, opaque(s));
    }
    ma = block_max(ma, red);
    if (FT) mb = block_max(mb, red);
    const float na = -ma * sl2, nb = -mb * sl2;
    // ---- exponentials, twice; eq. (11)
    float sum = 0.f;
    int bad = 0;
    for (int j = tid; j < nvalid; j += 256) {
      const float s = src[j];
      float ea = ex2(__builtin_fmaf(s, sl2, na));
      if (INJ && attempt == 0)
        for (int f = f0; f < f1; ++f)
          if (a.faults[f].stage == FTDEC_ST_EXP && a.faults[f].col == j) ea = flip(ea, a.faults[f].bit);
      if (FT) {
        const float eb = ex2(__builtin_fmaf(opaque(s), sl2, nb));
        if (!(__builtin_fabsf(ea - eb) < a.eps)) {
          bad = 1;
          log_softmax_event(a, bh, FTDEC_ST_EXP, row, j);
        }
        sum += 0.5f * (ea + eb);
      } else {
        sum += ea;
      }
    }
    if (FT && block_or(bad, redi)) {
      if (tid == 0) atomicAdd(a.retried, 1ull);
      continue;
    }
    const float l = block_sum(sum, red);
    const float inv = 1.0f / l;
    // ---- normalised weights; eq. (12)
    float psum = 0.f;
    // (causal: GEMM II stops at the last query of the row's 256-query tile; the weights beyond are never read)
    const int jend = a.causal && (row / 256 + 1) * 256 < a.Np ? (row / 256 + 1) * 256 : a.Np;
    for (int j = tid; j < jend; j += 256) {
      float p = 0.f;
      if (j < nvalid) {
        const float s = src[j];
        float ea = ex2(__builtin_fmaf(s, sl2, na));
        if (INJ && attempt == 0)
          for (int f = f0; f < f1; ++f)
            if (a.faults[f].stage == FTDEC_ST_EXP && a.faults[f].col == j) ea = flip(ea, a.faults[f].bit);
        const float e = FT ? 0.5f * (ea + ex2(__builtin_fmaf(opaque(s), sl2, nb))) : ea;
        p = e * inv;
        if (INJ && attempt == 0)
          for (int f = f0; f < f1; ++f)
            if (a.faults[f].stage == FTDEC_ST_PNORM && a.faults[f].col == j) p = flip(p, a.faults[f].bit);
        psum += p;
      }
      dst[j] = (_Float16)p;
    }
    if (!FT) break;
    psum = block_sum(psum, red);
    if (__builtin_fabsf(psum - 1.0f) < a.eps) break;
    if (tid == 0) {
      log_softmax_event(a, bh, FTDEC_ST_PNORM, row, -1);
      atomicAdd(a.retried, 1ull);
    }
  }
}

// V [N][d] (fp16 or bf16 patterns) -> V^T [d][Np] in fp16, columns beyond N zero.  One workgroup per 64 keys.
__global__ __launch_bounds__(256) void ftdec_transpose_v(const uint16_t* __restrict__ v, _Float16* __restrict__ vt, int N, int Np,
                                                         int d, int bf16) {
  __shared__ _Float16 tile[64][257];
  const int bh = blockIdx.y, k0 = blockIdx.x * 64, tid = threadIdx.x;
  const uint16_t* src = v + (size_t)bh * N * d;
  _Float16* dst = vt + (size_t)bh * d * Np;
  for (int e = tid; e < 64 * d; e += 256) {
    const int r = e / d, f = e % d, key = k0 + r;
    float x = 0.f;
    if (key < N) {
      const uint16_t u = src[(size_t)key * d + f];
      x = bf16 ? __builtin_bit_cast(float, (uint32_t)u << 16) : (float)__builtin_bit_cast(_Float16, u);
    }
    tile[r][f] = (_Float16)x;
  }
  __syncthreads();
  for (int e = tid; e < 64 * d; e += 256) {
    const int f = e / 64, r = e % 64, key = k0 + r;
    if (key < Np) dst[(size_t)f * Np + key] = tile[r][f];
  }
}

__global__ void ftdec_reset(int32_t* counters, uint32_t* resmax, int n, unsigned long long* retried) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) { counters[i] = 0; resmax[i] = 0u; }
  if (i == 0) *retried = 0ull;
}

}  // namespace ftdec

using namespace ftdec;

struct ftdec_ctx {
  ftdec_config cfg;
  int BH = 0, N = 0, Np = 0, d = 0, Tm = 0, Tn1 = 0;
  // device
  float* S = nullptr;
  _Float16* P = nullptr;
  _Float16* vt = nullptr;
  uint16_t* wc1 = nullptr;       // [BH][Tn1][32][d]
  uint16_t* wc2 = nullptr;       // [BH][1][32][Np]
  ftgemm_event* g_events = nullptr;   // [2*BH][cap]
  int32_t* counters = nullptr;        // [2*BH] GEMM logs, [2*BH] the softmax log
  uint32_t* resmax = nullptr;         // [2*BH + 1]
  ftdec_event* s_events = nullptr;
  unsigned long long* retried = nullptr;
  ftgemm::GFault* d_gfaults = nullptr;
  SFault* d_sfaults = nullptr;
  ftgemm::GFault* h_gfaults = nullptr;   // pinned
  SFault* h_sfaults = nullptr;           // pinned
  int fault_cap = 0;
  int64_t bytes_total = 0, bytes_sp = 0;
  size_t softmax_lds = 0;
  std::vector<ftdec_event> events;
  std::vector<int32_t> h_counters;
  std::vector<ftgemm_event> h_gev;
  hipStream_t last_stream = nullptr;
  bool ran = false, timing = false;
  hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
  std::string err;
};

static thread_local std::string g_dec_err;
static int dfail(ftdec_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_dec_err = msg;
  return code;
}
#define DHIP_TRY(ctx, expr)                                                                     \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess)                                                                       \
      return dfail(ctx, e_ == hipErrorOutOfMemory ? FTDEC_ENOMEM : FTDEC_EHIP,                  \
                   std::string(#expr) + ": " + hipGetErrorString(e_));                          \
  } while (0)

static void drelease(ftdec_ctx* c) {
  if (!c) return;
  (void)hipFree(c->S); (void)hipFree(c->P); (void)hipFree(c->vt); (void)hipFree(c->wc1); (void)hipFree(c->wc2);
  (void)hipFree(c->g_events); (void)hipFree(c->counters); (void)hipFree(c->resmax); (void)hipFree(c->s_events);
  (void)hipFree(c->retried); (void)hipFree(c->d_gfaults); (void)hipFree(c->d_sfaults);
  if (c->h_gfaults) (void)hipHostFree(c->h_gfaults);
  if (c->h_sfaults) (void)hipHostFree(c->h_sfaults);
  for (hipEvent_t e : c->ev) if (e) (void)hipEventDestroy(e);
  delete c;
}

typedef void (*softmax_fn)(const SArgs);
static softmax_fn select_softmax(bool ft, bool inject) {
  if (ft) return inject ? ftdec_softmax<true, true> : ftdec_softmax<true, false>;
  return inject ? ftdec_softmax<false, true> : ftdec_softmax<false, false>;
}

extern "C" int ftdec_create(const ftdec_config* cfg, ftdec_ctx** out) {
  if (!cfg || !out) return dfail(nullptr, FTDEC_EINVAL, "null argument");
  *out = nullptr;
  if (cfg->struct_size != sizeof(ftdec_config)) return dfail(nullptr, FTDEC_EINVAL, "struct_size mismatch");
  if (cfg->batch < 1 || cfg->heads < 1 || cfg->seq < 1) return dfail(nullptr, FTDEC_EINVAL, "batch, heads, seq must be >= 1");
  if ((long long)cfg->batch * cfg->heads > 65535) return dfail(nullptr, FTDEC_EUNSUPPORTED, "batch*heads > 65535");
  if (cfg->head_dim < 8 || cfg->head_dim % 8 != 0 || cfg->head_dim > 256) return dfail(nullptr, FTDEC_EUNSUPPORTED, "head_dim must be a multiple of 8, at most 256");
  if (cfg->in_dtype != FTDEC_F16 && cfg->in_dtype != FTDEC_BF16) return dfail(nullptr, FTDEC_EINVAL, "in_dtype must be F16 or BF16");
  if (cfg->causal != 0 && cfg->causal != 1) return dfail(nullptr, FTDEC_EINVAL, "causal must be 0 or 1");
  if (cfg->ft_mode != FTDEC_FT_OFF && cfg->ft_mode != FTDEC_FT_CORRECT) return dfail(nullptr, FTDEC_EINVAL, "ft_mode must be OFF or CORRECT");
  if ((long long)cfg->batch * cfg->heads * cfg->seq > 0x7FFFFFFFll) return dfail(nullptr, FTDEC_EUNSUPPORTED, "batch*heads*seq too large");
  ftdec_ctx* c = new (std::nothrow) ftdec_ctx();
  if (!c) return dfail(nullptr, FTDEC_ENOMEM, "out of host memory");
  c->cfg = *cfg;
  ftdec_config& e = c->cfg;
  if (!(e.softmax_scale > 0.f)) e.softmax_scale = 1.0f / std::sqrt((float)e.head_dim);
  if (!(e.tau_rel > 0.f)) e.tau_rel = 1.0f / 32768.0f;
  if (!(e.eps_dmr > 0.f)) e.eps_dmr = 1.0f / 4096.0f;
  if (e.max_events <= 0) e.max_events = 4096;
  c->BH = e.batch * e.heads; c->N = e.seq; c->Np = (e.seq + 7) & ~7; c->d = e.head_dim;
  c->Tm = (c->N + ftgemm::GBM - 1) / ftgemm::GBM;
  c->Tn1 = (c->N + ftgemm::GBN - 1) / ftgemm::GBN;
  c->fault_cap = 1 << 16;
  hipError_t he = hipSetDevice(e.device);
  if (he != hipSuccess) { int rc = dfail(nullptr, FTDEC_EHIP, std::string("hipSetDevice: ") + hipGetErrorString(he)); delete c; return rc; }
  const size_t BH = c->BH, N = c->N, Np = c->Np, d = c->d, cap = e.max_events;
  struct { void** p; size_t bytes; bool sp; } allocs[] = {
      {(void**)&c->S, BH * N * N * 4, true}, {(void**)&c->P, BH * N * Np * 2, true}, {(void**)&c->vt, BH * d * Np * 2, false},
      {(void**)&c->wc1, BH * c->Tn1 * ftgemm::GCK * d * 2, false}, {(void**)&c->wc2, BH * ftgemm::GCK * Np * 2, false},
      {(void**)&c->g_events, 2 * BH * cap * sizeof(ftgemm_event), false}, {(void**)&c->counters, (2 * BH + 1) * 4, false},
      {(void**)&c->resmax, (2 * BH + 1) * 4, false}, {(void**)&c->s_events, cap * sizeof(ftdec_event), false},
      {(void**)&c->retried, 8, false}, {(void**)&c->d_gfaults, sizeof(ftgemm::GFault) * c->fault_cap, false},
      {(void**)&c->d_sfaults, sizeof(SFault) * c->fault_cap, false}};
  for (auto& al : allocs) {
    he = hipMalloc(al.p, al.bytes);
    if (he == hipSuccess) he = hipMemset(*al.p, 0, al.bytes);
    if (he != hipSuccess) {
      int rc = dfail(nullptr, he == hipErrorOutOfMemory ? FTDEC_ENOMEM : FTDEC_EHIP, std::string("allocating device scratch: ") + hipGetErrorString(he));
      drelease(c);
      return rc;
    }
    c->bytes_total += (int64_t)al.bytes;
    if (al.sp) c->bytes_sp += (int64_t)al.bytes;
  }
  he = hipHostMalloc((void**)&c->h_gfaults, sizeof(ftgemm::GFault) * c->fault_cap, hipHostMallocDefault);
  if (he == hipSuccess) he = hipHostMalloc((void**)&c->h_sfaults, sizeof(SFault) * c->fault_cap, hipHostMallocDefault);
  if (he == hipSuccess) he = ftgemm::gemm_allow_lds(c->d);
  if (he == hipSuccess) he = ftgemm::gemm_allow_lds(c->Np);
  // the softmax row is staged in LDS when it fits next to the reduction scratch
  c->softmax_lds = N * 4 <= 32 * 1024 ? N * 4 : 0;
  for (int v = 0; v < 4 && he == hipSuccess; ++v)
    he = hipFuncSetAttribute((const void*)select_softmax((v & 1) != 0, (v & 2) != 0), hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
  if (he == hipSuccess) he = hipDeviceSynchronize();
  if (he != hipSuccess) {
    int rc = dfail(nullptr, FTDEC_EHIP, std::string("context set-up: ") + hipGetErrorString(he));
    drelease(c);
    return rc;
  }
  *out = c;
  return FTDEC_OK;
}

extern "C" int ftdec_get_config(const ftdec_ctx* c, ftdec_config* effective) {
  if (!c || !effective) return FTDEC_EINVAL;
  *effective = c->cfg;
  return FTDEC_OK;
}

extern "C" int ftdec_footprint(const ftdec_ctx* c, int64_t* total_bytes, int64_t* s_and_p_bytes) {
  if (!c || !total_bytes || !s_and_p_bytes) return FTDEC_EINVAL;
  *total_bytes = c->bytes_total;
  *s_and_p_bytes = c->bytes_sp;
  return FTDEC_OK;
}

extern "C" int ftdec_forward(ftdec_ctx* c, const void* q, const void* k, const void* v, void* o,
                             const ftdec_fault* faults, int32_t n_faults, void* hip_stream) {
  if (!c) return FTDEC_EINVAL;
  if (!q || !k || !v || !o) return dfail(c, FTDEC_EINVAL, "null tensor pointer");
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return dfail(c, FTDEC_EINVAL, "tensor pointers must be 16-byte aligned");
  if (n_faults < 0 || (n_faults > 0 && !faults)) return dfail(c, FTDEC_EINVAL, "bad fault list");
  if (n_faults > c->fault_cap) return dfail(c, FTDEC_EINVAL, "too many faults (limit 65536)");
  const ftdec_config& e = c->cfg;
  const int BH = c->BH, N = c->N, Np = c->Np, d = c->d;
  const bool ft = e.ft_mode != FTDEC_FT_OFF, bf = e.in_dtype == FTDEC_BF16;
  hipStream_t st = (hipStream_t)hip_stream;
  DHIP_TRY(c, hipSetDevice(e.device));

  // ---- fault list: GEMM faults grouped by (stage, head), softmax faults sorted by (head, row)
  std::vector<int> g_off(2 * (size_t)BH + 1, 0);
  int n_g = 0, n_s = 0;
  if (n_faults > 0) {
    std::vector<std::pair<long long, ftgemm::GFault>> gf;
    std::vector<SFault> sf;
    for (int i = 0; i < n_faults; ++i) {
      const ftdec_fault& f = faults[i];
      bool ok = f.b >= 0 && f.b < e.batch && f.h >= 0 && f.h < e.heads && f.row >= 0 && f.row < N && f.bit >= 0 && f.bit <= 31 &&
                f.stage >= FTDEC_ST_GEMM1 && f.stage <= FTDEC_ST_GEMM2 && f.col >= 0;
      if (ok && f.stage == FTDEC_ST_GEMM2) ok = f.col < d;
      if (ok && f.stage == FTDEC_ST_GEMM1) ok = f.col < N;
      if (ok && (f.stage == FTDEC_ST_EXP || f.stage == FTDEC_ST_PNORM)) ok = f.col < N && (!e.causal || f.col <= f.row);
      if (!ok) {
        char msg[160];
        snprintf(msg, sizeof msg, "fault %d (b=%d h=%d stage=%d row=%d col=%d bit=%d) names a masked or out-of-range position",
                 i, f.b, f.h, f.stage, f.row, f.col, f.bit);
        return dfail(c, FTDEC_EINVAL, msg);
      }
      const int bh = f.b * e.heads + f.h;
      if (f.stage == FTDEC_ST_GEMM1 || f.stage == FTDEC_ST_GEMM2)
        gf.push_back({(long long)(f.stage == FTDEC_ST_GEMM1 ? 0 : BH) + bh, ftgemm::GFault{f.row, f.col, f.bit}});
      else
        sf.push_back(SFault{bh * N + f.row, f.col, f.bit, f.stage});
    }
    std::stable_sort(gf.begin(), gf.end(), [](const auto& x, const auto& y) { return x.first < y.first; });
    std::stable_sort(sf.begin(), sf.end(), [](const SFault& x, const SFault& y) { return x.key < y.key; });
    n_g = (int)gf.size(); n_s = (int)sf.size();
    for (int i = 0; i < n_g; ++i) { c->h_gfaults[i] = gf[i].second; g_off[gf[i].first + 1]++; }
    for (size_t i = 0; i < 2 * (size_t)BH; ++i) g_off[i + 1] += g_off[i];
    for (int i = 0; i < n_s; ++i) c->h_sfaults[i] = sf[i];
    if (n_g) DHIP_TRY(c, hipMemcpyAsync(c->d_gfaults, c->h_gfaults, sizeof(ftgemm::GFault) * n_g, hipMemcpyHostToDevice, st));
    if (n_s) DHIP_TRY(c, hipMemcpyAsync(c->d_sfaults, c->h_sfaults, sizeof(SFault) * n_s, hipMemcpyHostToDevice, st));
    DHIP_TRY(c, hipStreamSynchronize(st));     // the staging buffers may be rewritten by the next call
  }

  const int n_cnt = 2 * BH + 1;
  ftdec_reset<<<(n_cnt + 255) / 256, 256, 0, st>>>(c->counters, c->resmax, n_cnt, c->retried);
  if (c->timing) DHIP_TRY(c, hipEventRecord(c->ev[0], st));
  const size_t cap = e.max_events;
  auto gemm_args = [&](int which, int bh) {
    ftgemm::GArgs a;
    std::memset(&a, 0, sizeof a);
    a.out_dtype = FTGEMM_F32;
    a.tau_rel = e.tau_rel; a.tau_abs = 0.f; a.correct = 1; a.transposed = 0;
    const int slot = which * BH + bh;
    a.faults = c->d_gfaults + g_off[slot];
    a.n_faults = g_off[slot + 1] - g_off[slot];
    a.events = c->g_events + (size_t)slot * cap;
    a.ev_count = c->counters + slot;
    a.max_events = e.max_events;
    a.resmax = c->resmax + slot;
    return a;
  };

  // ---- 1. ABFT-GEMM I: S = Q K^T (tokens = queries, weight rows = keys).  Without a fault list all
  // heads go out as one batched launch; a fault list is applied head by head.
  const uint16_t* q16 = reinterpret_cast<const uint16_t*>(q);
  const uint16_t* k16 = reinterpret_cast<const uint16_t*>(k);
  const long long wc1_stride = (long long)c->Tn1 * ftgemm::GCK * d;
  if (ft) DHIP_TRY(c, ftgemm::gemm_launch_encode_w(k16, c->wc1, N, d, bf, st, BH, (long long)N * d, wc1_stride));
  for (int bh = 0; bh < (n_g ? BH : 1); ++bh) {
    ftgemm::GArgs a = gemm_args(0, bh);
    a.x = q16 + (size_t)bh * N * d; a.w = k16 + (size_t)bh * N * d; a.wc = c->wc1 + (size_t)bh * wc1_stride;
    a.y = c->S + (size_t)bh * N * N;
    a.M = N; a.N = N; a.K = d; a.Tm = c->Tm; a.Tn = c->Tn1;
    if (!n_g) {
      a.bs_x = a.bs_w = (long long)N * d; a.bs_wc = wc1_stride; a.bs_y_bytes = (long long)N * N * 4; a.bs_events = (long long)cap;
      a.skip_upper = e.causal;      // score tiles above the diagonal are never read by the softmax (with a fault
                                    // list the matrix is computed in full: a fault may name any score)
    }
    DHIP_TRY(c, ftgemm::gemm_launch(a, ft, a.n_faults > 0, bf, st, n_g ? 1 : BH));
  }
  if (c->timing) DHIP_TRY(c, hipEventRecord(c->ev[1], st));

  // ---- 2. DMR row-softmax, all heads in one launch
  {
    SArgs a;
    a.S = c->S; a.P = c->P; a.N = N; a.Np = Np; a.H = e.heads; a.causal = e.causal;
    a.scale_log2 = e.softmax_scale * 1.4426950408889634f;
    a.eps = e.eps_dmr;
    a.use_lds = c->softmax_lds ? 1 : 0;
    a.faults = c->d_sfaults; a.n_faults = n_s;
    a.events = c->s_events; a.ev_count = c->counters + 2 * BH; a.max_events = e.max_events;
    a.retried = c->retried;
    hipLaunchKernelGGL(select_softmax(ft, n_s > 0), dim3(N, BH), dim3(256), c->softmax_lds, st, a);
    DHIP_TRY(c, hipGetLastError());
  }
  if (c->timing) DHIP_TRY(c, hipEventRecord(c->ev[2], st));

  // ---- 3. ABFT-GEMM II: O = P V per head (tokens = queries, weight rows = the features of V^T)
  ftdec_transpose_v<<<dim3((Np + 63) / 64, BH), 256, 0, st>>>(reinterpret_cast<const uint16_t*>(v), c->vt, N, Np, d, bf ? 1 : 0);
  DHIP_TRY(c, hipGetLastError());
  const uint16_t* vt16 = reinterpret_cast<const uint16_t*>(c->vt);
  const uint16_t* p16 = reinterpret_cast<const uint16_t*>(c->P);
  const long long wc2_stride = (long long)ftgemm::GCK * Np;
  if (ft) DHIP_TRY(c, ftgemm::gemm_launch_encode_w(vt16, c->wc2, d, Np, false, st, BH, (long long)d * Np, wc2_stride));
  for (int bh = 0; bh < (n_g ? BH : 1); ++bh) {
    ftgemm::GArgs a = gemm_args(1, bh);
    a.x = p16 + (size_t)bh * N * Np; a.w = vt16 + (size_t)bh * d * Np; a.wc = c->wc2 + (size_t)bh * wc2_stride;
    a.y = reinterpret_cast<float*>(o) + (size_t)bh * N * d;
    a.M = N; a.N = d; a.K = Np; a.Tm = c->Tm; a.Tn = 1;
    if (!n_g) {
      a.bs_x = (long long)N * Np; a.bs_w = (long long)d * Np; a.bs_wc = wc2_stride; a.bs_y_bytes = (long long)N * d * 4;
      a.bs_events = (long long)cap;
      a.k_lower = e.causal;         // P is lower-triangular: keys beyond a tile's last query contribute nothing
    }
    DHIP_TRY(c, ftgemm::gemm_launch(a, ft, a.n_faults > 0, false, st, n_g ? 1 : BH));
  }
  if (c->timing) DHIP_TRY(c, hipEventRecord(c->ev[3], st));
  c->last_stream = st;
  c->ran = true;
  return FTDEC_OK;
}

extern "C" int ftdec_report(ftdec_ctx* c, ftdec_report_view* out) {
  if (!c || !out) return FTDEC_EINVAL;
  if (!c->ran) return dfail(c, FTDEC_EINVAL, "no forward call to report on");
  const ftdec_config& e = c->cfg;
  DHIP_TRY(c, hipSetDevice(e.device));
  DHIP_TRY(c, hipStreamSynchronize(c->last_stream));
  const int BH = c->BH, cap = e.max_events;
  c->h_counters.resize(2 * (size_t)BH + 1);
  DHIP_TRY(c, hipMemcpy(c->h_counters.data(), c->counters, c->h_counters.size() * 4, hipMemcpyDeviceToHost));
  unsigned long long retried = 0;
  DHIP_TRY(c, hipMemcpy(&retried, c->retried, 8, hipMemcpyDeviceToHost));
  c->events.clear();
  int dropped = 0;
  for (int slot = 0; slot < 2 * BH; ++slot) {
    const int count = c->h_counters[slot], stored = std::min(count, cap);
    dropped += count - stored;
    if (!stored) continue;
    c->h_gev.resize(stored);
    DHIP_TRY(c, hipMemcpy(c->h_gev.data(), c->g_events + (size_t)slot * cap, sizeof(ftgemm_event) * stored, hipMemcpyDeviceToHost));
    const int bh = slot % BH;
    for (const ftgemm_event& g : c->h_gev)
      c->events.push_back(ftdec_event{bh / e.heads, bh % e.heads, slot < BH ? FTDEC_ST_GEMM1 : FTDEC_ST_GEMM2, g.row, g.col, g.action});
  }
  {
    const int count = c->h_counters[2 * BH], stored = std::min(count, cap);
    dropped += count - stored;
    const size_t base = c->events.size();
    c->events.resize(base + stored);
    if (stored) DHIP_TRY(c, hipMemcpy(c->events.data() + base, c->s_events, sizeof(ftdec_event) * stored, hipMemcpyDeviceToHost));
  }
  std::sort(c->events.begin(), c->events.end(), [](const ftdec_event& x, const ftdec_event& y) {
    if (x.b != y.b) return x.b < y.b;
    if (x.h != y.h) return x.h < y.h;
    if (x.stage != y.stage) return x.stage < y.stage;
    if (x.row != y.row) return x.row < y.row;
    return x.col < y.col;
  });
  out->n_events = (int32_t)c->events.size();
  out->n_events_dropped = dropped;
  out->events = c->events.data();
  out->retried_rows = (int64_t)retried;
  return FTDEC_OK;
}

extern "C" int ftdec_set_timing(ftdec_ctx* c, int32_t enabled) {
  if (!c) return FTDEC_EINVAL;
  DHIP_TRY(c, hipSetDevice(c->cfg.device));
  if (enabled)
    for (hipEvent_t& e : c->ev)
      if (!e) DHIP_TRY(c, hipEventCreate(&e));
  c->timing = enabled != 0;
  return FTDEC_OK;
}

extern "C" int ftdec_get_timing(ftdec_ctx* c, float ms[3]) {
  if (!c || !ms) return FTDEC_EINVAL;
  if (!c->timing || !c->ran) return dfail(c, FTDEC_EINVAL, "timing is not enabled or no forward has run");
  DHIP_TRY(c, hipSetDevice(c->cfg.device));
  DHIP_TRY(c, hipEventSynchronize(c->ev[3]));
  for (int i = 0; i < 3; ++i) DHIP_TRY(c, hipEventElapsedTime(&ms[i], c->ev[i], c->ev[i + 1]));
  return FTDEC_OK;
}

extern "C" int ftdec_destroy(ftdec_ctx* c) {
  if (!c) return FTDEC_EINVAL;
  (void)hipSetDevice(c->cfg.device);
  (void)hipDeviceSynchronize();
  drelease(c);
  return FTDEC_OK;
}

extern "C" const char* ftdec_last_error(const ftdec_ctx* c) {
  return c ? c->err.c_str() : g_dec_err.c_str();
}
