// Device code of the fault-tolerant fused attention library (gfx950 / CDNA4 only).
//
// Data flow of one forward call (Algorithm 1 of the paper, all steps):
//
//   encode kernels   K -> per key tile: 64 fp16 key rows followed by 32 checksum rows
//                    (tensor checksums of eq. (13), (14), stride 8, weights 1 and l+1, each
//                    stored as an fp16 high word and an fp16 low word);
//                    V -> per key tile: V^T in fp16 (feature-major, keys permuted to the order in
//                    which the MFMA accumulator of GEMM I hands out scores) followed by 32
//                    checksum rows of V.
//   main kernel      one workgroup per (batch, head, row tile); loop over key tiles:
//                    GEMM I (+checksum block) -> max -> exp -> product-form check -> row-sum ->
//                    GEMM II with rescale (+checksum block); after the loop: row-sum range check,
//                    normalisation, sum-form check, store.
//
// Register layout.  Scores are computed transposed, S^T = K_j Q_i^T, with the 32x32x16 fp16 MFMA.
// A lane then owns ONE query (column lane%32) and, per 32-key block, the 16 keys
// 8*g + 4*(lane/32) + r (g, r in 0..3).  Key index mod 8 is 4*(lane/32)+r, so the four stride-8
// checksum classes a lane sees are fixed and all folds of a class sit in the lane's own registers:
// encoding, verification and correction need no cross-lane traffic (the property the paper's
// strided layout is built for, Section 3.3), and a row reduction needs exactly one exchange
// between lane and lane^32.  Checksum rows 8*w + c (w: c1 high, c1 low, c2 high, c2 low) of
// the extra MFMA block land in register 4*w + r of the lane that owns class c = 4*(lane/32)+r.
// GEMM II is computed as O^T = V_j^T P^T, which gives the output features the same layout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "ftattn.h"

namespace ftattn {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

constexpr int BN = 64;        // keys per tile (B_c)
constexpr int CKR = 32;       // checksum rows per tile: {c1 hi, c1 lo, c2 hi, c2 lo} x 8 classes
constexpr int NFOLD_K = BN / 8;
constexpr float LN2 = 0.6931471805599453f;

struct DevFault { int32_t stage, kv_tile, row, col, bit; };

struct KArgs {
  const _Float16* q;       // [BH][N][D] fp16
  const _Float16* kc;      // [BH][Tj][BN + CKR][D]
  const _Float16* vt;      // [BH][Tj][D + CKR][BN]
  void* o;                 // [BH][N][D], fp32 / fp16 / bf16
  int32_t out_dtype;
  int32_t N, H, Ti, Tj;
  float scale;             // sigma
  float scale_log2;        // sigma * log2(e)
  float eps1, tau_fast, tau_o, delta_l;
  int32_t correct;         // 1: repair, 0: detect only
  const DevFault* faults;  // sorted by (bh, row tile, kv_tile)
  const int32_t* fault_off;  // [BH*Ti + 1] or nullptr
  ftattn_event* events;
  int32_t* ev_count;
  int32_t max_events;
  uint32_t* resmax;        // [BH][Ti][4], float bits of non-negative values
  unsigned long long* recheck;
};

// ------------------------------------------------------------------ small helpers

__device__ __forceinline__ float as_f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float lg2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float fmax2(float a, float b) { return __builtin_fmaxf(a, b); }
__device__ __forceinline__ bool finitef(float x) { return (as_u(x) & 0x7F800000u) != 0x7F800000u; }

// value held by lane^32
__device__ __forceinline__ float xchg32(float x, int hi) {
  auto r = __builtin_amdgcn_permlane32_swap(as_u(x), as_u(x), false, false);
  return as_f(hi ? r[0] : r[1]);
}
__device__ __forceinline__ float max32(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(as_u(x), as_u(x), false, false);
  return fmax2(as_f(r[0]), as_f(r[1]));
}
__device__ __forceinline__ float sum32(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(as_u(x), as_u(x), false, false);
  return as_f(r[0]) + as_f(r[1]);
}
__device__ __forceinline__ bool wave_any(bool p) { return __builtin_amdgcn_ballot_w64(p) != 0ull; }

__device__ __forceinline__ float flip_if(float x, bool c, int bit) {
  return as_f(as_u(x) ^ (c ? (1u << bit) : 0u));
}

__device__ __forceinline__ void log_event(const KArgs& a, int bh, int check, int kv_tile, int row, int col,
                                          float res, int action) {
  int idx = atomicAdd(a.ev_count, 1);
  if (idx < a.max_events) {
    ftattn_event e;
    e.b = bh / a.H; e.h = bh % a.H; e.check = check; e.kv_tile = kv_tile; e.row = row; e.col = col;
    e.residual = res; e.action = action;
    a.events[idx] = e;
  }
}

// LDS tile addressing.  Rows are stored unpadded so that a wave-wide direct-to-LDS load of 64
// consecutive 16-byte chunks is one instruction; bank conflicts of the MFMA operand reads are
// avoided by XOR-ing the chunk index with a function of the row.
template <int D> __device__ __forceinline__ int swz_k(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
__device__ __forceinline__ int swz_v(int row) { return (row >> 1) & 7; }

template <int D> __device__ __forceinline__ half8 lds_k(const char* buf, int row, int chunk) {
  return *reinterpret_cast<const half8*>(buf + row * (D * 2) + ((chunk ^ swz_k<D>(row)) << 4));
}
__device__ __forceinline__ half8 lds_v(const char* buf, int row, int chunk) {
  return *reinterpret_cast<const half8*>(buf + row * (BN * 2) + ((chunk ^ swz_v(row)) << 4));
}

// 16 bytes per lane from global memory straight into LDS at (wave-uniform base + 16*lane).
// Issued as an opaque instruction so that the compiler does not serialise it against later LDS
// reads: completion is awaited explicitly with s_waitcnt vmcnt before the barrier that publishes
// the tile.
__device__ __forceinline__ void gload_lds16(const void* g, const char* lds_dst) {
  uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)lds_dst;
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(base) : "memory", "m0");
}

template <int D> struct TileBytes {
  static constexpr int K = (BN + CKR) * D * 2;
  static constexpr int V = (D + CKR) * BN * 2;
};

// position of a key of a 32-key block in the lane/register layout of the S^T accumulator
//   key (in block) = 8*g + 4*hi + r   <->  lane half hi, register v = 4*g + r
__device__ __forceinline__ int key_of(int kb, int v, int hi) { return 32 * kb + 8 * (v >> 2) + 4 * hi + (v & 3); }

// ------------------------------------------------------------------ encode kernels

__device__ __forceinline__ float load_as_float(const void* p, size_t idx, int dtype) {
  if (dtype == FTATTN_F16) return (float)reinterpret_cast<const _Float16*>(p)[idx];
  return as_f((uint32_t)reinterpret_cast<const uint16_t*>(p)[idx] << 16);
}

// bf16 -> fp16 copy of Q (fp16 input is used in place)
__global__ void ftattn_convert_q(const uint16_t* __restrict__ in, _Float16* __restrict__ out, size_t n) {
  size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 8;
  if (i + 8 <= n) {
    uint4v raw = *reinterpret_cast<const uint4v*>(in + i);
    half8 r;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      r[2 * k] = (_Float16)as_f(raw[k] << 16);
      r[2 * k + 1] = (_Float16)as_f(raw[k] & 0xFFFF0000u);
    }
    *reinterpret_cast<half8*>(out + i) = r;
  } else {
    for (; i < n; ++i) out[i] = (_Float16)as_f((uint32_t)in[i] << 16);
  }
}

// One workgroup per (key tile, head): fp16 key rows followed by the four checksum words of
// check1[c,:] = sum_l K[c+8l,:] and check2[c,:] = sum_l (l+1) K[c+8l,:]   (eq. (13), (14)).
template <int D>
__global__ __launch_bounds__(256) void ftattn_encode_k(const void* __restrict__ k, int dtype, _Float16* __restrict__ kc,
                                                       int N, int Tj, int with_checksums) {
  __shared__ float tile[BN][D + 1];
  const int j = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
  _Float16* out = kc + ((size_t)bh * Tj + j) * ((BN + CKR) * D);
  for (int e = tid; e < BN * D; e += 256) {
    int r = e / D, c = e % D, key = j * BN + r;
    float x = key < N ? load_as_float(k, ((size_t)bh * N + key) * D + c, dtype) : 0.f;
    _Float16 hx = (_Float16)x;
    out[r * D + c] = hx;
    tile[r][c] = (float)hx;
  }
  if (!with_checksums) return;
  __syncthreads();
  for (int e = tid; e < 8 * D; e += 256) {
    int cls = e / D, c = e % D;
    float c1 = 0.f, c2 = 0.f;
#pragma unroll
    for (int l = 0; l < NFOLD_K; ++l) {
      float x = tile[cls + 8 * l][c];
      c1 += x;
      c2 += (float)(l + 1) * x;
    }
    _Float16 h1 = (_Float16)c1, h2 = (_Float16)c2;
    out[(BN + cls) * D + c] = h1;
    out[(BN + 8 + cls) * D + c] = (_Float16)(c1 - (float)h1);
    out[(BN + 16 + cls) * D + c] = h2;
    out[(BN + 24 + cls) * D + c] = (_Float16)(c2 - (float)h2);
  }
}

// position of key kl (0..63) inside the permuted key axis of the V^T tile
__device__ __forceinline__ int vt_pos(int kl) {
  int kb = kl >> 5, g = (kl >> 3) & 3, hi = (kl >> 2) & 1, r = kl & 3;
  return 32 * kb + 16 * hi + 8 * (g >> 1) + 4 * (g & 1) + r;
}

// One workgroup per (key tile, head): V^T in fp16 followed by the checksum rows of
// check1[key, c] = sum_l V[key, c+8l] and check2 with weights l+1.
template <int D>
__global__ __launch_bounds__(256) void ftattn_encode_v(const void* __restrict__ v, int dtype, _Float16* __restrict__ vt,
                                                       int N, int Tj, int with_checksums) {
  __shared__ float tile[BN][D + 1];
  const int j = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
  _Float16* out = vt + ((size_t)bh * Tj + j) * ((D + CKR) * BN);
  for (int e = tid; e < BN * D; e += 256) {
    int r = e / D, c = e % D, key = j * BN + r;
    float x = key < N ? load_as_float(v, ((size_t)bh * N + key) * D + c, dtype) : 0.f;
    tile[r][c] = (float)(_Float16)x;
  }
  __syncthreads();
  for (int e = tid; e < D * BN; e += 256) {
    int f = e / BN, kl = e % BN;
    out[f * BN + vt_pos(kl)] = (_Float16)tile[kl][f];
  }
  if (!with_checksums) return;
  for (int e = tid; e < 8 * BN; e += 256) {
    int cls = e / BN, kl = e % BN;
    float c1 = 0.f, c2 = 0.f;
#pragma unroll
    for (int l = 0; l < D / 8; ++l) {
      float x = tile[kl][cls + 8 * l];
      c1 += x;
      c2 += (float)(l + 1) * x;
    }
    _Float16 h1 = (_Float16)c1, h2 = (_Float16)c2;
    int p = vt_pos(kl);
    out[(D + cls) * BN + p] = h1;
    out[(D + 8 + cls) * BN + p] = (_Float16)(c1 - (float)h1);
    out[(D + 16 + cls) * BN + p] = h2;
    out[(D + 24 + cls) * BN + p] = (_Float16)(c2 - (float)h2);
  }
}

// clears the event counter, the recheck counter and the residual maxima (a fill kernel rather
// than a memset so that a caller may capture the forward call in a graph)
__global__ void ftattn_reset(int32_t* ev_count, unsigned long long* recheck, uint32_t* resmax, int n_resmax) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i == 0) { *ev_count = 0; *recheck = 0ull; }
  if (i < n_resmax) resmax[i] = 0u;
}

}  // namespace ftattn
