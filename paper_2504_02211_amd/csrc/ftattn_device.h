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
  const void* q;           // [BH][N][D] fp16 or bf16 (q_bf16)
  int32_t q_bf16;
  const _Float16* kc;      // [BH][Tj][BN + CKR][D]
  const _Float16* vt;      // [BH][Tj][D + CKR][BN]
  void* o;                 // [BH][N][D], fp32 / fp16 / bf16
  int32_t out_dtype;
  int32_t N, H, Ti, Tj;
  float scale;             // sigma
  float scale_log2;        // sigma * log2(e)
  float eps1, tau_fast, tau_o, delta_l;
  int32_t correct;         // 1: repair, 0: detect only
  int32_t rowsum_fold;     // 1: the row-sum is an extra fold of checksum class 0 of the value tiles
  float rescale_margin;    // (lazy mode) the reference maximum is renewed beyond this, natural-log units
  const DevFault* faults;  // sorted by (bh, row tile, kv_tile)
  const int32_t* fault_off;  // [BH*Ti + 1] or nullptr
  ftattn_event* events;
  int32_t* ev_count;
  int32_t max_events;
  uint32_t* resmax;        // [BH][Ti][4], float bits of non-negative values
  unsigned long long* recheck;
  uint32_t* range;         // FTATTN_RANGE_* bits of this call (operands that do not survive the conversion to fp16)
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

// FTATTN_RANGE_* bits of 8 consecutive bf16 patterns: a finite value of magnitude 65536 or more
// becomes Inf in fp16; a non-zero one below 2^-24 loses every significant bit (zero or the smallest
// subnormal).  Values between 2^-24 and 2^-14 become fp16 subnormals, an absolute error below 2^-25,
// and are not flagged; neither are Inf / NaN inputs, which are the caller's.
__device__ __forceinline__ uint32_t bf16_range_bits(uint4v raw) {
  uint32_t bits = 0u;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
#pragma unroll
    for (int hlf = 0; hlf < 2; ++hlf) {
      const uint32_t m = (hlf ? raw[k] >> 16 : raw[k]) & 0x7FFFu;
      if (m >= 0x4780u && m < 0x7F80u) bits |= FTATTN_RANGE_OPERAND_OVERFLOW;
      if (m != 0u && m < 0x3380u) bits |= FTATTN_RANGE_OPERAND_UNDERFLOW;
    }
  }
  return bits;
}

// 8 consecutive 16-bit inputs (fp16 or bf16 patterns) -> fp16
__device__ __forceinline__ half8 to_half8(uint4v raw, bool bf16) {
  if (!bf16) return __builtin_bit_cast(half8, raw);
  half8 r;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    r[2 * k] = (_Float16)as_f(raw[k] << 16);
    r[2 * k + 1] = (_Float16)as_f(raw[k] & 0xFFFF0000u);
  }
  return r;
}

// Key tile j of head bh by the first D threads of a workgroup, one thread per (checksum class,
// 16-byte chunk of a row): the thread converts the 8 rows of its class to fp16 and forms, in fp32
// registers, the four checksum words of check1[c,:] = sum_l K[c+8l,:] and
// check2[c,:] = sum_l (l+1) K[c+8l,:]  (eq. (13), (14)).
template <int D>
__device__ __forceinline__ void encode_k_tile(const void* __restrict__ k, int bf16, _Float16* __restrict__ kc,
                                              int N, int Tj, int with_checksums, int j, int bh, int tid, uint32_t* range) {
  constexpr int KCH = D / 8;
  const int cls = tid / KCH, ch = tid % KCH;
  const uint16_t* src = reinterpret_cast<const uint16_t*>(k) + (size_t)bh * N * D + ch * 8;
  _Float16* out = kc + ((size_t)bh * Tj + j) * ((BN + CKR) * D) + ch * 8;
  float c1[8], c2[8];
  uint32_t rbits = 0u;
#pragma unroll
  for (int x = 0; x < 8; ++x) { c1[x] = 0.f; c2[x] = 0.f; }
#pragma unroll
  for (int l = 0; l < NFOLD_K; ++l) {
    const int r = cls + 8 * l, key = j * BN + r;
    uint4v raw = (uint4v)0u;
    if (key < N) raw = *reinterpret_cast<const uint4v*>(src + (size_t)key * D);
    if (bf16) rbits |= bf16_range_bits(raw);
    const half8 h = to_half8(raw, bf16 != 0);
    *reinterpret_cast<half8*>(out + r * D) = h;
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const float v = (float)h[x];
      c1[x] += v;
      c2[x] += (float)(l + 1) * v;
    }
  }
  if (!with_checksums) {
    if (rbits) atomicOr(range, rbits);
    return;
  }
  half8 w0, w1, w2, w3;
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    w0[x] = (_Float16)c1[x]; w1[x] = (_Float16)(c1[x] - (float)w0[x]);
    w2[x] = (_Float16)c2[x]; w3[x] = (_Float16)(c2[x] - (float)w2[x]);
    // a checksum beyond the fp16 range (the second one reaches 36 times the largest key value)
    if ((finitef(c1[x]) && !finitef((float)w0[x])) || (finitef(c2[x]) && !finitef((float)w2[x]))) rbits |= FTATTN_RANGE_CHECKSUM_OVERFLOW;
  }
  if (rbits) atomicOr(range, rbits);
  *reinterpret_cast<half8*>(out + (BN + cls) * D) = w0;
  *reinterpret_cast<half8*>(out + (BN + 8 + cls) * D) = w1;
  *reinterpret_cast<half8*>(out + (BN + 16 + cls) * D) = w2;
  *reinterpret_cast<half8*>(out + (BN + 24 + cls) * D) = w3;
}

// position of key kl (0..63) inside the permuted key axis of the V^T tile
__device__ __forceinline__ int vt_pos(int kl) {
  int kb = kl >> 5, g = (kl >> 3) & 3, hi = (kl >> 2) & 1, r = kl & 3;
  return 32 * kb + 16 * hi + 8 * (g >> 1) + 4 * (g & 1) + r;
}
// ... and the key that sits at position p
__device__ __forceinline__ int vt_key(int p) {
  int kb = p >> 5, hi = (p >> 4) & 1, G = (p >> 3) & 1, b = (p >> 2) & 1, r = p & 3;
  return 32 * kb + 16 * G + 8 * b + 4 * hi + r;
}

// Value tile j of head bh by a whole workgroup of 256 threads: V^T in fp16 (16-byte loads,
// transposition through LDS, 16-byte stores) followed by the checksum rows of
// check1[key, c] = sum_l V[key, c+8l] and check2 with weights l+1.
template <int D>
__device__ __forceinline__ void encode_v_tile(const void* __restrict__ v, int bf16, _Float16* __restrict__ vt,
                                              int N, int Tj, int with_checksums, int j, int bh, int tid, uint32_t* range) {
  uint32_t rbits = 0u;
  // with_checksums == 2: class 0 also folds a column of ones at feature index D (fold D/8), which
  // makes the first checksum of class 0 carry the row-sum through GEMM II
  constexpr int KCH = D / 8, PITCH = D + 8;
  __shared__ __attribute__((aligned(16))) _Float16 tile[BN * PITCH];
  __shared__ __attribute__((aligned(16))) _Float16 cks[CKR * BN];
  const uint16_t* src = reinterpret_cast<const uint16_t*>(v) + (size_t)bh * N * D;
  _Float16* out = vt + ((size_t)bh * Tj + j) * ((D + CKR) * BN);
  for (int e = tid; e < BN * KCH; e += 256) {
    const int r = e / KCH, ch = e % KCH, key = j * BN + r;
    uint4v raw = (uint4v)0u;
    if (key < N) raw = *reinterpret_cast<const uint4v*>(src + (size_t)key * D + ch * 8);
    if (bf16) rbits |= bf16_range_bits(raw);
    *reinterpret_cast<half8*>(tile + r * PITCH + ch * 8) = to_half8(raw, bf16 != 0);
  }
  __syncthreads();
  for (int e = tid; e < D * 8; e += 256) {
    const int f = e >> 3, pc = e & 7;
    half8 h;
#pragma unroll
    for (int x = 0; x < 8; ++x) h[x] = tile[vt_key(8 * pc + x) * PITCH + f];
    *reinterpret_cast<half8*>(out + f * BN + 8 * pc) = h;
  }
  if (!with_checksums) {
    if (rbits) atomicOr(range, rbits);
    return;
  }
  for (int e = tid; e < 8 * BN; e += 256) {
    const int cls = e / BN, kl = e % BN;
    float c1 = 0.f, c2 = 0.f;
#pragma unroll
    for (int l = 0; l < D / 8; ++l) {
      const float x = (float)tile[kl * PITCH + cls + 8 * l];
      c1 += x;
      c2 += (float)(l + 1) * x;
    }
    if (with_checksums == 2 && cls == 0 && j * BN + kl < N) { c1 += 1.0f; c2 += (float)(D / 8 + 1); }
    const _Float16 h1 = (_Float16)c1, h2 = (_Float16)c2;
    if ((finitef(c1) && !finitef((float)h1)) || (finitef(c2) && !finitef((float)h2))) rbits |= FTATTN_RANGE_CHECKSUM_OVERFLOW;
    const int p = vt_pos(kl);
    cks[cls * BN + p] = h1;
    cks[(8 + cls) * BN + p] = (_Float16)(c1 - (float)h1);
    cks[(16 + cls) * BN + p] = h2;
    cks[(24 + cls) * BN + p] = (_Float16)(c2 - (float)h2);
  }
  __syncthreads();
  *reinterpret_cast<half8*>(out + D * BN + tid * 8) = *reinterpret_cast<const half8*>(cks + tid * 8);
  if (rbits) atomicOr(range, rbits);
}

// Everything the fused pass needs before it starts, in one launch (Algorithm 1: "Encode tensor
// checksum"): grid (key tiles, heads, 2); the workgroups with blockIdx.z == 0 encode the value tiles
// and clear the event counter, the recheck counter and the residual maxima (a store per thread
// rather than a memset, so that a caller may capture the forward call in a graph), those with
// blockIdx.z == 1 encode the key tiles.
template <int D>
__global__ __launch_bounds__(256) void ftattn_prepare(const void* __restrict__ k, const void* __restrict__ v, int bf16,
                                                      _Float16* __restrict__ kc, _Float16* __restrict__ vt, int N, int Tj,
                                                      int k_checksums, int v_checksums, int32_t* ev_count,
                                                      unsigned long long* recheck, uint32_t* resmax, int n_resmax,
                                                      uint32_t* range, uint32_t* range_next) {
  const int j = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
  if (blockIdx.z == 0) {
    const long long i = ((long long)bh * Tj + j) * 256 + tid;
    // (the range word of THIS call is set by many workgroups of this launch, so it cannot be cleared
    // here: each call clears the word the next call will use)
    if (i == 0) { *ev_count = 0; *recheck = 0ull; *range_next = 0u; }
    if (i < n_resmax) resmax[i] = 0u;
    encode_v_tile<D>(v, bf16, vt, N, Tj, v_checksums, j, bh, tid, range);
  } else if (tid < D) {
    encode_k_tile<D>(k, bf16, kc, N, Tj, k_checksums, j, bh, tid, range);
  }
}

}  // namespace ftattn
