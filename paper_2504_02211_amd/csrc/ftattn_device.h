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

// Asynchronous copy of one encoded key tile and one encoded value tile into LDS.
template <int D, int NW, bool FT>
__device__ __forceinline__ void load_tiles(const _Float16* kc_tile, const _Float16* vt_tile, char* bufk, char* bufv,
                                           int wave, int lane) {
  constexpr int KCH = D / 8;                       // 16-byte chunks per key row
  constexpr int K_INSTR = (FT ? BN + CKR : BN) * KCH / 64;
  constexpr int V_INSTR = (FT ? D + CKR : D) * (BN / 8) / 64;
#pragma unroll
  for (int i = 0; i < (K_INSTR + NW - 1) / NW; ++i) {
    int ins = i * NW + wave;
    if (K_INSTR % NW == 0 || ins < K_INSTR) {
      int L = ins * 64 + lane;
      int row = L / KCH, c = (L % KCH) ^ swz_k<D>(row);
      const _Float16* g = kc_tile + row * D + c * 8;
      char* dst = bufk + __builtin_amdgcn_readfirstlane(ins) * 1024;
      gload_lds16(g, dst);
    }
  }
#pragma unroll
  for (int i = 0; i < (V_INSTR + NW - 1) / NW; ++i) {
    int ins = i * NW + wave;
    if (V_INSTR % NW == 0 || ins < V_INSTR) {
      int L = ins * 64 + lane;
      int row = L / 8, c = (L % 8) ^ swz_v(row);
      const _Float16* g = vt_tile + row * BN + c * 8;
      char* dst = bufv + __builtin_amdgcn_readfirstlane(ins) * 1024;
      gload_lds16(g, dst);
    }
  }
}

// ------------------------------------------------------------------ main kernel

template <int D> struct TileBytes {
  static constexpr int K = (BN + CKR) * D * 2;
  static constexpr int V = (D + CKR) * BN * 2;
};

// position of a key of a 32-key block in the lane/register layout of the S^T accumulator
//   key (in block) = 8*g + 4*hi + r   <->  lane half hi, register v = 4*g + r
__device__ __forceinline__ int key_of(int kb, int v, int hi) { return 32 * kb + 8 * (v >> 2) + 4 * hi + (v & 3); }

template <int D, int NW, int NQ, bool FT, bool CAUSAL>
__global__ __launch_bounds__(NW * 64) void ftattn_main(const KArgs a) {
  constexpr int BM = NW * NQ * 32;
  constexpr int NSLAB = D / 16;     // k-slabs of GEMM I
  constexpr int NFB = D / 32;       // 32-feature blocks of O^T
  constexpr int NFOLD_V = D / 8;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int STAGE = TileBytes<D>::K + TileBytes<D>::V;   // one K tile followed by one V^T tile

  // ---- workgroup -> (head, row tile).  Workgroup ids go round-robin over the 8 XCDs; give each
  // XCD a contiguous range of work so that workgroups sharing K/V of a head share an L2.
  const int total = gridDim.x;
  int logical;
  {
    int id = blockIdx.x, xcd = id & 7, slot = id >> 3, qn = total >> 3, rn = total & 7;
    logical = xcd * qn + (xcd < rn ? xcd : rn) + slot;
  }
  const int bh = logical / a.Ti;
  const int ti = CAUSAL ? a.Ti - 1 - (logical % a.Ti) : (logical % a.Ti);   // heavy row tiles first
  const int tid = threadIdx.x, lane = tid & 63, lq = lane & 31, hi = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int N = a.N;
  const int row0_cta = ti * BM;
  const int row0_w = row0_cta + wave * (NQ * 32);
  const int last_row_cta = (row0_cta + BM < N ? row0_cta + BM : N) - 1;
  const int nj = CAUSAL ? (last_row_cta / BN + 1) : a.Tj;
  const float sl2 = a.scale_log2;

  const _Float16* kc_head = a.kc + (size_t)bh * a.Tj * ((BN + CKR) * D);
  const _Float16* vt_head = a.vt + (size_t)bh * a.Tj * ((D + CKR) * BN);

  // faults of this workgroup
  int fcur = 0, fend = 0;
  const DevFault* __restrict__ F = a.faults;
  if (a.fault_off != nullptr) { fcur = a.fault_off[bh * a.Ti + ti]; fend = a.fault_off[bh * a.Ti + ti + 1]; }

  load_tiles<D, NW, FT>(kc_head, vt_head, smem, smem + TileBytes<D>::K, wave, lane);

  // ---- Q_i^T as MFMA B operand: lane (query lq, half hi) holds Q[row][16*slab + 8*hi .. +7]
  half8 qf[NQ][NSLAB];
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    int row = row0_w + g * 32 + lq;
    const _Float16* qp = a.q + ((size_t)bh * N + (row < N ? row : 0)) * D + 8 * hi;
#pragma unroll
    for (int sl = 0; sl < NSLAB; ++sl) {
      half8 v = *reinterpret_cast<const half8*>(qp + 16 * sl);
      if (row >= N) v = (half8)(_Float16)0;
      qf[g][sl] = v;
    }
  }

  float16v o[NQ][NFB], oc[NQ];
  float m_run[NQ], l_part[NQ], l_low[NQ], dev_max = 0.f;
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
#pragma unroll
    for (int fb = 0; fb < NFB; ++fb) o[g][fb] = (float16v)0.f;
    oc[g] = (float16v)0.f;
    m_run[g] = -__builtin_inff(); l_part[g] = 0.f; l_low[g] = 0.f;
  }
  unsigned rechecks = 0;

  for (int j = 0; j < nj; ++j) {
    const int k0 = j * BN;
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's part of tile j is in LDS
    __syncthreads();                      // everyone's part is; everyone is done with the other buffer
    if (j + 1 < nj)
      load_tiles<D, NW, FT>(kc_head + (size_t)(j + 1) * ((BN + CKR) * D), vt_head + (size_t)(j + 1) * ((D + CKR) * BN),
                            smem + ((j + 1) & 1) * STAGE, smem + ((j + 1) & 1) * STAGE + TileBytes<D>::K, wave, lane);
    const char* bk = smem + (j & 1) * STAGE;
    const char* bv = bk + TileBytes<D>::K;
    const bool tile_has_fault = fcur < fend && F[fcur].kv_tile == j;

    // which of this wave's query groups take part in this tile, and which see a mask
    bool g_on[NQ], g_mask[NQ];
    bool any_on = false;
#pragma unroll
    for (int g = 0; g < NQ; ++g) {
      int r0 = row0_w + g * 32;
      g_on[g] = r0 < N && (!CAUSAL || k0 <= r0 + 31);
      g_mask[g] = (CAUSAL && k0 + BN - 1 > r0) || (k0 + BN > N);
      any_on |= g_on[g];
    }

    if (any_on) {
      // ================= GEMM I: S^T = K_j Q^T, checksum block = K^c Q^T  (eq. (15), (16))
      float16v s[NQ][2], sc[NQ];
#pragma unroll
      for (int g = 0; g < NQ; ++g) { s[g][0] = (float16v)0.f; s[g][1] = (float16v)0.f; sc[g] = (float16v)0.f; }
#pragma unroll
      for (int sl = 0; sl < NSLAB; ++sl) {
        half8 a0 = lds_k<D>(bk, lq, 2 * sl + hi);
        half8 a1 = lds_k<D>(bk, 32 + lq, 2 * sl + hi);
        half8 ac;
        if (FT) ac = lds_k<D>(bk, 64 + lq, 2 * sl + hi);
#pragma unroll
        for (int g = 0; g < NQ; ++g) {
          if (g_on[g]) {
            s[g][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, qf[g][sl], s[g][0], 0, 0, 0);
            s[g][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, qf[g][sl], s[g][1], 0, 0, 0);
            if (FT) sc[g] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ac, qf[g][sl], sc[g], 0, 0, 0);
          }
        }
      }

      // ---- injection point: raw scores
      if (tile_has_fault) {
        for (int fi = fcur; fi < fend && F[fi].kv_tile == j; ++fi) {
          if (F[fi].stage != FTATTN_ST_S) continue;
          int lr = F[fi].row - row0_w, kl = F[fi].col - k0, bit = F[fi].bit;
          bool mine = lr >= 0 && lr < NQ * 32 && lane == (lr & 31) + 32 * ((kl & 7) >> 2);
          int tg = lr >> 5, tkb = kl >> 5, tv = 4 * ((kl & 31) >> 3) + (kl & 3);
#pragma unroll
          for (int g = 0; g < NQ; ++g)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int v = 0; v < 16; ++v) s[g][kb][v] = flip_if(s[g][kb][v], mine && tg == g && tkb == kb && tv == v, bit);
        }
      }

      half8 ph[NQ][2][2];     // P^T in fp16, B operand of GEMM II: [group][key block][8-key half]
      float alpha[NQ];
#pragma unroll
      for (int g = 0; g < NQ; ++g) {
        alpha[g] = 1.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) { ph[g][kb][0] = (half8)(_Float16)0; ph[g][kb][1] = (half8)(_Float16)0; }
        if (!g_on[g]) continue;
        const int row = row0_w + g * 32 + lq;
        float p[2][16];
        float mx, m_new, negm;
        bool recheck = g_mask[g];

        if (!g_mask[g]) {
          // ============ reduce max, exp (fast path: no masked entry in this tile)
          mx = s[g][0][0];
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmax2(mx, s[g][kb][v]);
          mx = max32(mx);
          m_new = fmax2(m_run[g], mx);
          negm = -m_new * sl2;
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) p[kb][v] = ex2(__builtin_fmaf(s[g][kb][v], sl2, negm));
        } else {
          // ============ same with the causal / sequence-end mask applied per element
          mx = -__builtin_inff();
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              int key = k0 + key_of(kb, v, hi);
              bool ok = key < N && (!CAUSAL || key <= row);
              mx = fmax2(mx, ok ? s[g][kb][v] : -__builtin_inff());
            }
          mx = max32(mx);
          m_new = fmax2(m_run[g], mx);
          negm = -m_new * sl2;
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              int key = k0 + key_of(kb, v, hi);
              bool ok = key < N && (!CAUSAL || key <= row);
              p[kb][v] = ok ? ex2(__builtin_fmaf(s[g][kb][v], sl2, negm)) : 0.f;
            }
        }

        // ---- injection point: exponentials
        if (tile_has_fault) {
          for (int fi = fcur; fi < fend && F[fi].kv_tile == j; ++fi) {
            if (F[fi].stage != FTATTN_ST_EXP) continue;
            int lr = F[fi].row - row0_w, kl = F[fi].col - k0, bit = F[fi].bit;
            bool mine = lr >= 0 && (lr >> 5) == g && lane == (lr & 31) + 32 * ((kl & 7) >> 2);
            int tkb = kl >> 5, tv = 4 * ((kl & 31) >> 3) + (kl & 3);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int v = 0; v < 16; ++v) p[kb][v] = flip_if(p[kb][v], mine && tkb == kb && tv == v, bit);
          }
        }

        if (FT) {
          if (!g_mask[g]) {
            // ============ unified product-form check of GEMM I, subtraction and exp
            // (Algorithm 1, first "if"; Section 3.4 case 2).  For class c the product of its 8
            // exponentials must equal exp2(sl2*check1 - 8*m).  Both sides are divided by that
            // prediction, two factors at a time, so the running product stays near one.
            bool bad = false;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              float chk = sc[g][r] + sc[g][4 + r];
              float e = __builtin_fmaf(chk, sl2, (float)NFOLD_K * negm);
              float s2 = ex2(e * (-2.0f / NFOLD_K));
              float pr = ((p[0][r] * p[0][4 + r]) * s2) * ((p[0][8 + r] * p[0][12 + r]) * s2);
              pr *= ((p[1][r] * p[1][4 + r]) * s2) * ((p[1][8 + r] * p[1][12 + r]) * s2);
              float dv = __builtin_fabsf(pr - 1.0f);
              bad |= !(dv <= a.tau_fast);
              dev_max = fmax2(dev_max, dv <= a.tau_fast ? dv : 0.f);   // largest deviation that passed
            }
            recheck = wave_any(bad);
            if (recheck) ++rechecks;
          }
          if (recheck) {
            // ============ exact re-evaluation (rare: a fast check tripped, or the tile is masked).
            // lambda = ln prod P - (sigma*check1_eff - n_valid*m) = sum_l (ln P_l - x_l) - sigma*R1.
            bool lin_fixed = false;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              float chk1 = sc[g][r] + sc[g][4 + r];
              float sum1 = 0.f, E = 0.f;
              int nvalid = 0;
#pragma unroll
              for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) {
                  int v = 4 * gg + r, key = k0 + key_of(kb, v, hi);
                  bool ok = key < N && (!CAUSAL || key <= row);
                  float sv = s[g][kb][v];
                  sum1 += sv;
                  float t = __builtin_fmaf(sv, sl2, negm);
                  float pe = ex2(t);
                  if (ok) {
                    ++nvalid;
                    if (as_u(pe) != as_u(p[kb][v])) E += lg2(p[kb][v]) - t;
                  }
                }
              float R1 = chk1 - sum1;
              float lam = LN2 * E - a.scale * R1;
              bool det = nvalid > 0 && !(__builtin_fabsf(lam) <= a.eps1);
              if (det) {
                bool linear = !(a.scale * __builtin_fabsf(R1) <= 0.5f * a.eps1);
                if (linear) {
                  float chk2 = sc[g][8 + r] + sc[g][12 + r];
                  float sum2 = 0.f, big = -1.f;
                  int l_big = -1;
#pragma unroll
                  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int gg = 0; gg < 4; ++gg) {
                      float sv = s[g][kb][4 * gg + r];
                      sum2 += (float)(4 * kb + gg + 1) * sv;
                      float mag = finitef(sv) ? __builtin_fabsf(sv) : __builtin_inff();
                      if (mag > big) { big = mag; l_big = 4 * kb + gg; } else if (mag == big) { l_big = -1; }
                    }
                  float ratio = (chk2 - sum2) / R1;
                  int lstar = -1;
                  if (finitef(ratio)) {
                    float c = __builtin_rintf(ratio) - 1.0f;
                    if (c >= 0.f && c < (float)NFOLD_K) lstar = (int)c;
                  } else {
                    lstar = l_big;   // residuals left the fp32 range: the fold of overwhelming size
                  }
                  int col = lstar >= 0 ? k0 + 32 * (lstar >> 2) + 8 * (lstar & 3) + 4 * hi + r : -1;
                  bool fix = a.correct && lstar >= 0;
                  log_event(a, bh, FTATTN_CHECK_S, j, row, col, lam, fix ? 1 : 0);
                  if (fix) {
                    float rest = 0.f;
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                      for (int gg = 0; gg < 4; ++gg)
                        if (4 * kb + gg != lstar) rest += s[g][kb][4 * gg + r];
                    float val = chk1 - rest;
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                      for (int gg = 0; gg < 4; ++gg)
                        if (4 * kb + gg == lstar) s[g][kb][4 * gg + r] = val;
                    lin_fixed = true;
                  }
                } else {
#pragma unroll
                  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int gg = 0; gg < 4; ++gg) {
                      int v = 4 * gg + r, key = k0 + key_of(kb, v, hi);
                      bool ok = key < N && (!CAUSAL || key <= row);
                      float pe = ex2(__builtin_fmaf(s[g][kb][v], sl2, negm));
                      if (ok && as_u(pe) != as_u(p[kb][v])) {
                        log_event(a, bh, FTATTN_CHECK_EXP, j, row, key, lam, a.correct ? 1 : 0);
                        if (a.correct) p[kb][v] = pe;
                      }
                    }
                }
              }
            }
            // a repaired score changes the row's maximum and exponentials: recompute the row
            // (the exchange is a wave-wide operation: evaluate it outside any per-lane short circuit)
            const float partner_fixed = xchg32(lin_fixed ? 1.f : 0.f, hi);
            bool redo = lin_fixed | (partner_fixed != 0.f);
            if (wave_any(redo)) {
              float mx2 = -__builtin_inff();
#pragma unroll
              for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                  int key = k0 + key_of(kb, v, hi);
                  bool ok = key < N && (!CAUSAL || key <= row);
                  mx2 = fmax2(mx2, ok ? s[g][kb][v] : -__builtin_inff());
                }
              mx2 = max32(mx2);
              if (redo) {
                mx = mx2;
                m_new = fmax2(m_run[g], mx);
                negm = -m_new * sl2;
              }
#pragma unroll
              for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                  int key = k0 + key_of(kb, v, hi);
                  bool ok = key < N && (!CAUSAL || key <= row);
                  float pe = ok ? ex2(__builtin_fmaf(s[g][kb][v], sl2, negm)) : 0.f;
                  if (redo) p[kb][v] = pe;
                }
            }
          }
        }

        // ============ reduce sum (row-sum and its lower bound carried with the same rescale)
        float al = ex2(__builtin_fmaf(m_run[g], sl2, negm));
        float ps = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) ps += p[kb][v];
        l_part[g] = l_part[g] * al + ps;
        if (FT) l_low[g] = l_low[g] * al + ex2(__builtin_fmaf(mx, sl2, negm));
        m_run[g] = m_new;
        alpha[g] = al;

        // ---- injection point: row-sum
        if (tile_has_fault) {
          for (int fi = fcur; fi < fend && F[fi].kv_tile == j; ++fi) {
            if (F[fi].stage != FTATTN_ST_ROWSUM) continue;
            int lr = F[fi].row - row0_w;
            bool mine = lr >= 0 && (lr >> 5) == g && lq == (lr & 31);
            float full = sum32(l_part[g]);
            float flipped = flip_if(full, true, F[fi].bit);
            if (mine) l_part[g] = hi ? 0.f : flipped;
          }
        }

        // P -> fp16 in B-operand order: registers 8n..8n+7 of a key block feed MFMA n
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int i = 0; i < 8; ++i) ph[g][kb][n][i] = (_Float16)p[kb][8 * n + i];
      }

      // ================= GEMM II with rescale: O^T = diag(alpha) O^T + V_j^T P^T  (+ checksum block)
#pragma unroll
      for (int g = 0; g < NQ; ++g) {
        if (g_on[g] && wave_any(alpha[g] != 1.f)) {
#pragma unroll
          for (int fb = 0; fb < NFB; ++fb) o[g][fb] *= alpha[g];
          if (FT) oc[g] *= alpha[g];
        }
      }
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int n = 0; n < 2; ++n) {
#pragma unroll
          for (int fb = 0; fb < NFB; ++fb) {
            half8 av = lds_v(bv, 32 * fb + lq, 4 * kb + 2 * hi + n);
#pragma unroll
            for (int g = 0; g < NQ; ++g)
              if (g_on[g]) o[g][fb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, ph[g][kb][n], o[g][fb], 0, 0, 0);
          }
          if (FT) {
            half8 av = lds_v(bv, D + lq, 4 * kb + 2 * hi + n);
#pragma unroll
            for (int g = 0; g < NQ; ++g)
              if (g_on[g]) oc[g] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, ph[g][kb][n], oc[g], 0, 0, 0);
          }
        }

      // ---- injection point: output accumulator
      if (tile_has_fault) {
        for (int fi = fcur; fi < fend && F[fi].kv_tile == j; ++fi) {
          if (F[fi].stage != FTATTN_ST_OACC) continue;
          int lr = F[fi].row - row0_w, col = F[fi].col, bit = F[fi].bit;
          bool mine = lr >= 0 && lr < NQ * 32 && lane == (lr & 31) + 32 * ((col & 7) >> 2);
          int tg = lr >> 5, tfb = col >> 5, tv = 4 * ((col & 31) >> 3) + (col & 3);
#pragma unroll
          for (int g = 0; g < NQ; ++g)
#pragma unroll
            for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
              for (int v = 0; v < 16; ++v) o[g][fb][v] = flip_if(o[g][fb][v], mine && tg == g && tfb == fb && tv == v, bit);
        }
      }
    }
    if (tile_has_fault)
      while (fcur < fend && F[fcur].kv_tile == j) ++fcur;
  }

  // ================= after the loop: row-sum range check, normalisation, sum-form check, store
  float rmax_o = 0.f, rmax_u = 0.f, rmax_l = 0.f;
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    const int row = row0_w + g * 32 + lq;
    const bool real = row < N;
    float l = sum32(l_part[g]);
    if (FT) {
      float U = CAUSAL ? (float)(row + 1 < N ? row + 1 : N) : (float)N;
      float lo = l_low[g];
      bool detl = real && !(lo * (1.f - a.delta_l) <= l && l <= U * (1.f + a.delta_l));
      if (!detl && real) { rmax_u = fmax2(rmax_u, l / U); rmax_l = fmax2(rmax_l, lo / l); }
      if (detl) {
        if (hi == 0) log_event(a, bh, FTATTN_CHECK_L, -1, row, 0, l, a.correct ? 1 : 0);
        if (a.correct) l = lo;     // the approximation of Section 3.4, "optimized EFTA"
      }
    }
    float inv = 1.0f / l;
#pragma unroll
    for (int fb = 0; fb < NFB; ++fb) o[g][fb] *= inv;
    if (FT) {
      oc[g] *= inv;
      bool bad = false;
      float R[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float sum1 = 0.f;
#pragma unroll
        for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
          for (int gg = 0; gg < 4; ++gg) sum1 += o[g][fb][4 * gg + r];
        R[r] = (oc[g][r] + oc[g][4 + r]) - sum1;
        bool d = real && !(__builtin_fabsf(R[r]) <= a.tau_o);
        bad |= d;
        if (!d && real) rmax_o = fmax2(rmax_o, __builtin_fabsf(R[r]));
      }
      if (wave_any(bad)) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (real && !(__builtin_fabsf(R[r]) <= a.tau_o)) {
            float chk1 = oc[g][r] + oc[g][4 + r], chk2 = oc[g][8 + r] + oc[g][12 + r];
            float sum2 = 0.f, big = -1.f;
            int l_big = -1;
#pragma unroll
            for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
              for (int gg = 0; gg < 4; ++gg) {
                float ov = o[g][fb][4 * gg + r];
                sum2 += (float)(4 * fb + gg + 1) * ov;
                float mag = finitef(ov) ? __builtin_fabsf(ov) : __builtin_inff();
                if (mag > big) { big = mag; l_big = 4 * fb + gg; } else if (mag == big) { l_big = -1; }
              }
            float ratio = (chk2 - sum2) / R[r];
            int lstar = -1;
            if (finitef(ratio)) {
              float c = __builtin_rintf(ratio) - 1.0f;
              if (c >= 0.f && c < (float)NFOLD_V) lstar = (int)c;
            } else {
              lstar = l_big;
            }
            int col = lstar >= 0 ? 8 * lstar + 4 * hi + r : -1;
            bool fix = a.correct && lstar >= 0;
            log_event(a, bh, FTATTN_CHECK_O, -1, row, col, R[r], fix ? 1 : 0);
            if (fix) {
              float rest = 0.f;
#pragma unroll
              for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
                for (int gg = 0; gg < 4; ++gg)
                  if (4 * fb + gg != lstar) rest += o[g][fb][4 * gg + r];
              float val = chk1 - rest;
#pragma unroll
              for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
                for (int gg = 0; gg < 4; ++gg)
                  if (4 * fb + gg == lstar) o[g][fb][4 * gg + r] = val;
            }
          }
        }
      }
    }
    // ---- store: lane holds features 32*fb + 8*gg + 4*hi + (0..3) of its query
    if (real) {
      size_t base = ((size_t)bh * N + row) * D;
#pragma unroll
      for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {
          int f = 32 * fb + 8 * gg + 4 * hi;
          float x0 = o[g][fb][4 * gg], x1 = o[g][fb][4 * gg + 1], x2 = o[g][fb][4 * gg + 2], x3 = o[g][fb][4 * gg + 3];
          if (a.out_dtype == FTATTN_F32) {
            float4 v = make_float4(x0, x1, x2, x3);
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.o) + base + f) = v;
          } else if (a.out_dtype == FTATTN_F16) {
            _Float16 hv[4] = {(_Float16)x0, (_Float16)x1, (_Float16)x2, (_Float16)x3};
            *reinterpret_cast<uint2*>(reinterpret_cast<_Float16*>(a.o) + base + f) = *reinterpret_cast<uint2*>(hv);
          } else {
            uint32_t u[4] = {as_u(x0), as_u(x1), as_u(x2), as_u(x3)};
            uint16_t bv16[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              uint32_t rnd = ((u[i] >> 16) & 1u) + 0x7FFFu;
              bv16[i] = (u[i] & 0x7F800000u) == 0x7F800000u ? (uint16_t)(u[i] >> 16) : (uint16_t)((u[i] + rnd) >> 16);
            }
            *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.o) + base + f) = *reinterpret_cast<uint2*>(bv16);
          }
        }
    }
  }

  if (FT) {
    // largest statistics that passed, per row tile (non-negative floats order like their bits)
    uint32_t* rm = a.resmax + ((size_t)bh * a.Ti + ti) * 4;
    float vals[4] = {dev_max, rmax_o, rmax_u, rmax_l};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float v = vals[i];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v = fmax2(v, __shfl_xor(v, off));
      if (lane == 0) atomicMax(rm + i, as_u(v));
    }
    if (lane == 0 && rechecks) atomicAdd(a.recheck, (unsigned long long)rechecks);
  }
}

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
