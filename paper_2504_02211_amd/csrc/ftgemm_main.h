// Fault-tolerant linear layer Y = X W^T for gfx950 / CDNA4: the strided ABFT of Section 3.3 of
// the paper (tensor checksums of eq. (13), (14); checksum products of eq. (15), (16); location
// and repair as stated after eq. (16)) on a plain fp16 or bf16 GEMM with fp32 accumulation.
//
// Execution shape.  One workgroup computes a 256-token x 256-feature tile of Y; the 256 features
// are exactly one checksum block.  Eight waves of 64 lanes; wave w owns tokens 32w .. 32w+31 and
// ALL 256 features of the tile, as eight 32x32 accumulator blocks of Y^T = W X^T (32x32x16 fp16
// or bf16 MFMA: the weight rows are the A operand, the token rows the B operand) plus one block for the
// 32 checksum rows.  A lane then holds one token (column lane%32) and, per block, the features
// 8*g + 4*(lane/32) + r: feature index mod 8 is 4*(lane/32)+r, so all 32 folds of the four
// checksum classes a lane sees are in the lane's own registers and verification, location and
// repair need no exchange between lanes or waves (the property the strided layout is built for).
//
// The K dimension is walked in steps of 64 through two LDS stages filled by direct global-to-LDS
// loads; the tiles are stored unpadded with the 16-byte chunk index XOR-ed with a function of the
// row, which keeps the MFMA operand reads free of bank conflicts.
#pragma once
#include "ftattn_main.h"
#include "ftgemm.h"

namespace ftgemm {

using ftattn::half8;
using ftattn::float16v;
using ftattn::as_u;
using ftattn::as_f;
using ftattn::fmax2;
using ftattn::finitef;
using ftattn::flip_if;
using ftattn::wave_any;
using ftattn::gload_lds16_off;
using ftattn::wait_vmcnt;
using ftattn::phase_barrier;

constexpr int GBM = 256;      // tokens per workgroup tile
constexpr int GBN = 256;      // output features per workgroup tile = one checksum block
constexpr int GBK = 64;       // K step
constexpr int GCK = 32;       // checksum rows per block: {c1 hi, c1 lo, c2 hi, c2 lo} x 8 classes
constexpr int GFOLD = GBN / 8;
constexpr int GWAVES = 8;     // waves per workgroup
constexpr int ROWB = GBK * 2; // bytes per tile row in LDS

struct GFault { int32_t row, col, bit; };

typedef __bf16 bf8 __attribute__((ext_vector_type(8)));

// 16-bit storage helpers (fp16 or bf16 bit patterns)
template <bool BF> __device__ __forceinline__ float to_f32(uint16_t u) {
  if (BF) return as_f((uint32_t)u << 16);
  return (float)__builtin_bit_cast(_Float16, u);
}
// round-to-nearest-even to the storage type (Inf / NaN pass through)
template <bool BF> __device__ __forceinline__ uint16_t from_f32(float x) {
  if (!BF) return __builtin_bit_cast(uint16_t, (_Float16)x);
  const uint32_t u = as_u(x);
  if ((u & 0x7F800000u) == 0x7F800000u) return (uint16_t)(u >> 16);
  return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

struct GArgs {
  const uint16_t* x;       // [M][K] fp16 or bf16 patterns
  const uint16_t* w;       // [N][K]
  const uint16_t* wc;      // [Tn][GCK][K] checksum rows of W, same type
  void* y;                 // [M][N] fp32, or the input type
  int32_t out_dtype;
  int32_t M, N, K, Tm, Tn;
  float tau_rel, tau_abs;
  int32_t correct;
  const GFault* faults;
  int32_t n_faults;
  ftgemm_event* events;
  int32_t* ev_count;
  int32_t max_events;
  uint32_t* resmax;        // float bits of a non-negative value
  // batch of independent products (blockIdx.y): element strides between consecutive problems of x, w,
  // wc and the event log, byte stride of y; counters and residual maxima are one per problem.  All
  // zero for a single product.
  long long bs_x, bs_w, bs_wc, bs_y_bytes, bs_events;
  int32_t skip_upper;      // 1: output tiles that lie entirely above the diagonal (first feature > last token) are
                           // not computed and not written (the score matrix of a causal attention: nobody reads them)
  int32_t k_lower;         // 1: x is lower-triangular (the weights of a causal attention): contraction steps beyond the
                           // last token of the tile multiply zeros and are skipped
  int32_t transposed;      // 1: the kernel's (token, feature) is the caller's (column, row) of Y: checksums over the
                           // caller's token rows; results are stored, and events named, with the two exchanged
};

template <bool FT> struct GStage {
  static constexpr int XBYTES = GBM * ROWB;
  static constexpr int WBYTES = GBN * ROWB;
  static constexpr int CBYTES = FT ? GCK * ROWB : 0;
  static constexpr int BYTES = XBYTES + WBYTES + CBYTES;
  static constexpr int NLOAD = FT ? 9 : 8;        // 1 KB load instructions per wave and stage
  // 1 KB behind the two stages takes the loads of pieces that do not exist (no further K step,
  // or a wave without a checksum piece), so that every wave issues the same instructions
  static constexpr int DUMP = 1024;
  static constexpr int LDS_TOTAL = 2 * BYTES + DUMP;
};

// Tensor checksums of the weight rows of every 256-feature block (eq. (13), (14)): thread =
// (class c, 16-byte chunk of K); it folds the 32 rows c, c+8, ... of its block in fp32 and
// stores each of the two sums as a high word and a low word of the input type (high = the sum
// rounded, low = the remainder rounded).  Rows beyond N count as zero.
template <bool BF>
__global__ __launch_bounds__(256) void ftgemm_encode_w(const uint16_t* __restrict__ w, uint16_t* __restrict__ wc,
                                                       int N, int K, long long bs_w = 0, long long bs_wc = 0) {
  typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));
  w += (size_t)blockIdx.z * bs_w;        // batch of weight matrices
  wc += (size_t)blockIdx.z * bs_wc;
  const int tn = blockIdx.x, tid = threadIdx.x;
  const int cls = tid >> 5, ch = blockIdx.y * 32 + (tid & 31);
  if (ch * 8 >= K) return;
  float c1[8], c2[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { c1[e] = 0.f; c2[e] = 0.f; }
  for (int l = 0; l < GFOLD; ++l) {
    const int n = tn * GBN + cls + 8 * l;
    if (n >= N) break;
    const u16x8 h = *reinterpret_cast<const u16x8*>(w + (size_t)n * K + ch * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float v = to_f32<BF>(h[e]);
      c1[e] += v;
      c2[e] += (float)(l + 1) * v;
    }
  }
  u16x8 w0, w1, w2, w3;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    w0[e] = from_f32<BF>(c1[e]); w1[e] = from_f32<BF>(c1[e] - to_f32<BF>(w0[e]));
    w2[e] = from_f32<BF>(c2[e]); w3[e] = from_f32<BF>(c2[e] - to_f32<BF>(w2[e]));
  }
  uint16_t* out = wc + (size_t)tn * GCK * K + ch * 8;
  *reinterpret_cast<u16x8*>(out + (size_t)(cls) * K) = w0;
  *reinterpret_cast<u16x8*>(out + (size_t)(8 + cls) * K) = w1;
  *reinterpret_cast<u16x8*>(out + (size_t)(16 + cls) * K) = w2;
  *reinterpret_cast<u16x8*>(out + (size_t)(24 + cls) * K) = w3;
}

static __global__ void ftgemm_reset(int32_t* ev_count, uint32_t* resmax) {
  if (threadIdx.x == 0 && blockIdx.x == 0) { *ev_count = 0; *resmax = 0u; }
}

__device__ __forceinline__ void log_gemm_event(const GArgs& a, int row, int col, float res, int action) {
  int idx = atomicAdd(a.ev_count, 1);
  if (idx < a.max_events) {
    ftgemm_event e;
    e.row = a.transposed ? col : row; e.col = a.transposed ? row : col; e.residual = res; e.action = action;
    a.events[idx] = e;
  }
}

// RAG: K is not a multiple of the K step (the last step is partly empty); a separate instantiation so that the
// regular case carries none of its selects
template <bool FT, bool INJ, bool BF, bool RAG = false>
__global__ __launch_bounds__(GWAVES * 64) void ftgemm_main(const GArgs a0) {
  GArgs a = a0;
  {
    const size_t by = blockIdx.y;          // problem of the batch
    a.x += by * a0.bs_x; a.w += by * a0.bs_w; a.wc += by * a0.bs_wc;
    a.y = reinterpret_cast<char*>(a0.y) + by * a0.bs_y_bytes;
    a.events += by * a0.bs_events; a.ev_count += by; a.resmax += by;
  }
  using S = GStage<FT>;
  constexpr int NA = FT ? 9 : 8;          // A operands (32-row blocks of W, + the checksum block) per k-step
  constexpr int NKS = GBK / 16;           // k-steps of 16 per stage
  constexpr int NOPS = NKS * NA;
  constexpr int RING = 6;
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  // ---- workgroup -> output tile.  Workgroup ids go round-robin over the 8 XCDs; each XCD gets a
  // contiguous range of tiles, and tiles are numbered in groups of 8 token tiles x all feature
  // tiles, feature-major inside a group, so that the workgroups an XCD runs together share
  // weight rows and token rows in its L2.
  const int total = gridDim.x;
  int logical;
  {
    int id = blockIdx.x, xcd = id & 7, slot = id >> 3, qn = total >> 3, rn = total & 7;
    logical = xcd * qn + (xcd < rn ? xcd : rn) + slot;
  }
  int tm, tn;
  {
    constexpr int GM = 8;
    const int gsz = GM * a.Tn, g = logical / gsz, first = g * GM;
    const int gm = a.Tm - first < GM ? a.Tm - first : GM;
    const int in_g = logical - g * gsz;
    tm = first + in_g % gm;
    tn = in_g / gm;
  }
  const int tid = threadIdx.x, lane = tid & 63, lq = lane & 31, hi = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int M = a.M, N = a.N, K = a.K;
  const int m0 = tm * GBM, n0 = tn * GBN;
  if (a.skip_upper && n0 > m0 + GBM - 1) return;      // (the whole workgroup, before any barrier)
  const int nkb = (K + GBK - 1) / GBK;
  const int krem = K - (nkb - 1) * GBK;     // columns of the last K step (GBK unless K is ragged; K is a multiple of 8)
  const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;

  // ---- per-lane source offsets of this wave's load instructions.  Instruction `ins` of a stage
  // fills LDS bytes [1024*ins, 1024*ins + 1024): 32 of them cover the token rows, 32 the weight
  // rows, 4 the checksum rows.  Rows beyond the matrix are clamped to its last row (their
  // results are never used).  In the last K step of a ragged K a chunk beyond column K is fetched
  // from the first chunk of that step instead (valid memory); its products are switched off by
  // zeroing the token operand of those columns below.
  uint32_t off[S::NLOAD], offl[S::NLOAD];
#pragma unroll
  for (int i = 0; i < S::NLOAD; ++i) {
    const int ins = wave + 8 * i;
    int L, r, rows_left;
    if (i < 4) { L = ins * 64 + lane; rows_left = M - m0; }
    else if (i < 8) { L = (ins - 32) * 64 + lane; rows_left = N - n0; }
    else { L = ((ins - 64) & 3) * 64 + lane; rows_left = GCK; }
    r = L >> 3;
    const int c = (L & 7) ^ ((r >> 1) & 7);
    if (r > rows_left - 1) r = rows_left - 1;
    off[i] = ((uint32_t)r * (uint32_t)K + (uint32_t)c * 8u) * 2u;
    offl[i] = RAG ? ((uint32_t)r * (uint32_t)K + (c * 8 < krem ? (uint32_t)c * 8u : 0u)) * 2u : off[i];
  }
  const uint16_t* xb = a.x + (size_t)m0 * K;
  const uint16_t* wb = a.w + (size_t)n0 * K;
  const uint16_t* cb = FT ? a.wc + (size_t)tn * GCK * K : a.w;
  const uint32_t dump = smem_base + 2u * S::BYTES;
  auto issue_piece = [&](int i, int kb, int st, bool real_piece) __attribute__((always_inline)) {
    const bool ok = real_piece && (i < 8 || wave < 4);
    const uint32_t dst = ok ? smem_base + (uint32_t)st * S::BYTES + (uint32_t)(wave + 8 * i) * 1024u : dump;
    const size_t koff = real_piece ? (size_t)kb * GBK : 0;
    const uint32_t o = RAG && kb >= nkb - 1 ? offl[i] : off[i];      // (the loads that go to the dump area stay inside the rows too)
    if (i < 4) gload_lds16_off(xb + koff, o, dst);
    else if (i < 8) gload_lds16_off(wb + koff, o, dst);
    else gload_lds16_off(cb + koff, o, dst);
  };

  float16v acc[8], sc;
#pragma unroll
  for (int y = 0; y < 8; ++y) acc[y] = (float16v)0.f;
  sc = (float16v)0.f;

  // operand addresses inside a stage: row 32*y + lq of the weight tile (row 256 + lq: checksum
  // rows), row 32*wave + lq of the token tile, chunk (2*ks + hi) XOR-ed with (row/2)%8
  const int swz = (lq >> 1) & 7;
  const char* wrow = smem + S::XBYTES + lq * ROWB;
  const char* xrow = smem + (32 * wave + lq) * ROWB;

#pragma unroll
  for (int i = 0; i < S::NLOAD; ++i) issue_piece(i, 0, 0, true);

  int nkb_run = nkb;                       // (the ragged-K handling below stays keyed to the full count)
  if (a.k_lower) { const int lim = (m0 + GBM + GBK - 1) / GBK; nkb_run = lim < nkb ? lim : nkb; }
  for (int kb = 0; kb < nkb_run; ++kb) {
    const int st = kb & 1;
    wait_vmcnt<0>();                       // this wave's pieces of stage st have landed
    phase_barrier();                       // ... everyone's; and everyone is done reading the other stage
    const bool more = kb + 1 < nkb_run;
    const char* wst = wrow + st * S::BYTES;
    const char* xst = xrow + st * S::BYTES;
    half8 xf[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) xf[ks] = *reinterpret_cast<const half8*>(xst + (((2 * ks + hi) ^ swz) << 4));
    if (RAG && kb == nkb - 1) {
      // ragged K: the columns beyond K take no part (whatever the weight operand holds there)
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks)
        if ((2 * ks + hi) * 8 >= krem) xf[ks] = (half8)(_Float16)0.f;
    }
    half8 buf[RING];
    auto load_op = [&](int k) __attribute__((always_inline)) -> half8 {
      const int ks = k / NA, y = k % NA;
      return *reinterpret_cast<const half8*>(wst + y * (32 * ROWB) + (((2 * ks + hi) ^ swz) << 4));
    };
#pragma unroll
    for (int k = 0; k < RING - 1; ++k) buf[k] = load_op(k);
#pragma unroll
    for (int k = 0; k < NOPS; ++k) {
      if (k + RING - 1 < NOPS) buf[(k + RING - 1) % RING] = load_op(k + RING - 1);
      // the next stage is requested at the start of this one: its latency budget is one K step
      if (k < S::NLOAD) issue_piece(k, kb + 1, st ^ 1, more);
      const half8 av = buf[k % RING];
      const int ks = k / NA, y = k % NA;
      float16v& dst = y < 8 ? acc[y] : sc;
      if (BF) dst = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf8, av), __builtin_bit_cast(bf8, xf[ks]), dst, 0, 0, 0);
      else dst = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, xf[ks], dst, 0, 0, 0);
    }
  }

  wait_vmcnt<0>();                         // (the last step's loads went to the dump area)

  // ================= after the last accumulation step: injection, verification, repair, store
  const int row = m0 + 32 * wave + lq;
  const bool real = row < M;
  // features beyond N (clamped weight rows) must not enter the folds
  if (n0 + GBN > N) {
#pragma unroll
    for (int y = 0; y < 8; ++y)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int col = n0 + 32 * y + 8 * (v >> 2) + 4 * hi + (v & 3);
        if (col >= N) acc[y][v] = 0.f;
      }
  }
  if (INJ) {
    for (int fi = 0; fi < a.n_faults; ++fi) {
      const GFault f = a.faults[fi];
      const int lc = f.col - n0;
      if (lc < 0 || lc >= GBN) continue;
      const bool mine = f.row == row && hi == ((lc & 7) >> 2);
      const int ty = lc >> 5, tv = 4 * ((lc & 31) >> 3) + (lc & 3);
#pragma unroll
      for (int y = 0; y < 8; ++y)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[y][v] = flip_if(acc[y][v], mine && ty == y && tv == v, f.bit);
    }
  }
  if (FT) {
    // fold of the 32 results of each class against the first checksum product (eq. (15))
    bool bad = false, det[4];
    float stat_max = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float sum1 = 0.f, mag = 0.f;
#pragma unroll
      for (int y = 0; y < 8; ++y)
#pragma unroll
        for (int g = 0; g < 4; ++g) { sum1 += acc[y][4 * g + r]; mag += __builtin_fabsf(acc[y][4 * g + r]); }
      const float R = (sc[r] + sc[4 + r]) - sum1;
      const float thr = a.tau_abs + a.tau_rel * mag;
      det[r] = real && (!(__builtin_fabsf(R) <= thr) || !finitef(R));
      bad |= det[r];
      if (!det[r] && real && thr > 0.f) stat_max = fmax2(stat_max, __builtin_fabsf(R) / thr);
    }
    if (wave_any(bad)) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (!det[r]) continue;
        const float chk1 = sc[r] + sc[4 + r], chk2 = sc[8 + r] + sc[12 + r];
        float sum1 = 0.f, sum2 = 0.f, big = -1.f;
        int l_big = -1;
#pragma unroll
        for (int y = 0; y < 8; ++y)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const float v = acc[y][4 * g + r];
            sum1 += v;
            sum2 += (float)(4 * y + g + 1) * v;
            const float m = finitef(v) ? __builtin_fabsf(v) : __builtin_inff();
            if (m > big) { big = m; l_big = 4 * y + g; } else if (m == big) { l_big = -1; }
          }
        const float r1 = chk1 - sum1;
        const float ratio = (chk2 - sum2) / r1;
        int lstar = -1;
        if (finitef(ratio)) {
          const float c = __builtin_rintf(ratio) - 1.0f;
          if (c >= 0.f && c < (float)GFOLD) lstar = (int)c;
        } else {
          lstar = l_big;        // residuals left the fp32 range: the fold of overwhelming size
        }
        int col = lstar >= 0 ? n0 + 8 * lstar + 4 * hi + r : -1;
        if (col >= N) { col = -1; lstar = -1; }
        const bool fix = a.correct && lstar >= 0;
        log_gemm_event(a, row, col, r1, fix ? 1 : 0);
        if (fix) {
          float rest = 0.f;
#pragma unroll
          for (int y = 0; y < 8; ++y)
#pragma unroll
            for (int g = 0; g < 4; ++g)
              if (4 * y + g != lstar) rest += acc[y][4 * g + r];
          const float val = chk1 - rest;
#pragma unroll
          for (int y = 0; y < 8; ++y)
#pragma unroll
            for (int g = 0; g < 4; ++g)
              if (4 * y + g == lstar) acc[y][4 * g + r] = val;
        }
      }
    }
    float v = stat_max;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmax2(v, __shfl_xor(v, o));
    if (lane == 0 && v > 0.f) atomicMax(a.resmax, as_u(v));
  }

  // ---- store: the lane holds features n0 + 32*y + 8*g + 4*hi + (0..3) of its token
  if (real && a.transposed) {
    // Y is [N][M] seen from here: consecutive lanes (tokens) write consecutive elements of one row
#pragma unroll
    for (int y = 0; y < 8; ++y)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int col = n0 + 32 * y + 8 * (v >> 2) + 4 * hi + (v & 3);
        if (col < N) {
          const size_t at = (size_t)col * M + row;
          if (a.out_dtype == FTGEMM_F32) reinterpret_cast<float*>(a.y)[at] = acc[y][v];
          else reinterpret_cast<uint16_t*>(a.y)[at] = from_f32<BF>(acc[y][v]);
        }
      }
  } else if (real) {
    const size_t base = (size_t)row * N;
    const bool vec = (N & 3) == 0;
#pragma unroll
    for (int y = 0; y < 8; ++y)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + 32 * y + 8 * g + 4 * hi;
        const float x0 = acc[y][4 * g], x1 = acc[y][4 * g + 1], x2 = acc[y][4 * g + 2], x3 = acc[y][4 * g + 3];
        if (vec && col + 3 < N) {
          if (a.out_dtype == FTGEMM_F32) {
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.y) + base + col) = make_float4(x0, x1, x2, x3);
          } else {
            uint16_t hv[4] = {from_f32<BF>(x0), from_f32<BF>(x1), from_f32<BF>(x2), from_f32<BF>(x3)};
            *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.y) + base + col) = *reinterpret_cast<uint2*>(hv);
          }
        } else {
          const float xs[4] = {x0, x1, x2, x3};
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (col + e < N) {
              if (a.out_dtype == FTGEMM_F32) reinterpret_cast<float*>(a.y)[base + col + e] = xs[e];
              else reinterpret_cast<uint16_t*>(a.y)[base + col + e] = from_f32<BF>(xs[e]);
            }
        }
      }
  }
}

// Launch helpers defined next to the kernels' instantiations (ftgemm.hip), for other host code of
// the library that runs the same protected product on buffers of its own (the decoupled attention
// baseline).  None of them allocates or synchronises.
hipError_t gemm_allow_lds(int k);
hipError_t gemm_launch_encode_w(const uint16_t* w, uint16_t* wc, int n, int k, bool bf16, hipStream_t st,
                                int batch = 1, long long bs_w = 0, long long bs_wc = 0);
hipError_t gemm_launch(const GArgs& a, bool ft, bool inject, bool bf16, hipStream_t st, int batch = 1);

}  // namespace ftgemm
