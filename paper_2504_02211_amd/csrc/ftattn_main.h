// The fused fault-tolerant attention kernel (gfx950 / CDNA4): Algorithm 1 of the paper from
// GEMM I to the final store, for one (batch, head, query row tile) per workgroup.
//
// Execution shape.  Wave w of a workgroup owns queries 32w .. 32w+31 of the row tile.
//  * head_dim 128: eight waves (256-query row tiles), one workgroup per CU.  The waves form two
//    groups of four (one wave of each group per SIMD) that run half an iteration apart: while one
//    group is in its MATRIX phase (GEMM II of key tile i and GEMM I of key tile i+1, back to back
//    on the MFMA pipe) the other is in its SOFTMAX phase (max, exp, product-form check, row-sum,
//    rescale: vector ALU only), and at every workgroup barrier they trade places.  Key / value
//    tiles arrive in LDS by direct global-to-LDS loads into a ring of three stages.
//  * head_dim 64: four waves (128-query row tiles), two independent workgroups per CU, so that a
//    SIMD again holds two waves, which the hardware interleaves as it finds them; one barrier per
//    iteration, a ring of two stages.  With the smaller head the softmax phase is about twice the
//    matrix phase, and the strict alternation would leave the matrix pipe and one of the two waves
//    idle half of the time; free-running waves keep the vector ALU busy from both.
// In either shape stage u of the ring holds V_u^T and K_{u+1}, the two operands one matrix phase reads.
//
// Register layout: see ftattn_device.h (scores transposed, one query per lane, the four
// stride-8 checksum classes of a lane and all their folds in the lane's own registers).
#pragma once
#include "ftattn_device.h"

namespace ftattn {

// waves per workgroup, query rows per workgroup and ring stages, by head_dim (see above)
constexpr int nwave_of(int d) { return d == 64 ? 4 : 8; }
constexpr int bm_of(int d) { return nwave_of(d) * 32; }
constexpr int nstage_of(int d) { return nwave_of(d) == 8 ? 3 : 2; }

template <int D, bool FT> struct Unit {
  static constexpr int KROWS = FT ? BN + CKR : BN;
  static constexpr int VROWS = FT ? D + CKR : D;
  static constexpr int KBYTES = KROWS * D * 2;
  static constexpr int VBYTES = VROWS * BN * 2;
  static constexpr int BYTES = KBYTES + VBYTES;
  static constexpr int K_INSTR = KBYTES / 1024;     // one instruction moves 64 lanes x 16 bytes
  static constexpr int V_INSTR = VBYTES / 1024;
  static constexpr int NWAVE = nwave_of(D), NSTAGE = nstage_of(D);
  static constexpr int KPW = (K_INSTR + NWAVE - 1) / NWAVE;
  static constexpr int VPW = (V_INSTR + NWAVE - 1) / NWAVE;
  // Every wave issues NLOAD instructions per unit; a wave that has no real piece left (uneven
  // split, or no further unit to fetch) aims the instruction at a 1 KB dump area behind the ring,
  // so that the counted waits below hold for every wave in every iteration.
  static constexpr int NLOAD = KPW + VPW;
  static constexpr int DUMP = 1024;
  static constexpr int LDS_TOTAL = NSTAGE * BYTES + DUMP;
  static_assert(K_INSTR >= NWAVE && V_INSTR >= NWAVE, "every wave owns at least one piece of each tile");
  static_assert((NSTAGE - 1) * NLOAD <= 15, "counted waits use a 4-bit immediate");
  static_assert(NWAVE == 8 || 2 * LDS_TOTAL <= 160 * 1024, "two workgroups per CU");
};

// 16 bytes per lane from (uniform base + per-lane byte offset) straight into LDS at
// (uniform LDS address + 16*lane).  Opaque to the compiler on purpose (see gload_lds16 above); no
// memory clobber, so that operand reads of other ring stages may be scheduled around it.  Ordering
// against barriers and counted waits is kept because all of them are side-effecting instructions.
__device__ __forceinline__ void gload_lds16_off(const void* base, uint32_t byte_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_addr) : "m0");
}

struct yes { static constexpr bool value = true; };
struct no { static constexpr bool value = false; };

template <int N> __device__ __forceinline__ void wait_vmcnt() { __builtin_amdgcn_s_waitcnt(0x0F70 | N); }

__device__ __forceinline__ void phase_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
}

// Value that the compiler must take as new: a second evaluation built on it is not merged with the first.
__device__ __forceinline__ float opaque(float x) { asm volatile("" : "+v"(x)); return x; }
__device__ __forceinline__ half2v opaque(half2v x) { asm volatile("" : "+v"(x)); return x; }

// PS >= 1: verification after every step (the paper's EFTA before the unified verification of
// Section 3.4): GEMM I is verified on its own in every iteration, the row-sum against its range
// and the unnormalised output accumulator against its checksum after every GEMM II.
// PS == 2: in addition the softmax is protected by duplication (eq. (11), (12)) instead of the
// product-form check and the range restriction: maximum, exponentials and reduce-sum are
// evaluated twice and compared bit by bit; a third evaluation settles a difference.
// PS == 3: unified verification with the traditional checksum instead of the strided one (the
// comparison of Section 3.3 / 4.2): one class over the whole tile row (64 keys) and one over all
// features, i.e. stride 1 in eq. (13).  Its checksum values are the sums over the eight stride-8
// classes of the same encoded tiles (c1 = sum_c c1_c, c2 = sum_c 8 c2_c + (c - 7) c1_c), so the
// matrix work is the same; what changes is that a row has one residual per key tile, formed by
// the two lanes of a query together, and can name one element of 64 (of D for the output).
template <int D, bool FT, bool CAUSAL, bool INJ, int PS = 0>
__global__ __launch_bounds__(nwave_of(D) * 64, nwave_of(D) == 8 ? 1 : 2) void ftattn_main(const KArgs a) {
  static_assert(FT || PS == 0 || PS == 4, "the verification modes are modes of the protected kernel");
  constexpr bool DMR = PS == 2;
  constexpr bool STEP = PS == 1 || PS == 2;
  constexpr bool EW = PS == 3;
  // PS == 4 (an extension): the subtracted maximum is a reference that is renewed only when the running
  // maximum exceeds it by more than a margin; in all other iterations the rescale factor is exactly
  // one and the rescale of the output falls away.  Exponentials then reach e^margin; every identity of
  // Algorithm 1 holds with the reference in place of the maximum (Section 3.4, case 1).
  constexpr bool LAZY = PS == 4;
  using U = Unit<D, FT>;
  constexpr int NWAVE = U::NWAVE, BM = NWAVE * 32, NSTAGE = U::NSTAGE;
  constexpr bool ALT = NWAVE == 8;      // two wave groups alternating between the phases (else: free-running waves)
  constexpr int NSLAB = D / 16;     // k-slabs of GEMM I
  constexpr int NFB = D / 32;       // 32-feature blocks of O^T
  constexpr int NFOLD_V = D / 8;
  constexpr int KCH = D / 8;        // 16-byte chunks per key row
  constexpr int KT_ELEMS = (BN + CKR) * D, VT_ELEMS = (D + CKR) * BN;
  extern __shared__ __attribute__((aligned(1024))) char smem[];

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
  const int grp = ALT ? wave >> 2 : 0;
  const int N = a.N;
  const int row0_cta = ti * BM;
  const int row0_w = row0_cta + wave * 32;
  const int last_row_cta = (row0_cta + BM < N ? row0_cta + BM : N) - 1;
  const int nj = CAUSAL ? (last_row_cta / BN + 1) : a.Tj;         // key tiles of the workgroup
  int nj_w = 0;                                                   // key tiles this wave takes part in
  if (row0_w < N) {
    int last_row_w = (row0_w + 32 < N ? row0_w + 32 : N) - 1;
    nj_w = CAUSAL ? (last_row_w / BN + 1) : a.Tj;
  }
  const int row = row0_w + lq;
  const float sl2 = a.scale_log2;

  const _Float16* kc_head = a.kc + (size_t)bh * a.Tj * KT_ELEMS;
  const _Float16* vt_head = a.vt + (size_t)bh * a.Tj * VT_ELEMS;
  const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;

  // ---- per-lane source offsets of this wave's load instructions (the same for every tile).
  // Instruction wave + 8*i of a tile reads rows 512/chunks-per-row further down than instruction
  // wave, i.e. 8192 bytes further in either tile, and the swizzle of a row does not change over
  // that distance: one offset per tile kind is kept, the rest is added to the scalar base.
  uint32_t koff0, voff0;
  {
    const int L = wave * 64 + lane;
    const int rk = L / KCH, ck = (L % KCH) ^ swz_k<D>(rk);
    koff0 = (uint32_t)(rk * D + ck * 8) * 2u;
    const int rv = L / 8, cv = (L % 8) ^ swz_v(rv);
    voff0 = (uint32_t)(rv * BN + cv * 8) * 2u;
  }
  constexpr int PIECE_STEP = NWAVE * 64 * 8;      // halfs between the sources of consecutive pieces of a wave
  static_assert((NWAVE * 64 / KCH) * D == PIECE_STEP && (NWAVE * 64 / 8) * BN == PIECE_STEP, "piece stride");
  // unit u = { V_u^T, K_{u+1} } goes to stage (u+1) mod 3.  A unit is fetched in NLOAD pieces per
  // wave; the pieces of one unit are spread over a matrix phase (see matrix_stream).
  uint32_t ld_lds = 0;
  const _Float16* ld_kt = kc_head;
  const _Float16* ld_vt = vt_head;
  bool ld_real = false;
  const uint32_t dump = smem_base + (uint32_t)NSTAGE * U::BYTES;
  auto prepare_unit = [&](int u, bool real) __attribute__((always_inline)) {
    const int st = (u + 1) % NSTAGE;
    ld_lds = smem_base + (uint32_t)st * U::BYTES;
    const int jk = u + 1 < a.Tj ? u + 1 : a.Tj - 1, jv = u > 0 ? (u < a.Tj ? u : a.Tj - 1) : 0;
    ld_kt = kc_head + (size_t)jk * KT_ELEMS;
    ld_vt = vt_head + (size_t)jv * VT_ELEMS;
    ld_real = real;
  };
  auto issue_piece = [&](int n) __attribute__((always_inline)) {
    if (n < U::KPW) {
      const int ins = wave + NWAVE * n;
      const bool have = (n + 1) * NWAVE <= U::K_INSTR || ins < U::K_INSTR;     // (a piece this wave does not have reads piece 0 again)
      const bool ok = ld_real && have;
      gload_lds16_off(ld_kt + (have ? n * PIECE_STEP : 0), koff0, ok ? ld_lds + (uint32_t)ins * 1024u : dump);
    } else {
      const int m = n - U::KPW, ins = wave + NWAVE * m;
      const bool have = (m + 1) * NWAVE <= U::V_INSTR || ins < U::V_INSTR;
      const bool ok = ld_real && have;
      gload_lds16_off(ld_vt + (have ? m * PIECE_STEP : 0), voff0, ok ? ld_lds + (uint32_t)U::KBYTES + (uint32_t)ins * 1024u : dump);
    }
  };
  auto issue_unit = [&](int u, bool real) __attribute__((always_inline)) {
    prepare_unit(u, real);
#pragma unroll
    for (int n = 0; n < U::NLOAD; ++n) issue_piece(n);
  };

  // faults of this workgroup
  int fcur = 0, fend = 0;
  const DevFault* __restrict__ F = a.faults;
  if (INJ && a.fault_off != nullptr) { fcur = a.fault_off[bh * a.Ti + ti]; fend = a.fault_off[bh * a.Ti + ti + 1]; }

  issue_unit(-1, true);
  issue_unit(0, true);
  if (ALT) issue_unit(1, nj >= 2);

  // ---- Q_i^T as MFMA B operand: lane (query lq, half hi) holds Q[row][16*slab + 8*hi .. +7]
  // (bf16 queries are converted here: exact for magnitudes in the fp16 normal range)
  half8 qf[NSLAB];
  {
    const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q) + ((size_t)bh * N + (row < N ? row : 0)) * D + 8 * hi;
    uint32_t qbits = 0u;
#pragma unroll
    for (int sl = 0; sl < NSLAB; ++sl) {
      uint4v raw = *reinterpret_cast<const uint4v*>(qp + 16 * sl);
      if (row >= N) raw = (uint4v)0u;
      if (a.q_bf16) qbits |= bf16_range_bits(raw);
      qf[sl] = to_half8(raw, a.q_bf16 != 0);
    }
    if (qbits) atomicOr(a.range, qbits);
  }

  float16v o[NFB], oc, s[2], sc;
  half8 ph[2][2];             // P^T in fp16, B operand of GEMM II: [key block][8-key half]
  float p[2][16];             // exp(S - m) of the key tile in flight, fp32
  float ps[2][2];             // its row-sum, one partial per quarter
  float ps2[2][2];            // (duplication mode) the second evaluation of the same
  float l2_part = 0.f, l_prev = 0.f;
  float al = 1.f;             // e^{m_old - m_new} of the key tile in flight
#pragma unroll
  for (int fb = 0; fb < NFB; ++fb) o[fb] = (float16v)0.f;
  oc = (float16v)0.f;
  float m_run = -__builtin_inff(), l_part = 0.f, l_low = 0.f, dev_max = 0.f;
  float m_true = -__builtin_inff();       // (LAZY) the running maximum; m_run is then the reference
  // the maximum to subtract after a key tile whose maximum is mxv (Algorithm 1: m_ij = max(m_i,j-1, rowmax))
  auto renewed = [&](const float mxv) __attribute__((always_inline)) -> float {
    if (!LAZY) return fmax2(m_run, mxv);
    const float mt = fmax2(m_true, mxv);
    return (mt - m_run) * a.scale > a.rescale_margin ? mt : m_run;      // (a reference of -inf is always renewed)
  };
  unsigned rechecks = 0;

  // The matrix phase as one stream of (LDS operand read, MFMA) pairs: first GEMM II of a key tile,
  //   O^T += V_j^T P^T (+ checksum block; the rescale was applied in the softmax phase),
  // then GEMM I of the next key tile,
  //   S^T = K_j Q^T, checksum block = K^c Q^T  (eq. (15), (16)).
  // The wave that runs this phase has the MFMA pipe of its SIMD to itself (its partner wave is in
  // the softmax phase), so the LDS latency must be hidden inside the stream: operand k+RING-1 is
  // requested before MFMA k is issued, and the scheduler is told to keep exactly that order.
  constexpr int NA2 = FT ? NFB + 1 : NFB;      // A operands per k-step of GEMM II
  constexpr int NA1 = FT ? 3 : 2;              // A operands per k-slab of GEMM I
  constexpr int RING = 6;
  // P -> fp16 in B-operand order: registers 8n..8n+7 of key block kb feed the MFMAs of k-step
  // t = 2*kb + n of GEMM II.  The row-sum adds up the converted pairs, the values GEMM II
  // multiplies (dot product with (1, 1), fp32 accumulation).  Quarter 0 is converted at the end of
  // the softmax phase; quarters 1..3 are converted inside the matrix phase, each ahead of its
  // k-step, where the vector instructions run in the shadow of the wave's own MFMAs.
  auto convert_quarter = [&](const int t) __attribute__((always_inline)) {
    const int kb = t >> 1, n = t & 1;
    ps[kb][n] = 0.f;
#pragma unroll
    for (int x = 0; x < 8; x += 2) {
      half2v pr2;
      pr2[0] = (_Float16)p[kb][8 * n + x]; pr2[1] = (_Float16)p[kb][8 * n + x + 1];
      ph[kb][n][x] = pr2[0]; ph[kb][n][x + 1] = pr2[1];
      const half2v ones = {(_Float16)1.f, (_Float16)1.f};
      ps[kb][n] = __builtin_amdgcn_fdot2(pr2, ones, ps[kb][n], false);
      if (DMR) ps2[kb][n] = __builtin_amdgcn_fdot2(opaque(pr2), ones, x == 0 ? 0.f : ps2[kb][n], false);
    }
  };
  // reduce sum (Algorithm 1): one expression for every evaluation, so that they round alike
  auto rowsum_update = [&](float l_old, const float (&q4)[2][2]) __attribute__((always_inline)) -> float {
    return l_old * al + ((q4[0][0] + q4[0][1]) + (q4[1][0] + q4[1][1]));
  };
  // Operand addresses.  Row 32*y + lq of a K tile, chunk (2*sl + hi) XOR swizzle(lq), is at
  //   (tile + lq*row_bytes + ((hi ^ swizzle) << 4)) ^ (sl << 5), plus y*32 rows as an immediate:
  // the XOR only touches the chunk bits because every tile starts at a multiple of the row size.
  // One per-lane constant per tile kind serves all operands (likewise for V^T, whose chunk is
  // 4*(t>>1) + (t&1) XOR 2*hi); nothing per-lane has to follow the ring of stages.
  const uint32_t lane_k = (uint32_t)(lq * (D * 2) + ((hi ^ swz_k<D>(lq)) << 4));
  const uint32_t lane_v = (uint32_t)(lq * (BN * 2) + (((2 * hi) ^ swz_v(lq)) << 4));
  static_assert(U::BYTES % (D * 2) == 0 && U::KBYTES % (D * 2) == 0 && U::BYTES % (BN * 2) == 0 && U::KBYTES % (BN * 2) == 0,
                "tiles start at multiples of their row size");
  auto lds_rd = [](uint32_t addr) __attribute__((always_inline)) -> half8 {
    return *reinterpret_cast<const __attribute__((address_space(3))) half8*>((uintptr_t)addr);
  };
  auto matrix_stream = [&](uint32_t bv, uint32_t bk, auto do2_tag, auto do1_tag, auto ld_tag) __attribute__((always_inline)) {
    const uint32_t ak = bk + lane_k, av0 = bv + lane_v;
    constexpr bool DO2 = decltype(do2_tag)::value, DO1 = decltype(do1_tag)::value, LD = decltype(ld_tag)::value;
    constexpr int N2 = DO2 ? 4 * NA2 : 0, N1 = DO1 ? NSLAB * NA1 : 0, NOPS = N2 + N1;
    if (DO1) {
      s[0] = (float16v)0.f; s[1] = (float16v)0.f;
      if (FT) sc = (float16v)0.f;
    }
    half8 buf[RING];
    auto load_op = [&](int k) __attribute__((always_inline)) -> half8 {
      if (k < N2) {
        const int t = k / NA2, x = k % NA2;
        return lds_rd((av0 ^ (uint32_t)((4 * (t >> 1) + (t & 1)) << 4)) + (uint32_t)(x * 32 * BN * 2));
      }
      const int kk = k - N2, sl = kk / NA1, y = kk % NA1;
      return lds_rd((ak ^ (uint32_t)(sl << 5)) + (uint32_t)(y * 32 * D * 2));
    };
#pragma unroll
    for (int k = 0; k < RING - 1 && k < NOPS; ++k) buf[k] = load_op(k);
#pragma unroll
    for (int k = 0; k < NOPS; ++k) {
      if (k + RING - 1 < NOPS) buf[(k + RING - 1) % RING] = load_op(k + RING - 1);
      // one piece of the next-but-one unit every few MFMAs, so that the memory pipeline never backs up
      if (LD && k % (NOPS / U::NLOAD) == 1 && k / (NOPS / U::NLOAD) < U::NLOAD) issue_piece(k / (NOPS / U::NLOAD));
      const half8 av = buf[k % RING];
      if (DO2 && k < 3 * NA2 && k % NA2 == 0) convert_quarter(k / NA2 + 1);     // one k-step ahead of its use
      if (DO2 && k == 3 * NA2) {
        l_part = rowsum_update(l_part, ps);
        if (DMR) l2_part = rowsum_update(opaque(l2_part), ps2);
      }
      if (k < N2) {
        const int t = k / NA2, x = k % NA2;
        if (x < NFB) o[x] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, ph[t >> 1][t & 1], o[x], 0, 0, 0);
        else oc = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, ph[t >> 1][t & 1], oc, 0, 0, 0);
      } else {
        const int kk = k - N2, sl = kk / NA1, y = kk % NA1;
        if (y < 2) s[y] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, qf[sl], s[y], 0, 0, 0);
        else sc = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, qf[sl], sc, 0, 0, 0);
      }
    }
    // pin the order: RING-1 reads, then (MFMA, read) pairs, then the remaining MFMAs
    __builtin_amdgcn_sched_group_barrier(0x100, RING - 1, 0);
#pragma unroll
    for (int k = 0; k + RING - 1 < NOPS; ++k) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, RING - 1, 0);
  };
  // Sum-form check of the output accumulator against its checksums (Algorithm 1, last "if"; text
  // after eq. (16) for location and repair): class r of the lane, folds o[fb][4*gg + r].  `thr` is
  // the threshold in the units the accumulator is in, `tile` the key tile reported with an event
  // (-1 after the loop), `xfold` / `xv` the extra fold of class 0 in the exact row-sum mode.
  float rmax_o = 0.f;
  auto sum_check = [&](const float thr, const int tile, const bool real, const bool xf, const float xv, const bool track) -> bool {
    if (EW) {
      // one class over all D features of the row (fold index = feature), from both lanes of the query
      float sum1 = 0.f, chk1 = 0.f;
#pragma unroll
      for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum1 += o[fb][v];
#pragma unroll
      for (int r = 0; r < 4; ++r) chk1 += oc[r] + oc[4 + r];
      sum1 = sum32(sum1); chk1 = sum32(chk1);
      const float R1 = chk1 - sum1;
      const bool d = real && !(__builtin_fabsf(R1) <= thr);
      if (track && !d && real) rmax_o = fmax2(rmax_o, __builtin_fabsf(R1));
      if (!wave_any(d)) return false;
      float chk2 = 0.f, sum2 = 0.f, big = -1.f;
      int l_big = -1;
#pragma unroll
      for (int r = 0; r < 4; ++r)
        chk2 += 8.0f * (oc[8 + r] + oc[12 + r]) + (float)(4 * hi + r - 7) * (oc[r] + oc[4 + r]);
#pragma unroll
      for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int l = 32 * fb + 8 * (v >> 2) + 4 * hi + (v & 3);
          const float ov = o[fb][v];
          sum2 += (float)(l + 1) * ov;
          const float mag = finitef(ov) ? __builtin_fabsf(ov) : __builtin_inff();
          if (mag > big) { big = mag; l_big = l; } else if (mag == big) { l_big = -1; }
        }
      chk2 = sum32(chk2); sum2 = sum32(sum2);
      {
        const float bigp = xchg32(big, hi);
        const int lp = (int)xchg32((float)l_big, hi);
        if (bigp > big) l_big = lp; else if (bigp == big) l_big = -1;
      }
      int lstar = -1;
      {
        const float ratio = (chk2 - sum2) / R1;
        if (finitef(ratio)) {
          const float c = __builtin_rintf(ratio) - 1.0f;
          if (c >= 0.f && c < (float)D) lstar = (int)c;
        } else {
          lstar = l_big;
        }
      }
      if (!d) lstar = -1;
      float rest = 0.f;
#pragma unroll
      for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (32 * fb + 8 * (v >> 2) + 4 * hi + (v & 3) != lstar) rest += o[fb][v];
      rest = sum32(rest);
      if (d) {
        const bool fix = a.correct && lstar >= 0;
        if (hi == 0) log_event(a, bh, FTATTN_CHECK_O, tile, row, lstar, R1, fix ? 1 : 0);
        if (fix) {
          const float val = chk1 - rest;
#pragma unroll
          for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
            for (int v = 0; v < 16; ++v)
              if (32 * fb + 8 * (v >> 2) + 4 * hi + (v & 3) == lstar) o[fb][v] = val;
        }
      }
      return true;       // events may have been written
    }
    bool bad = false;
    float R[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float sum1 = 0.f;
#pragma unroll
      for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) sum1 += o[fb][4 * gg + r];
      if (r == 0 && xf) sum1 += xv;      // the normalised extra fold of class 0
      R[r] = (oc[r] + oc[4 + r]) - sum1;
      bool d = real && !(__builtin_fabsf(R[r]) <= thr);
      bad |= d;
      if (track && !d && real) rmax_o = fmax2(rmax_o, __builtin_fabsf(R[r]));
    }
    if (wave_any(bad)) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (real && !(__builtin_fabsf(R[r]) <= thr)) {
          float chk1 = oc[r] + oc[4 + r], chk2 = oc[8 + r] + oc[12 + r];
          float sum2 = 0.f, big = -1.f;
          int l_big = -1;
#pragma unroll
          for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
              float ov = o[fb][4 * gg + r];
              sum2 += (float)(4 * fb + gg + 1) * ov;
              float mag = finitef(ov) ? __builtin_fabsf(ov) : __builtin_inff();
              if (mag > big) { big = mag; l_big = 4 * fb + gg; } else if (mag == big) { l_big = -1; }
            }
          const bool xfold = r == 0 && xf;      // class 0 has the row-sum as fold NFOLD_V
          if (xfold) {
            sum2 += (float)(NFOLD_V + 1) * xv;
            float mag = finitef(xv) ? __builtin_fabsf(xv) : __builtin_inff();
            if (mag > big) { big = mag; l_big = NFOLD_V; } else if (mag == big) { l_big = -1; }
          }
          float ratio = (chk2 - sum2) / R[r];
          int lstar = -1;
          if (finitef(ratio)) {
            float c = __builtin_rintf(ratio) - 1.0f;
            if (c >= 0.f && c < (float)(xfold ? NFOLD_V + 1 : NFOLD_V)) lstar = (int)c;
          } else {
            lstar = l_big;
          }
          if (xfold && lstar == NFOLD_V) continue;             // the row-sum itself: reported by its own check
          int col = lstar >= 0 ? 8 * lstar + 4 * hi + r : -1;
          bool fix = a.correct && lstar >= 0;
          log_event(a, bh, FTATTN_CHECK_O, tile, row, col, R[r], fix ? 1 : 0);
          if (fix) {
            float rest = xfold ? xv : 0.f;
#pragma unroll
            for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
              for (int gg = 0; gg < 4; ++gg)
                if (4 * fb + gg != lstar) rest += o[fb][4 * gg + r];
            float val = chk1 - rest;
#pragma unroll
            for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
              for (int gg = 0; gg < 4; ++gg)
                if (4 * fb + gg == lstar) o[fb][4 * gg + r] = val;
          }
        }
      }
      return true;       // events may have been written
    }
    return false;
  };

  // ---- prologue: the first key tile's scores; group 1 starts one barrier later than group 0
  wait_vmcnt<(NSTAGE - 1) * U::NLOAD>();          // unit -1 has landed
  phase_barrier();
  if (ALT && grp == 1) phase_barrier();
  if (nj_w > 0) matrix_stream(smem_base, smem_base, no{}, yes{}, no{});
  if (ALT) {
    if (grp == 1) wait_vmcnt<U::NLOAD>();         // unit 0
    phase_barrier();
  }

  for (int i = 0; i < nj; ++i) {
    const int k0 = i * BN;
    const bool on = i < nj_w;
    const uint32_t stage = smem_base + (uint32_t)((i + 1) % NSTAGE) * U::BYTES;
    const bool tile_has_fault = INJ && fcur < fend && F[fcur].kv_tile == i;

    // =========================================================== softmax phase
    if (on) {
      const bool g_mask = (CAUSAL && k0 + BN - 1 > row0_w) || (k0 + BN > N);

      // ---- injection point: raw scores
      if (tile_has_fault) {
        for (int fi = fcur; fi < fend && F[fi].kv_tile == i; ++fi) {
          if (F[fi].stage != FTATTN_ST_S) continue;
          int lr = F[fi].row - row0_w, kl = F[fi].col - k0, bit = F[fi].bit;
          bool mine = lr >= 0 && lr < 32 && lane == lr + 32 * ((kl & 7) >> 2);
          int tkb = kl >> 5, tv = 4 * ((kl & 31) >> 3) + (kl & 3);
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) s[kb][v] = flip_if(s[kb][v], mine && tkb == kb && tv == v, bit);
        }
      }

      float mx, m_new, negm;
      bool recheck = g_mask;

      if (!g_mask) {
        // ============ reduce max, exp (fast path: no masked entry in this tile)
        float m0 = fmax2(s[0][0], s[0][1]), m1 = fmax2(s[1][0], s[1][1]);
#pragma unroll
        for (int v = 2; v < 16; v += 2) {
          m0 = fmax2(fmax2(m0, s[0][v]), s[0][v + 1]);
          m1 = fmax2(fmax2(m1, s[1][v]), s[1][v + 1]);
        }
        mx = max32(fmax2(m0, m1));
        m_new = renewed(mx);
        negm = -m_new * sl2;
        // all 32 arguments first, then all 32 exponentials, in place: neighbouring instructions are
        // independent, where (argument, exponential) pairs through one temporary would each wait
        // for the other
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) p[kb][v] = __builtin_fmaf(s[kb][v], sl2, negm);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) p[kb][v] = ex2(p[kb][v]);
      } else {
        // ============ same with the causal / sequence-end mask applied per element
        mx = -__builtin_inff();
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            int key = k0 + key_of(kb, v, hi);
            bool ok = key < N && (!CAUSAL || key <= row);
            mx = fmax2(mx, ok ? s[kb][v] : -__builtin_inff());
          }
        mx = max32(mx);
        m_new = renewed(mx);
        negm = -m_new * sl2;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            int key = k0 + key_of(kb, v, hi);
            bool ok = key < N && (!CAUSAL || key <= row);
            p[kb][v] = ok ? ex2(__builtin_fmaf(s[kb][v], sl2, negm)) : 0.f;
          }
      }

      // ---- injection point: exponentials
      if (tile_has_fault) {
        for (int fi = fcur; fi < fend && F[fi].kv_tile == i; ++fi) {
          if (F[fi].stage != FTATTN_ST_EXP) continue;
          int lr = F[fi].row - row0_w, kl = F[fi].col - k0, bit = F[fi].bit;
          bool mine = lr >= 0 && lr < 32 && lane == lr + 32 * ((kl & 7) >> 2);
          int tkb = kl >> 5, tv = 4 * ((kl & 31) >> 3) + (kl & 3);
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) p[kb][v] = flip_if(p[kb][v], mine && tkb == kb && tv == v, bit);
        }
      }

      if (FT) {
        if (!g_mask) {
          // ============ unified product-form check of GEMM I, subtraction and exp
          // (Algorithm 1, first "if"; Section 3.4 case 2).  For class c the product of its 8
          // exponentials must equal exp2(sl2*check1 - 8*m).  Both sides are divided by that
          // prediction, two factors at a time, so the running product stays near one.
          bool bad = false;
          float dv[4] = {0.f, 0.f, 0.f, 0.f};
          // (2^(-e/4) per pair of factors, e = sl2*check1 + 8*negm the predicted log2 of the product)
          const float c_chk = sl2 * (-2.0f / NFOLD_K), c_m = -2.0f * negm;
          if (DMR) {
            // second evaluation of the maximum and of every exponential (eq. (11), (12)), compared bit
            // by bit; a third evaluation settles a differing maximum here, a differing exponential in
            // the exact path below
            float m0 = fmax2(opaque(s[0][0]), s[0][1]), m1 = fmax2(opaque(s[1][0]), s[1][1]);
#pragma unroll
            for (int v = 2; v < 16; v += 2) {
              m0 = fmax2(fmax2(m0, s[0][v]), s[0][v + 1]);
              m1 = fmax2(fmax2(m1, s[1][v]), s[1][v + 1]);
            }
            const float mxb = max32(fmax2(m0, m1));
            if (wave_any(as_u(mxb) != as_u(mx))) {
              float mc = opaque(s[0][0]);
#pragma unroll
              for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) mc = fmax2(mc, s[kb][v]);
              mc = max32(mc);
              if (as_u(mc) == as_u(mxb)) mx = mxb;          // two of three agree on the duplicate
              m_new = renewed(mx);
              negm = -m_new * sl2;
              bad = true;                                    // every exponential is looked at again below
            }
            uint32_t diff = 0u;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int v = 0; v < 16; ++v) diff |= as_u(ex2(__builtin_fmaf(opaque(s[kb][v]), sl2, negm))) ^ as_u(p[kb][v]);
            bad |= diff != 0u;
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float chk = sc[r] + sc[4 + r];
            if (!DMR) {
              float s2 = ex2(__builtin_fmaf(chk, c_chk, c_m));
              float pr = ((p[0][r] * p[0][4 + r]) * s2) * ((p[0][8 + r] * p[0][12 + r]) * s2);
              pr *= ((p[1][r] * p[1][4 + r]) * s2) * ((p[1][8 + r] * p[1][12 + r]) * s2);
              if (EW) dv[r] = pr;
              else {
                dv[r] = pr - 1.0f;
                bad |= !(__builtin_fabsf(dv[r]) <= a.tau_fast);
              }
            }
            if (STEP) {
              // strided ABFT of GEMM I alone (eq. (15)): same sum order as the exact evaluation below
              float sum1 = 0.f;
#pragma unroll
              for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) sum1 += s[kb][4 * gg + r];
              bad |= !(a.scale * __builtin_fabsf(chk - sum1) <= 0.5f * a.eps1);
            }
          }
          if (EW) {
            // one class per row: the product of all 64 exponentials, from both lanes of the query
            const float pl = (dv[0] * dv[1]) * (dv[2] * dv[3]);
            dv[0] = pl * xchg32(pl, hi) - 1.0f;
            bad = !(__builtin_fabsf(dv[0]) <= a.tau_fast);
          }
          recheck = wave_any(bad);
          if (recheck) ++rechecks;
          else if (EW) {
            dev_max = fmax2(dev_max, __builtin_fabsf(dv[0]));
          } else {
            // largest deviation that passed (two three-input maxima; the values are finite here)
            asm("v_max3_f32 %0, %0, |%1|, |%2|" : "+v"(dev_max) : "v"(dv[0]), "v"(dv[1]));
            asm("v_max3_f32 %0, %0, |%1|, |%2|" : "+v"(dev_max) : "v"(dv[2]), "v"(dv[3]));
          }
        }
        if (recheck) {
          // ============ exact re-evaluation (rare: a fast check tripped, or the tile is masked).
          // lambda = ln prod P - (sigma*check1_eff - n_valid*m) = sum_l (ln P_l - x_l) - sigma*R1.
          bool lin_fixed = false, logged = false;
          if (EW) {
            // the whole tile row as one class (fold index = position of the key in the tile): every
            // sum is the lane's half plus its partner's, formed by all lanes alike (the exchanges
            // are wave-wide operations); only the event and the writes depend on the outcome
            float sum1 = 0.f, sum2 = 0.f, E = 0.f, chk1 = 0.f, chk2 = 0.f, big = -1.f;
            int nvalid = 0, l_big = -1;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float c1 = sc[r] + sc[4 + r];
              chk1 += c1;
              chk2 += 8.0f * (sc[8 + r] + sc[12 + r]) + (float)(4 * hi + r - 7) * c1;
            }
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int l = key_of(kb, v, hi), key = k0 + l;
                const bool ok = key < N && (!CAUSAL || key <= row);
                const float sv = s[kb][v];
                sum1 += sv;
                sum2 += (float)(l + 1) * sv;
                const float mag = finitef(sv) ? __builtin_fabsf(sv) : __builtin_inff();
                if (mag > big) { big = mag; l_big = l; } else if (mag == big) { l_big = -1; }
                const float t = __builtin_fmaf(sv, sl2, negm);
                const float pe = ex2(t);
                if (ok) {
                  ++nvalid;
                  if (as_u(pe) != as_u(p[kb][v])) E += lg2(p[kb][v]) - t;
                }
              }
            sum1 = sum32(sum1); sum2 = sum32(sum2); E = sum32(E); chk1 = sum32(chk1); chk2 = sum32(chk2);
            nvalid += (int)xchg32((float)nvalid, hi);
            {
              const float bigp = xchg32(big, hi);
              const int lp = (int)xchg32((float)l_big, hi);
              if (bigp > big) l_big = lp; else if (bigp == big) l_big = -1;
            }
            const float R1 = chk1 - sum1;
            const float lam = LN2 * E - a.scale * R1;
            const bool linear = !(a.scale * __builtin_fabsf(R1) <= 0.5f * a.eps1);
            const bool det = nvalid > 0 && !(__builtin_fabsf(lam) <= a.eps1);
            int lstar = -1;
            {
              const float ratio = (chk2 - sum2) / R1;
              if (finitef(ratio)) {
                const float c = __builtin_rintf(ratio) - 1.0f;
                if (c >= 0.f && c < (float)BN) lstar = (int)c;
              } else {
                lstar = l_big;
              }
            }
            if (!(det && linear)) lstar = -1;
            float rest = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int v = 0; v < 16; ++v)
                if (key_of(kb, v, hi) != lstar) rest += s[kb][v];
            rest = sum32(rest);
            if (det) {
              logged = true;
              if (linear) {
                const bool fix = a.correct && lstar >= 0;
                if (hi == 0) log_event(a, bh, FTATTN_CHECK_S, i, row, lstar >= 0 ? k0 + lstar : -1, lam, fix ? 1 : 0);
                if (fix) {
                  const float val = chk1 - rest;
#pragma unroll
                  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                      if (key_of(kb, v, hi) == lstar) s[kb][v] = val;
                  lin_fixed = true;
                }
              } else {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                  for (int v = 0; v < 16; ++v) {
                    const int key = k0 + key_of(kb, v, hi);
                    const bool ok = key < N && (!CAUSAL || key <= row);
                    const float pe = ex2(__builtin_fmaf(s[kb][v], sl2, negm));
                    if (ok && as_u(pe) != as_u(p[kb][v])) {
                      log_event(a, bh, FTATTN_CHECK_EXP, i, row, key, lam, a.correct ? 1 : 0);
                      if (a.correct) p[kb][v] = pe;
                    }
                  }
              }
            }
          }
#pragma unroll
          for (int r = 0; r < 4 && !EW; ++r) {
            float chk1 = sc[r] + sc[4 + r];
            float sum1 = 0.f, E = 0.f;
            int nvalid = 0;
            bool differs = false;       // an exponential that is not what its re-evaluation gives
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int gg = 0; gg < 4; ++gg) {
                int v = 4 * gg + r, key = k0 + key_of(kb, v, hi);
                bool ok = key < N && (!CAUSAL || key <= row);
                float sv = s[kb][v];
                sum1 += sv;
                float t = __builtin_fmaf(sv, sl2, negm);
                float pe = ex2(t);
                if (ok) {
                  ++nvalid;
                  if (as_u(pe) != as_u(p[kb][v])) { E += lg2(p[kb][v]) - t; differs = true; }
                }
              }
            float R1 = chk1 - sum1;
            float lam = LN2 * E - a.scale * R1;
            const bool linear = !(a.scale * __builtin_fabsf(R1) <= 0.5f * a.eps1);
            bool det = nvalid > 0 && (DMR ? (linear || differs) : (!(__builtin_fabsf(lam) <= a.eps1) || (STEP && linear)));
            if (det) {
              logged = true;
              if (linear) {
                float chk2 = sc[8 + r] + sc[12 + r];
                float sum2 = 0.f, big = -1.f;
                int l_big = -1;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                  for (int gg = 0; gg < 4; ++gg) {
                    float sv = s[kb][4 * gg + r];
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
                log_event(a, bh, FTATTN_CHECK_S, i, row, col, lam, fix ? 1 : 0);
                if (fix) {
                  float rest = 0.f;
#pragma unroll
                  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int gg = 0; gg < 4; ++gg)
                      if (4 * kb + gg != lstar) rest += s[kb][4 * gg + r];
                  float val = chk1 - rest;
#pragma unroll
                  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int gg = 0; gg < 4; ++gg)
                      if (4 * kb + gg == lstar) s[kb][4 * gg + r] = val;
                  lin_fixed = true;
                }
              } else {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                  for (int gg = 0; gg < 4; ++gg) {
                    int v = 4 * gg + r, key = k0 + key_of(kb, v, hi);
                    bool ok = key < N && (!CAUSAL || key <= row);
                    float pe = ex2(__builtin_fmaf(s[kb][v], sl2, negm));
                    if (ok && as_u(pe) != as_u(p[kb][v])) {
                      log_event(a, bh, FTATTN_CHECK_EXP, i, row, key, lam, a.correct ? 1 : 0);
                      if (a.correct) p[kb][v] = pe;
                    }
                  }
              }
            }
          }
          // the event log's stores complete out of order with loads: drain before the counted waits
          if (wave_any(logged)) wait_vmcnt<0>();
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
                mx2 = fmax2(mx2, ok ? s[kb][v] : -__builtin_inff());
              }
            mx2 = max32(mx2);
            if (redo) {
              mx = mx2;
              m_new = renewed(mx);
              negm = -m_new * sl2;
            }
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                int key = k0 + key_of(kb, v, hi);
                bool ok = key < N && (!CAUSAL || key <= row);
                float pe = ok ? ex2(__builtin_fmaf(s[kb][v], sl2, negm)) : 0.f;
                if (redo) p[kb][v] = pe;
              }
          }
        }
      }

      // ============ rescale factor, lower bound of the row-sum (carried with the same rescale as the
      // row-sum itself, which is completed in the matrix phase), first quarter of P in fp16
      if (LAZY) m_true = fmax2(m_true, mx);
      // e^{m_old - m_new}, formed from the difference so that an unchanged maximum gives exactly one (the
      // product m_old * sl2 against the rounded m_new * sl2 would leave a rounding residue, and with it a
      // rescale of the whole output by 1 + 2^-23)
      al = ex2((m_run - m_new) * sl2);
      if (FT) l_low = l_low * al + ex2(__builtin_fmaf(mx, sl2, negm));
      m_run = m_new;
      convert_quarter(0);

      // ============ rescale of the running output (Algorithm 1: diag(e^{m_old - m_new}) O)
      if (wave_any(al != 1.f)) {
#pragma unroll
        for (int fb = 0; fb < NFB; ++fb) o[fb] *= al;
        if (FT) oc *= al;
      }
    }
    if (ALT) {
      if (grp == 0) wait_vmcnt<U::NLOAD>();       // unit i (unit i+1 may still be in flight)
    } else {
      wait_vmcnt<0>();                            // unit i (nothing younger has been requested)
    }
    phase_barrier();                              // ... everyone's pieces; and everyone is past the reads of the stage refilled next

    // =========================================================== matrix phase
    prepare_unit(ALT ? i + 2 : i + 1, (ALT ? i + 2 : i + 1) < nj);
    __builtin_amdgcn_s_setprio(1);
    // (after a wave's last key tile GEMM I runs on a tile it does not need: same code, result unused)
    if (DMR) l_prev = l_part;
    if (on) matrix_stream(stage + (uint32_t)U::KBYTES, stage, yes{}, yes{}, yes{});
    else {
#pragma unroll
      for (int n = 0; n < U::NLOAD; ++n) issue_piece(n);
    }
    __builtin_amdgcn_s_setprio(0);

    // ---- injection point: row-sum (right after the update of this iteration)
    if (tile_has_fault) {
      if (on) {
        for (int fi = fcur; fi < fend && F[fi].kv_tile == i; ++fi) {
          if (F[fi].stage != FTATTN_ST_ROWSUM) continue;
          int lr = F[fi].row - row0_w;
          bool mine = lr >= 0 && lr < 32 && lq == lr;
          float full = sum32(l_part);
          float flipped = flip_if(full, true, F[fi].bit);
          if (mine) l_part = hi ? 0.f : flipped;
        }
      }
    }
    // ---- injection point: output accumulator
    if (tile_has_fault) {
      if (on) {
        for (int fi = fcur; fi < fend && F[fi].kv_tile == i; ++fi) {
          if (F[fi].stage != FTATTN_ST_OACC) continue;
          int lr = F[fi].row - row0_w, col = F[fi].col, bit = F[fi].bit;
          bool mine = lr >= 0 && lr < 32 && lane == lr + 32 * ((col & 7) >> 2);
          int tfb = col >> 5, tv = 4 * ((col & 31) >> 3) + (col & 3);
#pragma unroll
          for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[fb][v] = flip_if(o[fb][v], mine && tfb == fb && tv == v, bit);
        }
      }
      while (fcur < fend && F[fcur].kv_tile == i) ++fcur;
    }
    if (STEP && on) {
      // ---- verification of this iteration's reduce-sum (range so far, Section 3.4 case 3) and of
      // GEMM II with the rescale (sum-form check on the unnormalised accumulator)
      const bool real = row < N;
      float l = sum32(l_part);
      const int seen = k0 + BN < N ? k0 + BN : N;
      const float Ub = (float)(CAUSAL && row + 1 < seen ? row + 1 : seen);
      if (DMR) {
        // the two evaluations of the reduce-sum; a third one, from the fp16 P still in registers,
        // settles a difference
        const bool dl = as_u(l_part) != as_u(l2_part);
        if (wave_any(real && dl)) {
          float q3[2][2];
          const half2v ones = {(_Float16)1.f, (_Float16)1.f};
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int n = 0; n < 2; ++n) {
              q3[kb][n] = 0.f;
#pragma unroll
              for (int x = 0; x < 8; x += 2) {
                half2v pr2 = {ph[kb][n][x], ph[kb][n][x + 1]};
                q3[kb][n] = __builtin_amdgcn_fdot2(opaque(pr2), ones, q3[kb][n], false);
              }
            }
          const float l3 = rowsum_update(opaque(l_prev), q3);
          const bool row_dl = dl | (xchg32(dl ? 1.f : 0.f, hi) != 0.f);
          if (real && row_dl && hi == 0) log_event(a, bh, FTATTN_CHECK_L, i, row, 0, l, a.correct ? 1 : 0);
          if (a.correct && dl) {
            if (as_u(l3) == as_u(l2_part)) l_part = l2_part; else if (as_u(l3) == as_u(l_part)) l2_part = l_part;
          }
          l = sum32(l_part);
          wait_vmcnt<0>();    // the event log's stores complete out of order with loads: drain before the counted waits
        }
      }
      const bool detl = !DMR && real && !(l_low * (1.f - a.delta_l) <= l && l <= Ub * (1.f + a.delta_l));
      if (wave_any(detl)) {
        if (detl) {
          if (hi == 0) log_event(a, bh, FTATTN_CHECK_L, i, row, 0, l, a.correct ? 1 : 0);
          if (a.correct) { l = l_low; l_part = hi ? 0.f : l_low; }
        }
        wait_vmcnt<0>();      // the event log's stores complete out of order with loads: drain before the counted waits
      }
      if (sum_check(a.tau_o * l, i, real, false, 0.f, false)) wait_vmcnt<0>();
    }
    if (ALT) {
      if (grp == 1) wait_vmcnt<U::NLOAD>();       // unit i+1 (unit i+2 may still be in flight)
      phase_barrier();
    }
  }
  if (ALT && grp == 0) phase_barrier();

  // ================= after the loop: row-sum range check, normalisation, sum-form check, store
  float rmax_u = 0.f, rmax_l = 0.f;
  {
    const bool real = row < N;
    float l = sum32(l_part);
    const bool lfold = FT && a.rowsum_fold != 0;
    if (FT && lfold) {
      // The row-sum as fold NFOLD_V of checksum class 0 (held by the lane half hi == 0, register
      // r == 0): the row-sum the checksum implies against the accumulated one, in units of the
      // row-sum; on a mismatch the location rule over the NFOLD_V + 1 folds decides whether the
      // row-sum is the wrong element, and if so it is replaced by the implied one.
      float sumx = 0.f;
#pragma unroll
      for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) sumx += o[fb][4 * gg];
      const float chk1 = oc[0] + oc[4];
      const float lc = chk1 - sumx;
      const float rr = (lc - l) / lc;
      const bool detl = real && hi == 0 && (!(__builtin_fabsf(rr) <= a.tau_o) || !finitef(rr));
      if (!detl && real && hi == 0) rmax_u = fmax2(rmax_u, __builtin_fabsf(rr));
      if (wave_any(detl)) {
        if (detl) {
          const float chk2 = oc[8] + oc[12];
          float sum2 = (float)(NFOLD_V + 1) * l;
          float big = finitef(l) ? __builtin_fabsf(l) : __builtin_inff();
          int l_big = NFOLD_V;
#pragma unroll
          for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
              const float ov = o[fb][4 * gg];
              sum2 += (float)(4 * fb + gg + 1) * ov;
              const float mag = finitef(ov) ? __builtin_fabsf(ov) : __builtin_inff();
              if (mag > big) { big = mag; l_big = 4 * fb + gg; } else if (mag == big) { l_big = -1; }
            }
          const float ratio = (chk2 - sum2) / (lc - l);
          int lstar = -1;
          if (finitef(ratio)) {
            const float c = __builtin_rintf(ratio) - 1.0f;
            if (c >= 0.f && c < (float)(NFOLD_V + 1)) lstar = (int)c;
          } else {
            lstar = l_big;
          }
          if (lstar == NFOLD_V) {
            log_event(a, bh, FTATTN_CHECK_L, -1, row, 0, rr, a.correct ? 1 : 0);
            if (a.correct) l = lc;
          }
        }
      }
      // the other half of the row takes the row-sum of the half that checked it
      const float lp = xchg32(l, hi);
      if (hi == 1) l = lp;
    }
    if (FT && !lfold && !DMR) {
      float Ub = CAUSAL ? (float)(row + 1 < N ? row + 1 : N) : (float)N;
      if (LAZY) Ub *= ex2((m_true - m_run) * sl2);      // exponentials reach exp(running maximum - reference)
      float lo = l_low;
      bool detl = real && !(lo * (1.f - a.delta_l) <= l && l <= Ub * (1.f + a.delta_l));
      if (!detl && real) { rmax_u = fmax2(rmax_u, l / Ub); rmax_l = fmax2(rmax_l, lo / l); }
      if (detl) {
        if (hi == 0) log_event(a, bh, FTATTN_CHECK_L, -1, row, 0, l, a.correct ? 1 : 0);
        if (a.correct) l = lo;     // the approximation of Section 3.4, "optimized EFTA"
      }
    }
    float inv = 1.0f / l;
#pragma unroll
    for (int fb = 0; fb < NFB; ++fb) o[fb] *= inv;
    if (FT) {
      oc *= inv;
      (void)sum_check(a.tau_o, -1, real, lfold && hi == 0, l * inv, true);
    }
    // ---- store: lane holds features 32*fb + 8*gg + 4*hi + (0..3) of its query
    if (real) {
      size_t base = ((size_t)bh * N + row) * D;
#pragma unroll
      for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {
          int f = 32 * fb + 8 * gg + 4 * hi;
          float x0 = o[fb][4 * gg], x1 = o[fb][4 * gg + 1], x2 = o[fb][4 * gg + 2], x3 = o[fb][4 * gg + 3];
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
            for (int x = 0; x < 4; ++x) {
              uint32_t rnd = ((u[x] >> 16) & 1u) + 0x7FFFu;
              bv16[x] = (u[x] & 0x7F800000u) == 0x7F800000u ? (uint16_t)(u[x] >> 16) : (uint16_t)((u[x] + rnd) >> 16);
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
    for (int x = 0; x < 4; ++x) {
      float v = vals[x];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v = fmax2(v, __shfl_xor(v, off));
      if (lane == 0) atomicMax(rm + x, as_u(v));
    }
    if (lane == 0 && rechecks) atomicAdd(a.recheck, (unsigned long long)rechecks);
  }
}

}  // namespace ftattn
