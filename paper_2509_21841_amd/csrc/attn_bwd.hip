// Backward of causal varlen attention, deterministic and atomics-free: two kernels.
//   attn_bwd_dq   owns a block of query rows, walks the visible key tiles:  S^T = K Q^T, dP^T = V dO^T,
//                 dS^T = P^T o (dP^T - D), dQ^T += K^T dS^T.  Also computes D_i = dO_i . O_i and stores it.
//   attn_bwd_dkdv owns a block of key rows, walks the query tiles at or after it and the query heads of its
//                 KV group:  S = Q K^T, dP = dO V^T, dV^T += dO^T P, dK^T += Q^T dS.
// Both recompute P from the forward's LSE. In each kernel the accumulator of the first two products already
// has the register layout the third/fourth product needs as its B operand; the transposed A operands
// (K^T, Q^T, dO^T) come from the row-major LDS tiles through the transposing LDS read.
#include <type_traits>
#include "zp_common.h"

struct zp_bwd_params {
  const __bf16 *q, *k, *v, *o, *dout;
  int64_t q_stride, k_stride, v_stride, o_stride, do_stride;
  const float *lse;   // [Hq][T]
  float *dvec;        // [Hq][T] scratch: -D_i = -(dO_i . O_i)
  float *lse2;        // [Hq][T] scratch: -LSE_i / scale
  const zp_tile *dq_tiles;
  const zp_tile *kv_tiles;
  const zp_tile *kv_tiles_short;  // key blocks with few query tiles: run by the two-workgroups-per-CU kernel (d = 128)
  int32_t n_dq_tiles, n_kv_tiles, n_kv_tiles_short, Hq, Hkv, grp, T;
  float scale_log2, scale;
  __bf16 *dq, *dk, *dv;      // outputs (bf16, overwritten) ...
  int64_t dq_stride, dkv_stride;
  int32_t accumulate;        // ... or, when set, float accumulators of the same shapes that the results are ADDED to
  zp_work_split work_dq, work_kv, work_kv_short;  // work hand-out of the three launches (counters set by the C ABI, the rest by the launcher)
};

namespace {

constexpr int BWD_NT = 256;
constexpr float LOG2E = 1.4426950408889634f;

template <int D>
__device__ __forceinline__ void store_acc_rows(__bf16 *dst, const f32x16 (&acc)[D / 32], float mul) {
#pragma unroll
  for (int db = 0; db < D / 32; db++)
#pragma unroll
    for (int b = 0; b < 4; b++) {
      bf16x4 v4 = {(__bf16)(acc[db][4 * b] * mul), (__bf16)(acc[db][4 * b + 1] * mul),
                   (__bf16)(acc[db][4 * b + 2] * mul), (__bf16)(acc[db][4 * b + 3] * mul)};
      *(bf16x4 *)(dst + db * 32 + b * 8) = v4;
    }
}

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// accumulate variant of store_acc_rows: dst is float, the scaled accumulator is added to what is there
template <int D>
__device__ __forceinline__ void add_acc_rows(float *dst, const f32x16 (&acc)[D / 32], float mul) {
#pragma unroll
  for (int db = 0; db < D / 32; db++)
#pragma unroll
    for (int b = 0; b < 4; b++) {
      f32x4 cur = *(const f32x4 *)(dst + db * 32 + b * 8);
      cur[0] += acc[db][4 * b] * mul; cur[1] += acc[db][4 * b + 1] * mul;
      cur[2] += acc[db][4 * b + 2] * mul; cur[3] += acc[db][4 * b + 3] * mul;
      *(f32x4 *)(dst + db * 32 + b * 8) = cur;
    }
}

// ------------------------------------------------------------------------------------------- dQ
// One 32-key half of a K/V tile for one wave: S^T and dP^T chains, dS^T, then dQ^T += K^T dS^T.
// `piece(integral_constant<int, kk>)` is called once per 16-wide k-step of the chains when PIECES is set: the caller
// issues one asynchronous copy of the next tile there. Every step is fenced and the copies are ordered against every
// LDS access, so they end up one per MFMA pair -- far enough apart that none waits for the address unit behind the
// copies of the other waves. Kb, Vb: byte offsets of the K and V tile from the base the lane offsets carry.
template <int D, bool MASK, bool PIECES, class Piece>
__device__ __forceinline__ void dq_half(int Kb, int Vb, int kb, const bf16x8 (&qreg)[D / 16],
                                        const bf16x8 (&doreg)[D / 16], f32x16 (&dq_acc)[D / 32], float c_log2,
                                        float lse2, const f32x16 &negD, int j0, int hi, int nvis_lane,
                                        const zp_lds_offsets<D> &lo, Piece &&piece) {
  constexpr int KK = D / 16, DB = D / 32;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // the dP^T chain starts from -D (a lane holds one query, so the seed is the same in all 16 registers and lives in
  // registers for the whole kernel): the accumulator then holds dP - D
  // the LDS operand reads stay two k-steps ahead of the MFMAs that use them; every step is fenced so that the
  // copies keep their distance
  f32x16 s = zero, dp = negD;
  bf16x8 ka[KK], va[KK];
  ka[0] = lo.rows_at(Kb, kb, 0); va[0] = lo.rows_at(Vb, kb, 0);
  ka[1] = lo.rows_at(Kb, kb, 1); va[1] = lo.rows_at(Vb, kb, 1);
  zp_static_for<KK>([&](auto kk) {
    constexpr int k = kk.value;
    __builtin_amdgcn_sched_barrier(0);
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[k], qreg[k], s, 0, 0, 0);
    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[k], doreg[k], dp, 0, 0, 0);
    if constexpr (k + 2 < KK) { ka[k + 2] = lo.rows_at(Kb, kb, k + 2); va[k + 2] = lo.rows_at(Vb, kb, k + 2); }
    if constexpr (PIECES) piece(kk);
  });
  __builtin_amdgcn_sched_barrier(0);
  bf16x8 dsb[2];
#pragma unroll
  for (int r = 0; r < 16; r++) {
    float pv = zp_exp2(__builtin_fmaf(s[r], c_log2, -lse2));
    if (MASK) {
      const int j = j0 + kb * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
      if (j >= nvis_lane) pv = 0.f;
    }
    dsb[r >> 3][r & 7] = (__bf16)(pv * dp[r]);
  }
#pragma unroll
  for (int m = 0; m < 2; m++)
#pragma unroll
    for (int db = 0; db < DB; db++)
      dq_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo.tr_at(Kb, kb, m, db), dsb[m], dq_acc[db], 0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);
}

// Two waves per SIMD (two workgroups of four waves per CU, 64 KB of LDS each). An MFMA takes about 20 cycles of the
// issuing wave's vector issue time, and a wave issues its LDS, scalar and wait instructions one after the other as
// well; with a second wave on the SIMD all of that runs under the other wave's MFMAs. Working through a tile in two
// 32-key halves keeps the wave within the 256 registers this needs.
template <int D>
__global__ __launch_bounds__(BWD_NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dq_kernel(zp_bwd_params p) {
  constexpr int TILEB = 64 * D * 2;
  constexpr int LOADS = 2 * zp_stager<D>::LOADS;  // async loads one wave issues per staged K/V tile pair
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char *Ks = smem;               // [2][64][D]
  char *Vs = smem + 2 * TILEB;   // [2][64][D]

  const int item = zp_item_of_block(p.work_dq, (int *)(smem + 4 * TILEB));
  if (item < 0) return;
  int unit, hh;
  zp_block_to_unit(item, p.grp, unit, hh);
  if (unit >= p.n_dq_tiles * p.Hkv) return;
  const int tile_idx = unit / p.Hkv, g = unit - tile_idx * p.Hkv;
  const int h = g * p.grp + hh;
  const zp_tile t = p.dq_tiles[tile_idx];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int ql = lane & 31, hi = lane >> 5;
  const int row = w * 32 + ql;
  const bool row_ok = row < t.q_rows;
  const int64_t tok = (int64_t)t.q_tok0 + row;

  auto nvis_of = [&](int r) {
    int n = t.q_pos0 + r - t.k_pos0 + 1;
    return n < 0 ? 0 : (n > t.k_len ? t.k_len : n);
  };
  const int nvis_lane = nvis_of(row);
  const int nvis_w_min = nvis_of(w * 32), nvis_w_max = nvis_of(w * 32 + 31);
  const int n_kt = (nvis_of(t.q_rows - 1) + 63) / 64;

  zp_stager<D> kst, vst;
  kst.init(p.k + (int64_t)t.k_tok0 * p.k_stride + (int64_t)g * D, p.k_stride, tid);
  vst.init(p.v + (int64_t)t.k_tok0 * p.v_stride + (int64_t)g * D, p.v_stride, tid);
  zp_lds_offsets<D> lo;
  lo.init_abs(lane, smem);

  // Row operands first, the first tile copy right behind them (the two memory latencies overlap), their first use
  // after that. The explicit wait before the first barrier covers all of it and tells the compiler that the register
  // operands have arrived (a wait of its own inside the key loop would drain the copies in flight every iteration).
  bf16x8 qreg[D / 16], doreg[D / 16], oreg[D / 16];
  {
    const __bf16 *qp = p.q + tok * p.q_stride + (int64_t)h * D + 8 * hi;
    const __bf16 *dop = p.dout + tok * p.do_stride + (int64_t)h * D + 8 * hi;
    const __bf16 *op = p.o + tok * p.o_stride + (int64_t)h * D + 8 * hi;
#pragma unroll
    for (int kk = 0; kk < D / 16; kk++) {
      if (row_ok) {
        qreg[kk] = *(const bf16x8 *)(qp + 16 * kk);
        doreg[kk] = *(const bf16x8 *)(dop + 16 * kk);
        oreg[kk] = *(const bf16x8 *)(op + 16 * kk);
      } else {
        qreg[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        doreg[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        oreg[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      }
    }
  }
  float lse_nat = 0.f;
  if (row_ok) lse_nat = p.lse[(int64_t)h * p.T + tok];
  if (n_kt > 0) {
    kst.issue(Ks, 0, t.k_len);
    vst.issue(Vs, 0, t.k_len);
  }
  float dsum = 0.f;
#pragma unroll
  for (int kk = 0; kk < D / 16; kk++)
#pragma unroll
    for (int e = 0; e < 8; e++) dsum += (float)doreg[kk][e] * (float)oreg[kk][e];
  const float Dq = zp_pair_sum(dsum);
  float lse2 = 0.f;
  if (row_ok) {
    lse2 = lse_nat * LOG2E;
    if (hi == 0) {
      // negated and pre-divided so that the second kernel can seed its MFMA accumulators with them
      p.dvec[(int64_t)h * p.T + tok] = -Dq;
      p.lse2[(int64_t)h * p.T + tok] = -lse_nat / p.scale;
    }
  }

  f32x16 dq_acc[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) dq_acc[i][r] = 0.f;
  const float c_log2 = p.scale_log2;

  zp_wait_async();
  __syncthreads();

  f32x16 negD;
#pragma unroll
  for (int r = 0; r < 16; r++) negD[r] = -Dq;
  constexpr int PW = zp_stager<D>::PER_WAVE;
  // one key tile out of LDS buffer BUF (compile-time, so that every LDS address is a register plus an immediate)
  auto key_tile = [&](int it, auto BUF) {
    constexpr int buf = decltype(BUF)::value;
    const int j0 = it * 64;
    const bool compute = j0 < nvis_w_max;
    const bool masked = j0 + 64 > nvis_w_min;
    // the next tile is fetched inside the first half of this tile's arithmetic when it has 64 valid keys and this
    // wave computes an unmasked tile (the common case), else in front of it
    const bool fetch = it + 1 < n_kt;
    const bool fused = fetch && compute && !masked && j0 + 128 <= t.k_len;
    if (fetch && !fused) {
      kst.issue(Ks + (buf ^ 1) * TILEB, j0 + 64, t.k_len);
      vst.issue(Vs + (buf ^ 1) * TILEB, j0 + 64, t.k_len);
    }
    // the same copies one load at a time, K and V alternating (2 * PW loads = one per k-step)
    // (the sources are worked out unconditionally: a value defined under a branch would not stay in scalar registers)
    const void *pc_k = zp_uniform_ptr(kst.base + (int64_t)(j0 + 64) * kst.stride);
    const void *pc_v = zp_uniform_ptr(vst.base + (int64_t)(j0 + 64) * vst.stride);
    auto stage_piece = [&](auto n) {
      constexpr int N = decltype(n)::value, i = N / 2;
      static_assert(2 * PW == D / 16, "one copy per k-step");
      if constexpr (N % 2 == 0)
        zp_dma16_so(pc_k, kst.off[i], __builtin_amdgcn_readfirstlane(zp_lds_addr(Ks + (buf ^ 1) * TILEB) + (kst.w * PW + i) * 1024));
      else
        zp_dma16_so(pc_v, vst.off[i], __builtin_amdgcn_readfirstlane(zp_lds_addr(Vs + (buf ^ 1) * TILEB) + (vst.w * PW + i) * 1024));
    };
    if (compute) {
      constexpr int Kb = buf * TILEB, Vb = (2 + buf) * TILEB;  // byte offsets of the tiles from smem
      if (masked) {
        dq_half<D, true, false>(Kb, Vb, 0, qreg, doreg, dq_acc, c_log2, lse2, negD, j0, hi, nvis_lane, lo, stage_piece);
        dq_half<D, true, false>(Kb, Vb, 1, qreg, doreg, dq_acc, c_log2, lse2, negD, j0, hi, nvis_lane, lo, stage_piece);
      } else if (fused) {
        dq_half<D, false, true>(Kb, Vb, 0, qreg, doreg, dq_acc, c_log2, lse2, negD, j0, hi, nvis_lane, lo, stage_piece);
        dq_half<D, false, false>(Kb, Vb, 1, qreg, doreg, dq_acc, c_log2, lse2, negD, j0, hi, nvis_lane, lo, stage_piece);
      } else {
        dq_half<D, false, false>(Kb, Vb, 0, qreg, doreg, dq_acc, c_log2, lse2, negD, j0, hi, nvis_lane, lo, stage_piece);
        dq_half<D, false, false>(Kb, Vb, 1, qreg, doreg, dq_acc, c_log2, lse2, negD, j0, hi, nvis_lane, lo, stage_piece);
      }
    }
    zp_wait_async();
    __syncthreads();
  };
  for (int it = 0; it < n_kt; it += 2) {
    key_tile(it, std::integral_constant<int, 0>{});
    if (it + 1 < n_kt) key_tile(it + 1, std::integral_constant<int, 1>{});
  }

  if (row_ok) {
    if (p.accumulate) add_acc_rows<D>((float *)p.dq + tok * p.dq_stride + (int64_t)h * D + 4 * hi, dq_acc, p.scale);
    else store_acc_rows<D>(p.dq + tok * p.dq_stride + (int64_t)h * D + 4 * hi, dq_acc, p.scale);
  }
}

// ------------------------------------------------------------------------------------------- dK, dV
// Tile fields: k_tok0/k_len/k_pos0 = this block of key rows; q_tok0/q_rows/q_pos0 = the query rows of the
// same sequence from the first one that can see the block's first key to the end of the sequence.
//
// One wave per SIMD (the 128 accumulator registers of dK^T and dV^T plus the K/V operands leave no room for
// two), so latency is hidden inside the wave: per 64-query tile the two 32-query blocks are software
// pipelined -- LDS operands are fetched a phase ahead, the exp/scale arithmetic of one block is interleaved
// with the MFMAs of the other.

// Two neighbouring elements (registers r, r + 1 of the accumulators) of P and dS of a 32-query block, packed as bf16.
// The accumulators were seeded with -LSE/scale and -D, so P = exp2(S c) and dS = P dP.
template <bool MASK>
__device__ __forceinline__ void dkdv_pair(const f32x16 &s, const f32x16 &dp, int r, int qb, int hi, int qpos0,
                                          int kpos, int qpos_end, float c_log2, unsigned &p_pk, unsigned &ds_pk) {
  float p0 = zp_exp2(s[r] * c_log2), p1 = zp_exp2(s[r + 1] * c_log2);
  if (MASK) {
    const int qpos = qpos0 + qb * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
    if (qpos < kpos || qpos >= qpos_end) p0 = 0.f;
    if (qpos + 1 < kpos || qpos + 1 >= qpos_end) p1 = 0.f;
  }
  const bf16x2 pp = {(__bf16)p0, (__bf16)p1};
  const bf16x2 dd = {(__bf16)(p0 * dp[r]), (__bf16)(p1 * dp[r + 1])};
  p_pk = __builtin_bit_cast(unsigned, pp);
  ds_pk = __builtin_bit_cast(unsigned, dd);
}

// One 64-query tile = two 32-query blocks in four phases of D / 16 steps, two MFMAs per step:
//   A: S,dP(0) | B: S,dP(1) || P,dS(0) | C: dV,dK(0) || P,dS(1) | D: dV,dK(1) || the caller's copies
// A wave issues in order, so the overlap is written into the program order: every step is fenced, its two LDS
// operands are requested two steps ahead (each phase thereby reads what its own MFMAs consume, 1/4 of the tile's
// LDS traffic), and an empty volatile asm that takes the step's results as in/out operands pins its MFMAs and vector
// arithmetic to the step. `piece(integral_constant<int, n>)` is called after the n-th MFMA of phase D
// (n = 0 .. 4 * D / 32 - 1): the caller's asynchronous copies of a later tile are issued there, one load between two
// MFMAs.
template <int D, bool MASK, class Piece>
__device__ __forceinline__ void dkdv_tile(const char *Qb, const char *Ob, const float *Lb, const float *Db,
                                          const bf16x8 (&kreg)[D / 16], const bf16x8 (&vreg)[D / 16],
                                          f32x16 (&dk_acc)[D / 32], f32x16 (&dv_acc)[D / 32], int qpos0, int kpos,
                                          int qpos_end, float c_log2, int hi, const zp_lds_offsets<D> &lo,
                                          Piece &&piece) {
  constexpr int KK = D / 16, DB = D / 32, PPS = 8 / KK;  // steps per phase; pairs of P/dS elements per step
  f32x16 s[2], dp[2];
  auto load_seed = [&](int qb) {  // -LSE/scale and -D of the 16 query rows this lane holds
#pragma unroll
    for (int b = 0; b < 4; b++) {
      const f32x4 l4 = *(const ZP_LDS f32x4 *)((const ZP_LDS char *)Lb + (qb * 32 + 8 * b + 4 * hi) * 4);
      const f32x4 d4 = *(const ZP_LDS f32x4 *)((const ZP_LDS char *)Db + (qb * 32 + 8 * b + 4 * hi) * 4);
#pragma unroll
      for (int c = 0; c < 4; c++) { s[qb][4 * b + c] = l4[c]; dp[qb][4 * b + c] = d4[c]; }
    }
  };
  // operand pair of global step t (phase t / KK, step t % KK): rows of Q,dO for A and B, transposed pieces of dO,Q
  // for C and D
  bf16x8 x[4 * KK], y[4 * KK];
  auto load_ops = [&](auto tt) {
    constexpr int t = decltype(tt)::value, ph = t / KK, k = t % KK;
    if constexpr (ph < 2) { x[t] = lo.rows(Qb, ph, k); y[t] = lo.rows(Ob, ph, k); }
    else { x[t] = lo.tr(Ob, ph - 2, k / DB, k % DB); y[t] = lo.tr(Qb, ph - 2, k / DB, k % DB); }
  };
  unsigned ppk[2][8], dpk[2][8];

  load_seed(0);
  load_ops(std::integral_constant<int, 0>{});
  load_ops(std::integral_constant<int, 1>{});
  // A
  zp_static_for<KK>([&](auto kk) {
    constexpr int k = kk.value, t = k;
    __builtin_amdgcn_sched_barrier(0);
    s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[t], kreg[k], s[0], 0, 0, 0);
    dp[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(y[t], vreg[k], dp[0], 0, 0, 0);
    load_ops(std::integral_constant<int, t + 2>{});
    if constexpr (k == KK / 2) load_seed(1);
    asm volatile("" : "+v"(s[0]), "+v"(dp[0]));
  });
  // B
  zp_static_for<KK>([&](auto kk) {
    constexpr int k = kk.value, t = KK + k;
    __builtin_amdgcn_sched_barrier(0);
    s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[t], kreg[k], s[1], 0, 0, 0);
    dp[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(y[t], vreg[k], dp[1], 0, 0, 0);
#pragma unroll
    for (int q = 0; q < PPS; q++)
      dkdv_pair<MASK>(s[0], dp[0], 2 * (PPS * k + q), 0, hi, qpos0, kpos, qpos_end, c_log2, ppk[0][PPS * k + q], dpk[0][PPS * k + q]);
    load_ops(std::integral_constant<int, t + 2>{});
    if constexpr (PPS == 1) asm volatile("" : "+v"(s[1]), "+v"(dp[1]), "+v"(ppk[0][k]), "+v"(dpk[0][k]));
    else asm volatile("" : "+v"(s[1]), "+v"(dp[1]), "+v"(ppk[0][2 * k]), "+v"(dpk[0][2 * k]), "+v"(ppk[0][2 * k + 1]), "+v"(dpk[0][2 * k + 1]));
  });
  auto pack4 = [](const unsigned (&v)[8], int m) {
    return __builtin_bit_cast(bf16x8, (u32x4){v[4 * m], v[4 * m + 1], v[4 * m + 2], v[4 * m + 3]});
  };
  const bf16x8 pb0[2] = {pack4(ppk[0], 0), pack4(ppk[0], 1)}, dsb0[2] = {pack4(dpk[0], 0), pack4(dpk[0], 1)};
  // C
  zp_static_for<KK>([&](auto kk) {
    constexpr int k = kk.value, t = 2 * KK + k, m = k / DB, db = k % DB;
    __builtin_amdgcn_sched_barrier(0);
    dv_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[t], pb0[m], dv_acc[db], 0, 0, 0);
    dk_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(y[t], dsb0[m], dk_acc[db], 0, 0, 0);
#pragma unroll
    for (int q = 0; q < PPS; q++)
      dkdv_pair<MASK>(s[1], dp[1], 2 * (PPS * k + q), 1, hi, qpos0, kpos, qpos_end, c_log2, ppk[1][PPS * k + q], dpk[1][PPS * k + q]);
    load_ops(std::integral_constant<int, t + 2>{});
    if constexpr (PPS == 1) asm volatile("" : "+v"(dv_acc[db]), "+v"(dk_acc[db]), "+v"(ppk[1][k]), "+v"(dpk[1][k]));
    else asm volatile("" : "+v"(dv_acc[db]), "+v"(dk_acc[db]), "+v"(ppk[1][2 * k]), "+v"(dpk[1][2 * k]), "+v"(ppk[1][2 * k + 1]), "+v"(dpk[1][2 * k + 1]));
  });
  const bf16x8 pb1[2] = {pack4(ppk[1], 0), pack4(ppk[1], 1)}, dsb1[2] = {pack4(dpk[1], 0), pack4(dpk[1], 1)};
  // D
  zp_static_for<KK>([&](auto kk) {
    constexpr int k = kk.value, t = 3 * KK + k, m = k / DB, db = k % DB;
    __builtin_amdgcn_sched_barrier(0);
    dv_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[t], pb1[m], dv_acc[db], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    piece(std::integral_constant<int, 2 * k>{});
    __builtin_amdgcn_sched_barrier(0);
    dk_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(y[t], dsb1[m], dk_acc[db], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    piece(std::integral_constant<int, 2 * k + 1>{});
    if constexpr (k + 2 < KK) load_ops(std::integral_constant<int, t + 2>{});
  });
  __builtin_amdgcn_sched_barrier(0);
}

template <int D>
__global__ __launch_bounds__(BWD_NT) __attribute__((amdgpu_waves_per_eu(D == 64 ? 2 : 1, D == 64 ? 2 : 1))) void attn_bwd_dkdv_kernel(zp_bwd_params p) {
  constexpr int TILEB = 64 * D * 2;
  constexpr int NBUF = 4;                       // tiles are fetched three iterations ahead
  constexpr int LOADS = 2 * (TILEB / 4096) + 2; // async loads one wave issues per staged tile
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char *Qs = smem;                              // [NBUF][64][D]
  char *Os = smem + NBUF * TILEB;               // [NBUF][64][D]  (dO)
  float *Ls = (float *)(smem + 2 * NBUF * TILEB);  // [NBUF][64] -LSE / scale
  float *Ds = Ls + NBUF * 64;                   // [NBUF][64] -D

  const int unit = zp_item_of_block(p.work_kv, (int *)(Ds + NBUF * 64));
  if (unit < 0 || unit >= p.n_kv_tiles * p.Hkv) return;
  const int tile_idx = unit / p.Hkv, g = unit - tile_idx * p.Hkv;
  const zp_tile t = p.kv_tiles[tile_idx];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int kl = lane & 31, hi = lane >> 5;
  const int krow = w * 32 + kl;
  const bool key_ok = krow < t.k_len;
  const int64_t ktok = (int64_t)t.k_tok0 + krow;
  const int kpos = t.k_pos0 + krow;

  bf16x8 kreg[D / 16], vreg[D / 16];
  {
    const __bf16 *kp = p.k + ktok * p.k_stride + (int64_t)g * D + 8 * hi;
    const __bf16 *vp = p.v + ktok * p.v_stride + (int64_t)g * D + 8 * hi;
#pragma unroll
    for (int kk = 0; kk < D / 16; kk++) {
      if (key_ok) {
        kreg[kk] = *(const bf16x8 *)(kp + 16 * kk);
        vreg[kk] = *(const bf16x8 *)(vp + 16 * kk);
      } else {
        kreg[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        vreg[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      }
    }
  }

  f32x16 dk_acc[D / 32], dv_acc[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) { dk_acc[i][r] = 0.f; dv_acc[i][r] = 0.f; }
  const float c_log2 = p.scale_log2;

  const int n_qt = (t.q_rows + 63) / 64;
  const int n_it = n_qt * p.grp;  // iterations: query tiles outermost (last tile first), heads of the group innermost

  zp_stager<D> qst, ost;
  qst.init(p.q + (int64_t)t.q_tok0 * p.q_stride + (int64_t)g * p.grp * D, p.q_stride, tid);
  ost.init(p.dout + (int64_t)t.q_tok0 * p.do_stride + (int64_t)g * p.grp * D, p.do_stride, tid);
  zp_lds_offsets<D> lo;
  lo.init(lane);
  // Iteration order: query tiles from the END of the sequence backwards, the heads of the group innermost.
  // Workgroups of one sequence that start together then read the same (tile, head) at the same time and
  // share it in L2; the diagonal (masked) tiles come last.
  int st_hh = 0, st_qt = n_qt - 1;
  auto stage = [&](int buf) {
    const int hh = st_hh, i0 = st_qt * 64;
    const int h = g * p.grp + hh;
    if (++st_hh == p.grp) { st_hh = 0; st_qt--; }
    qst.issue(Qs + buf * TILEB, i0, t.q_rows, (int64_t)hh * D);
    ost.issue(Os + buf * TILEB, i0, t.q_rows, (int64_t)hh * D);
    const int64_t base = (int64_t)h * p.T + t.q_tok0;
    zp_stage_async_f32x64(Ls + buf * 64, p.lse2 + base, i0, t.q_rows - 1, lane);
    zp_stage_async_f32x64(Ds + buf * 64, p.dvec + base, i0, t.q_rows - 1, lane);
  };
  // The same copies for a tile of 64 valid rows, cut into pieces that dkdv_tile issues between the MFMAs of its
  // last phase: piece 0 is the scalar address arithmetic, every later piece one load (same order as `stage`).
  constexpr int PW = zp_stager<D>::PER_WAVE;
  const void *pc_q = nullptr, *pc_o = nullptr, *pc_l = nullptr, *pc_d = nullptr;
  unsigned pc_buf = 0;
  auto stage_piece = [&](auto n) {
    constexpr int N = decltype(n)::value;
    if constexpr (N == 0) {
      const int hh = st_hh, i0 = st_qt * 64;
      const int h = g * p.grp + hh;
      if (++st_hh == p.grp) { st_hh = 0; st_qt--; }
      pc_q = zp_uniform_ptr(qst.base + (int64_t)i0 * qst.stride + (int64_t)hh * D);
      pc_o = zp_uniform_ptr(ost.base + (int64_t)i0 * ost.stride + (int64_t)hh * D);
      const int64_t base = (int64_t)h * p.T + t.q_tok0 + i0;
      pc_l = zp_uniform_ptr(p.lse2 + base);
      pc_d = zp_uniform_ptr(p.dvec + base);
    } else if constexpr (N <= PW) {
      zp_dma16_so(pc_q, qst.off[N - 1], __builtin_amdgcn_readfirstlane(zp_lds_addr(Qs) + pc_buf * TILEB + (qst.w * PW + N - 1) * 1024));
    } else if constexpr (N <= 2 * PW) {
      zp_dma16_so(pc_o, ost.off[N - PW - 1], __builtin_amdgcn_readfirstlane(zp_lds_addr(Os) + pc_buf * TILEB + (ost.w * PW + N - PW - 1) * 1024));
    } else if constexpr (N == 2 * PW + 1) {
      zp_dma4_so(pc_l, lane * 4, __builtin_amdgcn_readfirstlane(zp_lds_addr(Ls) + pc_buf * 256));
    } else if constexpr (N == 2 * PW + 2) {
      zp_dma4_so(pc_d, lane * 4, __builtin_amdgcn_readfirstlane(zp_lds_addr(Ds) + pc_buf * 256));
    }
  };
  auto no_piece = [](auto) {};

  // prologue: tile 0 is requested right behind the K/V register operands (the two memory latencies overlap) and
  // one explicit wait covers both -- it also tells the compiler that the register operands have arrived (a wait of
  // its own inside the loop would drain the copies in flight every iteration); tiles 1 and 2 follow and stay in flight
  if (n_it > 0) stage(0);
  zp_wait_async();
  if (n_it > 1) stage(1);
  if (n_it > 2) stage(2);
  __syncthreads();

  const int kpos_w_min = t.k_pos0 + w * 32, kpos_w_max = t.k_pos0 + w * 32 + 31;
  const int qpos_end = t.q_pos0 + t.q_rows;

  int buf = 0, cur_qt = n_qt - 1, cur_hh = 0;
  for (int it = 0; it < n_it; it++) {
    const int i0 = cur_qt * 64;
    if (++cur_hh == p.grp) { cur_hh = 0; cur_qt--; }
    const int ahead = n_it - 1 - it;  // tiles after this one
    const int qpos0 = t.q_pos0 + i0;  // position of the tile's first query
    const bool compute = qpos0 + 63 >= kpos_w_min;  // otherwise every query of the tile precedes every key of this wave
    const bool masked = qpos0 < kpos_w_max || qpos0 + 64 > qpos_end;
    // the tile three iterations ahead is fetched inside this tile's arithmetic when it is a full tile and this
    // wave computes an unmasked one (the common case), else in front of it
    const bool fetch = ahead >= NBUF - 1;
    const bool fused = fetch && compute && !masked && st_qt * 64 + 64 <= t.q_rows;
    pc_buf = (buf + NBUF - 1) & (NBUF - 1);
    if (fetch && !fused) stage(pc_buf);

    if (compute) {
      const char *Qb = Qs + buf * TILEB;
      const char *Ob = Os + buf * TILEB;
      if (masked)
        dkdv_tile<D, true>(Qb, Ob, Ls + buf * 64, Ds + buf * 64, kreg, vreg, dk_acc, dv_acc, qpos0, kpos, qpos_end, c_log2, hi, lo, no_piece);
      else if (fused)
        dkdv_tile<D, false>(Qb, Ob, Ls + buf * 64, Ds + buf * 64, kreg, vreg, dk_acc, dv_acc, qpos0, kpos, qpos_end, c_log2, hi, lo, stage_piece);
      else
        dkdv_tile<D, false>(Qb, Ob, Ls + buf * 64, Ds + buf * 64, kreg, vreg, dk_acc, dv_acc, qpos0, kpos, qpos_end, c_log2, hi, lo, no_piece);
    }
    // the next tile must have landed; the ones behind it may stay in flight
    if (ahead >= NBUF - 1) zp_wait_async_upto<(NBUF - 2) * LOADS>();
    else if (ahead == 2) zp_wait_async_upto<LOADS>();
    else zp_wait_async();
    __syncthreads();
    buf = (buf + 1) & (NBUF - 1);
  }

  if (key_ok) {
    if (p.accumulate) {
      add_acc_rows<D>((float *)p.dk + ktok * p.dkv_stride + (int64_t)g * D + 4 * hi, dk_acc, p.scale);
      add_acc_rows<D>((float *)p.dv + ktok * p.dkv_stride + (int64_t)g * D + 4 * hi, dv_acc, 1.0f);
    } else {
      store_acc_rows<D>(p.dk + ktok * p.dkv_stride + (int64_t)g * D + 4 * hi, dk_acc, p.scale);
      store_acc_rows<D>(p.dv + ktok * p.dkv_stride + (int64_t)g * D + 4 * hi, dv_acc, 1.0f);
    }
  }
}

// ---------------------------------------------------------------------------- dK, dV at head dimension 128
// The LDS read addresses of zp_lds_offsets with three registers instead of sixteen: the swizzle XORs the 16-byte
// chunk index with a function of the row, so the offsets of the k-steps (row pattern) and of the 32-column blocks
// (transposed pattern) differ from the first one by an XOR with a constant -- also after a multiple of 256 bytes
// (tile, row block) has been added.
struct dkdv_lds_addr {
  unsigned row0, tr0[2];
  __device__ __forceinline__ void init(int lane) {
    zp_lds_offsets<128> lo;
    lo.init(lane);
    row0 = lo.row_off[0]; tr0[0] = lo.tr_off[0][0]; tr0[1] = lo.tr_off[1][0];
  }
  // base = LDS address of the tile + the lane's first offset + the row block, see rows_base / tr_base
  __device__ __forceinline__ unsigned rows_base(const char *tile, int blk) const { return zp_lds_addr(tile) + row0 + blk * 32 * 256; }
  static __device__ __forceinline__ bf16x8 rows(unsigned base, int kk) {
    return *(const ZP_LDS bf16x8 *)(unsigned long long)(base ^ (unsigned)(kk << 5));
  }
  __device__ __forceinline__ unsigned tr_base(const char *tile, int blk, int j) const { return zp_lds_addr(tile) + tr0[j] + blk * 32 * 256; }
  static __device__ __forceinline__ bf16x8 tr(unsigned b0, unsigned b1, int m, int db) {
    const unsigned o = (unsigned)(db << 6);
    s16x4 u0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ZP_LDS s16x4 *)(unsigned long long)((b0 ^ o) + m * 16 * 256));
    s16x4 u1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ZP_LDS s16x4 *)(unsigned long long)((b1 ^ o) + m * 16 * 256));
    return zp_cat(__builtin_bit_cast(bf16x4, u0), __builtin_bit_cast(bf16x4, u1));
  }
};

template <int D, bool MASK, bool PIECES, class Piece>
__device__ __forceinline__ void dkdv_block(const char *Qb, const char *Ob, const float *Lb, const float *Db, int qb,
                                           const bf16x8 (&kreg)[D / 16], const char *Vt, int vkb,
                                           f32x16 (&dk_acc)[D / 32], f32x16 (&dv_acc)[D / 32], int qpos0, int kpos,
                                           int qpos_end, float c_log2, int hi, const dkdv_lds_addr &la,
                                           Piece &&piece) {
  constexpr int KK = D / 16, DB = D / 32;
  f32x16 s, dp;
#pragma unroll
  for (int b = 0; b < 4; b++) {  // -LSE/scale and -D of the 16 query rows this lane holds
    const f32x4 l4 = *(const ZP_LDS f32x4 *)((const ZP_LDS char *)Lb + (qb * 32 + 8 * b + 4 * hi) * 4);
    const f32x4 d4 = *(const ZP_LDS f32x4 *)((const ZP_LDS char *)Db + (qb * 32 + 8 * b + 4 * hi) * 4);
#pragma unroll
    for (int c = 0; c < 4; c++) { s[4 * b + c] = l4[c]; dp[4 * b + c] = d4[c]; }
  }
  // Four runs of eight MFMAs -- S, dP, dV^T, dK^T -- each a fenced pipeline with its LDS operands two steps ahead;
  // the last two steps of a run request the first operands of the next one. One run at a time keeps the operands in
  // flight at 24 registers (all four streams two steps ahead would not fit beside the accumulators). The empty asm
  // in every step keeps the compiler from working out all the addresses of a run ahead of it.
  unsigned xb = la.rows_base(Qb, qb), yb = la.rows_base(Ob, qb), vb = la.rows_base(Vt, vkb);
  unsigned xt0 = la.tr_base(Ob, qb, 0), xt1 = la.tr_base(Ob, qb, 1), yt0 = la.tr_base(Qb, qb, 0), yt1 = la.tr_base(Qb, qb, 1);
  bf16x8 x[KK], y[KK], v[KK], xt[2 * DB], yt[2 * DB];
  x[0] = la.rows(xb, 0); x[1] = la.rows(xb, 1);
  zp_static_for<KK>([&](auto kk) {
    constexpr int k = kk.value;
    __builtin_amdgcn_sched_barrier(0);
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[k], kreg[k], s, 0, 0, 0);
    asm volatile("" : "+v"(xb), "+v"(yb), "+v"(vb));
    if constexpr (k + 2 < KK) x[k + 2] = la.rows(xb, k + 2);
    else { y[k + 2 - KK] = la.rows(yb, k + 2 - KK); v[k + 2 - KK] = la.rows(vb, k + 2 - KK); }
    if constexpr (PIECES) piece(kk);
  });
  zp_static_for<KK>([&](auto kk) {
    constexpr int k = kk.value;
    __builtin_amdgcn_sched_barrier(0);
    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(y[k], v[k], dp, 0, 0, 0);
    asm volatile("" : "+v"(yb), "+v"(vb), "+v"(xt0), "+v"(xt1));
    if constexpr (k + 2 < KK) { y[k + 2] = la.rows(yb, k + 2); v[k + 2] = la.rows(vb, k + 2); }
    else xt[k + 2 - KK] = la.tr(xt0, xt1, (k + 2 - KK) / DB, (k + 2 - KK) % DB);
  });
  __builtin_amdgcn_sched_barrier(0);
  unsigned ppk[8], dpk[8];
#pragma unroll
  for (int q = 0; q < 8; q++) dkdv_pair<MASK>(s, dp, 2 * q, qb, hi, qpos0, kpos, qpos_end, c_log2, ppk[q], dpk[q]);
  const bf16x8 pb[2] = {__builtin_bit_cast(bf16x8, (u32x4){ppk[0], ppk[1], ppk[2], ppk[3]}),
                        __builtin_bit_cast(bf16x8, (u32x4){ppk[4], ppk[5], ppk[6], ppk[7]})};
  const bf16x8 dsb[2] = {__builtin_bit_cast(bf16x8, (u32x4){dpk[0], dpk[1], dpk[2], dpk[3]}),
                         __builtin_bit_cast(bf16x8, (u32x4){dpk[4], dpk[5], dpk[6], dpk[7]})};
  zp_static_for<2 * DB>([&](auto ii) {
    constexpr int i = ii.value, m = i / DB, db = i % DB;
    __builtin_amdgcn_sched_barrier(0);
    dv_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xt[i], pb[m], dv_acc[db], 0, 0, 0);
    asm volatile("" : "+v"(xt0), "+v"(xt1), "+v"(yt0), "+v"(yt1));
    if constexpr (i + 2 < 2 * DB) xt[i + 2] = la.tr(xt0, xt1, (i + 2) / DB, (i + 2) % DB);
    else yt[i + 2 - 2 * DB] = la.tr(yt0, yt1, (i + 2 - 2 * DB) / DB, (i + 2 - 2 * DB) % DB);
  });
  zp_static_for<2 * DB>([&](auto ii) {
    constexpr int i = ii.value, m = i / DB, db = i % DB;
    __builtin_amdgcn_sched_barrier(0);
    dk_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(yt[i], dsb[m], dk_acc[db], 0, 0, 0);
    asm volatile("" : "+v"(yt0), "+v"(yt1));
    if constexpr (i + 2 < 2 * DB) yt[i + 2] = la.tr(yt0, yt1, (i + 2) / DB, (i + 2) % DB);
  });
  __builtin_amdgcn_sched_barrier(0);
}


#ifndef ZP_DKDV_NBUF
#define ZP_DKDV_NBUF 2
#endif
// Two waves per SIMD for head dimension 128 as well: two independent workgroups of four waves per CU (80 KB of LDS
// each), a wave holding its K operands (32 registers) and its dK^T/dV^T accumulators (128) and working on 32-query
// tiles, one block's S and dP at a time; the V operands do not fit beside them in 256 registers and are read from
// LDS, where the workgroup's 128 V rows are staged once. An MFMA takes about 20 cycles of its wave's vector issue
// time and the wave's LDS, scalar and wait instructions issue in line with it; a second wave on the SIMD, from a
// workgroup that meets its own barriers, runs under all of that.
__global__ __launch_bounds__(BWD_NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dkdv128_kernel(zp_bwd_params p) {
  constexpr int D = 128, QT = 32;
  constexpr int TILEB = QT * D * 2;                // a staged tile: 32 query rows
  constexpr int NBUF = ZP_DKDV_NBUF;               // staging buffers (three would not fit two workgroups per CU with the seeds)
  typedef zp_stager<D, 8> stager;                  // 4 waves x 2 wave-loads = the first 32 rows of its 64-row pattern
  constexpr int PW = stager::PER_WAVE;
  constexpr int LOADS = 2 * PW + 2;                // async loads one wave issues per staged tile
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char *Qs = smem;                                 // [NBUF][32][D]
  char *Os = smem + NBUF * TILEB;                  // [NBUF][32][D]  (dO)
  char *Vs = smem + 2 * NBUF * TILEB;              // [2][64][D]: the workgroup's V rows, staged once
  float *Ls = (float *)(Vs + 2 * 64 * D * 2);      // [NBUF][32] -LSE / scale
  float *Ds = Ls + NBUF * QT;                      // [NBUF][32] -D

  const int unit = zp_item_of_block(p.work_kv_short, (int *)(Ds + NBUF * QT));
  if (unit < 0 || unit >= p.n_kv_tiles_short * p.Hkv) return;
  const int tile_idx = unit / p.Hkv, g = unit - tile_idx * p.Hkv;
  const zp_tile t = p.kv_tiles_short[tile_idx];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int kl = lane & 31, hi = lane >> 5;
  const int krow = w * 32 + kl;
  const bool key_ok = krow < t.k_len;
  const int64_t ktok = (int64_t)t.k_tok0 + krow;
  const int kpos = t.k_pos0 + krow;

  // K operands in registers; V operands from LDS (rows past the block's last key repeat it: a key column never
  // mixes with another, and those columns are not stored)
  bf16x8 kreg[D / 16];
  {
    const __bf16 *kp = p.k + ktok * p.k_stride + (int64_t)g * D + 8 * hi;
#pragma unroll
    for (int kk = 0; kk < D / 16; kk++) {
      if (key_ok) kreg[kk] = *(const bf16x8 *)(kp + 16 * kk);
      else kreg[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
  }

  f32x16 dk_acc[D / 32], dv_acc[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) { dk_acc[i][r] = 0.f; dv_acc[i][r] = 0.f; }
  const float c_log2 = p.scale_log2;

  const int n_qt = (t.q_rows + QT - 1) / QT;
  const int n_it = n_qt * p.grp;  // iterations: query tiles outermost (last tile first), heads of the group innermost

  stager qst, ost;
  qst.init(p.q + (int64_t)t.q_tok0 * p.q_stride + (int64_t)g * p.grp * D, p.q_stride, tid);
  ost.init(p.dout + (int64_t)t.q_tok0 * p.do_stride + (int64_t)g * p.grp * D, p.do_stride, tid);
  dkdv_lds_addr la;
  la.init(lane);
  {
    zp_stager<D> vst;
    vst.init(p.v + (int64_t)t.k_tok0 * p.v_stride + (int64_t)g * D, p.v_stride, tid);
    vst.issue(Vs, 0, t.k_len);
    vst.issue(Vs + 64 * D * 2, 64, t.k_len);
  }
  const char *Vt = Vs + (w >> 1) * (64 * D * 2);
  const int vkb = w & 1;
  // 32 floats of a row vector, one per lane of the lower half-wave (rows past the last valid one repeat it)
  auto stage_f32x32 = [&](float *dst, const float *src, int first, int last_valid) {
    int i = first + (lane & 31);
    if (i > last_valid) i = last_valid;
    if (lane < 32) zp_dma4(src + i, __builtin_amdgcn_readfirstlane(zp_lds_addr(dst)));
  };
  int st_hh = 0, st_qt = n_qt - 1;
  auto stage = [&](int buf) {
    const int hh = st_hh, i0 = st_qt * QT;
    const int h = g * p.grp + hh;
    if (++st_hh == p.grp) { st_hh = 0; st_qt--; }
    qst.issue(Qs + buf * TILEB, i0, t.q_rows, (int64_t)hh * D);
    ost.issue(Os + buf * TILEB, i0, t.q_rows, (int64_t)hh * D);
    const int64_t base = (int64_t)h * p.T + t.q_tok0;
    stage_f32x32(Ls + buf * QT, p.lse2 + base, i0, t.q_rows - 1);
    stage_f32x32(Ds + buf * QT, p.dvec + base, i0, t.q_rows - 1);
  };
  // the same copies for a tile of 32 valid rows, one per k-step of the S chain (piece 0: the scalar addresses)
  const void *pc_q = nullptr, *pc_o = nullptr, *pc_l = nullptr, *pc_d = nullptr;
  unsigned pc_buf = 0;
  auto stage_piece = [&](auto n) {
    constexpr int N = decltype(n)::value;
    static_assert(2 * PW + 3 <= D / 16, "the copies of a tile fit the steps of one chain");
    if constexpr (N == 0) {
      const int hh = st_hh, i0 = st_qt * QT;
      const int h = g * p.grp + hh;
      if (++st_hh == p.grp) { st_hh = 0; st_qt--; }
      pc_q = zp_uniform_ptr(qst.base + (int64_t)i0 * qst.stride + (int64_t)hh * D);
      pc_o = zp_uniform_ptr(ost.base + (int64_t)i0 * ost.stride + (int64_t)hh * D);
      const int64_t base = (int64_t)h * p.T + t.q_tok0 + i0;
      pc_l = zp_uniform_ptr(p.lse2 + base);
      pc_d = zp_uniform_ptr(p.dvec + base);
    } else if constexpr (N <= PW) {
      zp_dma16_so(pc_q, qst.off[N - 1], __builtin_amdgcn_readfirstlane(zp_lds_addr(Qs) + pc_buf * TILEB + (qst.w * PW + N - 1) * 1024));
    } else if constexpr (N <= 2 * PW) {
      zp_dma16_so(pc_o, ost.off[N - PW - 1], __builtin_amdgcn_readfirstlane(zp_lds_addr(Os) + pc_buf * TILEB + (ost.w * PW + N - PW - 1) * 1024));
    } else if constexpr (N == 2 * PW + 1) {
      if (lane < 32) zp_dma4_so(pc_l, lane * 4, __builtin_amdgcn_readfirstlane(zp_lds_addr(Ls) + pc_buf * (QT * 4)));
    } else if constexpr (N == 2 * PW + 2) {
      if (lane < 32) zp_dma4_so(pc_d, lane * 4, __builtin_amdgcn_readfirstlane(zp_lds_addr(Ds) + pc_buf * (QT * 4)));
    }
  };
  auto no_piece = [](auto) {};

  if (n_it > 0) stage(0);
  zp_wait_async();
#pragma unroll
  for (int b = 1; b < NBUF - 1; b++)
    if (n_it > b) stage(b);
  __syncthreads();

  const int kpos_w_min = t.k_pos0 + w * 32, kpos_w_max = t.k_pos0 + w * 32 + 31;
  const int qpos_end = t.q_pos0 + t.q_rows;

  int buf = 0, cur_qt = n_qt - 1, cur_hh = 0;
  for (int it = 0; it < n_it; it++) {
    const int i0 = cur_qt * QT;
    if (++cur_hh == p.grp) { cur_hh = 0; cur_qt--; }
    const int ahead = n_it - 1 - it;        // tiles after this one
    const int qpos0 = t.q_pos0 + i0;        // position of the tile's first query
    const bool compute = qpos0 + QT - 1 >= kpos_w_min;  // otherwise every query of the tile precedes every key of this wave
    const bool masked = qpos0 < kpos_w_max || qpos0 + QT > qpos_end;
    // the tile NBUF - 1 iterations ahead is fetched inside this tile's S chain when it is a full tile and this wave
    // computes an unmasked one (the common case), else in front
    const bool fetch = ahead >= NBUF - 1;
    const bool fused = fetch && compute && !masked && st_qt * QT + QT <= t.q_rows;
    pc_buf = buf == 0 ? NBUF - 1 : buf - 1;
    if (fetch && !fused) stage(pc_buf);

    if (compute) {
      const char *Qb = Qs + buf * TILEB;
      const char *Ob = Os + buf * TILEB;
      if (masked)
        dkdv_block<D, true, false>(Qb, Ob, Ls + buf * QT, Ds + buf * QT, 0, kreg, Vt, vkb, dk_acc, dv_acc, qpos0, kpos, qpos_end, c_log2, hi, la, no_piece);
      else if (fused)
        dkdv_block<D, false, true>(Qb, Ob, Ls + buf * QT, Ds + buf * QT, 0, kreg, Vt, vkb, dk_acc, dv_acc, qpos0, kpos, qpos_end, c_log2, hi, la, stage_piece);
      else
        dkdv_block<D, false, false>(Qb, Ob, Ls + buf * QT, Ds + buf * QT, 0, kreg, Vt, vkb, dk_acc, dv_acc, qpos0, kpos, qpos_end, c_log2, hi, la, no_piece);
    }
    // the next tile must have landed; the one behind it may stay in flight
    if (ahead >= NBUF - 1) zp_wait_async_upto<(NBUF - 2) * LOADS>();
    else zp_wait_async();
    __syncthreads();
    buf = buf + 1 == NBUF ? 0 : buf + 1;
  }

  if (key_ok) {
    if (p.accumulate) {
      add_acc_rows<D>((float *)p.dk + ktok * p.dkv_stride + (int64_t)g * D + 4 * hi, dk_acc, p.scale);
      add_acc_rows<D>((float *)p.dv + ktok * p.dkv_stride + (int64_t)g * D + 4 * hi, dv_acc, 1.0f);
    } else {
      store_acc_rows<D>(p.dk + ktok * p.dkv_stride + (int64_t)g * D + 4 * hi, dk_acc, p.scale);
      store_acc_rows<D>(p.dv + ktok * p.dkv_stride + (int64_t)g * D + 4 * hi, dv_acc, 1.0f);
    }
  }
}

}  // namespace

extern "C" void zp_prof_begin(const char *name, hipStream_t stream);
extern "C" void zp_prof_end(hipStream_t stream);

extern "C" int zp_attn_bwd_block_rows(int d, int which) { (void)d; (void)which; return 128; }

extern "C" int zp_launch_attn_bwd(const zp_bwd_params *p_in, int d, hipStream_t stream) {
  zp_bwd_params params = *p_in;
  zp_bwd_params *p = &params;
  const int dq_units = p->n_dq_tiles * p->Hkv;
  const int kv_units = p->n_kv_tiles * p->Hkv;
  // item numbering padded to a multiple of 8 (one residue per XCD); the kernels drop the padding
  int32_t *c = p->work_dq.counters;
  const int dq_grid = zp_plan_work_split(p->work_dq, c, ((dq_units + 7) / 8) * 8 * p->grp);
  const int kv_grid = zp_plan_work_split(p->work_kv, c ? c + ZP_COUNTER_BYTES / 4 : nullptr, ((kv_units + 7) / 8) * 8);
  const int kv_units_short = p->n_kv_tiles_short * p->Hkv;   // only ever non-zero at d = 128
  const int kv_short_grid = zp_plan_work_split(p->work_kv_short, c ? c + 2 * (ZP_COUNTER_BYTES / 4) : nullptr, ((kv_units_short + 7) / 8) * 8);
  if (dq_units > 0) {
    zp_prof_begin("attn_bwd_dq", stream);
    if (d == 128) hipLaunchKernelGGL((attn_bwd_dq_kernel<128>), dim3(dq_grid), dim3(BWD_NT), 4 * 64 * 128 * 2 + 16, stream, *p);
    else hipLaunchKernelGGL((attn_bwd_dq_kernel<64>), dim3(dq_grid), dim3(BWD_NT), 4 * 64 * 64 * 2 + 16, stream, *p);
    zp_prof_end(stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  if (kv_units > 0) {
    zp_prof_begin("attn_bwd_dkdv", stream);
    if (d == 128) hipLaunchKernelGGL((attn_bwd_dkdv_kernel<128>), dim3(kv_grid), dim3(BWD_NT), 8 * 64 * 128 * 2 + 2048 + 16, stream, *p);
    else hipLaunchKernelGGL((attn_bwd_dkdv_kernel<64>), dim3(kv_grid), dim3(BWD_NT), 8 * 64 * 64 * 2 + 2048 + 16, stream, *p);
    zp_prof_end(stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  if (kv_units_short > 0) {
    zp_prof_begin("attn_bwd_dkdv_short", stream);
    hipLaunchKernelGGL(attn_bwd_dkdv128_kernel, dim3(kv_short_grid), dim3(BWD_NT),
                       2 * ZP_DKDV_NBUF * 32 * 128 * 2 + 2 * 64 * 128 * 2 + 2 * ZP_DKDV_NBUF * 32 * 4 + 16, stream, *p);
    zp_prof_end(stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}
