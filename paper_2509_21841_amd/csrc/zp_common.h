// Shared device-side types and small helpers for the gfx950 kernels of the attention engine.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include <utility>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define ZP_LDS __attribute__((address_space(3)))

// One unit of attention work: a block of query rows against one run of keys of the same sequence.
// Whole sequences and (Q chunk, KV chunk) pairs (Sec. 3.2) both reduce to this.
struct zp_tile {
  int32_t q_tok0;    // first packed query token of the block
  int32_t q_rows;    // query rows in the block
  int32_t q_pos0;    // position of the first query row inside its sequence
  int32_t k_tok0;    // first packed token of the key run
  int32_t k_len;     // keys in the run
  int32_t k_pos0;    // position of the first key inside the sequence
  int32_t out_row0;  // first output row (packed token, or partial-result row)
  int32_t aux;       // kernel specific
};

// How a launch hands its work items to workgroups. The XCDs of a chip do not run equally fast (on the boxes measured
// the same four finish an equal share 4-8 % later than the other four), and the hardware deals workgroups to them
// round-robin, so with one item per workgroup the fast ones idle at the end. Items 0 .. n_static-1 are therefore taken
// by number (workgroup b runs item b, on XCD b % 8, no cost), and the last ones -- the cheapest of the launch -- are
// claimed at run time from one counter per XCD by the workgroups behind them, of which the launch holds more than
// there are items left: a workgroup whose own XCD has none left takes one from a neighbour, surplus workgroups exit.
// A claim costs its workgroup an atomic round trip (about a microsecond), so launches of light items claim the last
// eighth and launches of heavy items (dyn_div = 2) the last half.
// counters: 8 ints, ZP_COUNTER_STRIDE apart, zero before the launch. n_items and n_static are multiples of 8.
#define ZP_COUNTER_STRIDE 32
#define ZP_COUNTER_BYTES (8 * ZP_COUNTER_STRIDE * 4)
struct zp_work_split {
  int32_t *counters;
  int32_t n_items, n_static;
  int32_t dyn_div;  // 1 / dyn_div of the items are claimed at run time (0: the default, 8)
};
// Host side: the split and the grid of a launch of n_items (a multiple of 8) items.
inline int zp_plan_work_split(zp_work_split &ws, int32_t *counters, int n_items) {
  ws.counters = counters;
  ws.n_items = n_items;
  if (n_items < 8 * 128 || counters == nullptr) {  // small launches: every item by number
    ws.n_static = n_items;
    return n_items;
  }
  const int div = ws.dyn_div >= 2 ? ws.dyn_div : 8;
  ws.n_static = (n_items / 8 * (div - 1) / div) * 8;
  const int n_dyn = n_items - ws.n_static;
  return ws.n_static + ((n_dyn * 3 / 2 + 7) / 8) * 8;
}
// Device side: the item of this workgroup, or -1 if there is none left for it. `slot` is one int of LDS. All threads
// of the workgroup must call it (it holds a barrier for the workgroups that claim).
__device__ __forceinline__ int zp_item_of_block(const zp_work_split &ws, int *slot) {
  const int b = blockIdx.x;
  if (b < ws.n_static) return b;
  if (threadIdx.x == 0) {
    const int per = (ws.n_items - ws.n_static) >> 3, x = b & 7;
    int item = -1;
    for (int j = 0; j < 8 && item < 0; j++) {
      const int y = (x + j) & 7;
      const int k = atomicAdd(ws.counters + y * ZP_COUNTER_STRIDE, 1);
      if (k < per) item = ws.n_static + 8 * k + y;
    }
    *slot = item;
  }
  __syncthreads();
  return __builtin_amdgcn_readfirstlane(*slot);
}

// Parameters shared by the attention kernels. Strides are token strides in elements.
struct zp_attn_params {
  const __bf16 *q, *k, *v;
  int64_t q_stride, k_stride, v_stride;
  const zp_tile *tiles;
  int32_t n_tiles, Hq, Hkv, grp;
  float scale_log2;  // scale * log2(e)
  float scale;
  void *o;           // bf16 [.][Hq][d] (whole) or float [part_rows][Hq][d] (partial)
  int64_t o_stride;  // token stride of o in elements
  float *lse;        // [Hq][lse_stride]
  int64_t lse_stride;
  int32_t update;    // partial kernel only: merge the result into the running (o, lse) found at the output rows
  zp_work_split work;  // which workgroups take their item by number and which claim one (set by the launcher)
};

// blockIdx -> (unit, head-in-group). Workgroups are dealt to the 8 XCDs round-robin by blockIdx, so
// units (tile, kv head) are dealt round-robin too -- the cost-sorted list stays balanced across XCDs --
// while the grp query heads of one unit get consecutive slots on the SAME XCD and share K/V in its L2.
__device__ __forceinline__ void zp_block_to_unit(int bid, int grp, int &unit, int &hh) {
  int x = bid & 7, y = bid >> 3;
  hh = y % grp;
  unit = (y / grp) * 8 + x;
}

__device__ __forceinline__ float zp_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Three-operand maximum in one VALU operation (operands are finite or -inf here, never NaN). Inline assembly is
// invisible to the compiler's hazard checks: never feed it a register an MFMA has just written unless an ordinary
// instruction that reads the same accumulator comes first (data-dependently), which makes the compiler insert the
// required wait states.
__device__ __forceinline__ float zp_max3(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}
// max / sum across the two lanes l and l^32 that hold the two halves of one 32x32 MFMA column.
__device__ __forceinline__ float zp_pair_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float zp_pair_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 16-byte LDS read and the gfx950 transposing 8-byte LDS read.
__device__ __forceinline__ bf16x8 zp_lds_read16(const char *smem, int off) {
  return *(const ZP_LDS bf16x8 *)((const ZP_LDS char *)smem + off);
}
// Within each group of 16 lanes, lane i passes the address of 4 consecutive 16-bit elements of row i/4,
// columns 4*(i%4)..+3 of a 4x16 block, and receives column i of rows 0..3.
__device__ __forceinline__ bf16x4 zp_lds_read_tr(const char *smem, int off) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ZP_LDS s16x4 *)((ZP_LDS char *)smem + off));
  return __builtin_bit_cast(bf16x4, v);
}

__device__ __forceinline__ bf16x8 zp_cat(bf16x4 a, bf16x4 b) {
  return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Swizzle for LDS tiles that are read BOTH row-wise (16 lanes: 16 consecutive rows, same 16-byte chunk) and
// with the transposing read (32 lanes: 4 consecutive rows x 64 contiguous bytes): the 16-byte chunk index is
// XORed with the row's low four bits with their two 2-bit fields swapped, which spreads both patterns over
// all banks. `chunk` is the 16-byte chunk index in the row; returns the byte offset of that chunk.
template <int D>
__device__ __forceinline__ int zp_swz(int row, int chunk) {
  if (D == 128) return row * 256 + ((chunk ^ (((row & 3) << 2) | ((row >> 2) & 3))) << 4);
  return row * 128 + ((chunk ^ (((row & 1) << 2) | ((row >> 1) & 3))) << 4);
}
// Byte offset of element column `col` (multiple of 4) of row `row` under zp_swz.
template <int D>
__device__ __forceinline__ int zp_swz_col(int row, int col) {
  return zp_swz<D>(row, col >> 3) + ((col & 7) << 1);
}

// ---- asynchronous global -> LDS copies -------------------------------------------------------------
// The direct-to-LDS loads are issued from inline assembly so that they stay truly asynchronous: the
// compiler does not track them, inserts no waits for them, and its workgroup barriers do not drain them.
// Ordering is explicit: zp_wait_async*() before the barrier that publishes a staged tile. Each lane's bytes
// land at (wave-uniform LDS base in M0) + lane * size. The compiler checks no hardware hazard for inline assembly,
// so each block pads itself: s_mov m0 plus s_nop 3 put five wait states between any vector instruction that
// wrote the scalar base (a v_readlane restoring a spilled SGPR, a v_readfirstlane) and the load that reads it,
// and cover the one wait state M0 needs before a direct-to-LDS load.
__device__ __forceinline__ unsigned zp_lds_addr(const void *p) {
  return (unsigned)(unsigned long long)(ZP_LDS const char *)p;
}
__device__ __forceinline__ void zp_dma16(const void *g, unsigned lds_base_uniform) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 3\n\tglobal_load_lds_dwordx4 %0, off\n" ::"v"(g), "s"(lds_base_uniform) : "memory");
}
__device__ __forceinline__ void zp_dma4(const void *g, unsigned lds_base_uniform) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 3\n\tglobal_load_lds_dword %0, off\n" ::"v"(g), "s"(lds_base_uniform) : "memory");
}

// Copy of 64 consecutive floats (one per lane), issued by every wave of the workgroup to the same
// destination so that all waves have the same number of loads in flight.
__device__ __forceinline__ void zp_stage_async_f32x64(float *lds_dst, const float *gsrc, int first, int last_valid,
                                                      int lane) {
  int i = first + lane;
  if (i > last_valid) i = last_valid;
  zp_dma4(gsrc + i, __builtin_amdgcn_readfirstlane(zp_lds_addr(lds_dst)));
}
// wait for every outstanding vector-memory operation of this wave (vmcnt = 0), nothing else
__device__ __forceinline__ void zp_wait_async() { __builtin_amdgcn_s_waitcnt(0x0F70); }
// wait until at most N vector-memory operations of this wave are outstanding (N compile-time, <= 63)
template <int N>
__device__ __forceinline__ void zp_wait_async_upto() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// 16-byte direct-to-LDS load addressed as (wave-uniform 64-bit base) + (per-lane 32-bit byte offset)
__device__ __forceinline__ void zp_dma16_so(const void *sbase_uniform, unsigned voff, unsigned lds_base_uniform) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 3\n\tglobal_load_lds_dwordx4 %0, %1\n" ::"v"(voff), "s"(sbase_uniform),
               "s"(lds_base_uniform)
               : "memory");
}
// the same with 4 bytes per lane
__device__ __forceinline__ void zp_dma4_so(const void *sbase_uniform, unsigned voff, unsigned lds_base_uniform) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 3\n\tglobal_load_lds_dword %0, %1\n" ::"v"(voff), "s"(sbase_uniform),
               "s"(lds_base_uniform)
               : "memory");
}
__device__ __forceinline__ const void *zp_uniform_ptr(const void *p) {
  unsigned long long v = (unsigned long long)p;
  unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return (const void *)(((unsigned long long)hi << 32) | lo);
}

// Per-thread state of the asynchronous [64][D] tile copy: the lane's byte offsets inside a tile are worked
// out once (they carry the LDS swizzle); issuing a tile is then scalar address arithmetic plus the loads.
// `init` takes the tensor base of the row run and the token stride (64 * stride * 2 bytes must fit 32 bits);
// `issue` copies rows row0 .. row0+63 (rows past rows_total clamp to the last valid row).
template <int D, int NW = 4>
struct zp_stager {
  static constexpr int PER_WAVE = 64 * D * 2 / 1024 / NW;  // 1 KiB wave-loads per wave (NW = 4: the four waves share a 64-row tile; NW = 8: they cover its first 32 rows)
  static constexpr int LOADS = PER_WAVE;
  unsigned off[PER_WAVE];  // bytes from the tile's first row
  int64_t stride;
  const __bf16 *base;
  int w, lane;
  __device__ __forceinline__ static void row_chunk(int blk, int lane, int &r, int &c) {
    if (D == 128) {
      r = blk * 4 + (lane >> 4);
      c = (lane & 15) ^ (((r & 3) << 2) | ((r >> 2) & 3));
    } else {
      r = blk * 8 + (lane >> 3);
      c = (lane & 7) ^ (((r & 1) << 2) | ((r >> 1) & 3));
    }
  }
  __device__ __forceinline__ void init(const __bf16 *gbase, int64_t tok_stride, int tid) {
    lane = tid & 63;
    w = __builtin_amdgcn_readfirstlane(tid >> 6);
    stride = tok_stride;
    base = gbase;
#pragma unroll
    for (int n = 0; n < PER_WAVE; n++) {
      int r, c;
      row_chunk(w * PER_WAVE + n, lane, r, c);
      off[n] = (unsigned)(((int64_t)r * tok_stride + c * 8) * 2);
    }
  }
  // extra: a wave-uniform element offset added to every source address (e.g. head * D)
  __device__ __forceinline__ void issue(char *lds_tile, int row0, int rows_total, int64_t extra = 0) const {
    const unsigned lds0 = __builtin_amdgcn_readfirstlane(zp_lds_addr(lds_tile));
    if (row0 + 64 <= rows_total) {
      const void *sb = zp_uniform_ptr(base + (int64_t)row0 * stride + extra);
#pragma unroll
      for (int n = 0; n < PER_WAVE; n++) zp_dma16_so(sb, off[n], lds0 + (w * PER_WAVE + n) * 1024);
    } else {
#pragma unroll
      for (int n = 0; n < PER_WAVE; n++) {
        int r, c;
        row_chunk(w * PER_WAVE + n, lane, r, c);
        int gr = row0 + r;
        if (gr > rows_total - 1) gr = rows_total - 1;
        zp_dma16(base + (int64_t)gr * stride + c * 8 + extra, lds0 + (w * PER_WAVE + n) * 1024);
      }
    }
  }
};

// LDS read offsets of one lane for the two MFMA operand patterns of a [64][D] zp_swz tile, worked out once.
// rows(kb, kk): 16 bytes of row 32*kb + (lane%32), head-dim elements 16*kk + 8*(lane/32) ..+7  (row-major operand)
// tr(kb, m, j, db): transposed 4-row piece for k-slots 4j..4j+3 of MFMA m of 32-row block kb, columns 32*db + lane%32
template <int D>
struct zp_lds_offsets {
  int row_off[D / 16];      // + kb * 32 * ROWB
  int tr_off[2][D / 32];    // [j][db], + (kb * 32 + m * 16) * ROWB
  static constexpr int ROWB = D * 2;
  __device__ __forceinline__ void init(int lane) {
    const int r32 = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < D / 16; kk++) row_off[kk] = zp_swz<D>(r32, 2 * kk + hi);
    const int g16 = lane >> 4, i16 = lane & 15;
    const int trow = 4 * (g16 >> 1) + (i16 >> 2);
    const int tcol = 16 * (g16 & 1) + 4 * (i16 & 3);
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int db = 0; db < D / 32; db++) tr_off[j][db] = zp_swz_col<D>(8 * j + trow, db * 32 + tcol);
  }
  // Absolute form: the lane's offsets include the LDS address of `base` from then on, and the *_at readers take a
  // tile's byte offset from `base` -- with a compile-time offset every read is a register plus an immediate (the
  // pointer form costs one vector add per read for the base, which the compiler only knows as a relocation).
  __device__ __forceinline__ void init_abs(int lane, const char *base) {
    init(lane);
    const int b = (int)(unsigned)(unsigned long long)(const ZP_LDS char *)base;
#pragma unroll
    for (int kk = 0; kk < D / 16; kk++) {
      row_off[kk] += b;
      asm volatile("" : "+v"(row_off[kk]));  // opaque from here on: the compiler would otherwise split the sum again and redo the add at every read
    }
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int db = 0; db < D / 32; db++) {
        tr_off[j][db] += b;
        asm volatile("" : "+v"(tr_off[j][db]));
      }
  }
  __device__ __forceinline__ bf16x8 rows_at(int tile_off, int kb, int kk) const {
    return *(const ZP_LDS bf16x8 *)(unsigned long long)(unsigned)(row_off[kk] + tile_off + kb * 32 * ROWB);
  }
  __device__ __forceinline__ bf16x8 tr_at(int tile_off, int kb, int m, int db) const {
    const int o = tile_off + (kb * 32 + m * 16) * ROWB;
    s16x4 u0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ZP_LDS s16x4 *)(unsigned long long)(unsigned)(tr_off[0][db] + o));
    s16x4 u1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ZP_LDS s16x4 *)(unsigned long long)(unsigned)(tr_off[1][db] + o));
    return zp_cat(__builtin_bit_cast(bf16x4, u0), __builtin_bit_cast(bf16x4, u1));
  }
  // the swizzle depends on row % 16 only (D = 128) / row % 8 (D = 64), so blocks of 32 and 16 rows shift by a constant
  __device__ __forceinline__ bf16x8 rows(const char *tile, int kb, int kk) const {
    return zp_lds_read16(tile, row_off[kk] + kb * 32 * ROWB);
  }
  __device__ __forceinline__ bf16x8 tr(const char *tile, int kb, int m, int db) const {
    const int o = (kb * 32 + m * 16) * ROWB;
    return zp_cat(zp_lds_read_tr(tile, tr_off[0][db] + o), zp_lds_read_tr(tile, tr_off[1][db] + o));
  }
};

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <class F, int... I>
__device__ __forceinline__ void zp_static_for_impl(F &&f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void zp_static_for(F &&f) {
  zp_static_for_impl(f, std::make_integer_sequence<int, N>{});
}
