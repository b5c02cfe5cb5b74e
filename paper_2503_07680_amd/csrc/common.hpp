// Device-side building blocks shared by the gfx950 attention kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hbp.h"

namespace hbp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kThreads = 256;  // 4 wavefronts per workgroup, one per SIMD

// v_mfma_f32_32x32x16_bf16: D[32x32] += A[32x16] * B[16x32].
// Lane l supplies A[l%32][8*(l/32)..+7] and B[8*(l/32)..+7][l%32]; it receives
// D[8*b + 4*(l/32) + v][l%32] in element 4*b + v (b,v in 0..3).
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

typedef short s16x4 __attribute__((ext_vector_type(4)));

// The same MFMA with its accumulator forced into the vector register file.  In kernels that also
// keep long-lived accumulators in the accumulation file the compiler would put EVERY MFMA result
// there and copy it out element by element before any vector arithmetic; scores that feed exp()
// right away are better produced in place.  Written as inline asm, so the wait states between an
// MFMA result and its first vector read are the caller's duty: see mfma_results_ready().
__device__ __forceinline__ f32x16 mfma32_vgpr_first(bf16x8 a, bf16x8 b) {
  f32x16 d;
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "v"(b));
  return d;
}
// first MFMA of a chain whose accumulator starts from another register tuple (left untouched)
__device__ __forceinline__ f32x16 mfma32_vgpr_from(bf16x8 a, bf16x8 b, const f32x16& c0) {
  f32x16 d;
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(d) : "v"(a), "v"(b), "v"(c0));
  return d;
}
__device__ __forceinline__ void mfma32_vgpr(f32x16& c, bf16x8 a, bf16x8 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
}
// Orders every later read of x and y after 19 idle issue cycles that follow the MFMAs which
// produced them (the longest wait the ISA asks for between a matrix result and a vector read).
__device__ __forceinline__ void mfma_results_ready(f32x16& x, f32x16& y) {
  asm volatile("s_nop 15\n\ts_nop 3" : "+v"(x), "+v"(y));
}

union Frag {
  bf16x8 v;
  u32x4 u;
  uint32_t w[4];
  s16x4 h[2];
};

// two fp32 -> packed bf16 pair (round to nearest even), low half = a
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

// acc + lo(w) + hi(w) for a packed bf16 pair (v_dot2c_f32_bf16 with a vector of ones)
__device__ __forceinline__ float add_bf16_pair(float acc, uint32_t w) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, 0x3f803f80u),
                                         acc, false);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

// max over a lane and its partner lane^32 (one v_permlane32_swap: r[0] = {lo half of x, lo half of
// x}, r[1] = {hi half of x, hi half of x} when both inputs are x)
__device__ __forceinline__ float max_with_other_half(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Store one 32x32 accumulator block as bf16: the lane's column (a query or key row of the output, at
// `row`: dim 0 of the block's 32 dims) and, of its 16 values, element 4b+v = dim 8b + 4hh + v.  The two
// half-waves exchange every second group of four, so that a lane ends up with 8 consecutive dims and
// writes 16 bytes at a time (two stores per block instead of four).  Called by all lanes (the exchange
// needs both halves); only lanes with `valid` store.
__device__ __forceinline__ void store_block_bf16(uint16_t* row, const f32x16& acc, float scale, int hh, bool valid) {
#pragma unroll
  for (int bp = 0; bp < 2; ++bp) {
    const int e = 8 * bp;  // elements e..e+3: dims 16bp + 4hh + v; e+4..e+7: dims 16bp + 8 + 4hh + v
    const uint32_t y0 = pack_bf16(acc[e] * scale, acc[e + 1] * scale), y1 = pack_bf16(acc[e + 2] * scale, acc[e + 3] * scale);
    const uint32_t x0 = pack_bf16(acc[e + 4] * scale, acc[e + 5] * scale), x1 = pack_bf16(acc[e + 6] * scale, acc[e + 7] * scale);
    const auto s0 = __builtin_amdgcn_permlane32_swap(y0, x0, false, false);
    const auto s1 = __builtin_amdgcn_permlane32_swap(y1, x1, false, false);
    // lower half-wave: dims 16bp + 0..7, upper: 16bp + 8..15
    if (valid) *(u32x4*)(row + 16 * bp + 8 * hh) = u32x4{s0[0], s1[0], s0[1], s1[1]};
  }
}

// ---- LDS tiles in their natural [row][dim] layout, 16-byte chunks XOR-swizzled -----------------
// Chunk c of row r sits at chunk position c ^ f(r).  Two access patterns have to stay free of bank
// conflicts (a bank line is 16 chunks): 16 consecutive rows read at one chunk index (row-major MFMA
// operand, 16-byte reads), and the 4 rows x 4 consecutive chunks that one half of a transposing read
// touches.
//  * 256-byte rows (16 chunks): a row starts at bank 0, so f must take 16 values over 16 rows and
//    separate the 4 rows of a transposing read into the four quarters of the line:
//    f(r) = ((r&3)<<2) | ((r>>2)&3).
//  * 128- and 384-byte rows (8 or 24 chunks): rows alternate between the two halves of the bank line
//    (r*8 mod 16), so only the low three chunk bits may be permuted (the result must stay inside the
//    row) and f must be a bijection onto 0..7 over the 8 even rows of a 16-row window (same for the
//    odd rows), with the two even (odd) rows of every aligned group of four differing in bit 2:
//    f(r) = (bit1(r)<<2) | (bit3(r)<<1) | bit2(r).
//    (Taking the 16-chunk f modulo 8 instead gave two-way conflicts on 33-43 % of the LDS cycles of
//    the d_qk = 192 kernels.)
__device__ __forceinline__ int swz_g(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
__device__ __forceinline__ int swz_h(int row) { return (((row >> 1) & 1) << 2) | (((row >> 3) & 1) << 1) | ((row >> 2) & 1); }
template <int D>
__device__ __forceinline__ int swz(int chunk, int row) {
  static_assert(D / 8 == 16 || D / 8 == 8 || D / 8 == 24, "row of 8, 16 or 24 chunks");
  return chunk ^ (D / 8 == 16 ? swz_g(row) : swz_h(row));
}

// Asynchronous global -> LDS copy of a [ROWS][D] bf16 tile (row stride `stride` elements), with
// the swizzle applied on the global side: each wave instruction fills 1 KiB of contiguous LDS
// (lane i -> bytes 16i..16i+15).  Rows >= rows_valid re-read the last valid row (never out of
// bounds; their products are masked by the caller).  lds_tile must be 1 KiB aligned.
template <int D, int ROWS>
__device__ __forceinline__ void async_tile_load(const uint16_t* g, int64_t stride, int rows_valid,
                                                char* lds_tile, int wave, int lane) {
  constexpr int RB = D * 2;
  constexpr int N_INSTR = ROWS * RB / 1024;
  const int last = rows_valid - 1;
#pragma unroll
  for (int ii = 0; ii < (N_INSTR + 3) / 4; ++ii) {
    const int inst = wave + 4 * ii;
    if (N_INSTR % 4 != 0 && inst >= N_INSTR) break;
    const int pos = inst * 1024 + lane * 16;
    const int row = pos / RB, cpos = (pos % RB) / 16;
    const int c = swz<D>(cpos, row);
    const int grow = row < last ? row : last;
    const uint16_t* src = g + (int64_t)grow * stride + 8 * c;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)(lds_tile + inst * 1024),
                                     16, 0, 0);
  }
}

// One 16-byte-per-lane global -> LDS copy: lane i writes LDS bytes [lds_addr + 16 i, +16).  The
// global address is a wave-uniform 64-bit base plus a 32-bit per-lane byte offset, so no per-lane
// 64-bit address arithmetic is needed.  Completion is tracked by vmcnt like any vector load.
__device__ __forceinline__ void async_copy16(const void* base_uniform, uint32_t lane_byte_off,
                                             uint32_t lds_addr_uniform) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_addr_uniform), "v"(lane_byte_off), "s"(base_uniform)
      : "memory", "m0");
}

// 4-byte-per-lane variant: lane i writes LDS bytes [lds_addr + 4 i, +4).
__device__ __forceinline__ void async_copy4(const void* base_uniform, uint32_t lane_byte_off,
                                            uint32_t lds_addr_uniform) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dword %1, %2"
      :
      : "s"(lds_addr_uniform), "v"(lane_byte_off), "s"(base_uniform)
      : "memory", "m0");
}

__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// Tile copy with the lane-dependent part (LDS row, swizzled chunk) packed once per kernel.  Rows
// >= rows_valid re-read the last valid row (never out of bounds; the caller masks their products).
template <int D, int ROWS>
struct TileLoader {
  static constexpr int RB = D * 2;
  static constexpr int N_INSTR = ROWS * RB / 1024;
  static constexpr int PER_WAVE = (N_INSTR + 3) / 4;
  uint32_t rc[PER_WAVE];  // (row << 16) | byte offset of the source chunk inside its row

  __device__ __forceinline__ void init(int wave, int lane) {
#pragma unroll
    for (int ii = 0; ii < PER_WAVE; ++ii) {
      const int pos = (wave + 4 * ii) * 1024 + lane * 16;
      const int row = pos / RB, cpos = (pos % RB) / 16;
      rc[ii] = ((uint32_t)row << 16) | (uint32_t)(swz<D>(cpos, row) * 16);
    }
  }
  // One of this wave's PER_WAVE copy instructions (so a caller can spread them between other
  // work: a burst of copies stalls the issuing wave behind the 64 B/clk address path).
  // g: first row of the tile (wave-uniform); row * stride_bytes fits 32 bits.
  __device__ __forceinline__ void issue_one(int ii, const uint16_t* g, uint32_t stride_bytes, int rows_valid,
                                            const char* lds_tile, int wave) const {
    const int inst = wave + 4 * ii;
    if (N_INSTR % 4 != 0 && inst >= N_INSTR) return;
    const uint32_t last = (uint32_t)(rows_valid - 1);
    const uint32_t row = rc[ii] >> 16;
    const uint32_t off = __umul24(row < last ? row : last, stride_bytes) + (rc[ii] & 0xffffu);
    async_copy16(g, off, lds_address(lds_tile) + inst * 1024);
  }
  __device__ __forceinline__ void issue(const uint16_t* g, uint32_t stride_bytes, int rows_valid,
                                        const char* lds_tile, int wave) const {
#pragma unroll
    for (int ii = 0; ii < PER_WAVE; ++ii) issue_one(ii, g, stride_bytes, rows_valid, lds_tile, wave);
  }
};

// The same copy with the per-lane source offsets of a FULL tile (all ROWS rows valid) kept ready, so
// that such a copy costs no vector arithmetic at all and can be dropped between MFMAs one at a time.
// A tile with fewer valid rows recomputes its (clamped) offsets from the lane id.
template <int D, int ROWS, int NW = 4>
struct FullTileLoader {
  static constexpr int RB = D * 2;
  static constexpr int N_INSTR = ROWS * RB / 1024;
  static constexpr int PER_WAVE = (N_INSTR + NW - 1) / NW;  // NW waves share the tile's copies
  uint32_t off[PER_WAVE];  // row * stride_bytes + byte offset of the source chunk inside its row

  static __device__ __forceinline__ bool has(int ii, int wave) { return N_INSTR % NW == 0 || wave + NW * ii < N_INSTR; }
  __device__ __forceinline__ void init(int wave, int lane, uint32_t stride_bytes) {
#pragma unroll
    for (int ii = 0; ii < PER_WAVE; ++ii) {
      const int pos = (wave + NW * ii) * 1024 + lane * 16;
      const int row = pos / RB, cpos = (pos % RB) / 16;
      off[ii] = (uint32_t)row * stride_bytes + (uint32_t)(swz<D>(cpos, row) * 16);
    }
  }
  // copy ii of this wave, every row of the tile valid
  __device__ __forceinline__ void issue_full(int ii, const uint16_t* g, const char* lds_tile, int wave) const {
    if (!has(ii, wave)) return;
    async_copy16(g, off[ii], lds_address(lds_tile) + (wave + NW * ii) * 1024);
  }
  // copy ii of this wave, rows >= rows_valid re-read the last valid row
  __device__ __forceinline__ void issue_clamped(int ii, const uint16_t* g, uint32_t stride_bytes, int rows_valid,
                                                const char* lds_tile, int wave, int lane) const {
    if (!has(ii, wave)) return;
    asm volatile("" : "+v"(lane));  // recomputed here each time: not worth registers held across the main loops
    const int pos = (wave + NW * ii) * 1024 + lane * 16;
    const int row = pos / RB, cpos = (pos % RB) / 16;
    const int last = rows_valid - 1;
    const uint32_t o = (uint32_t)(row < last ? row : last) * stride_bytes + (uint32_t)(swz<D>(cpos, row) * 16);
    async_copy16(g, o, lds_address(lds_tile) + (wave + NW * ii) * 1024);
  }
  __device__ __forceinline__ void issue_one(int ii, const uint16_t* g, uint32_t stride_bytes, int rows_valid,
                                            const char* lds_tile, int wave, int lane) const {
    if (rows_valid >= ROWS) issue_full(ii, g, lds_tile, wave);
    else issue_clamped(ii, g, stride_bytes, rows_valid, lds_tile, wave, lane);
  }
  __device__ __forceinline__ void issue(const uint16_t* g, uint32_t stride_bytes, int rows_valid,
                                        const char* lds_tile, int wave, int lane) const {
    if (rows_valid >= ROWS) {
#pragma unroll
      for (int ii = 0; ii < PER_WAVE; ++ii) issue_full(ii, g, lds_tile, wave);
    } else {
#pragma unroll
      for (int ii = 0; ii < PER_WAVE; ++ii) issue_clamped(ii, g, stride_bytes, rows_valid, lds_tile, wave, lane);
    }
  }
};

// all of this wave's outstanding global loads (including global -> LDS copies) have completed
__device__ __forceinline__ void wait_async_loads() {
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), expcnt and lgkmcnt left at their maxima
}

// ds_read_b64_tr_b16: within each group of 16 lanes, lane i receives element i%4 of the 8-byte
// words addressed by lanes i/4, i/4+4, i/4+8, i/4+12 of the group.
__device__ __forceinline__ s16x4 lds_read_tr16(const char* addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)addr);
}

// the same read from an absolute LDS address held as an integer
__device__ __forceinline__ s16x4 lds_read_tr16_at(uint32_t lds_addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)lds_addr);
}

// A chain of L MFMAs whose A operands come from LDS, with the reads running PD fragments ahead of
// their use.  load(i) returns fragment i, mma(i, frag) consumes it.  prefill()/run() are split so a
// caller can start the first reads before unrelated arithmetic and drain the chain after it.
template <int L, int PD>
struct LdsChain {
  Frag ring[PD];
  template <class Load>
  __device__ __forceinline__ void prefill(Load load) {
#pragma unroll
    for (int i = 0; i < PD && i < L; ++i) ring[i] = load(i);
    __builtin_amdgcn_sched_barrier(0);
  }
  template <class Load, class Mma>
  __device__ __forceinline__ void run(Load load, Mma mma) {
#pragma unroll
    for (int i = 0; i < L; ++i) {
      mma(i, ring[i % PD]);
      if (i + PD < L) ring[i % PD] = load(i + PD);
      __builtin_amdgcn_sched_barrier(0);  // keep the read-ahead distance: no hoisting or sinking
    }
  }
  // Same, with NS slices of independent vector arithmetic spread evenly behind the MFMAs: they
  // execute in the MFMAs' shadow (the matrix pipe runs asynchronously to the issuing wave).
  template <int NS, class Load, class Mma, class Slice>
  __device__ __forceinline__ void run_with(Load load, Mma mma, Slice slice) {
#pragma unroll
    for (int i = 0; i < L; ++i) {
      mma(i, ring[i % PD]);
      if (i + PD < L) ring[i % PD] = load(i + PD);
#pragma unroll
      for (int sl = i * NS / L; sl < (i + 1) * NS / L; ++sl) slice(sl);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
};

// Position of contraction index w (0..15) inside a 16-element chunk of a transposed LDS tile.
// An MFMA whose B operand is taken straight from an accumulator sees, in lane half hh, the
// eight rows {4hh+v, 8+4hh+v : v=0..3}; storing row w at slot 8*((w%8)/4) + 4*(w/8) + w%4
// makes those eight rows one contiguous 16-byte read at offset 8*hh.
__device__ __forceinline__ int tslot(int w) { return (((w & 7) >> 2) << 3) + ((w >> 3) << 2) + (w & 3); }

__device__ __forceinline__ uint32_t hw_id_reg() {
  // s_getreg_b32 HW_REG_HW_ID (id 4), offset 0, size 32
  return __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 4);
}
__device__ __forceinline__ uint32_t xcc_id_reg() {
  // s_getreg_b32 HW_REG_XCC_ID (id 20), offset 0, size 32
  return __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 20);
}

// ---- work queues, one per accelerator die (XCD) ------------------------------------------------
// Each die has its own L2, so work is dealt by kv head: queue x holds the items of the kv heads kvh
// with kvh % 8 == x.  All workgroups of a die then stream the same K/V (or the same Q/dO) and share
// it through that die's L2.  When a die has several kv heads they are taken kHeadGroup at a time:
// within a group the order is the worklist's (longest first), tile by tile with the group's heads
// innermost, so that at any time the die's 32 workgroups sit on about 32 / kHeadGroup neighbouring
// tiles of each of these heads and share that head's stream (with all of a die's heads innermost,
// 16 of them for 128 kv heads, only two workgroups would).  A workgroup serves its own die's queue
// first and then steals from the others, so every item is done whatever the head count and the tail
// stays balanced.  Counters are 128 bytes apart.
constexpr int kNumXcd = 8;
constexpr int kCounterStride = 32;  // in int32
constexpr int kHeadGroup = 2;  // measured on 128 kv heads: 1 and 2 alike, 4 is 2 % slower, all 16 at once 12 %

struct Taken {
  int tile_idx;  // < 0: every queue is exhausted
  int head;      // kvh * per_kv + sub
  int q_cur, q_tried;
};

// One thread takes the next item.  q_cur / q_tried: that thread's cursor over the queues.  A real
// call, everything passed and returned by value in registers: inlined into the persistent kernels
// its temporaries cost them registers they do not have (two of them would spill).
// steal_stride (odd): how the cursor moves on from an exhausted queue; different workgroups of a die use
// different strides, so they do not all descend on the same other queue.
__device__ __attribute__((noinline)) Taken take_item(int32_t* counters, int n_tiles, int Hkv, int per_kv, int q_cur,
                                                      int q_tried, int steal_stride) {
  while (q_tried < kNumXcd) {
    const int nk = Hkv > q_cur ? (Hkv - q_cur + kNumXcd - 1) / kNumXcd : 0;  // kv heads of this die
    const int len = n_tiles * nk * per_kv;
    if (len > 0) {
      const int j = atomicAdd(counters + q_cur * kCounterStride, 1);
      if (j < len) {
        const int per_group = n_tiles * kHeadGroup * per_kv;  // items of a full group of heads
        const int full = nk / kHeadGroup;
        int grp = j / per_group, jj = j - grp * per_group, size = kHeadGroup;
        if (grp >= full) {  // the last, smaller group
          grp = full;
          jj = j - full * per_group;
          size = nk - full * kHeadGroup;
        }
        const int per_tile = size * per_kv;
        const int rem = jj % per_tile;
        return Taken{jj / per_tile, (q_cur + kNumXcd * (grp * kHeadGroup + rem / per_kv)) * per_kv + rem % per_kv,
                     q_cur, q_tried};
      }
    }
    q_cur = (q_cur + steal_stride) & (kNumXcd - 1);
    ++q_tried;
  }
  return Taken{-1, 0, q_cur, q_tried};
}

struct WorkQueues {
  int32_t* counters;
  int n_tiles, Hkv, per_kv;  // per_kv: heads per kv head inside one item group (g, or 1)
};

// Workgroup barrier that orders LDS traffic only: waits for this wave's LDS operations, not for its
// outstanding global stores (the results a previous item is still writing out).
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Race-hunting build (-DHBP_RACE_HUNT, a second library next to the release one): a full fence of the
// workgroup - this wave's tile copies and LDS operations complete, then a barrier - at the end of every
// phase of the forward and of every tile or step of the backward kernels.  The release build gets by with
// one barrier per tile and relies on which buffer each phase still reads; if that reasoning were wrong
// somewhere, the two builds would differ.  The arithmetic and its order are the same, so they must agree
// bit for bit.  Every call site is reached by all wavefronts of the workgroup equally often.
__device__ __forceinline__ void race_fence() {
#ifdef HBP_RACE_HUNT
  wait_async_loads();
  __syncthreads();
#endif
}

// Workgroup-wide fetch of the next item: thread 0 takes it, everybody reads it back as scalars.
// slot: two ints of LDS that nobody else touches between the surrounding barriers.
__device__ __forceinline__ bool next_item(const WorkQueues& wq, int* slot, int tid, int& q_cur, int& q_tried,
                                          int& tile_idx, int& head) {
  // the slot is addressed as LDS (not through a generic pointer: that becomes flat accesses, each
  // followed by a wait for every outstanding global store of the previous item)
  volatile __attribute__((address_space(3))) int* const box =
      (volatile __attribute__((address_space(3))) int*)(uintptr_t)lds_address(slot);
  lds_barrier();  // all LDS reads of the previous item are finished
  if (tid == 0) {
    const Taken tk = take_item(wq.counters, wq.n_tiles, wq.Hkv, wq.per_kv, q_cur, q_tried,
                               2 * ((blockIdx.x >> 3) & 3) + 1);
    q_cur = tk.q_cur;
    q_tried = tk.q_tried;
    box[0] = tk.tile_idx;
    box[1] = tk.head;
  }
  lds_barrier();
  tile_idx = __builtin_amdgcn_readfirstlane(box[0]);
  head = __builtin_amdgcn_readfirstlane(box[1]);
  lds_barrier();
  return tile_idx >= 0;
}

struct FwdParams {
  const uint16_t *q, *k, *v;
  uint16_t* o;
  float* lse;
  const int32_t* cu;
  const hbp_tile* tiles;
  int32_t n_tiles, n_samples, T, Hq, Hkv, g;
  int64_t q_st, q_sh, k_st, k_sh, v_st, v_sh, o_st, o_sh;
  float scale_log2;  // softmax scale * log2(e)
  int32_t* counter;
  hbp_profile_rec* prof;
  int32_t n_split;   // the query heads of a kv head are dealt to the dies in this many parts (see heads_split)
};

struct BwdParams {
  const uint16_t *q, *k, *v, *o, *d_o;
  const float* lse;
  uint16_t *dq, *dk, *dv;
  float* D;     // [Hq,T] rowsum(dO * O)
  float* lse2;  // [Hq,T] LSE * log2(e)
  const int32_t* cu;
  const hbp_tile* tiles;    // key tiles (dK/dV kernel)
  const hbp_tile* q_tiles;  // query tiles (dQ kernel)
  int32_t n_tiles, n_q_tiles, n_samples, T, Hq, Hkv, g;
  int64_t q_st, q_sh, k_st, k_sh, v_st, v_sh, o_st, o_sh;
  float scale, scale_log2;
  int32_t *counter, *counter_dq;
  hbp_profile_rec *prof, *prof_dq;
  // With fewer kv heads than dies the g query heads of a kv head are cut into n_split parts, each a
  // work item of its own (so that every die has a queue and no item loops over too many heads).  In
  // the dK/dV kernel the parts of a kv head then produce partial sums: fp32, [n_split][T][Hkv][dim],
  // added up in part order by a reduce kernel.
  int32_t n_split, n_split_dq;
  float *dk_part, *dv_part;
};

// In how many parts the `units` schedulable units of a kv head (query heads, or pairs of them) are
// dealt out: the smallest divisor of units that gives every die a queue, else units itself.
inline int heads_split(int n_kv_heads, int units) {
  for (int s = 1; s <= units; ++s)
    if (units % s == 0 && n_kv_heads * s >= 8) return s;
  return units;
}

struct CeParams {  // packed cross-entropy
  const uint16_t* logits;
  int64_t stride_t;  // elements
  int32_t T, V, n_samples, normalizer;
  const int32_t* labels;
  const int32_t* cu;
  float t_ave;
  uint16_t* dlogits;   // may be null
  float* token_loss;   // [T]
  float* weighted;     // [T] workspace: w_r CE_r
  int32_t* counts;     // [n_samples] workspace: loss tokens per sample
  float* weights;      // [n_samples] workspace
  int32_t* row_start;  // [kCeMaxWorkgroups + 1] workspace: first row of every workgroup of the main kernel
  float* loss_out;
};
constexpr int kCeMaxWorkgroups = 2048;

// launchers implemented in the .hip files; return hipError_t as int
// ev0/ev1: optional events recorded around the persistent main kernel
// n_cu: compute units to fill (the kernel picks its own workgroup shape and grid)
int launch_fwd(int d_qk, int d_v, const FwdParams& p, int tile_rows, int n_cu, hipStream_t s, hipEvent_t ev0,
               hipEvent_t ev1);
// ev: {dkdv start, dkdv stop, dq start, dq stop}, entries may be null
int launch_bwd(int d_qk, int d_v, const BwdParams& p, int grid_dq, int grid_dkdv, hipStream_t s, hipEvent_t* ev);
size_t bwd_partial_floats(int T, int Hkv, int g, int dim);  // per tensor; 0 when the dK/dV kernel needs no partial sums
int launch_zero_counters(int32_t* counters, hipStream_t s);  // the kNumXcd forward counters
int launch_packed_ce(const CeParams& p, int n_cu, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);

}  // namespace hbp
