// Forward kernel: causal attention inside each sample of a packed buffer, gfx950.
//
// One work item = (query tile, one or two query heads of a kv head).  A persistent grid takes items
// from per-die queues in worklist order (longest causal cost first).  Per item the workgroup (eight
// wavefronts of 32 query rows each: two heads x 128 rows, or one head x 256 rows; four for one head x
// 128 rows) walks the sample's keys from the sample start to the diagonal.
//
//   S^T = K Q^T      K tile from LDS (A operand), Q fragments held in registers (B operand);
//                    the accumulator then has one query per lane column, its keys in-lane, so
//                    the row max/sum needs a single exchange with lane^32.
//   P^T -> bf16      used directly as the B operand of the next product (no shuffle);
//   O^T += V^T P^T   V tile kept in its natural [key][dim] layout in LDS and read with the
//                    transposing LDS load, in the key order the accumulator rows have.
//
// K and V tiles (64 keys) go global -> LDS directly (no staging registers), double buffered, with
// an XOR swizzle of the 16-byte chunks applied on the global side.  exp is taken in base 2 with
// scale*log2(e) folded into one multiplier.
//
// Software pipeline inside each wave.  Keys are processed in blocks of 32; block b goes through
//   A(b): S^T block (MFMA)   M(b): online softmax of the block (vector ALU)   B(b): O^T += V^T P^T (MFMA)
// and the wave executes "phases": phase b issues the MFMAs of A(b+1) and B(b-1), alternating, with
// the vector instructions of M(b) spread a few at a time behind them.  A vector instruction
// overlaps only MFMAs of its own wave, and only about four fit behind each MFMA, so this spreading
// is what keeps the matrix pipe busy.  One workgroup barrier per 64-key tile: K(t) and V(t-1) are
// last read in phase 2t, so at the barrier before phase 2t+1 the copies of K(t+2) and V(t+1) are
// issued into the buffers they leave.
#include <type_traits>

#include "common.hpp"

namespace hbp {

template <int DQK, int DV>
struct FwdWave {
  static constexpr int BN = 64;
  static constexpr int KRB = DQK * 2, VRB = DV * 2;  // bytes per LDS row
  static constexpr int K_TILE = BN * KRB, V_TILE = BN * VRB;
  static constexpr int NC = DQK / 16;   // MFMAs of A: contraction chunks of QK^T
  static constexpr int NEB = DV / 32;   // 32-wide blocks of the head dim of V
  static constexpr int NB = 2 * NEB;    // MFMAs of B
  static constexpr int TOTAL = NC + NB; // MFMAs per phase; a multiple of PD
  static constexpr int PD = 4;          // LDS read-ahead depth of the operand ring
  static constexpr int NSL = 17;        // exp slices: 1..16 = elements, 17 = drain
  static constexpr int EA = NSL * 2 * NC / (2 * NC + NB);  // exp slices placed behind the A MFMAs
  static constexpr int NMP = 4;         // pieces of the diagonal block's mask

  // LDS layout: [K buf0][K buf1][V buf0][V buf1].  The offsets below are absolute LDS addresses
  // (workgroup base and current buffer included), so a read needs no address arithmetic.
  uint32_t koff[NC];     // this lane's K fragments
  uint32_t voff[2][NEB]; // this lane's V^T fragments
  Frag qf[NC];
  Frag ring[PD];         // operand read-ahead; runs on across phase boundaries
  f32x16 oacc[NEB];
  f32x16 s[2];           // s[b & 1] = scores of block b
  Frag pf[2][2];         // pf[b & 1][j] = probabilities of block b, key chunk j
  float scale_log2;
  int q_in, hh;
  // Online softmax state.  m_run: reference the probabilities are taken against (times log2 e): the
  // maximum of the row's first block, moved up when a later block rises well above it (see
  // range_check); l_run: this lane's part of the row sum.
  float m_run, l_run, pmax;
  float p_cur, p_even, psum;

  // `add`: a compile-time byte offset on top of the lane's offsets (the hot loop names the other tile
  // buffer this way, as part of the read's immediate, instead of moving the offsets every tile)
  __device__ __forceinline__ Frag k_frag(int blk_in_tile, int c, int add = 0) const {
    Frag f;
    f.u = *(const __attribute__((address_space(3))) u32x4*)(uintptr_t)(koff[c] + (32 * blk_in_tile * KRB + add));
    return f;
  }
  __device__ __forceinline__ Frag v_frag(int blk_in_tile, int i, int add = 0) const {  // i = (j, eb), eb fastest
    const int eb = i % NEB, j = i / NEB;
    const uint32_t base = (32 * blk_in_tile + 16 * j) * VRB + add;
    Frag f;
    f.h[0] = lds_read_tr16_at(voff[0][eb] + base);
    f.h[1] = lds_read_tr16_at(voff[1][eb] + base);
    return f;
  }
  // first PD operands of a phase that reads K block `blk_in_tile`
  __device__ __forceinline__ void preload_k(int blk_in_tile, int add = 0) {
#pragma unroll
    for (int i = 0; i < PD; ++i) ring[i] = k_frag(blk_in_tile, i, add);
  }

  // Values produced by the slices are consumed a phase later, behind a branch; without an anchor
  // the compiler sinks their whole computation out of the MFMA shadow to just before that use.
  template <class T>
  static __device__ __forceinline__ void pin(T& x) {
    asm volatile("" : "+v"(x));
  }

  // A(0) alone (pipeline prologue): s[0] = K_0 Q^T
  __device__ __forceinline__ void first_scores() {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[0][i] = 0.f;
    LdsChain<NC, PD> c;
    auto load = [&](int i) { return k_frag(0, i); };
    c.prefill(load);
    c.run(load, [&](int i, const Frag& f) { s[0] = mfma32(f.v, qf[i].v, s[0]); });
  }

  // The reference of a row.  Probabilities are exp2(s c - m_run) against a reference that O and l share,
  // so the result does not depend on it; it starts as the maximum of the row's first block of 32 keys.
  // No later block computes its row maximum up front.  Instead the block's probabilities are taken against
  // the reference as it stands, and their sum tells whether that was good enough: a lane's sum of 16
  // probabilities above 2^8 means that some score lies well above the reference, and only then
  // (range_check, a wave-uniform branch that ordinary data takes for a few early blocks of an item) the
  // true maximum of the block is computed, the reference moves there, O and l are rescaled and the block's
  // probabilities are taken again.  A row's largest score so far thus never lies more than 8 (in log2)
  // above its reference, as with a maximum computed for every block, and a dominant key still gets the
  // probability 1 exactly; but the hot loop carries no row maximum at all: per element one fma, one exp2,
  // one add and half a conversion.
  //
  // Block 0 (scores in s[0]): mask (d: causal threshold of this lane, element i is masked iff
  // 8 (i>>2) + (i&3) > d), maximum, reference.
  __device__ __forceinline__ void first_reference(int d) {
    pmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (8 * (i >> 2) + (i & 3) > d) s[0][i] = -INFINITY;
      pmax = fmaxf(pmax, s[0][i]);
    }
    m_run = max_with_other_half(pmax) * scale_log2;  // scale > 0; finite: key 0 of the sample is visible to every row
    l_run = 0.f;
  }
  // causal mask of a later block (scores in s[par]), four elements per piece
  __device__ __forceinline__ void mask_piece(int par, int d, int piece) {
#pragma unroll
    for (int i = 4 * piece; i < 4 * piece + 4; ++i)
      if (8 * (i >> 2) + (i & 3) > d) s[par][i] = -INFINITY;
  }
  // After the exp slices of a block (scores still in s[par], probabilities in pf[par], this lane's sum in
  // psum): if any lane's sum says that the block rose above the reference (or is not a number at all),
  // move the references to the rows' true maxima, rescale O and l, and take the block's probabilities
  // again.  Then the sum joins l.
  __device__ __forceinline__ void range_check(int par) {
    if (__builtin_amdgcn_ballot_w64(!(psum < 0x1p8f)) != 0) {
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[par][i]);
      const float m_new = fmaxf(m_run, max_with_other_half(mx) * scale_log2);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[eb][i] *= alpha;
      psum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[par][e], scale_log2, -m_run));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[par][e + 1], scale_log2, -m_run));
        psum += p0;
        psum += p1;
        pf[par][e >> 3].w[(e & 7) >> 1] = pack_bf16(p0, p1);
      }
    }
    l_run += psum;
  }
  // causal threshold for the block that starts at in-sample key k_blk; a lane-constant.  Kept
  // opaque so the compares stay "constant vs one register" instead of sixteen precomputed
  // per-lane thresholds.
  __device__ __forceinline__ int mask_threshold(int k_blk, bool masked) const {
    int d = masked ? q_in - (k_blk + 4 * hh) : 0x7fffffff;
    asm volatile("" : "+v"(d));
    return d;
  }
  // a new block becomes the current one
  __device__ __forceinline__ void adopt() { psum = 0.f; }
  // exp of the current block (scores in s[par]).  Elements go through two stages one slice apart
  // (exp of element e next to the sum/pack of element e-1) so no instruction waits on the one
  // before it.  sl = 1..NSL.
  __device__ __forceinline__ void exp_slice(int par, int sl) {
    const float p_prev = p_cur;
    if (sl <= 16) {
      p_cur = __builtin_amdgcn_exp2f(__builtin_fmaf(s[par][sl - 1], scale_log2, -m_run));
      pin(p_cur);
    }
    if (sl >= 2) {
      const int e = sl - 2;  // element whose exp was issued one slice ago
      psum += p_prev;        // unrounded: LSE must not inherit the bf16 rounding of P
      pin(psum);
      if (e & 1) {
        pf[par][e >> 3].w[(e & 7) >> 1] = pack_bf16(p_even, p_prev);
        pin(pf[par][e >> 3].w[(e & 7) >> 1]);
      } else {
        p_even = p_prev;
      }
    }
  }

  // What phase b of a wave consists of.  The wave's blocks are 0..nb-1; block nb-1 is the diagonal
  // one, the only one that needs the causal compare.
  struct Parts {
    bool a;     // A(b+1) and, on the diagonal, the mask of block b+1:  b+1 < nb
    bool e;     // exp of block b:                             b < nb
    bool b;     // B(b-1):                                     1 <= b <= nb
    bool mask;  // block b+1 is the diagonal block
  };
  static __device__ __forceinline__ Parts parts_of(int b, int nb) {
    return Parts{b + 1 < nb, b < nb, b >= 1 && b <= nb, b + 2 == nb};
  }

  // Phase b (PAR = b & 1).  MFMAs: A(b+1) then B(b-1), both on block 1-PAR of their tiles.  Behind
  // them: the exp slices of block b and, where block b+1 is the diagonal one, behind the B MFMAs (when
  // its scores are complete) the pieces of its mask; at the end the check whether block b rose above
  // the rows' references (range_check).  HOT: every part present and no mask, known
  // at compile time; otherwise `pt` says (wave-uniform) which parts run.  With part a the ring must
  // hold the first PD K fragments on entry; an odd phase leaves the ring holding those of the
  // following even phase (same K tile, no barrier in between).  k_next: in-sample index of the
  // first key of block b+1.  KADD, VADD: byte offsets of the K and V tile buffers this phase reads,
  // relative to where the lane's offsets point.
  template <int PAR, bool HOT, int KADD = 0, int VADD = 0, class Copy>
  __device__ __forceinline__ void phase(int k_next, Parts pt, Copy copy) {
    constexpr int NXT = 1 - PAR;
    const bool do_a = HOT || pt.a, do_e = HOT || pt.e, do_b = HOT || pt.b;
    int d = 0;
    if (!HOT) d = mask_threshold(k_next, pt.mask);
    if (do_e) adopt();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < TOTAL; ++j) {
      if (j < NC) {
        if (do_a) {
          if (j == 0) {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            s[NXT] = mfma32(ring[0].v, qf[0].v, zero);
          } else {
            s[NXT] = mfma32(ring[j % PD].v, qf[j].v, s[NXT]);
          }
        }
      } else if (do_b) {
        const int i = j - NC;
        oacc[i % NEB] = mfma32(ring[j % PD].v, pf[NXT][i / NEB].v, oacc[i % NEB]);
      }
      const int jn = j + PD;  // operand to fetch now
      if (jn < NC) {
        if (do_a) ring[jn % PD] = k_frag(NXT, jn, KADD);
      } else if (jn < TOTAL) {
        if (do_b) ring[jn % PD] = v_frag(NXT, jn - NC, VADD);
      } else if (PAR == 1) {
        ring[jn % PD] = k_frag(PAR, jn - TOTAL, KADD);
      }
      if (do_e) {
        const int lo = j < NC ? j * EA / NC : EA + (j - NC) * (NSL - EA) / NB;
        const int hi = j < NC ? (j + 1) * EA / NC : EA + (j - NC + 1) * (NSL - EA) / NB;
#pragma unroll
        for (int sl = lo; sl < hi; ++sl) exp_slice(PAR, sl + 1);
      }
      if (!HOT && do_a && pt.mask && j >= NC) {  // the scores of block b+1 are complete: mask the diagonal block
#pragma unroll
        for (int piece = 0; piece < NMP; ++piece) {
          const int slot = 2 + piece * (NB - 2) / NMP;
          if ((slot < NB ? slot : NB - 1) == j - NC) mask_piece(NXT, d, piece);
        }
      }
      copy(j);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (do_e) range_check(PAR);
  }
  template <int PAR>
  __device__ __forceinline__ void any_phase(int b, int nb) {
    const Parts pt = parts_of(b, nb);
    if (pt.a || pt.e || pt.b) phase<PAR, false>(32 * (b + 1), pt, [](int) {});
  }
};

// HP: query heads per workgroup, TP: 128-row query tiles per workgroup (HP * TP <= 2).  With
// HP = 2 the workgroup has eight wavefronts, four per head, and both heads (same kv head) work off
// the same K/V tiles in LDS, which halves the L2 -> LDS copy traffic per MFMA; it needs an even
// group size.  With TP = 2 the eight wavefronts take 32 rows each of a tile of up to 256 rows of one
// head and share the K/V stream in the same way (every wavefront stops at its own diagonal): the
// form for odd group sizes, multi-head attention included.  Either way a compute unit holds eight
// wavefronts.
template <int DQK, int DV, int HP, int TP>
__global__ __launch_bounds__(kThreads * HP * TP, 2 / (HP * TP)) void fwd_kernel(const FwdParams p) {
  static_assert(HP * TP <= 2, "eight wavefronts per compute unit");
  constexpr int NW = 4 * HP * TP;
  using W = FwdWave<DQK, DV>;
  constexpr int BM = 128 * TP, BN = W::BN;
  constexpr int KRB = W::KRB, VRB = W::VRB, K_TILE = W::K_TILE, V_TILE = W::V_TILE;
  constexpr int NC = W::NC, NEB = W::NEB;

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  char* const k_lds = smem;
  char* const v_lds = smem + 2 * K_TILE;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rw = wave % (4 * TP);  // which 32 rows of the query tile
  const int lane = tid & 63, l32 = lane & 31, hh = lane >> 5;

  W w;
  const uint32_t lds0 = lds_address(smem);
  w.hh = hh;
  w.scale_log2 = p.scale_log2;
  // per-lane LDS byte offsets of the A operands (row part that does not depend on the 32-key block)
#pragma unroll
  for (int c = 0; c < NC; ++c) w.koff[c] = lds0 + l32 * KRB + swz<DQK>(2 * c + hh, l32) * 16;
  {
    const int G = lane >> 4, s = lane & 15;
    const int k8 = 4 * hh + (s >> 2);
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int eb = 0; eb < NEB; ++eb) {
        const int c = 4 * eb + 2 * (G & 1) + ((s & 3) >> 1);
        w.voff[r][eb] = lds0 + 2 * K_TILE + (8 * r + k8) * VRB + swz<DV>(c, 8 * r + k8) * 16 + (s & 1) * 8;
      }
  }
  const uint32_t k_stride_b = (uint32_t)p.k_st * 2, v_stride_b = (uint32_t)p.v_st * 2;
  FullTileLoader<DQK, BN, NW> k_loader;
  FullTileLoader<DV, BN, NW> v_loader;
  k_loader.init(wave, lane, k_stride_b);
  v_loader.init(wave, lane, v_stride_b);

  uint32_t n_done = 0;
  uint64_t t_first = 0, t_last = 0, t_busy = 0;

  const WorkQueues wq{p.counter, p.n_tiles, p.Hkv * p.n_split, p.g / HP / p.n_split};
  int q_cur = xcc_id_reg() & (kNumXcd - 1), q_tried = 0;
  for (;;) {
    int tile_idx, h;
    if (!next_item(wq, (int*)smem, tid, q_cur, q_tried, tile_idx, h)) break;
    h = h * HP + wave / (4 * TP);  // this wave's head
    uint64_t t0 = 0;
    if (p.prof && tid == 0) {
      t0 = wall_clock64();
      if (n_done == 0) t_first = t0;
    }

    const hbp_tile tl = p.tiles[tile_idx];
    bool ok = tl.sample >= 0 && tl.sample < p.n_samples;
    int s0 = 0, s1 = 0;
    if (ok) {
      s0 = p.cu[tl.sample];
      s1 = p.cu[tl.sample + 1];
      // tiles start a multiple of 32 rows into their sample: each wave then has exactly one key
      // block that crosses its diagonal
      ok = s0 >= 0 && s1 <= p.T && s0 <= tl.row_begin && tl.row_begin < tl.row_end &&
           tl.row_end <= s1 && tl.row_end - tl.row_begin <= BM && (tl.row_begin - s0) % 32 == 0;
    }
    if (ok) {
      const int r0 = tl.row_begin, r1 = tl.row_end;
      const int kh = h / p.g;
      const int qw0 = r0 - s0 + 32 * rw;  // in-sample index of this wave's first query
      const int my_row = r0 + 32 * rw + l32;
      const bool row_valid = my_row < r1;
      const bool wave_active = r0 + 32 * rw < r1;
      const int nb = wave_active ? qw0 / 32 + 1 : 0;  // this wave's key blocks are 0..nb-1

      const int n_keys = r1 - s0;  // keys 0..n_keys-1 (in-sample) are needed by this tile
      const int nkt = (n_keys + BN - 1) / BN;  // nb <= 2 nkt
      const uint16_t* kbase = p.k + (int64_t)s0 * p.k_st + (int64_t)kh * p.k_sh;
      const uint16_t* vbase = p.v + (int64_t)s0 * p.v_st + (int64_t)kh * p.v_sh;
      auto issue_k = [&](int t) {
        if (t < nkt)
          k_loader.issue(kbase + (int64_t)t * BN * p.k_st, k_stride_b, n_keys - t * BN, k_lds + (t & 1) * K_TILE, wave, lane);
      };
      auto issue_v = [&](int t) {
        if (t < nkt)
          v_loader.issue(vbase + (int64_t)t * BN * p.v_st, v_stride_b, n_keys - t * BN, v_lds + (t & 1) * V_TILE, wave, lane);
      };
      issue_k(0);
      issue_v(0);
      issue_k(1);

      // Q fragments (B operand of S^T = K Q^T): lane holds query l32, dims 16c+8hh..+7
      {
        const uint16_t* qp = p.q + (int64_t)my_row * p.q_st + (int64_t)h * p.q_sh + 8 * hh;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          if (row_valid) w.qf[c].u = *(const u32x4*)(qp + 16 * c);
          else w.qf[c].u = u32x4{0, 0, 0, 0};
        }
      }
#pragma unroll
      for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
        for (int i = 0; i < 16; ++i) w.oacc[eb][i] = 0.f;
      w.m_run = 0.f;
      w.l_run = 0.f;
      w.q_in = qw0 + l32;
      w.p_cur = w.p_even = w.psum = 0.f;

      int k_buf = 0, v_buf = 0;  // buffers the LDS offsets currently point at
      auto point_k = [&](int buf) {
        if (buf != k_buf) {
          const int d = buf ? K_TILE : -K_TILE;
#pragma unroll
          for (int c = 0; c < NC; ++c) w.koff[c] += d;
          k_buf = buf;
        }
      };
      auto point_v = [&](int buf) {
        if (buf != v_buf) {
          const int d = buf ? V_TILE : -V_TILE;
#pragma unroll
          for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int eb = 0; eb < NEB; ++eb) w.voff[r][eb] += d;
          v_buf = buf;
        }
      };
      auto tile_sync = [&](int t) {  // between phases 2t and 2t+1
        wait_async_loads();
        __syncthreads();  // K(t+1) and V(t) have landed; K(t) and V(t-1) are no longer read
        point_k((t + 1) & 1);
        point_v(t & 1);
      };
      auto tile_barrier = [&](int t) {  // the same, with the next copies issued in one go
        tile_sync(t);
        issue_k(t + 2);
        issue_v(t + 1);
      };

      wait_async_loads();
      __syncthreads();  // K(0), V(0), K(1) have landed
      if (nb > 0) {
        w.first_scores();
        w.preload_k(1);
        w.first_reference(w.mask_threshold(0, nb == 1));
      }

      // Tiles whose two phases both run every part unmasked (phases 1 .. nb-3) get a loop of
      // their own with one code variant; every wave passes nkt barriers in total.
      const int t_hot_end = nb >= 6 ? (nb - 4) / 2 + 1 : 1;  // hot tiles are 1 .. t_hot_end-1
      int t = 0;
      if (nkt > 0) {
        w.template any_phase<0>(0, nb);
        race_fence();
        tile_barrier(0);
        w.preload_k(0);
        w.template any_phase<1>(1, nb);
        race_fence();
        t = 1;
      }
      // One hot tile t: phase 2t reads K tile t and V tile t-1, phase 2t+1 reads K tile t+1 and V tile t.
      // TPAR = t & 1 as a compile-time constant: the lane's offsets stay on buffer 0 and the other buffer
      // is part of each read's immediate offset; TPAR < 0: the offsets follow the buffers (16 vector adds
      // per tile, but one copy of the code).
      auto hot_tile = [&](auto tpar, int t) {
        constexpr int TPAR = decltype(tpar)::value;
        constexpr bool IMM = TPAR >= 0;
        w.template phase<0, true, IMM ? TPAR * K_TILE : 0, IMM ? (1 - TPAR) * V_TILE : 0>(
            64 * t + 32, typename W::Parts{}, [](int) {});
        race_fence();
        if constexpr (IMM) {
          wait_async_loads();
          __syncthreads();  // K(t+1) and V(t) have landed; K(t) and V(t-1) are no longer read
        } else {
          tile_sync(t);
        }
        w.preload_k(0, IMM ? (1 - TPAR) * K_TILE : 0);
        // the copies of K(t+2) and V(t+1) go out one at a time behind this phase's MFMAs (a burst
        // of them would hold the wave for as long as the address path takes to drain)
        const uint16_t* kg = kbase + (int64_t)(t + 2) * BN * p.k_st;
        const uint16_t* vg = vbase + (int64_t)(t + 1) * BN * p.v_st;
        const int k_valid = n_keys - (t + 2) * BN, v_valid = n_keys - (t + 1) * BN;
        const char* k_dst = k_lds + (IMM ? TPAR : t & 1) * K_TILE;
        const char* v_dst = v_lds + (IMM ? 1 - TPAR : (t + 1) & 1) * V_TILE;
        constexpr int NKC = decltype(k_loader)::PER_WAVE, NVC = decltype(v_loader)::PER_WAVE;
        constexpr int GAP = W::TOTAL / (NKC + NVC) > 0 ? W::TOTAL / (NKC + NVC) : 1;
        w.template phase<1, true, IMM ? (1 - TPAR) * K_TILE : 0, IMM ? TPAR * V_TILE : 0>(
            64 * t + 64, typename W::Parts{}, [&](int j) {
#pragma unroll
              for (int c = 0; c < NKC + NVC; ++c) {
                const int slot = c * GAP < W::TOTAL ? c * GAP : W::TOTAL - 1;
                if (slot != j) continue;
                if (c < NKC) {
                  if (k_valid > 0) k_loader.issue_one(c, kg, k_stride_b, k_valid, k_dst, wave, lane);
                } else {
                  v_loader.issue_one(c - NKC, vg, v_stride_b, v_valid, v_dst, wave, lane);
                }
              }
            });
        race_fence();
      };
      // Two copies of the hot tile need a few registers more; at head size 192 they are not there.
      if constexpr (DQK <= 128) {
        if (t + 1 < t_hot_end) {
          point_k(0);
          point_v(0);
        }
        for (; t + 1 < t_hot_end; t += 2) {  // t is odd here: the hot tiles start at tile 1
          hot_tile(std::integral_constant<int, 1>{}, t);
          hot_tile(std::integral_constant<int, 0>{}, t + 1);
        }
        if (t > 0) {  // back to offsets that follow the buffers: K tile t, V tile t-1 are read next
          point_k(t & 1);
          point_v((t - 1) & 1);
        }
      }
      for (; t < t_hot_end; ++t) hot_tile(std::integral_constant<int, -1>{}, t);
      for (; t < nkt; ++t) {
        w.template any_phase<0>(2 * t, nb);
        race_fence();
        tile_barrier(t);
        w.preload_k(0);
        w.template any_phase<1>(2 * t + 1, nb);
        race_fence();
      }
      // B of the last block when the wave's blocks fill every tile: V(nkt-1) is still in LDS and
      // the offsets already point at it
      if (nb == 2 * nkt) w.template any_phase<0>(nb, nb);
      point_k(0);
      point_v(0);

      // finalise: O = acc / l, LSE = (m + log2 l) * ln 2
      const float l_tot = w.l_run + xor32(w.l_run);
      {
        const float inv = 1.f / l_tot;
        uint16_t* op = p.o + (int64_t)my_row * p.o_st + (int64_t)h * p.o_sh;
#pragma unroll
        for (int eb = 0; eb < NEB; ++eb) store_block_bf16(op + 32 * eb, w.oacc[eb], inv, hh, row_valid);
        if (row_valid && hh == 0)
          p.lse[(int64_t)h * p.T + my_row] = (w.m_run + log2f(l_tot)) * 0.6931471805599453f;
      }
    }
    if (p.prof && tid == 0) {
      const uint64_t t1 = wall_clock64();
      t_busy += t1 - t0;
      t_last = t1;
      ++n_done;
    }
  }
  if (p.prof && tid == 0) {
    hbp_profile_rec r;
    r.hw_id = hw_id_reg();
    r.xcc_id = xcc_id_reg();
    r.n_items = n_done;
    r.reserved = 0;
    r.first_tick = t_first;
    r.last_tick = t_last;
    r.busy_ticks = t_busy;
    p.prof[blockIdx.x] = r;
  }
}

__global__ void zero_counters_kernel(int32_t* c) {
  if (threadIdx.x < kNumXcd) c[threadIdx.x * kCounterStride] = 0;
}

int launch_zero_counters(int32_t* counters, hipStream_t s) {
  hipLaunchKernelGGL(zero_counters_kernel, dim3(1), dim3(64), 0, s, counters);
  return (int)hipGetLastError();
}

template <int DQK, int DV, int HP, int TP>
static int launch_fwd_hp(const FwdParams& p, int n_cu, hipStream_t s) {
  constexpr int lds_bytes = 2 * 64 * (DQK * 2 + DV * 2);
  static bool attr_set = false;
  if (!attr_set) {
    const hipError_t e = hipFuncSetAttribute((const void*)fwd_kernel<DQK, DV, HP, TP>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return (int)e;
    attr_set = true;
  }
  const int64_t n_items = (int64_t)p.n_tiles * (p.Hq / HP), cap = (int64_t)n_cu * (2 / (HP * TP));
  const int grid = (int)(n_items < cap ? n_items : cap);
  hipLaunchKernelGGL((fwd_kernel<DQK, DV, HP, TP>), dim3(grid), dim3(kThreads * HP * TP), lds_bytes, s, p);
  return (int)hipGetLastError();
}
// tile_rows: rows per query tile of the worklist, 128 or (odd group sizes only) 256
template <int DQK, int DV>
static int launch_fwd_t(const FwdParams& p, int tile_rows, int n_cu, hipStream_t s) {
  if (p.g % 2 == 0) return tile_rows == 128 ? launch_fwd_hp<DQK, DV, 2, 1>(p, n_cu, s) : (int)hipErrorInvalidValue;
  return tile_rows == 256 ? launch_fwd_hp<DQK, DV, 1, 2>(p, n_cu, s) : launch_fwd_hp<DQK, DV, 1, 1>(p, n_cu, s);
}

int launch_fwd(int d_qk, int d_v, const FwdParams& p, int tile_rows, int n_cu, hipStream_t s,
               hipEvent_t ev0, hipEvent_t ev1) {
  if (ev0 && hipEventRecord(ev0, s) != hipSuccess) return (int)hipErrorInvalidValue;
  int e;
  if (d_qk == 64 && d_v == 64) e = launch_fwd_t<64, 64>(p, tile_rows, n_cu, s);
  else if (d_qk == 128 && d_v == 128) e = launch_fwd_t<128, 128>(p, tile_rows, n_cu, s);
  else if (d_qk == 192 && d_v == 128) e = launch_fwd_t<192, 128>(p, tile_rows, n_cu, s);
  else return (int)hipErrorInvalidValue;
  if (e == 0 && ev1 && hipEventRecord(ev1, s) != hipSuccess) return (int)hipErrorInvalidValue;
  return e;
}

}  // namespace hbp
