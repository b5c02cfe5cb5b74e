// Backward kernels: dQ, dK, dV of causal attention inside each sample of a packed buffer, gfx950.
//
// (1) prepass   D[h,r] = sum_x dO[r,h,x] O[r,h,x]; resets the scheduler counters of (2) and (3).
// (2) dq        query-tile major, same skeleton as the forward: work item = (query tile of <=128
//               rows, query head); K and V tiles of 64 keys stream through LDS; per 32-key block
//                   S^T  = K Q^T,  dP^T = V dO^T          (one query per lane column)
//                   dS^T = exp2(S^T c - LSE log2e) (dP^T - D)      (the dP^T accumulator starts at -D)
//                   dQ^T += K^T dS^T                      (K^T by transposing LDS reads)
// (3) dkdv      key-tile major: work item = (key tile of <=128 keys, kv head); each wavefront keeps
//               the K and V fragments of its 32 keys and the dK^T / dV^T accumulators in registers
//               while Q and dO blocks of 64 rows stream through LDS, for every query head of the
//               group (the GQA reduction happens in the accumulators):
//                   S  = Q K^T,  dP = dO V^T               (one key per lane column)
//                   P  = exp2(S c - LSE log2e),  dS = P (dP - D)
//                   dV^T += dO^T P,  dK^T += Q^T dS        (transposing LDS reads of dO and Q)
// No atomics: dQ has its own pass (S and dP are recomputed there), so every output is written
// once and the results are bit-stable from run to run.
#include <type_traits>

#include "common.hpp"

namespace hbp {

constexpr float kLog2e = 1.4426950408889634f;

struct ProfAcc {
  uint32_t n_done = 0;
  uint64_t t_first = 0, t_last = 0, t_busy = 0, t0 = 0;
};
__device__ __forceinline__ void prof_begin(ProfAcc& a, const hbp_profile_rec* prof, int tid) {
  if (prof && tid == 0) {
    a.t0 = wall_clock64();
    if (a.n_done == 0) a.t_first = a.t0;
  }
}
__device__ __forceinline__ void prof_end(ProfAcc& a, const hbp_profile_rec* prof, int tid) {
  if (prof && tid == 0) {
    const uint64_t t1 = wall_clock64();
    a.t_busy += t1 - a.t0;
    a.t_last = t1;
    ++a.n_done;
  }
}
__device__ __forceinline__ void prof_write(const ProfAcc& a, hbp_profile_rec* prof, int tid) {
  if (prof && tid == 0) {
    hbp_profile_rec r;
    r.hw_id = hw_id_reg();
    r.xcc_id = xcc_id_reg();
    r.n_items = a.n_done;
    r.reserved = 0;
    r.first_tick = a.t_first;
    r.last_tick = a.t_last;
    r.busy_ticks = a.t_busy;
    prof[blockIdx.x] = r;
  }
}

// ------------------------------------------------------------------------------------- dQ
// Two workgroups per compute unit where the kernel fits 256 registers (d_qk <= 128): the second
// wavefront on each SIMD fills the issue slots the first one leaves open.
template <int DQK, int DV>
__global__ __launch_bounds__(kThreads, DQK <= 128 ? 2 : 1) void bwd_dq_kernel(const BwdParams p) {
  constexpr int BM = 128, BN = 64;
  constexpr int KRB = DQK * 2, VRB = DV * 2;
  constexpr int K_TILE = BN * KRB, V_TILE = BN * VRB;
  constexpr int NC = DQK / 16, NCV = DV / 16, NDB = DQK / 32;
  constexpr int PD = DQK == 128 ? 3 : 4;  // read-ahead depth: at d = 128 the kernel is two registers short of its 256 with 4
  // Scores in the vector file (asm MFMA): needs a kernel that compiles without spills (checked at build
  // time); the builtin form stays as the fallback.
  constexpr bool kVgprScores = true;

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  // [K buf0][K buf1][V buf0][V buf1]
  char* const k_lds = smem;
  char* const v_lds = smem + 2 * K_TILE;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hh = lane >> 5;

  // Absolute LDS addresses of this lane's fragments: workgroup base and current buffer included
  // (toggled once per tile), so a read needs no address arithmetic.
  const uint32_t lds0 = lds_address(smem);
  // With equal row sizes (d_qk = d_v) a lane's V fragments sit exactly two K tiles behind its K fragments
  // (both buffers toggle together), so one set of addresses serves both.
  constexpr bool kSameRows = DQK == DV;
  uint32_t koff[NC], vnoff[kSameRows ? 1 : NCV], ktoff[2][NDB];
#pragma unroll
  for (int c = 0; c < NC; ++c) koff[c] = lds0 + l32 * KRB + swz<DQK>(2 * c + hh, l32) * 16;
  if (!kSameRows) {
#pragma unroll
    for (int c = 0; c < NCV; ++c) vnoff[c] = lds0 + 2 * K_TILE + l32 * VRB + swz<DV>(2 * c + hh, l32) * 16;
  }
  {
    const int G = lane >> 4, s = lane & 15;
    const int k8 = 4 * hh + (s >> 2);
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        const int c = 4 * db + 2 * (G & 1) + ((s & 3) >> 1);
        ktoff[r][db] = lds0 + (8 * r + k8) * KRB + swz<DQK>(c, 8 * r + k8) * 16 + (s & 1) * 8;
      }
  }

  TileLoader<DQK, BN> k_loader;
  TileLoader<DV, BN> v_loader;  // same lane pattern as k_loader when the row sizes agree: then only that one is kept
  k_loader.init(wave, lane);
  if (!kSameRows) v_loader.init(wave, lane);
  const uint32_t k_stride_b = (uint32_t)p.k_st * 2, v_stride_b = (uint32_t)p.v_st * 2;

  ProfAcc pa;
  const WorkQueues wq{p.counter_dq, p.n_q_tiles, p.Hkv * p.n_split_dq, p.g / p.n_split_dq};
  int q_cur = xcc_id_reg() & (kNumXcd - 1), q_tried = 0;
  for (;;) {
    int tile_idx, h;
    if (!next_item(wq, (int*)smem, tid, q_cur, q_tried, tile_idx, h)) break;
    prof_begin(pa, p.prof_dq, tid);

    const hbp_tile tl = p.q_tiles[tile_idx];
    bool ok = tl.sample >= 0 && tl.sample < p.n_samples;
    int s0 = 0, s1 = 0;
    if (ok) {
      s0 = p.cu[tl.sample];
      s1 = p.cu[tl.sample + 1];
      ok = s0 >= 0 && s1 <= p.T && s0 <= tl.row_begin && tl.row_begin < tl.row_end &&
           tl.row_end <= s1 && tl.row_end - tl.row_begin <= BM;
    }
    if (ok) {
      const int r0 = tl.row_begin, r1 = tl.row_end;
      const int kh = h / p.g;
      const int qw0 = r0 - s0 + 32 * wave;
      const int my_row = r0 + 32 * wave + l32;
      const bool row_valid = my_row < r1;
      const bool wave_active = r0 + 32 * wave < r1;
      const int n_keys = r1 - s0;
      const int nkt = (n_keys + BN - 1) / BN;
      const uint16_t* kbase = p.k + (int64_t)s0 * p.k_st + (int64_t)kh * p.k_sh;
      const uint16_t* vbase = p.v + (int64_t)s0 * p.v_st + (int64_t)kh * p.v_sh;

      // copy `slot` of this wave's share of key tile kt (K first, then V)
      constexpr int NKCP = decltype(k_loader)::PER_WAVE, NVCP = decltype(v_loader)::PER_WAVE;
      auto issue_slot = [&](int kt, int slot) {
        const int k_off = kt * BN;
        const int valid = n_keys - k_off;
        if (slot < NKCP) {
          k_loader.issue_one(slot, kbase + (int64_t)k_off * p.k_st, k_stride_b, valid, k_lds + (kt & 1) * K_TILE, wave);
        } else if constexpr (kSameRows) {
          k_loader.issue_one(slot - NKCP, vbase + (int64_t)k_off * p.v_st, v_stride_b, valid, v_lds + (kt & 1) * V_TILE, wave);
        } else {
          v_loader.issue_one(slot - NKCP, vbase + (int64_t)k_off * p.v_st, v_stride_b, valid, v_lds + (kt & 1) * V_TILE, wave);
        }
      };
      auto issue = [&](int kt) {
#pragma unroll
        for (int slot = 0; slot < NKCP + NVCP; ++slot) issue_slot(kt, slot);
      };
      issue(0);

      Frag qf[NC], dof[NCV];
      float lse2 = INFINITY, Dv = 0.f;  // +inf: rows past the tile end get probability 0
      {
        const uint16_t* qp = p.q + (int64_t)my_row * p.q_st + (int64_t)h * p.q_sh + 8 * hh;
        const uint16_t* dop = p.d_o + (int64_t)my_row * p.o_st + (int64_t)h * p.o_sh + 8 * hh;
#pragma unroll
        for (int c = 0; c < NC; ++c) qf[c].u = row_valid ? *(const u32x4*)(qp + 16 * c) : u32x4{0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < NCV; ++c) dof[c].u = row_valid ? *(const u32x4*)(dop + 16 * c) : u32x4{0, 0, 0, 0};
        if (row_valid) {
          lse2 = p.lse2[(int64_t)h * p.T + my_row];
          Dv = p.D[(int64_t)h * p.T + my_row];
        }
      }
      // the dP^T accumulator of every block starts at -D of the lane's query (one value per lane): the
      // subtraction in dS = P (dP - D) then comes out of the MFMAs
      f32x16 negD;
#pragma unroll
      for (int i = 0; i < 16; ++i) negD[i] = -Dv;
      asm volatile("" : "+v"(negD));
      f32x16 dqacc[NDB];
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dqacc[db][i] = 0.f;
      const int q_in = qw0 + l32;

      // One 32-key block: sd = (S^T, dP^T - D) products, sm = dS^T = exp2(c S^T - LSE2)(dP^T - D),
      // gr = dQ^T += K^T dS^T.  Interior tiles pipeline their two blocks inside the wave:
      //     sd(0) | sd(1) + sm(0) | gr(0) + sm(1) first half | gr(1) first half + sm(1) rest | gr(1) rest
      struct Blk {
        f32x16 s, dp;
        Frag dsf[2];
      };
      // buf: a compile-time tile buffer on top of where the lane's offsets point (the interior loop names
      // the second buffer this way, in the reads' immediate offsets, instead of moving the offsets per tile)
      auto sd_load = [&](int blk, int buf = 0) {
        return [&, blk, buf](int i) {
          const int ka = 32 * blk * KRB + buf * K_TILE, va = 32 * blk * VRB + buf * V_TILE;
          Frag a;
          if (i < NC) a.u = *(const __attribute__((address_space(3))) u32x4*)(uintptr_t)(koff[i] + ka);
          else if (kSameRows) a.u = *(const __attribute__((address_space(3))) u32x4*)(uintptr_t)(koff[i - NC] + (2 * K_TILE + va));
          else a.u = *(const __attribute__((address_space(3))) u32x4*)(uintptr_t)(vnoff[i - NC] + va);
          return a;
        };
      };
      auto sd_mma = [&](Blk& x) {
        return [&](int i, const Frag& a) {
          if (kVgprScores) {
            if (i == 0) x.s = mfma32_vgpr_first(a.v, qf[0].v);
            else if (i < NC) mfma32_vgpr(x.s, a.v, qf[i].v);
            else if (i == NC) x.dp = mfma32_vgpr_from(a.v, dof[0].v, negD);  // starts at -D: ends as dP - D
            else mfma32_vgpr(x.dp, a.v, dof[i - NC].v);
          } else {
            if (i == 0 || i == NC) {
              f32x16 z;
#pragma unroll
              for (int e = 0; e < 16; ++e) z[e] = 0.f;
              if (i == 0) x.s = mfma32(a.v, qf[0].v, z);
              else x.dp = mfma32(a.v, dof[0].v, negD);
            } else if (i < NC) {
              x.s = mfma32(a.v, qf[i].v, x.s);
            } else {
              x.dp = mfma32(a.v, dof[i - NC].v, x.dp);
            }
          }
        };
      };
      auto gr_frag = [&](int blk, int j, int db, int buf = 0) {
        const uint32_t base = (32 * blk + 16 * j) * KRB + buf * K_TILE;
        Frag a;
        a.h[0] = lds_read_tr16_at(ktoff[0][db] + base);
        a.h[1] = lds_read_tr16_at(ktoff[1][db] + base);
        return a;
      };
      // slices 0..16 of a block: slice k issues exp for element k (k < 16) and finishes element
      // k-1 (k > 0); element e = 4b+v <-> key 32 blk + 8b + 4hh + v of the tile, query column q_in
      float e_cur = 0.f, ds_even = 0.f;
      auto sm_slice = [&](Blk& x, int kb, int k, auto masked) {
        const float e_prev = e_cur;
        if (k < 16) e_cur = __builtin_amdgcn_exp2f(__builtin_fmaf(x.s[k], p.scale_log2, -lse2));
        if (k > 0) {
          const int e = k - 1;
          float pr = e_prev;
          if (decltype(masked)::value) {
            if (kb + 8 * (e >> 2) + 4 * hh + (e & 3) > q_in) pr = 0.f;
          }
          const float ds = pr * x.dp[e];
          if (e & 1) x.dsf[e >> 3].w[(e & 7) >> 1] = pack_bf16(ds_even, ds);
          else ds_even = ds;
        }
      };

      int cur_buf = 0;
      auto point_offsets_at = [&](int buf) {
        const int dk = buf ? K_TILE : -K_TILE, dv = buf ? V_TILE : -V_TILE;
#pragma unroll
        for (int c = 0; c < NC; ++c) koff[c] += dk;
        if (!kSameRows) {
#pragma unroll
          for (int c = 0; c < NCV; ++c) vnoff[c] += dv;
        }
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
          for (int db = 0; db < NDB; ++db) ktoff[r][db] += dk;
        cur_buf = buf;
      };
      // copies_now: the next tile's copies go out here in one go; an interior tile spreads them behind the MFMAs
      // of its first chain instead (a tile follows every interior tile)
      auto begin_tile = [&](int kt, bool point = true, bool copies_now = true) {
        race_fence();
        wait_async_loads();
        __syncthreads();
        if (copies_now && kt + 1 < nkt) issue(kt + 1);
        if (point && (kt & 1) != cur_buf) point_offsets_at(kt & 1);
      };

      const int n_interior = wave_active ? min(nkt, (qw0 + 1) / BN) : 0;
      // One interior tile.  BUF = kt & 1 as a compile-time constant: the lane's offsets stay on buffer 0
      // and the reads carry the buffer in their immediate offsets; BUF < 0: the offsets follow the buffers.
      auto interior_tile = [&](auto bufc, int kt) {
        constexpr int BUF = decltype(bufc)::value < 0 ? 0 : decltype(bufc)::value;
        begin_tile(kt, decltype(bufc)::value < 0, false);
        const int k_off = kt * BN;
        Blk x0, x1;
        LdsChain<NC + NCV, PD> c1;
        c1.prefill(sd_load(0, BUF));
        c1.template run_with<NKCP + NVCP>(sd_load(0, BUF), sd_mma(x0), [&](int slot) { issue_slot(kt + 1, slot); });
        c1.prefill(sd_load(1, BUF));
        if (kVgprScores) mfma_results_ready(x0.s, x0.dp);
        c1.template run_with<17>(sd_load(1, BUF), sd_mma(x1), [&](int k) { sm_slice(x0, k_off, k, std::false_type{}); });
        // gr(0) (2*NDB MFMAs) then gr(1) j=0 (NDB) then gr(1) j=1 (NDB), with sm(1) spread so that
        // dS chunk j of block 1 is complete before the MFMAs that read it
        constexpr int LG = 4 * NDB;
        auto g_load = [&](int i) {
          const int blk = i / (2 * NDB), j = (i / NDB) & 1, db = i % NDB;
          return gr_frag(blk, j, db, BUF);
        };
        LdsChain<LG, PD> c2;
        c2.prefill(g_load);
        if (kVgprScores) mfma_results_ready(x1.s, x1.dp);
#pragma unroll
        for (int i = 0; i < LG; ++i) {
          const int blk = i / (2 * NDB), j = (i / NDB) & 1, db = i % NDB;
          Blk& x = blk ? x1 : x0;
          dqacc[db] = mfma32(c2.ring[i % PD].v, x.dsf[j].v, dqacc[db]);
          if (i + PD < LG) c2.ring[i % PD] = g_load(i + PD);
          // sm(1): slices 0..8 behind gr(0) (chunk 0 of block 1 done), 9..16 behind gr(1) j=0
          constexpr int A = 2 * NDB, B = NDB;
          if (i < A) {
#pragma unroll
            for (int k = i * 9 / A; k < (i + 1) * 9 / A; ++k) sm_slice(x1, k_off + 32, k, std::false_type{});
          } else if (i < A + B) {
#pragma unroll
            for (int k = 9 + (i - A) * 8 / B; k < 9 + (i - A + 1) * 8 / B; ++k)
              sm_slice(x1, k_off + 32, k, std::false_type{});
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      int kt = 0;  // the offsets point at buffer 0 here
      for (; kt + 1 < n_interior; kt += 2) {
        interior_tile(std::integral_constant<int, 0>{}, kt);
        interior_tile(std::integral_constant<int, 1>{}, kt + 1);
      }
      for (; kt < n_interior; ++kt) interior_tile(std::integral_constant<int, -1>{}, kt);
      for (; kt < nkt; ++kt) {  // tiles that touch the diagonal: plain masked path, block by block
        begin_tile(kt);
        const int k_off = kt * BN;
        if (!wave_active || k_off > qw0 + 31) continue;
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
          const int kb = k_off + 32 * blk;
          if (kb > qw0 + 31) continue;
          Blk x;
          LdsChain<NC + NCV, PD> c1;
          c1.prefill(sd_load(blk));
          c1.run(sd_load(blk), sd_mma(x));
          auto g_load = [&](int i) { return gr_frag(blk, i / NDB, i % NDB); };
          LdsChain<2 * NDB, PD> c2;
          c2.prefill(g_load);
          if (kVgprScores) mfma_results_ready(x.s, x.dp);
#pragma unroll
          for (int k = 0; k < 17; ++k) sm_slice(x, kb, k, std::true_type{});
          __builtin_amdgcn_sched_barrier(0);
          c2.run(g_load, [&](int i, const Frag& a) { dqacc[i % NDB] = mfma32(a.v, x.dsf[i / NDB].v, dqacc[i % NDB]); });
        }
      }
      if (cur_buf) point_offsets_at(0);

      {
        uint16_t* dqp = p.dq + (int64_t)my_row * p.q_st + (int64_t)h * p.q_sh;
#pragma unroll
        for (int db = 0; db < NDB; ++db) store_block_bf16(dqp + 32 * db, dqacc[db], p.scale, hh, row_valid);
      }
    }
    prof_end(pa, p.prof_dq, tid);
  }
  prof_write(pa, p.prof_dq, tid);
}

// ----------------------------------------------------------------------------------- dK, dV
template <int DQK, int DV>
__global__ __launch_bounds__(kThreads, 1) void bwd_dkdv_kernel(const BwdParams p) {
  constexpr int BN = 128, BQ = 64;
  constexpr int QRB = DQK * 2, ORB = DV * 2;
  constexpr int Q_TILE = BQ * QRB, O_TILE = BQ * ORB;
  constexpr int NC = DQK / 16, NCV = DV / 16, NDB = DQK / 32, NEB = DV / 32;

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  // [Q buf0][Q buf1][dO buf0][dO buf1][lse buf0|buf1][D buf0|buf1]
  char* const q_lds = smem;
  char* const o_lds = smem + 2 * Q_TILE;
  float* const lse_lds = (float*)(smem + 2 * Q_TILE + 2 * O_TILE);
  float* const d_lds = lse_lds + 2 * BQ;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hh = lane >> 5;

  // Absolute LDS addresses of this lane's fragments in buffer 0 (workgroup base included): a read
  // needs no address arithmetic, the buffer and the sub-block go into its immediate offset.
  const uint32_t lds0 = lds_address(smem);
  uint32_t qoff[NC], dooff[NCV], qtoff[2][NDB], dotoff[2][NEB];
#pragma unroll
  for (int c = 0; c < NC; ++c) qoff[c] = lds0 + l32 * QRB + swz<DQK>(2 * c + hh, l32) * 16;
#pragma unroll
  for (int c = 0; c < NCV; ++c) dooff[c] = lds0 + 2 * Q_TILE + l32 * ORB + swz<DV>(2 * c + hh, l32) * 16;
  {
    const int G = lane >> 4, s = lane & 15;
    const int k8 = 4 * hh + (s >> 2);
#pragma unroll
    for (int r = 0; r < 2; ++r) {
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        const int c = 4 * db + 2 * (G & 1) + ((s & 3) >> 1);
        qtoff[r][db] = lds0 + (8 * r + k8) * QRB + swz<DQK>(c, 8 * r + k8) * 16 + (s & 1) * 8;
      }
#pragma unroll
      for (int eb = 0; eb < NEB; ++eb) {
        const int c = 4 * eb + 2 * (G & 1) + ((s & 3) >> 1);
        dotoff[r][eb] = lds0 + 2 * Q_TILE + (8 * r + k8) * ORB + swz<DV>(c, 8 * r + k8) * 16 + (s & 1) * 8;
      }
    }
  }
  // LDS addresses of this lane's LSE2 / D rows inside the current buffer
  uint32_t lseoff = lds0 + 2 * Q_TILE + 2 * O_TILE + 16 * hh;
  uint32_t dvoff = lseoff + 2 * BQ * 4;

  const uint32_t q_stride_b = (uint32_t)p.q_st * 2, o_stride_b = (uint32_t)p.o_st * 2;
  FullTileLoader<DQK, BQ> q_loader;
  FullTileLoader<DV, BQ> o_loader;
  q_loader.init(wave, lane, q_stride_b);
  o_loader.init(wave, lane, o_stride_b);

  // Both tile buffers start out as zeros: an idle step (see the step loop) multiplies whatever the
  // second buffer holds by zero operands, and that must not be the NaN patterns of unwritten LDS.
  for (int i = tid * 16; i < 2 * Q_TILE + 2 * O_TILE + 4 * BQ * (int)sizeof(float); i += kThreads * 16)
    *(u32x4*)(smem + i) = u32x4{0, 0, 0, 0};
  __syncthreads();

  ProfAcc pa;
  // Work item = (key tile, kv head, part of its query heads): with n_split > 1 the g heads of a kv head
  // are cut into n_split runs of g_item heads, each an item of its own.
  const WorkQueues wq{p.counter, p.n_tiles, p.Hkv * p.n_split, 1};
  const int g_item = p.g / p.n_split;
  int q_cur = xcc_id_reg() & (kNumXcd - 1), q_tried = 0;
  for (;;) {
    int tile_idx, vh;
    if (!next_item(wq, (int*)smem, tid, q_cur, q_tried, tile_idx, vh)) break;
    const int kh = vh / p.n_split, part = vh - kh * p.n_split;
    const int head0 = vh * g_item;  // first query head of the item
    prof_begin(pa, p.prof, tid);

    const hbp_tile tl = p.tiles[tile_idx];
    bool ok = tl.sample >= 0 && tl.sample < p.n_samples;
    int s0 = 0, s1 = 0;
    if (ok) {
      s0 = p.cu[tl.sample];
      s1 = p.cu[tl.sample + 1];
      ok = s0 >= 0 && s1 <= p.T && s0 <= tl.row_begin && tl.row_begin < tl.row_end &&
           tl.row_end <= s1 && tl.row_end - tl.row_begin <= BN;
    }
    if (ok) {
      const int s_len = s1 - s0;
      const int k0_in = tl.row_begin - s0;
      const int kw0_in = k0_in + 32 * wave;
      const int my_key = tl.row_begin + 32 * wave + l32;
      const bool key_valid = my_key < tl.row_end;
      const bool wave_active = tl.row_begin + 32 * wave < tl.row_end;
      const int key_in = kw0_in + l32;

      const int qb_start = (k0_in / BQ) * BQ;
      const int nqb = (s_len - qb_start + BQ - 1) / BQ;
      const int n_steps = nqb * g_item;

      // Step order: the query blocks from the LAST one of the sample down to the tile's own, and for each
      // block the g query heads of the group.  Every key tile of a sample needs a suffix of the same
      // blocks, so the workgroups of a die (they work on tiles of the same kv head) ask for the same
      // block at about the same time and it comes from that die's L2 once, not from HBM once per tile.
      // That only works while they walk in step: 32 workgroups two blocks apart put 8 MB between two
      // uses of a block, more than the L2 holds.  The w workgroups that share a kv head take the tiles
      // of a long sample w at a time, longest first.  Tiles 0..w-1 start together and end BN/BQ blocks
      // apart (each is that much shorter than the one before); their workgroups then take tiles
      // w..2w-1 one after the other, BN/BQ blocks apart.  Such a tile starts as many blocks below the top
      // as it starts late (where the first tile of its set is by then) and does the blocks it skipped at
      // the end; that set of w tiles ends together, the next one starts together, and so on in turns.  The
      // order is a function of the tile number alone, so the results do not depend on timing.
      // (With fewer than 8 workgroups per kv head there is little to share and the plain order is kept.)
      const int w_share = (int)gridDim.x / min(p.Hkv * p.n_split, kNumXcd * kHeadGroup);  // heads in work at a time
      int skip = w_share >= 8 && ((tl.tile / w_share) & 1) ? (tl.tile % w_share) * (BN / BQ) : 0;
      skip = max(0, min(skip, nqb - 1));
      const int first_blk = nqb - 1 - skip;
      // the blocks are taken in the order first_blk .. 0, then nqb-1 .. first_blk+1, g steps each
      // Copies are issued in step order; the source pointers of the next block to copy are carried
      // along instead of being recomputed from the step number.
      const int64_t first_row = (int64_t)s0 + qb_start + (int64_t)first_blk * BQ;
      const uint16_t* q_blk = p.q + first_row * p.q_st + (int64_t)head0 * p.q_sh;
      const uint16_t* o_blk = p.d_o + first_row * p.o_st + (int64_t)head0 * p.o_sh;
      const float* row_blk = (wave == 0 ? p.lse2 : p.D) + (int64_t)head0 * p.T + first_row;
      const uint16_t* q_src = q_blk;
      const uint16_t* o_src = o_blk;
      const float* row_src = row_blk;
      int blk_next = first_blk, head_next = 0;
      // The copies of a step's operands are issued one at a time (slot 0 .. N_COPY-1), so that they can sit
      // behind the MFMAs of the step before; taking the last slot moves the source on to the next step.
      // qb_in[buf]: first query row (in-sample) of the block whose copies went to buffer buf.
      constexpr int NQC = decltype(q_loader)::PER_WAVE, NOC = decltype(o_loader)::PER_WAVE;
      constexpr int N_COPY = NQC + NOC + 1;
      int qb_in[2] = {0, 0};
      // FULL: all BQ rows of the block exist (no clamping of the source rows, no vector arithmetic at all)
      auto issue_copy = [&](int slot, int buf, auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        const int valid = FULL ? BQ : s_len - qb_start - blk_next * BQ;  // >= 1; < BQ only for the sample's last block
        if (slot < NQC) {
          if (FULL) q_loader.issue_full(slot, q_src, q_lds + buf * Q_TILE, wave);
          else q_loader.issue_one(slot, q_src, q_stride_b, valid, q_lds + buf * Q_TILE, wave, lane);
        } else if (slot < NQC + NOC) {
          if (FULL) o_loader.issue_full(slot - NQC, o_src, o_lds + buf * O_TILE, wave);
          else o_loader.issue_one(slot - NQC, o_src, o_stride_b, valid, o_lds + buf * O_TILE, wave, lane);
        } else {
          if (wave < 2) {
            // issued through the same untracked path as the tiles: the compiler must not see an LDS
            // write here, or it would drain every outstanding copy before the next LDS read
            const int row = lane < valid ? lane : valid - 1;
            const float* dst = (wave == 0 ? lse_lds : d_lds) + buf * BQ;
            async_copy4(row_src, (uint32_t)row * 4u, lds_address(dst));
          }
          qb_in[buf] = qb_start + blk_next * BQ;
          if (++head_next == g_item) {  // on to the block before; from the tile's own block to the sample's last
            head_next = 0;
            const int64_t jump = blk_next == 0 ? (int64_t)(nqb - 1) * BQ : -(int64_t)BQ;
            blk_next = blk_next == 0 ? nqb - 1 : blk_next - 1;
            q_blk += jump * p.q_st;
            o_blk += jump * p.o_st;
            row_blk += jump;
            q_src = q_blk;
            o_src = o_blk;
            row_src = row_blk;
          } else {
            q_src += p.q_sh;
            o_src += p.o_sh;
            row_src += p.T;
          }
        }
      };
      auto next_is_full = [&]() { return s_len - qb_start - blk_next * BQ >= BQ; };
      auto issue_next = [&](int buf) {  // all of a step's copies in one go
#pragma unroll
        for (int slot = 0; slot < N_COPY; ++slot) issue_copy(slot, buf, std::false_type{});
      };
      if (n_steps > 0) issue_next(0);

      // register-resident B operands of this wave's 32 keys: lane column = key l32
      Frag knat[NC], vnat[NCV];
      {
        const uint16_t* kp = p.k + (int64_t)my_key * p.k_st + (int64_t)kh * p.k_sh + 8 * hh;
        const uint16_t* vp = p.v + (int64_t)my_key * p.v_st + (int64_t)kh * p.v_sh + 8 * hh;
#pragma unroll
        for (int c = 0; c < NC; ++c) knat[c].u = key_valid ? *(const u32x4*)(kp + 16 * c) : u32x4{0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < NCV; ++c) vnat[c].u = key_valid ? *(const u32x4*)(vp + 16 * c) : u32x4{0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < NCV; ++c) vnat[c].u ^= u32x4{0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};
      }
      f32x16 dkt[NDB], dvt[NEB];
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dkt[db][i] = 0.f;
#pragma unroll
      for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
        for (int i = 0; i < 16; ++i) dvt[eb][i] = 0.f;

      // One 32-query x 32-key sub-block: sd = (S, dP) products, sm = probabilities and dS,
      // gr = dV^T / dK^T updates.  Away from the diagonal two sub-blocks are software-pipelined
      // inside the wave so the vector arithmetic of one is spread, one element per MFMA, behind the
      // other's MFMAs (the matrix pipe leaves about half of each MFMA's issue time free):
      //     sd(A) | sd(B) + sm(A) | gr(A) + sm(B) | gr(B)
      // Blocks that touch the diagonal or the sample tail take the plain masked path.
      struct Sub {
        f32x16 s, dp;
        Frag pb[2], dsb[2];
      };
      constexpr int kPD = 3;  // LDS read-ahead depth (fragments)
      // active: a step of the item (not the idle one that makes the count even); has_next: another step
      // follows, whose operands this step copies into the other buffer.
      auto do_step = [&](auto buf_tag, bool active, bool has_next) {
        // the step's buffer is a compile-time constant: it goes into the immediate offset of every LDS
        // read (two copies of the step's code instead of 34 address updates per step)
        constexpr int BUF = decltype(buf_tag)::value;
        const int qb = qb_in[BUF];
        auto sd_load = [&](int sub) {
          return [&, sub](int i) {
            Frag a;
            if (i < NC) a.u = *(const __attribute__((address_space(3))) u32x4*)(uintptr_t)(qoff[i] + 32 * sub * QRB + BUF * Q_TILE);
            else a.u = *(const __attribute__((address_space(3))) u32x4*)(uintptr_t)(dooff[i - NC] + 32 * sub * ORB + BUF * O_TILE);
            return a;
          };
        };
        // The asm form (scores produced in the vector file) needs a kernel that compiles without
        // register spills: spill copies next to an asm MFMA would bypass the compiler's hazard
        // handling.  Every instantiation does (a build-time test checks it); the builtin form stays
        // as the fallback should one stop doing so.
        constexpr bool kVgprScores = true;
        auto sd_mma = [&](Sub& x) {
          return [&](int i, const Frag& a) {
            if (kVgprScores) {
              if (i == 0) x.s = mfma32_vgpr_first(a.v, knat[0].v);
              else if (i < NC) mfma32_vgpr(x.s, a.v, knat[i].v);
              else if (i == NC) mfma32_vgpr(x.dp, a.v, vnat[0].v);
              else mfma32_vgpr(x.dp, a.v, vnat[i - NC].v);
            } else {
              if (i == 0 || i == NC) {
                f32x16 z;
#pragma unroll
                for (int e = 0; e < 16; ++e) z[e] = 0.f;
                if (i == 0) x.s = mfma32(a.v, knat[0].v, z);
                else x.dp = mfma32(a.v, vnat[0].v, z);
              } else if (i < NC) {
                x.s = mfma32(a.v, knat[i].v, x.s);
              } else {
                x.dp = mfma32(a.v, vnat[i - NC].v, x.dp);
              }
            }
          };
        };
        auto gr_load = [&](int sub) {
          return [&, sub](int i) {
            Frag a;
            if (i < 2 * NEB) {
              const int eb = i % NEB, j = i / NEB;
              const uint32_t base = (32 * sub + 16 * j) * ORB + BUF * O_TILE;
              a.h[0] = lds_read_tr16_at(dotoff[0][eb] + base);
              a.h[1] = lds_read_tr16_at(dotoff[1][eb] + base);
            } else {
              const int db = (i - 2 * NEB) % NDB, j = (i - 2 * NEB) / NDB;
              const uint32_t base = (32 * sub + 16 * j) * QRB + BUF * Q_TILE;
              a.h[0] = lds_read_tr16_at(qtoff[0][db] + base);
              a.h[1] = lds_read_tr16_at(qtoff[1][db] + base);
            }
            return a;
          };
        };
        auto gr_mma = [&](Sub& x) {
          return [&](int i, const Frag& a) {
            if (i < 2 * NEB) dvt[i % NEB] = mfma32(a.v, x.pb[i / NEB].v, dvt[i % NEB]);
            else dkt[(i - 2 * NEB) % NDB] = mfma32(a.v, x.dsb[(i - 2 * NEB) / NDB].v, dkt[(i - 2 * NEB) % NDB]);
          };
        };
        // element i = 4b+v of the accumulators <-> query q0 + 8b + 4hh + v, key column key_in.
        // The per-element arithmetic  pr = exp2(c*s - lse2);  ds = pr * (D - dP)  is issued in two
        // stages one slice apart (stage 1 of element i next to stage 2 of element i-1), so that no
        // vector instruction waits on the one just before it; LSE2 of the 4 query rows of group b is
        // read from LDS one group ahead (rows_prefetch(sub, 0) before the chain).  D - dP comes
        // straight out of the MFMAs: the accumulator starts as D (init_dp) and V is held negated, so
        // no subtraction is left for the vector unit; dS and dK carry the opposite sign until the
        // final scaling.
        f32x4 l4, l4n;
        float e_cur = 0.f;  // exp of element i (stage 1)
        float pr_even = 0.f, ds_even = 0.f;
        auto rows_prefetch = [&](int sub, int b) {
          l4n = *(const __attribute__((address_space(3))) f32x4*)(uintptr_t)(lseoff + (32 * sub + 8 * b + BUF * BQ) * 4);
        };
        // the dP accumulator of a sub-block starts as D (V is held negated: it ends as D - dP)
        auto init_dp = [&](Sub& x, int sub) {
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            const f32x4 t = *(const __attribute__((address_space(3))) f32x4*)(uintptr_t)(dvoff + (32 * sub + 8 * b + BUF * BQ) * 4);
#pragma unroll
            for (int v = 0; v < 4; ++v) x.dp[4 * b + v] = t[v];
          }
        };
        auto stage2 = [&](Sub& x, int sub, int i, float e_val, auto masked) {
          const int b = i >> 2, v = i & 3;
          float pr = e_val;
          if (decltype(masked)::value) {
            const int q_in = qb + 32 * sub + 8 * b + 4 * hh + v;
            if (key_in > q_in || q_in >= s_len) pr = 0.f;
          }
          const float ds = pr * x.dp[i];
          if (i & 1) {
            x.pb[b >> 1].w[2 * (b & 1) + (v >> 1)] = pack_bf16(pr_even, pr);
            x.dsb[b >> 1].w[2 * (b & 1) + (v >> 1)] = pack_bf16(ds_even, ds);
          } else {
            pr_even = pr;
            ds_even = ds;
          }
        };
        // slices 0..16: slice i runs stage 1 of element i (i < 16) and stage 2 of element i-1 (i > 0)
        auto sm_slice = [&](Sub& x, int sub, int i, auto masked) {
          const float e_prev = e_cur;
          if (i < 16) {
            const int b = i >> 2, v = i & 3;
            if (v == 0) {
              l4 = l4n;
              if (b < 3) rows_prefetch(sub, b + 1);
            }
            e_cur = __builtin_amdgcn_exp2f(__builtin_fmaf(x.s[i], p.scale_log2, -l4[v]));
          }
          if (i > 0) stage2(x, sub, i - 1, e_prev, masked);
        };
        // Every update of the dK^T / dV^T accumulators of a step is issued from ONE place (the two gr
        // chains at the end), whatever path computed the probabilities: with updates in several
        // branches the compiler keeps a second set of the 128 accumulator registers and copies one
        // set to the other in every step (one vector instruction per register).
        //
        // The step opens with the first LDS reads of sub-block A, which depend on nothing but the buffer: a
        // single wave per SIMD has nothing else to run while they are under way, so everything that can wait
        // (the step's flags, the copies for the next step) comes after them, and the copies go out one by one
        // behind the first MFMA chain, which carries no vector arithmetic (measured per step of 3600 clocks:
        // 800 clocks from the last MFMA of a step to the first of the next with the bookkeeping, a burst of
        // copies and the reads one after the other; 350 this way, and the copies cost the chain 340).
        Sub xa, xb;
        LdsChain<NC + NCV, kPD> c1;
        c1.prefill(sd_load(0));
        init_dp(xa, 0);  // behind the operand reads: only the first dP MFMA needs it
        // not in reach: the block lies above this wave's keys, or this is the idle step that makes the count even
        const bool in_reach = wave_active && active && qb + BQ - 1 >= kw0_in;
        const bool need_a = in_reach && qb + 31 >= kw0_in;           // qb < s_len always holds
        const bool need_b = in_reach && qb + 63 >= kw0_in && qb + 32 < s_len;
        const bool any_mask = kw0_in + 31 > qb || qb + 63 >= s_len;  // diagonal or sample tail in reach
        const bool pair = need_a && need_b && !any_mask;
        if (pair) {
          // a next block with all its rows (every block but a sample's last) is copied slot by slot behind
          // the MFMAs; the clamped form needs vector arithmetic and registers, and goes out up front.  One
          // chain for both cases: with the chain on two paths the compiler joins the score registers by
          // copies placed right behind the asm MFMAs, before their results exist.
          const bool behind = has_next && next_is_full();
          if (has_next && !behind) issue_next(1 - BUF);
          c1.template run_with<N_COPY>(sd_load(0), sd_mma(xa), [&](int slot) {
            if (behind) issue_copy(slot, 1 - BUF, std::true_type{});
          });
          rows_prefetch(0, 0);
          init_dp(xb, 1);
          c1.prefill(sd_load(1));
          if (kVgprScores) mfma_results_ready(xa.s, xa.dp);
          c1.template run_with<16>(sd_load(1), sd_mma(xb), [&](int i) { sm_slice(xa, 0, i, std::false_type{}); });
          sm_slice(xa, 0, 16, std::false_type{});
        } else {
          // sub-block A: masked, finished here.  Sub-block B: its probabilities are formed by the same
          // unmasked slices as on the fast path (behind the first gr chain below), so the mask goes
          // into the scores instead: -inf gives exp2 = 0 (the scale is positive) and dS = 0 (dP - D).
          if (has_next) issue_next(1 - BUF);
          if (need_a) {
            c1.run(sd_load(0), sd_mma(xa));
            rows_prefetch(0, 0);
            if (kVgprScores) mfma_results_ready(xa.s, xa.dp);
#pragma unroll
            for (int i = 0; i < 17; ++i) sm_slice(xa, 0, i, std::true_type{});
          } else {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
              xa.pb[j].u = u32x4{0, 0, 0, 0};
              xa.dsb[j].u = u32x4{0, 0, 0, 0};
            }
          }
          if (need_b) {
            init_dp(xb, 1);
            c1.prefill(sd_load(1));
            c1.run(sd_load(1), sd_mma(xb));
            if (kVgprScores) mfma_results_ready(xb.s, xb.dp);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int q_in = qb + 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
              if (key_in > q_in || q_in >= s_len) xb.s[i] = -INFINITY;
            }
          } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              xb.s[i] = -INFINITY;
              xb.dp[i] = 0.f;
            }
          }
        }
        rows_prefetch(1, 0);
        __builtin_amdgcn_sched_barrier(0);
        LdsChain<2 * NEB + 2 * NDB, kPD> c2;
        c2.prefill(gr_load(0));
        if (kVgprScores) mfma_results_ready(xb.s, xb.dp);
        c2.template run_with<16>(gr_load(0), gr_mma(xa), [&](int i) { sm_slice(xb, 1, i, std::false_type{}); });
        sm_slice(xb, 1, 16, std::false_type{});
        c2.prefill(gr_load(1));
        c2.run(gr_load(1), gr_mma(xb));
      };

      // Two steps per iteration, one on each buffer, with no branch between them: the accumulators are
      // updated at two places that follow each other, never on alternative paths.  An odd number of
      // steps is rounded up by an idle step (zero operands).
      for (int step = 0; step < n_steps; step += 2) {
        wait_async_loads();
        __syncthreads();
        do_step(std::integral_constant<int, 0>{}, true, step + 1 < n_steps);
        race_fence();
        wait_async_loads();
        __syncthreads();
        do_step(std::integral_constant<int, 1>{}, step + 1 < n_steps, step + 2 < n_steps);
        race_fence();
      }

      if (p.n_split == 1) {
        uint16_t* dkp = p.dk + (int64_t)my_key * p.k_st + (int64_t)kh * p.k_sh;
        uint16_t* dvp = p.dv + (int64_t)my_key * p.v_st + (int64_t)kh * p.v_sh;
#pragma unroll
        for (int db = 0; db < NDB; ++db) store_block_bf16(dkp + 32 * db, dkt[db], -p.scale, hh, key_valid);
#pragma unroll
        for (int eb = 0; eb < NEB; ++eb) store_block_bf16(dvp + 32 * eb, dvt[eb], 1.0f, hh, key_valid);
      } else if (key_valid) {
        // this part's sums, fp32, [part][key][kv head][dim]; the reduce kernel adds the parts up
        const int64_t row = ((int64_t)part * p.T + my_key) * p.Hkv + kh;
        float* dkp = p.dk_part + row * DQK + 4 * hh;
        float* dvp = p.dv_part + row * DV + 4 * hh;
        const float ksc = -p.scale;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int b = 0; b < 4; ++b)
            *(f32x4*)(dkp + 32 * db + 8 * b) = f32x4{dkt[db][4 * b] * ksc, dkt[db][4 * b + 1] * ksc,
                                                       dkt[db][4 * b + 2] * ksc, dkt[db][4 * b + 3] * ksc};
#pragma unroll
        for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
          for (int b = 0; b < 4; ++b)
            *(f32x4*)(dvp + 32 * eb + 8 * b) = f32x4{dvt[eb][4 * b], dvt[eb][4 * b + 1], dvt[eb][4 * b + 2], dvt[eb][4 * b + 3]};
      }
    }
    prof_end(pa, p.prof, tid);
  }
  prof_write(pa, p.prof, tid);
}

// dK, dV = sum over the parts of the partial sums of the key-tile kernel, in part order.  One workgroup
// per key tile of the worklist (only rows covered by a tile are written, as without parts); a thread
// handles four consecutive dims of one (key, kv head).
template <int DQK, int DV>
__global__ __launch_bounds__(kThreads) void bwd_reduce_parts_kernel(const BwdParams p) {
  const hbp_tile tl = p.tiles[blockIdx.x];
  if (tl.sample < 0 || tl.sample >= p.n_samples) return;
  const int s0 = p.cu[tl.sample], s1 = p.cu[tl.sample + 1];
  if (!(s0 >= 0 && s1 <= p.T && s0 <= tl.row_begin && tl.row_begin < tl.row_end && tl.row_end <= s1 &&
        tl.row_end - tl.row_begin <= 128))
    return;
  constexpr int QK4 = DQK / 4, V4 = DV / 4;
  const int n_rows = tl.row_end - tl.row_begin;
  const int64_t n_units = (int64_t)n_rows * p.Hkv * (QK4 + V4);
  for (int64_t u = threadIdx.x; u < n_units; u += kThreads) {
    const int c = (int)(u % (QK4 + V4));
    const int64_t rk = u / (QK4 + V4);
    const int kh = (int)(rk % p.Hkv);
    const int64_t key = tl.row_begin + rk / p.Hkv;
    const bool is_k = c < QK4;
    const int dim = is_k ? DQK : DV, x = 4 * (is_k ? c : c - QK4);
    const float* src = (is_k ? p.dk_part : p.dv_part) + (key * p.Hkv + kh) * dim + x;
    const int64_t part_stride = (int64_t)p.T * p.Hkv * dim;
    f32x4 acc = *(const f32x4*)src;
    for (int part = 1; part < p.n_split; ++part) {
      const f32x4 v = *(const f32x4*)(src + part * part_stride);
      acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
    }
    uint16_t* dst = is_k ? p.dk + key * p.k_st + (int64_t)kh * p.k_sh + x : p.dv + key * p.v_st + (int64_t)kh * p.v_sh + x;
    *(u32x2*)dst = u32x2{pack_bf16(acc[0], acc[1]), pack_bf16(acc[2], acc[3])};
  }
}

size_t bwd_partial_floats(int T, int Hkv, int g, int dim) {
  const int n_split = heads_split(Hkv, g);
  return n_split > 1 ? (size_t)n_split * (size_t)T * (size_t)Hkv * (size_t)dim : 0;
}

// D[h,r] = sum_x dO[r,h,x] O[r,h,x], LSE2 = LSE*log2(e); resets both scheduler counters.
template <int DV>
__global__ __launch_bounds__(kThreads) void bwd_prepass_kernel(const BwdParams p) {
  constexpr int LPR = DV / 8;  // lanes per (row, head): 16 bytes of O and dO each
  if (blockIdx.x == 0 && threadIdx.x < kNumXcd) {
    p.counter[threadIdx.x * kCounterStride] = 0;
    p.counter_dq[threadIdx.x * kCounterStride] = 0;
  }
  const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t rh = gid / LPR;
  const int part = (int)(gid % LPR);
  const bool valid = rh < (int64_t)p.T * p.Hq;
  float acc = 0.f;
  if (valid) {
    const int64_t r = rh / p.Hq;
    const int h = (int)(rh % p.Hq);
    const int64_t off = r * p.o_st + (int64_t)h * p.o_sh + 8 * part;
    const u32x4 a = *(const u32x4*)(p.o + off);
    const u32x4 b = *(const u32x4*)(p.d_o + off);
#pragma unroll
    for (int i = 0; i < 4; ++i) acc += bf16_lo(a[i]) * bf16_lo(b[i]) + bf16_hi(a[i]) * bf16_hi(b[i]);
  }
#pragma unroll
  for (int m = LPR / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
  if (valid && part == 0) {
    const int64_t r = rh / p.Hq;
    const int h = (int)(rh % p.Hq);
    p.D[(int64_t)h * p.T + r] = acc;
    p.lse2[(int64_t)h * p.T + r] = p.lse[(int64_t)h * p.T + r] * kLog2e;
  }
}

template <int DQK, int DV>
static int launch_bwd_t(const BwdParams& p, int grid_dq, int grid_dkdv, hipStream_t s, hipEvent_t* ev) {
  constexpr int lds_dq = 2 * 64 * (DQK * 2 + DV * 2);
  constexpr int lds_dkdv = 2 * 64 * (DQK * 2 + DV * 2) + 4 * 64 * (int)sizeof(float);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)bwd_dq_kernel<DQK, DV>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_dq);
    if (e != hipSuccess) return (int)e;
    e = hipFuncSetAttribute((const void*)bwd_dkdv_kernel<DQK, DV>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_dkdv);
    if (e != hipSuccess) return (int)e;
    attr_set = true;
  }
  const int64_t pre_threads = (int64_t)p.T * p.Hq * (DV / 8);
  const unsigned pre_grid = (unsigned)((pre_threads + kThreads - 1) / kThreads);
  hipLaunchKernelGGL((bwd_prepass_kernel<DV>), dim3(pre_grid ? pre_grid : 1), dim3(kThreads), 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return (int)e;
  if (grid_dkdv > 0) {
    if (ev[0] && hipEventRecord(ev[0], s) != hipSuccess) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL((bwd_dkdv_kernel<DQK, DV>), dim3(grid_dkdv), dim3(kThreads), lds_dkdv, s, p);
    e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
    if (p.n_split > 1) {
      hipLaunchKernelGGL((bwd_reduce_parts_kernel<DQK, DV>), dim3(p.n_tiles), dim3(kThreads), 0, s, p);
      e = hipGetLastError();
      if (e != hipSuccess) return (int)e;
    }
    if (ev[1] && hipEventRecord(ev[1], s) != hipSuccess) return (int)hipErrorInvalidValue;
  }
  if (grid_dq > 0) {
    if (ev[2] && hipEventRecord(ev[2], s) != hipSuccess) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL((bwd_dq_kernel<DQK, DV>), dim3(grid_dq), dim3(kThreads), lds_dq, s, p);
    e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
    if (ev[3] && hipEventRecord(ev[3], s) != hipSuccess) return (int)hipErrorInvalidValue;
  }
  return (int)e;
}

int launch_bwd(int d_qk, int d_v, const BwdParams& p, int grid_dq, int grid_dkdv, hipStream_t s,
               hipEvent_t* ev) {
  if (d_qk == 64 && d_v == 64) return launch_bwd_t<64, 64>(p, grid_dq, grid_dkdv, s, ev);
  if (d_qk == 128 && d_v == 128) return launch_bwd_t<128, 128>(p, grid_dq, grid_dkdv, s, ev);
  if (d_qk == 192 && d_v == 128) return launch_bwd_t<192, 128>(p, grid_dq, grid_dkdv, s, ev);
  return (int)hipErrorInvalidValue;
}

}  // namespace hbp
