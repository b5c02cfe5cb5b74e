// Forward kernel: causal attention inside each sample of a packed buffer, gfx950.
//
// One work item = (query tile of <=128 rows, query head).  A persistent grid takes items from
// an atomic counter in worklist order (longest causal cost first).  Per item the workgroup
// (4 wavefronts, 32 query rows each) walks the sample's key tiles of 64 keys from the sample
// start to the diagonal:
//   S^T = K Q^T      K tile from LDS (A operand), Q fragments held in registers (B operand);
//                    the accumulator then has one query per lane column, its keys in-lane, so
//                    the row max/sum needs a single exchange with lane^32.
//   P^T -> bf16      used directly as the B operand of the next product (no shuffle);
//   O^T += V^T P^T   V tile kept in its natural [key][dim] layout in LDS and read with the
//                    transposing LDS load, in the key order the accumulator rows have.
// K and V tiles go global -> LDS directly (no staging registers), double buffered, with an XOR
// swizzle of the 16-byte chunks applied on the global side.  exp is taken in base 2 with
// scale*log2(e) folded into one multiplier.
#include "common.hpp"

namespace hbp {

// One key tile (64 keys = two blocks of 32) for one wavefront (32 query rows).  MASKED: the tile
// reaches past the wave's first query row, so the causal compare is applied; interior tiles skip it.
//
// Each 32-key block is one online-softmax step.  The two blocks are software-pipelined inside the
// wave so that the softmax arithmetic of a block is issued, a few instructions at a time, behind the
// MFMAs of the neighbouring product (a vector instruction only overlaps MFMAs of its own wave, and
// only a handful fit behind each):
//     S(0) | S(1) + softmax(0) | PV(0) + softmax(1) | PV(1)
// LDS operand reads run PD fragments ahead of the MFMAs that consume them.  koff / voff are byte
// offsets from `lds` that already contain the current buffer's base.
template <int DQK, int DV, bool MASKED>
__device__ __forceinline__ void fwd_tile(const char* lds, const int (&koff)[DQK / 16],
                                         const int (&voff)[2][DV / 32], const Frag (&qf)[DQK / 16],
                                         f32x16 (&oacc)[DV / 32], float& m_run, float& l_run,
                                         float scale_log2, int k_off, int q_in, int hh) {
  constexpr int KRB = DQK * 2, VRB = DV * 2;
  constexpr int NC = DQK / 16, NEB = DV / 32;
  constexpr int PD = 4;
  constexpr int NSL = 18;  // softmax slices per block: 0 = row max, 1..16 = elements, 17 = drain

  f32x16 s[2];
  Frag pf[2][2];  // [blk][j]
#pragma unroll
  for (int blk = 0; blk < 2; ++blk)
#pragma unroll
    for (int i = 0; i < 16; ++i) s[blk][i] = 0.f;

  auto k_load = [&](int blk) {
    return [&, blk](int c) {
      Frag f;
      f.u = *(const u32x4*)(lds + 32 * blk * KRB + koff[c]);
      return f;
    };
  };
  auto s_mma = [&](int blk) {
    return [&, blk](int c, const Frag& f) { s[blk] = mfma32(f.v, qf[c].v, s[blk]); };
  };
  auto v_load = [&](int blk) {  // step (j, eb), eb fastest
    return [&, blk](int i) {
      const int eb = i % NEB, j = i / NEB;
      const char* base = lds + (32 * blk + 16 * j) * VRB;
      Frag f;
      f.h[0] = lds_read_tr16(base + voff[0][eb]);
      f.h[1] = lds_read_tr16(base + voff[1][eb]);
      return f;
    };
  };
  auto pv_mma = [&](int blk) {
    return [&, blk](int i, const Frag& f) { oacc[i % NEB] = mfma32(f.v, pf[blk][i / NEB].v, oacc[i % NEB]); };
  };

  // softmax of one block, cut in slices.  Elements go through two stages one slice apart (exp of
  // element e next to the sum/pack of element e-1) so no instruction waits on its predecessor.
  float p_cur = 0.f, p_even = 0.f, psum = 0.f, alpha_deferred = 1.f;
  bool rescale_deferred = false;
  auto sm_slice = [&](int blk, int sl, bool defer_o_rescale) {
    if (sl == 0) {
      float mx = -INFINITY;
      // element i holds key k_off + 32 blk + 4 hh + (8 (i>>2) + (i&3)): masked iff that constant
      // exceeds d.  d is kept opaque so the compare stays "constant vs one register" instead of
      // sixteen precomputed per-lane thresholds held across the whole loop.
      int d = q_in - (k_off + 32 * blk + 4 * hh);
      if (MASKED) asm volatile("" : "+v"(d));
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        if (MASKED) {
          if (8 * (i >> 2) + (i & 3) > d) s[blk][i] = -INFINITY;
        }
        mx = fmaxf(mx, s[blk][i]);
      }
      mx = max_with_other_half(mx) * scale_log2;  // scale > 0: max commutes with the scaling
      // Lazy rescale: the running reference m_run only moves when some row's maximum grew by more
      // than 2^8; until then probabilities are taken relative to the old reference (they stay
      // below 2^8, and O and l share the reference, so the result is unchanged).
      if (__builtin_amdgcn_ballot_w64(mx > m_run + 8.0f) != 0) {
        const float m_new = fmaxf(m_run, mx);  // finite: key 0 of the sample is visible to every row
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        l_run *= alpha;
        if (defer_o_rescale) {  // O is being accumulated by MFMAs in flight: scale it after them
          alpha_deferred = alpha;
          rescale_deferred = true;
        } else {
#pragma unroll
          for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[eb][i] *= alpha;
        }
      }
      psum = 0.f;
      return;
    }
    const float p_prev = p_cur;
    if (sl <= 16) {
      const int e = sl - 1;
      p_cur = __builtin_amdgcn_exp2f(__builtin_fmaf(s[blk][e], scale_log2, -m_run));
    }
    if (sl >= 2) {
      const int e = sl - 2;  // element whose exp was issued one slice ago
      psum += p_prev;        // unrounded: LSE must not inherit the bf16 rounding of P
      if (e & 1) pf[blk][e >> 3].w[(e & 7) >> 1] = pack_bf16(p_even, p_prev);
      else p_even = p_prev;
    }
    if (sl == NSL - 1) l_run += psum;
  };

  LdsChain<NC, PD> cs;
  cs.prefill(k_load(0));
  cs.run(k_load(0), s_mma(0));
  cs.prefill(k_load(1));
  cs.template run_with<NSL>(k_load(1), s_mma(1), [&](int sl) { sm_slice(0, sl, false); });
  LdsChain<2 * NEB, PD> cv;
  cv.prefill(v_load(0));
  cv.template run_with<NSL>(v_load(0), pv_mma(0), [&](int sl) { sm_slice(1, sl, true); });
  cv.prefill(v_load(1));
  if (rescale_deferred) {
#pragma unroll
    for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[eb][i] *= alpha_deferred;
  }
  cv.run(v_load(1), pv_mma(1));
}

template <int DQK, int DV>
__global__ __launch_bounds__(kThreads, 2) void fwd_kernel(const FwdParams p) {
  constexpr int BM = 128, BN = 64;
  constexpr int KRB = DQK * 2, VRB = DV * 2;  // bytes per LDS row
  constexpr int K_TILE = BN * KRB, V_TILE = BN * VRB;
  constexpr int NC = DQK / 16;   // contraction chunks of QK^T
  constexpr int NEB = DV / 32;   // 32-wide blocks of the head dim of V

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  // [K buf0][K buf1][V buf0][V buf1]
  char* const k_lds = smem;
  char* const v_lds = smem + 2 * K_TILE;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hh = lane >> 5;

  // per-lane LDS byte offsets of the A operands (row part that does not depend on the 32-key block)
  int koff[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) koff[c] = l32 * KRB + swz<DQK>(2 * c + hh, l32) * 16;
  int voff[2][NEB];
  {
    const int G = lane >> 4, s = lane & 15;
    const int k8 = 4 * hh + (s >> 2);
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int eb = 0; eb < NEB; ++eb) {
        const int c = 4 * eb + 2 * (G & 1) + ((s & 3) >> 1);
        voff[r][eb] = 2 * K_TILE + (8 * r + k8) * VRB + swz<DV>(c, 8 * r + k8) * 16 + (s & 1) * 8;
      }
  }
  TileLoader<DQK, BN> k_loader;
  TileLoader<DV, BN> v_loader;
  k_loader.init(wave, lane);
  v_loader.init(wave, lane);
  const uint32_t k_stride_b = (uint32_t)p.k_st * 2, v_stride_b = (uint32_t)p.v_st * 2;

  uint32_t n_done = 0;
  uint64_t t_first = 0, t_last = 0, t_busy = 0;

  const WorkQueues wq{p.counter, p.n_tiles, p.Hkv, p.g};
  int q_cur = xcc_id_reg() & (kNumXcd - 1), q_tried = 0;
  for (;;) {
    int tile_idx, h;
    if (!next_item(wq, (int*)smem, tid, q_cur, q_tried, tile_idx, h)) break;
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
      ok = s0 >= 0 && s1 <= p.T && s0 <= tl.row_begin && tl.row_begin < tl.row_end &&
           tl.row_end <= s1 && tl.row_end - tl.row_begin <= BM;
    }
    if (ok) {
      const int r0 = tl.row_begin, r1 = tl.row_end;
      const int kh = h / p.g;
      const int qw0 = r0 - s0 + 32 * wave;  // in-sample index of this wave's first query
      const int my_row = r0 + 32 * wave + l32;
      const bool row_valid = my_row < r1;
      const bool wave_active = r0 + 32 * wave < r1;

      const int n_keys = r1 - s0;  // keys 0..n_keys-1 (in-sample) are needed by this tile
      const int nkt = (n_keys + BN - 1) / BN;
      const uint16_t* kbase = p.k + (int64_t)s0 * p.k_st + (int64_t)kh * p.k_sh;
      const uint16_t* vbase = p.v + (int64_t)s0 * p.v_st + (int64_t)kh * p.v_sh;

      auto issue = [&](int kt) {
        const int k_off = kt * BN;
        const int valid = n_keys - k_off;  // >= 1
        k_loader.issue(kbase + (int64_t)k_off * p.k_st, k_stride_b, valid, k_lds + (kt & 1) * K_TILE, wave);
        v_loader.issue(vbase + (int64_t)k_off * p.v_st, v_stride_b, valid, v_lds + (kt & 1) * V_TILE, wave);
      };
      issue(0);

      // Q fragments (B operand of S^T = K Q^T): lane holds query l32, dims 16c+8hh..+7
      Frag qf[NC];
      {
        const uint16_t* qp = p.q + (int64_t)my_row * p.q_st + (int64_t)h * p.q_sh + 8 * hh;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          if (row_valid) qf[c].u = *(const u32x4*)(qp + 16 * c);
          else qf[c].u = u32x4{0, 0, 0, 0};
        }
      }

      f32x16 oacc[NEB];
#pragma unroll
      for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[eb][i] = 0.f;
      float m_run = -INFINITY, l_run = 0.f;
      const int q_in = qw0 + l32;

      int cur_buf = 0;
      auto point_offsets_at = [&](int buf) {  // move every LDS offset to the other buffer
        const int dk = buf ? K_TILE : -K_TILE, dv = buf ? V_TILE : -V_TILE;
#pragma unroll
        for (int c = 0; c < NC; ++c) koff[c] += dk;
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
          for (int eb = 0; eb < NEB; ++eb) voff[r][eb] += dv;
        cur_buf = buf;
      };
      auto begin_tile = [&](int kt) {
        wait_async_loads();
        __syncthreads();  // tile kt has landed for every wave; tile kt-1 is no longer read
        if (kt + 1 < nkt) issue(kt + 1);
        if ((kt & 1) != cur_buf) point_offsets_at(kt & 1);
      };
      // Interior tiles (entirely below this wave's first query row) and diagonal tiles run in two
      // separate loops, one code variant each; every wave still passes nkt barriers in total.
      const int n_interior = wave_active ? min(nkt, (qw0 + 1) / BN) : 0;
      int kt = 0;
      for (; kt < n_interior; ++kt) {
        begin_tile(kt);
        fwd_tile<DQK, DV, false>(smem, koff, voff, qf, oacc, m_run, l_run, p.scale_log2, kt * BN, q_in, hh);
      }
      for (; kt < nkt; ++kt) {
        begin_tile(kt);
        if (wave_active && kt * BN <= qw0 + 31)  // else: nothing at or below the diagonal
          fwd_tile<DQK, DV, true>(smem, koff, voff, qf, oacc, m_run, l_run, p.scale_log2, kt * BN, q_in, hh);
      }
      if (cur_buf) point_offsets_at(0);

      // finalise: O = acc / l, LSE = (m + log2 l) * ln 2
      const float l_tot = l_run + xor32(l_run);
      if (row_valid) {
        const float inv = 1.f / l_tot;
        uint16_t* op = p.o + (int64_t)my_row * p.o_st + (int64_t)h * p.o_sh + 4 * hh;
#pragma unroll
        for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            u32x2 w = {pack_bf16(oacc[eb][4 * b] * inv, oacc[eb][4 * b + 1] * inv),
                       pack_bf16(oacc[eb][4 * b + 2] * inv, oacc[eb][4 * b + 3] * inv)};
            *(u32x2*)(op + 32 * eb + 8 * b) = w;
          }
        if (hh == 0)
          p.lse[(int64_t)h * p.T + my_row] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
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

template <int DQK, int DV>
static int launch_fwd_t(const FwdParams& p, int grid, hipStream_t s) {
  constexpr int lds_bytes = 2 * 64 * (DQK * 2 + DV * 2);
  static bool attr_set = false;
  if (!attr_set) {
    const hipError_t e = hipFuncSetAttribute((const void*)fwd_kernel<DQK, DV>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return (int)e;
    attr_set = true;
  }
  hipLaunchKernelGGL((fwd_kernel<DQK, DV>), dim3(grid), dim3(kThreads), lds_bytes, s, p);
  return (int)hipGetLastError();
}

int launch_fwd(int d_qk, int d_v, const FwdParams& p, int grid, hipStream_t s, hipEvent_t ev0,
               hipEvent_t ev1) {
  if (ev0 && hipEventRecord(ev0, s) != hipSuccess) return (int)hipErrorInvalidValue;
  int e;
  if (d_qk == 64 && d_v == 64) e = launch_fwd_t<64, 64>(p, grid, s);
  else if (d_qk == 128 && d_v == 128) e = launch_fwd_t<128, 128>(p, grid, s);
  else if (d_qk == 192 && d_v == 128) e = launch_fwd_t<192, 128>(p, grid, s);
  else return (int)hipErrorInvalidValue;
  if (e == 0 && ev1 && hipEventRecord(ev1, s) != hipSuccess) return (int)hipErrorInvalidValue;
  return e;
}

}  // namespace hbp
