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

// One key tile (64 keys) for one wavefront (32 query rows).  MASKED: the tile reaches past the
// wave's first query row, so the causal compare is applied; interior tiles skip it entirely.
// LDS operand reads run PD fragments ahead of the MFMAs that consume them.
template <int DQK, int DV, bool MASKED>
__device__ __forceinline__ void fwd_tile(const char* kt_lds, const char* vt_lds, const int (&koff)[DQK / 16],
                                         const int (&voff)[2][DV / 32], const Frag (&qf)[DQK / 16],
                                         f32x16 (&oacc)[DV / 32], float& m_run, float& l_run,
                                         float scale_log2, int k_off, int q_in, int hh) {
  constexpr int KRB = DQK * 2, VRB = DV * 2;
  constexpr int NC = DQK / 16, NEB = DV / 32;
  constexpr int PD = 4;

  f32x16 sacc[2];
#pragma unroll
  for (int blk = 0; blk < 2; ++blk)
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[blk][i] = 0.f;
  {
    constexpr int L = 2 * NC;
    Frag ring[PD];
#pragma unroll
    for (int i = 0; i < PD; ++i) ring[i].u = *(const u32x4*)(kt_lds + 32 * (i / NC) * KRB + koff[i % NC]);
#pragma unroll
    for (int i = 0; i < L; ++i) {
      sacc[i / NC] = mfma32(ring[i % PD].v, qf[i % NC].v, sacc[i / NC]);
      if (i + PD < L)
        ring[i % PD].u = *(const u32x4*)(kt_lds + 32 * ((i + PD) / NC) * KRB + koff[(i + PD) % NC]);
      __builtin_amdgcn_sched_barrier(0);  // keep the read-ahead distance: no hoisting of later reads
    }
  }
  // first V fragments: their LDS latency hides under the softmax arithmetic
  constexpr int LV = 4 * NEB;  // steps (blk, j, eb), eb fastest
  Frag vring[PD];
  auto load_v = [&](int i) {
    const int eb = i % NEB, bj = i / NEB;  // bj = 2*blk + j
    const char* base = vt_lds + 16 * bj * VRB;
    Frag f;
    f.h[0] = lds_read_tr16(base + voff[0][eb]);
    f.h[1] = lds_read_tr16(base + voff[1][eb]);
    return f;
  };
#pragma unroll
  for (int i = 0; i < PD; ++i) vring[i] = load_v(i);
  __builtin_amdgcn_sched_barrier(0);

  float mx = -INFINITY;
#pragma unroll
  for (int blk = 0; blk < 2; ++blk)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (MASKED) {
        const int key_in = k_off + 32 * blk + 8 * (i >> 2) + 4 * hh + (i & 3);
        if (key_in > q_in) sacc[blk][i] = -INFINITY;
      }
      mx = fmaxf(mx, sacc[blk][i]);
    }
  mx = max_with_other_half(mx) * scale_log2;  // scale > 0: max commutes with the scaling
  // Lazy rescale: the running reference m_run only moves when some row's maximum grew by more
  // than 2^8; until then probabilities are taken relative to the old reference (they stay below
  // 2^8, exact in fp32/bf16 range, and O and l use the same reference so the result is unchanged).
  if (__builtin_amdgcn_ballot_w64(mx > m_run + 8.0f) != 0) {
    const float m_new = fmaxf(m_run, mx);  // finite: key 0 of the sample is visible to every row
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    l_run *= alpha;
#pragma unroll
    for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[eb][i] *= alpha;
  }
  Frag pf[4];  // index 2*blk + j
  float psum = 0.f;
#pragma unroll
  for (int blk = 0; blk < 2; ++blk)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[blk][8 * j + 2 * w], scale_log2, -m_run));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[blk][8 * j + 2 * w + 1], scale_log2, -m_run));
        pf[2 * blk + j].w[w] = pack_bf16(p0, p1);
        psum += p0 + p1;  // unrounded: LSE must not inherit the bf16 rounding of P
      }
  l_run += psum;
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < LV; ++i) {
    oacc[i % NEB] = mfma32(vring[i % PD].v, pf[i / NEB].v, oacc[i % NEB]);
    if (i + PD < LV) vring[i % PD] = load_v(i + PD);
    __builtin_amdgcn_sched_barrier(0);
  }
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
        voff[r][eb] = (8 * r + k8) * VRB + swz<DV>(c, 8 * r + k8) * 16 + (s & 1) * 8;
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

      for (int kt = 0; kt < nkt; ++kt) {
        wait_async_loads();
        __syncthreads();  // tile kt has landed for every wave; tile kt-1 is no longer read
        if (kt + 1 < nkt) issue(kt + 1);

        const int k_off = kt * BN;
        if (!wave_active || k_off > qw0 + 31) continue;  // nothing at or below the diagonal
        const char* kt_lds = k_lds + (kt & 1) * K_TILE;
        const char* vt_lds = v_lds + (kt & 1) * V_TILE;
        if (k_off + BN - 1 > qw0)
          fwd_tile<DQK, DV, true>(kt_lds, vt_lds, koff, voff, qf, oacc, m_run, l_run, p.scale_log2, k_off, q_in, hh);
        else
          fwd_tile<DQK, DV, false>(kt_lds, vt_lds, koff, voff, qf, oacc, m_run, l_run, p.scale_log2, k_off, q_in, hh);
      }

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
