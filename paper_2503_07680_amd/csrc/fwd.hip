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
//   O^T += V^T P^T   V tile stored transposed in LDS with the contraction index permuted to
//                    match the accumulator's row order.
// exp is taken in base 2 with scale*log2(e) folded into one multiplier.
#include "common.hpp"

namespace hbp {

template <int DQK, int DV>
__global__ __launch_bounds__(kThreads, (DQK <= 64 ? 2 : 1)) void fwd_kernel(const FwdParams p) {
  constexpr int BM = 128, BN = 64;
  constexpr int KP = DQK + 8;                        // LDS pitch of a K row (elements)
  constexpr int VP = BN + 8;                         // LDS pitch of a V^T row
  constexpr int NC = DQK / 16;                       // contraction chunks of QK^T
  constexpr int NEB = DV / 32;                       // 32-wide blocks of the head dim of V
  constexpr int K_PIECES = BN * (DQK / 8) / kThreads;  // 16-byte pieces per thread
  constexpr int V_UNITS = (BN / 4) * (DV / 2) / kThreads;  // (4 keys x 2 cols) units per thread

  __shared__ __attribute__((aligned(16))) uint16_t Ks[BN * KP];
  __shared__ __attribute__((aligned(16))) uint16_t Vt[DV * VP];
  __shared__ int s_item;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hh = lane >> 5;

  uint32_t n_done = 0;
  uint64_t t_first = 0, t_last = 0, t_busy = 0;

  for (;;) {
    if (tid == 0) s_item = atomicAdd(p.counter, 1);
    __syncthreads();
    const int item = s_item;
    __syncthreads();
    if (item >= p.n_tiles * p.Hq) break;
    uint64_t t0 = 0;
    if (p.prof && tid == 0) {
      t0 = wall_clock64();
      if (n_done == 0) t_first = t0;
    }

    const int h = item % p.Hq;
    const hbp_tile tl = p.tiles[item / p.Hq];
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

      const int n_keys = r1 - s0;  // keys 0..n_keys-1 (in-sample) are needed by this tile
      const int nkt = (n_keys + BN - 1) / BN;
      const uint16_t* kbase = p.k + (int64_t)s0 * p.k_st + (int64_t)kh * p.k_sh;
      const uint16_t* vbase = p.v + (int64_t)s0 * p.v_st + (int64_t)kh * p.v_sh;

      u32x4 kreg[K_PIECES];
      uint32_t vreg[V_UNITS][4];

      auto load_tile = [&](int kt) {
        const int k_off = kt * BN;
#pragma unroll
        for (int i = 0; i < K_PIECES; ++i) {
          const int pi = tid + kThreads * i;
          const int row = pi / (DQK / 8), c8 = pi % (DQK / 8);
          if (k_off + row < n_keys)
            kreg[i] = *(const u32x4*)(kbase + (int64_t)(k_off + row) * p.k_st + 8 * c8);
          else
            kreg[i] = u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < V_UNITS; ++i) {
          const int u = tid + kThreads * i;
          const int cp = u % (DV / 2), rg = u / (DV / 2);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int row = k_off + 4 * rg + j;
            vreg[i][j] = row < n_keys ? *(const uint32_t*)(vbase + (int64_t)row * p.v_st + 2 * cp) : 0u;
          }
        }
      };
      auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < K_PIECES; ++i) {
          const int pi = tid + kThreads * i;
          const int row = pi / (DQK / 8), c8 = pi % (DQK / 8);
          *(u32x4*)&Ks[row * KP + 8 * c8] = kreg[i];
        }
#pragma unroll
        for (int i = 0; i < V_UNITS; ++i) {
          const int u = tid + kThreads * i;
          const int cp = u % (DV / 2), rg = u / (DV / 2);
          const int pos = 16 * (rg >> 2) + tslot(4 * (rg & 3));
          const uint32_t a0 = vreg[i][0], a1 = vreg[i][1], a2 = vreg[i][2], a3 = vreg[i][3];
          u32x2 lo = {(a0 & 0xffffu) | (a1 << 16), (a2 & 0xffffu) | (a3 << 16)};
          u32x2 hi = {(a0 >> 16) | (a1 & 0xffff0000u), (a2 >> 16) | (a3 & 0xffff0000u)};
          *(u32x2*)&Vt[(2 * cp) * VP + pos] = lo;
          *(u32x2*)&Vt[(2 * cp + 1) * VP + pos] = hi;
        }
      };

      load_tile(0);
      for (int kt = 0; kt < nkt; ++kt) {
        __syncthreads();  // every wave is done reading the previous tile
        store_tile();
        __syncthreads();
        if (kt + 1 < nkt) load_tile(kt + 1);  // in flight while this tile is computed

        const int k_off = kt * BN;
        if (!wave_active || k_off > qw0 + 31) continue;  // nothing at or below the diagonal

        f32x16 sacc[2];
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[blk][i] = 0.f;
#pragma unroll
          for (int c = 0; c < NC; ++c) {
            Frag kf;
            kf.u = *(const u32x4*)&Ks[(32 * blk + l32) * KP + 16 * c + 8 * hh];
            sacc[blk] = mfma32(kf.v, qf[c].v, sacc[blk]);
          }
        }
        // scale into the base-2 domain, causal mask on tiles that reach past the wave's first row
        const bool need_mask = k_off + BN - 1 > qw0;
        const int q_in = qw0 + l32;
        float mx = -INFINITY;
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            float x = sacc[blk][i] * p.scale_log2;
            if (need_mask) {
              const int key_in = k_off + 32 * blk + 8 * (i >> 2) + 4 * hh + (i & 3);
              if (key_in > q_in) x = -INFINITY;
            }
            sacc[blk][i] = x;
            mx = fmaxf(mx, x);
          }
        mx = fmaxf(mx, xor32(mx));
        const float m_new = fmaxf(m_run, mx);  // finite: key 0 of the sample is visible to every row
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
        Frag pf[2][2];
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
              const float p0 = __builtin_amdgcn_exp2f(sacc[blk][8 * j + 2 * w] - m_new);
              const float p1 = __builtin_amdgcn_exp2f(sacc[blk][8 * j + 2 * w + 1] - m_new);
              psum += p0 + p1;
              pf[blk][j].w[w] = pack_bf16(p0, p1);
            }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[eb][i] *= alpha;
#pragma unroll
        for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
          for (int blk = 0; blk < 2; ++blk)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
              Frag vf;
              vf.u = *(const u32x4*)&Vt[(32 * eb + l32) * VP + 32 * blk + 16 * j + 8 * hh];
              oacc[eb] = mfma32(vf.v, pf[blk][j].v, oacc[eb]);
            }
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

__global__ void zero_counter_kernel(int32_t* c) {
  if (threadIdx.x == 0) *c = 0;
}

int launch_zero_counter(int32_t* counter, hipStream_t s) {
  hipLaunchKernelGGL(zero_counter_kernel, dim3(1), dim3(64), 0, s, counter);
  return (int)hipGetLastError();
}

int launch_fwd(int d_qk, int d_v, const FwdParams& p, int grid, hipStream_t s, hipEvent_t ev0,
               hipEvent_t ev1) {
  if (ev0 && hipEventRecord(ev0, s) != hipSuccess) return (int)hipErrorInvalidValue;
  if (d_qk == 64 && d_v == 64)
    hipLaunchKernelGGL((fwd_kernel<64, 64>), dim3(grid), dim3(kThreads), 0, s, p);
  else if (d_qk == 128 && d_v == 128)
    hipLaunchKernelGGL((fwd_kernel<128, 128>), dim3(grid), dim3(kThreads), 0, s, p);
  else if (d_qk == 192 && d_v == 128)
    hipLaunchKernelGGL((fwd_kernel<192, 128>), dim3(grid), dim3(kThreads), 0, s, p);
  else
    return (int)hipErrorInvalidValue;
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess && ev1 && hipEventRecord(ev1, s) != hipSuccess) return (int)hipErrorInvalidValue;
  return (int)e;
}

}  // namespace hbp
