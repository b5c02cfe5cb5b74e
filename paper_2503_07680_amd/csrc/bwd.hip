// Backward kernels: dQ, dK, dV of causal attention inside each sample of a packed buffer.
//
// (1) prepass:  D[h,r] = sum_x dO[r,h,x] O[r,h,x]  and zeroing of the fp32 dQ accumulator.
// (2) main:     one work item = (key tile of <=128 keys, kv head), served longest cost first by
//               a persistent grid.  Each of the 4 wavefronts owns 32 keys: their K and V
//               fragments and the dK^T / dV^T accumulators stay in registers while the
//               workgroup walks the query blocks (32 rows) at or below the diagonal, for every
//               query head of the kv head's group.  Per block and wavefront, five MFMA products:
//                   S  = Q K^T            (accumulator: one key per lane column, queries in-lane)
//                   dP = dO V^T
//                   P  = exp2(S*c - LSE*log2e),  dS = P (dP - D)
//                   dV^T += dO^T P        (P taken straight from the accumulator as B operand)
//                   dK^T += Q^T dS
//                   dQ   += dS K          (dS transposed through a per-wave LDS patch)
//               dQ partial sums go to the fp32 accumulator with hardware float atomics.
// (3) convert:  dQ = bf16(scale * accumulator).
#include "common.hpp"

namespace hbp {

template <int DQK, int DV>
__global__ __launch_bounds__(kThreads, 1) void bwd_kernel(const BwdParams p) {
  constexpr int BN = 128, BQ = 32;
  constexpr int NC = DQK / 16, NCV = DV / 16;   // contraction chunks of S and dP
  constexpr int NDB = DQK / 32, NEB = DV / 32;  // 32-wide output blocks of dK/dQ and dV
  constexpr int QP = DQK + 8, OP = DV + 8;      // pitches of the natural Q / dO blocks
  constexpr int TP = BQ + 8;                    // pitch of the transposed blocks and of dS
  constexpr int Q_UNITS = (BQ / 4) * (DQK / 2) / kThreads;
  constexpr int O_UNITS = (BQ / 4) * (DV / 2) / kThreads;

  __shared__ __attribute__((aligned(16))) uint16_t Qs[BQ * QP];
  __shared__ __attribute__((aligned(16))) uint16_t dOs[BQ * OP];
  __shared__ __attribute__((aligned(16))) uint16_t Qt[DQK * TP];
  __shared__ __attribute__((aligned(16))) uint16_t dOt[DV * TP];
  __shared__ __attribute__((aligned(16))) uint16_t dSs[4 * BQ * TP];
  __shared__ __attribute__((aligned(16))) float lse_s[BQ];
  __shared__ __attribute__((aligned(16))) float D_s[BQ];
  __shared__ int s_item;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hh = lane >> 5;
  constexpr float kLog2e = 1.4426950408889634f;

  uint32_t n_done = 0;
  uint64_t t_first = 0, t_last = 0, t_busy = 0;

  for (;;) {
    if (tid == 0) s_item = atomicAdd(p.counter, 1);
    __syncthreads();
    const int item = s_item;
    __syncthreads();
    if (item >= p.n_tiles * p.Hkv) break;
    uint64_t t0 = 0;
    if (p.prof && tid == 0) {
      t0 = wall_clock64();
      if (n_done == 0) t_first = t0;
    }

    const int kh = item % p.Hkv;
    const hbp_tile tl = p.tiles[item / p.Hkv];
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
      const int k0_in = tl.row_begin - s0;             // in-sample index of the tile's first key
      const int kw0_in = k0_in + 32 * wave;            // ... of this wave's first key
      const int my_key = tl.row_begin + 32 * wave + l32;  // absolute row of this lane's key column
      const bool key_valid = my_key < tl.row_end;
      const bool wave_active = tl.row_begin + 32 * wave < tl.row_end;

      // register-resident operands of this wave's 32 keys
      Frag knat[NC], vnat[NCV], ktr[NDB][2];
      {
        const uint16_t* kp = p.k + (int64_t)my_key * p.k_st + (int64_t)kh * p.k_sh + 8 * hh;
        const uint16_t* vp = p.v + (int64_t)my_key * p.v_st + (int64_t)kh * p.v_sh + 8 * hh;
#pragma unroll
        for (int c = 0; c < NC; ++c) knat[c].u = key_valid ? *(const u32x4*)(kp + 16 * c) : u32x4{0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < NCV; ++c) vnat[c].u = key_valid ? *(const u32x4*)(vp + 16 * c) : u32x4{0, 0, 0, 0};
        // B operand of dQ = dS K: lane column d = 32db + l32, contraction rows = keys 16j+8hh+i
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
              const int key_a = tl.row_begin + 32 * wave + 16 * j + 8 * hh + 2 * w;
              const uint16_t* ka = p.k + (int64_t)key_a * p.k_st + (int64_t)kh * p.k_sh + 32 * db + l32;
              const uint32_t lo = key_a < tl.row_end ? (uint32_t)ka[0] : 0u;
              const uint32_t hi = key_a + 1 < tl.row_end ? (uint32_t)ka[p.k_st] : 0u;
              ktr[db][j].w[w] = lo | (hi << 16);
            }
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

      const int qb_start = (k0_in / BQ) * BQ;
      const int nqb = (s_len - qb_start + BQ - 1) / BQ;  // query blocks per head
      const int n_steps = nqb * p.g;

      uint32_t qreg[Q_UNITS][4], oreg[O_UNITS][4];
      float lse_reg = 0.f, D_reg = 0.f;

      auto load_block = [&](int step) {
        const int hq = kh * p.g + step / nqb;
        const int qb = qb_start + (step % nqb) * BQ;
        const uint16_t* qb_ptr = p.q + (int64_t)(s0 + qb) * p.q_st + (int64_t)hq * p.q_sh;
        const uint16_t* ob_ptr = p.d_o + (int64_t)(s0 + qb) * p.o_st + (int64_t)hq * p.o_sh;
#pragma unroll
        for (int i = 0; i < Q_UNITS; ++i) {
          const int u = tid + kThreads * i;
          const int cp = u % (DQK / 2), rg = u / (DQK / 2);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int row = 4 * rg + j;
            qreg[i][j] = qb + row < s_len ? *(const uint32_t*)(qb_ptr + (int64_t)row * p.q_st + 2 * cp) : 0u;
          }
        }
#pragma unroll
        for (int i = 0; i < O_UNITS; ++i) {
          const int u = tid + kThreads * i;
          const int cp = u % (DV / 2), rg = u / (DV / 2);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int row = 4 * rg + j;
            oreg[i][j] = qb + row < s_len ? *(const uint32_t*)(ob_ptr + (int64_t)row * p.o_st + 2 * cp) : 0u;
          }
        }
        if (tid < BQ) {
          const bool v = qb + tid < s_len;
          // +inf for rows past the sample end makes their probabilities exactly zero
          lse_reg = v ? p.lse[(int64_t)hq * p.T + s0 + qb + tid] * kLog2e : INFINITY;
          D_reg = v ? p.D[(int64_t)hq * p.T + s0 + qb + tid] : 0.f;
        }
      };
      auto store_block = [&]() {
#pragma unroll
        for (int i = 0; i < Q_UNITS; ++i) {
          const int u = tid + kThreads * i;
          const int cp = u % (DQK / 2), rg = u / (DQK / 2);
          const int pos = 16 * (rg >> 2) + tslot(4 * (rg & 3));
          const uint32_t a0 = qreg[i][0], a1 = qreg[i][1], a2 = qreg[i][2], a3 = qreg[i][3];
#pragma unroll
          for (int j = 0; j < 4; ++j) *(uint32_t*)&Qs[(4 * rg + j) * QP + 2 * cp] = qreg[i][j];
          u32x2 lo = {(a0 & 0xffffu) | (a1 << 16), (a2 & 0xffffu) | (a3 << 16)};
          u32x2 hi = {(a0 >> 16) | (a1 & 0xffff0000u), (a2 >> 16) | (a3 & 0xffff0000u)};
          *(u32x2*)&Qt[(2 * cp) * TP + pos] = lo;
          *(u32x2*)&Qt[(2 * cp + 1) * TP + pos] = hi;
        }
#pragma unroll
        for (int i = 0; i < O_UNITS; ++i) {
          const int u = tid + kThreads * i;
          const int cp = u % (DV / 2), rg = u / (DV / 2);
          const int pos = 16 * (rg >> 2) + tslot(4 * (rg & 3));
          const uint32_t a0 = oreg[i][0], a1 = oreg[i][1], a2 = oreg[i][2], a3 = oreg[i][3];
#pragma unroll
          for (int j = 0; j < 4; ++j) *(uint32_t*)&dOs[(4 * rg + j) * OP + 2 * cp] = oreg[i][j];
          u32x2 lo = {(a0 & 0xffffu) | (a1 << 16), (a2 & 0xffffu) | (a3 << 16)};
          u32x2 hi = {(a0 >> 16) | (a1 & 0xffff0000u), (a2 >> 16) | (a3 & 0xffff0000u)};
          *(u32x2*)&dOt[(2 * cp) * TP + pos] = lo;
          *(u32x2*)&dOt[(2 * cp + 1) * TP + pos] = hi;
        }
        if (tid < BQ) {
          lse_s[tid] = lse_reg;
          D_s[tid] = D_reg;
        }
      };

      uint16_t* my_dS = dSs + wave * BQ * TP;

      if (n_steps > 0) load_block(0);
      for (int step = 0; step < n_steps; ++step) {
        __syncthreads();
        store_block();
        __syncthreads();
        const int hq = kh * p.g + step / nqb;
        const int qb = qb_start + (step % nqb) * BQ;
        if (step + 1 < n_steps) load_block(step + 1);
        if (!wave_active || qb + BQ - 1 < kw0_in) continue;  // block lies above this wave's keys

        f32x16 sacc, dpacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.f, dpacc[i] = 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          Frag a;
          a.u = *(const u32x4*)&Qs[l32 * QP + 16 * c + 8 * hh];
          sacc = mfma32(a.v, knat[c].v, sacc);
        }
#pragma unroll
        for (int c = 0; c < NCV; ++c) {
          Frag a;
          a.u = *(const u32x4*)&dOs[l32 * OP + 16 * c + 8 * hh];
          dpacc = mfma32(a.v, vnat[c].v, dpacc);
        }
        // accumulator element 4b+v <-> query row qb + 8b + 4hh + v, key column kw0_in + l32
        const bool need_mask = kw0_in + 31 > qb;
        const int key_in = kw0_in + l32;
        Frag pb[2], dsb[2];
        float dsv[16];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const f32x4 l4 = *(const f32x4*)&lse_s[8 * b + 4 * hh];
          const f32x4 d4 = *(const f32x4*)&D_s[8 * b + 4 * hh];
          float pv[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            float pr = __builtin_amdgcn_exp2f(sacc[4 * b + v] * p.scale_log2 - l4[v]);
            if (need_mask && key_in > qb + 8 * b + 4 * hh + v) pr = 0.f;
            pv[v] = pr;
            dsv[4 * b + v] = pr * (dpacc[4 * b + v] - d4[v]);
          }
          pb[b >> 1].w[2 * (b & 1)] = pack_bf16(pv[0], pv[1]);
          pb[b >> 1].w[2 * (b & 1) + 1] = pack_bf16(pv[2], pv[3]);
          dsb[b >> 1].w[2 * (b & 1)] = pack_bf16(dsv[4 * b], dsv[4 * b + 1]);
          dsb[b >> 1].w[2 * (b & 1) + 1] = pack_bf16(dsv[4 * b + 2], dsv[4 * b + 3]);
        }
        // dV^T += dO^T P ; dK^T += Q^T dS  (contraction over the 32 query rows, two chunks of 16)
#pragma unroll
        for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            Frag a;
            a.u = *(const u32x4*)&dOt[(32 * eb + l32) * TP + 16 * j + 8 * hh];
            dvt[eb] = mfma32(a.v, pb[j].v, dvt[eb]);
          }
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            Frag a;
            a.u = *(const u32x4*)&Qt[(32 * db + l32) * TP + 16 * j + 8 * hh];
            dkt[db] = mfma32(a.v, dsb[j].v, dkt[db]);
          }
        // transpose dS through this wave's LDS patch: [query][key]
#pragma unroll
        for (int b = 0; b < 4; ++b) {
#pragma unroll
          for (int v = 0; v < 4; v += 2) {
            const uint32_t w = dsb[b >> 1].w[2 * (b & 1) + (v >> 1)];
            my_dS[(8 * b + 4 * hh + v) * TP + l32] = (uint16_t)(w & 0xffffu);
            my_dS[(8 * b + 4 * hh + v + 1) * TP + l32] = (uint16_t)(w >> 16);
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // dQ[q, d] += sum_key dS[q,key] K[key,d]
        float* dq_row = p.dq_acc + ((int64_t)(s0 + qb) * p.Hq + hq) * DQK + l32;
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          f32x16 dq;
#pragma unroll
          for (int i = 0; i < 16; ++i) dq[i] = 0.f;
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            Frag a;
            a.u = *(const u32x4*)&my_dS[l32 * TP + 16 * j + 8 * hh];
            dq = mfma32(a.v, ktr[db][j].v, dq);
          }
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int row = 8 * (i >> 2) + 4 * hh + (i & 3);
            if (qb + row < s_len)
              unsafeAtomicAdd(dq_row + (int64_t)row * p.Hq * DQK + 32 * db, dq[i]);
          }
        }
        __builtin_amdgcn_wave_barrier();
      }

      // store dK = scale * dK^T^T, dV = dV^T^T : lane column = key, 4 consecutive dims per element group
      if (key_valid) {
        uint16_t* dkp = p.dk + (int64_t)my_key * p.k_st + (int64_t)kh * p.k_sh + 4 * hh;
        uint16_t* dvp = p.dv + (int64_t)my_key * p.v_st + (int64_t)kh * p.v_sh + 4 * hh;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            u32x2 w = {pack_bf16(dkt[db][4 * b] * p.scale, dkt[db][4 * b + 1] * p.scale),
                       pack_bf16(dkt[db][4 * b + 2] * p.scale, dkt[db][4 * b + 3] * p.scale)};
            *(u32x2*)(dkp + 32 * db + 8 * b) = w;
          }
#pragma unroll
        for (int eb = 0; eb < NEB; ++eb)
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            u32x2 w = {pack_bf16(dvt[eb][4 * b], dvt[eb][4 * b + 1]),
                       pack_bf16(dvt[eb][4 * b + 2], dvt[eb][4 * b + 3])};
            *(u32x2*)(dvp + 32 * eb + 8 * b) = w;
          }
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

// D[h,r] = sum_x dO[r,h,x] O[r,h,x]; zero the fp32 dQ accumulator row (r,h); reset the counter.
template <int DQK, int DV>
__global__ __launch_bounds__(kThreads) void bwd_prepass_kernel(const BwdParams p) {
  constexpr int LPR = DV / 8;          // lanes per (row, head): 16 bytes of O and dO each
  constexpr int ZPL = DQK / LPR;       // accumulator floats zeroed per lane
  if (blockIdx.x == 0 && threadIdx.x == 0) *p.counter = 0;
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
    float* z = p.dq_acc + rh * DQK + (int64_t)part * ZPL;
#pragma unroll
    for (int i = 0; i < ZPL; i += 4) *(f32x4*)(z + i) = f32x4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int m = LPR / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
  if (valid && part == 0) {
    const int64_t r = rh / p.Hq;
    const int h = (int)(rh % p.Hq);
    p.D[(int64_t)h * p.T + r] = acc;
  }
}

// dQ = bf16(scale * accumulator)
template <int DQK>
__global__ __launch_bounds__(kThreads) void bwd_convert_kernel(const BwdParams p) {
  constexpr int CPR = DQK / 8;  // 8-element chunks per (row, head)
  const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t rh = gid / CPR;
  const int part = (int)(gid % CPR);
  if (rh >= (int64_t)p.T * p.Hq) return;
  const int64_t r = rh / p.Hq;
  const int h = (int)(rh % p.Hq);
  const float* a = p.dq_acc + rh * DQK + 8 * part;
  const f32x4 x = *(const f32x4*)a, y = *(const f32x4*)(a + 4);
  u32x4 w = {pack_bf16(x[0] * p.scale, x[1] * p.scale), pack_bf16(x[2] * p.scale, x[3] * p.scale),
             pack_bf16(y[0] * p.scale, y[1] * p.scale), pack_bf16(y[2] * p.scale, y[3] * p.scale)};
  *(u32x4*)(p.dq + r * p.q_st + (int64_t)h * p.q_sh + 8 * part) = w;
}

template <int DQK, int DV>
static int launch_bwd_t(const BwdParams& p, int grid, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
  const int64_t rh = (int64_t)p.T * p.Hq;
  const int64_t pre_threads = rh * (DV / 8);
  const int64_t cvt_threads = rh * (DQK / 8);
  const unsigned pre_grid = (unsigned)((pre_threads + kThreads - 1) / kThreads);
  const unsigned cvt_grid = (unsigned)((cvt_threads + kThreads - 1) / kThreads);
  hipLaunchKernelGGL((bwd_prepass_kernel<DQK, DV>), dim3(pre_grid ? pre_grid : 1), dim3(kThreads), 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return (int)e;
  if (grid > 0) {
    if (ev0 && hipEventRecord(ev0, s) != hipSuccess) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL((bwd_kernel<DQK, DV>), dim3(grid), dim3(kThreads), 0, s, p);
    e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
    if (ev1 && hipEventRecord(ev1, s) != hipSuccess) return (int)hipErrorInvalidValue;
  }
  if (cvt_grid > 0) {
    hipLaunchKernelGGL((bwd_convert_kernel<DQK>), dim3(cvt_grid), dim3(kThreads), 0, s, p);
    e = hipGetLastError();
  }
  return (int)e;
}

int launch_bwd(int d_qk, int d_v, const BwdParams& p, int grid, hipStream_t s, hipEvent_t ev0,
               hipEvent_t ev1) {
  if (d_qk == 64 && d_v == 64) return launch_bwd_t<64, 64>(p, grid, s, ev0, ev1);
  if (d_qk == 128 && d_v == 128) return launch_bwd_t<128, 128>(p, grid, s, ev0, ev1);
  if (d_qk == 192 && d_v == 128) return launch_bwd_t<192, 128>(p, grid, s, ev0, ev1);
  return (int)hipErrorInvalidValue;
}

}  // namespace hbp
