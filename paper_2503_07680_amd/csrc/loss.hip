// Packed cross-entropy with the paper's loss normalisers (Section 4.3, normaliser equation), forward
// and backward in one pass over the logits, gfx950.
//
//   token loss      CE_r = logsumexp(z_r) - z_r[label_r]                     (rows with label < 0: none)
//   loss            sum_r w_r CE_r,  w_r by normaliser: token-mean 1 / sum_i T_i, sample-mean
//                   1 / (T_i B_l) for the row's sample i, stable 1 / (B_l T_ave)
//   d loss / d z_r  w_r (softmax(z_r) - onehot(label_r))
//
// HBM-bound: every logit is read once and every gradient written once.  One workgroup of 1024 threads
// owns a row at a time and holds the whole row in registers as packed bf16 (up to 163840 entries:
// 20 loads of 16 bytes per thread, each load instruction of the workgroup covering 16 KiB of
// consecutive addresses), so the row maximum, the sum of exponentials and the gradient are all
// computed from that one read; the registers of a chunk are refilled with the next row while the
// gradient of this one is still being written.  Longer rows are streamed twice (running maximum and
// rescaled sum in the first pass; the second read mostly hits L2/MALL).
// The weighted token losses go to a workspace array and are summed by one workgroup in a fixed order,
// so the loss is bit-stable from run to run.
#include "common.hpp"

namespace hbp {

constexpr int kCeThreads = 1024;
constexpr int kCeChunk = kCeThreads * 8;  // logits covered by one load instruction of the workgroup
constexpr float kLog2eF = 1.4426950408889634f;
constexpr float kLn2F = 0.6931471805599453f;

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) x = fmaxf(x, __shfl_xor(x, m, 64));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
  return x;
}
// block-wide reduction over 1024 threads through 16 LDS slots; every thread gets the result
template <bool IS_MAX>
__device__ __forceinline__ float block_reduce(float x, float* slots, int tid) {
  x = IS_MAX ? wave_max(x) : wave_sum(x);
  __syncthreads();  // the slots may still be read from the previous reduction
  if ((tid & 63) == 0) slots[tid >> 6] = x;
  __syncthreads();
  float r = slots[0];
#pragma unroll
  for (int i = 1; i < kCeThreads / 64; ++i) r = IS_MAX ? fmaxf(r, slots[i]) : r + slots[i];
  return r;
}

// loss tokens per sample
__global__ __launch_bounds__(256) void ce_count_kernel(const CeParams p) {
  __shared__ int part[4];
  const int i = blockIdx.x;
  const int a = max(p.cu[i], 0), b = min(p.cu[i + 1], p.T);  // a malformed list cannot take a read out of bounds
  int n = 0;
  for (int r = a + (int)threadIdx.x; r < b; r += 256) n += p.labels[r] >= 0 && p.labels[r] < p.V;
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) n += __shfl_xor(n, m, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = n;
  __syncthreads();
  if (threadIdx.x == 0) p.counts[i] = part[0] + part[1] + part[2] + part[3];
  // a row that belongs to no sample has weight 0 (the weight kernel fills in the others)
  for (int r = i * 256 + (int)threadIdx.x; r < p.T; r += gridDim.x * 256) p.weighted[r] = 0.f;
}

// per-sample weight of a token's cross-entropy, written to every row of the sample (weighted[r] holds
// the row's weight until the main kernel replaces it with weight x loss); one workgroup per sample
__global__ __launch_bounds__(256) void ce_weight_kernel(const CeParams p) {
  __shared__ float part[4];
  const int tid = threadIdx.x, i = blockIdx.x;
  float total = 0.f;
  if (p.normalizer == HBP_LOSS_TOKEN_MEAN) {  // same order in every workgroup: the same bits
    for (int j = tid; j < p.n_samples; j += 256) total += (float)p.counts[j];
    total = wave_sum(total);
    if ((tid & 63) == 0) part[tid >> 6] = total;
    __syncthreads();
    total = (part[0] + part[1]) + (part[2] + part[3]);
  }
  const float c = (float)p.counts[i];
  float w;
  if (p.normalizer == HBP_LOSS_TOKEN_MEAN) w = total > 0.f ? 1.0f / total : 0.f;
  else if (p.normalizer == HBP_LOSS_SAMPLE_MEAN) w = c > 0.f ? 1.0f / (c * (float)p.n_samples) : 0.f;
  else w = 1.0f / ((float)p.n_samples * p.t_ave);
  if (tid == 0) p.weights[i] = w;
  const int a = max(p.cu[i], 0), b = min(p.cu[i + 1], p.T);
  for (int r = a + tid; r < b; r += 256) p.weighted[r] = w;
}

// NCH: 16-byte loads per thread that cover a row when HOLD (row kept in registers); with !HOLD the
// row is streamed in kCeChunk pieces, twice.  In the HOLD form the registers of a chunk are refilled
// with the same chunk of the workgroup's NEXT row as soon as its gradient is stored, so the reads of
// one row are in flight behind the arithmetic and the stores of the row before it.
//
// Softmax statistics: every thread takes the maximum m_t and the sum s_t = sum exp(z - m_t) of its own
// logits; (m, s) pairs are merged per wave and then through LDS, s = sum_t s_t exp(m_t - m).  One
// workgroup barrier per row: the LDS slots alternate between two sets from row to row.
template <int NCH, bool HOLD>
__global__ __launch_bounds__(kCeThreads) void ce_main_kernel(const CeParams p) {
  __shared__ float slot_m[2][kCeThreads / 64], slot_s[2][kCeThreads / 64];
  const int tid = threadIdx.x;
  const u32x4 kNegInf = {0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u};  // bf16 -inf pairs
  u32x4 held[HOLD ? NCH : 1];
  auto has_loss = [&](int label) { return label >= 0 && label < p.V; };  // an out-of-range label: no loss
  // chunks c of a row with an entry for this thread: c * kCeChunk + tid * 8 < V
  const int my_chunks = max(0, (p.V - tid * 8 + kCeChunk - 1) / kCeChunk);
  const uint32_t byte_in_chunk = tid * 16;
  // The value again, opaque to the optimiser: keeps it from computing every chunk's predicate and
  // address ahead of the loops and holding them in registers the row needs.
  auto fresh = [](auto x) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("" : "+v"(x));
#endif
    return x;
  };
  // Same for the held row between two passes over it: without this the unpacked fp32 values of one
  // pass are kept for the next one (8 registers per chunk instead of 4).
  auto forget_unpacked = [&]() {
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
    for (int c = 0; c < (HOLD ? NCH : 1); ++c) asm volatile("" : "+v"(held[c]));
#endif
  };
  auto chunk_ptr = [&](const uint16_t* row, int c) {  // uniform base + one per-thread offset
    return (u32x4*)((char*)(row + c * kCeChunk) + fresh(byte_in_chunk));
  };
  auto load_chunk = [&](const uint16_t* row, int c) {
    return c < fresh(my_chunks) ? __builtin_nontemporal_load((const u32x4*)chunk_ptr(row, c)) : kNegInf;
  };
  // -inf stands for "no entry": its exponent offset is taken as 0 so that no inf - inf appears
  auto finite_or_zero = [](float m) { return m == -INFINITY ? 0.f : m; };
  int r = blockIdx.x;
  int label = r < p.T ? p.labels[r] : -1;
  if (HOLD && r < p.T && has_loss(label)) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) held[c] = load_chunk(p.logits + (int64_t)r * p.stride_t, c);
  }
  for (int parity = 0; r < p.T;) {
    const int r_next = r + gridDim.x;
    const int label_next = r_next < p.T ? p.labels[r_next] : -1;
    const bool fetch_next = HOLD && r_next < p.T && has_loss(label_next);
    const bool live = has_loss(label);  // a row without a loss: zero loss, zero gradient, no arithmetic
    const uint16_t* row = p.logits + (int64_t)r * p.stride_t;
    const uint16_t* row_next = p.logits + (int64_t)r_next * p.stride_t;
    uint16_t* grow = p.dlogits ? p.dlogits + (int64_t)r * p.V : nullptr;
    float lse2w = 0.f, w = 0.f, z_label = 0.f;
    if (live) {
      w = p.weighted[r];  // the row's weight, put there by ce_weight_kernel
      z_label = __uint_as_float((uint32_t)row[label] << 16);
      float mx = -INFINITY, s = 0.f;
      auto chunk_max = [&](const u32x4& v, float m) {
#pragma unroll
        for (int k = 0; k < 4; ++k) m = fmaxf(m, fmaxf(bf16_lo(v[k]), bf16_hi(v[k])));
        return m;
      };
      auto chunk_sum = [&](const u32x4& v, float m2) {  // base 2 with log2(e) folded into the multiplier
        float a = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          a += __builtin_amdgcn_exp2f(__builtin_fmaf(bf16_lo(v[k]), kLog2eF, -m2));
          a += __builtin_amdgcn_exp2f(__builtin_fmaf(bf16_hi(v[k]), kLog2eF, -m2));
        }
        return a;
      };
      if (HOLD) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
          mx = chunk_max(held[c], mx);
          __builtin_amdgcn_sched_barrier(0);  // one chunk at a time: bounds the temporaries
        }
        forget_unpacked();
        const float m2 = finite_or_zero(mx) * kLog2eF;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
          s += chunk_sum(held[c], m2);
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
        // one pass: the running sum is rescaled when the running maximum moves
        for (int c = 0; c < my_chunks; ++c) {
          {
            const u32x4 v = *chunk_ptr(row, c);
            const float m_new = chunk_max(v, mx);
            s *= __builtin_amdgcn_exp2f((finite_or_zero(mx) - finite_or_zero(m_new)) * kLog2eF);
            s += chunk_sum(v, finite_or_zero(m_new) * kLog2eF);
            mx = m_new;
          }
        }
      }
      // wave, then workgroup
      const float m_wave = wave_max(mx);
      s *= __builtin_amdgcn_exp2f((finite_or_zero(mx) - finite_or_zero(m_wave)) * kLog2eF);
      s = wave_sum(s);
      if ((tid & 63) == 0) {
        slot_m[parity][tid >> 6] = m_wave;
        slot_s[parity][tid >> 6] = s;
      }
      __syncthreads();
      float m_row = slot_m[parity][0];
#pragma unroll
      for (int i = 1; i < kCeThreads / 64; ++i) m_row = fmaxf(m_row, slot_m[parity][i]);
      const float m_row0 = finite_or_zero(m_row);
      float s_row = 0.f;
#pragma unroll
      for (int i = 0; i < kCeThreads / 64; ++i)
        s_row += slot_s[parity][i] * __builtin_amdgcn_exp2f((finite_or_zero(slot_m[parity][i]) - m_row0) * kLog2eF);
      const float lse2 = m_row0 * kLog2eF + __builtin_amdgcn_logf(s_row);  // log2-sum-exp2 of the row
      const float ce = lse2 * kLn2F - z_label;
      lse2w = lse2 - __builtin_amdgcn_logf(w);  // w exp2(x - lse2) = exp2(x - lse2w)
      if (tid == 0) {
        p.token_loss[r] = ce;
        p.weighted[r] = w * ce;
      }
      parity ^= 1;  // per row WITH a barrier: a set is written again only after the barrier of the row between
    } else if (tid == 0) {
      p.token_loss[r] = 0.f;
      p.weighted[r] = 0.f;
    }
    // gradient w (softmax - onehot): the one entry at the label is patched in by the thread that holds it
    const int label_chunk = label / kCeChunk, label_tid = (label % kCeChunk) >> 3;
    auto chunk_grad = [&](const u32x4& v, int c) {
      u32x4 g;
#pragma unroll
      for (int k = 0; k < 4; ++k)
        g[k] = pack_bf16(__builtin_amdgcn_exp2f(__builtin_fmaf(bf16_lo(v[k]), kLog2eF, -lse2w)),
                         __builtin_amdgcn_exp2f(__builtin_fmaf(bf16_hi(v[k]), kLog2eF, -lse2w)));
      if (c == label_chunk && tid == label_tid) {
        const float a = __builtin_amdgcn_exp2f(__builtin_fmaf(z_label, kLog2eF, -lse2w)) - w;
        const uint32_t bits = pack_bf16(a, 0.f) & 0xffffu;
        const int k_label = (label >> 1) & 3;
#pragma unroll
        for (int k = 0; k < 4; ++k)
          if (k == k_label) g[k] = (label & 1) ? (g[k] & 0xffffu) | (bits << 16) : (g[k] & 0xffff0000u) | bits;
      }
      __builtin_nontemporal_store(g, chunk_ptr(grow, c));
    };
    if (HOLD) {
      forget_unpacked();
      // the only place (after the first row) where the held registers are written
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        if (grow && c < fresh(my_chunks)) {
          if (live) chunk_grad(held[c], c);
          else __builtin_nontemporal_store(u32x4{0, 0, 0, 0}, chunk_ptr(grow, c));
        }
        if (fetch_next) held[c] = load_chunk(row_next, c);
        __builtin_amdgcn_sched_barrier(0);  // keep the refill behind the store: hoisted loads would need a second set of registers
      }
    } else if (grow) {
      for (int c = 0; c < my_chunks; ++c) {
        if (live) chunk_grad(*chunk_ptr(row, c), c);
        else __builtin_nontemporal_store(u32x4{0, 0, 0, 0}, chunk_ptr(grow, c));
      }
    }
    r = r_next;
    label = label_next;
  }
}

// loss = sum of the weighted token losses, fixed order
__global__ __launch_bounds__(kCeThreads) void ce_reduce_kernel(const CeParams p) {
  __shared__ float slots[kCeThreads / 64];
  const int tid = threadIdx.x;
  float acc = 0.f;
  for (int r = tid; r < p.T; r += kCeThreads) acc += p.weighted[r];
  acc = block_reduce<false>(acc, slots, tid);
  if (tid == 0) *p.loss_out = acc;
}

// grid = the workgroups resident at once (a persistent loop over rows; a second round of workgroups
// would start with an empty pipeline)
template <int NCH, bool HOLD>
static void launch_main(const CeParams& p, int n_cu, hipStream_t s) {
  static int per_cu = 0;  // same on every device of this part
  if (per_cu == 0) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, ce_main_kernel<NCH, HOLD>, kCeThreads, 0) != hipSuccess || n < 1) n = 1;
    per_cu = n;
  }
  const int64_t resident = (int64_t)per_cu * n_cu;
  const int grid = p.T < resident ? p.T : (int)resident;
  hipLaunchKernelGGL((ce_main_kernel<NCH, HOLD>), dim3(grid), dim3(kCeThreads), 0, s, p);
}

int launch_packed_ce(const CeParams& p, int n_cu, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
  if (p.n_samples > 0) {
    hipLaunchKernelGGL(ce_count_kernel, dim3(p.n_samples), dim3(256), 0, s, p);
    hipLaunchKernelGGL(ce_weight_kernel, dim3(p.n_samples), dim3(256), 0, s, p);
  }
  if (p.T > 0) {
    if (ev0 && hipEventRecord(ev0, s) != hipSuccess) return (int)hipErrorInvalidValue;
    const int chunks = (p.V + kCeChunk - 1) / kCeChunk;
    if (chunks <= 2) launch_main<2, true>(p, n_cu, s);
    else if (chunks <= 4) launch_main<4, true>(p, n_cu, s);
    else if (chunks <= 8) launch_main<8, true>(p, n_cu, s);
    else if (chunks <= 16) launch_main<16, true>(p, n_cu, s);
    else if (chunks <= 20) launch_main<20, true>(p, n_cu, s);
    else launch_main<1, false>(p, n_cu, s);
    if (ev1 && hipEventRecord(ev1, s) != hipSuccess) return (int)hipErrorInvalidValue;
  }
  hipLaunchKernelGGL(ce_reduce_kernel, dim3(1), dim3(kCeThreads), 0, s, p);
  return (int)hipGetLastError();
}

}  // namespace hbp
