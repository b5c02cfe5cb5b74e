// Packed cross-entropy with the paper's loss normalisers (Section 4.3, normaliser equation), forward
// and backward in one pass over the logits, gfx950.
//
//   token loss      CE_r = logsumexp(z_r) - z_r[label_r]                     (rows with label < 0: none)
//   loss            sum_r w_r CE_r,  w_r by normaliser: token-mean 1 / sum_i T_i, sample-mean
//                   1 / (T_i B_l) for the row's sample i, stable 1 / (B_l T_ave)
//   d loss / d z_r  w_r (softmax(z_r) - onehot(label_r))
//
// HBM-bound: every logit is read once and every gradient written once.  One workgroup of 1024 threads
// owns a row at a time and holds the whole row in registers as packed bf16 (up to 131072 entries:
// 16 loads of 16 bytes per thread, each load instruction of the workgroup covering 16 KiB of
// consecutive addresses), so the row maximum, the sum of exponentials and the gradient are all
// computed from that one read.  Longer rows are streamed twice (the second read mostly hits L2/MALL).
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
}

// per-sample weight of a token's cross-entropy
__global__ __launch_bounds__(kCeThreads) void ce_weight_kernel(const CeParams p) {
  __shared__ float slots[kCeThreads / 64];
  const int tid = threadIdx.x;
  float total = 0.f;  // exact in fp32 up to 2^24 tokens per term; summed as float of ints <= 2^31 is fine for a weight
  for (int i = tid; i < p.n_samples; i += kCeThreads) total += (float)p.counts[i];
  total = block_reduce<false>(total, slots, tid);
  for (int i = tid; i < p.n_samples; i += kCeThreads) {
    const float c = (float)p.counts[i];
    float w;
    if (p.normalizer == HBP_LOSS_TOKEN_MEAN) w = total > 0.f ? 1.0f / total : 0.f;
    else if (p.normalizer == HBP_LOSS_SAMPLE_MEAN) w = c > 0.f ? 1.0f / (c * (float)p.n_samples) : 0.f;
    else w = 1.0f / ((float)p.n_samples * p.t_ave);
    p.weights[i] = w;
  }
}

__device__ __forceinline__ int sample_of_row(const int32_t* cu, int n_samples, int r) {
  int lo = 0, hi = n_samples;  // cu[lo] <= r < cu[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu[mid] <= r) lo = mid;
    else hi = mid;
  }
  return lo;
}

// NCH: 16-byte loads per thread that cover a row when HOLD (row kept in registers); with !HOLD the
// row is streamed in kCeChunk pieces, twice.  In the HOLD form the registers of a chunk are refilled
// with the same chunk of the workgroup's NEXT row as soon as its gradient is stored, so the reads of
// one row are in flight behind the arithmetic and the stores of the row before it.
template <int NCH, bool HOLD>
__global__ __launch_bounds__(kCeThreads) void ce_main_kernel(const CeParams p) {
  __shared__ float slots[kCeThreads / 64];
  const int tid = threadIdx.x;
  const u32x4 kNegInf = {0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u};  // bf16 -inf pairs
  u32x4 held[HOLD ? NCH : 1];
  auto has_loss = [&](int label) { return label >= 0 && label < p.V; };  // an out-of-range label: no loss
  auto load_chunk = [&](const uint16_t* row, int c) {
    const int e = c * kCeChunk + tid * 8;
    return e < p.V ? __builtin_nontemporal_load((const u32x4*)(row + e)) : kNegInf;
  };
  int r = blockIdx.x;
  int label = r < p.T ? p.labels[r] : -1;
  if (HOLD && r < p.T && has_loss(label)) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) held[c] = load_chunk(p.logits + (int64_t)r * p.stride_t, c);
  }
  for (; r < p.T;) {
    const int r_next = r + gridDim.x;
    const int label_next = r_next < p.T ? p.labels[r_next] : -1;
    const bool fetch_next = HOLD && r_next < p.T && has_loss(label_next);
    const bool live = has_loss(label);  // a row without a loss: zero loss, zero gradient, no arithmetic
    const uint16_t* row = p.logits + (int64_t)r * p.stride_t;
    const uint16_t* row_next = p.logits + (int64_t)r_next * p.stride_t;
    uint16_t* grow = p.dlogits ? p.dlogits + (int64_t)r * p.V : nullptr;
    const int n_chunks = HOLD ? NCH : (p.V + kCeChunk - 1) / kCeChunk;
    float lse2 = 0.f, w = 0.f;
    if (live) {
      // maximum
      float mx = -INFINITY;
      auto chunk_max = [&](const u32x4& v) {
#pragma unroll
        for (int k = 0; k < 4; ++k) mx = fmaxf(mx, fmaxf(bf16_lo(v[k]), bf16_hi(v[k])));
      };
      if (HOLD) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
          chunk_max(held[c]);
          __builtin_amdgcn_sched_barrier(0);  // one chunk at a time: bounds the temporaries
        }
      } else {
        for (int c = 0; c < n_chunks; ++c) {
          const int e = c * kCeChunk + tid * 8;
          if (e < p.V) chunk_max(*(const u32x4*)(row + e));
        }
      }
      mx = block_reduce<true>(mx, slots, tid);
      const float m2 = mx * kLog2eF;
      // sum of exponentials, base 2 with log2(e) folded into the multiplier
      float s = 0.f;
      auto chunk_sum = [&](const u32x4& v) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          s += __builtin_amdgcn_exp2f(__builtin_fmaf(bf16_lo(v[k]), kLog2eF, -m2));
          s += __builtin_amdgcn_exp2f(__builtin_fmaf(bf16_hi(v[k]), kLog2eF, -m2));
        }
      };
      if (HOLD) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
          chunk_sum(held[c]);
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
        for (int c = 0; c < n_chunks; ++c) {
          const int e = c * kCeChunk + tid * 8;
          if (e < p.V) chunk_sum(*(const u32x4*)(row + e));
        }
      }
      s = block_reduce<false>(s, slots, tid);
      lse2 = m2 + __builtin_amdgcn_logf(s);  // log2-sum-exp2 of the row
      const float z_label = __uint_as_float((uint32_t)row[label] << 16);
      const float ce = lse2 * kLn2F - z_label;
      w = p.weights[sample_of_row(p.cu, p.n_samples, r)];
      if (tid == 0) {
        p.token_loss[r] = ce;
        p.weighted[r] = w * ce;
      }
    } else if (tid == 0) {
      p.token_loss[r] = 0.f;
      p.weighted[r] = 0.f;
    }
    auto chunk_grad = [&](const u32x4& v, int e) {
      u32x4 g;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        float a = w * __builtin_amdgcn_exp2f(__builtin_fmaf(bf16_lo(v[k]), kLog2eF, -lse2));
        float b = w * __builtin_amdgcn_exp2f(__builtin_fmaf(bf16_hi(v[k]), kLog2eF, -lse2));
        if (e + 2 * k == label) a -= w;
        if (e + 2 * k + 1 == label) b -= w;
        g[k] = pack_bf16(a, b);
      }
      __builtin_nontemporal_store(g, (u32x4*)(grow + e));
    };
    if (HOLD) {
      // the only place (after the first row) where the held registers are written
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const int e = c * kCeChunk + tid * 8;
        if (grow && e < p.V) {
          if (live) chunk_grad(held[c], e);
          else __builtin_nontemporal_store(u32x4{0, 0, 0, 0}, (u32x4*)(grow + e));
        }
        if (fetch_next) held[c] = load_chunk(row_next, c);
        __builtin_amdgcn_sched_barrier(0);  // keep the refill behind the store: hoisted loads would need a second set of registers
      }
    } else if (grow) {
      for (int c = 0; c < n_chunks; ++c) {
        const int e = c * kCeChunk + tid * 8;
        if (e < p.V) {
          if (live) chunk_grad(*(const u32x4*)(row + e), e);
          else __builtin_nontemporal_store(u32x4{0, 0, 0, 0}, (u32x4*)(grow + e));
        }
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
    hipLaunchKernelGGL(ce_weight_kernel, dim3(1), dim3(kCeThreads), 0, s, p);
  }
  if (p.T > 0) {
    if (ev0 && hipEventRecord(ev0, s) != hipSuccess) return (int)hipErrorInvalidValue;
    const int chunks = (p.V + kCeChunk - 1) / kCeChunk;
    if (chunks <= 2) launch_main<2, true>(p, n_cu, s);
    else if (chunks <= 4) launch_main<4, true>(p, n_cu, s);
    else if (chunks <= 8) launch_main<8, true>(p, n_cu, s);
    else if (chunks <= 16) launch_main<16, true>(p, n_cu, s);
    else launch_main<1, false>(p, n_cu, s);
    if (ev1 && hipEventRecord(ev1, s) != hipSuccess) return (int)hipErrorInvalidValue;
  }
  hipLaunchKernelGGL(ce_reduce_kernel, dim3(1), dim3(kCeThreads), 0, s, p);
  return (int)hipGetLastError();
}

}  // namespace hbp
