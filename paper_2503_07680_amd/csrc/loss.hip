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

// Rows to workgroups: workgroup k of the main kernel takes the consecutive rows
// [row_start[k], row_start[k + 1]), cut so that every range carries the same memory traffic (a row
// with a loss is read and written, one without is only written, or skipped when no gradient is asked
// for).  row_start[k] = the first row whose preceding rows cost at least k / n_ranges of the total.
__device__ __forceinline__ int row_cost(int label, int V, bool with_grad) {
  return (label >= 0 && label < V ? 8 : 0) + (with_grad ? 8 : 0) + 1;
}
__global__ __launch_bounds__(kCeThreads) void ce_partition_kernel(const CeParams p, int n_ranges) {
  __shared__ int64_t part[kCeThreads];
  const int tid = threadIdx.x;
  const bool with_grad = p.dlogits != nullptr;
  const int slice = (p.T + kCeThreads - 1) / kCeThreads;
  const int a = min(tid * slice, p.T), b = min(a + slice, p.T);
  int64_t mine = 0;
  for (int r = a; r < b; ++r) mine += row_cost(p.labels[r], p.V, with_grad);
  part[tid] = mine;
  __syncthreads();
  for (int d = 1; d < kCeThreads; d <<= 1) {  // inclusive scan
    const int64_t add = tid >= d ? part[tid - d] : 0;
    __syncthreads();
    part[tid] += add;
    __syncthreads();
  }
  const int64_t total = part[kCeThreads - 1];
  int64_t before = part[tid] - mine;  // cost of the rows before row a
  if (tid == 0) p.row_start[0] = 0;
  for (int r = a; r < b; ++r) {
    const int64_t after = before + row_cost(p.labels[r], p.V, with_grad);
    // ranges k with before < k total / n_ranges <= after begin at row r + 1
    for (int64_t k = before * n_ranges / total + 1; k <= after * n_ranges / total; ++k) p.row_start[k] = r + 1;
    before = after;
  }
}

// NCH: 16-byte loads per thread that cover a row when HOLD (row kept in registers); with !HOLD the
// row is streamed in kCeChunk pieces, twice.
//
// Softmax statistics: every thread keeps a running maximum m_t and sum s_t = sum exp(z - m_t) over its
// own logits, chunk by chunk (the sum is rescaled when the maximum moves); the (m, s) pairs are merged
// per wave and then through LDS, s = sum_t s_t exp(m_t - m).  One workgroup barrier per row: the LDS
// slots alternate between two sets from row to row.
//
// HOLD form, one loop over the chunks per row with all of the row's memory traffic AND arithmetic in
// it: step c computes and stores chunk c of THIS row's gradient, refills the chunk's registers with
// chunk c of the workgroup's NEXT row, and adds chunk c - kLag of the next row (loaded kLag steps
// earlier) to that row's statistics.  A compute unit cannot queue a whole row of memory operations, so
// arithmetic outside this loop would run with the memory pipe idle.
#ifndef HBP_CE_LAG
#define HBP_CE_LAG 2
#endif
constexpr int kLag = HBP_CE_LAG;
constexpr int kRowBatch = 256;  // rows whose scalars are staged in LDS at a time

template <int NCH, bool HOLD, bool WITH_GRAD>
__global__ __launch_bounds__(kCeThreads) void ce_main_kernel(const CeParams p) {
  __shared__ float slot_m[2][kCeThreads / 64], slot_s[2][kCeThreads / 64];
  const int tid = threadIdx.x;
  const u32x4 kNegInf = {0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u};  // bf16 -inf pairs
  u32x4 held[HOLD ? NCH : 1];
  auto has_loss = [&](int label) { return label >= 0 && label < p.V; };  // an out-of-range label: no loss
  // HOLD: NCH = ceil(V / kCeChunk) exactly, so every chunk but the last has an entry for every thread
  // and the last one for the threads with tail_valid: which chunk needs a predicate is known at
  // compile time, and the chunk loops are straight-line code.
  const int last_chunk = HOLD ? NCH - 1 : (p.V + kCeChunk - 1) / kCeChunk - 1;
  const bool tail_valid = last_chunk * kCeChunk + tid * 8 < p.V;
  const int my_chunks = last_chunk + (tail_valid ? 1 : 0);
  const uint32_t byte_in_chunk = tid * 16;
  const uint32_t byte_in_tail = tail_valid ? byte_in_chunk : 0;  // a thread without an entry reads the chunk's first
  // The value again, opaque to the optimiser: keeps it from computing every chunk's predicate and
  // address ahead of the loops and holding them in registers the row needs.
  auto fresh = [](auto x) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("" : "+v"(x));
#endif
    return x;
  };
  auto chunk_ptr = [&](const uint16_t* row, int c) {  // uniform base + one per-thread offset
    return (u32x4*)((char*)(row + c * kCeChunk) + fresh(byte_in_chunk));
  };
  // Unconditional for every thread (a predicated load would have to be waited for at once to merge it
  // with the "no entry" value): the partial chunk is masked where it is used, see entries().
  auto load_chunk = [&](const uint16_t* row, int c) {
    const uint32_t off = c == last_chunk ? byte_in_tail : byte_in_chunk;
    return __builtin_nontemporal_load((const u32x4*)((const char*)(row + c * kCeChunk) + fresh(off)));
  };
  auto entries = [&](const u32x4& v, int c) {  // the chunk as held, "no entry" = -inf
    u32x4 x = v;
    if (c == last_chunk) x = tail_valid ? v : kNegInf;
    return x;
  };

  // -inf stands for "no entry": its exponent offset is taken as 0 so that no inf - inf appears
  auto finite_or_zero = [](float m) { return m == -INFINITY ? 0.f : m; };
  // running (maximum, sum of exponentials) of this thread's entries, base 2 with log2(e) folded in
  float mx = -INFINITY, sm = 0.f;
  auto add_to_stats = [&](const u32x4& v) {
    float m_new = mx;
#pragma unroll
    for (int k = 0; k < 4; ++k) m_new = fmaxf(m_new, fmaxf(bf16_lo(v[k]), bf16_hi(v[k])));
    const float m2 = finite_or_zero(m_new) * kLog2eF;
    float a = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      a += __builtin_amdgcn_exp2f(__builtin_fmaf(bf16_lo(v[k]), kLog2eF, -m2));
      a += __builtin_amdgcn_exp2f(__builtin_fmaf(bf16_hi(v[k]), kLog2eF, -m2));
    }
    sm = sm * __builtin_amdgcn_exp2f(__builtin_fmaf(finite_or_zero(mx), kLog2eF, -m2)) + a;
    mx = m_new;
  };
  // Per-row scalars (label, weight, logit at the label) of the workgroup's next kRowBatch rows, staged
  // in LDS by one thread per row.  Read from global memory inside the row loop they would have to be
  // waited for with every outstanding store and load of the chunk pipeline (the counter is in order).
  __shared__ int row_label[kRowBatch];
  __shared__ float row_weight[kRowBatch], row_zlabel[kRowBatch];
  const int row_end = p.row_start[blockIdx.x + 1];
  auto stage_rows = [&](int first_row) {  // rows first_row + i, i < kRowBatch
    __syncthreads();                       // the entries of the batch before have all been read
    if (tid < kRowBatch) {
      const int64_t rr = (int64_t)first_row + tid;
      int lab = -1;
      float wt = 0.f, zl = 0.f;
      if (rr < row_end) {
        lab = p.labels[rr];
        if (has_loss(lab)) {
          wt = p.weighted[rr];  // the row's weight, put there by ce_weight_kernel
          zl = __uint_as_float((uint32_t)p.logits[rr * p.stride_t + lab] << 16);
        } else {
          lab = -1;
        }
      }
      row_label[tid] = lab;
      row_weight[tid] = wt;
      row_zlabel[tid] = zl;
    }
    __syncthreads();
  };
  int r = p.row_start[blockIdx.x];
  if (r >= row_end) return;
  stage_rows(r);
  int label = row_label[0];  // -1: no loss
  float w = row_weight[0], z_label = row_zlabel[0];
  if (HOLD && label >= 0) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) held[c] = load_chunk(p.logits + (int64_t)r * p.stride_t, c);
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      add_to_stats(entries(held[c], c));
      __builtin_amdgcn_sched_barrier(0);  // one chunk at a time: bounds the temporaries
    }
  }
  for (int parity = 0, i_next = 1; r < row_end; ++i_next) {
    const int r_next = r + 1;
    if (i_next % kRowBatch == 0 && r_next < row_end) stage_rows(r_next);
    const int label_next = r_next < row_end ? row_label[i_next % kRowBatch] : -1;
    const float w_next = row_weight[i_next % kRowBatch], z_label_next = row_zlabel[i_next % kRowBatch];
    const bool fetch_next = HOLD && label_next >= 0;
    const bool live = label >= 0;  // a row without a loss: zero loss, zero gradient, no arithmetic
    const uint16_t* row = p.logits + (int64_t)r * p.stride_t;
    const uint16_t* row_next = p.logits + (int64_t)r_next * p.stride_t;
    uint16_t* grow = WITH_GRAD ? p.dlogits + (int64_t)r * p.V : nullptr;
    float lse2w = 0.f;
    if (live) {
      if (!HOLD) {
        for (int c = 0; c < my_chunks; ++c) add_to_stats(*chunk_ptr(row, c));
      }
      // wave, then workgroup
      const float m_wave = wave_max(mx);
      sm *= __builtin_amdgcn_exp2f((finite_or_zero(mx) - finite_or_zero(m_wave)) * kLog2eF);
      sm = wave_sum(sm);
      if ((tid & 63) == 0) {
        slot_m[parity][tid >> 6] = m_wave;
        slot_s[parity][tid >> 6] = sm;
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
    mx = -INFINITY;  // from here on: the statistics of the next row
    sm = 0.f;
    // gradient w (softmax - onehot): the one entry at the label is patched in by the thread that holds it
    const int label_chunk = label / kCeChunk, label_tid = (label % kCeChunk) >> 3;
    auto chunk_grad = [&](const u32x4& v, int c) {  // zeros for a row without a loss
      u32x4 g = {0, 0, 0, 0};
      if (live) {
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
      }
      return g;
    };
    if (HOLD) {
      // the only place (after the first row) where the held registers are written
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        // No store or load of this loop sits in a branch on a uniform condition (the arithmetic does):
        // with one there the compiler waits for ALL outstanding memory operations at every use of a
        // loaded chunk instead of for that chunk's load.
        if (WITH_GRAD) {
          const u32x4 g = chunk_grad(held[c], c);
          if (c < NCH - 1) __builtin_nontemporal_store(g, chunk_ptr(grow, c));
          else if (tail_valid) __builtin_nontemporal_store(g, chunk_ptr(grow, c));
        }
        if (fetch_next) {
          held[c] = load_chunk(row_next, c);
          if (c >= kLag) add_to_stats(entries(held[c - kLag], c - kLag));
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the refill behind the store: hoisted loads would need a second set of registers
      }
      if (fetch_next) {
#pragma unroll
        for (int c = NCH > kLag ? NCH - kLag : 0; c < NCH; ++c) {
          add_to_stats(entries(held[c], c));
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    } else if (WITH_GRAD) {
      for (int c = 0; c < my_chunks; ++c) __builtin_nontemporal_store(chunk_grad(*chunk_ptr(row, c), c), chunk_ptr(grow, c));
    }
    r = r_next;
    label = label_next;
    w = w_next;
    z_label = z_label_next;
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

// Workgroups resident at once per compute unit.  The main kernel's grid is that times the compute
// units: a persistent loop over rows; a second batch of workgroups would start with an empty pipeline.
template <int NCH, bool HOLD, bool WITH_GRAD>
static int main_per_cu() {
  static int per_cu = 0;  // same on every device of this part
  if (per_cu == 0) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, ce_main_kernel<NCH, HOLD, WITH_GRAD>, kCeThreads, 0) != hipSuccess || n < 1) n = 1;
    per_cu = n;
  }
  return per_cu;
}
template <int NCH, bool HOLD, bool WITH_GRAD>
static void launch_main_g(const CeParams& p, int n_cu, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
  int64_t grid = (int64_t)main_per_cu<NCH, HOLD, WITH_GRAD>() * n_cu;
  if (grid > kCeMaxWorkgroups) grid = kCeMaxWorkgroups;
  if (grid > p.T) grid = p.T;
  hipLaunchKernelGGL(ce_partition_kernel, dim3(1), dim3(kCeThreads), 0, s, p, (int)grid);
  if (ev0) (void)hipEventRecord(ev0, s);
  hipLaunchKernelGGL((ce_main_kernel<NCH, HOLD, WITH_GRAD>), dim3((unsigned)grid), dim3(kCeThreads), 0, s, p);
  if (ev1) (void)hipEventRecord(ev1, s);
}
template <int NCH, bool HOLD>
static void launch_main(const CeParams& p, int n_cu, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
  if (p.dlogits) launch_main_g<NCH, HOLD, true>(p, n_cu, s, ev0, ev1);
  else launch_main_g<NCH, HOLD, false>(p, n_cu, s, ev0, ev1);
}

int launch_packed_ce(const CeParams& p, int n_cu, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
  if (p.n_samples > 0) {
    hipLaunchKernelGGL(ce_count_kernel, dim3(p.n_samples), dim3(256), 0, s, p);
    hipLaunchKernelGGL(ce_weight_kernel, dim3(p.n_samples), dim3(256), 0, s, p);
  }
  if (p.T > 0) {
    const int chunks = (p.V + kCeChunk - 1) / kCeChunk;
    switch (chunks) {
#define HBP_CE_HELD(N) case N: launch_main<N, true>(p, n_cu, s, ev0, ev1); break;
      HBP_CE_HELD(1) HBP_CE_HELD(2) HBP_CE_HELD(3) HBP_CE_HELD(4) HBP_CE_HELD(5)
      HBP_CE_HELD(6) HBP_CE_HELD(7) HBP_CE_HELD(8) HBP_CE_HELD(9) HBP_CE_HELD(10)
      HBP_CE_HELD(11) HBP_CE_HELD(12) HBP_CE_HELD(13) HBP_CE_HELD(14) HBP_CE_HELD(15)
      HBP_CE_HELD(16) HBP_CE_HELD(17) HBP_CE_HELD(18) HBP_CE_HELD(19) HBP_CE_HELD(20)
#undef HBP_CE_HELD
      default: launch_main<1, false>(p, n_cu, s, ev0, ev1);
    }
  }
  hipLaunchKernelGGL(ce_reduce_kernel, dim3(1), dim3(kCeThreads), 0, s, p);
  return (int)hipGetLastError();
}

}  // namespace hbp
