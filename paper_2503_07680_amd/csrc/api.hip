// C ABI: argument validation on the host, then kernel launches on the caller's stream.
#include <climits>
#include <cmath>
#include <cstring>
#include <mutex>

#include "common.hpp"

namespace {

constexpr int kNumCU = 256;          // MI355X: 8 accelerator dies x 32 compute units
constexpr size_t kCounterBytes = 2048;  // two sets of 8 per-die counters, 128 bytes apart
constexpr int64_t kMaxTokenStride = int64_t{1} << 22;  // elements; see check_desc
constexpr int kTileRows = 128;       // rows per query / key tile of every kernel (the forward also takes 256)

bool dims_supported(int d_qk, int d_v) {
  return (d_qk == 64 && d_v == 64) || (d_qk == 128 && d_v == 128) || (d_qk == 192 && d_v == 128);
}


struct Strides {
  int64_t q_st, q_sh, k_st, k_sh, v_st, v_sh, o_st, o_sh;
};

hbp_status check_desc(const hbp_attn_desc* d, Strides* st) {
  if (!d) return HBP_ERR_INVALID_ARG;
  if (d->total_tokens < 0 || d->n_samples < 0 || d->n_q_heads <= 0 || d->n_kv_heads <= 0 ||
      d->d_qk <= 0 || d->d_v <= 0)
    return HBP_ERR_INVALID_ARG;
  if (!std::isfinite(d->softmax_scale)) return HBP_ERR_INVALID_ARG;
  if (d->n_q_heads % d->n_kv_heads) return HBP_ERR_SHAPE;
  if (!dims_supported(d->d_qk, d->d_v)) return HBP_ERR_UNSUPPORTED;
  if (d->fwd_tile_rows != 0 && d->fwd_tile_rows != kTileRows &&
      !(d->fwd_tile_rows == 2 * kTileRows && (d->n_q_heads / d->n_kv_heads) % 2 == 1))
    return HBP_ERR_INVALID_ARG;
  auto fix = [](int64_t s, int64_t dense) { return s == 0 ? dense : s; };
  st->q_sh = fix(d->q_stride_h, d->d_qk);
  st->q_st = fix(d->q_stride_t, (int64_t)d->n_q_heads * d->d_qk);
  st->k_sh = fix(d->k_stride_h, d->d_qk);
  st->k_st = fix(d->k_stride_t, (int64_t)d->n_kv_heads * d->d_qk);
  st->v_sh = fix(d->v_stride_h, d->d_v);
  st->v_st = fix(d->v_stride_t, (int64_t)d->n_kv_heads * d->d_v);
  st->o_sh = fix(d->o_stride_h, d->d_v);
  st->o_st = fix(d->o_stride_t, (int64_t)d->n_q_heads * d->d_v);
  // every stride must hold its row and keep 16-byte vector accesses aligned
  const int64_t all[8] = {st->q_st, st->q_sh, st->k_st, st->k_sh, st->v_st, st->v_sh, st->o_st, st->o_sh};
  for (int64_t s : all)
    if (s <= 0 || (s % 8) != 0) return HBP_ERR_SHAPE;
  if (st->q_sh < d->d_qk || st->k_sh < d->d_qk || st->v_sh < d->d_v || st->o_sh < d->d_v)
    return HBP_ERR_SHAPE;
  if (st->q_st < d->d_qk || st->k_st < d->d_qk || st->v_st < d->d_v || st->o_st < d->d_v)
    return HBP_ERR_SHAPE;
  // The kernels form (row of a tile) * (token stride in bytes) in 32 bits, the tile copies with a 24-bit
  // multiply: a token stride must stay below 2^23 elements.  The bound is 2^22 (8 MiB per token).
  if (st->q_st > kMaxTokenStride || st->k_st > kMaxTokenStride || st->v_st > kMaxTokenStride ||
      st->o_st > kMaxTokenStride)
    return HBP_ERR_SHAPE;
  return HBP_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct BwdLayout {
  size_t d_off, lse2_off, dk_part_off, dv_part_off, total;
};

BwdLayout bwd_layout(const hbp_attn_desc* d) {
  BwdLayout l;
  l.d_off = kCounterBytes;
  const size_t rows = align_up((size_t)d->n_q_heads * d->total_tokens * sizeof(float), 256);
  l.lse2_off = l.d_off + rows;
  const int g = d->n_q_heads / d->n_kv_heads;
  l.dk_part_off = l.lse2_off + rows;
  l.dv_part_off = l.dk_part_off + align_up(hbp::bwd_partial_floats(d->total_tokens, d->n_kv_heads, g, d->d_qk) * sizeof(float), 256);
  l.total = l.dv_part_off + align_up(hbp::bwd_partial_floats(d->total_tokens, d->n_kv_heads, g, d->d_v) * sizeof(float), 256);
  return l;
}

float resolve_scale(const hbp_attn_desc* d) {
  return d->softmax_scale > 0.f ? d->softmax_scale : 1.0f / std::sqrt((float)d->d_qk);
}

hipEvent_t g_events[4][2] = {{nullptr, nullptr}, {nullptr, nullptr}, {nullptr, nullptr}, {nullptr, nullptr}};

// the schedulers count (tile, head) items in 32-bit integers
bool item_count_fits(int32_t n_tiles, int32_t n_heads) { return (int64_t)n_tiles * n_heads <= INT32_MAX; }

int grid_for(int64_t n_items, int blocks_per_cu) {
  const int64_t cap = (int64_t)kNumCU * blocks_per_cu;
  return (int)(n_items < cap ? n_items : cap);
}

}  // namespace

extern "C" const char* hbp_status_string(hbp_status s) {
  switch (s) {
    case HBP_OK: return "ok";
    case HBP_ERR_INVALID_ARG: return "invalid argument";
    case HBP_ERR_SHAPE: return "inconsistent shape or stride";
    case HBP_ERR_UNSUPPORTED: return "unsupported head dimensions";
    case HBP_ERR_CAPACITY: return "output array too small";
    case HBP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case HBP_ERR_DEVICE: return "HIP runtime error at launch";
    case HBP_ERR_NO_MEMORY: return "out of host memory";
    case HBP_ERR_STATIC_LIMIT: return "problem needs more scratch than the library's static buffer holds";
    default: return "unknown status";
  }
}

namespace {
struct CeLayout {
  size_t weighted_off, token_loss_off, counts_off, weights_off, row_start_off, total;
};
CeLayout ce_layout(int32_t T, int32_t n) {
  CeLayout l;
  l.weighted_off = 0;
  l.token_loss_off = align_up((size_t)T * sizeof(float), 256);
  l.counts_off = l.token_loss_off + align_up((size_t)T * sizeof(float), 256);
  l.weights_off = l.counts_off + align_up((size_t)n * sizeof(int32_t), 256);
  l.row_start_off = l.weights_off + align_up((size_t)n * sizeof(float), 256);
  l.total = l.row_start_off + align_up((size_t)(hbp::kCeMaxWorkgroups + 1) * sizeof(int32_t), 256) + 256;
  return l;
}
}  // namespace

extern "C" hbp_status hbp_packed_ce_workspace_bytes(int32_t total_tokens, int32_t n_samples, size_t* bytes_out) {
  if (!bytes_out || total_tokens < 0 || n_samples < 0) return HBP_ERR_INVALID_ARG;
  *bytes_out = ce_layout(total_tokens, n_samples).total;
  return HBP_OK;
}

extern "C" hbp_status hbp_packed_ce(const void* logits, int64_t logit_stride_t, int32_t total_tokens,
                                    int32_t vocab, const int32_t* labels, const int32_t* cu_seqlens,
                                    int32_t n_samples, int32_t normalizer, float t_ave, void* dlogits_or_null,
                                    float* loss_out, float* token_loss_or_null, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  if (total_tokens < 0 || n_samples < 0 || vocab < 1 || !loss_out) return HBP_ERR_INVALID_ARG;
  if (normalizer != HBP_LOSS_TOKEN_MEAN && normalizer != HBP_LOSS_SAMPLE_MEAN && normalizer != HBP_LOSS_STABLE)
    return HBP_ERR_INVALID_ARG;
  if (normalizer == HBP_LOSS_STABLE && !(t_ave > 0.f)) return HBP_ERR_INVALID_ARG;
  if (total_tokens > 0 && (!logits || !labels || !cu_seqlens || n_samples < 1)) return HBP_ERR_INVALID_ARG;
  const int64_t stride = logit_stride_t ? logit_stride_t : vocab;
  if (stride < vocab) return HBP_ERR_SHAPE;
  if (vocab % 8 || stride % 8 || !aligned16(logits) || !aligned16(dlogits_or_null)) return HBP_ERR_UNSUPPORTED;
  const CeLayout lay = ce_layout(total_tokens, n_samples);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < lay.total)
    return HBP_ERR_WORKSPACE;
  char* ws = static_cast<char*>(workspace);
  hbp::CeParams p;
  p.logits = static_cast<const uint16_t*>(logits);
  p.stride_t = stride;
  p.T = total_tokens;
  p.V = vocab;
  p.n_samples = n_samples;
  p.normalizer = normalizer;
  p.labels = labels;
  p.cu = cu_seqlens;
  p.t_ave = t_ave;
  p.dlogits = static_cast<uint16_t*>(dlogits_or_null);
  p.weighted = reinterpret_cast<float*>(ws + lay.weighted_off);
  p.token_loss = token_loss_or_null ? token_loss_or_null : reinterpret_cast<float*>(ws + lay.token_loss_off);
  p.counts = reinterpret_cast<int32_t*>(ws + lay.counts_off);
  p.weights = reinterpret_cast<float*>(ws + lay.weights_off);
  p.row_start = reinterpret_cast<int32_t*>(ws + lay.row_start_off);
  p.loss_out = loss_out;
  if (hbp::launch_packed_ce(p, kNumCU, static_cast<hipStream_t>(stream), g_events[HBP_LOSS][0],
                            g_events[HBP_LOSS][1]) != 0)
    return HBP_ERR_DEVICE;
  return HBP_OK;
}

namespace {
// nothing but independent MFMAs: four accumulators per wave, operands in registers.  The operands are
// pseudo-random bf16 values of magnitude 0.5 .. 1 with random signs: what the matrix pipes sustain
// depends on the data (the part is power-limited), and constants would flatter the figure by a fifth.
__global__ __launch_bounds__(512) void mfma_probe_kernel(float* sink, int n_groups) {
  hbp::Frag a, b;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t h = (uint32_t)(blockIdx.x * 512 + threadIdx.x) * 4u + (uint32_t)i;
    h *= 2654435761u;
    h ^= h >> 15;
    h *= 2246822519u;
    h ^= h >> 13;
    a.w[i] = (h & 0x807f807fu) | 0x3f003f00u;
    h *= 3266489917u;
    h ^= h >> 16;
    b.w[i] = (h & 0x807f807fu) | 0x3f003f00u;
  }
  hbp::f32x16 c[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) c[j][i] = 0.f;
  for (int it = 0; it < n_groups; ++it) {
#pragma unroll
    for (int j = 0; j < 4; ++j) c[j] = hbp::mfma32(a.v, b.v, c[j]);
  }
  sink[blockIdx.x * blockDim.x + threadIdx.x] = c[0][3] + c[1][3] + c[2][3] + c[3][3];
}
}  // namespace

extern "C" hbp_status hbp_mfma_probe(int32_t n_cu, int32_t mfma_per_wave, float* sink, void* stream) {
  if (!sink || n_cu < 1 || mfma_per_wave < 4) return HBP_ERR_INVALID_ARG;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(n_cu), dim3(512), 0, static_cast<hipStream_t>(stream), sink,
                     mfma_per_wave / 4);
  return hipGetLastError() == hipSuccess ? HBP_OK : HBP_ERR_DEVICE;
}

extern "C" hbp_status hbp_set_kernel_events(int32_t which, void* start_event, void* stop_event) {
  if (which != HBP_FWD && which != HBP_BWD && which != HBP_BWD_DQ && which != HBP_LOSS) return HBP_ERR_INVALID_ARG;
  if ((start_event == nullptr) != (stop_event == nullptr)) return HBP_ERR_INVALID_ARG;
  g_events[which][0] = static_cast<hipEvent_t>(start_event);
  g_events[which][1] = static_cast<hipEvent_t>(stop_event);
  return HBP_OK;
}

extern "C" hbp_status hbp_tile_rows(int32_t d_qk, int32_t d_v, int32_t which, int32_t* rows_out) {
  if (!rows_out) return HBP_ERR_INVALID_ARG;
  if (which != HBP_FWD && which != HBP_BWD) return HBP_ERR_INVALID_ARG;
  if (!dims_supported(d_qk, d_v)) return HBP_ERR_UNSUPPORTED;
  *rows_out = kTileRows;
  return HBP_OK;
}

extern "C" hbp_status hbp_fwd_tile_rows(const hbp_attn_desc* desc, int32_t* rows_out) {
  if (!desc || !rows_out) return HBP_ERR_INVALID_ARG;
  if (desc->n_q_heads <= 0 || desc->n_kv_heads <= 0) return HBP_ERR_INVALID_ARG;
  if (desc->n_q_heads % desc->n_kv_heads) return HBP_ERR_SHAPE;
  if (!dims_supported(desc->d_qk, desc->d_v)) return HBP_ERR_UNSUPPORTED;
  *rows_out = (desc->n_q_heads / desc->n_kv_heads) % 2 == 1 ? 2 * kTileRows : kTileRows;
  return HBP_OK;
}

extern "C" hbp_status hbp_workspace_bytes(const hbp_attn_desc* desc, int32_t which, size_t* bytes_out) {
  if (!bytes_out) return HBP_ERR_INVALID_ARG;
  if (which != HBP_FWD && which != HBP_BWD) return HBP_ERR_INVALID_ARG;
  Strides st;
  const hbp_status s = check_desc(desc, &st);
  if (s != HBP_OK) return s;
  *bytes_out = which == HBP_FWD ? kCounterBytes : bwd_layout(desc).total;
  return HBP_OK;
}

extern "C" hbp_status hbp_profile_capacity(const hbp_attn_desc* desc, int32_t which, int32_t* n_records_out) {
  if (!n_records_out) return HBP_ERR_INVALID_ARG;
  if (which != HBP_FWD && which != HBP_BWD && which != HBP_BWD_DQ) return HBP_ERR_INVALID_ARG;
  Strides st;
  const hbp_status s = check_desc(desc, &st);
  if (s != HBP_OK) return s;
  *n_records_out = kNumCU * (which == HBP_BWD ? 1 : 2);
  return HBP_OK;
}

extern "C" hbp_status hbp_varlen_attn_fwd(const hbp_attn_desc* desc, const void* q, const void* k,
                                          const void* v, const int32_t* cu_seqlens,
                                          const hbp_tile* q_tiles, int32_t n_q_tiles, void* o,
                                          float* lse, void* workspace, size_t workspace_bytes,
                                          hbp_profile_rec* profile, void* stream) {
  Strides st;
  const hbp_status s = check_desc(desc, &st);
  if (s != HBP_OK) return s;
  if (n_q_tiles < 0 || !item_count_fits(n_q_tiles, desc->n_q_heads)) return HBP_ERR_INVALID_ARG;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < kCounterBytes)
    return HBP_ERR_WORKSPACE;
  if (desc->total_tokens == 0 || n_q_tiles == 0) return HBP_OK;
  if (!q || !k || !v || !o || !lse || !cu_seqlens || !q_tiles) return HBP_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return HBP_ERR_INVALID_ARG;

  hbp::FwdParams p;
  std::memset(&p, 0, sizeof(p));
  p.q = static_cast<const uint16_t*>(q);
  p.k = static_cast<const uint16_t*>(k);
  p.v = static_cast<const uint16_t*>(v);
  p.o = static_cast<uint16_t*>(o);
  p.lse = lse;
  p.cu = cu_seqlens;
  p.tiles = q_tiles;
  p.n_tiles = n_q_tiles;
  p.n_samples = desc->n_samples;
  p.T = desc->total_tokens;
  p.Hq = desc->n_q_heads;
  p.Hkv = desc->n_kv_heads;
  p.g = desc->n_q_heads / desc->n_kv_heads;
  p.q_st = st.q_st; p.q_sh = st.q_sh; p.k_st = st.k_st; p.k_sh = st.k_sh;
  p.v_st = st.v_st; p.v_sh = st.v_sh; p.o_st = st.o_st; p.o_sh = st.o_sh;
  p.scale_log2 = resolve_scale(desc) * 1.4426950408889634f;
  p.counter = static_cast<int32_t*>(workspace);
  p.prof = profile;
  p.n_split = hbp::heads_split(p.Hkv, p.g % 2 == 0 ? p.g / 2 : p.g);  // even groups: items are pairs of heads

  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (hbp::launch_zero_counters(p.counter, hs) != 0) return HBP_ERR_DEVICE;
  if (hbp::launch_fwd(desc->d_qk, desc->d_v, p, desc->fwd_tile_rows ? desc->fwd_tile_rows : kTileRows, kNumCU, hs, g_events[HBP_FWD][0], g_events[HBP_FWD][1]) != 0) return HBP_ERR_DEVICE;
  return HBP_OK;
}

namespace {

// Scratch of the entry point that takes no workspace: one array per GPU, held from the moment the
// library's code is loaded on that GPU until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; the device address is looked up once per device (static_scratch).
constexpr size_t kStaticScratchBytes = HBP_STATIC_SCRATCH_BYTES;  // 64 MiB of per-row scalars + counters
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (each GPU has its own copy at its own address).
hbp_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HBP_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return HBP_ERR_DEVICE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return HBP_OK;
}

// Shared by both backward entry points.  use_static: the workspace is the library's static array.
hbp_status bwd_impl(const hbp_attn_desc* desc, const void* q, const void* k, const void* v, const void* o,
                    const float* lse, const void* d_o, const int32_t* cu_seqlens, const hbp_tile* q_tiles,
                    int32_t n_q_tiles, const hbp_tile* kv_tiles, int32_t n_kv_tiles, void* dq, void* dk, void* dv,
                    void* workspace, size_t workspace_bytes, bool use_static, hbp_profile_rec* profile,
                    hbp_profile_rec* profile_dq, void* stream) {
  Strides st;
  const hbp_status s = check_desc(desc, &st);
  if (s != HBP_OK) return s;
  if (n_kv_tiles < 0 || n_q_tiles < 0) return HBP_ERR_INVALID_ARG;
  if (!item_count_fits(n_q_tiles, desc->n_q_heads) || !item_count_fits(n_kv_tiles, desc->n_q_heads))
    return HBP_ERR_INVALID_ARG;
  const BwdLayout lay = bwd_layout(desc);
  if (use_static) {
    if (lay.total > kStaticScratchBytes) return HBP_ERR_STATIC_LIMIT;
  } else if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < lay.total) {
    return HBP_ERR_WORKSPACE;
  }
  if (desc->total_tokens == 0) return HBP_OK;
  if (!q || !k || !v || !o || !lse || !d_o || !cu_seqlens || !dq || !dk || !dv) return HBP_ERR_INVALID_ARG;
  if ((n_kv_tiles > 0 && !kv_tiles) || (n_q_tiles > 0 && !q_tiles)) return HBP_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) ||
      !aligned16(dq) || !aligned16(dk) || !aligned16(dv))
    return HBP_ERR_INVALID_ARG;

  hbp::BwdParams p;
  std::memset(&p, 0, sizeof(p));
  p.q = static_cast<const uint16_t*>(q);
  p.k = static_cast<const uint16_t*>(k);
  p.v = static_cast<const uint16_t*>(v);
  p.o = static_cast<const uint16_t*>(o);
  p.d_o = static_cast<const uint16_t*>(d_o);
  p.lse = lse;
  p.dq = static_cast<uint16_t*>(dq);
  p.dk = static_cast<uint16_t*>(dk);
  p.dv = static_cast<uint16_t*>(dv);
  if (use_static) {
    const hbp_status ss = static_scratch(&workspace);
    if (ss != HBP_OK) return ss;
  }
  char* ws = static_cast<char*>(workspace);
  p.counter = reinterpret_cast<int32_t*>(ws);
  p.counter_dq = reinterpret_cast<int32_t*>(ws + 1024);
  p.D = reinterpret_cast<float*>(ws + lay.d_off);
  p.lse2 = reinterpret_cast<float*>(ws + lay.lse2_off);
  p.cu = cu_seqlens;
  p.tiles = kv_tiles;
  p.n_tiles = n_kv_tiles;
  p.q_tiles = q_tiles;
  p.n_q_tiles = n_q_tiles;
  p.prof_dq = profile_dq;
  p.n_samples = desc->n_samples;
  p.T = desc->total_tokens;
  p.Hq = desc->n_q_heads;
  p.Hkv = desc->n_kv_heads;
  p.g = desc->n_q_heads / desc->n_kv_heads;
  p.q_st = st.q_st; p.q_sh = st.q_sh; p.k_st = st.k_st; p.k_sh = st.k_sh;
  p.v_st = st.v_st; p.v_sh = st.v_sh; p.o_st = st.o_st; p.o_sh = st.o_sh;
  p.scale = resolve_scale(desc);
  p.scale_log2 = p.scale * 1.4426950408889634f;
  p.prof = profile;
  p.n_split = hbp::heads_split(p.Hkv, p.g);
  p.n_split_dq = p.n_split;
  p.dk_part = reinterpret_cast<float*>(ws + lay.dk_part_off);
  p.dv_part = reinterpret_cast<float*>(ws + lay.dv_part_off);

  const int grid_dkdv = grid_for((int64_t)n_kv_tiles * p.Hkv * p.n_split, 1);
  const int grid_dq = grid_for((int64_t)n_q_tiles * p.Hq, 2);
  hipEvent_t ev[4] = {g_events[HBP_BWD][0], g_events[HBP_BWD][1], g_events[HBP_BWD_DQ][0], g_events[HBP_BWD_DQ][1]};
  if (hbp::launch_bwd(desc->d_qk, desc->d_v, p, grid_dq, grid_dkdv, static_cast<hipStream_t>(stream), ev) != 0)
    return HBP_ERR_DEVICE;
  return HBP_OK;
}

}  // namespace

extern "C" hbp_status hbp_varlen_attn_bwd(const hbp_attn_desc* desc, const void* q, const void* k,
                                          const void* v, const void* o, const float* lse,
                                          const void* d_o, const int32_t* cu_seqlens,
                                          const hbp_tile* q_tiles, int32_t n_q_tiles,
                                          const hbp_tile* kv_tiles, int32_t n_kv_tiles, void* dq,
                                          void* dk, void* dv, void* workspace,
                                          size_t workspace_bytes, hbp_profile_rec* profile,
                                          hbp_profile_rec* profile_dq, void* stream) {
  return bwd_impl(desc, q, k, v, o, lse, d_o, cu_seqlens, q_tiles, n_q_tiles, kv_tiles, n_kv_tiles, dq, dk, dv,
                  workspace, workspace_bytes, false, profile, profile_dq, stream);
}

extern "C" hbp_status hbp_varlen_attn_bwd_static(const hbp_attn_desc* desc, const void* q, const void* k,
                                                 const void* v, const void* o, const float* lse,
                                                 const void* d_o, const int32_t* cu_seqlens,
                                                 const hbp_tile* q_tiles, int32_t n_q_tiles,
                                                 const hbp_tile* kv_tiles, int32_t n_kv_tiles, void* dq,
                                                 void* dk, void* dv, hbp_profile_rec* profile,
                                                 hbp_profile_rec* profile_dq, void* stream) {
  return bwd_impl(desc, q, k, v, o, lse, d_o, cu_seqlens, q_tiles, n_q_tiles, kv_tiles, n_kv_tiles, dq, dk, dv,
                  nullptr, 0, true, profile, profile_dq, stream);
}
