// The extern "C" boundary declared in include/kvh.h: argument validation on the host, then
// kernel launches on the caller's stream.  No allocation, no state, no synchronisation.
#include "kvh_common.hpp"

namespace kvh {

namespace {

constexpr int kMaxItems = 65535;   // gridDim.z
constexpr int kMaxLayers = 32767;  // gridDim.y = 2 * l

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(int l, int n, int c) {
  if (l < 1 || l > kMaxLayers || n < 1 || c < kGroup || c % kGroup != 0) return KVH_E_SHAPE;
  return KVH_OK;
}

int check_view(const kvh_kv_view* v) {
  if (v == nullptr || v->k == nullptr || v->v == nullptr) return KVH_E_ARG;
  if (v->layer_stride < 0 || v->token_stride < 0) return KVH_E_ARG;
  if (!aligned16(v->k) || !aligned16(v->v) || v->layer_stride % 8 != 0 || v->token_stride % 8 != 0) return KVH_E_ALIGN;
  return KVH_OK;
}

// A destination whose rows are closer together than c elements would have rows written over each other.
int check_dst_view(const kvh_kv_view* v, int c) {
  if (int rc = check_view(v)) return rc;
  return v->token_stride < c ? KVH_E_ARG : KVH_OK;
}

__device__ __forceinline__ void uintx4_nt_store(uint4* p, const uint4& v) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 x = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(x, reinterpret_cast<__attribute__((address_space(1))) u32x4*>(reinterpret_cast<uintptr_t>(p)));
}

__global__ __launch_bounds__(kBlockThreads) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                              size_t n16) {
  size_t i = (size_t)blockIdx.x * (kBlockThreads * 4) + threadIdx.x;
  uint4 r[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (i + (size_t)u * kBlockThreads < n16) r[u] = src[i + (size_t)u * kBlockThreads];
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (i + (size_t)u * kBlockThreads < n16) dst[i + (size_t)u * kBlockThreads] = r[u];
}

// Traffic generator with a chosen read : write mix and no arithmetic: a thread handles units of R 16-byte loads and
// W 16-byte stores (each a full 1 KiB per wave), 4 units per thread.  What is stored depends on what was loaded, and
// a pure read stream stores one word only under a condition that never holds, so no access can be optimised away.
template <int R, int W>
__global__ __launch_bounds__(kBlockThreads) void stream_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                                size_t n_units) {
  constexpr int U = 4;
  const size_t base = (size_t)blockIdx.x * (kBlockThreads * U);
  uint4 acc = make_uint4(threadIdx.x, 1u, 2u, 3u);
  uint4 r[U][R > 0 ? R : 1];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t unit = base + (size_t)u * kBlockThreads + threadIdx.x;
    if (unit < n_units) {
#pragma unroll
      for (int j = 0; j < R; ++j) r[u][j] = src[(unit - threadIdx.x) * R + (size_t)j * kBlockThreads + threadIdx.x];
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t unit = base + (size_t)u * kBlockThreads + threadIdx.x;
    if (unit < n_units) {
#pragma unroll
      for (int j = 0; j < R; ++j) {
        acc.x ^= r[u][j].x; acc.y ^= r[u][j].y; acc.z ^= r[u][j].z; acc.w ^= r[u][j].w;
      }
#pragma unroll
      for (int j = 0; j < W; ++j) {
        uintx4_nt_store(&dst[(unit - threadIdx.x) * W + (size_t)j * kBlockThreads + threadIdx.x], acc);
      }
    }
  }
  if (W == 0 && (acc.x & acc.y & acc.z & acc.w) == 0xfffffffeu) dst[0] = acc;  // never true in practice: keeps the loads alive
}

template <int R, int W>
int launch_stream(void* dst, const void* src, size_t n_units, hipStream_t stream) {
  const size_t per_block = (size_t)kBlockThreads * 4;
  const size_t blocks = (n_units + per_block - 1) / per_block;
  if (blocks == 0 || blocks > 0x7fffffffu) return KVH_E_SIZE;
  hipLaunchKernelGGL((stream_kernel<R, W>), dim3((unsigned)blocks), dim3(kBlockThreads), 0, stream,
                     static_cast<uint4*>(dst), static_cast<const uint4*>(src), n_units);
  KVH_HIP_CHECK_LAUNCH();
  return KVH_OK;
}

}  // namespace
}  // namespace kvh

using namespace kvh;

// ---- self-test of the short quotient forms ------------------------------------------------------
// Every finite fp32 value from 2^-100 up (what the range of a non-degenerate group of finite values can be) goes
// through range_over_levels and levels_over_range and through the divisions they stand for; out[0..2] count the
// values where r / L differs at 8 / 4 / 2 bits, out[3..5] where L / r does.
namespace {
constexpr uint32_t kSelftestFirst = 0x0d800000u;  // 2^-100
constexpr uint32_t kSelftestEnd = 0x7f800000u;    // +infinity, not included

__device__ __forceinline__ bool same_float(float a, float b) { return __float_as_uint(a) == __float_as_uint(b); }

template <int BITS>
__device__ __forceinline__ void selftest_one(float r, unsigned& bad_scale, unsigned& bad_inv) {
  constexpr float L = float((1 << BITS) - 1);
  // the divisor and dividend reach the divisions through an opaque copy so that no rewrite can merge the two sides
  float ro = r, Lo = L;
  asm volatile("" : "+v"(ro), "+v"(Lo));
  bad_scale += same_float(range_over_levels<BITS>(r), ro / Lo) ? 0u : 1u;
  bad_inv += same_float(levels_over_range<BITS>(r), Lo / ro) ? 0u : 1u;
}

__global__ void __launch_bounds__(kBlockThreads) selftest_division_kernel(unsigned long long* out) {
  unsigned bad[6] = {0, 0, 0, 0, 0, 0};
  const uint64_t stride = (uint64_t)gridDim.x * kBlockThreads;
  for (uint64_t u = kSelftestFirst + (uint64_t)blockIdx.x * kBlockThreads + threadIdx.x; u < kSelftestEnd; u += stride) {
    const float r = __uint_as_float((uint32_t)u);
    selftest_one<8>(r, bad[0], bad[3]);
    selftest_one<4>(r, bad[1], bad[4]);
    selftest_one<2>(r, bad[2], bad[5]);
  }
#pragma unroll
  for (int k = 0; k < 6; ++k)
    if (bad[k] != 0) atomicAdd(&out[k], (unsigned long long)bad[k]);
}
}  // namespace

static int launch_selftest_division(unsigned long long* mismatches_dev, hipStream_t stream) {
  hipLaunchKernelGGL(selftest_division_kernel, dim3(8192), dim3(kBlockThreads), 0, stream, mismatches_dev);
  return hipGetLastError() == hipSuccess ? KVH_OK : KVH_E_HIP;
}

namespace kvh {
namespace {
thread_local TimingEvents t_timing = {nullptr, nullptr};
}
TimingEvents take_timing_events() {
  const TimingEvents ev = t_timing;
  t_timing = TimingEvents{nullptr, nullptr};
  return ev;
}
}  // namespace kvh

extern "C" {

int kvh_num_levels(void) { return 3; }

int kvh_level_bits(int level) { return level_bits(level); }

size_t kvh_blob_size(int l, int n_tokens, int c, int level) {
  int bits = level_bits(level);
  if (bits < 0 || check_shape(l, n_tokens, c) != KVH_OK) return 0;
  return kHeaderBytes + (size_t)l * layer_geom(n_tokens, c, bits).layer_bytes();
}

int kvh_encode(const kvh_kv_view* kv, kvh_dtype dt, int l, int N, int c, int level, void* blob_dev, size_t blob_cap,
               void* stream) {
  if (blob_dev == nullptr || (dt != KVH_F16 && dt != KVH_BF16)) return KVH_E_ARG;
  if (int rc = check_view(kv)) return rc;
  if (level_bits(level) < 0) return KVH_E_LEVEL;
  if (int rc = check_shape(l, N, c)) return rc;
  if (blob_cap < kvh_blob_size(l, N, c, level)) return KVH_E_SIZE;
  if (!aligned16(blob_dev)) return KVH_E_ALIGN;
  EncodeParams a{};
  a.items = nullptr;
  a.one = kvh_enc_item{blob_dev, 0, N, level};
  a.k = static_cast<const uint16_t*>(kv->k);
  a.v = static_cast<const uint16_t*>(kv->v);
  a.layer_stride = kv->layer_stride;
  a.token_stride = kv->token_stride;
  a.l = l;
  a.c = c;
  a.split = kNoSplit;
  return launch_encode(a, dt, 1, N, static_cast<hipStream_t>(stream));
}

int kvh_encode_chunked(const kvh_kv_view* kv, kvh_dtype dt, int l, int N, int c, int chunk, const int8_t* levels,
                       void* blobs_dev, const size_t* blob_offsets, size_t cap, void* stream) {
  if (blobs_dev == nullptr || levels == nullptr || blob_offsets == nullptr || (dt != KVH_F16 && dt != KVH_BF16))
    return KVH_E_ARG;
  if (int rc = check_view(kv)) return rc;
  if (int rc = check_shape(l, N, c)) return rc;
  if (chunk < kGroup || chunk % kGroup != 0) return KVH_E_SHAPE;
  if (!aligned16(blobs_dev)) return KVH_E_ALIGN;
  const int n_chunks = (N + chunk - 1) / chunk;
  // validate everything before the first launch
  for (int i = 0; i < n_chunks; ++i) {
    const int n = (i + 1) * (int64_t)chunk <= N ? chunk : N - i * chunk;
    if (level_bits(levels[i]) < 0) return KVH_E_LEVEL;
    if (blob_offsets[i] % 16 != 0) return KVH_E_ALIGN;
    const size_t need = kvh_blob_size(l, n, c, levels[i]);
    if (blob_offsets[i] > cap || cap - blob_offsets[i] < need) return KVH_E_SIZE;
  }
  EncodeParams a{};
  a.items = nullptr;
  a.k = static_cast<const uint16_t*>(kv->k);
  a.v = static_cast<const uint16_t*>(kv->v);
  a.layer_stride = kv->layer_stride;
  a.token_stride = kv->token_stride;
  a.l = l;
  a.c = c;
  a.split = kNoSplit;
  // the descriptors ride in the kernel arguments, kInlineItems chunks per launch
  for (int i0 = 0; i0 < n_chunks; i0 += kInlineItems) {
    const int cnt = n_chunks - i0 < kInlineItems ? n_chunks - i0 : kInlineItems;
    for (int j = 0; j < cnt; ++j) {
      const int i = i0 + j;
      const int n = (i + 1) * (int64_t)chunk <= N ? chunk : N - i * chunk;
      a.inline_items[j] = kvh_enc_item{static_cast<uint8_t*>(blobs_dev) + blob_offsets[i], (int64_t)i * chunk, n, levels[i]};
    }
    a.n_inline = cnt;
    if (int rc = launch_encode(a, dt, cnt, chunk, static_cast<hipStream_t>(stream))) return rc;
  }
  return KVH_OK;
}

int kvh_encode_batch(const kvh_enc_item* items_dev, int n_items, int max_tokens_per_item, kvh_dtype dt, int l, int c,
                     const kvh_kv_view* src, void* stream) {
  if (items_dev == nullptr || n_items < 1 || n_items > kMaxItems || (dt != KVH_F16 && dt != KVH_BF16)) return KVH_E_ARG;
  if (int rc = check_view(src)) return rc;
  if (int rc = check_shape(l, max_tokens_per_item, c)) return rc;
  EncodeParams a{};
  a.items = items_dev;
  a.k = static_cast<const uint16_t*>(src->k);
  a.v = static_cast<const uint16_t*>(src->v);
  a.layer_stride = src->layer_stride;
  a.token_stride = src->token_stride;
  a.l = l;
  a.c = c;
  a.split = kNoSplit;
  return launch_encode(a, dt, n_items, max_tokens_per_item, static_cast<hipStream_t>(stream));
}

int kvh_decode(const void* blob_dev, kvh_dtype dt, int l, int n_tokens, int c, int level, const kvh_kv_view* dst,
               int64_t dst_token0, const int32_t* page_table_dev, int block_tokens, int32_t* status_dev, void* stream) {
  if (blob_dev == nullptr || (dt != KVH_F16 && dt != KVH_BF16) || dst_token0 < 0) return KVH_E_ARG;
  if (int rc = check_dst_view(dst, c)) return rc;
  if (level_bits(level) < 0) return KVH_E_LEVEL;
  if (int rc = check_shape(l, n_tokens, c)) return rc;
  if (page_table_dev != nullptr && block_tokens < 1) return KVH_E_ARG;
  if (dst_token0 + n_tokens > INT32_MAX) return KVH_E_ARG;
  if (!aligned16(blob_dev)) return KVH_E_ALIGN;
  DecodeParams a{};
  a.items = nullptr;
  a.one = kvh_item{blob_dev, n_tokens, level, dst_token0, page_table_dev};
  a.k = static_cast<uint16_t*>(dst->k);
  a.v = static_cast<uint16_t*>(dst->v);
  a.layer_stride = dst->layer_stride;
  a.token_stride = dst->token_stride;
  a.status = status_dev;
  a.l = l;
  a.c = c;
  a.block_tokens = page_table_dev != nullptr ? block_tokens : 1;
  a.split = kNoSplit;
  return launch_decode(a, dt, 1, n_tokens, static_cast<hipStream_t>(stream));
}

int kvh_decode_chunked(const void* blobs_dev, const size_t* blob_offsets, const int8_t* levels, kvh_dtype dt, int l, int N,
                       int c, int chunk, const kvh_kv_view* dst, int64_t dst_token0, const int32_t* page_table_dev,
                       int block_tokens, int32_t* status_dev, void* stream) {
  if (blobs_dev == nullptr || blob_offsets == nullptr || levels == nullptr || (dt != KVH_F16 && dt != KVH_BF16) ||
      dst_token0 < 0)
    return KVH_E_ARG;
  if (int rc = check_dst_view(dst, c)) return rc;
  if (int rc = check_shape(l, N, c)) return rc;
  if (chunk < kGroup || chunk % kGroup != 0) return KVH_E_SHAPE;
  if (page_table_dev != nullptr && block_tokens < 1) return KVH_E_ARG;
  if (dst_token0 + N > INT32_MAX) return KVH_E_ARG;
  if (!aligned16(blobs_dev)) return KVH_E_ALIGN;
  const int n_chunks = (N + chunk - 1) / chunk;
  for (int i = 0; i < n_chunks; ++i) {  // validate everything before the first launch
    if (level_bits(levels[i]) < 0) return KVH_E_LEVEL;
    if (blob_offsets[i] % 16 != 0) return KVH_E_ALIGN;
  }
  DecodeParams a{};
  a.items = nullptr;
  a.k = static_cast<uint16_t*>(dst->k);
  a.v = static_cast<uint16_t*>(dst->v);
  a.layer_stride = dst->layer_stride;
  a.token_stride = dst->token_stride;
  a.l = l;
  a.c = c;
  a.block_tokens = page_table_dev != nullptr ? block_tokens : 1;
  a.split = kNoSplit;
  // the descriptors ride in the kernel arguments, kInlineItems chunks per launch
  for (int i0 = 0; i0 < n_chunks; i0 += kInlineItems) {
    const int cnt = n_chunks - i0 < kInlineItems ? n_chunks - i0 : kInlineItems;
    for (int j = 0; j < cnt; ++j) {
      const int i = i0 + j;
      const int n = (i + 1) * (int64_t)chunk <= N ? chunk : N - i * chunk;
      a.inline_items[j] = kvh_item{static_cast<const uint8_t*>(blobs_dev) + blob_offsets[i], n, levels[i],
                                   dst_token0 + (int64_t)i * chunk, page_table_dev};
    }
    a.n_inline = cnt;
    a.status = status_dev != nullptr ? status_dev + i0 : nullptr;
    if (int rc = launch_decode(a, dt, cnt, chunk, static_cast<hipStream_t>(stream))) return rc;
  }
  return KVH_OK;
}

int kvh_decode_batch(const kvh_item* items_dev, int n_items, int max_tokens_per_item, kvh_dtype dt, int l, int c,
                     const kvh_kv_view* dst, int block_tokens, int32_t* status_dev, void* stream) {
  if (items_dev == nullptr || n_items < 1 || n_items > kMaxItems || (dt != KVH_F16 && dt != KVH_BF16) ||
      block_tokens < 1)
    return KVH_E_ARG;
  if (int rc = check_dst_view(dst, c)) return rc;
  if (int rc = check_shape(l, max_tokens_per_item, c)) return rc;
  DecodeParams a{};
  a.items = items_dev;
  a.k = static_cast<uint16_t*>(dst->k);
  a.v = static_cast<uint16_t*>(dst->v);
  a.layer_stride = dst->layer_stride;
  a.token_stride = dst->token_stride;
  a.status = status_dev;
  a.l = l;
  a.c = c;
  a.block_tokens = block_tokens;
  a.split = kNoSplit;
  return launch_decode(a, dt, n_items, max_tokens_per_item, static_cast<hipStream_t>(stream));
}

int kvh_kept_tokens(int N, int sink, int window) {
  if (N < 1 || sink < 0 || window < 0 || (int64_t)sink + window < 1) return 0;
  return (int64_t)sink + window >= N ? N : sink + window;
}

int kvh_encode_kept(const kvh_kv_view* kv, kvh_dtype dt, int l, int N, int c, int sink, int window, int level,
                    void* blob_dev, size_t blob_cap, void* stream) {
  if (blob_dev == nullptr || (dt != KVH_F16 && dt != KVH_BF16)) return KVH_E_ARG;
  if (int rc = check_view(kv)) return rc;
  if (level_bits(level) < 0) return KVH_E_LEVEL;
  const int n = kvh_kept_tokens(N, sink, window);
  if (n < 1) return KVH_E_SHAPE;
  if (int rc = check_shape(l, n, c)) return rc;
  if (blob_cap < kvh_blob_size(l, n, c, level)) return KVH_E_SIZE;
  if (!aligned16(blob_dev)) return KVH_E_ALIGN;
  EncodeParams a{};
  a.items = nullptr;
  a.one = kvh_enc_item{blob_dev, 0, n, level};
  a.k = static_cast<const uint16_t*>(kv->k);
  a.v = static_cast<const uint16_t*>(kv->v);
  a.layer_stride = kv->layer_stride;
  a.token_stride = kv->token_stride;
  a.l = l;
  a.c = c;
  const bool drops = n < N;
  a.split = drops ? sink : kNoSplit;  // kept token t >= sink is source token t + (N - window - sink)
  a.jump = drops ? (int64_t)N - window - sink : 0;
  a.hdr_orig_tokens = (uint32_t)N;
  a.hdr_sink = (uint32_t)sink;
  a.hdr_window = (uint32_t)window;
  return launch_encode(a, dt, 1, n, static_cast<hipStream_t>(stream));
}

int kvh_decode_kept(const void* blob_dev, kvh_dtype dt, int l, int N, int c, int sink, int window, int level,
                    const kvh_kv_view* dst, int64_t dst_token0, int compact, const int32_t* page_table_dev,
                    int block_tokens, int32_t* status_dev, void* stream) {
  if (blob_dev == nullptr || (dt != KVH_F16 && dt != KVH_BF16) || dst_token0 < 0) return KVH_E_ARG;
  if (int rc = check_dst_view(dst, c)) return rc;
  if (level_bits(level) < 0) return KVH_E_LEVEL;
  const int n = kvh_kept_tokens(N, sink, window);
  if (n < 1) return KVH_E_SHAPE;
  if (int rc = check_shape(l, n, c)) return rc;
  if (page_table_dev != nullptr && block_tokens < 1) return KVH_E_ARG;
  if (dst_token0 + N > INT32_MAX) return KVH_E_ARG;
  if (!aligned16(blob_dev)) return KVH_E_ALIGN;
  DecodeParams a{};
  a.items = nullptr;
  a.one = kvh_item{blob_dev, n, level, dst_token0, page_table_dev};
  a.k = static_cast<uint16_t*>(dst->k);
  a.v = static_cast<uint16_t*>(dst->v);
  a.layer_stride = dst->layer_stride;
  a.token_stride = dst->token_stride;
  a.status = status_dev;
  a.l = l;
  a.c = c;
  a.block_tokens = page_table_dev != nullptr ? block_tokens : 1;
  const bool hops = n < N && !compact;
  a.split = hops ? sink : kNoSplit;
  a.jump = hops ? (int64_t)N - window - sink : 0;
  a.hdr_orig_tokens = (uint32_t)N;
  a.hdr_sink = (uint32_t)sink;
  a.hdr_window = (uint32_t)window;
  return launch_decode(a, dt, 1, n, static_cast<hipStream_t>(stream));
}

int kvh_transcode(const void* src_dev, kvh_dtype dt, int l, int n_tokens, int c, int level_in, int level_out,
                  void* dst_dev, size_t dst_cap, int32_t* status_dev, void* stream) {
  if (src_dev == nullptr || dst_dev == nullptr || (dt != KVH_F16 && dt != KVH_BF16)) return KVH_E_ARG;
  if (level_bits(level_in) < 0 || level_bits(level_out) < 0) return KVH_E_LEVEL;
  if (level_in == kRawLevel || level_out == kRawLevel) return KVH_E_LEVEL;  // raw blobs hold rows, not codes
  if (int rc = check_shape(l, n_tokens, c)) return rc;
  const size_t size_in = kvh_blob_size(l, n_tokens, c, level_in), size_out = kvh_blob_size(l, n_tokens, c, level_out);
  if (dst_cap < size_out) return KVH_E_SIZE;
  if (!aligned16(src_dev) || !aligned16(dst_dev)) return KVH_E_ALIGN;
  const uintptr_t s = reinterpret_cast<uintptr_t>(src_dev), d = reinterpret_cast<uintptr_t>(dst_dev);
  if (s < d + size_out && d < s + size_in) return KVH_E_ARG;  // overlapping buffers
  TranscodeParams a{};
  a.items = nullptr;
  a.one = kvh_tc_item{src_dev, dst_dev, n_tokens, level_in, level_out, 0};
  a.status = status_dev;
  a.l = l;
  a.c = c;
  return launch_transcode(a, dt, 1, n_tokens, static_cast<hipStream_t>(stream));
}

int kvh_transcode_batch(const kvh_tc_item* items_dev, int n_items, int max_tokens_per_item, kvh_dtype dt, int l, int c,
                        int32_t* status_dev, void* stream) {
  if (items_dev == nullptr || n_items < 1 || n_items > kMaxItems || (dt != KVH_F16 && dt != KVH_BF16)) return KVH_E_ARG;
  if (int rc = check_shape(l, max_tokens_per_item, c)) return rc;
  TranscodeParams a{};
  a.items = items_dev;
  a.status = status_dev;
  a.l = l;
  a.c = c;
  return launch_transcode(a, dt, n_items, max_tokens_per_item, static_cast<hipStream_t>(stream));
}

int kvh_encode_kept_batch(const kvh_kept_enc_item* items_dev, int n_items, int max_kept_tokens_per_item, kvh_dtype dt,
                          int l, int c, const kvh_kv_view* src, void* stream) {
  if (items_dev == nullptr || n_items < 1 || n_items > kMaxItems || (dt != KVH_F16 && dt != KVH_BF16)) return KVH_E_ARG;
  if (int rc = check_view(src)) return rc;
  if (int rc = check_shape(l, max_kept_tokens_per_item, c)) return rc;
  EncodeParams a{};
  a.kept_items = items_dev;
  a.k = static_cast<const uint16_t*>(src->k);
  a.v = static_cast<const uint16_t*>(src->v);
  a.layer_stride = src->layer_stride;
  a.token_stride = src->token_stride;
  a.l = l;
  a.c = c;
  a.split = kNoSplit;
  return launch_encode(a, dt, n_items, max_kept_tokens_per_item, static_cast<hipStream_t>(stream));
}

int kvh_decode_kept_batch(const kvh_kept_item* items_dev, int n_items, int max_tokens_per_item, kvh_dtype dt, int l,
                          int c, const kvh_kv_view* dst, int block_tokens, int32_t* status_dev, void* stream) {
  if (items_dev == nullptr || n_items < 1 || n_items > kMaxItems || (dt != KVH_F16 && dt != KVH_BF16) ||
      block_tokens < 1)
    return KVH_E_ARG;
  if (int rc = check_dst_view(dst, c)) return rc;
  if (int rc = check_shape(l, max_tokens_per_item, c)) return rc;
  DecodeParams a{};
  a.kept_items = items_dev;
  a.k = static_cast<uint16_t*>(dst->k);
  a.v = static_cast<uint16_t*>(dst->v);
  a.layer_stride = dst->layer_stride;
  a.token_stride = dst->token_stride;
  a.status = status_dev;
  a.l = l;
  a.c = c;
  a.block_tokens = block_tokens;
  a.split = kNoSplit;
  return launch_decode(a, dt, n_items, max_tokens_per_item, static_cast<hipStream_t>(stream));
}

int kvh_copy_probe(void* dst_dev, const void* src_dev, size_t bytes, void* stream) {
  if (dst_dev == nullptr || src_dev == nullptr || bytes == 0) return KVH_E_ARG;
  if (bytes % 16 != 0 || !aligned16(dst_dev) || !aligned16(src_dev)) return KVH_E_ALIGN;
  const size_t n16 = bytes / 16;
  const size_t per_block = (size_t)kBlockThreads * 4;
  const size_t blocks = (n16 + per_block - 1) / per_block;
  if (blocks > 0x7fffffffu) return KVH_E_SIZE;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(kBlockThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<uint4*>(dst_dev), static_cast<const uint4*>(src_dev), n16);
  KVH_HIP_CHECK_LAUNCH();
  return KVH_OK;
}

int kvh_stream_probe(void* dst_dev, const void* src_dev, size_t n_units, int reads_per_unit, int writes_per_unit,
                     void* stream) {
  // whole groups of 256 units only: the j-th access of a group is laid out behind the (j-1)-th of all its threads
  if (dst_dev == nullptr || src_dev == nullptr || n_units == 0 || n_units % kBlockThreads != 0) return KVH_E_ARG;
  if (!aligned16(dst_dev) || !aligned16(src_dev)) return KVH_E_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  switch (reads_per_unit * 16 + writes_per_unit) {
    case 1 * 16 + 0: return launch_stream<1, 0>(dst_dev, src_dev, n_units, s);
    case 0 * 16 + 1: return launch_stream<0, 1>(dst_dev, src_dev, n_units, s);
    case 1 * 16 + 1: return launch_stream<1, 1>(dst_dev, src_dev, n_units, s);
    case 1 * 16 + 2: return launch_stream<1, 2>(dst_dev, src_dev, n_units, s);
    case 1 * 16 + 4: return launch_stream<1, 4>(dst_dev, src_dev, n_units, s);
    case 1 * 16 + 8: return launch_stream<1, 8>(dst_dev, src_dev, n_units, s);
    case 2 * 16 + 1: return launch_stream<2, 1>(dst_dev, src_dev, n_units, s);
    case 4 * 16 + 1: return launch_stream<4, 1>(dst_dev, src_dev, n_units, s);
    case 8 * 16 + 1: return launch_stream<8, 1>(dst_dev, src_dev, n_units, s);
    default: return KVH_E_ARG;
  }
}

int kvh_time_next_launch(void* start_event, void* stop_event) {
  if (start_event == nullptr || stop_event == nullptr) return KVH_E_ARG;
  kvh::t_timing = kvh::TimingEvents{static_cast<hipEvent_t>(start_event), static_cast<hipEvent_t>(stop_event)};
  return KVH_OK;
}

int kvh_selftest_division(uint64_t* mismatches_dev, void* stream) {
  if (mismatches_dev == nullptr || (reinterpret_cast<uintptr_t>(mismatches_dev) & 7u) != 0) return KVH_E_ARG;
  return launch_selftest_division(reinterpret_cast<unsigned long long*>(mismatches_dev),
                                  static_cast<hipStream_t>(stream));
}

const char* kvh_strerror(int status) {
  switch (status) {
    case KVH_OK: return "ok";
    case KVH_E_ARG: return "bad argument (null pointer, dtype, offset, block size or item count)";
    case KVH_E_LEVEL: return "level outside 0..3 (or the raw level where only quantised levels are allowed)";
    case KVH_E_SHAPE: return "bad shape (l, n >= 1; c and chunk multiples of 128)";
    case KVH_E_SIZE: return "blob capacity too small";
    case KVH_E_ALIGN: return "pointer or stride breaks the 16-byte alignment rule";
    case KVH_E_HIP: return "kernel launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
