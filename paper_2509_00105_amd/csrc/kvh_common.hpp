// Shared pieces of the HIP implementation: blob geometry, the 16-bit float conversions and
// the per-group parameters.  gfx950 only.  Nothing here is used by the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/kvh.h"

#include <cstddef>

// The kernels read job descriptors as raw 16-byte words and the binding builds them as packed records:
// the layouts below are part of the ABI.
static_assert(sizeof(kvh_enc_item) == 24 && offsetof(kvh_enc_item, src_token0) == 8 &&
                  offsetof(kvh_enc_item, n_tokens) == 16 && offsetof(kvh_enc_item, level) == 20,
              "kvh_enc_item layout");
static_assert(sizeof(kvh_item) == 32 && offsetof(kvh_item, n_tokens) == 8 && offsetof(kvh_item, level) == 12 &&
                  offsetof(kvh_item, dst_token0) == 16 && offsetof(kvh_item, page_table) == 24,
              "kvh_item layout");
static_assert(sizeof(kvh_kept_enc_item) == 32 && offsetof(kvh_kept_enc_item, src_token0) == 8 &&
                  offsetof(kvh_kept_enc_item, orig_tokens) == 16 && offsetof(kvh_kept_enc_item, sink) == 20 &&
                  offsetof(kvh_kept_enc_item, window) == 24 && offsetof(kvh_kept_enc_item, level) == 28,
              "kvh_kept_enc_item layout");
static_assert(sizeof(kvh_kept_item) == 48 && offsetof(kvh_kept_item, n_tokens) == 8 && offsetof(kvh_kept_item, level) == 12 &&
                  offsetof(kvh_kept_item, dst_token0) == 16 && offsetof(kvh_kept_item, page_table) == 24 &&
                  offsetof(kvh_kept_item, orig_tokens) == 32 && offsetof(kvh_kept_item, sink) == 36 &&
                  offsetof(kvh_kept_item, window) == 40 && offsetof(kvh_kept_item, compact) == 44,
              "kvh_kept_item layout");
static_assert(sizeof(kvh_tc_item) == 32 && offsetof(kvh_tc_item, dst) == 8 && offsetof(kvh_tc_item, n_tokens) == 16 &&
                  offsetof(kvh_tc_item, level_in) == 20 && offsetof(kvh_tc_item, level_out) == 24,
              "kvh_tc_item layout");
static_assert(sizeof(kvh_load_item) == 48 && offsetof(kvh_load_item, n_tokens) == 8 && offsetof(kvh_load_item, level) == 12 &&
                  offsetof(kvh_load_item, dst_token0) == 16 && offsetof(kvh_load_item, page_table) == 24 &&
                  offsetof(kvh_load_item, orig_tokens) == 32 && offsetof(kvh_load_item, compact) == 44,
              "kvh_load_item layout");

namespace kvh {

constexpr int kGroup = 128;        // tokens per K group and channels per V group
constexpr int kHeaderBytes = 64;
constexpr int kWave = 64;          // CDNA wavefront
constexpr int kLaneCh = 8;         // channels owned by one lane: 8 x 16 bit = one 128-bit access
constexpr int kStripCh = kWave * kLaneCh;  // 512 channels = 1 KiB of 16-bit data per wave access
constexpr int kBlockThreads = 256; // 4 waves
constexpr int kWavesPerBlock = kBlockThreads / kWave;
constexpr uint32_t kMagic = 0x3148564Bu;  // "KVH1" read as a little-endian u32

constexpr int kRawLevel = 3;  // full quality: 16 bits per element, rows stored as they are, no metadata
__host__ __device__ inline int level_bits(int level) {
  return level == 0 ? 8 : level == 1 ? 4 : level == 2 ? 2 : level == kRawLevel ? 16 : -1;
}
__host__ __device__ inline size_t pad16(size_t x) { return (x + 15) & ~size_t(15); }

// Byte sizes of the four sections of one layer.
struct LayerGeom {
  size_t kmeta, codes, vmeta;  // kcodes and vcodes have the same size
  size_t row_bytes;            // one packed token row
  __host__ __device__ size_t layer_bytes() const { return kmeta + vmeta + 2 * codes; }
};

__host__ __device__ inline LayerGeom layer_geom(int n, int c, int bits) {
  LayerGeom g;
  g.row_bytes = size_t(c) * bits / 8;
  g.kmeta = bits == 16 ? 0 : pad16(size_t((n + kGroup - 1) / kGroup) * c * 4);  // the raw level has no groups
  g.codes = pad16(size_t(n) * g.row_bytes);
  g.vmeta = bits == 16 ? 0 : pad16(size_t(n) * (c / kGroup) * 4);
  return g;
}

// ---- 16-bit float <-> fp32 ------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ float t16_to_f32(uint32_t bits16) {
  if constexpr (DT == KVH_F16) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);  // v_cvt_f32_f16, exact
  } else {
    return __builtin_bit_cast(float, bits16 << 16);
  }
}

// Round to nearest even.  Finite inputs only (a NaN would not stay a NaN in the bf16 branch).
template <int DT>
__device__ __forceinline__ uint32_t f32_to_t16(float f) {
  if constexpr (DT == KVH_F16) {
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);  // v_cvt_f16_f32 under the default RNE mode
  } else {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  }
}

// ---- wave-uniform values ------------------------------------------------------------------------
// A job descriptor fetched from memory arrives in vector registers although every lane holds the same
// value.  Moving it to scalar registers lets row indices, bounds tests and base addresses derived from
// it run on the scalar unit instead of costing vector instructions per row.
__device__ __forceinline__ int32_t uniform(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint64_t uniform(uint64_t v) {
  return (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(uint32_t)v) |
         (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(uint32_t)(v >> 32)) << 32;
}
__device__ __forceinline__ int64_t uniform(int64_t v) { return (int64_t)uniform((uint64_t)v); }
template <typename T>
__device__ __forceinline__ T* uniform(T* p) {
  return reinterpret_cast<T*>(uniform((uint64_t)reinterpret_cast<uintptr_t>(p)));
}

// Load through the scalar data cache: for read-only data at a wave-uniform address (job descriptors, blob headers).
// The result arrives in scalar registers after a much shorter round trip than a vector load's, and needs no
// readfirstlane.  Only ever used for loads.
#ifndef KVH_SCALAR_DESC
#define KVH_SCALAR_DESC 1
#endif
template <typename T>
__device__ __forceinline__ T sload(const void* p) {
  return *reinterpret_cast<const __attribute__((address_space(4))) T*>(reinterpret_cast<uintptr_t>(p));
}

// ---- the two quotients of a group -------------------------------------------------------------
// scale = r / L and inv = L / r are defined as correctly rounded fp32 divisions.  The IEEE division sequence costs
// about eleven instructions; the forms below cost four (a reciprocal, a product, the exact residual by one fma, one
// corrected quotient by another) and return the same bits for every range a group of finite values can have, at
// L = 3, 15, 255.  That is a property of this chip's reciprocal instruction, established by running all of those
// ranges through both forms and both divisions (kvh_selftest_division does it in about a second, and the GPU tests
// call it).
template <int BITS>
__device__ __forceinline__ float range_over_levels(float r) {  // r / L
  constexpr float L = float((1 << BITS) - 1);
  constexpr float kInvL = 1.0f / L;
  const float q = r * kInvL;
  return __builtin_fmaf(__builtin_fmaf(-q, L, r), kInvL, q);
}
template <int BITS>
__device__ __forceinline__ float levels_over_range(float r) {  // L / r, r >= 2^-100
  // everything runs on r / 16 and L / 16 (exact scalings that leave the quotient as it is): the reciprocal of a range
  // near the top of fp32 would be subnormal otherwise
  constexpr float L16 = float((1 << BITS) - 1) * 0x1p-4f;
  const float rr = r * 0x1p-4f;
  const float y = __builtin_amdgcn_rcpf(rr);
  const float q = L16 * y;
  return __builtin_fmaf(__builtin_fmaf(-q, rr, L16), y, q);
}

// ---- group parameters -------------------------------------------------------------------------
// meta = mn | mx << 16 (raw 16-bit patterns as stored in the blob).
struct GroupParams {
  float mn;      // f32(mn)
  float scale;   // r / L, or 0 for a degenerate group
  uint32_t top;  // what code L decodes to: mx, or mn for a degenerate group
};

template <int DT, int BITS>
__device__ __forceinline__ GroupParams decode_params(uint32_t meta) {
  GroupParams p;
  p.mn = t16_to_f32<DT>(meta & 0xffffu);
  float r = t16_to_f32<DT>(meta >> 16) - p.mn;
  bool degenerate = r < 0x1p-100f;
  p.scale = degenerate ? 0.0f : range_over_levels<BITS>(r);
  p.top = degenerate ? (meta & 0xffffu) : (meta >> 16);
  return p;
}

template <int BITS>
__device__ __forceinline__ float encode_inv(float mn, float mx) {
  float r = mx - mn;
  return r < 0x1p-100f ? 0.0f : levels_over_range<BITS>(r);
}

// ---- kernel parameter blocks and launchers (defined next to their kernels) -----------------------
// Jobs that travel inside the kernel arguments: the chunked calls have their descriptors in host arrays, and
// this many per launch reach the kernel without any device memory of the library's own.
constexpr int kInlineItems = 32;

struct DecodeParams {
  const kvh_item* items;  // device array of jobs, or nullptr: decode `one` (or the inline jobs)
  const kvh_kept_item* kept_items;  // device array of jobs that may be token-dropped (then `items` is nullptr)
  kvh_item one;
  uint16_t* k;
  uint16_t* v;
  int64_t layer_stride, token_stride;  // elements
  int32_t* status;                     // nullable; indexed by item
  int l, c, block_tokens;
  int max_tokens;  // rows the grid covers per item: an item with more tokens is refused on the device
  int row_tile;  // block order chosen by the launcher: blocks of a plane that are taken before the next plane (see decode_kernel)
  // Token-dropped entries (single-item calls only): token t >= split lands `jump` rows further on,
  // and the header must carry these three words (all zero for an ordinary blob).
  int32_t split;
  int64_t jump;
  uint32_t hdr_orig_tokens, hdr_sink, hdr_window;
  int n_inline;  // > 0: the jobs are inline_items[0 .. n_inline), read from the kernel-argument segment
  kvh_item inline_items[kInlineItems];
};

struct EncodeParams {
  const kvh_enc_item* items;  // device array of jobs, or nullptr: encode `one` (or the inline jobs)
  const kvh_kept_enc_item* kept_items;  // device array of token-dropping jobs (then `items` is nullptr)
  kvh_enc_item one;
  const uint16_t* k;
  const uint16_t* v;
  int64_t layer_stride, token_stride;  // elements
  int l, c;
  int max_tokens;  // rows the grid covers per item: an item with more tokens is skipped on the device
  // Token-dropped entries (single-item calls only): token t >= split is read `jump` rows further on,
  // and the header records these three words (all zero for an ordinary blob).
  int32_t split;
  int64_t jump;
  uint32_t hdr_orig_tokens, hdr_sink, hdr_window;
  int n_inline;  // > 0: the jobs are inline_items[0 .. n_inline), read from the kernel-argument segment
  int plane_group;  // block order: (layer, K|V) planes that consecutive blocks cycle through (set by the launcher)
  kvh_enc_item inline_items[kInlineItems];
};

// Address of a member of the kernel's (single, by-value) parameter block inside the kernel-argument segment.
#define KVH_KERNARG_MEMBER(TYPE, MEMBER) \
  (reinterpret_cast<uintptr_t>(__builtin_amdgcn_kernarg_segment_ptr()) + offsetof(TYPE, MEMBER))

constexpr int32_t kNoSplit = 0x7fffffff;

// Token dropping as the kernels see it: kept token t >= split sits `jump` rows further on in the full
// entry; the three header words are what the blob records (all zero for an ordinary blob).
struct DropInfo {
  int32_t split;
  int64_t jump;
  uint32_t orig_tokens, sink, window;
};

struct TranscodeParams {
  const kvh_tc_item* items;  // device array of jobs, or nullptr: transcode `one`
  kvh_tc_item one;
  int32_t* status;           // nullable; indexed by item
  int l, c;
  int max_tokens;            // rows the grid covers per item: an item with more tokens is refused on the device
};

int launch_decode(const DecodeParams& a, int dt, int n_items, int max_tokens, hipStream_t stream);
int launch_encode(const EncodeParams& a, int dt, int n_items, int max_tokens, hipStream_t stream);
int launch_transcode(const TranscodeParams& a, int dt, int n_items, int max_tokens, hipStream_t stream);

// Launch timing.  A caller that wants the duration of one launch itself (not of the launch plus the queue
// packets that bracketing events add around it) hands over two events with kvh_time_next_launch; the next kernel
// this thread launches through launch_kernel records them at its own start and end.
struct TimingEvents {
  hipEvent_t start, stop;
};
TimingEvents take_timing_events();  // the pair set for this thread, cleared by the call

template <typename... Args>
inline void launch_kernel(void (*kernel)(Args...), dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t stream,
                          Args... args) {
  const TimingEvents ev = take_timing_events();
  if (ev.start != nullptr || ev.stop != nullptr)
    hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, ev.start, ev.stop, 0u, args...);
  else
    hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, args...);
}

#define KVH_HIP_CHECK_LAUNCH()                          \
  do {                                                  \
    if (hipGetLastError() != hipSuccess) return KVH_E_HIP; \
  } while (0)

}  // namespace kvh
