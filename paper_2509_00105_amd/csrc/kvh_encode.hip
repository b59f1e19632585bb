// Level encoder: per-group min/max, quantise to b bits, bit-pack and write the blob
// ("compress a KV-cache entry with the quantisation method at a rate"; Design section, and
// the per-channel-K / per-token-V quantiser named in Preliminary Results).  Single pass: each
// input element is read from HBM once.
//   K (statistics over 128 tokens of a channel): a block owns one token-group x one 512-channel
//     strip; each of its 8 waves keeps 16 token rows (16 x 128-bit per lane) in registers,
//     reduces its rows per channel, the 8 partial results meet in LDS, then every wave
//     quantises its own registers.
//   V (statistics over the 128 channels of a head): a head is 16 lanes x 8 channels, reduced
//     with a 4-step butterfly inside the wave.
#include "kvh_common.hpp"

namespace kvh {

constexpr int kEncWaves = 8;                          // waves per block
constexpr int kEncThreads = kEncWaves * kWave;        // 512
constexpr int kEncRows = 16;                          // rows per wave
constexpr int kEncTile = kEncRows * kEncWaves;        // 128 tokens per block = one K group
static_assert(kEncTile == kGroup, "a K block must cover exactly one token-group");

template <int DT>
__device__ __forceinline__ void unpack8(const uint4& d, float (&x)[8]) {
  const uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    x[2 * j] = t16_to_f32<DT>(w[j] & 0xffffu);
    x[2 * j + 1] = t16_to_f32<DT>(w[j] >> 16);
  }
}

// fp32 value that came from a 16-bit value -> its bit pattern, with -0 stored as +0.
template <int DT>
__device__ __forceinline__ uint32_t exact_bits(float f) {
  uint32_t b;
  if constexpr (DT == KVH_F16) {
    b = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
  } else {
    b = __builtin_bit_cast(uint32_t, f) >> 16;
  }
  return b == 0x8000u ? 0u : b;
}

template <int BITS>
__device__ __forceinline__ uint32_t quantise1(float x, float mn, float inv) {
  constexpr float L = float((1 << BITS) - 1);
  float t = (x - mn) * inv;                 // two roundings: compiled with -ffp-contract=off
  float r = __builtin_rintf(t);             // v_rndne_f32: ties to even
  r = __builtin_fminf(__builtin_fmaxf(r, 0.0f), L);
  return (uint32_t)r;
}

// Pack 8 codes LSB-first and store the BITS bytes they occupy.
template <int BITS>
__device__ __forceinline__ void store_codes(uint8_t* p, const uint32_t (&q)[8]) {
  if constexpr (BITS == 8) {
    uint2 w = {q[0] | q[1] << 8 | q[2] << 16 | q[3] << 24, q[4] | q[5] << 8 | q[6] << 16 | q[7] << 24};
    *reinterpret_cast<uint2*>(p) = w;
  } else if constexpr (BITS == 4) {
    uint32_t w = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) w |= q[j] << (4 * j);
    *reinterpret_cast<uint32_t*>(p) = w;
  } else {
    uint32_t w = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) w |= q[j] << (2 * j);
    *reinterpret_cast<uint16_t*>(p) = (uint16_t)w;
  }
}

template <int DT, int BITS>
__device__ __forceinline__ void encode_k_block(const EncodeParams& a, const kvh_enc_item& it, uint8_t* layer_base,
                                               const LayerGeom& geo, int lam, int g, int strip, float* red) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const int n = it.n_tokens;
  const int c = a.c;
  const int ch0 = strip * kStripCh + lane * kLaneCh;
  const bool active = ch0 < c;
  const int t_first = g * kGroup + wave * kEncRows;
  const uint16_t* src = a.k + (int64_t)lam * a.layer_stride + ch0;

  // Rows past the end of the blob re-read its last row: a duplicate never changes a min or max.
  uint4 d[kEncRows];
  if (active) {
#pragma unroll
    for (int i = 0; i < kEncRows; ++i) {
      int t = t_first + i;
      t = t < n ? t : n - 1;
      d[i] = *reinterpret_cast<const uint4*>(src + (it.src_token0 + t) * a.token_stride);
    }
  } else {
#pragma unroll
    for (int i = 0; i < kEncRows; ++i) d[i] = make_uint4(0, 0, 0, 0);
  }
  float mn[8], mx[8];
  unpack8<DT>(d[0], mn);
#pragma unroll
  for (int j = 0; j < 8; ++j) mx[j] = mn[j];
#pragma unroll
  for (int i = 1; i < kEncRows; ++i) {
    float x[8];
    unpack8<DT>(d[i], x);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      mn[j] = __builtin_fminf(mn[j], x[j]);
      mx[j] = __builtin_fmaxf(mx[j], x[j]);
    }
  }
  // red[0][wave][512] = partial minima, red[1][wave][512] = partial maxima
  float* rmn = red + (0 * kEncWaves + wave) * kStripCh + lane * kLaneCh;
  float* rmx = red + (1 * kEncWaves + wave) * kStripCh + lane * kLaneCh;
  *reinterpret_cast<float4*>(rmn) = make_float4(mn[0], mn[1], mn[2], mn[3]);
  *reinterpret_cast<float4*>(rmn + 4) = make_float4(mn[4], mn[5], mn[6], mn[7]);
  *reinterpret_cast<float4*>(rmx) = make_float4(mx[0], mx[1], mx[2], mx[3]);
  *reinterpret_cast<float4*>(rmx + 4) = make_float4(mx[4], mx[5], mx[6], mx[7]);
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kEncWaves; ++w) {
    const float* pmn = red + (0 * kEncWaves + w) * kStripCh + lane * kLaneCh;
    const float* pmx = red + (1 * kEncWaves + w) * kStripCh + lane * kLaneCh;
    float4 a0 = *reinterpret_cast<const float4*>(pmn), a1 = *reinterpret_cast<const float4*>(pmn + 4);
    float4 b0 = *reinterpret_cast<const float4*>(pmx), b1 = *reinterpret_cast<const float4*>(pmx + 4);
    const float am[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
    const float bm[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      mn[j] = __builtin_fminf(mn[j], am[j]);
      mx[j] = __builtin_fmaxf(mx[j], bm[j]);
    }
  }
  if (!active) return;

  uint32_t meta[8];
  float inv[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    uint32_t lo = exact_bits<DT>(mn[j]), hi = exact_bits<DT>(mx[j]);
    meta[j] = lo | hi << 16;
    mn[j] = t16_to_f32<DT>(lo);
    inv[j] = encode_inv<BITS>(mn[j], t16_to_f32<DT>(hi));
  }
  if (wave == 0) {
    uint4* mp = reinterpret_cast<uint4*>(layer_base + ((size_t)g * c + ch0) * 4);
    mp[0] = make_uint4(meta[0], meta[1], meta[2], meta[3]);
    mp[1] = make_uint4(meta[4], meta[5], meta[6], meta[7]);
  }
  uint8_t* codes = layer_base + geo.kmeta + (size_t)ch0 * BITS / 8;
#pragma unroll
  for (int i = 0; i < kEncRows; ++i) {
    int t = t_first + i;
    if (t < n) {
      float x[8];
      uint32_t q[8];
      unpack8<DT>(d[i], x);
#pragma unroll
      for (int j = 0; j < 8; ++j) q[j] = quantise1<BITS>(x[j], mn[j], inv[j]);
      store_codes<BITS>(codes + (size_t)t * geo.row_bytes, q);
    }
  }
}

template <int DT, int BITS>
__device__ __forceinline__ void encode_v_block(const EncodeParams& a, const kvh_enc_item& it, uint8_t* layer_base,
                                               const LayerGeom& geo, int lam, int tile, int strip) {
  constexpr int kBatch = 8;  // rows in flight per wave
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const int n = it.n_tokens;
  const int c = a.c;
  const int heads = c / kGroup;
  const int ch0 = strip * kStripCh + lane * kLaneCh;
  const bool active = ch0 < c;
  const int t_first = tile * kEncTile + wave * kEncRows;
  const uint16_t* src = a.v + (int64_t)lam * a.layer_stride + (active ? ch0 : 0);
  uint8_t* vmeta = layer_base + geo.kmeta + geo.codes;
  uint8_t* codes = vmeta + geo.vmeta + (size_t)ch0 * BITS / 8;

  for (int i0 = 0; i0 < kEncRows; i0 += kBatch) {
    if (t_first + i0 >= n) break;  // wave-uniform
    uint4 d[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      int t = t_first + i0 + i;
      t = t < n ? t : n - 1;
      // lanes beyond c re-read the row's first channels; their results are never stored
      d[i] = *reinterpret_cast<const uint4*>(src + (it.src_token0 + t) * a.token_stride);
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      int t = t_first + i0 + i;
      float x[8];
      unpack8<DT>(d[i], x);
      float mn = x[0], mx = x[0];
#pragma unroll
      for (int j = 1; j < 8; ++j) {
        mn = __builtin_fminf(mn, x[j]);
        mx = __builtin_fmaxf(mx, x[j]);
      }
#pragma unroll
      for (int m = 1; m < 16; m <<= 1) {  // butterfly over the 16 lanes of a head
        mn = __builtin_fminf(mn, __shfl_xor(mn, m));
        mx = __builtin_fmaxf(mx, __shfl_xor(mx, m));
      }
      if (active && t < n) {
        uint32_t lo = exact_bits<DT>(mn), hi = exact_bits<DT>(mx);
        if ((lane & 15) == 0)
          *reinterpret_cast<uint32_t*>(vmeta + ((size_t)t * heads + (ch0 / kGroup)) * 4) = lo | hi << 16;
        float fmn = t16_to_f32<DT>(lo);
        float inv = encode_inv<BITS>(fmn, t16_to_f32<DT>(hi));
        uint32_t q[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) q[j] = quantise1<BITS>(x[j], fmn, inv);
        store_codes<BITS>(codes + (size_t)t * geo.row_bytes, q);
      }
    }
  }
  // zero the padding that rounds the vmeta section up to 16 bytes
  if (strip == 0 && threadIdx.x == 0 && (tile + 1) * kEncTile >= n) {
    size_t used = (size_t)n * heads * 4;
    for (size_t o = used; o < geo.vmeta; o += 4) *reinterpret_cast<uint32_t*>(vmeta + o) = 0u;
  }
}

// grid = (token-groups x strips, 2 * l, items)
template <int DT>
__global__ __launch_bounds__(kEncThreads) void encode_kernel(EncodeParams a) {
  __shared__ float red[2 * kEncWaves * kStripCh];  // 32 KiB
  kvh_enc_item it;
  if (a.items != nullptr) {
    it = a.items[blockIdx.z];
  } else {
    it = a.one;
  }
  const int nstrips = (a.c + kStripCh - 1) / kStripCh;
  const int tile = blockIdx.x / nstrips;
  const int strip = blockIdx.x - tile * nstrips;
  const int bits = level_bits(it.level);
  if (bits < 0 || it.n_tokens < 1 || tile * kEncTile >= it.n_tokens) return;  // block-uniform
  const LayerGeom geo = layer_geom(it.n_tokens, a.c, bits);
  uint8_t* blob = static_cast<uint8_t*>(it.blob);
  const int lam = blockIdx.y >> 1;
  const bool is_v = blockIdx.y & 1;

  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < kHeaderBytes / 4) {
    const uint64_t total = kHeaderBytes + (uint64_t)a.l * geo.layer_bytes();
    uint32_t w = 0;
    switch (threadIdx.x) {
      case 0: w = kMagic; break;
      case 1: w = 1u | (uint32_t)DT << 16 | (uint32_t)bits << 24; break;
      case 2: w = (uint32_t)a.l; break;
      case 3: w = (uint32_t)it.n_tokens; break;
      case 4: w = (uint32_t)a.c; break;
      case 5: w = (uint32_t)kGroup | (uint32_t)kGroup << 16; break;
      case 6: w = (uint32_t)total; break;
      case 7: w = (uint32_t)(total >> 32); break;
      default: break;
    }
    reinterpret_cast<uint32_t*>(blob)[threadIdx.x] = w;
  }
  uint8_t* layer_base = blob + kHeaderBytes + (size_t)lam * geo.layer_bytes();
  if (!is_v) {
    switch (bits) {
      case 8: encode_k_block<DT, 8>(a, it, layer_base, geo, lam, tile, strip, red); break;
      case 4: encode_k_block<DT, 4>(a, it, layer_base, geo, lam, tile, strip, red); break;
      default: encode_k_block<DT, 2>(a, it, layer_base, geo, lam, tile, strip, red); break;
    }
  } else {
    switch (bits) {
      case 8: encode_v_block<DT, 8>(a, it, layer_base, geo, lam, tile, strip); break;
      case 4: encode_v_block<DT, 4>(a, it, layer_base, geo, lam, tile, strip); break;
      default: encode_v_block<DT, 2>(a, it, layer_base, geo, lam, tile, strip); break;
    }
  }
}

int launch_encode(const EncodeParams& a, int dt, int n_items, int max_tokens, hipStream_t stream) {
  const int nstrips = (a.c + kStripCh - 1) / kStripCh;
  const int tiles = (max_tokens + kEncTile - 1) / kEncTile;
  dim3 grid((unsigned)(tiles * nstrips), (unsigned)(2 * a.l), (unsigned)n_items);
  if (dt == KVH_F16)
    hipLaunchKernelGGL(encode_kernel<KVH_F16>, grid, dim3(kEncThreads), 0, stream, a);
  else
    hipLaunchKernelGGL(encode_kernel<KVH_BF16>, grid, dim3(kEncThreads), 0, stream, a);
  KVH_HIP_CHECK_LAUNCH();
  return KVH_OK;
}

}  // namespace kvh
