// Level decoder: unpack b-bit codes, dequantise with the stored (min, max) of each group and
// write fp16/bf16 KV rows, contiguous or through a page table (the "decompression" whose
// overhead the paper's estimator profiles; Design section).  Pure streaming kernel: every
// lane owns 8 channels, so every store is one 128-bit access and a wave writes 1 KiB of a
// token row per instruction; K metadata (per channel) lives in registers across the rows of
// a tile, V metadata (per token and head) is fetched by one lane per group and broadcast.
#include "kvh_common.hpp"

namespace kvh {

constexpr int kDecRows = 16;                            // rows per wave
constexpr int kDecTile = kDecRows * kWavesPerBlock;     // 64 tokens per block (divides the K group)

template <int BITS>
struct Codes;
template <>
struct Codes<8> {
  uint2 w;
  __device__ __forceinline__ void load(const uint8_t* p) { w = *reinterpret_cast<const uint2*>(p); }
  __device__ __forceinline__ uint32_t get(int j) const { return ((j < 4 ? w.x : w.y) >> (8 * (j & 3))) & 0xffu; }
};
template <>
struct Codes<4> {
  uint32_t w;
  __device__ __forceinline__ void load(const uint8_t* p) { w = *reinterpret_cast<const uint32_t*>(p); }
  __device__ __forceinline__ uint32_t get(int j) const { return (w >> (4 * j)) & 0xfu; }
};
template <>
struct Codes<2> {
  uint32_t w;
  __device__ __forceinline__ void load(const uint8_t* p) { w = *reinterpret_cast<const uint16_t*>(p); }
  __device__ __forceinline__ uint32_t get(int j) const { return (w >> (2 * j)) & 0x3u; }
};

template <int DT, int BITS>
__device__ __forceinline__ uint32_t dequant1(uint32_t q, const GroupParams& p) {
  constexpr uint32_t L = (1u << BITS) - 1u;
  float y = __builtin_fmaf((float)q, p.scale, p.mn);
  // The definition rounds twice (fma to fp32, then fp32 to the 16-bit type).  Keep the compiler
  // from merging the two into a mixed-precision fma that rounds once straight to fp16.
  asm("" : "+v"(y));
  uint32_t h = f32_to_t16<DT>(y);
  return q == L ? p.top : h;
}

// Physical row of logical position s.
__device__ __forceinline__ int32_t physical_row(int64_t s, const int32_t* page_table, int block_tokens) {
  if (page_table == nullptr) return (int32_t)s;
  uint32_t su = (uint32_t)s, bt = (uint32_t)block_tokens;
  uint32_t blk = su / bt;
  return page_table[blk] * block_tokens + (int32_t)(su - blk * bt);
}

template <int DT, int BITS>
__device__ __forceinline__ void decode_tile(const DecodeParams& a, const kvh_item& it, const uint8_t* layer_base,
                                            const LayerGeom& geo, int lam, bool is_v, int t_begin, int strip) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const int n = it.n_tokens;
  const int c = a.c;
  const int ch0 = strip * kStripCh + lane * kLaneCh;
  const bool active = ch0 < c;
  const int t_first = t_begin + wave;  // this wave's rows: t_first + 4 * i

  // Row i's destination is computed by lane i, then handed to the whole wave.
  int32_t my_row = 0;
  {
    int t = t_first + kWavesPerBlock * (lane & (kDecRows - 1));
    if (t < n) my_row = physical_row(it.dst_token0 + t, it.page_table, a.block_tokens);
  }
  int32_t rows[kDecRows];
#pragma unroll
  for (int i = 0; i < kDecRows; ++i) rows[i] = __builtin_amdgcn_readlane(my_row, i);

  const uint8_t* kmeta = layer_base;
  const uint8_t* kcodes = kmeta + geo.kmeta;
  const uint8_t* vmeta = kcodes + geo.codes;
  const uint8_t* vcodes = vmeta + geo.vmeta;
  uint16_t* dst = (is_v ? a.v : a.k) + (int64_t)lam * a.layer_stride + ch0;
  const uint8_t* codes = (is_v ? vcodes : kcodes) + (size_t)ch0 * BITS / 8;

  if (!is_v) {
    if (!active) return;
    const int g = t_begin / kGroup;
    const uint4* mp = reinterpret_cast<const uint4*>(kmeta + ((size_t)g * c + ch0) * 4);
    uint4 m0 = mp[0], m1 = mp[1];
    const uint32_t meta[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
    GroupParams gp[kLaneCh];
#pragma unroll
    for (int j = 0; j < kLaneCh; ++j) gp[j] = decode_params<DT, BITS>(meta[j]);

    Codes<BITS> cw[kDecRows];
#pragma unroll
    for (int i = 0; i < kDecRows; ++i) {
      int t = t_first + kWavesPerBlock * i;
      t = t < n ? t : n - 1;
      cw[i].load(codes + (size_t)t * geo.row_bytes);
    }
#pragma unroll
    for (int i = 0; i < kDecRows; ++i) {
      int t = t_first + kWavesPerBlock * i;
      if (t < n) {
        uint32_t h[kLaneCh];
#pragma unroll
        for (int j = 0; j < kLaneCh; ++j) h[j] = dequant1<DT, BITS>(cw[i].get(j), gp[j]);
        uint4 out = {h[0] | h[1] << 16, h[2] | h[3] << 16, h[4] | h[5] << 16, h[6] | h[7] << 16};
        *reinterpret_cast<uint4*>(dst + (int64_t)rows[i] * a.token_stride) = out;
      }
    }
  } else {
    // One lane per (row, head) group of this wave's 16 rows x 4 heads fetches and prepares the
    // parameters; every row then pulls its group's values from that lane.
    const int heads = c / kGroup;
    GroupParams mine = {0.0f, 0.0f, 0u};
    {
      int t = t_first + kWavesPerBlock * (lane >> 2);
      int head = strip * (kStripCh / kGroup) + (lane & 3);
      if (t < n && head < heads) {
        uint32_t meta = *reinterpret_cast<const uint32_t*>(vmeta + ((size_t)t * heads + head) * 4);
        mine = decode_params<DT, BITS>(meta);
      }
    }
    Codes<BITS> cw[kDecRows];
    if (active) {
#pragma unroll
      for (int i = 0; i < kDecRows; ++i) {
        int t = t_first + kWavesPerBlock * i;
        t = t < n ? t : n - 1;
        cw[i].load(codes + (size_t)t * geo.row_bytes);
      }
    }
#pragma unroll
    for (int i = 0; i < kDecRows; ++i) {
      int t = t_first + kWavesPerBlock * i;
      int src = i * 4 + (lane >> 4);
      GroupParams p;
      p.mn = __shfl(mine.mn, src);
      p.scale = __shfl(mine.scale, src);
      p.top = __shfl(mine.top, src);
      if (active && t < n) {
        uint32_t h[kLaneCh];
#pragma unroll
        for (int j = 0; j < kLaneCh; ++j) h[j] = dequant1<DT, BITS>(cw[i].get(j), p);
        uint4 out = {h[0] | h[1] << 16, h[2] | h[3] << 16, h[4] | h[5] << 16, h[6] | h[7] << 16};
        *reinterpret_cast<uint4*>(dst + (int64_t)rows[i] * a.token_stride) = out;
      }
    }
  }
}

__device__ __forceinline__ bool header_matches(const uint8_t* blob, int dt, int bits, int l, int n, int c,
                                               size_t total) {
  const uint4* h = reinterpret_cast<const uint4*>(blob);
  uint4 a = h[0], b = h[1];
  return a.x == kMagic && a.y == (1u | (uint32_t)dt << 16 | (uint32_t)bits << 24) && a.z == (uint32_t)l &&
         a.w == (uint32_t)n && b.x == (uint32_t)c && b.y == ((uint32_t)kGroup | (uint32_t)kGroup << 16) &&
         b.z == (uint32_t)total && b.w == (uint32_t)((uint64_t)total >> 32);
}

// grid = (token tiles x strips, 2 * l, items)
template <int DT>
__global__ __launch_bounds__(kBlockThreads) void decode_kernel(DecodeParams a) {
  const int item_idx = blockIdx.z;
  kvh_item it;
  if (a.items != nullptr) {
    it = a.items[item_idx];
  } else {
    it = a.one;
  }
  const int nstrips = (a.c + kStripCh - 1) / kStripCh;
  const int tile = blockIdx.x / nstrips;
  const int strip = blockIdx.x - tile * nstrips;
  const int t_begin = tile * kDecTile;
  if (it.n_tokens < 1 || t_begin >= it.n_tokens) return;
  const int bits = level_bits(it.level);
  const uint8_t* blob = static_cast<const uint8_t*>(it.blob);
  bool ok = bits > 0;
  LayerGeom geo = layer_geom(it.n_tokens, a.c, ok ? bits : 8);
  if (ok) ok = header_matches(blob, DT, bits, a.l, it.n_tokens, a.c, kHeaderBytes + (size_t)a.l * geo.layer_bytes());
  if (!ok) {
    if (a.status != nullptr && threadIdx.x == 0) a.status[item_idx] = KVH_DEV_HEADER_MISMATCH;
    return;
  }
  const int lam = blockIdx.y >> 1;
  const bool is_v = blockIdx.y & 1;
  const uint8_t* layer_base = blob + kHeaderBytes + (size_t)lam * geo.layer_bytes();
  switch (bits) {
    case 8: decode_tile<DT, 8>(a, it, layer_base, geo, lam, is_v, t_begin, strip); break;
    case 4: decode_tile<DT, 4>(a, it, layer_base, geo, lam, is_v, t_begin, strip); break;
    default: decode_tile<DT, 2>(a, it, layer_base, geo, lam, is_v, t_begin, strip); break;
  }
}

int launch_decode(const DecodeParams& a, int dt, int n_items, int max_tokens, hipStream_t stream) {
  const int nstrips = (a.c + kStripCh - 1) / kStripCh;
  const int tiles = (max_tokens + kDecTile - 1) / kDecTile;
  dim3 grid((unsigned)(tiles * nstrips), (unsigned)(2 * a.l), (unsigned)n_items);
  if (dt == KVH_F16)
    hipLaunchKernelGGL(decode_kernel<KVH_F16>, grid, dim3(kBlockThreads), 0, stream, a);
  else
    hipLaunchKernelGGL(decode_kernel<KVH_BF16>, grid, dim3(kBlockThreads), 0, stream, a);
  KVH_HIP_CHECK_LAUNCH();
  return KVH_OK;
}

}  // namespace kvh
