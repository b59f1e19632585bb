// Level encoder: per-group min/max, quantise to b bits, bit-pack and write the blob
// (compression of a KV-cache entry with the quantisation method at a rate; Design section, and
// the per-channel-K / per-token-V quantiser named in Preliminary Results).  Single pass: each
// input element is read from HBM once.
//   K (statistics over 128 tokens of a channel): a block owns one token-group x one 512-channel
//     strip; each of its 8 waves keeps 16 token rows (16 x 128-bit per lane) in registers,
//     reduces its rows per channel, the 8 partial results meet in LDS, then every wave
//     quantises its own registers.
//   V (statistics over the 128 channels of a head): a head is 16 lanes x 8 channels, reduced
//     with a 4-step rotate-and-combine inside the 16-lane DPP row.
// Quantised codes are produced with the packed float->u8 convert, which rounds to nearest even
// and inserts the byte in one instruction; narrow codes are routed to their byte at that point.
#include "kvh_common.hpp"

namespace kvh {

constexpr int kEncWaves = 8;                          // waves per block
constexpr int kEncThreads = kEncWaves * kWave;        // 512
constexpr int kEncRows = 16;                          // rows per wave
constexpr int kEncTile = kEncRows * kEncWaves;        // 128 tokens per block = one K group
static_assert(kEncTile == kGroup, "a K block must cover exactly one token-group");

typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

template <typename T>
__device__ __forceinline__ T gload(const void* p) {
  return *reinterpret_cast<const __attribute__((address_space(1))) T*>(reinterpret_cast<uintptr_t>(p));
}
template <typename T>
__device__ __forceinline__ void gstore(void* p, T v) {
  *reinterpret_cast<__attribute__((address_space(1))) T*>(reinterpret_cast<uintptr_t>(p)) = v;
}

#ifndef KVH_ENC_NT
#define KVH_ENC_NT 1  // non-temporal stores of the packed codes
#endif
#ifndef KVH_ENC_NTL
#define KVH_ENC_NTL 1  // non-temporal loads of the 16-bit rows
#endif
// Rows of a V wave whose statistics are reduced together (16, 8, 4 or 2).  Fewer operations with larger batches,
// earlier stores with smaller ones; measured on the 8K-token shape (% of HBM peak at 8 / 4 / 2 bits): batches of 16:
// 76.2 / 76.5 / 75.8, of 8: 76.1 / 76.3 / 75.8, of 4: 76.6 / 78.0 / 77.6, of 2: 77.2 / 77.9 / 75.1.
#ifndef KVH_ENC_VBATCH
#define KVH_ENC_VBATCH 4
#endif
template <typename T>
__device__ __forceinline__ T gload_rows(const void* p) {
#if KVH_ENC_NTL
  return __builtin_nontemporal_load(reinterpret_cast<const __attribute__((address_space(1))) T*>(reinterpret_cast<uintptr_t>(p)));
#else
  return *reinterpret_cast<const __attribute__((address_space(1))) T*>(reinterpret_cast<uintptr_t>(p));
#endif
}
template <typename T>
__device__ __forceinline__ void gstore_codes(void* p, T v) {
#if KVH_ENC_NT
  __builtin_nontemporal_store(v, reinterpret_cast<__attribute__((address_space(1))) T*>(reinterpret_cast<uintptr_t>(p)));
#else
  gstore<T>(p, v);
#endif
}

template <int DT>
__device__ __forceinline__ void unpack8(const uintx4& d, float (&x)[8]) {
  const uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if constexpr (DT == KVH_F16) {
      x[2 * j] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[j] & 0xffffu));
      x[2 * j + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[j] >> 16));
    } else {
      x[2 * j] = __builtin_bit_cast(float, w[j] << 16);
      x[2 * j + 1] = __builtin_bit_cast(float, w[j] & 0xffff0000u);
    }
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

// t = (x - mn) * inv: two roundings (the file is compiled with -ffp-contract=off).  For finite
// input 0 <= t <= L * (1 + 2^-23), so rounding to nearest even never leaves [0, L].
__device__ __forceinline__ float position(float x, float mn, float inv) { return (x - mn) * inv; }

// Four positions -> four code bytes in one word (byte j = code j).  The convert rounds to
// nearest even and saturates to [0, 255].
__device__ __forceinline__ uint32_t codes4(float t0, float t1, float t2, float t3) {
  uint32_t a = __builtin_amdgcn_cvt_pk_u8_f32(t0, 0, 0u);
  a = __builtin_amdgcn_cvt_pk_u8_f32(t1, 1, a);
  a = __builtin_amdgcn_cvt_pk_u8_f32(t2, 2, a);
  return __builtin_amdgcn_cvt_pk_u8_f32(t3, 3, a);
}

// Two positions -> two code bytes (bytes 0 and 1 of the result).
__device__ __forceinline__ uint32_t codes2(float t0, float t1) {
  return __builtin_amdgcn_cvt_pk_u8_f32(t1, 1, __builtin_amdgcn_cvt_pk_u8_f32(t0, 0, 0u));
}

// Quantise 8 elements and store the BITS bytes they occupy (LSB-first packing).
// param(j) returns {mn, inv} of channel j.  The convert puts a code into any byte of a word, so
// narrow codes are routed at that point: word i receives, in its byte k, the code that belongs i
// fields above the bottom of output byte k, and the words are merged with one shift-or each.
// (For finite input every code is <= L, so fields never overlap.)
template <int BITS, typename P>
__device__ __forceinline__ void quantise_store8(uint8_t* p, const float (&x)[8], P&& param) {
  float t[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) t[j] = position(x[j], param(j).x, param(j).y);
  if constexpr (BITS == 8) {
    uintx2 w = {codes4(t[0], t[1], t[2], t[3]), codes4(t[4], t[5], t[6], t[7])};
    gstore_codes<uintx2>(p, w);
  } else if constexpr (BITS == 4) {
    gstore_codes<uint32_t>(p, codes4(t[0], t[2], t[4], t[6]) | codes4(t[1], t[3], t[5], t[7]) << 4);
  } else {
    gstore_codes<uint16_t>(p, (uint16_t)(codes2(t[0], t[4]) | codes2(t[1], t[5]) << 2 | codes2(t[2], t[6]) << 4 |
                                   codes2(t[3], t[7]) << 6));
  }
}

template <int DT, int BITS>
__device__ __forceinline__ void encode_k_block(const EncodeParams& a, const kvh_enc_item& it, uint8_t* layer_base,
                                               const LayerGeom& geo, int lam, int g, int strip, float* red,
                                               int split, int64_t jump) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = it.n_tokens;
  const int c = a.c;
  const int ch_raw = strip * kStripCh + lane * kLaneCh;
  const bool active = ch_raw < c;
  const int ch0 = active ? ch_raw : 0;  // idle lanes of a partial strip shadow lane 0 and never store
  const int t_first = g * kGroup + wave * kEncRows;
  const uint8_t* src = reinterpret_cast<const uint8_t*>(a.k + (int64_t)lam * a.layer_stride);  // wave-uniform
  const uint32_t lane_src_off = (uint32_t)ch0 * 2u;

  // Rows past the end of the blob re-read its last row: a duplicate never changes a min or max.
  uintx4 d[kEncRows];
#pragma unroll
  for (int i = 0; i < kEncRows; ++i) {
    int t = t_first + i;
    t = t < n ? t : n - 1;
    d[i] = gload_rows<uintx4>(uniform(src + (it.src_token0 + t + (t >= split ? jump : 0)) * a.token_stride * 2) + lane_src_off);
  }
  float mn[8], mx[8];
  if constexpr (DT == KVH_BF16) {
    // bf16: the odd channels (upper halves) are compared in their words as they are, the even ones after a shift;
    // the lower half of a word only extends the mantissa and never carries a value past its 16-bit neighbour
    auto word = [&](int i, int q) { return q == 0 ? d[i].x : q == 1 ? d[i].y : q == 2 ? d[i].z : d[i].w; };
    auto as_f = [](uint32_t w) { return __builtin_bit_cast(float, w); };
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t w0 = word(0, q), w1 = word(1, q);
      mn[2 * q] = __builtin_fminf(as_f(w0 << 16), as_f(w1 << 16));
      mx[2 * q] = __builtin_fmaxf(as_f(w0 << 16), as_f(w1 << 16));
      mn[2 * q + 1] = __builtin_fminf(as_f(w0), as_f(w1));
      mx[2 * q + 1] = __builtin_fmaxf(as_f(w0), as_f(w1));
    }
#pragma unroll
    for (int i = 2; i < kEncRows; i += 2) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t w0 = word(i, q), w1 = word(i + 1, q);
        mn[2 * q] = __builtin_fminf(__builtin_fminf(mn[2 * q], as_f(w0 << 16)), as_f(w1 << 16));
        mx[2 * q] = __builtin_fmaxf(__builtin_fmaxf(mx[2 * q], as_f(w0 << 16)), as_f(w1 << 16));
        mn[2 * q + 1] = __builtin_fminf(__builtin_fminf(mn[2 * q + 1], as_f(w0)), as_f(w1));
        mx[2 * q + 1] = __builtin_fmaxf(__builtin_fmaxf(mx[2 * q + 1], as_f(w0)), as_f(w1));
      }
    }
  } else {
    unpack8<DT>(d[0], mn);
#pragma unroll
    for (int j = 0; j < 8; ++j) mx[j] = mn[j];
    {
      float x1[8];
      unpack8<DT>(d[1], x1);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        mn[j] = __builtin_fminf(mn[j], x1[j]);
        mx[j] = __builtin_fmaxf(mx[j], x1[j]);
      }
    }
#pragma unroll
    for (int i = 2; i < kEncRows; i += 2) {  // two rows per step: three-operand min / max
      float x0[8], x1[8];
      unpack8<DT>(d[i], x0);
      unpack8<DT>(d[i + 1], x1);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        mn[j] = __builtin_fminf(__builtin_fminf(mn[j], x0[j]), x1[j]);
        mx[j] = __builtin_fmaxf(__builtin_fmaxf(mx[j], x0[j]), x1[j]);
      }
      __builtin_amdgcn_sched_barrier(0);  // keep the unpacked floats of different rows from piling up in registers
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
  // The rows are unpacked a second time for quantisation.  Hide them from common-subexpression
  // elimination, or the compiler keeps all 128 unpacked floats alive across the barrier.
#pragma unroll
  for (int i = 0; i < kEncRows; ++i) {
    uint32_t w0 = d[i].x, w1 = d[i].y, w2 = d[i].z, w3 = d[i].w;
    asm volatile("" : "+v"(w0), "+v"(w1), "+v"(w2), "+v"(w3));
    d[i] = uintx4{w0, w1, w2, w3};
  }
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

  uint32_t meta[8];
  float2 par[8];  // {mn, inv}
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    uint32_t lo = exact_bits<DT>(mn[j]), hi = exact_bits<DT>(mx[j]);
    meta[j] = lo | hi << 16;
    par[j].x = t16_to_f32<DT>(lo);
    par[j].y = encode_inv<BITS>(par[j].x, t16_to_f32<DT>(hi));
    // The eight channels are independent, and the scheduler would interleave them all, which costs more registers
    // than the kernel has left here (the 16 rows stay in registers across this point).  Spilled registers come back
    // through loads in the middle of the store loop, and a wait for such a load also waits for every store issued
    // before it: 3-5 such stalls per block, 3 points of throughput.  The empty statement ties the next channel's
    // inputs to this channel's results, so the channels are prepared one after the other and nothing spills.
    if (j + 1 < 8) asm volatile("" : "+v"(par[j].x), "+v"(par[j].y), "+v"(meta[j]), "+v"(mn[j + 1]), "+v"(mx[j + 1]));
  }
  if (!active) return;
  if (wave == 0) {
    uint8_t* mp = layer_base + ((size_t)g * c + ch0) * 4;
    uintx4 m0 = {meta[0], meta[1], meta[2], meta[3]}, m1 = {meta[4], meta[5], meta[6], meta[7]};
    gstore<uintx4>(mp, m0);
    gstore<uintx4>(mp + 16, m1);
  }
  uint8_t* codes = layer_base + geo.kmeta;  // wave-uniform
  const uint32_t lane_code_off = (uint32_t)ch0 * BITS / 8;
#pragma unroll
  for (int i = 0; i < kEncRows; ++i) {
    int t = t_first + i;
    if (t < n) {  // wave-uniform
      float x[8];
      unpack8<DT>(d[i], x);
      quantise_store8<BITS>(uniform(codes + (size_t)t * geo.row_bytes) + lane_code_off, x, [&](int j) { return par[j]; });
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Raw level: the rows of the block's tile and strip go into the blob as they are (K rows, then V rows, per layer).
template <int DT>
__device__ __forceinline__ void encode_raw_block(const EncodeParams& a, const kvh_enc_item& it, uint8_t* layer_base,
                                                 const LayerGeom& geo, int lam, bool is_v, int tile, int strip, int split,
                                                 int64_t jump) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = it.n_tokens;
  const int ch_raw = strip * kStripCh + lane * kLaneCh;
  const bool active = ch_raw < a.c;
  const int ch0 = active ? ch_raw : 0;
  const int t_first = tile * kEncTile + wave * kEncRows;
  if (t_first >= n) return;  // wave-uniform
  const uint8_t* src = reinterpret_cast<const uint8_t*>((is_v ? a.v : a.k) + (int64_t)lam * a.layer_stride);
  uint8_t* rows = layer_base + (is_v ? geo.codes : 0);  // kmeta and vmeta are empty at this level
  uintx4 d[kEncRows];
#pragma unroll
  for (int i = 0; i < kEncRows; ++i) {
    int t = t_first + i;
    t = t < n ? t : n - 1;
    d[i] = gload_rows<uintx4>(uniform(src + (it.src_token0 + t + (t >= split ? jump : 0)) * a.token_stride * 2) + (uint32_t)ch0 * 2u);
  }
#pragma unroll
  for (int i = 0; i < kEncRows; ++i) {
    const int t = t_first + i;
    if (t < n && active) gstore_codes<uintx4>(uniform(rows + (size_t)t * geo.row_bytes) + (uint32_t)ch0 * 2u, d[i]);
  }
}

// ---- V statistics: a reduce-scatter over the 16 lanes of a head --------------------------------------
// A wave holds 16 rows; a head is one DPP row of 16 lanes.  Instead of an all-reduce per row (after which all 16
// lanes would prepare the same parameters 16 times over), the 16 per-row partials of a lane are folded in four
// halving steps so that lane j of a head ends up with the minimum and maximum of row j alone: 15 combine-and-select
// steps per lane for all 16 rows, parameters prepared once per (row, head), and row i's two parameters fetched
// back by every lane with a row broadcast when row i is quantised.
template <typename F, int... I>
__device__ __forceinline__ void for_each_index(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
constexpr int kDppRor8 = 0x128;    // row_ror:8, lane L reads lane L - 8 (mod 16): its partner across bit 3
constexpr int kDppPlus4 = 0x12C;   // row_ror:12, lane L reads lane L + 4 (mod 16)
constexpr int kDppMinus4 = 0x124;  // row_ror:4, lane L reads lane L - 4 (mod 16)
constexpr int kDppXor2 = 0x4E;     // quad_perm [2,3,0,1]
constexpr int kDppXor1 = 0xB1;     // quad_perm [1,0,3,2]
constexpr int kDppRowBcast = 0x150;  // + i: every lane of a row reads lane i of that row

// One fold.  p0 and p1 are this lane's partials of two rows that differ in the row-index bit which the lane bit
// `bit` decides: the lane keeps the row whose bit equals its own and folds in its partner's partial of that row.
// FROM_UP reads the partner of a lane whose bit is clear, FROM_DOWN that of a lane whose bit is set; each is only
// right for its half of the lanes, and the select takes the right one.
template <bool IS_MIN, int FROM_UP, int FROM_DOWN>
__device__ __forceinline__ float fold16(float p0, float p1, bool bit) {
  const float a = dpp_f<FROM_UP>(p0), b = dpp_f<FROM_DOWN>(p1);
  const float lo = IS_MIN ? __builtin_fminf(a, p0) : __builtin_fmaxf(a, p0);
  const float hi = IS_MIN ? __builtin_fminf(b, p1) : __builtin_fmaxf(b, p1);
  return bit ? hi : lo;
}
// A batch of R rows (16, 8 or 4).  in[k] = this lane's partial of rows 2k / 2k + 1 of the batch, already folded over
// lane bit 0 (so in[k] belongs to row 2k + (lane & 1)).  The remaining row-index bits are folded over lane bits
// 1 .. log2(R) - 1; over the lane bits above that the partials are all-reduced, so that the full reduction of row r
// ends up in every lane with (lane & (R - 1)) == r, lane r among them.
template <bool IS_MIN, int R>
__device__ __forceinline__ float reduce_scatter(const float (&in)[R / 2], int lane) {
  auto both = [](float v, float o) { return IS_MIN ? __builtin_fminf(v, o) : __builtin_fmaxf(v, o); };
  if constexpr (R == 16) {
    float c[4], e[2];
#pragma unroll
    for (int m = 0; m < 4; ++m) c[m] = fold16<IS_MIN, kDppXor2, kDppXor2>(in[2 * m], in[2 * m + 1], (lane & 2) != 0);
#pragma unroll
    for (int q = 0; q < 2; ++q) e[q] = fold16<IS_MIN, kDppPlus4, kDppMinus4>(c[2 * q], c[2 * q + 1], (lane & 4) != 0);
    return fold16<IS_MIN, kDppRor8, kDppRor8>(e[0], e[1], (lane & 8) != 0);
  } else if constexpr (R == 8) {
    float c[2];
#pragma unroll
    for (int m = 0; m < 2; ++m) c[m] = fold16<IS_MIN, kDppXor2, kDppXor2>(in[2 * m], in[2 * m + 1], (lane & 2) != 0);
    const float e = fold16<IS_MIN, kDppPlus4, kDppMinus4>(c[0], c[1], (lane & 4) != 0);
    return both(dpp_f<kDppRor8>(e), e);
  } else if constexpr (R == 4) {
    float c = fold16<IS_MIN, kDppXor2, kDppXor2>(in[0], in[1], (lane & 2) != 0);
    c = both(dpp_f<kDppMinus4>(c), c);
    return both(dpp_f<kDppRor8>(c), c);
  } else {
    static_assert(R == 2, "batches of 16, 8, 4 or 2 rows");
    float c = both(dpp_f<kDppXor2>(in[0]), in[0]);
    c = both(dpp_f<kDppMinus4>(c), c);
    return both(dpp_f<kDppRor8>(c), c);
  }
}

// Minimum and maximum of the 8 values of one lane and row.  For bf16 the upper halves are compared as they sit in
// their words: the lower half only extends the mantissa, which never carries a value past its 16-bit neighbour, so
// the upper 16 bits of the result are those of the true extreme (the sign of a zero aside, which the metadata
// drops anyway).
template <int DT>
__device__ __forceinline__ void row_minmax(const uintx4& d, float& mn, float& mx) {
  if constexpr (DT == KVH_BF16) {
    // (the words are copied out first: a bit cast applied to a vector element directly reads element 0)
    const uint32_t w0 = d.x, w1 = d.y, w2 = d.z, w3 = d.w;
    const float h0 = __builtin_bit_cast(float, w0), h1 = __builtin_bit_cast(float, w1);
    const float h2 = __builtin_bit_cast(float, w2), h3 = __builtin_bit_cast(float, w3);
    const float l0 = __builtin_bit_cast(float, w0 << 16), l1 = __builtin_bit_cast(float, w1 << 16);
    const float l2 = __builtin_bit_cast(float, w2 << 16), l3 = __builtin_bit_cast(float, w3 << 16);
    mn = __builtin_fminf(__builtin_fminf(h0, h1), h2);
    mx = __builtin_fmaxf(__builtin_fmaxf(h0, h1), h2);
    mn = __builtin_fminf(__builtin_fminf(mn, h3), l0);
    mx = __builtin_fmaxf(__builtin_fmaxf(mx, h3), l0);
    mn = __builtin_fminf(__builtin_fminf(mn, l1), l2);
    mx = __builtin_fmaxf(__builtin_fmaxf(mx, l1), l2);
    mn = __builtin_fminf(mn, l3);
    mx = __builtin_fmaxf(mx, l3);
  } else {
    float x[8];
    unpack8<DT>(d, x);
    mn = __builtin_fminf(__builtin_fminf(x[0], x[1]), x[2]);
    mx = __builtin_fmaxf(__builtin_fmaxf(x[0], x[1]), x[2]);
    mn = __builtin_fminf(__builtin_fminf(mn, x[3]), x[4]);
    mx = __builtin_fmaxf(__builtin_fmaxf(mx, x[3]), x[4]);
    mn = __builtin_fminf(__builtin_fminf(mn, x[5]), x[6]);
    mx = __builtin_fmaxf(__builtin_fmaxf(mx, x[5]), x[6]);
    mn = __builtin_fminf(mn, x[7]);
    mx = __builtin_fmaxf(mx, x[7]);
  }
}

template <int DT, int BITS>
__device__ __forceinline__ void encode_v_block(const EncodeParams& a, const kvh_enc_item& it, uint8_t* layer_base,
                                               const LayerGeom& geo, int lam, int tile, int strip, int split,
                                               int64_t jump) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = it.n_tokens;
  const int c = a.c;
  const int heads = c / kGroup;
  const int ch_raw = strip * kStripCh + lane * kLaneCh;
  const bool active = ch_raw < c;  // uniform over the 16 lanes of a head
  const int ch0 = active ? ch_raw : 0;
  const int t_first = tile * kEncTile + wave * kEncRows;
  const uint8_t* src = reinterpret_cast<const uint8_t*>(a.v + (int64_t)lam * a.layer_stride);  // wave-uniform
  const uint32_t lane_src_off = (uint32_t)ch0 * 2u;
  uint8_t* vmeta = layer_base + geo.kmeta + geo.codes;
  uint8_t* codes = vmeta + geo.vmeta;  // wave-uniform
  const uint32_t lane_code_off = (uint32_t)ch0 * BITS / 8;

  if (t_first < n) {  // wave-uniform
    uintx4 d[kEncRows];  // all 16 rows of the wave are requested before the first one is used
#pragma unroll
    for (int i = 0; i < kEncRows; ++i) {
      int t = t_first + i;
      t = t < n ? t : n - 1;
      d[i] = gload_rows<uintx4>(uniform(src + (it.src_token0 + t + (t >= split ? jump : 0)) * a.token_stride * 2) + lane_src_off);
    }
    // The 16 rows are taken in batches of R, in the order their loads return: statistics of a batch, its metadata
    // words and parameters (lane r of a head takes row r of the batch), then its rows are quantised and stored
    // while the loads of the next batch are still arriving.
    constexpr int R = KVH_ENC_VBATCH;
    static_assert(kEncRows % R == 0 && (R == 16 || R == 8 || R == 4 || R == 2), "batches of 16, 8, 4 or 2 rows");
    auto batch = [&](auto b_idx) {
      constexpr int r0 = decltype(b_idx)::value * R;
      float pmn[R / 2], pmx[R / 2];
#pragma unroll
      for (int k = 0; k < R / 2; ++k) {
        float mn0, mx0, mn1, mx1;
        row_minmax<DT>(d[r0 + 2 * k], mn0, mx0);
        row_minmax<DT>(d[r0 + 2 * k + 1], mn1, mx1);
        pmn[k] = fold16<true, kDppXor1, kDppXor1>(mn0, mn1, (lane & 1) != 0);
        pmx[k] = fold16<false, kDppXor1, kDppXor1>(mx0, mx1, (lane & 1) != 0);
      }
      const float mn_own = reduce_scatter<true, R>(pmn, lane);
      const float mx_own = reduce_scatter<false, R>(pmx, lane);
      const uint32_t lo = exact_bits<DT>(mn_own), hi = exact_bits<DT>(mx_own);
      const int t_own = t_first + r0 + (lane & (R - 1));
      if (active && (lane & 15) < R && t_own < n)
        gstore<uint32_t>(vmeta + ((size_t)t_own * heads + ch0 / kGroup) * 4, lo | hi << 16);
      float2 own;
      own.x = t16_to_f32<DT>(lo);
      own.y = encode_inv<BITS>(own.x, t16_to_f32<DT>(hi));
      auto row = [&](auto idx) {
        constexpr int r = decltype(idx)::value;
        constexpr int i = r0 + r;
        const int t = t_first + i;
        if (t < n) {  // wave-uniform; the row address is formed on the scalar unit, outside the per-lane test
          uint8_t* code_row = uniform(codes + (size_t)t * geo.row_bytes);
          float2 par;
          par.x = dpp_f<kDppRowBcast + r>(own.x);
          par.y = dpp_f<kDppRowBcast + r>(own.y);
          if (active) {
            // the row is unpacked a second time here; the copy below keeps the compiler from holding the first
            // unpacking of all rows in registers instead (which spills)
            uintx4 w = d[i];
            asm volatile("" : "+v"(w));
            float x[8];
            unpack8<DT>(w, x);
            quantise_store8<BITS>(code_row + lane_code_off, x, [&](int) { return par; });
          }
        }
      };
      for_each_index(row, std::make_integer_sequence<int, R>{});
    };
    for_each_index(batch, std::make_integer_sequence<int, kEncRows / R>{});
  }
  // zero the padding that rounds the vmeta section up to 16 bytes
  if (strip == 0 && threadIdx.x == 0 && (tile + 1) * kEncTile >= n) {
    size_t used = (size_t)n * heads * 4;
    for (size_t o = used; o < geo.vmeta; o += 4) gstore<uint32_t>(vmeta + o, 0u);
  }
}


// grid = (token-groups x strips, 2 * l, items)
template <int DT>
__global__ __launch_bounds__(kEncThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void encode_kernel(EncodeParams a) {
  __shared__ float red[2 * kEncWaves * kStripCh];  // 32 KiB
  kvh_enc_item it;
  DropInfo drop = {kNoSplit, 0, 0u, 0u, 0u};  // ordinary batch items are never token-dropped
  const kvh_enc_item* items = a.items;
  if (a.n_inline > 0) items = reinterpret_cast<const kvh_enc_item*>(KVH_KERNARG_MEMBER(EncodeParams, inline_items));
  if (items != nullptr) {
    const kvh_enc_item* p = items + blockIdx.z;
#if KVH_SCALAR_DESC
    uintx4 lo = sload<uintx4>(p);
    uintx2 hi = sload<uintx2>(reinterpret_cast<const uint8_t*>(p) + 16);
#else
    uintx4 lo = gload<uintx4>(p);
    uintx2 hi = gload<uintx2>(reinterpret_cast<const uint8_t*>(p) + 16);
#endif
    it.blob = reinterpret_cast<void*>((uint64_t)lo.x | (uint64_t)lo.y << 32);
    it.src_token0 = (int64_t)((uint64_t)lo.z | (uint64_t)lo.w << 32);
    it.n_tokens = (int32_t)hi.x;
    it.level = (int32_t)hi.y;
  } else if (a.kept_items != nullptr) {
    const kvh_kept_enc_item* p = a.kept_items + blockIdx.z;
#if KVH_SCALAR_DESC
    uintx4 lo = sload<uintx4>(p), hi = sload<uintx4>(reinterpret_cast<const uint8_t*>(p) + 16);
#else
    uintx4 lo = gload<uintx4>(p), hi = gload<uintx4>(reinterpret_cast<const uint8_t*>(p) + 16);
#endif
    it.blob = reinterpret_cast<void*>((uint64_t)lo.x | (uint64_t)lo.y << 32);
    it.src_token0 = (int64_t)((uint64_t)lo.z | (uint64_t)lo.w << 32);
    const int32_t orig = uniform((int32_t)hi.x), sink = uniform((int32_t)hi.y), window = uniform((int32_t)hi.z);
    it.level = (int32_t)hi.w;
    const bool ok = orig >= 1 && sink >= 0 && window >= 0 && (int64_t)sink + window >= 1;
    const int64_t sw = (int64_t)sink + window;
    it.n_tokens = ok ? (int32_t)(sw >= orig ? orig : sw) : 0;  // nothing kept: the item is skipped below
    drop.orig_tokens = (uint32_t)orig;
    drop.sink = (uint32_t)sink;
    drop.window = (uint32_t)window;
    if (ok && sw < orig) {
      drop.split = sink;
      drop.jump = (int64_t)orig - window - sink;
    }
  } else {
    it = a.one;
    drop = DropInfo{a.split, a.jump, a.hdr_orig_tokens, a.hdr_sink, a.hdr_window};
  }
  it.blob = uniform(it.blob);
  it.src_token0 = uniform(it.src_token0);
  it.n_tokens = uniform(it.n_tokens);
  it.level = uniform(it.level);
  const int split = drop.split;
  const int64_t jump = drop.jump;
  const int nstrips = (a.c + kStripCh - 1) / kStripCh;
  // Block order: consecutive blocks of the dispatch order take the same tile of the `plane_group` consecutive
  // (layer, K|V) planes of a group, then the next tile of those planes; the groups follow each other (the last one
  // may be smaller).  The launcher chooses the group size.
  int lay_kv, bx;
  {
    const int lin_xy = blockIdx.y * gridDim.x + blockIdx.x;
    const int planes = gridDim.y, per_plane = gridDim.x;
    const int group = a.plane_group < 1 ? 1 : a.plane_group < planes ? a.plane_group : planes;
    const int full = planes / group;
    const int g = lin_xy / (group * per_plane);
    const int first = (g < full ? g : full) * group;            // first plane of this block's group
    const int size = g < full ? group : planes - full * group;  // planes in it
    const int j = lin_xy - first * per_plane;
    lay_kv = first + j % size;
    bx = j / size;
  }
  const int tile = bx / nstrips;
  const int strip = bx - tile * nstrips;
  const int bits = level_bits(it.level);
  // block-uniform; an item with more tokens than the grid covers is skipped as a whole (no header either), so
  // that a later decode of its blob reports a mismatch instead of reading sections that were never written
  if (bits < 0 || it.n_tokens < 1 || it.n_tokens > a.max_tokens || tile * kEncTile >= it.n_tokens) return;
  const LayerGeom geo = layer_geom(it.n_tokens, a.c, bits);
  uint8_t* blob = static_cast<uint8_t*>(it.blob);
  const int lam = lay_kv >> 1;
  const bool is_v = lay_kv & 1;

  if (bx == 0 && lay_kv == 0 && threadIdx.x < kHeaderBytes / 4) {
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
      case 8: w = drop.orig_tokens; break;
      case 9: w = drop.sink; break;
      case 10: w = drop.window; break;
      default: break;
    }
    gstore<uint32_t>(blob + 4 * threadIdx.x, w);
  }
  uint8_t* layer_base = blob + kHeaderBytes + (size_t)lam * geo.layer_bytes();
  if (bits == 16) {
    encode_raw_block<DT>(a, it, layer_base, geo, lam, is_v, tile, strip, split, jump);
    return;
  }
  if (!is_v) {
    switch (bits) {
      case 8: encode_k_block<DT, 8>(a, it, layer_base, geo, lam, tile, strip, red, split, jump); break;
      case 4: encode_k_block<DT, 4>(a, it, layer_base, geo, lam, tile, strip, red, split, jump); break;
      default: encode_k_block<DT, 2>(a, it, layer_base, geo, lam, tile, strip, red, split, jump); break;
    }
  } else {
    switch (bits) {
      case 8: encode_v_block<DT, 8>(a, it, layer_base, geo, lam, tile, strip, split, jump); break;
      case 4: encode_v_block<DT, 4>(a, it, layer_base, geo, lam, tile, strip, split, jump); break;
      default: encode_v_block<DT, 2>(a, it, layer_base, geo, lam, tile, strip, split, jump); break;
    }
  }
}

int launch_encode(const EncodeParams& a, int dt, int n_items, int max_tokens, hipStream_t stream) {
  const int nstrips = (a.c + kStripCh - 1) / kStripCh;
  const int tiles = (max_tokens + kEncTile - 1) / kEncTile;
  dim3 grid((unsigned)(tiles * nstrips), (unsigned)(2 * a.l), (unsigned)n_items);
  EncodeParams b = a;
  b.max_tokens = max_tokens;
  // Plane group.  With the dispatcher dealing consecutive blocks to the 8 XCDs in turn, groups of 8 make every XCD
  // stream through one plane at a time; that is the default.  Long items do better with the two planes of a layer
  // alone (their sections of a blob are megabytes apart, and fewer planes at a time keep the writes together), and
  // short items of a source within 1 GiB with all planes in one group.  Measured at 8 / 4 / 2 bits, % of HBM peak:
  //   80 x 32768 tokens in 512-token items, all planes / groups of 8:  74.7 / 72.0 / 67.4   76.0 / 76.2 / 73.2
  //   32 x 8192 tokens in 256-token items (the benchmark's rotation):   71.4 / 76.3 / 74.5   69.9 / 74.3 / 73.5
  //   32 x 8192 tokens in one item, all / 8 / 2 (the kernel alone):     72.6 / 66.0 / 64.0   73.3 / 73.4 / 70.3   74.4 / 73.8 / 74.7
  //   32 x 32768 tokens in one item, all / 8 / 2:                       75.0 / 61.3 / 67.9   76.1 / 73.9 / 71.2   75.2 / 75.5 / 75.5
  //   32 x 32768 tokens in 2048-token items, all / 8 / 2:               74.7 / 75.5 / 69.3   75.5 / 77.5 / 78.0   74.3 / 76.5 / 75.9
  const bool near = (int64_t)a.l * a.layer_stride * 2 <= ((int64_t)1 << 29);
  b.plane_group = max_tokens >= 8192 ? 2 : near && max_tokens <= 512 ? 2 * a.l : 8;
  if (dt == KVH_F16)
    launch_kernel(encode_kernel<KVH_F16>, grid, dim3(kEncThreads), 0u, stream, b);
  else
    launch_kernel(encode_kernel<KVH_BF16>, grid, dim3(kEncThreads), 0u, stream, b);
  KVH_HIP_CHECK_LAUNCH();
  return KVH_OK;
}

}  // namespace kvh
