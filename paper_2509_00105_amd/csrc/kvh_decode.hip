// Level decoder: unpack b-bit codes, dequantise with the stored (min, max) of each group and
// write fp16/bf16 KV rows, contiguous or through a page table (the decompression whose
// cost the paper's estimator profiles; Design section).
//
// Streaming kernel.  The unit of work is one wave decoding 8 consecutive token rows of a
// 1024-channel span (two 512-channel segments), i.e. 16 KiB of contiguous output when c = 1024.
// A lane owns 8 channels per segment, so each store is one 128-bit access and the wave writes
// 1 KiB of a row per instruction.  A block is 8 such units: 64 consecutive rows of one span, which
// always lie in one K token-group.  K metadata (per channel) is turned into fp32 parameters either
// once per block, two channels per thread, and handed to the waves through 12 KiB of LDS (8 bits),
// or by every wave for the channels of its own lanes, with no barrier (4 and 2 bits); V metadata
// (per token and head) is prepared by one lane per group and broadcast inside the wave, and V blocks
// never meet at a barrier.  The rare groups whose top code does not land exactly on the stored
// maximum select a slower row loop through a uniform branch.  Stores are non-temporal, at 8 and 4
// bits also device-scoped; which form each level takes is measured, see kStoreThrough and kOwnK.
#include <type_traits>

#include "kvh_common.hpp"

namespace kvh {

#ifndef KVH_DEC_NT
#define KVH_DEC_NT 1  // non-temporal stores: decoded KV is not re-read by this kernel
#endif
#ifndef KVH_DEC_NTL
#define KVH_DEC_NTL 0  // non-temporal loads of the packed codes
#endif
#ifndef KVH_DEC_WAVES
#define KVH_DEC_WAVES 8
#endif
constexpr int kDecWaves = KVH_DEC_WAVES;                         // units per block
constexpr int kDecThreads = kDecWaves * kWave;
constexpr int kDecSegs = 2;                                      // 512-channel segments per wave
constexpr int kDecSpanCh = kDecSegs * kStripCh;                 // channels covered by one wave
constexpr int kDecHeads = kDecSpanCh / kGroup;                  // V groups per row of a unit
constexpr int kDecRows = kWave / kDecHeads;                     // token rows per wave: one lane per V group
#ifndef KVH_DEC_KOWN
#define KVH_DEC_KOWN -1  // K parameters prepared by every wave for itself: 1 always, 0 never, -1 per code width
#endif
#ifndef KVH_DEC_SUB
#define KVH_DEC_SUB 1
#endif
constexpr int kDecSub = KVH_DEC_SUB;                            // units a wave decodes one after the other
constexpr int kDecBlockRows = kDecRows * kDecSub * kDecWaves;   // token rows per block
static_assert(kGroup % kDecBlockRows == 0, "a block must not straddle K token-groups");
constexpr int kDecPrep = kDecSpanCh / kDecThreads;               // K channels of the block's span a thread prepares
static_assert(kDecThreads * kDecPrep == kDecSpanCh && (kDecPrep == 1 || kDecPrep == 2 || kDecPrep == 4), "K channels per thread");

typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

// Load through a pointer known to be in global memory (scalar or clang vector types only).
template <typename T>
__device__ __forceinline__ T gload(const uint8_t* p) {
  return *reinterpret_cast<const __attribute__((address_space(1))) T*>(reinterpret_cast<uintptr_t>(p));
}

// Same, for the streamed code words.
template <typename T>
__device__ __forceinline__ T gload_stream(const uint8_t* p) {
#if KVH_DEC_NTL
  return __builtin_nontemporal_load(
      reinterpret_cast<const __attribute__((address_space(1))) T*>(reinterpret_cast<uintptr_t>(p)));
#else
  return gload<T>(p);
#endif
}

// 16-byte store of decoded values, never re-read by this kernel: non-temporal.  With THROUGH the store also carries
// device scope (sc1), which makes the L2 pass the line on at once instead of holding it until it is evicted; the
// data written is the same.  Which levels gain from it is measured, see kStoreThrough below.  (The builtin has no
// form with both hints, hence the instruction is spelled out; it costs the immediate offsets the compiler would
// otherwise fold, two additions per store.  The s_nop is the wait state this chip family wants between a store of more
// than 8 bytes and a write to the registers that held its data; the compiler inserts it after its own stores and
// cannot see into this one.)
#ifndef KVH_DEC_THROUGH
#define KVH_DEC_THROUGH -1  // device-scope stores: 1 always, 0 never, -1 per code width
#endif
template <bool THROUGH>
__device__ __forceinline__ void gstore16(uint16_t* p, const uint4& v) {
  auto* g = reinterpret_cast<__attribute__((address_space(1))) uintx4*>(reinterpret_cast<uintptr_t>(p));
  uintx4 x = {v.x, v.y, v.z, v.w};
  if constexpr (THROUGH) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 0" ::"v"(g), "v"(x) : "memory");
  } else {
#if KVH_DEC_NT
    __builtin_nontemporal_store(x, g);
#else
    *g = x;
#endif
  }
}
// Six shapes from 1 to 16 GiB (8K to 128K tokens, 32 and 80 layers), % of HBM peak, plain / device-scope stores, each
// with the better K-parameter form: 8 bits 70.8 / 73.4 on average (better on every shape, +1.3 to +3.3), 4 bits
// 73.4 / 76.8 (every shape, +0.9 to +6.2), 2 bits 73.9 / 74.0 (from -5 on the 8K shape to +3).
template <int BITS>
constexpr bool kStoreThrough = KVH_DEC_THROUGH < 0 ? (BITS == 8 || BITS == 4) : KVH_DEC_THROUGH != 0;

typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Two fp32 values -> two 16-bit values in one word (element 0 in the low half), each rounded to
// nearest even.  gfx950 has packed converts for both types.
template <int DT>
__device__ __forceinline__ uint32_t pack2(float a, float b) {
  floatx2 f = {a, b};
  if constexpr (DT == KVH_F16) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, halfx2));
  } else {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
  }
}

template <int BITS>
struct Codes;
template <>
struct Codes<8> {
  uintx2 w;
  __device__ __forceinline__ void load(const uint8_t* p) { w = gload_stream<uintx2>(p); }
  __device__ __forceinline__ uint32_t get(int j) const { return ((j < 4 ? w.x : w.y) >> (8 * (j & 3))) & 0xffu; }
};
template <>
struct Codes<4> {
  uint32_t w;
  __device__ __forceinline__ void load(const uint8_t* p) { w = gload_stream<uint32_t>(p); }
  __device__ __forceinline__ uint32_t get(int j) const { return (w >> (4 * j)) & 0xfu; }
};
template <>
struct Codes<2> {
  uint32_t w;
  __device__ __forceinline__ void load(const uint8_t* p) { w = gload_stream<uint16_t>(p); }
  __device__ __forceinline__ uint32_t get(int j) const { return (w >> (2 * j)) & 0x3u; }
};

// fp32 reconstruction of one code; the 16-bit rounding happens in pack2.
__device__ __forceinline__ float recon(uint32_t q, float scale, float mn) {
  float y = __builtin_fmaf((float)q, scale, mn);
  // The definition rounds twice (fma to fp32, then fp32 to the 16-bit type).  Keep the compiler
  // from merging the two into a mixed-precision fma that rounds once straight to fp16.
  asm("" : "+v"(y));
  return y;
}

// Does code L need the explicit "decode to the stored maximum" rule for this group?
template <int DT, int BITS>
__device__ __forceinline__ bool top_needs_fix(const GroupParams& p) {
  constexpr uint32_t L = (1u << BITS) - 1u;
  return (pack2<DT>(recon(L, p.scale, p.mn), 0.0f) & 0xffffu) != p.top;
}

// Dequantise the 8 codes of one lane for one row.  param(j) gives the parameters of channel j.
template <int DT, int BITS, bool FIX, typename P>
__device__ __forceinline__ uint4 dequant8(const Codes<BITS>& cw, P&& param) {
  constexpr uint32_t L = (1u << BITS) - 1u;
  uint32_t w[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const GroupParams& p0 = param(2 * j);
    const GroupParams& p1 = param(2 * j + 1);
    uint32_t q0 = cw.get(2 * j), q1 = cw.get(2 * j + 1);
    w[j] = pack2<DT>(recon(q0, p0.scale, p0.mn), recon(q1, p1.scale, p1.mn));
    if constexpr (FIX) {
      if (q0 == L) w[j] = (w[j] & 0xffff0000u) | p0.top;
      if (q1 == L) w[j] = (w[j] & 0x0000ffffu) | (p1.top << 16);
    }
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// Physical row of logical position s, in two halves: row = entry * block_tokens + rest.  The page-table entry is
// only requested here; the product is formed by the caller after the unit's other loads have been issued, so that
// the first use of the entry does not hold them back by one trip to memory (a multiplication right behind the load
// makes the wave wait for it before it requests its codes).  Without a page table entry = 0 and rest = s.
struct RowRef {
  int32_t entry, rest;
};
__device__ __forceinline__ RowRef physical_row(int64_t s, const int32_t* page_table, int block_tokens) {
  if (page_table == nullptr) return {0, (int32_t)s};
  uint32_t su = (uint32_t)s, bt = (uint32_t)block_tokens;
  uint32_t blk = su / bt;
  return {gload<int32_t>(reinterpret_cast<const uint8_t*>(page_table + blk)), (int32_t)(su - blk * bt)};
}
__device__ __forceinline__ int32_t row_of(const RowRef& r, int block_tokens) { return r.entry * block_tokens + r.rest; }

struct HeaderWords {
  uintx4 a, b, c;
};
__device__ __forceinline__ HeaderWords load_header(const uint8_t* blob) {  // blob is wave-uniform
#if KVH_SCALAR_DESC
  return {sload<uintx4>(blob), sload<uintx4>(blob + 16), sload<uintx4>(blob + 32)};
#else
  return {gload<uintx4>(blob), gload<uintx4>(blob + 16), gload<uintx4>(blob + 32)};
#endif
}
__device__ __forceinline__ bool header_matches(const HeaderWords& h, int dt, int bits, int l, int n, int c,
                                               size_t total, uint32_t orig_tokens, uint32_t sink, uint32_t window) {
  return h.a.x == kMagic && h.a.y == (1u | (uint32_t)dt << 16 | (uint32_t)bits << 24) && h.a.z == (uint32_t)l &&
         h.a.w == (uint32_t)n && h.b.x == (uint32_t)c && h.b.y == ((uint32_t)kGroup | (uint32_t)kGroup << 16) &&
         h.b.z == (uint32_t)total && h.b.w == (uint32_t)((uint64_t)total >> 32) && h.c.x == orig_tokens &&
         h.c.y == sink && h.c.z == window;
}

// One wave's share of a block: kDecSub units of kDecRows consecutive rows each, one after the other.  Every load a
// unit needs (page-table entries, metadata, codes; for the first unit also the header) is issued up front so that
// their latencies overlap; the header verdict is taken before anything is stored.  (The compiler is free to move
// loads whose results are only needed past the verdict below it, and does so with the code words; keeping them in
// front of it was measured and changes nothing.)  The caller guarantees
// kvh_blob_size(l, n_tokens, c, level) readable bytes at the blob pointer, so these loads stay inside the buffer
// whatever the header says.
template <int DT, int BITS>
__device__ __forceinline__ void decode_unit(const DecodeParams& a, const kvh_item& it, int item_idx, int lam, bool is_v,
                                            int t0_wave, int span, float* kshare, int t0_block, const DropInfo& drop) {
  const int lane = threadIdx.x & (kWave - 1);
  const int n = it.n_tokens;
  const int c = a.c;
  const uint8_t* blob = static_cast<const uint8_t*>(it.blob);
  const LayerGeom geo = layer_geom(n, c, BITS);
  const HeaderWords hdr = load_header(blob);

  // segment s of this lane: 8 channels starting at ch[s]; idle lanes of a partial span shadow
  // channel 0 and never store
  bool active[kDecSegs];
  uint32_t ch[kDecSegs];
#pragma unroll
  for (int s = 0; s < kDecSegs; ++s) {
    int raw = span * kDecSpanCh + s * kStripCh + lane * kLaneCh;
    active[s] = raw < c;
    ch[s] = active[s] ? (uint32_t)raw : 0u;
  }

  const uint8_t* kmeta = blob + kHeaderBytes + (size_t)lam * geo.layer_bytes();
  const uint8_t* kcodes = kmeta + geo.kmeta;
  const uint8_t* vmeta = kcodes + geo.codes;
  const uint8_t* vcodes = vmeta + geo.vmeta;
  uint16_t* dst = (is_v ? a.v : a.k) + (int64_t)lam * a.layer_stride;
  const uint8_t* codes = is_v ? vcodes : kcodes;
  const int heads = c / kGroup;

  // what one unit loads: the destination row of row i (computed by lane i), the V metadata word of group
  // (row lane / H, head lane % H), and the code words
  RowRef my_ref = {0, 0};
  uint32_t vm = 0;
  bool v_owner = false;
  Codes<BITS> cw[kDecRows][kDecSegs];
  auto load_unit = [&](int t0) {
    {
      int t = t0 + (lane & (kDecRows - 1));
      const int64_t hop = t >= drop.split ? drop.jump : 0;
      my_ref = RowRef{0, 0};
      if (t < n) my_ref = physical_row(it.dst_token0 + t + hop, it.page_table, a.block_tokens);
    }
    if (is_v) {
      int t = t0 + lane / kDecHeads;
      int head = span * kDecHeads + lane % kDecHeads;
      v_owner = t < n && head < heads;
      vm = 0;
      if (v_owner) vm = gload<uint32_t>(vmeta + ((size_t)t * heads + head) * 4);
    }
#pragma unroll
    for (int i = 0; i < kDecRows; ++i) {
      int t = t0 + i;
      t = t < n ? t : n - 1;  // rows past the end re-read the last row and are not stored
#pragma unroll
      for (int s = 0; s < kDecSegs; ++s) cw[i][s].load(codes + (size_t)t * geo.row_bytes + ch[s] * BITS / 8);
    }
  };

  // K parameters, one of two ways.  Shared: every thread of the block prepares kDecPrep channels of the span, the
  // results meet in LDS behind one barrier.  Own: every wave prepares the 16 channels of each of its lanes itself
  // (8 times the arithmetic, which the short quotient forms made cheap, and 8 times the metadata reads, from L2), and
  // no wave waits for another.  Which is faster depends on the level and on the store form; average over the six
  // shapes named at kStoreThrough, shared / own: 8 bits (device-scope stores) 73.4 / 72.4 %, 4 bits (device-scope)
  // 73.0 / 76.8 %, 2 bits (plain non-temporal) 73.0 / 73.9 %.
  constexpr bool kOwnK = KVH_DEC_KOWN < 0 ? BITS != 8 : KVH_DEC_KOWN != 0;
  static_assert(!kOwnK || kDecSub == 1, "the own-parameter form takes one unit per wave");
  // K metadata: the channels of the span this thread prepares for the whole block
  uint32_t kwords[kDecPrep] = {};
  const int pc = span * kDecSpanCh + (int)threadIdx.x * kDecPrep;
  const bool pact = !kOwnK && !is_v && pc < c;  // c is a multiple of 128, so the thread's channels are all inside or all outside
  if (pact) {
    const uint8_t* mp = kmeta + ((size_t)(t0_block / kGroup) * c + pc) * 4;
    if constexpr (kDecPrep == 1) {
      kwords[0] = gload<uint32_t>(mp);
    } else if constexpr (kDecPrep == 2) {
      const uintx2 m = gload<uintx2>(mp);
      kwords[0] = m.x; kwords[1] = m.y;
    } else {
      const uintx4 m = gload<uintx4>(mp);
      kwords[0] = m.x; kwords[1] = m.y; kwords[2] = m.z; kwords[3] = m.w;
    }
  }
  uintx4 own_meta[kDecSegs][2] = {};
  if (kOwnK && !is_v) {
#pragma unroll
    for (int s = 0; s < kDecSegs; ++s) {
      const uint8_t* mp = kmeta + ((size_t)(t0_block / kGroup) * c + ch[s]) * 4;
      own_meta[s][0] = gload<uintx4>(mp);
      own_meta[s][1] = gload<uintx4>(mp + 16);
    }
  }
  load_unit(t0_wave);

  if (!header_matches(hdr, DT, BITS, a.l, n, c, kHeaderBytes + (size_t)a.l * geo.layer_bytes(), drop.orig_tokens,
                      drop.sink, drop.window)) {
    if (a.status != nullptr && lane == 0) a.status[item_idx] = KVH_DEV_HEADER_MISMATCH;
    return;
  }

  // the row loop of one unit, instantiated with and without the explicit top-code rule
  int32_t rows[kDecRows];
  auto run = [&](int t0, auto fix_tag, auto&& param_of) {
    constexpr bool FIX = decltype(fix_tag)::value;
#pragma unroll
    for (int i = 0; i < kDecRows; ++i) {
      if (t0 + i < n) {  // wave-uniform
        uint16_t* row = dst + (int64_t)rows[i] * a.token_stride;
#pragma unroll
        for (int s = 0; s < kDecSegs; ++s) {
          uint4 out = dequant8<DT, BITS, FIX>(cw[i][s], param_of(i, s));
          if (active[s]) gstore16<kStoreThrough<BITS>>(row + ch[s], out);
        }
      }
    }
  };
  using Yes = std::integral_constant<bool, true>;
  using No = std::integral_constant<bool, false>;

  if (!is_v) {
    // Every thread of the block prepares its channels of the span; the three arrays (minimum, scale,
    // top code) meet in LDS and every wave then picks up the 16 channels its lanes own.  All waves of
    // a K block reach the barrier, also those whose rows lie past the end of the blob.
    GroupParams gp[kDecSegs][kLaneCh];
    bool fix = false;
    if constexpr (kOwnK) {
    if (t0_wave >= n) return;  // wave-uniform; no barrier in this form
#pragma unroll
    for (int s = 0; s < kDecSegs; ++s) {
      const uint32_t w[kLaneCh] = {own_meta[s][0].x, own_meta[s][0].y, own_meta[s][0].z, own_meta[s][0].w,
                                   own_meta[s][1].x, own_meta[s][1].y, own_meta[s][1].z, own_meta[s][1].w};
#pragma unroll
      for (int j = 0; j < kLaneCh; ++j) {
        gp[s][j] = decode_params<DT, BITS>(w[j]);
        fix |= active[s] && top_needs_fix<DT, BITS>(gp[s][j]);
      }
    }
    {
      const bool any_fix = __builtin_amdgcn_ballot_w64(fix) != 0;
      auto param_of = [&](int, int s) { return [&gp, s](int j) -> const GroupParams& { return gp[s][j]; }; };
      const int32_t my_row = row_of(my_ref, a.block_tokens);
#pragma unroll
      for (int i = 0; i < kDecRows; ++i) rows[i] = __builtin_amdgcn_readlane(my_row, i);
      if (any_fix) run(t0_wave, Yes{}, param_of); else run(t0_wave, No{}, param_of);
      return;
    }
    }
    {
#pragma unroll
      for (int e = 0; e < kDecPrep; ++e) {
        GroupParams p = decode_params<DT, BITS>(kwords[e]);
        fix |= pact && top_needs_fix<DT, BITS>(p);
        const int lc = (int)threadIdx.x * kDecPrep + e;
        kshare[lc] = p.mn;
        kshare[kDecSpanCh + lc] = p.scale;
        kshare[2 * kDecSpanCh + lc] = __builtin_bit_cast(float, p.top);
      }
    }
    const bool any_fix = __syncthreads_or(fix);
    if (t0_wave >= n) return;  // wave-uniform, after the barrier
    // The common path never touches `top`; reading it only where the rule is needed keeps that path's register
    // count down.
    auto k_units = [&](auto fix_tag) {
      constexpr bool FIX = decltype(fix_tag)::value;
#pragma unroll
      for (int s = 0; s < kDecSegs; ++s) {
        const int base = s * kStripCh + lane * kLaneCh;
#pragma unroll
        for (int j = 0; j < kLaneCh; ++j) {
          gp[s][j].mn = kshare[base + j];
          gp[s][j].scale = kshare[kDecSpanCh + base + j];
          gp[s][j].top = FIX ? __builtin_bit_cast(uint32_t, kshare[2 * kDecSpanCh + base + j]) : 0u;
        }
      }
      auto param_of = [&](int, int s) { return [&gp, s](int j) -> const GroupParams& { return gp[s][j]; }; };
      auto unit = [&](int u) {
        const int t0 = t0_wave + u * kDecRows;
        if (u > 0) {
          if (t0 >= n) return;  // wave-uniform
          load_unit(t0);
        }
        const int32_t my_row = row_of(my_ref, a.block_tokens);
#pragma unroll
        for (int i = 0; i < kDecRows; ++i) rows[i] = __builtin_amdgcn_readlane(my_row, i);
        run(t0, fix_tag, param_of);
      };
      unit(0);
      if constexpr (kDecSub > 1) unit(1);
      if constexpr (kDecSub > 2) unit(2);
      if constexpr (kDecSub > 3) unit(3);
    };
    if (any_fix) k_units(Yes{}); else k_units(No{});
  } else {
    if (t0_wave >= n) return;  // wave-uniform; V waves never meet at a barrier
    auto unit = [&](int u) {
      const int t0 = t0_wave + u * kDecRows;
      if (u > 0) {
        if (t0 >= n) return;  // wave-uniform
        load_unit(t0);
      }
      const int32_t my_row = row_of(my_ref, a.block_tokens);
#pragma unroll
      for (int i = 0; i < kDecRows; ++i) rows[i] = __builtin_amdgcn_readlane(my_row, i);
      GroupParams mine = {0.0f, 0.0f, 0u};
      bool fix = false;
      if (v_owner) {
        mine = decode_params<DT, BITS>(vm);
        fix = top_needs_fix<DT, BITS>(mine);
      }
      const bool any_fix = __builtin_amdgcn_ballot_w64(fix) != 0;
      // every (row, segment) pulls its group's three values from the lane that prepared them
      auto param_of = [&](int i, int s) {
        int src = i * kDecHeads + s * (kStripCh / kGroup) + (lane >> 4);
        GroupParams p;
        p.mn = __shfl(mine.mn, src);
        p.scale = __shfl(mine.scale, src);
        p.top = __shfl(mine.top, src);
        return [p](int) -> const GroupParams& { return p; };
      };
      if (any_fix) run(t0, Yes{}, param_of); else run(t0, No{}, param_of);
    };
    unit(0);
    if constexpr (kDecSub > 1) unit(1);
    if constexpr (kDecSub > 2) unit(2);
    if constexpr (kDecSub > 3) unit(3);
  }
}

// Raw level: a unit copies its rows from the blob (K rows, then V rows, per layer) to their destination rows.
template <int DT>
__device__ __forceinline__ void decode_raw_unit(const DecodeParams& a, const kvh_item& it, int item_idx, int lam, bool is_v,
                                                int t0_wave, int span, const DropInfo& drop) {
  const int lane = threadIdx.x & (kWave - 1);
  const int n = it.n_tokens;
  const int c = a.c;
  const uint8_t* blob = static_cast<const uint8_t*>(it.blob);
  const LayerGeom geo = layer_geom(n, c, 16);
  const HeaderWords hdr = load_header(blob);
  bool active[kDecSegs];
  uint32_t ch[kDecSegs];
#pragma unroll
  for (int s = 0; s < kDecSegs; ++s) {
    int raw = span * kDecSpanCh + s * kStripCh + lane * kLaneCh;
    active[s] = raw < c;
    ch[s] = active[s] ? (uint32_t)raw : 0u;
  }
  const uint8_t* rows_in = blob + kHeaderBytes + (size_t)lam * geo.layer_bytes() + (is_v ? geo.codes : 0);
  uint16_t* dst = (is_v ? a.v : a.k) + (int64_t)lam * a.layer_stride;
  const bool ok = header_matches(hdr, DT, 16, a.l, n, c, kHeaderBytes + (size_t)a.l * geo.layer_bytes(), drop.orig_tokens,
                                 drop.sink, drop.window);
  if (!ok) {
    if (a.status != nullptr && lane == 0) a.status[item_idx] = KVH_DEV_HEADER_MISMATCH;
    return;
  }
#pragma unroll
  for (int u = 0; u < kDecSub; ++u) {
    const int t0 = t0_wave + u * kDecRows;
    if (t0 >= n) return;  // wave-uniform
    RowRef my_ref = {0, 0};
    {
      int t = t0 + (lane & (kDecRows - 1));
      const int64_t hop = t >= drop.split ? drop.jump : 0;
      if (t < n) my_ref = physical_row(it.dst_token0 + t + hop, it.page_table, a.block_tokens);
    }
    uintx4 d[kDecRows][kDecSegs];
#pragma unroll
    for (int i = 0; i < kDecRows; ++i) {
      int t = t0 + i;
      t = t < n ? t : n - 1;  // rows past the end re-read the last row and are not stored
#pragma unroll
      for (int s = 0; s < kDecSegs; ++s) d[i][s] = gload_stream<uintx4>(rows_in + (size_t)t * geo.row_bytes + ch[s] * 2u);
    }
    const int32_t my_row = row_of(my_ref, a.block_tokens);
#pragma unroll
    for (int i = 0; i < kDecRows; ++i) {
      const int32_t r = __builtin_amdgcn_readlane(my_row, i);
      if (t0 + i < n) {  // wave-uniform
        uint16_t* row = dst + (int64_t)r * a.token_stride;
#pragma unroll
        for (int s = 0; s < kDecSegs; ++s)
          if (active[s]) gstore16<kStoreThrough<16>>(row + ch[s], make_uint4(d[i][s].x, d[i][s].y, d[i][s].z, d[i][s].w));
      }
    }
  }
}

// grid = (64-row blocks x spans, 2 * l, items); span fastest; wave w of a block takes rows 8 w .. 8 w + 7 of its 64.
// Waves per SIMD the register allocation is held to (0 = compiler's choice).  The kernel needs about 100 registers,
// which would let two blocks (16 waves) share a CU; the write stream does better with fewer waves in flight.  Measured
// on the 8K-token shape with plain non-temporal stores, 8 / 4 / 2 bits, % of HBM peak in the benchmark's rotation:
// 16 waves per CU 68.4 / 71.6 / 71.3, this setting (allocation raised to three waves per SIMD, one block per CU)
// 70.4 / 73.8 / 74.5, two waves per SIMD 71.0 / 69.2 / 67.1; with the device-scope stores of the 8- and 4-bit levels
// the order is the same (16 waves per CU 70.6 / 73.6 / 72.8, this setting 73.0 / 70.9 / 69.3 before each level had its
// own store and parameter form, two waves per SIMD 71.7 / 68.5 / 66.2).
#ifndef KVH_DEC_WPE
#define KVH_DEC_WPE 3
#endif
#if KVH_DEC_WPE
#define KVH_DEC_OCC __attribute__((amdgpu_waves_per_eu(KVH_DEC_WPE, KVH_DEC_WPE)))
#else
#define KVH_DEC_OCC
#endif
template <int DT>
__global__ __launch_bounds__(kDecThreads) KVH_DEC_OCC void decode_kernel(DecodeParams a) {
  const int item_idx = blockIdx.z;
  // Block order: `row_tile` consecutive 64-row blocks of a plane, then the same rows of the next (layer, K|V)
  // plane, and so on through all planes, then the next tile of rows (the last tile may be smaller).  1 walks the
  // planes first, anything from the number of blocks per plane upwards walks plane by plane.
  int lay_kv, bx;
  {
    const int lin_xy = blockIdx.y * gridDim.x + blockIdx.x;
    const int per_plane = gridDim.x, planes = gridDim.y;
    const int rt = a.row_tile < 1 ? 1 : a.row_tile < per_plane ? a.row_tile : per_plane;
    const int full = per_plane / rt;
    const int tile = lin_xy / (rt * planes);
    const int first = (tile < full ? tile : full) * rt;          // first block (within a plane) of this tile
    const int size = tile < full ? rt : per_plane - full * rt;   // blocks per plane in it
    const int j = lin_xy - first * planes;
    lay_kv = j / size;
    bx = first + j % size;
  }
  kvh_item it;
  DropInfo drop = {kNoSplit, 0, 0u, 0u, 0u};  // ordinary batch items are never token-dropped
  bool consistent = true;
  const kvh_item* items = a.items;
  if (a.n_inline > 0) items = reinterpret_cast<const kvh_item*>(KVH_KERNARG_MEMBER(DecodeParams, inline_items));
  if (items != nullptr) {
    const uint8_t* p = reinterpret_cast<const uint8_t*>(items + item_idx);
#if KVH_SCALAR_DESC
    uintx4 lo = sload<uintx4>(p), hi = sload<uintx4>(p + 16);
#else
    uintx4 lo = gload<uintx4>(p), hi = gload<uintx4>(p + 16);
#endif
    it.blob = reinterpret_cast<const void*>((uint64_t)lo.x | (uint64_t)lo.y << 32);
    it.n_tokens = (int32_t)lo.z;
    it.level = (int32_t)lo.w;
    it.dst_token0 = (int64_t)((uint64_t)hi.x | (uint64_t)hi.y << 32);
    it.page_table = reinterpret_cast<const int32_t*>((uint64_t)hi.z | (uint64_t)hi.w << 32);
  } else if (a.kept_items != nullptr) {
    const uint8_t* p = reinterpret_cast<const uint8_t*>(a.kept_items + item_idx);
#if KVH_SCALAR_DESC
    uintx4 lo = sload<uintx4>(p), hi = sload<uintx4>(p + 16), ex = sload<uintx4>(p + 32);
#else
    uintx4 lo = gload<uintx4>(p), hi = gload<uintx4>(p + 16), ex = gload<uintx4>(p + 32);
#endif
    it.blob = reinterpret_cast<const void*>((uint64_t)lo.x | (uint64_t)lo.y << 32);
    it.n_tokens = (int32_t)lo.z;
    it.level = (int32_t)lo.w;
    it.dst_token0 = (int64_t)((uint64_t)hi.x | (uint64_t)hi.y << 32);
    it.page_table = reinterpret_cast<const int32_t*>((uint64_t)hi.z | (uint64_t)hi.w << 32);
    const uint32_t orig = (uint32_t)uniform((int32_t)ex.x), sink = (uint32_t)uniform((int32_t)ex.y),
                   window = (uint32_t)uniform((int32_t)ex.z);
    const bool compact = uniform((int32_t)ex.w) != 0;
    if ((orig | sink | window) != 0) {
      const uint64_t sw = (uint64_t)sink + window;
      const uint32_t kept = sw >= orig ? orig : (uint32_t)sw;
      consistent = orig <= 0x7fffffffu && sink <= 0x7fffffffu && window <= 0x7fffffffu && kept >= 1 &&
                   kept == (uint32_t)uniform(it.n_tokens);
      drop.orig_tokens = orig;
      drop.sink = sink;
      drop.window = window;
      if (consistent && kept < orig && !compact) {
        drop.split = (int32_t)sink;
        drop.jump = (int64_t)orig - window - sink;
      }
    }
  } else {
    it = a.one;
    drop = DropInfo{a.split, a.jump, a.hdr_orig_tokens, a.hdr_sink, a.hdr_window};
  }
  it.blob = uniform(it.blob);
  it.n_tokens = uniform(it.n_tokens);
  it.level = uniform(it.level);
  it.dst_token0 = uniform(it.dst_token0);
  it.page_table = uniform(it.page_table);
  // An item with more tokens than the grid covers, or whose rows leave the 31-bit row range, is refused as a
  // whole: partial output with a clean status word would be worse than none.
  {
    const int64_t reach = drop.split != kNoSplit ? (int64_t)drop.orig_tokens : (int64_t)it.n_tokens;
    if (it.n_tokens > a.max_tokens || it.dst_token0 < 0 || it.dst_token0 + reach > 0x7fffffffLL) consistent = false;
  }
  __shared__ float kshare[3 * kDecSpanCh];  // K parameters of the block's span: minima, scales, top codes
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nspans = (a.c + kDecSpanCh - 1) / kDecSpanCh;
  const int strip = bx % nspans;
  const int t0_block = (bx / nspans) * kDecBlockRows;
  const int t0 = t0_block + wave * (kDecRows * kDecSub);
  if (it.n_tokens < 1 || t0_block >= it.n_tokens) return;  // block-uniform
  const int lam = lay_kv >> 1;
  const bool is_v = lay_kv & 1;
  switch (consistent ? it.level : -1) {
    case 0: decode_unit<DT, 8>(a, it, item_idx, lam, is_v, t0, strip, kshare, t0_block, drop); break;
    case 1: decode_unit<DT, 4>(a, it, item_idx, lam, is_v, t0, strip, kshare, t0_block, drop); break;
    case 2: decode_unit<DT, 2>(a, it, item_idx, lam, is_v, t0, strip, kshare, t0_block, drop); break;
    case kRawLevel: decode_raw_unit<DT>(a, it, item_idx, lam, is_v, t0, strip, drop); break;
    default:
      if (a.status != nullptr && (threadIdx.x & (kWave - 1)) == 0) a.status[item_idx] = KVH_DEV_HEADER_MISMATCH;
      break;
  }
}

int launch_decode(const DecodeParams& a, int dt, int n_items, int max_tokens, hipStream_t stream) {
  const int nspans = (a.c + kDecSpanCh - 1) / kDecSpanCh;
  const unsigned gx = (unsigned)(((max_tokens + kDecBlockRows - 1) / kDecBlockRows) * nspans);
  dim3 grid(gx, (unsigned)(2 * a.l), (unsigned)n_items);
  DecodeParams b = a;
  b.max_tokens = max_tokens;
  // Row tile.  Destination planes within 1 GiB of each other: planes first (one block per plane and turn), worth
  // 1-2 % there over anything longer.  Beyond that: four blocks (256 rows) per plane and turn for items of up to
  // 8,192 tokens, plane by plane for longer ones.  Measured on ten tensors of 2.5 to 16 GiB (8 to 80 layers, 8K to
  // 128K tokens) against walking plane by plane, the kernel alone, 8 / 4 / 2 bits in points of HBM peak: items of 512
  // tokens -1.4 to +3.9 / -1.6 to +5.3 / -0.4 to +4.9, of 1,024 tokens +0.9 to +8.9 / +1.0 to +11.8 / +2.2 to +9.2
  // (walking plane by plane has a hole there, 67-69 % on most tensors), of 4,096 tokens -1.8 to +5.1 / -1.0 to +6.9 /
  // -3.6 to +6.2; one item of 16,384 tokens +0.8 to +4.3 / -6.3 to +1.0 / -3.4 to +1.1, hence the limit.  Tiles of
  // 2 are a point below tiles of 4, tiles of 8 two to four, tiles of 16 are the hole again.
  const bool near = (int64_t)a.l * a.layer_stride * 2 <= ((int64_t)1 << 29);
  b.row_tile = near ? 1 : max_tokens <= 8192 ? 4 : 0x7fffffff;
  if (dt == KVH_F16)
    launch_kernel(decode_kernel<KVH_F16>, grid, dim3(kDecThreads), 0u, stream, b);
  else
    launch_kernel(decode_kernel<KVH_BF16>, grid, dim3(kDecThreads), 0u, stream, b);
  KVH_HIP_CHECK_LAUNCH();
  return KVH_OK;
}

}  // namespace kvh
