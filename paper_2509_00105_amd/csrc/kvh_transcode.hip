// Level transcoder: re-compress a stored blob from b_in to b_out bits per element without ever
// writing 16-bit KV to memory (the policy's step that compresses a stored entry further; Design section,
// marginal utility drop).  The result is, byte for byte, encode(decode(blob)).
//
// Why no statistics pass is needed: in a blob written by the encoder (or by this kernel) every
// group holds code 0 and code L.  Code 0 decodes to the stored minimum exactly, code L to the
// stored maximum, and every other code to something in between, so the minimum and maximum of
// the decoded group are the stored ones and the re-encoded group keeps its metadata word.  The
// one exception is a degenerate group (range below 2^-100): all its elements decode to the
// minimum, so its new word is (mn, mn).  With the statistics known up front the kernel is a
// pure stream: code in -> fp32 reconstruction -> rounding to the 16-bit type -> position in the
// same range at the new rate -> code out.
//
// Block = 8 waves x 16 token rows = one K token-group x a 1024-channel span; a lane owns 16
// consecutive channels, so a wave moves one whole code row of the span per access (16 / 8 / 4
// bytes per lane at 8 / 4 / 2 bits).  K parameters (per channel) are prepared once per block,
// two channels per thread, and shared through LDS; V parameters (per token and head) are
// prepared by one lane per group and broadcast inside the wave.  When the whole code -> code map
// of a group fits one register (4 -> 2 and the pairs that start from 2 bits) the "parameters"
// are that map, built by running the arithmetic once per input code, and an element costs a
// shift and a funnel shift.
#include <type_traits>

#include "kvh_common.hpp"

namespace kvh {

#ifndef KVH_TC_NT
#define KVH_TC_NT 1  // non-temporal stores of the output codes
#endif

#ifndef KVH_TC_WPE
#define KVH_TC_WPE 4  // waves per SIMD the register allocation is held to (0 = compiler's choice): two blocks per CU
#endif
#if KVH_TC_WPE
#define KVH_TC_OCC __attribute__((amdgpu_waves_per_eu(KVH_TC_WPE, KVH_TC_WPE)))
#else
#define KVH_TC_OCC
#endif

constexpr int kTcWaves = 8;
constexpr int kTcThreads = kTcWaves * kWave;      // 512
constexpr int kTcLaneCh = 16;                     // channels per lane
constexpr int kTcSpanCh = kWave * kTcLaneCh;      // 1024 channels per wave access
constexpr int kTcRows = kGroup / kTcWaves;        // 16 rows per wave
constexpr int kTcBatch = 8;                       // rows in flight per wave
constexpr int kTcSpanHeads = kTcSpanCh / kGroup;  // 8 V groups per row of a span
static_assert(kTcBatch * kTcSpanHeads == kWave, "one lane per V group of a batch");
static_assert(kTcThreads * 2 == kTcSpanCh, "two K channels per thread");

typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

namespace {

template <typename T>
__device__ __forceinline__ T gload(const uint8_t* p) {
  return *reinterpret_cast<const __attribute__((address_space(1))) T*>(reinterpret_cast<uintptr_t>(p));
}
#ifndef KVH_TC_NTL
#define KVH_TC_NTL 1  // non-temporal loads of the input codes
#endif
template <typename T>
__device__ __forceinline__ T gload_codes(const uint8_t* p) {
#if KVH_TC_NTL
  return __builtin_nontemporal_load(reinterpret_cast<const __attribute__((address_space(1))) T*>(reinterpret_cast<uintptr_t>(p)));
#else
  return gload<T>(p);
#endif
}
template <typename T>
__device__ __forceinline__ void gstore(uint8_t* p, T v) {
  *reinterpret_cast<__attribute__((address_space(1))) T*>(reinterpret_cast<uintptr_t>(p)) = v;
}
template <typename T>
__device__ __forceinline__ void gstore_stream(uint8_t* p, T v) {
#if KVH_TC_NT
  __builtin_nontemporal_store(v, reinterpret_cast<__attribute__((address_space(1))) T*>(reinterpret_cast<uintptr_t>(p)));
#else
  gstore<T>(p, v);
#endif
}

// Two fp32 values -> two 16-bit values in one word, each rounded to nearest even.
template <int DT>
__device__ __forceinline__ uint32_t pack2(float a, float b) {
  floatx2 f = {a, b};
  if constexpr (DT == KVH_F16) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, halfx2));
  } else {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
  }
}

// fp32 reconstruction of a code.  The definition rounds twice (fma to fp32, then to the 16-bit
// type); the empty asm keeps the compiler from merging the two into one mixed-precision fma.
__device__ __forceinline__ float recon(float q, float scale, float mn) {
  float y = __builtin_fmaf(q, scale, mn);
  asm("" : "+v"(y));
  return y;
}

// The 16 input codes of a lane.  spread() lays them out one per byte (4 words), so that each code
// then costs a single byte->float convert; the empty asm keeps the compiler from undoing that
// into one bit-field extract plus one convert per code.
__device__ __forceinline__ uint32_t opaque(uint32_t x) {
  asm("" : "+v"(x));
  return x;
}
template <int BITS>
struct InCodes;
template <>
struct InCodes<8> {
  uintx4 w;
  __device__ __forceinline__ void load(const uint8_t* p) { w = gload_codes<uintx4>(p); }
  __device__ __forceinline__ float get(const uint32_t (&e)[4], int j) const { return (float)((e[j >> 2] >> (8 * (j & 3))) & 0xffu); }
  __device__ __forceinline__ void spread(uint32_t (&e)[4]) const {
    e[0] = w.x; e[1] = w.y; e[2] = w.z; e[3] = w.w;
  }
};
template <>
struct InCodes<4> {
  uintx2 w;
  __device__ __forceinline__ void load(const uint8_t* p) { w = gload_codes<uintx2>(p); }
  // e[0] / e[1] = even / odd nibbles of the first word, e[2] / e[3] of the second
  __device__ __forceinline__ void spread(uint32_t (&e)[4]) const {
    e[0] = opaque(w.x & 0x0f0f0f0fu);
    e[1] = opaque((w.x >> 4) & 0x0f0f0f0fu);
    e[2] = opaque(w.y & 0x0f0f0f0fu);
    e[3] = opaque((w.y >> 4) & 0x0f0f0f0fu);
  }
  __device__ __forceinline__ float get(const uint32_t (&e)[4], int j) const {
    return (float)((e[(j >> 3) * 2 + (j & 1)] >> (8 * ((j & 7) >> 1))) & 0xffu);
  }
};
template <>
struct InCodes<2> {
  uint32_t w;
  __device__ __forceinline__ void load(const uint8_t* p) { w = gload_codes<uint32_t>(p); }
  // e[k] holds codes k, k + 4, k + 8, k + 12 in its four bytes
  __device__ __forceinline__ void spread(uint32_t (&e)[4]) const {
#pragma unroll
    for (int k = 0; k < 4; ++k) e[k] = opaque((w >> (2 * k)) & 0x03030303u);
  }
  __device__ __forceinline__ float get(const uint32_t (&e)[4], int j) const {
    return (float)((e[j & 3] >> (8 * (j >> 2))) & 0xffu);
  }
};

// Four positions -> four code bytes in one word; the convert rounds to nearest even and
// saturates to [0, 255].
__device__ __forceinline__ uint32_t codes4(float t0, float t1, float t2, float t3) {
  uint32_t a = __builtin_amdgcn_cvt_pk_u8_f32(t0, 0, 0u);
  a = __builtin_amdgcn_cvt_pk_u8_f32(t1, 1, a);
  a = __builtin_amdgcn_cvt_pk_u8_f32(t2, 2, a);
  return __builtin_amdgcn_cvt_pk_u8_f32(t3, 3, a);
}

// Pack 16 positions into BITS-bit codes (channel order, LSB first) and store them.  The convert
// puts a code into any byte of a word, so narrow codes are routed at that point: word i receives,
// in its byte k, the code that belongs i fields above the bottom of output byte k, and the words
// are then merged with one shift-or each.  (For finite positions every code is <= L, so fields
// never overlap.)
template <int BITS>
__device__ __forceinline__ void store_codes16(uint8_t* p, const float (&t)[16]) {
  if constexpr (BITS == 8) {
    uintx4 o;
    o.x = codes4(t[0], t[1], t[2], t[3]);
    o.y = codes4(t[4], t[5], t[6], t[7]);
    o.z = codes4(t[8], t[9], t[10], t[11]);
    o.w = codes4(t[12], t[13], t[14], t[15]);
    gstore_stream<uintx4>(p, o);
  } else if constexpr (BITS == 4) {
    uintx2 o;
    o.x = codes4(t[0], t[2], t[4], t[6]) | codes4(t[1], t[3], t[5], t[7]) << 4;
    o.y = codes4(t[8], t[10], t[12], t[14]) | codes4(t[9], t[11], t[13], t[15]) << 4;
    gstore_stream<uintx2>(p, o);
  } else {
    uint32_t o = codes4(t[0], t[4], t[8], t[12]) | codes4(t[1], t[5], t[9], t[13]) << 2 |
                 codes4(t[2], t[6], t[10], t[14]) << 4 | codes4(t[3], t[7], t[11], t[15]) << 6;
    gstore_stream<uint32_t>(p, o);
  }
}

// Everything one group contributes to the arithmetic, as fp32.
struct TcParams {
  float mn;     // f32(mn)
  float scale;  // r / L_in, or 0 (degenerate)
  float inv;    // L_out / r, or 0 (degenerate)
  float top;    // what code L_in decodes to: f32(mx), or f32(mn) (degenerate)
};

// Parameters of a group from its metadata word; also the word the re-encoded group stores and
// whether code L_in needs the explicit "decode to the stored maximum" rule.
template <int DT, int BI, int BO>
__device__ __forceinline__ TcParams tc_params(uint32_t meta, uint32_t& out_meta, bool& fix) {
  constexpr float LI = float((1 << BI) - 1), LO = float((1 << BO) - 1);
  TcParams p;
  const uint32_t mn_bits = meta & 0xffffu, mx_bits = meta >> 16;
  p.mn = t16_to_f32<DT>(mn_bits);
  const float r = t16_to_f32<DT>(mx_bits) - p.mn;
  const bool degenerate = r < 0x1p-100f;
  p.scale = degenerate ? 0.0f : range_over_levels<BI>(r);  // correctly rounded quotients
  p.inv = degenerate ? 0.0f : levels_over_range<BO>(r);
  const uint32_t top_bits = degenerate ? mn_bits : mx_bits;
  p.top = t16_to_f32<DT>(top_bits);
  out_meta = mn_bits | top_bits << 16;
  fix = (pack2<DT>(recon(LI, p.scale, p.mn), 0.0f) & 0xffffu) != top_bits;
  return p;
}

// One row of a lane: 16 codes in, 16 codes out.  param(j) gives the parameters of channel j.
template <int DT, int BI, int BO, bool FIX, typename P>
__device__ __forceinline__ void transcode_row(uint8_t* out, const InCodes<BI>& cw, P&& param) {
  constexpr float LI = float((1 << BI) - 1);
  float t[kTcLaneCh];
  uint32_t e[4];
  cw.spread(e);
#pragma unroll
  for (int j = 0; j < kTcLaneCh; j += 2) {
    const TcParams& p0 = param(j);
    const TcParams& p1 = param(j + 1);
    const float q0 = cw.get(e, j), q1 = cw.get(e, j + 1);
    float x0, x1;
    if constexpr (DT == KVH_BF16) {
      // a bf16 value in the upper half of a word over a zero lower half is that value as fp32: one convert per
      // element rounds and widens at once (a pair packed together would need unpacking, half an operation more)
      x0 = __builtin_bit_cast(float, pack2<DT>(0.0f, recon(q0, p0.scale, p0.mn)));
      x1 = __builtin_bit_cast(float, pack2<DT>(0.0f, recon(q1, p1.scale, p1.mn)));
    } else {
      const uint32_t pk = pack2<DT>(recon(q0, p0.scale, p0.mn), recon(q1, p1.scale, p1.mn));
      x0 = t16_to_f32<DT>(pk & 0xffffu);
      x1 = t16_to_f32<DT>(pk >> 16);
    }
    if constexpr (FIX) {
      x0 = q0 == LI ? p0.top : x0;
      x1 = q1 == LI ? p1.top : x1;
    }
    // position in the range at the new rate: subtract, then multiply (two roundings)
    t[j] = (x0 - p0.mn) * p0.inv;
    t[j + 1] = (x1 - p1.mn) * p1.inv;
  }
  store_codes16<BO>(out, t);
}

// ---- narrow inputs: one small table per group ---------------------------------------------------
// With b_in <= 4 a group has at most 16 distinct input codes, so its whole code -> code map fits one
// register when 2^b_in * b_out <= 32 (4 -> 2, 2 -> 2, 2 -> 4, 2 -> 8).  The map is built by running
// the arithmetic above once per input code; an element then costs a shift and a funnel shift
// instead of seven floating-point instructions.
template <int BI, int BO>
constexpr bool kUseTable = (1 << BI) * BO <= 32;

template <int DT, int BI, int BO>
__device__ __forceinline__ uint32_t code_table(uint32_t meta, uint32_t& out_meta) {
  constexpr int NQ = 1 << BI;
  bool fix;
  const TcParams p = tc_params<DT, BI, BO>(meta, out_meta, fix);
  uint32_t table = 0;
#pragma unroll
  for (int q = 0; q < NQ; q += 2) {
    const uint32_t pk = pack2<DT>(recon((float)q, p.scale, p.mn), recon((float)(q + 1), p.scale, p.mn));
    const float x0 = t16_to_f32<DT>(pk & 0xffffu);
    const float x1 = q + 1 == NQ - 1 ? p.top : t16_to_f32<DT>(pk >> 16);  // the top code decodes to the stored maximum
    const uint32_t two = __builtin_amdgcn_cvt_pk_u8_f32((x1 - p.mn) * p.inv, 1,
                                                        __builtin_amdgcn_cvt_pk_u8_f32((x0 - p.mn) * p.inv, 0, 0u));
    table |= ((two & 0xffu) | ((two >> 8) & 0xffu) << BO) << (BO * q);
  }
  return table;
}

// Byte-wise shift amounts b_out * q for the 16 codes of a lane: code j sits in byte sh_byte(j) of
// e[sh_word(j)].
template <int BI, int BO>
struct Shifts;
template <int BO>
struct Shifts<4, BO> {
  static constexpr int S = BO == 2 ? 1 : BO == 4 ? 2 : 3;
  static constexpr uint32_t M = 0x0f0f0f0fu << S;
  static __device__ __forceinline__ void make(const InCodes<4>& cw, uint32_t (&e)[4]) {
    e[0] = opaque((cw.w.x << S) & M);
    e[1] = opaque((cw.w.x >> (4 - S)) & M);
    e[2] = opaque((cw.w.y << S) & M);
    e[3] = opaque((cw.w.y >> (4 - S)) & M);
  }
  static constexpr int word(int j) { return (j >> 3) * 2 + (j & 1); }
  static constexpr int byte(int j) { return (j & 7) >> 1; }
};
template <int BO>
struct Shifts<2, BO> {
  static constexpr int S = BO == 2 ? 1 : BO == 4 ? 2 : 3;
  static constexpr uint32_t M = 0x03030303u << S;
  static __device__ __forceinline__ void make(const InCodes<2>& cw, uint32_t (&e)[4]) {
#pragma unroll
    for (int k = 0; k < 4; ++k) e[k] = opaque((2 * k >= S ? cw.w >> (2 * k - S) : cw.w << (S - 2 * k)) & M);
  }
  static constexpr int word(int j) { return j & 3; }
  static constexpr int byte(int j) { return j >> 2; }
};

// One row of a lane through the tables.  table(j) gives the table of channel j.
template <int BI, int BO, typename T>
__device__ __forceinline__ void lookup_row(uint8_t* out, const InCodes<BI>& cw, T&& table) {
  using Sh = Shifts<BI, BO>;
  constexpr int kPer = 32 / BO;  // codes per output word
  uint32_t e[4];
  Sh::make(cw, e);
  uint32_t acc[kTcLaneCh / kPer] = {};
#pragma unroll
  for (int j = 0; j < kTcLaneCh; ++j) {
    const uint32_t x = table(j) >> ((e[Sh::word(j)] >> (8 * Sh::byte(j))) & 0xffu);
    // funnel shift: the low b_out bits of x enter at the top; after kPer steps code j sits at bit b_out * (j % kPer)
    acc[j / kPer] = __builtin_amdgcn_alignbit(x, acc[j / kPer], BO);
  }
  if constexpr (BO == 2) {
    gstore_stream<uint32_t>(out, acc[0]);
  } else if constexpr (BO == 4) {
    uintx2 o = {acc[0], acc[1]};
    gstore_stream<uintx2>(out, o);
  } else {
    uintx4 o = {acc[0], acc[1], acc[2], acc[3]};
    gstore_stream<uintx4>(out, o);
  }
}

// ---- 8 -> 2 bits: the code -> code map of a group as a polynomial of the input code ------------------
// The map f(q) of a group (reconstruct, round to the 16-bit type, re-position, round to a code) is a monotone step
// function of q with three steps, because every operation in it is monotone.  If some cheap monotone function
// g(q) is shown to round to f(q) at the last code before each step and at the first code of each step (and at both
// ends), the two agree at all 256 codes, and an element costs  byte -> float, g, float -> code  instead of the seven
// floating-point instructions of the definition.  Two forms of g are used:
//   standard  g(q) = q / 85: steps at 43, 128, 213, which is where the steps of a group lie unless the rounding to
//             the 16-bit type moves them (it does when the group sits far from zero compared with its range);
//             recognised by evaluating f at the six codes around those steps;
//   fitted    the parabola through the three step positions of the group, found by evaluating f itself, and
//             accepted only if evaluating it with the very instructions of the row loop reproduces f at the codes
//             around its steps and at both ends, with a slope that keeps it monotone.
// A group that passes neither test (a range of a few units in the last place, say) sends its block, or its batch
// of V rows, down the arithmetic route above.  Bit-exactness therefore never rests on the fit, only on the checks.
struct Quad {
  float a, b, c;  // g(q) = (a q + b) q + c
};
enum : uint32_t { kStandard = 0u, kFitted = 1u, kHard = 2u };

// f(q) by the definition (the top code decodes to the stored maximum).
template <int DT>
__device__ __forceinline__ uint32_t code82(float q, const TcParams& p) {
  const uint32_t pk = pack2<DT>(recon(q, p.scale, p.mn), 0.0f);
  float x = t16_to_f32<DT>(pk & 0xffffu);
  x = q == 255.0f ? p.top : x;
  return __builtin_amdgcn_cvt_pk_u8_f32((x - p.mn) * p.inv, 0, 0u);
}
// g(q) exactly as the row loop evaluates it
__device__ __forceinline__ float quad_value(float q, const Quad& g) { return __builtin_fmaf(__builtin_fmaf(g.a, q, g.b), q, g.c); }
__device__ __forceinline__ uint32_t quad_code(float q, const Quad& g) { return __builtin_amdgcn_cvt_pk_u8_f32(quad_value(q, g), 0, 0u); }

template <int DT>
__device__ __forceinline__ uint32_t classify82(const TcParams& p, Quad& g) {
  g = Quad{0.0f, 0.0f, 0.0f};
  if (p.inv == 0.0f) return kFitted;  // degenerate group: every code becomes 0, and so does g
  const bool standard = code82<DT>(42.0f, p) == 0u && code82<DT>(43.0f, p) == 1u && code82<DT>(127.0f, p) == 1u &&
                        code82<DT>(128.0f, p) == 2u && code82<DT>(212.0f, p) == 2u && code82<DT>(213.0f, p) == 3u;
  if (standard) {
    g.b = 1.0f / 85.0f;  // what a standard group contributes where its neighbours need the fitted form
    return kStandard;
  }
  // First code of each step.  The steps lie within a few codes of 43, 128, 213, so each is looked for from there,
  // one code at a time in the direction the two evaluations at the usual place point to; a step further away than
  // kReach codes makes the group a hard one.
  constexpr int kReach = 6;
  float t[3];
  bool found = true;
#pragma unroll
  for (int k = 1; k <= 3; ++k) {
    const float hi0 = k == 1 ? 43.0f : k == 2 ? 128.0f : 213.0f;
    const bool below = code82<DT>(hi0 - 1.0f, p) >= (uint32_t)k;  // the step is at or before the code below the usual place
    const bool above = code82<DT>(hi0, p) < (uint32_t)k;          // the step is after the usual place
    float tk = hi0;
    bool searching = below || above;
    const float dir = below ? -1.0f : 1.0f;
    float q = below ? hi0 - 1.0f : hi0;
#pragma unroll 1
    for (int step = 0; step < kReach && __builtin_amdgcn_ballot_w64(searching) != 0; ++step) {
      q += dir;
      const bool ge = code82<DT>(q, p) >= (uint32_t)k;
      if (searching && ge != below) {  // crossed the step: going up, q is its first code; going down, q + 1 is
        tk = below ? q + 1.0f : q;
        searching = false;
      }
    }
    found = found && !searching;
    t[k - 1] = tk;
  }
  if (!found || !(t[0] >= 1.0f && t[0] < t[1] && t[1] < t[2] && t[2] <= 255.0f)) return kHard;
  // parabola through (t_k - 1/2, k - 1/2); approximate reciprocals will do, the checks below are what counts
  const float x1 = t[0] - 0.5f, x2 = t[1] - 0.5f, x3 = t[2] - 0.5f;
  const float d1 = __builtin_amdgcn_rcpf(x2 - x1), d2 = __builtin_amdgcn_rcpf(x3 - x2);
  g.a = (d2 - d1) * __builtin_amdgcn_rcpf(x3 - x1);
  g.b = d1 - g.a * (x1 + x2);
  g.c = 0.5f - (g.a * x1 + g.b) * x1;
  bool ok = quad_code(0.0f, g) == 0u && quad_code(255.0f, g) == 3u;
#pragma unroll
  for (int k = 1; k <= 3; ++k) ok = ok && quad_code(t[k - 1] - 1.0f, g) == (uint32_t)(k - 1) && quad_code(t[k - 1], g) == (uint32_t)k;
  // slope at both ends well above what rounding errors in g could undo
  ok = ok && g.b >= 0x1p-9f && __builtin_fmaf(510.0f, g.a, g.b) >= 0x1p-9f;
  return ok ? kFitted : kHard;
}

// One row of a lane through g.  coef(j) gives the polynomial of channel j (unused when STANDARD).
template <bool STANDARD, typename C>
__device__ __forceinline__ void poly_row82(uint8_t* out, const InCodes<8>& cw, C&& coef) {
  constexpr float kStep = 1.0f / 85.0f;
  float t[kTcLaneCh];
  uint32_t e[4];
  cw.spread(e);
#pragma unroll
  for (int j = 0; j < kTcLaneCh; ++j) {
    const float q = cw.get(e, j);
    if constexpr (STANDARD) t[j] = q * kStep; else t[j] = quad_value(q, coef(j));
  }
  store_codes16<2>(out, t);
}

struct HeaderWords {
  uintx4 a, b, c;
};

// Header of the source blob against the call; the token-dropping words are accepted if they are
// all zero or describe an entry of which exactly n tokens are kept.
__device__ __forceinline__ bool source_header_ok(const HeaderWords& h, int dt, int bits, int l, int n, int c, size_t total) {
  const bool fields = h.a.x == kMagic && h.a.y == (1u | (uint32_t)dt << 16 | (uint32_t)bits << 24) && h.a.z == (uint32_t)l &&
                      h.a.w == (uint32_t)n && h.b.x == (uint32_t)c && h.b.y == ((uint32_t)kGroup | (uint32_t)kGroup << 16) &&
                      h.b.z == (uint32_t)total && h.b.w == (uint32_t)((uint64_t)total >> 32);
  const uint32_t orig = h.c.x, sink = h.c.y, window = h.c.z;
  const uint64_t sw = (uint64_t)sink + window;
  const bool plain = (orig | sink | window) == 0;
  const bool dropped = orig >= 1 && orig <= 0x7fffffffu && sw >= 1 && sw <= 0x7fffffffu &&
                       (sw >= orig ? orig : (uint32_t)sw) == (uint32_t)n;
  return fields && (plain || dropped);
}

template <int DT, int BI, int BO>
__device__ __forceinline__ void transcode_block(const TranscodeParams& a, const kvh_tc_item& it, int item_idx, int lam,
                                                bool is_v, int g, int span, TcParams* kpar, float* kquad,
                                                uint32_t* kflags) {
  using Yes = std::integral_constant<bool, true>;
  using No = std::integral_constant<bool, false>;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = it.n_tokens;
  const int c = a.c;
  const int heads = c / kGroup;
  const uint8_t* src = static_cast<const uint8_t*>(it.src);
  uint8_t* dst = static_cast<uint8_t*>(it.dst);
  const LayerGeom gi = layer_geom(n, c, BI), go = layer_geom(n, c, BO);
  const HeaderWords hdr = {gload<uintx4>(src), gload<uintx4>(src + 16), gload<uintx4>(src + 32)};

  const int ch_raw = span * kTcSpanCh + lane * kTcLaneCh;
  const bool active = ch_raw < c;  // idle lanes of a partial span shadow channel 0 and never store
  const uint32_t ch = active ? (uint32_t)ch_raw : 0u;
  const int t_first = g * kGroup + wave * kTcRows;

  const uint8_t* in_layer = src + kHeaderBytes + (size_t)lam * gi.layer_bytes();
  uint8_t* out_layer = dst + kHeaderBytes + (size_t)lam * go.layer_bytes();
  const uint8_t* in_codes = in_layer + gi.kmeta + (is_v ? gi.codes + gi.vmeta : 0) + ch * BI / 8;
  uint8_t* out_codes = out_layer + go.kmeta + (is_v ? go.codes + go.vmeta : 0) + ch * BO / 8;

  // Rows in flight per wave.  Narrow codes (2 registers a row or less) are loaded for all 16 rows of
  // the wave at once: one round trip to memory instead of two, and twice the bytes in flight.  With
  // 8-bit input a row takes 4 registers; a K wave also holds the parameters of its 16 channels
  // (48 registers), so it takes 4 rows at a time and a V wave 8.
  constexpr int kRowsK = BI == 8 ? kTcBatch / 2 : kTcRows;
  constexpr int kRowsV = BI == 8 ? kTcBatch : kTcRows;
  InCodes<BI> cw[kRowsV];
  auto load_batch = [&](int t0, auto rows_tag) {
#pragma unroll
    for (int i = 0; i < decltype(rows_tag)::value; ++i) {
      int t = t0 + i;
      t = t < n ? t : n - 1;  // rows past the end re-read the last row and are not stored
      cw[i].load(in_codes + (size_t)t * gi.row_bytes);
    }
  };
  // rows t0 .. t0 + rows - 1, held in cw[first ..]
  auto run_batch = [&](int t0, auto first_tag, auto rows_tag, auto fix_tag, auto&& param_of) {
    constexpr bool FIX = decltype(fix_tag)::value;
    constexpr int kFirst = decltype(first_tag)::value;
#pragma unroll
    for (int i = 0; i < decltype(rows_tag)::value; ++i) {
      if (t0 + i < n) {  // wave-uniform
        auto param = param_of(i);  // may shuffle across lanes: taken with the whole wave enabled
        if (active) transcode_row<DT, BI, BO, FIX>(out_codes + (size_t)(t0 + i) * go.row_bytes, cw[kFirst + i], param);
      }
      __builtin_amdgcn_sched_barrier(0);  // one row at a time: keeps the temporaries of different rows apart
    }
  };
  using Zero = std::integral_constant<int, 0>;
  using Eight = std::integral_constant<int, kTcBatch>;
  using Batch = std::integral_constant<int, kTcBatch>;
  using RowsK = std::integral_constant<int, kRowsK>;
  using RowsV = std::integral_constant<int, kRowsV>;

  // The caller guarantees kvh_blob_size(l, n_tokens, c, level_in) readable bytes at the source,
  // so the loads issued before the header verdict stay inside the buffer whatever it says.
  if (t_first < n) {
    if (is_v) load_batch(t_first, RowsV{}); else load_batch(t_first, RowsK{});
  }

  uintx2 km = {0u, 0u};
  const int pc = span * kTcSpanCh + (int)threadIdx.x * 2;  // the two K channels this thread prepares
  const bool pact = !is_v && pc < c;
  if (pact) km = gload<uintx2>(in_layer + ((size_t)g * c + pc) * 4);

  // block-uniform verdict: every thread reads the same header
  if (!source_header_ok(hdr, DT, BI, a.l, n, c, kHeaderBytes + (size_t)a.l * gi.layer_bytes())) {
    if (a.status != nullptr && threadIdx.x == 0) a.status[item_idx] = KVH_DEV_HEADER_MISMATCH;
    return;
  }
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < kHeaderBytes / 4) {
    const uint64_t total = kHeaderBytes + (uint64_t)a.l * go.layer_bytes();
    uint32_t w = 0;
    switch (threadIdx.x) {
      case 0: w = kMagic; break;
      case 1: w = 1u | (uint32_t)DT << 16 | (uint32_t)BO << 24; break;
      case 2: w = (uint32_t)a.l; break;
      case 3: w = (uint32_t)n; break;
      case 4: w = (uint32_t)c; break;
      case 5: w = (uint32_t)kGroup | (uint32_t)kGroup << 16; break;
      case 6: w = (uint32_t)total; break;
      case 7: w = (uint32_t)(total >> 32); break;
      case 8: w = hdr.c.x; break;  // token-dropping words are carried over
      case 9: w = hdr.c.y; break;
      case 10: w = hdr.c.z; break;
      default: break;
    }
    gstore<uint32_t>(dst + 4 * threadIdx.x, w);
  }

  if (!is_v) {
    uint32_t om[2] = {0u, 0u};
    const uint32_t meta[2] = {km.x, km.y};
    if constexpr (kUseTable<BI, BO>) {
      uint32_t* ktab = reinterpret_cast<uint32_t*>(kpar);  // [slot][lane], one word per channel
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int lc = (int)threadIdx.x * 2 + e;
        ktab[(lc % kTcLaneCh) * kWave + lc / kTcLaneCh] = code_table<DT, BI, BO>(meta[e], om[e]);
      }
      if (pact) {
        uintx2 o = {om[0], om[1]};
        gstore<uintx2>(out_layer + ((size_t)g * c + pc) * 4, o);
      }
      __syncthreads();
      if (t_first >= n) return;  // wave-uniform, after the barrier
      uint32_t tab[kTcLaneCh];
#pragma unroll
      for (int j = 0; j < kTcLaneCh; ++j) tab[j] = ktab[j * kWave + lane];
#pragma unroll
      for (int i = 0; i < kRowsK; ++i) {  // kRowsK == kTcRows here: the wave's rows are all loaded
        if (t_first + i < n && active)
          lookup_row<BI, BO>(out_codes + (size_t)(t_first + i) * go.row_bytes, cw[i], [&tab](int j) { return tab[j]; });
        __builtin_amdgcn_sched_barrier(0);
      }
      return;
    }
    bool fix = false;
    [[maybe_unused]] uint32_t worst = kStandard;  // 8 -> 2: the least tractable of this thread's channels
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      bool f;
      const TcParams p = tc_params<DT, BI, BO>(meta[e], om[e], f);
      fix |= pact && f;
      const int lc = (int)threadIdx.x * 2 + e;  // channel within the span; its user is lane lc / 16, slot lc % 16
      const int slot = (lc % kTcLaneCh) * kWave + lc / kTcLaneCh;
      kpar[slot] = p;
      if constexpr (BI == 8 && BO == 2) {
        Quad gq;
        const uint32_t cls = classify82<DT>(p, gq);
        if (pact && cls > worst) worst = cls;
        kquad[slot] = gq.a;
        kquad[kTcLaneCh * kWave + slot] = gq.b;
        kquad[2 * kTcLaneCh * kWave + slot] = gq.c;
      }
    }
    if (pact) {
      uintx2 o = {om[0], om[1]};
      gstore<uintx2>(out_layer + ((size_t)g * c + pc) * 4, o);
    }
    bool any_fix;
    if constexpr (BI == 8 && BO == 2) {
      // three block-wide verdicts through one barrier: every wave leaves its own in LDS
      const uint32_t mine = (__builtin_amdgcn_ballot_w64(fix) != 0 ? 1u : 0u) |
                            (__builtin_amdgcn_ballot_w64(worst != kStandard) != 0 ? 2u : 0u) |
                            (__builtin_amdgcn_ballot_w64(worst == kHard) != 0 ? 4u : 0u);
      if (lane == 0) kflags[wave] = mine;
      __syncthreads();
      uint32_t all = 0;
#pragma unroll
      for (int w = 0; w < kTcWaves; ++w) all |= kflags[w];
      all = (uint32_t)__builtin_amdgcn_readfirstlane((int)all);
      any_fix = (all & 1u) != 0;
      if ((all & 4u) == 0) {  // no hard group in the block: the polynomial route
        if (t_first >= n) return;  // wave-uniform, after the barrier
        auto poly_rows = [&](auto standard_tag) {
          constexpr bool STANDARD = decltype(standard_tag)::value;
          Quad gq[kTcLaneCh];
#pragma unroll
          for (int j = 0; j < kTcLaneCh; ++j) {
            gq[j].a = STANDARD ? 0.0f : kquad[j * kWave + lane];
            gq[j].b = STANDARD ? 0.0f : kquad[(kTcLaneCh + j) * kWave + lane];
            gq[j].c = STANDARD ? 0.0f : kquad[(2 * kTcLaneCh + j) * kWave + lane];
          }
#pragma unroll 1
          for (int t0 = t_first;;) {
#pragma unroll
            for (int i = 0; i < kRowsK; ++i) {
              if (t0 + i < n && active)
                poly_row82<STANDARD>(out_codes + (size_t)(t0 + i) * go.row_bytes, cw[i], [&gq](int j) -> const Quad& { return gq[j]; });
              __builtin_amdgcn_sched_barrier(0);
            }
            t0 += kRowsK;
            if (t0 >= t_first + kTcRows || t0 >= n) break;
            load_batch(t0, RowsK{});
          }
        };
        if ((all & 2u) == 0) poly_rows(Yes{}); else poly_rows(No{});
        return;
      }
    } else {
      any_fix = __syncthreads_or(fix);
    }
    if (t_first >= n) return;  // wave-uniform, after the barrier
    // The common path never touches `top`; reading it only where the rule is needed keeps that path's
    // register count down.
    auto k_rows = [&](auto fix_tag) {
      constexpr bool FIX = decltype(fix_tag)::value;
      TcParams p[kTcLaneCh];
#pragma unroll
      for (int j = 0; j < kTcLaneCh; ++j) {
        const TcParams& s = kpar[j * kWave + lane];
        p[j].mn = s.mn;
        p[j].scale = s.scale;
        p[j].inv = s.inv;
        p[j].top = FIX ? s.top : 0.0f;
      }
      auto param_of = [&](int) { return [&p](int j) -> const TcParams& { return p[j]; }; };
#pragma unroll 1
      for (int t0 = t_first;;) {
        run_batch(t0, Zero{}, RowsK{}, fix_tag, param_of);
        t0 += kRowsK;
        if (t0 >= t_first + kTcRows || t0 >= n) break;
        load_batch(t0, RowsK{});
      }
    };
    if (any_fix) k_rows(Yes{}); else k_rows(No{});
  } else {
    if (t_first >= n) return;  // wave-uniform; V waves never meet at a barrier
    const uint8_t* in_vmeta = in_layer + gi.kmeta + gi.codes;
    uint8_t* out_vmeta = out_layer + go.kmeta + go.codes;
    if constexpr (kUseTable<BI, BO>) {
      // the wave's 16 rows are loaded; their groups are prepared 8 rows (= 64 groups, one per lane) at a time
      uint32_t vm[2] = {0u, 0u};
      bool own[2];
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        const int t = t_first + sb * kTcBatch + lane / kTcSpanHeads;
        const int head = span * kTcSpanHeads + lane % kTcSpanHeads;
        own[sb] = t < n && head < heads;
        if (own[sb]) vm[sb] = gload<uint32_t>(in_vmeta + ((size_t)t * heads + head) * 4);
      }
      auto eight_rows = [&](auto sb_tag) {
        constexpr int sb = decltype(sb_tag)::value;
        const int t0 = t_first + sb * kTcBatch;
        uint32_t mine = 0;
        if (own[sb]) {
          const int t = t0 + lane / kTcSpanHeads;
          const int head = span * kTcSpanHeads + lane % kTcSpanHeads;
          uint32_t om;
          mine = code_table<DT, BI, BO>(vm[sb], om);
          gstore<uint32_t>(out_vmeta + ((size_t)t * heads + head) * 4, om);
        }
#pragma unroll
        for (int i = 0; i < kTcBatch; ++i) {
          if (t0 + i < n) {  // wave-uniform; the shuffle is taken with the whole wave enabled
            const uint32_t tab = __shfl(mine, i * kTcSpanHeads + lane / (kGroup / kTcLaneCh));
            if (active)
              lookup_row<BI, BO>(out_codes + (size_t)(t0 + i) * go.row_bytes, cw[sb * kTcBatch + i], [tab](int) { return tab; });
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      eight_rows(std::integral_constant<int, 0>{});
      if (t_first + kTcBatch < n) eight_rows(std::integral_constant<int, 1>{});
    } else {
#pragma unroll 1
      for (int t0 = t_first;;) {  // kRowsV rows from t0 on are loaded
        auto eight_rows = [&](auto first_tag) {
          const int tb = t0 + decltype(first_tag)::value;
          // lane -> the group (row tb + lane / 8, head lane % 8 of this span)
          const int t = tb + lane / kTcSpanHeads;
          const int head = span * kTcSpanHeads + lane % kTcSpanHeads;
          TcParams mine = {0.0f, 0.0f, 0.0f, 0.0f};
          bool fix = false;
          if (t < n && head < heads) {
            const size_t off = ((size_t)t * heads + head) * 4;
            uint32_t om;
            mine = tc_params<DT, BI, BO>(gload<uint32_t>(in_vmeta + off), om, fix);
            gstore<uint32_t>(out_vmeta + off, om);
          }
          const bool any_fix = __builtin_amdgcn_ballot_w64(fix) != 0;
          if constexpr (BI == 8 && BO == 2) {
            Quad gq;
            uint32_t cls = classify82<DT>(mine, gq);
            if (!(t < n && head < heads)) cls = kStandard;  // a lane without a group has no say
            if (__builtin_amdgcn_ballot_w64(cls == kHard) == 0) {
              const bool all_standard = __builtin_amdgcn_ballot_w64(cls != kStandard) == 0;
              constexpr int kFirst = decltype(first_tag)::value;
#pragma unroll
              for (int i = 0; i < kTcBatch; ++i) {
                if (tb + i < n) {  // wave-uniform; the shuffles are taken with the whole wave enabled
                  const int owner = i * kTcSpanHeads + lane / (kGroup / kTcLaneCh);
                  uint8_t* out_row = out_codes + (size_t)(tb + i) * go.row_bytes;
                  if (all_standard) {
                    if (active) poly_row82<true>(out_row, cw[kFirst + i], [&gq](int) -> const Quad& { return gq; });
                  } else {
                    const Quad gr = {__shfl(gq.a, owner), __shfl(gq.b, owner), __shfl(gq.c, owner)};
                    if (active) poly_row82<false>(out_row, cw[kFirst + i], [&gr](int) -> const Quad& { return gr; });
                  }
                }
                __builtin_amdgcn_sched_barrier(0);
              }
              return;
            }
          }
          auto param_of = [&](int i) {
            const int owner = i * kTcSpanHeads + lane / (kGroup / kTcLaneCh);
            TcParams p;
            p.mn = __shfl(mine.mn, owner);
            p.scale = __shfl(mine.scale, owner);
            p.inv = __shfl(mine.inv, owner);
            p.top = __shfl(mine.top, owner);
            return [p](int) -> const TcParams& { return p; };
          };
          if (any_fix) run_batch(tb, first_tag, Batch{}, Yes{}, param_of); else run_batch(tb, first_tag, Batch{}, No{}, param_of);
        };
        eight_rows(Zero{});
        if constexpr (kRowsV > kTcBatch) {
          if (t0 + kTcBatch < n) eight_rows(Eight{});
        }
        t0 += kRowsV;
        if (t0 >= t_first + kTcRows || t0 >= n) break;
        load_batch(t0, RowsV{});
      }
    }
    // zero the padding that rounds the vmeta section up to 16 bytes
    if (span == 0 && threadIdx.x == 0 && (g + 1) * kGroup >= n) {
      for (size_t o = (size_t)n * heads * 4; o < go.vmeta; o += 4) gstore<uint32_t>(out_vmeta + o, 0u);
    }
  }
}

}  // namespace

// grid = (token-groups x spans, 2 * l, items)
template <int DT>
__global__ __launch_bounds__(kTcThreads) KVH_TC_OCC void transcode_kernel(TranscodeParams a) {
  __shared__ TcParams kpar[kTcLaneCh * kWave];  // 16 KiB, [slot][lane]
  __shared__ float kquad[3 * kTcLaneCh * kWave];  // 12 KiB, [coefficient][slot][lane]: the 8 -> 2 polynomials
  __shared__ uint32_t kflags[kTcWaves];
  kvh_tc_item it;
  if (a.items != nullptr) {
    const uint8_t* p = reinterpret_cast<const uint8_t*>(a.items + blockIdx.z);
    uintx4 lo = gload<uintx4>(p), hi = gload<uintx4>(p + 16);
    it.src = reinterpret_cast<const void*>((uint64_t)lo.x | (uint64_t)lo.y << 32);
    it.dst = reinterpret_cast<void*>((uint64_t)lo.z | (uint64_t)lo.w << 32);
    it.n_tokens = (int32_t)hi.x;
    it.level_in = (int32_t)hi.y;
    it.level_out = (int32_t)hi.z;
    it.reserved = 0;
  } else {
    it = a.one;
  }
  it.src = uniform(it.src);
  it.dst = uniform(it.dst);
  it.n_tokens = uniform(it.n_tokens);
  it.level_in = uniform(it.level_in);
  it.level_out = uniform(it.level_out);
  const int nspans = (a.c + kTcSpanCh - 1) / kTcSpanCh;
  const int g = blockIdx.x / nspans;
  const int span = blockIdx.x - g * nspans;
  if (it.n_tokens < 1 || g * kGroup >= it.n_tokens) return;  // block-uniform
  const int lam = blockIdx.y >> 1;
  const bool is_v = blockIdx.y & 1;
  const int bi = level_bits(it.level_in), bo = level_bits(it.level_out);
  // refused: a level out of range, the raw level (no codes to transcode), more tokens than the grid covers
  if (bi < 0 || bo < 0 || bi > 8 || bo > 8 || it.n_tokens > a.max_tokens) {
    if (a.status != nullptr && threadIdx.x == 0) a.status[blockIdx.z] = KVH_DEV_HEADER_MISMATCH;
    return;
  }
#define KVH_TC_CASE(BI, BO) \
  case BI * 16 + BO: transcode_block<DT, BI, BO>(a, it, blockIdx.z, lam, is_v, g, span, kpar, kquad, kflags); break;
  switch (bi * 16 + bo) {
    KVH_TC_CASE(8, 8) KVH_TC_CASE(8, 4) KVH_TC_CASE(8, 2)
    KVH_TC_CASE(4, 8) KVH_TC_CASE(4, 4) KVH_TC_CASE(4, 2)
    KVH_TC_CASE(2, 8) KVH_TC_CASE(2, 4) KVH_TC_CASE(2, 2)
    default: break;
  }
#undef KVH_TC_CASE
}

int launch_transcode(const TranscodeParams& a, int dt, int n_items, int max_tokens, hipStream_t stream) {
  const int nspans = (a.c + kTcSpanCh - 1) / kTcSpanCh;
  const int groups = (max_tokens + kGroup - 1) / kGroup;
  dim3 grid((unsigned)(groups * nspans), (unsigned)(2 * a.l), (unsigned)n_items);
  TranscodeParams b = a;
  b.max_tokens = max_tokens;
  if (dt == KVH_F16)
    launch_kernel(transcode_kernel<KVH_F16>, grid, dim3(kTcThreads), 0u, stream, b);
  else
    launch_kernel(transcode_kernel<KVH_BF16>, grid, dim3(kTcThreads), 0u, stream, b);
  KVH_HIP_CHECK_LAUNCH();
  return KVH_OK;
}

}  // namespace kvh
