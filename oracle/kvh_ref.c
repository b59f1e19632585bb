/*
 * kvh_ref.c — CPU ORACLE of the KV-cache level codec.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, scalar C that states what compressing a KV-cache entry with the quantisation
 * method at a rate, and decompressing it on load, compute (AdaptCache: Introduction — lossy KV
 * compression by quantisation; Design — the executor applies the chosen method/rate, the
 * estimator profiles the decompression overhead; Preliminary Results — the quantiser is the
 * cited per-channel-K / per-token-V min-max quantiser, named rate: two bits).  The paper gives
 * no equations for the codec; every concrete choice below is a stated reading, listed in the
 * design notes of this repository, and pinned by the CPU tests (worked examples, closed
 * forms, invariants, brute force in exact arithmetic, conversions checked exhaustively
 * against independent libraries).
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call this file.
 * It shares no code, header, table or constant generator with the HIP implementation.
 *
 * Definition (one blob = n tokens of l layers x c channels of K and of V, c % 128 == 0,
 * level 0/1/2 -> b = 8/4/2 bits, L = 2^b - 1, T16 = fp16 or bf16):
 *   groups      K: (layer, token-group g = t / 128, channel)  -> up to 128 tokens of one channel
 *               V: (layer, token, channel-group h = ch / 128) -> 128 channels of one token
 *   statistics  mn / mx = numerically smallest / largest element (exact T16 values, -0 -> +0)
 *   parameters  r = f32(mx) - f32(mn);  r < 2^-100: scale = inv = 0 (degenerate group)
 *               else scale = r / L, inv = L / r        (fp32, each operation rounded once)
 *   quantise    q = clamp(nearbyintf((f32(x) - f32(mn)) * inv), 0, L)   (ties to even)
 *   pack        codes of one token row in channel order, LSB-first inside each byte
 *   dequantise  q == L and not degenerate: mx;  else T16_rne(fmaf(f32(q), scale, f32(mn)))
 *               (q == 0 therefore gives mn exactly; a degenerate group gives mn everywhere)
 *   token drop  the second method (keep the beginning and the end of an entry): of N tokens keep the first
 *               `sink` and the last `window`; the kept tokens, in order, are encoded as an ordinary blob of
 *               n = min(N, sink + window) tokens whose header also records (N, sink, window); decoding puts
 *               kept token i back at its original position, or at position i (compact).
 *   blob        64-byte header, then per layer: kmeta | kcodes | vmeta | vcodes, every section
 *               padded to a multiple of 16 bytes.
 *   raw level   level 3 stores an entry in full quality (one of the three choices the policy's greedy step has
 *               for an entry: evict, store in full quality, compress; Design section): b = 16, no groups, no
 *               metadata; per layer the n K rows and then the n V rows, every 16-bit pattern kept as it is
 *               (non-finite values included); header as above with bits = 16.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum { KVH_REF_F16 = 0, KVH_REF_BF16 = 1 };
enum {
  KVH_REF_OK = 0,
  KVH_REF_E_ARG = -1,
  KVH_REF_E_LEVEL = -2,
  KVH_REF_E_SHAPE = -3,
  KVH_REF_E_SIZE = -4,
  KVH_REF_E_ALIGN = -5,
  KVH_REF_E_HEADER = -7,
  KVH_REF_E_NONFINITE = -8
};

#define REF_GROUP 128
#define REF_HEADER_BYTES 64

/* ------------------------------------------------------------------------------------------
 * 16-bit float <-> fp32, written from the formats' definitions.
 * ---------------------------------------------------------------------------------------- */
static float bits_to_float(uint32_t u) {
  float f;
  memcpy(&f, &u, 4);
  return f;
}
static uint32_t float_to_bits(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  return u;
}

float kvh_ref_t16_to_f32(uint16_t h, int dt) {
  if (dt == KVH_REF_BF16) return bits_to_float((uint32_t)h << 16); /* top half of an fp32 */
  /* binary16: 1 sign, 5 exponent (bias 15), 10 fraction */
  int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
  float mag;
  if (e == 0)
    mag = ldexpf((float)m, -24); /* zero and subnormals: m * 2^-24 */
  else if (e == 31)
    mag = m ? NAN : INFINITY;
  else
    mag = ldexpf((float)(m | 1024), e - 25); /* (1 + m/1024) * 2^(e-15) */
  return sign ? -mag : mag;
}

uint16_t kvh_ref_f32_to_t16(float f, int dt) {
  uint32_t u = float_to_bits(f);
  uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
  uint32_t a = u & 0x7fffffffu; /* |f| as bits */
  if (dt == KVH_REF_BF16) {
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7fc0u);           /* NaN */
    uint32_t keep = u >> 16, rest = u & 0xffffu;                        /* round the low 16 bits */
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1; /* nearest, ties to even */
    return (uint16_t)keep;                                              /* carry may reach inf */
  }
  if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u); /* NaN */
  float mag = bits_to_float(a);
  if (mag >= 65520.0f) return (uint16_t)(sign | 0x7c00u); /* >= max + half ulp -> inf */
  if (mag < 0x1p-14f) {
    /* below the smallest normal: the fp16 grid is the integers times 2^-24 */
    float scaled = ldexpf(mag, 24);                  /* exact */
    uint16_t m = (uint16_t)nearbyintf(scaled);       /* ties to even; 1024 is the first normal */
    return (uint16_t)(sign | m);
  }
  uint32_t e = (a >> 23) - 127 + 15;  /* 1..30 */
  uint32_t frac = a & 0x7fffffu;      /* 23 fraction bits; keep 10, round 13 */
  uint32_t h = (e << 10) | (frac >> 13);
  uint32_t rest = frac & 0x1fffu;
  if (rest > 0x1000u || (rest == 0x1000u && (h & 1u))) h += 1; /* carry into the exponent is right */
  return (uint16_t)(sign | h);
}

/* ------------------------------------------------------------------------------------------
 * Level table and blob geometry.
 * ---------------------------------------------------------------------------------------- */
int kvh_ref_num_levels(void) { return 3; } /* the quantised levels 0..2; level 3 is the raw one */

int kvh_ref_level_bits(int level) {
  switch (level) {
    case 0: return 8;
    case 1: return 4;
    case 2: return 2;
    case 3: return 16; /* full quality: rows stored as they are */
    default: return -1;
  }
}

static size_t pad16(size_t x) { return (x + 15u) & ~(size_t)15u; }

static int shape_ok(int l, int n, int c) { return l >= 1 && n >= 1 && c >= REF_GROUP && c % REF_GROUP == 0; }

/* section sizes of one layer */
static size_t kmeta_bytes_q(int n, int c) { return pad16((size_t)((n + REF_GROUP - 1) / REF_GROUP) * (size_t)c * 4u); }
static size_t codes_bytes(int n, int c, int bits) { return pad16((size_t)n * ((size_t)c * (size_t)bits / 8u)); }
static size_t vmeta_bytes_q(int n, int c) { return pad16((size_t)n * (size_t)(c / REF_GROUP) * 4u); }
/* the raw level has no groups and therefore no metadata sections */
#define kmeta_bytes(n, c) (bits == 16 ? (size_t)0 : kmeta_bytes_q(n, c))
#define vmeta_bytes(n, c) (bits == 16 ? (size_t)0 : vmeta_bytes_q(n, c))

size_t kvh_ref_blob_size(int l, int n, int c, int level) {
  int bits = kvh_ref_level_bits(level);
  if (bits < 0 || !shape_ok(l, n, c)) return 0;
  size_t per_layer = kmeta_bytes(n, c) + vmeta_bytes(n, c) + 2 * codes_bytes(n, c, bits);
  return REF_HEADER_BYTES + (size_t)l * per_layer;
}

static void put_u16(uint8_t* p, uint16_t v) { p[0] = (uint8_t)(v & 0xff); p[1] = (uint8_t)(v >> 8); }
static void put_u32(uint8_t* p, uint32_t v) { for (int i = 0; i < 4; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
static void put_u64(uint8_t* p, uint64_t v) { for (int i = 0; i < 8; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
static uint16_t get_u16(const uint8_t* p) { return (uint16_t)(p[0] | (p[1] << 8)); }
static uint32_t get_u32(const uint8_t* p) { uint32_t v = 0; for (int i = 0; i < 4; ++i) v |= (uint32_t)p[i] << (8 * i); return v; }
static uint64_t get_u64(const uint8_t* p) { uint64_t v = 0; for (int i = 0; i < 8; ++i) v |= (uint64_t)p[i] << (8 * i); return v; }

static void write_header(uint8_t* blob, int dt, int bits, int l, int n, int c, uint64_t total, uint32_t orig_tokens,
                         uint32_t sink, uint32_t window) {
  memset(blob, 0, REF_HEADER_BYTES);
  blob[0] = 'K'; blob[1] = 'V'; blob[2] = 'H'; blob[3] = '1';
  put_u16(blob + 4, 1);               /* version */
  blob[6] = (uint8_t)dt;
  blob[7] = (uint8_t)bits;
  put_u32(blob + 8, (uint32_t)l);
  put_u32(blob + 12, (uint32_t)n);
  put_u32(blob + 16, (uint32_t)c);
  put_u16(blob + 20, REF_GROUP);      /* K group: tokens   */
  put_u16(blob + 22, REF_GROUP);      /* V group: channels */
  put_u64(blob + 24, total);
  put_u32(blob + 32, orig_tokens); /* 0: not a token-dropped entry */
  put_u32(blob + 36, sink);
  put_u32(blob + 40, window);
}

static int header_matches(const uint8_t* blob, int dt, int bits, int l, int n, int c, uint64_t total, uint32_t orig_tokens,
                          uint32_t sink, uint32_t window) {
  return blob[0] == 'K' && blob[1] == 'V' && blob[2] == 'H' && blob[3] == '1' && get_u16(blob + 4) == 1 &&
         blob[6] == dt && blob[7] == bits && get_u32(blob + 8) == (uint32_t)l && get_u32(blob + 12) == (uint32_t)n &&
         get_u32(blob + 16) == (uint32_t)c && get_u16(blob + 20) == REF_GROUP && get_u16(blob + 22) == REF_GROUP &&
         get_u64(blob + 24) == total && get_u32(blob + 32) == orig_tokens && get_u32(blob + 36) == sink &&
         get_u32(blob + 40) == window;
}

/* ------------------------------------------------------------------------------------------
 * The scalar steps: statistics, parameters, quantise, dequantise.
 * ---------------------------------------------------------------------------------------- */
static uint16_t canonical_zero(uint16_t bits) { return bits == 0x8000u ? 0 : bits; }

/* min and max of `count` elements spaced `stride` apart; returns nonzero if one is not finite */
static int group_minmax(const uint16_t* x, int64_t stride, int count, int dt, uint16_t* mn_bits, uint16_t* mx_bits) {
  uint16_t lo = x[0], hi = x[0];
  float flo = kvh_ref_t16_to_f32(lo, dt), fhi = flo;
  int bad = !isfinite(flo);
  for (int i = 1; i < count; ++i) {
    uint16_t b = x[(int64_t)i * stride];
    float f = kvh_ref_t16_to_f32(b, dt);
    if (!isfinite(f)) bad = 1;
    if (f < flo) { flo = f; lo = b; }
    if (f > fhi) { fhi = f; hi = b; }
  }
  *mn_bits = canonical_zero(lo);
  *mx_bits = canonical_zero(hi);
  return bad;
}

/* scale and inv of a group from its stored (min, max); returns 1 if the group is degenerate */
int kvh_ref_group_params(uint16_t mn_bits, uint16_t mx_bits, int dt, int bits, float* scale, float* inv) {
  float L = (float)((1 << bits) - 1);
  float r = kvh_ref_t16_to_f32(mx_bits, dt) - kvh_ref_t16_to_f32(mn_bits, dt);
  if (r < 0x1p-100f) {
    *scale = 0.0f;
    *inv = 0.0f;
    return 1;
  }
  *scale = r / L;
  *inv = L / r;
  return 0;
}

int kvh_ref_quantise(uint16_t x_bits, uint16_t mn_bits, float inv, int dt, int bits) {
  int L = (1 << bits) - 1;
  float d = kvh_ref_t16_to_f32(x_bits, dt) - kvh_ref_t16_to_f32(mn_bits, dt);
  float t = d * inv;
  float rt = nearbyintf(t); /* default rounding mode: to nearest, ties to even */
  if (!(rt > 0.0f)) return 0; /* also catches NaN so the cast below is always defined */
  if (rt >= (float)L) return L;
  return (int)rt;
}

uint16_t kvh_ref_dequantise(int q, uint16_t mn_bits, uint16_t mx_bits, int dt, int bits) {
  int L = (1 << bits) - 1;
  float scale, inv;
  int degenerate = kvh_ref_group_params(mn_bits, mx_bits, dt, bits, &scale, &inv);
  if (q == L && !degenerate) return mx_bits;
  float y = fmaf((float)q, scale, kvh_ref_t16_to_f32(mn_bits, dt));
  return kvh_ref_f32_to_t16(y, dt);
}

/* ------------------------------------------------------------------------------------------
 * Encode one blob.
 * k, v: host pointers to T16 [l][n][c] views with the given element strides (channel stride 1).
 * ---------------------------------------------------------------------------------------- */
int kvh_ref_encode(const uint16_t* k, const uint16_t* v, int64_t layer_stride, int64_t token_stride, int dt, int l,
                   int n, int c, int level, uint8_t* blob, size_t blob_cap) {
  if (!k || !v || !blob || (dt != KVH_REF_F16 && dt != KVH_REF_BF16)) return KVH_REF_E_ARG;
  int bits = kvh_ref_level_bits(level);
  if (bits < 0) return KVH_REF_E_LEVEL;
  if (!shape_ok(l, n, c)) return KVH_REF_E_SHAPE;
  size_t total = kvh_ref_blob_size(l, n, c, level);
  if (blob_cap < total) return KVH_REF_E_SIZE;

  const int per_byte = bits == 16 ? 1 : 8 / bits;
  const size_t row_bytes = (size_t)c * (size_t)bits / 8u;
  const int n_groups = (n + REF_GROUP - 1) / REF_GROUP;
  int nonfinite = 0;

  memset(blob, 0, total); /* padding bytes are zero */
  write_header(blob, dt, bits, l, n, c, (uint64_t)total, 0, 0, 0);
  uint8_t* p = blob + REF_HEADER_BYTES;

  for (int lam = 0; lam < l; ++lam) {
    const uint16_t* K = k + (int64_t)lam * layer_stride;
    const uint16_t* V = v + (int64_t)lam * layer_stride;
    uint8_t* kmeta = p;
    uint8_t* kcodes = kmeta + kmeta_bytes(n, c);
    uint8_t* vmeta = kcodes + codes_bytes(n, c, bits);
    uint8_t* vcodes = vmeta + vmeta_bytes(n, c);
    p = vcodes + codes_bytes(n, c, bits);

    if (bits == 16) { /* full quality: the rows as they are, K then V */
      for (int t = 0; t < n; ++t)
        for (int ch = 0; ch < c; ++ch) {
          put_u16(kcodes + ((size_t)t * c + ch) * 2, K[(int64_t)t * token_stride + ch]);
          put_u16(vcodes + ((size_t)t * c + ch) * 2, V[(int64_t)t * token_stride + ch]);
        }
      continue;
    }

    /* K: one group per (token-group, channel), statistics over tokens */
    for (int g = 0; g < n_groups; ++g) {
      int t0 = g * REF_GROUP;
      int cnt = n - t0 < REF_GROUP ? n - t0 : REF_GROUP;
      for (int ch = 0; ch < c; ++ch) {
        uint16_t mn, mx;
        float scale, inv;
        nonfinite |= group_minmax(K + (int64_t)t0 * token_stride + ch, token_stride, cnt, dt, &mn, &mx);
        put_u16(kmeta + ((size_t)g * c + ch) * 4, mn);
        put_u16(kmeta + ((size_t)g * c + ch) * 4 + 2, mx);
        kvh_ref_group_params(mn, mx, dt, bits, &scale, &inv);
        for (int i = 0; i < cnt; ++i) {
          int t = t0 + i;
          int q = kvh_ref_quantise(K[(int64_t)t * token_stride + ch], mn, inv, dt, bits);
          kcodes[(size_t)t * row_bytes + ch / per_byte] |= (uint8_t)(q << ((ch % per_byte) * bits));
        }
      }
    }
    /* V: one group per (token, 128-channel group), statistics over channels */
    for (int t = 0; t < n; ++t) {
      for (int h = 0; h < c / REF_GROUP; ++h) {
        uint16_t mn, mx;
        float scale, inv;
        const uint16_t* row = V + (int64_t)t * token_stride + h * REF_GROUP;
        nonfinite |= group_minmax(row, 1, REF_GROUP, dt, &mn, &mx);
        put_u16(vmeta + ((size_t)t * (c / REF_GROUP) + h) * 4, mn);
        put_u16(vmeta + ((size_t)t * (c / REF_GROUP) + h) * 4 + 2, mx);
        kvh_ref_group_params(mn, mx, dt, bits, &scale, &inv);
        for (int i = 0; i < REF_GROUP; ++i) {
          int ch = h * REF_GROUP + i;
          int q = kvh_ref_quantise(row[i], mn, inv, dt, bits);
          vcodes[(size_t)t * row_bytes + ch / per_byte] |= (uint8_t)(q << ((ch % per_byte) * bits));
        }
      }
    }
  }
  return nonfinite ? KVH_REF_E_NONFINITE : KVH_REF_OK;
}

/* ------------------------------------------------------------------------------------------
 * Decode one blob into a contiguous or paged destination.
 * kdst, vdst: host pointers to T16 [l][tokens][c] (contiguous) or [l][P][block_tokens][c] (paged)
 * with the given element strides.  Token t of the blob goes to logical position dst_token0 + t;
 * with a page table, logical position s lives in physical block page_table[s / block_tokens],
 * slot s % block_tokens.
 * ---------------------------------------------------------------------------------------- */
static int code_at(const uint8_t* row, int ch, int bits) {
  int per_byte = 8 / bits;
  return (row[ch / per_byte] >> ((ch % per_byte) * bits)) & ((1 << bits) - 1);
}

int kvh_ref_decode(const uint8_t* blob, size_t blob_len, int dt, int l, int n, int c, int level, uint16_t* kdst,
                   uint16_t* vdst, int64_t layer_stride, int64_t token_stride, int64_t dst_token0,
                   const int32_t* page_table, int block_tokens) {
  if (!blob || !kdst || !vdst || (dt != KVH_REF_F16 && dt != KVH_REF_BF16) || dst_token0 < 0) return KVH_REF_E_ARG;
  int bits = kvh_ref_level_bits(level);
  if (bits < 0) return KVH_REF_E_LEVEL;
  if (!shape_ok(l, n, c)) return KVH_REF_E_SHAPE;
  if (page_table && block_tokens < 1) return KVH_REF_E_ARG;
  size_t total = kvh_ref_blob_size(l, n, c, level);
  if (blob_len < total) return KVH_REF_E_SIZE;
  if (!header_matches(blob, dt, bits, l, n, c, (uint64_t)total, 0, 0, 0)) return KVH_REF_E_HEADER;

  const size_t row_bytes = (size_t)c * (size_t)bits / 8u;
  const uint8_t* p = blob + REF_HEADER_BYTES;
  for (int lam = 0; lam < l; ++lam) {
    const uint8_t* kmeta = p;
    const uint8_t* kcodes = kmeta + kmeta_bytes(n, c);
    const uint8_t* vmeta = kcodes + codes_bytes(n, c, bits);
    const uint8_t* vcodes = vmeta + vmeta_bytes(n, c);
    p = vcodes + codes_bytes(n, c, bits);
    for (int t = 0; t < n; ++t) {
      int64_t s = dst_token0 + t;
      int64_t row = page_table ? (int64_t)page_table[s / block_tokens] * block_tokens + s % block_tokens : s;
      uint16_t* krow = kdst + (int64_t)lam * layer_stride + row * token_stride;
      uint16_t* vrow = vdst + (int64_t)lam * layer_stride + row * token_stride;
      if (bits == 16) { /* full quality: the stored rows as they are */
        for (int ch = 0; ch < c; ++ch) {
          krow[ch] = get_u16(kcodes + ((size_t)t * c + ch) * 2);
          vrow[ch] = get_u16(vcodes + ((size_t)t * c + ch) * 2);
        }
        continue;
      }
      for (int ch = 0; ch < c; ++ch) {
        const uint8_t* km = kmeta + ((size_t)(t / REF_GROUP) * c + ch) * 4;
        const uint8_t* vm = vmeta + ((size_t)t * (c / REF_GROUP) + ch / REF_GROUP) * 4;
        krow[ch] = kvh_ref_dequantise(code_at(kcodes + (size_t)t * row_bytes, ch, bits), get_u16(km), get_u16(km + 2), dt, bits);
        vrow[ch] = kvh_ref_dequantise(code_at(vcodes + (size_t)t * row_bytes, ch, bits), get_u16(vm), get_u16(vm + 2), dt, bits);
      }
    }
  }
  return KVH_REF_OK;
}

/* Section offsets of layer `lam` inside a blob (for tests that inspect metadata and codes):
 * out[0..3] = byte offsets of kmeta, kcodes, vmeta, vcodes; out[4] = bytes of one packed row. */
int kvh_ref_section_offsets(int l, int n, int c, int level, int lam, uint64_t out[5]) {
  int bits = kvh_ref_level_bits(level);
  if (bits < 0) return KVH_REF_E_LEVEL;
  if (!shape_ok(l, n, c) || lam < 0 || lam >= l) return KVH_REF_E_SHAPE;
  size_t per_layer = kmeta_bytes(n, c) + vmeta_bytes(n, c) + 2 * codes_bytes(n, c, bits);
  size_t base = REF_HEADER_BYTES + (size_t)lam * per_layer;
  out[0] = base;
  out[1] = out[0] + kmeta_bytes(n, c);
  out[2] = out[1] + codes_bytes(n, c, bits);
  out[3] = out[2] + vmeta_bytes(n, c);
  out[4] = (uint64_t)c * (uint64_t)bits / 8u;
  return KVH_REF_OK;
}

/* Array forms of the two conversions (the exhaustive conversion tests call these). */
void kvh_ref_t16_to_f32_array(const uint16_t* in, float* out, size_t count, int dt) {
  for (size_t i = 0; i < count; ++i) out[i] = kvh_ref_t16_to_f32(in[i], dt);
}
void kvh_ref_f32_to_t16_array(const float* in, uint16_t* out, size_t count, int dt) {
  for (size_t i = 0; i < count; ++i) out[i] = kvh_ref_f32_to_t16(in[i], dt);
}

/* ------------------------------------------------------------------------------------------
 * Token dropping (the paper's second compression method: the Introduction motivates it with
 * contexts whose middle matters little compared with their start and their end; Preliminary
 * Results use it as the fixed-rate token-dropping baseline).  The paper gives no definition; the reading taken: keep the first `sink` and the
 * last `window` tokens of an entry of N tokens, drop the middle, and store the kept tokens at a
 * quantised level.  Written as the plain composition gather -> encode and decode -> scatter.
 * ---------------------------------------------------------------------------------------- */
#include <stdlib.h>

int kvh_ref_kept_tokens(int N, int sink, int window) {
  if (N < 1 || sink < 0 || window < 0 || sink + window < 1) return 0;
  return sink + window >= N ? N : sink + window;
}

/* original position of kept token i */
static int64_t kept_position(int i, int N, int sink, int window) {
  if (sink + window >= N) return i;
  return i < sink ? i : (int64_t)N - window + (i - sink);
}

int kvh_ref_encode_kept(const uint16_t* k, const uint16_t* v, int64_t layer_stride, int64_t token_stride, int dt, int l,
                        int N, int c, int sink, int window, int level, uint8_t* blob, size_t blob_cap) {
  if (!k || !v || !blob) return KVH_REF_E_ARG;
  int n = kvh_ref_kept_tokens(N, sink, window);
  if (n < 1) return KVH_REF_E_SHAPE;
  if (!shape_ok(l, n, c)) return KVH_REF_E_SHAPE;
  /* gather the kept rows into a dense [l][n][c] copy, then encode that */
  uint16_t* gk = (uint16_t*)malloc((size_t)l * n * c * 2);
  uint16_t* gv = (uint16_t*)malloc((size_t)l * n * c * 2);
  if (!gk || !gv) { free(gk); free(gv); return KVH_REF_E_SIZE; }
  for (int lam = 0; lam < l; ++lam)
    for (int i = 0; i < n; ++i) {
      int64_t t = kept_position(i, N, sink, window);
      memcpy(gk + ((size_t)lam * n + i) * c, k + lam * layer_stride + t * token_stride, (size_t)c * 2);
      memcpy(gv + ((size_t)lam * n + i) * c, v + lam * layer_stride + t * token_stride, (size_t)c * 2);
    }
  int rc = kvh_ref_encode(gk, gv, (int64_t)n * c, c, dt, l, n, c, level, blob, blob_cap);
  free(gk);
  free(gv);
  if (rc == KVH_REF_OK || rc == KVH_REF_E_NONFINITE) {
    put_u32(blob + 32, (uint32_t)N);
    put_u32(blob + 36, (uint32_t)sink);
    put_u32(blob + 40, (uint32_t)window);
  }
  return rc;
}

/* compact != 0: kept token i goes to logical position dst_token0 + i; else to dst_token0 + its
 * original position (rows of dropped tokens are left untouched). */
int kvh_ref_decode_kept(const uint8_t* blob, size_t blob_len, int dt, int l, int N, int c, int sink, int window, int level,
                        uint16_t* kdst, uint16_t* vdst, int64_t layer_stride, int64_t token_stride, int64_t dst_token0,
                        int compact, const int32_t* page_table, int block_tokens) {
  if (!blob || !kdst || !vdst || dst_token0 < 0) return KVH_REF_E_ARG;
  int bits = kvh_ref_level_bits(level);
  if (bits < 0) return KVH_REF_E_LEVEL;
  int n = kvh_ref_kept_tokens(N, sink, window);
  if (n < 1 || !shape_ok(l, n, c)) return KVH_REF_E_SHAPE;
  if (page_table && block_tokens < 1) return KVH_REF_E_ARG;
  size_t total = kvh_ref_blob_size(l, n, c, level);
  if (blob_len < total) return KVH_REF_E_SIZE;
  if (!header_matches(blob, dt, bits, l, n, c, (uint64_t)total, (uint32_t)N, (uint32_t)sink, (uint32_t)window))
    return KVH_REF_E_HEADER;
  /* decode into a dense temporary with the ordinary decoder (on a copy whose drop words are cleared), then scatter */
  uint8_t* plain = (uint8_t*)malloc(total);
  uint16_t* dk = (uint16_t*)malloc((size_t)l * n * c * 2);
  uint16_t* dv = (uint16_t*)malloc((size_t)l * n * c * 2);
  if (!plain || !dk || !dv) { free(plain); free(dk); free(dv); return KVH_REF_E_SIZE; }
  memcpy(plain, blob, total);
  memset(plain + 32, 0, 12);
  int rc = kvh_ref_decode(plain, total, dt, l, n, c, level, dk, dv, (int64_t)n * c, c, 0, NULL, 0);
  if (rc == KVH_REF_OK) {
    for (int lam = 0; lam < l; ++lam)
      for (int i = 0; i < n; ++i) {
        int64_t s = dst_token0 + (compact ? i : kept_position(i, N, sink, window));
        int64_t row = page_table ? (int64_t)page_table[s / block_tokens] * block_tokens + s % block_tokens : s;
        memcpy(kdst + lam * layer_stride + row * token_stride, dk + ((size_t)lam * n + i) * c, (size_t)c * 2);
        memcpy(vdst + lam * layer_stride + row * token_stride, dv + ((size_t)lam * n + i) * c, (size_t)c * 2);
      }
  }
  free(plain);
  free(dk);
  free(dv);
  return rc;
}

/* ------------------------------------------------------------------------------------------
 * Transcode: re-compress a stored entry from the level it is held at to another level (the
 * greedy step of the policy compresses an entry further, from rate m to rate n; Design section,
 * marginal utility drop).  Defined as nothing more than decode followed by encode; the
 * token-dropping words of the header are carried over unchanged.
 * ---------------------------------------------------------------------------------------- */
int kvh_ref_transcode(const uint8_t* blob_in, size_t len_in, int dt, int l, int n, int c, int level_in, int level_out,
                      uint8_t* blob_out, size_t cap_out) {
  if (!blob_in || !blob_out) return KVH_REF_E_ARG;
  int bits_in = kvh_ref_level_bits(level_in);
  if (bits_in < 0 || kvh_ref_level_bits(level_out) < 0) return KVH_REF_E_LEVEL;
  if (!shape_ok(l, n, c)) return KVH_REF_E_SHAPE;
  size_t total_in = kvh_ref_blob_size(l, n, c, level_in);
  size_t total_out = kvh_ref_blob_size(l, n, c, level_out);
  if (len_in < total_in || cap_out < total_out) return KVH_REF_E_SIZE;
  uint32_t orig = get_u32(blob_in + 32), sink = get_u32(blob_in + 36), window = get_u32(blob_in + 40);
  if (!header_matches(blob_in, dt, bits_in, l, n, c, (uint64_t)total_in, orig, sink, window)) return KVH_REF_E_HEADER;
  if ((orig | sink | window) != 0 &&
      (orig > 0x7fffffffu || sink > 0x7fffffffu || window > 0x7fffffffu || (uint64_t)sink + window > 0x7fffffffu ||
       kvh_ref_kept_tokens((int)orig, (int)sink, (int)window) != n))
    return KVH_REF_E_HEADER;
  uint8_t* plain = (uint8_t*)malloc(total_in);
  uint16_t* dk = (uint16_t*)malloc((size_t)l * n * c * 2);
  uint16_t* dv = (uint16_t*)malloc((size_t)l * n * c * 2);
  if (!plain || !dk || !dv) { free(plain); free(dk); free(dv); return KVH_REF_E_SIZE; }
  memcpy(plain, blob_in, total_in);
  memset(plain + 32, 0, 12);
  int rc = kvh_ref_decode(plain, total_in, dt, l, n, c, level_in, dk, dv, (int64_t)n * c, c, 0, NULL, 0);
  if (rc == KVH_REF_OK) rc = kvh_ref_encode(dk, dv, (int64_t)n * c, c, dt, l, n, c, level_out, blob_out, cap_out);
  if (rc == KVH_REF_OK) {
    put_u32(blob_out + 32, orig);
    put_u32(blob_out + 36, sink);
    put_u32(blob_out + 40, window);
  }
  free(plain);
  free(dk);
  free(dv);
  return rc;
}
