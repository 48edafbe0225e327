// Device-side pieces of the 3-axis rotary embedding shared by every kernel that rotates K or Q and
// has to produce the same bits: token geometry, cos/sin of a pair at a position, the rotation of
// eight elements, bf16 packing, and the per-page cos/sin table of the paged K write.
// (Convention: cascade_attn.h.  Included inside namespace ca { namespace { ... } }.)
#pragma once

struct alignas(16) U4 { uint32_t x, y, z, w; };

// Tensors that pass through once (the unrotated inputs, the rotated output) are read and written
// with the non-temporal hint, so that they do not displace the pool pages the attention kernel
// re-reads from the caches.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_nt;
__device__ __forceinline__ U4 load_once(const void* p) {
  const u32x4_nt t = __builtin_nontemporal_load(static_cast<const u32x4_nt*>(p));
  return U4{t[0], t[1], t[2], t[3]};
}
__device__ __forceinline__ void store_once(void* p, const U4& a) {
  const u32x4_nt t = {a.x, a.y, a.z, a.w};
  __builtin_nontemporal_store(t, static_cast<u32x4_nt*>(p));
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// two fp32 -> one dword of bf16 bits, round to nearest even (v_cvt_pk_bf16_f32)
typedef __attribute__((ext_vector_type(2))) float rd_f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 rd_bf16x2;
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const rd_f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, rd_bf16x2));
}

struct TokenPos { int f, y, x; };

__device__ __forceinline__ TokenPos token_pos(int64_t n, int64_t first_frame, int gh, int gw) {
  const int plane = gh * gw;
  TokenPos p;
  p.f = int(first_frame + n / plane);
  const int r = int(n % plane);
  p.y = r / gw;
  p.x = r % gw;
  return p;
}

// cos/sin of pair `pair` at a token position.  The angle pos * freq is formed and reduced to
// [-pi, pi] in fp64 (exact to ~1e-15 for any position).  FP64_TRIG evaluates sin/cos in fp64 (fp32
// storage: results correctly rounded to fp32); otherwise in fp32 on the reduced angle, whose error
// (~1e-7) is far below the bf16 rounding (4e-3) of what it multiplies, at a fraction of the cost.
template <bool FP64_TRIG>
__device__ __forceinline__ void pair_cs(const RopeGeom& g, const TokenPos& p, int pair, float* c, float* s) {
  const int pos = pair < g.pairs_t ? p.f : (pair < g.pairs_t + g.pairs_h ? p.y : p.x);
  const double ang = double(pos) * g.freq[pair];
  if (FP64_TRIG) {
    double sd, cd;
    sincos(ang, &sd, &cd);
    *c = float(cd);
    *s = float(sd);
  } else {
    const double turns = rint(ang * 0.15915494309189535);                 // nearest multiple of 2 pi
    const float r = float(fma(turns, -6.283185307179586, ang));
    sincosf(r, s, c);
  }
}

template <typename T> struct Vec8;
template <> struct Vec8<float> {
  float v[8];
  __device__ void load(const float* p) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  __device__ void store(float* p) const {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
  }
};
template <> struct Vec8<uint16_t> {
  float v[8];
  __device__ void load(const uint16_t* p) {
    const U4 a = load_once(p);
    v[0] = bf16_lo(a.x); v[1] = bf16_hi(a.x); v[2] = bf16_lo(a.y); v[3] = bf16_hi(a.y);
    v[4] = bf16_lo(a.z); v[5] = bf16_hi(a.z); v[6] = bf16_lo(a.w); v[7] = bf16_hi(a.w);
  }
  __device__ void store(uint16_t* p) const {
    U4 a;
    a.x = pack_bf16(v[0], v[1]); a.y = pack_bf16(v[2], v[3]);
    a.z = pack_bf16(v[4], v[5]); a.w = pack_bf16(v[6], v[7]);
    store_once(p, a);
  }
};

template <typename T>
__device__ __forceinline__ void rotate8(Vec8<T>& x, const float* c, const float* s) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float u = x.v[2 * j], w = x.v[2 * j + 1];
    x.v[2 * j] = fmaf(u, c[j], -(w * s[j]));
    x.v[2 * j + 1] = fmaf(u, s[j], w * c[j]);
  }
}

// cos/sin are shared by every head of a token and, per axis, by every token with the same frame,
// row or column: a workgroup tabulates them once per axis value present in a 128-token page (for
// a 30 x 52 grid: 2 frames x 22 pairs + 4 rows x 21 + 52 columns x 21 = 1220 evaluations instead
// of 128 tokens x 64 pairs = 8192) and its threads pick theirs from LDS.
// the token `step` tokens after p (step >= 0), without the divisions of token_pos
__device__ __forceinline__ TokenPos token_advance(TokenPos p, int step, int gh, int gw) {
  p.x += step;
  while (p.x >= gw) {
    p.x -= gw;
    ++p.y;
  }
  while (p.y >= gh) {
    p.y -= gh;
    ++p.f;
  }
  return p;
}

struct TrigTable {
  int32_t n_f, n_y, n_x;       // axis values tabulated: consecutive frames / rows (mod grid_h) / columns (mod grid_w)
};

struct TrigLayout {            // where the three axes start in the table, and the page's first token
  int off_y, off_x, total, pairs_w;
  TokenPos first;
};

__device__ __forceinline__ TrigLayout trig_layout(const RopeGeom& g, const TrigTable& tab, int tok0, int block_tokens,
                                                  int64_t first_frame) {
  TrigLayout l;
  l.pairs_w = g.head_dim / 2 - g.pairs_t - g.pairs_h;
  l.first = token_pos(min(tok0, block_tokens - 1), first_frame, g.grid_h, g.grid_w);
  l.off_y = tab.n_f * g.pairs_t;
  l.off_x = l.off_y + tab.n_y * g.pairs_h;
  l.total = l.off_x + tab.n_x * l.pairs_w;
  return l;
}

// entries t, t + stride, ... of the table of the page that starts at the layout's first token
__device__ __forceinline__ void trig_fill(const RopeGeom& g, const TrigLayout& l, float2* trig, int t, int stride) {
  for (int e = t; e < l.total; e += stride) {
    TokenPos p = l.first;
    int pair;
    if (e < l.off_y) {
      p.f = l.first.f + e / g.pairs_t;
      pair = e % g.pairs_t;
    } else if (e < l.off_x) {
      p.y = (l.first.y + (e - l.off_y) / g.pairs_h) % g.grid_h;
      pair = g.pairs_t + (e - l.off_y) % g.pairs_h;
    } else {
      p.x = (l.first.x + (e - l.off_x) / l.pairs_w) % g.grid_w;
      pair = g.pairs_t + g.pairs_h + (e - l.off_x) % l.pairs_w;
    }
    float cv, sv;
    pair_cs<false>(g, p, pair, &cv, &sv);
    trig[e] = make_float2(cv, sv);
  }
}

// cos/sin of pairs 4c .. 4c+3 at token p, from the table
__device__ __forceinline__ void trig_pick(const RopeGeom& g, const TrigLayout& l, const float2* trig, const TokenPos& p,
                                          int c, float* cs, float* sn) {
  const int rf = p.f - l.first.f;
  int ry = p.y - l.first.y, rx = p.x - l.first.x;         // both in (-grid, grid): one conditional add wraps them
  ry += ry < 0 ? g.grid_h : 0;
  rx += rx < 0 ? g.grid_w : 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int pair = c * 4 + j;
    const int e = pair < g.pairs_t ? rf * g.pairs_t + pair
                  : (pair < g.pairs_t + g.pairs_h ? l.off_y + ry * g.pairs_h + (pair - g.pairs_t)
                                                  : l.off_x + rx * l.pairs_w + (pair - g.pairs_t - g.pairs_h));
    const float2 v = trig[e];
    cs[j] = v.x;
    sn[j] = v.y;
  }
}

// Host side: which axis values a 128-token page can touch (consecutive tokens, so consecutive
// columns -- all of them once the page is longer than a row --, rows and frames), and the bytes of
// the table; n_f = 0 and 0 bytes if that exceeds max_bytes (then threads evaluate their own).
inline TrigTable trig_table_for(const RopeGeom& g, int page_tokens, size_t max_bytes, size_t* bytes) {
  const int plane = g.grid_h * g.grid_w;
  TrigTable tab;
  tab.n_x = g.grid_w < page_tokens ? g.grid_w : page_tokens;
  tab.n_y = page_tokens / g.grid_w + 2 < g.grid_h ? page_tokens / g.grid_w + 2 : g.grid_h;
  tab.n_f = page_tokens / plane + 2;
  const int pairs_w = g.head_dim / 2 - g.pairs_t - g.pairs_h;
  *bytes = sizeof(float2) * (size_t(tab.n_f) * g.pairs_t + size_t(tab.n_y) * g.pairs_h + size_t(tab.n_x) * pairs_w);
  if (*bytes > max_bytes) {
    tab.n_f = 0;
    *bytes = 0;
  }
  return tab;
}
