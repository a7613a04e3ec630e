// oscar_quantize_append: Canalized Rotation -> Omni-Token Scaling -> per-channel key
// quantization + per-token value quantization -> bit-packed page write, plus the
// 16-bit residual window (BufferQuantK / BufferQuantV of Algorithm "The OScaR
// algorithm"; key transform of App. "Implementation Details ...", "Overall Design";
// quantizer of Eq. 3-4).
//
// Every translation unit that includes this header is compiled with -ffp-contract=off:
// the encoder is an encoding, and its fp32 operation order is part of the format (codes
// must not depend on whether a multiply-add was fused).
//
// Work decomposition: one workgroup of 256 threads per (sequence, kv head, block of
// R=128 pending tokens).  A thread owns 8 channels (channel group cg) of token
// 16*pass+slot for pass = 0..7; the 16 lanes of a DPP row share a token, so
//   - the 128-point Hadamard butterfly runs 3 stages in registers and 4 stages across the
//     row.  Lanes are labelled so that the partner of every stage is one DPP control
//     (cg^1, cg^2: quad permutes; cg^4: half-row mirror; cg^8: row rotate by 8): no
//     LDS-crossbar shuffles, and a cross-lane butterfly is one instruction per element,
//     "own += partner * (+1 | -1)", which rounds like the fp32 add/sub the format
//     prescribes (rotate8),
//   - the token norm is a 16-lane butterfly sum over the same partners; on the prefill
//     path four tokens at a time, as a reduce-scatter over the quad, so that a lane takes
//     the square root and the reciprocal of one token instead of four
//     (key_transform_4tokens),
//   - per-channel min/max over tokens reduce over passes (packed fp16 registers), over the
//     4 token slots of a wave and over the 4 waves (LDS); each channel's Eq. 3-4 parameters
//     are computed once and handed to the 16 token slots through LDS,
//   - per-token value min/max reduce over 8 registers and 4|8|16 lanes of the row.
// Rotated keys are held as packed fp16 (that is what they are), values in their input
// type: about half the registers of an fp32 copy, which doubles the resident waves.
// A code is clamp(rint(x/Delta), -z, qmax-z) + z; codes of one packed word are summed in
// fp32 with their place values (exact: small integers) and converted once.  Both code
// images are built in LDS in their final page layout and leave with 16-byte stores.
#pragma once
#include "oscar_common.h"
#include <type_traits>

#include "oscar_rowops.h"

#ifndef OSCAR_ENC_EARLY_K
#define OSCAR_ENC_EARLY_K 1
#endif

struct AppendParams {
  const void* k;
  const void* v;
  int T;
  const int32_t* new_lens;
  oscar_cache c;
  PageGeom g;
  uint32_t flags;
};

// Three sets of encoder instantiations, each in a translation unit of its own (they compile
// side by side, and the register allocation of the published method does not depend on the
// variants' code):
//   XF_PUBLISHED  rotation on, L2 norm per (token, kv head): the switches are constants
//   XF_SWITCHED   rotation and scaling coefficient read from the configuration (the ablations)
//   XF_ALL_HEADS  one norm over all kv heads, with the norm pre-pass it needs
constexpr int XF_PUBLISHED = 0, XF_SWITCHED = 1, XF_ALL_HEADS = 2;
int oscar_launch_append_switched(const AppendParams& P, dim3 grid, hipStream_t st);
int oscar_launch_append_all_heads(const AppendParams& P, dim3 grid, hipStream_t st);

namespace {

constexpr int D = OSCAR_D;
constexpr int R = OSCAR_R;

// 16 bytes of the caller's K / V, which this launch reads exactly once: a non-temporal load
// (measured on a kernel that only moves the encoder's bytes in the encoder's pattern: 223 us
// against 254 us with plain loads for the 1.07 GB + 0.2 GB of a 262144-token prefill)
__device__ __forceinline__ uint4 load_once(const void* p) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Eight consecutive elements of the caller's type, held raw (packed) in registers.
template <typename IO> struct Raw8;
template <> struct Raw8<float> {
  uint4 a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = load_once(p);
    b = load_once(p + 4);
  }
  __device__ __forceinline__ void load_halves(const __half* p) {   // 8 fp16 values, kept in a
    a = *reinterpret_cast<const uint4*>(p);
    b = a;
  }
  __device__ __forceinline__ void store(float* p) const {
    reinterpret_cast<uint4*>(p)[0] = a;
    reinterpret_cast<uint4*>(p)[1] = b;
  }
  __device__ __forceinline__ void widen(float (&x)[8]) const {
    x[0] = __uint_as_float(a.x); x[1] = __uint_as_float(a.y);
    x[2] = __uint_as_float(a.z); x[3] = __uint_as_float(a.w);
    x[4] = __uint_as_float(b.x); x[5] = __uint_as_float(b.y);
    x[6] = __uint_as_float(b.z); x[7] = __uint_as_float(b.w);
  }
};
__device__ __forceinline__ void widen_halves(const uint4& r, float (&x)[8]) {
  const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __half2float(__ushort_as_half((unsigned short)(w[i] & 0xffffu)));
    x[2 * i + 1] = __half2float(__ushort_as_half((unsigned short)(w[i] >> 16)));
  }
}
template <> struct Raw8<__half> {
  uint4 a;
  __device__ __forceinline__ void load(const __half* p) { a = load_once(p); }
  __device__ __forceinline__ void load_halves(const __half* p) { load(p); }
  __device__ __forceinline__ void store(__half* p) const { *reinterpret_cast<uint4*>(p) = a; }
  __device__ __forceinline__ void widen(float (&x)[8]) const { widen_halves(a, x); }
};
template <> struct Raw8<__hip_bfloat16> {
  uint4 a;
  __device__ __forceinline__ void load(const __hip_bfloat16* p) { a = load_once(p); }
  __device__ __forceinline__ void load_halves(const __half* p) {
    a = *reinterpret_cast<const uint4*>(p);
  }
  __device__ __forceinline__ void store(__hip_bfloat16* p) const {
    *reinterpret_cast<uint4*>(p) = a;
  }
  __device__ __forceinline__ void widen(float (&x)[8]) const {
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(w[i] << 16);
      x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

// Keeps a value in a VGPR across an empty asm: stops the compiler from folding the
// fp32 multiply and the fp16 conversion below into one mixed-precision instruction that
// rounds the exact product once (the format rounds to fp32 first, then to fp16).
__device__ __forceinline__ float pin_f32(float x) {
  asm volatile("" : "+v"(x));
  return x;
}

__device__ __forceinline__ uint32_t half_bits(float x) {
  return (uint32_t)__half_as_ushort(__float2half_rn(x));
}
// fp16(a) in the low half, fp16(b) in the high half, both rounded to nearest even: one
// instruction on this chip (v_cvt_pk_f16_f32)
__device__ __forceinline__ uint32_t pack_halves(float a, float b) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

// value of lane j (a constant after unrolling) of the caller's quad
template <int CTRL> __device__ __forceinline__ float dpp_read(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float quad_bcast(float v, int j) {
  switch (j) {
    case 0: return dpp_read<0x00>(v);
    case 1: return dpp_read<0x55>(v);
    case 2: return dpp_read<0xAA>(v);
    default: return dpp_read<0xFF>(v);
  }
}
// sum of squares of the 128 rotated channels: balanced tree, adjacent pairs first
__device__ __forceinline__ float row_sumsq(const float (&x)[8]) {
  float t[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) t[i] = x[i] * x[i];
  float s = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
  s = s + partner<0>(s);
  s = s + partner<1>(s);
  s = s + partner<2>(s);
  s = s + partner<3>(s);
  return s;
}

// the same tree over |x|, and the maximum of |x| (App. "Ablation Study": alternative
// scaling coefficients)
__device__ __forceinline__ float row_sumabs(const float (&x)[8]) {
  float t[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) t[i] = fabsf(x[i]);
  float s = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
  s = s + partner<0>(s);
  s = s + partner<1>(s);
  s = s + partner<2>(s);
  s = s + partner<3>(s);
  return s;
}
__device__ __forceinline__ float row_maxabs(const float (&x)[8]) {
  float m = fabsf(x[0]);
#pragma unroll
  for (int i = 1; i < 8; ++i) m = fmaxf(m, fabsf(x[i]));
  m = fmaxf(m, partner<0>(m));
  m = fmaxf(m, partner<1>(m));
  m = fmaxf(m, partner<2>(m));
  m = fmaxf(m, partner<3>(m));
  return m;
}

// The switches of the key transform (uniform over a launch): rotation on/off and the
// OSCAR_SCALE_* coefficient.  Default-constructed = the method as published.
struct KeyXf {
  bool rotate = true;
  int scale_mode = OSCAR_SCALE_L2;
};
__device__ __forceinline__ KeyXf key_xf_of(const oscar_config& cfg) {
  KeyXf m;
  m.rotate = cfg.rotation == OSCAR_ROTATION_ON;
  m.scale_mode = cfg.scale_mode;
  return m;
}

template <typename META>
__device__ __forceinline__ uint4 key_transform8(float (&x)[8], const uint32_t (&sgn)[4],
                                                float& n_st, const KeyXf m = KeyXf()) {
  if (m.rotate) rotate8(x, sgn);
  float nf;
  if (m.scale_mode == OSCAR_SCALE_L2) {
    nf = round_meta<META>(sqrtf(row_sumsq(x)));
  } else if (m.scale_mode == OSCAR_SCALE_MAX) {
    nf = round_meta<META>(row_maxabs(x));
  } else if (m.scale_mode == OSCAR_SCALE_MEAN_ABS) {
    nf = round_meta<META>(row_sumabs(x) * (1.0f / (float)D));
  } else {
    nf = 1.0f;
  }
  float inv = (nf > 0.0f && !isinf(nf)) ? 1.0f / nf : 0.0f;
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    w[i] = pack_halves(pin_f32(x[2 * i] * inv), pin_f32(x[2 * i + 1] * inv));
  n_st = nf;
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// value of row lane r ^ 4: lanes 0-3 and 8-11 read four lanes up, the others four lanes down
__device__ __forceinline__ float same_position_next_quad(float v) {
  const int x = __builtin_bit_cast(int, v);
  int t = __builtin_amdgcn_update_dpp(0, x, 0x104 /* row_shl:4 */, 0xf, 0x5, false);
  t = __builtin_amdgcn_update_dpp(t, x, 0x114 /* row_shr:4 */, 0xf, 0xa, false);
  return __builtin_bit_cast(float, t);
}

// The published transform (rotation, L2 norm) of four tokens held by the same 16-lane row.
// The cross-lane part of the four sums of squares is a reduce-scatter over the quad followed
// by an all-reduce over the row's four quads (whose lanes hold channel groups that differ in
// bits 2 and 3): in the first stage a lane passes on the two
// sums its partner keeps and adds what it receives to the two it keeps, in the second stage
// one of one -- the additions of the balanced tree, operands in either order -- so that the
// lane at quad position j ends up with the complete sum of token j and takes one square root
// and one reciprocal for it; the four reciprocals come back by quad broadcast.
// n_own: the stored norm of token `qj` (the caller's position in its quad).
template <typename META>
__device__ __forceinline__ void key_transform_4tokens(float (&x)[4][8], const uint32_t (&sgn)[4],
                                                      int qj, float& n_own, uint4* ku) {
  float s[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    rotate8(x[j], sgn);
    float t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = x[j][i] * x[j][i];
    s[j] = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
  }
  const bool odd = (qj & 1) != 0, high = (qj & 2) != 0;
  const float k01 = odd ? s[1] : s[0], g01 = odd ? s[0] : s[1];
  const float k23 = odd ? s[3] : s[2], g23 = odd ? s[2] : s[3];
  const float t01 = k01 + partner<0>(g01);   // token 0 (even lanes) or 1 (odd lanes)
  const float t23 = k23 + partner<0>(g23);   // token 2 or 3
  const float kk = high ? t23 : t01, gg = high ? t01 : t23;
  float u = kk + partner<1>(gg);             // token qj, summed over this quad's channel groups
  // The other quad of the half-row holds the channel groups that differ in bit 2; the partner
  // there must sit at the same quad position (partner<2> mirrors the half-row and would hand
  // over another token's sum): row lane r ^ 4.
  u = u + same_position_next_quad(u);
  u = u + partner<3>(u);                     // row lane r ^ 8
  const float nf = round_meta<META>(sqrtf(u));
  const float inv = (nf > 0.0f && !isinf(nf)) ? 1.0f / nf : 0.0f;
  n_own = nf;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float iv = quad_bcast(inv, j);
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      w[i] = pack_halves(pin_f32(x[j][2 * i] * iv), pin_f32(x[j][2 * i + 1] * iv));
    ku[j] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// Same transform with a norm that is already known (rounded to its storage type).
__device__ __forceinline__ uint4 key_transform8_given(float (&x)[8], const uint32_t (&sgn)[4],
                                                      float nf, bool rotate) {
  if (rotate) rotate8(x, sgn);
  float inv = (nf > 0.0f && !isinf(nf)) ? 1.0f / nf : 0.0f;
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    w[i] = pack_halves(pin_f32(x[2 * i] * inv), pin_f32(x[2 * i + 1] * inv));
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// Token-wise norm over all kv heads (App. "Fused Hadamard-Norm Kernel": squared sums
// accumulated across heads): every head's vector of the token is rotated, its squared sum
// taken in the same tree order, the sums added in head order, one square root.
// row0 = this lane's 8 channels of head 0 of the token; heads are D elements apart.
// Heads are fetched four at a time; slots past the last head repeat it and add +0.
template <typename IO, typename META>
__device__ __forceinline__ float token_norm_all_heads(const IO* row0, int n_heads,
                                                      const uint32_t (&sgn)[4], bool rotate) {
  float s = 0.0f;
  for (int h0 = 0; h0 < n_heads; h0 += 4) {
    Raw8<IO> r[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int h = h0 + j < n_heads ? h0 + j : n_heads - 1;
      r[j].load(row0 + (size_t)h * D);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float x[8];
      r[j].widen(x);
      if (rotate) rotate8(x, sgn);
      const float sh = row_sumsq(x);
      s = s + (h0 + j < n_heads ? sh : 0.0f);
    }
  }
  return round_meta<META>(sqrtf(s));
}

// Eq. 3-4 parameters of one group, rounded to storage before use.
// zp_min: the zero-point is the group minimum itself (float zero-point form of the complexity
// appendix) instead of the integer of Eq. 3-4.
template <typename META, int BITS>
__device__ __forceinline__ void quant_params(float mn, float mx, bool zp_min, float& df, float& rd,
                                             float& z) {
  const float qmax = (float)((1 << BITS) - 1);
  float dl = (mx - mn) / qmax;
  df = round_meta<META>(dl);
  if (df == 0.0f) {
    df = round_meta<META>(fabsf(mn));
    if (df == 0.0f || isinf(df)) df = 1.0f;
  }
  rd = 1.0f / df;
  z = zp_min ? round_meta<META>(mn) : round_meta<META>(rintf(-mn * rd));
}

// packed fp16 min / max (finite inputs).  volatile like every asm block of this library: the
// one ordering problem ever found around such blocks (oscar_decode_mfma.hip, keep_tuple)
// needed a matrix instruction in flight, which this kernel does not have, and nothing is
// gained by letting the blocks move
__device__ __forceinline__ uint32_t pk_min_f16(uint32_t a, uint32_t b) {
  uint32_t r;
  asm volatile("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ uint32_t pk_max_f16(uint32_t a, uint32_t b) {
  uint32_t r;
  asm volatile("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float half_of(uint32_t w, int hi) {
  return __half2float(__ushort_as_half((unsigned short)(hi ? (w >> 16) : (w & 0xffffu))));
}

// Integer zero-point: clamp(rint(x * rd) + z, 0, qmax) - z, i.e. the code minus its
// zero-point (an integer in fp32), with lo = -z, hi = qmax - z.
// Float zero-point (ZPMIN): the code itself, clamp(rint((x - zero) * rd), 0, qmax), with
// lo = zero and hi unused.
template <bool ZPMIN, int BITS>
__device__ __forceinline__ float code_term(float x, float rd, float lo, float hi) {
  if (ZPMIN) return __builtin_amdgcn_fmed3f(rintf((x - lo) * rd), 0.0f, (float)((1 << BITS) - 1));
  return __builtin_amdgcn_fmed3f(rintf(x * rd), lo, hi);
}

struct SeqPlan {
  int n;          // tokens appended by this call
  int r0;         // residual tokens on entry
  int packed_pages;
  int nq;         // blocks quantized by this call
  int tail_len;   // residual tokens on exit
  bool ok;
};

__device__ __forceinline__ SeqPlan plan_sequence(const AppendParams& P, int b) {
  SeqPlan s;
  const int seq_len = P.c.seq_lens[b];
  s.r0 = P.c.res_lens[b];
  int n = P.new_lens ? P.new_lens[b] : P.T;
  n = n < 0 ? 0 : (n > P.T ? P.T : n);
  s.n = n;
  s.packed_pages = (seq_len - s.r0) / R;
  const int pending = s.r0 + n;
  const int nfull = pending / R, rem = pending % R;
  const bool eager = (P.flags & OSCAR_APPEND_EAGER) != 0;
  s.nq = (n > 0 && rem == 0 && !eager) ? nfull - 1 : nfull;
  if (n == 0) s.nq = 0;  // nothing arrives: a full residual keeps waiting
  s.tail_len = pending - s.nq * R;
  s.ok = (s.packed_pages + s.nq) <= P.c.max_pages_per_seq;
  return s;
}

template <int BITS> __device__ __forceinline__ constexpr float place_value(int i) {
  // 4^i (2-bit codes) or 16^i (4-bit codes)
  float v = 1.0f;
  for (int k = 0; k < i; ++k) v *= (float)(1 << BITS);
  return v;
}

// One token's 8 codes of a channel group -> one 16-bit (2-bit codes) or 32-bit (4-bit codes)
// piece of chunk (tile = tok/16, n = tok%16, q4 = cg/4) of the key-code page image.
// The code itself, clamp(rint(x * rd) + z, 0, qmax), from lo = -z: the form the packers take
// when a zero-point is so large that sums of (code - z) * place would leave the range in which
// fp32 holds every integer (|z| * 21845 < 2^24 for a word of eight 2-bit codes).
template <int BITS> __device__ __forceinline__ float code_exact(float x, float rd, float lo) {
  return __builtin_amdgcn_fmed3f(rintf(x * rd) - lo, 0.0f, (float)((1 << BITS) - 1));
}
// |z| up to this bound goes through the (code - z) form: every partial sum of a packed word
// stays an exactly representable integer (2-bit: 512 * 21845, 4-bit: 512 * 4369 < 2^24)
constexpr float kZeroPointFastBound = 512.0f;

// EXACT: integer zero-points past kZeroPointFastBound (wave-uniform choice of the caller).
template <bool ZPMIN, int BITS, bool EXACT>
__device__ __forceinline__ void key_codes(const uint4& ku, const float (&rd)[8], const float (&lo)[8],
                                          const float (&hi)[8], float zs0, float zs1,
                                          uint8_t* s_kimg, int tok, int cg) {
  float x[8];
  widen_halves(ku, x);
  const int off = chunk_offset(BITS, tok / 16, tok % 16, cg / 4) + (cg % 4) * BITS;
  auto term = [&](int e) {
    return EXACT ? code_exact<BITS>(x[e], rd[e], lo[e]) : code_term<ZPMIN, BITS>(x[e], rd[e], lo[e], hi[e]);
  };
  if (BITS == 2) {
    float w = EXACT ? 0.0f : zs0;
#pragma unroll
    for (int e = 0; e < 8; ++e) w = fmaf(term(e), place_value<BITS>(e), w);
    *reinterpret_cast<uint16_t*>(&s_kimg[off]) = (uint16_t)(uint32_t)w;
  } else {
    float w0 = EXACT ? 0.0f : zs0, w1 = EXACT ? 0.0f : zs1;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      w0 = fmaf(term(e), place_value<BITS>(e), w0);
      w1 = fmaf(term(e + 4), place_value<BITS>(e), w1);
    }
    *reinterpret_cast<uint32_t*>(&s_kimg[off]) = (uint32_t)w0 | ((uint32_t)w1 << 16);
  }
}

template <typename IO, typename META, int BITS, int KG, int XF>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(sizeof(IO) == 4 ? (XF == 2 ? 2 : 3) : 4))) void oscar_append_kernel(AppendParams P) {
  constexpr bool NORM_ALL = XF == XF_ALL_HEADS;
  constexpr int NGK = R / KG;        // key groups per page
  constexpr int PPG = KG / 16;       // passes per key group
  constexpr float QMAX = (float)((1 << BITS) - 1);
  constexpr int IMG = R * D * BITS / 8;   // bytes of one code image

  struct MinMax {
    uint4 mn, mx;   // packed fp16, the 8 channels of a channel group
  };
  __shared__ __align__(16) MinMax s_red[NGK][4][16];   // [group][wave][channel group]
  // per channel: 1/Delta, -z, qmax-z, z*place; channel 8*cg + e sits at slot 16*e + cg, so the
  // 16 lanes of a row (cg = 0..15) read 256 consecutive bytes (channel order would put them
  // 128 bytes apart: an 8-way bank conflict on every read)
  __shared__ __align__(16) float4 s_par[NGK][D];
  __shared__ __align__(16) uint8_t s_kimg[IMG];        // key-code page image
  // value-code page image, staged with 64 bytes of padding after every eighth of the image:
  // the lanes of a wave write pieces that are 1/8, 1/4 and 1/2 image apart, which would
  // otherwise all fall into the same 8 LDS banks
  __shared__ __align__(16) uint8_t s_vimg[IMG + 8 * 64];
  __shared__ __align__(16) META s_vmeta[2][4][R];
  __shared__ __align__(16) META s_norm[R];

  // kv head fastest: the workgroups that share a token block's rows in memory run together
  const int b = blockIdx.z, kvh = blockIdx.x, blk = blockIdx.y;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int slot = tid >> 4;                            // token of a pass
  const int cg = channel_group_of_row_lane(tid & 15);   // channels 8*cg .. 8*cg+7
  const int Hkv = P.c.cfg.n_kv_heads;
  const bool zp_min = P.c.cfg.zp_mode == OSCAR_ZP_MIN;
  const KeyXf xf = XF == XF_PUBLISHED ? KeyXf() : key_xf_of(P.c.cfg);
  uint32_t sgn[4];
#pragma unroll
  for (int st = 0; st < 4; ++st) sgn[st] = ((cg >> st) & 1) ? 0x80000000u : 0u;

  const SeqPlan sp = plan_sequence(P, b);
  do {  // one pass; "break" = this workgroup has nothing (more) to do
  if (sp.n <= 0) break;
  if (!sp.ok) {
    if (tid == 0 && blk == 0 && kvh == 0 && P.c.dev_status) *P.c.dev_status = OSCAR_ERR_CAPACITY;
    break;
  }
  const bool do_block = blk < sp.nq;
  const bool do_tail = (blk == 0);
  if (!do_block && !do_tail) break;
  // the page this block goes to, asked for now: behind the barrier below the workgroup would
  // wait for the answer
  const int phys = do_block ? P.c.block_table[(size_t)b * P.c.max_pages_per_seq + sp.packed_pages + blk] : 0;

  const IO* knew = reinterpret_cast<const IO*>(P.k);
  const IO* vnew = reinterpret_cast<const IO*>(P.v);
  const size_t res_base = ((size_t)b * Hkv + kvh) * R;
  __half* res_k = reinterpret_cast<__half*>(P.c.res_k) + res_base * D;
  IO* res_v = reinterpret_cast<IO*>(P.c.res_v) + res_base * D;
  META* res_norm = reinterpret_cast<META*>(P.c.res_norm) + res_base;

  // ---- phase 1: gather the block (old residual tokens first, then new tokens) and
  // transform the new keys; keys end up as packed fp16 K_u, values stay raw ----
  uint4 ku[8];
  Raw8<IO> vraw[8];
  float nrm[8];
  // batched_norms (uniform over the workgroup): the norms of tokens 16*(4*hb + j) + slot sit in
  // nrm_q[hb] of the lanes whose position in their quad is j, and nrm[] is unused
  bool batched_norms = false;
  float nrm_q[2] = {0.0f, 0.0f};
  // NORM_ALL: the norms of new tokens that end up in a page were written into that page's
  // norm slots (of every head) by oscar_token_norm_kernel, launched just before this kernel
  const META* pre_norm = nullptr;
  if (NORM_ALL && do_block) {
    const int phys0 = phys;
    pre_norm = reinterpret_cast<const META*>(reinterpret_cast<const uint8_t*>(P.c.k_norms) +
                                             ((size_t)phys0 * Hkv + kvh) * P.g.k_norms_bytes);
  }
  if (do_block && blk * R >= sp.r0) {
    // the whole block is new tokens (every block of a prefill): straight-line loads
    Raw8<IO> kraw[8];
    const size_t tok0 = (size_t)b * P.T + (size_t)(blk * R - sp.r0 + slot);
    const IO* kp = knew + (tok0 * Hkv + kvh) * D + cg * 8;
    const IO* vp = vnew + (tok0 * Hkv + kvh) * D + cg * 8;
    const size_t pstride = (size_t)16 * Hkv * D;
#pragma unroll
    for (int p = 0; p < 8; ++p) kraw[p].load(kp + p * pstride);
    // The values are not needed before the key codes are done: their loads go out behind the
    // first half of the key transform (held there by the fences), which keeps their 32
    // registers free while the transform is at its widest and spreads the workgroup's requests.
    auto load_values = [&]() {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int p = 0; p < 8; ++p) vraw[p].load(vp + p * pstride);
      __builtin_amdgcn_sched_barrier(0);
    };
    if (NORM_ALL) {
#pragma unroll
      for (int p = 0; p < 8; ++p) nrm[p] = to_f32<META>(pre_norm[tok_meta_pos(p * 16 + slot)]);
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        float x[8];
        kraw[p].widen(x);
        ku[p] = key_transform8_given(x, sgn, nrm[p], xf.rotate);
        if (p == 3) load_values();
      }
    } else if (XF == XF_PUBLISHED) {
      // the method as published: four tokens at a time, one square root and one reciprocal
      // per lane instead of four (key_transform_4tokens)
      batched_norms = true;
#pragma unroll
      for (int hb = 0; hb < 2; ++hb) {
        float x[4][8];
#pragma unroll
        for (int j = 0; j < 4; ++j) kraw[4 * hb + j].widen(x[j]);
        key_transform_4tokens<META>(x, sgn, tid & 3, nrm_q[hb], &ku[4 * hb]);
        if (hb == 0) load_values();
      }
    } else {
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        float x[8];
        kraw[p].widen(x);
        ku[p] = key_transform8<META>(x, sgn, nrm[p], xf);
        if (p == 3) load_values();
      }
    }
  } else if (do_block) {
    Raw8<IO> kraw[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int pi = blk * R + p * 16 + slot;  // index among pending tokens
      if (pi < sp.r0) {
        kraw[p].load_halves(res_k + (size_t)pi * D + cg * 8);
        nrm[p] = to_f32<META>(res_norm[pi]);
        vraw[p].load(res_v + (size_t)pi * D + cg * 8);
      } else {
        const size_t ti = (size_t)(pi - sp.r0);
        const size_t off = (((size_t)b * P.T + ti) * Hkv + kvh) * D + cg * 8;
        kraw[p].load(knew + off);
        vraw[p].load(vnew + off);
        nrm[p] = 0.0f;
      }
    }
    // the branch above is uniform per 16-lane token row; every row runs the transform (its
    // result is dropped for tokens that came from the residual, which are K_u already)
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int pi = blk * R + p * 16 + slot;
      const bool old = pi < sp.r0;
      float x[8], nn;
      kraw[p].widen(x);
      uint4 nu;
      if (NORM_ALL) {   // (rows that came from the residual drop the result)
        nn = to_f32<META>(pre_norm[tok_meta_pos(p * 16 + slot)]);
        nu = key_transform8_given(x, sgn, nn, xf.rotate);
      } else {
        nu = key_transform8<META>(x, sgn, nn, xf);
      }
      ku[p].x = old ? kraw[p].a.x : nu.x;
      ku[p].y = old ? kraw[p].a.y : nu.y;
      ku[p].z = old ? kraw[p].a.z : nu.z;
      ku[p].w = old ? kraw[p].a.w : nu.w;
      nrm[p] = old ? nrm[p] : nn;
    }
  }
  __syncthreads();  // every read of the old residual precedes the tail write below

  // ---- phase 2 (workgroup 0): new residual tail ----
  if (do_tail) {
    const int src0 = (sp.nq == 0) ? 0 : sp.nq * R - sp.r0;  // first new token of the tail
    const int dst0 = (sp.nq == 0) ? sp.r0 : 0;              // its residual slot
    const int cnt = sp.n - src0;                            // new tokens going to the residual
    for (int i0 = 0; i0 < cnt; i0 += 16) {
      const int i = i0 + slot;
      const int ic = i < cnt ? i : cnt - 1;
      const size_t off = (((size_t)b * P.T + (size_t)(src0 + ic)) * Hkv + kvh) * D + cg * 8;
      Raw8<IO> kin, vin;
      kin.load(knew + off);
      vin.load(vnew + off);
      float x[8], nn;
      kin.widen(x);
      uint4 nu;
      if (NORM_ALL) {
        nn = token_norm_all_heads<IO, META>(knew + off - (size_t)kvh * D, Hkv, sgn, xf.rotate);
        nu = key_transform8_given(x, sgn, nn, xf.rotate);
      } else {
        nu = key_transform8<META>(x, sgn, nn, xf);
      }
      if (i < cnt) {
        const int ds = dst0 + i;
        *reinterpret_cast<uint4*>(res_k + (size_t)ds * D + cg * 8) = nu;
        vin.store(res_v + (size_t)ds * D + cg * 8);
        if (cg == 0) res_norm[ds] = from_f32<META>(nn);
      }
    }
  }
  if (!do_block) break;

  // ---- phase 3: quantize the block held in registers ----
  const size_t pg = (size_t)phys * Hkv + kvh;
  uint8_t* o_kcodes = reinterpret_cast<uint8_t*>(P.c.k_codes) + pg * P.g.k_codes_bytes;
  META* o_kmeta = reinterpret_cast<META*>(reinterpret_cast<uint8_t*>(P.c.k_meta) + pg * P.g.k_meta_bytes);
  META* o_knorm = reinterpret_cast<META*>(reinterpret_cast<uint8_t*>(P.c.k_norms) + pg * P.g.k_norms_bytes);
  uint8_t* o_vcodes = reinterpret_cast<uint8_t*>(P.c.v_codes) + pg * P.g.v_codes_bytes;
  META* o_vmeta = reinterpret_cast<META*>(reinterpret_cast<uint8_t*>(P.c.v_meta) + pg * P.g.v_meta_bytes);

  // keys: per-channel min/max over the tokens of each group: passes, then the 4 token rows
  // of the wave, then (through LDS) the 4 waves
#pragma unroll
  for (int gk = 0; gk < NGK; ++gk) {
    uint32_t mn[4] = {ku[gk * PPG].x, ku[gk * PPG].y, ku[gk * PPG].z, ku[gk * PPG].w};
    uint32_t mx[4] = {mn[0], mn[1], mn[2], mn[3]};
#pragma unroll
    for (int p = 1; p < PPG; ++p) {
      const uint4 q = ku[gk * PPG + p];
      const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        mn[j] = pk_min_f16(mn[j], w[j]);
        mx[j] = pk_max_f16(mx[j], w[j]);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      mn[j] = pk_min_f16(mn[j], (uint32_t)__shfl_xor((int)mn[j], 16, 64));
      mx[j] = pk_max_f16(mx[j], (uint32_t)__shfl_xor((int)mx[j], 16, 64));
      mn[j] = pk_min_f16(mn[j], (uint32_t)__shfl_xor((int)mn[j], 32, 64));
      mx[j] = pk_max_f16(mx[j], (uint32_t)__shfl_xor((int)mx[j], 32, 64));
    }
    if (lane < 16) {
      s_red[gk][wave][cg].mn = make_uint4(mn[0], mn[1], mn[2], mn[3]);
      s_red[gk][wave][cg].mx = make_uint4(mx[0], mx[1], mx[2], mx[3]);
    }
  }
  if (batched_norms) {
    if ((tid & 15) < 4) {   // first quad of the token row: lane j holds the norms of passes j, 4 + j
#pragma unroll
      for (int hb = 0; hb < 2; ++hb)
        s_norm[tok_meta_pos((4 * hb + (tid & 3)) * 16 + slot)] = from_f32<META>(nrm_q[hb]);
    }
  } else if (cg == 0) {
#pragma unroll
    for (int p = 0; p < 8; ++p) s_norm[tok_meta_pos(p * 16 + slot)] = from_f32<META>(nrm[p]);
  }
  __syncthreads();

  // Eq. 3-4 parameters, once per channel and group: thread (slot < 8, cg) takes channel
  // 8*cg + slot, stores Delta and z (operand order, see kmeta_pos_of_chan) and leaves what
  // the coders need in LDS
  if (slot < 8) {
    const int e = slot, c = 8 * cg + e;
#pragma unroll
    for (int gk = 0; gk < NGK; ++gk) {
      uint32_t mnw = 0, mxw = 0;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t* rp = reinterpret_cast<const uint32_t*>(&s_red[gk][w][cg]);
        const uint32_t a = rp[e >> 1], bb = rp[4 + (e >> 1)];
        mnw = w == 0 ? a : pk_min_f16(mnw, a);
        mxw = w == 0 ? bb : pk_max_f16(mxw, bb);
      }
      float df, rd, z;
      quant_params<META, BITS>(half_of(mnw, e & 1), half_of(mxw, e & 1), zp_min, df, rd, z);
      // place value of this channel's code inside its packed word (4-bit: two 16-bit halves)
      const float place = ldexpf(1.0f, BITS * ((BITS == 2) ? e : (e & 3)));
      s_par[gk][16 * e + cg] = zp_min ? make_float4(rd, z, 0.0f, 0.0f)
                            : make_float4(rd, -z, QMAX - z, z * place);
      const int pos = kmeta_pos_of_chan(BITS, c);
      o_kmeta[(size_t)gk * D + pos] = from_f32<META>(df);
      o_kmeta[(size_t)(NGK + gk) * D + pos] = from_f32<META>(z);
    }
  }
  __syncthreads();

  // key codes: a token's 8 codes of this channel group form one 16-bit (2-bit codes) or
  // 32-bit (4-bit codes) piece of chunk (tile = tok/16, n = tok%16, q4 = cg/4)
#pragma unroll
  for (int gk = 0; gk < NGK; ++gk) {
    float rd[8], lo[8], hi[8], zs0 = 0.0f, zs1 = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float4 q = s_par[gk][16 * e + cg];
      rd[e] = q.x;
      lo[e] = q.y;
      hi[e] = q.z;
      if (BITS == 2 || e < 4) zs0 += q.w;
      else zs1 += q.w;
    }
    if (zp_min) {
#pragma unroll
      for (int p = gk * PPG; p < (gk + 1) * PPG; ++p)
        key_codes<true, BITS, false>(ku[p], rd, lo, hi, zs0, zs1, s_kimg, p * 16 + slot, cg);
    } else {
      // a nearly constant channel far from zero has a huge integer zero-point: the wave then
      // packs from the codes themselves (rare; the choice is uniform over the wave)
      bool big = false;
#pragma unroll
      for (int e = 0; e < 8; ++e) big |= fabsf(lo[e]) > kZeroPointFastBound;
      if (__any(big)) {
#pragma unroll
        for (int p = gk * PPG; p < (gk + 1) * PPG; ++p)
          key_codes<false, BITS, true>(ku[p], rd, lo, hi, zs0, zs1, s_kimg, p * 16 + slot, cg);
      } else {
#pragma unroll
        for (int p = gk * PPG; p < (gk + 1) * PPG; ++p)
          key_codes<false, BITS, false>(ku[p], rd, lo, hi, zs0, zs1, s_kimg, p * 16 + slot, cg);
      }
    }
  }

#if OSCAR_ENC_EARLY_K
  // the key-code image is complete: it leaves now, under the value phase, instead of with
  // everything else at the end of the workgroup (one more barrier)
  __syncthreads();
  {
    constexpr int NV = IMG / 16;
    const uint4* ksrc = reinterpret_cast<const uint4*>(&s_kimg[0]);
    uint4* kdst = reinterpret_cast<uint4*>(o_kcodes);
#pragma unroll
    for (int i = tid; i < NV; i += 256) kdst[i] = ksrc[i];
  }
#endif

  // values: per-token min/max over each group of v_group channels (8 registers, then the
  // 4 | 8 | 16 lanes of the group).  The thread's 8 tokens of one channel are the elements
  // e = pass of k-step kk = slot/4 in chunk (tile = c/16, n = c%16, q4 = slot%4): even
  // passes fill one byte (2-bit) / half-word (4-bit) of the piece, odd passes the other.
  {
    const int L = P.g.v_group / 8;  // lanes per value group: 4, 8 or 16
    float vmn[8], vmx[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      float v[8];
      vraw[p].widen(v);
      const float mn = min_finite(min3_finite(min3_finite(v[0], v[1], v[2]), v[3], v[4]),
                                  min3_finite(v[5], v[6], v[7]));
      const float mx = max_finite(max3_finite(max3_finite(v[0], v[1], v[2]), v[3], v[4]),
                                  max3_finite(v[5], v[6], v[7]));
      float rmn = partner_min<1>(partner_min<0>(mn)), rmx = partner_max<1>(partner_max<0>(mx));
      if (L > 4) { rmn = partner_min<2>(rmn); rmx = partner_max<2>(rmx); }
      if (L > 8) { rmn = partner_min<3>(rmn); rmx = partner_max<3>(rmx); }
      vmn[p] = rmn;
      vmx[p] = rmx;
    }
    // The 4 lanes of a quad always share a value group: lane j of the quad works out the
    // Eq. 3-4 parameters of passes 2j and 2j+1 and the quad reads them back by broadcast.
    const int qj = tid & 3;
    float prd[2], plo[2], phi[2], pz[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const float mn = qj == 0 ? vmn[i] : qj == 1 ? vmn[2 + i] : qj == 2 ? vmn[4 + i] : vmn[6 + i];
      const float mx = qj == 0 ? vmx[i] : qj == 1 ? vmx[2 + i] : qj == 2 ? vmx[4 + i] : vmx[6 + i];
      float df;
      quant_params<META, BITS>(mn, mx, zp_min, df, prd[i], pz[i]);
      plo[i] = zp_min ? pz[i] : -pz[i];
      phi[i] = QMAX - pz[i];
      if ((cg & (L - 1) & ~3) == 0) {   // first quad of its value group stores the metadata
        const int tok = (2 * qj + i) * 16 + slot, gv = cg >> (L == 4 ? 2 : L == 8 ? 3 : 4);
        s_vmeta[0][gv][tok_meta_pos(tok)] = from_f32<META>(df);
        s_vmeta[1][gv][tok_meta_pos(tok)] = from_f32<META>(pz[i]);
      }
    }
    float wv0[8], wv1[8], zv0 = 0.0f, zv1 = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) wv0[e] = wv1[e] = 0.0f;
    // mode 0: integer zero-point, (code - z) form; 1: float zero-point; 2: integer zero-point
    // past kZeroPointFastBound somewhere in the wave, the codes themselves
    auto code_values = [&](auto mode_tag) {
      constexpr int MODE = decltype(mode_tag)::value;
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        float v[8];
        vraw[p].widen(v);
        const float rd = quad_bcast(prd[p & 1], p >> 1);
        const float lo = quad_bcast(plo[p & 1], p >> 1);
        const float hi = quad_bcast(phi[p & 1], p >> 1);
        const float z = MODE == 0 ? quad_bcast(pz[p & 1], p >> 1) : 0.0f;
        const float pl = place_value<BITS>(p >> 1);
        float t[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
          t[e] = MODE == 1   ? code_term<true, BITS>(v[e], rd, lo, hi)
                 : MODE == 2 ? code_exact<BITS>(v[e], rd, lo)
                             : code_term<false, BITS>(v[e], rd, lo, hi);
        if ((p & 1) == 0) {
#pragma unroll
          for (int e = 0; e < 8; ++e) wv0[e] = fmaf(t[e], pl, wv0[e]);
          zv0 = fmaf(z, pl, zv0);
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) wv1[e] = fmaf(t[e], pl, wv1[e]);
          zv1 = fmaf(z, pl, zv1);
        }
      }
    };
    if (zp_min) {
      code_values(std::integral_constant<int, 1>());
    } else if (__any(fabsf(pz[0]) > kZeroPointFastBound || fabsf(pz[1]) > kZeroPointFastBound)) {
      code_values(std::integral_constant<int, 2>());
    } else {
      code_values(std::integral_constant<int, 0>());
    }
    const int kk = slot >> 2, q4 = slot & 3;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = 8 * cg + e;
      const uint32_t ev = (uint32_t)(wv0[e] + zv0), od = (uint32_t)(wv1[e] + zv1);
      const int lin = chunk_offset(BITS, c / 16, c % 16, q4);
      const int base = lin + (lin / (IMG / 8)) * 64;
      if (BITS == 2) {
        s_vimg[base + (kk >> 1) * 4 + (kk & 1)] = (uint8_t)ev;
        s_vimg[base + (kk >> 1) * 4 + 2 + (kk & 1)] = (uint8_t)od;
      } else {
        *reinterpret_cast<uint32_t*>(&s_vimg[base + kk * 4]) = ev | (od << 16);
      }
    }
  }
  __syncthreads();

  // ---- phase 4: coalesced page stores ----
  {
    constexpr int NV = IMG / 16;  // uint4 count: 256 (2-bit) or 512 (4-bit)
    const uint4* ksrc = reinterpret_cast<const uint4*>(&s_kimg[0]);
    const uint4* vsrc = reinterpret_cast<const uint4*>(&s_vimg[0]);
    uint4* kdst = reinterpret_cast<uint4*>(o_kcodes);
    uint4* vdst = reinterpret_cast<uint4*>(o_vcodes);
#pragma unroll
    for (int i = tid; i < NV; i += 256) {
#if !OSCAR_ENC_EARLY_K
      kdst[i] = ksrc[i];
#endif
      vdst[i] = vsrc[i + (i / (NV / 8)) * 4];   // un-pad: 4 x 16 bytes per eighth
    }
  }
  {
    // value metadata image: Delta[ngv][R] then zero[ngv][R], 16 bytes per thread (each plane of
    // the staging array holds 4 groups, of which the first ngv are in use)
    const int per16 = P.g.ngv * R * (int)sizeof(META) / 16;   // 16-byte pieces of a plane: <= 128
    if (tid < 2 * per16) {
      const int plane = tid >= per16 ? 1 : 0, idx = tid - plane * per16;
      reinterpret_cast<uint4*>(o_vmeta)[plane * per16 + idx] =
          reinterpret_cast<const uint4*>(&s_vmeta[plane][0][0])[idx];
    }
    if (tid < R * (int)sizeof(META) / 16)
      reinterpret_cast<uint4*>(o_knorm)[tid] = reinterpret_cast<const uint4*>(&s_norm[0])[tid];
  }
  } while (false);

  // ---- length update, folded in: the last workgroup to finish advances the lengths of all
  // sequences.  Every other workgroup consumed its loads of seq_lens / res_lens before it
  // took its ticket, so no fence is needed (an agent-scope fence per workgroup costs a
  // cache write-back each and nearly doubled the prefill time); the new lengths become
  // visible to later kernels at the end of this one. ----
  if (P.c.tickets) {
    __shared__ int s_last;
    __syncthreads();
    if (tid == 0) {
      const int total = (int)(gridDim.x * gridDim.y * gridDim.z);
      s_last = (atomicAdd(&P.c.tickets[0], 1) == total - 1) ? 1 : 0;
    }
    __syncthreads();
    if (s_last) {
      for (int bb = tid; bb < P.c.batch; bb += 256) {
        const SeqPlan q = plan_sequence(P, bb);
        if (q.n > 0 && q.ok) {
          P.c.seq_lens[bb] += q.n;
          P.c.res_lens[bb] = q.tail_len;
        }
      }
      if (tid == 0) P.c.tickets[0] = 0;
    }
  }
}

template <typename META>
__global__ void oscar_update_lens_kernel(AppendParams P) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= P.c.batch) return;
  const SeqPlan sp = plan_sequence(P, b);
  if (sp.n <= 0 || !sp.ok) return;
  P.c.seq_lens[b] += sp.n;
  P.c.res_lens[b] = sp.tail_len;
}

template <typename IO, typename META, int BITS, int XF>
int launch_kg(const AppendParams& P, dim3 grid, hipStream_t st) {
  switch (P.g.k_group) {
    case 32: hipLaunchKernelGGL((oscar_append_kernel<IO, META, BITS, 32, XF>), grid, dim3(256), 0, st, P); break;
    case 64: hipLaunchKernelGGL((oscar_append_kernel<IO, META, BITS, 64, XF>), grid, dim3(256), 0, st, P); break;
    case 128: hipLaunchKernelGGL((oscar_append_kernel<IO, META, BITS, 128, XF>), grid, dim3(256), 0, st, P); break;
    default: return OSCAR_ERR_UNSUPPORTED;
  }
  return OSCAR_OK;
}

template <typename IO, typename META, int XF>
int launch_bits(const AppendParams& P, dim3 grid, hipStream_t st) {
  if (P.g.bits == 2) return launch_kg<IO, META, 2, XF>(P, grid, st);
  if (P.g.bits == 4) return launch_kg<IO, META, 4, XF>(P, grid, st);
  return OSCAR_ERR_UNSUPPORTED;
}

template <typename IO, int XF>
int launch_meta(const AppendParams& P, dim3 grid, hipStream_t st) {
  int rc;
  if (P.c.cfg.meta_dtype == OSCAR_F16) {
    rc = launch_bits<IO, __half, XF>(P, grid, st);
    if (rc == OSCAR_OK && !P.c.tickets)
      hipLaunchKernelGGL((oscar_update_lens_kernel<__half>), dim3((P.c.batch + 63) / 64), dim3(64), 0, st, P);
  } else {
    rc = launch_bits<IO, float, XF>(P, grid, st);
    if (rc == OSCAR_OK && !P.c.tickets)
      hipLaunchKernelGGL((oscar_update_lens_kernel<float>), dim3((P.c.batch + 63) / 64), dim3(64), 0, st, P);
  }
  return rc;
}

// Token norms over all kv heads for the new tokens that this call moves into pages
// (pending index r0 <= pi < nq*R): one 16-lane row per token, 16 tokens per workgroup;
// the norm goes into the token's slot of the norm plane of every head's page, where the
// encoder kernel (launched next on the same stream) picks it up.  Tokens that stay in the
// residual window are left to the encoder kernel itself.
template <typename IO, typename META>
__global__ __launch_bounds__(256) void oscar_token_norm_kernel(AppendParams P) {
  const int b = blockIdx.y, tid = threadIdx.x;
  const int row_lane = tid & 15;
  const int cg = channel_group_of_row_lane(row_lane);
  const int Hkv = P.c.cfg.n_kv_heads;
  uint32_t sgn[4];
#pragma unroll
  for (int st = 0; st < 4; ++st) sgn[st] = ((cg >> st) & 1) ? 0x80000000u : 0u;
  const SeqPlan sp = plan_sequence(P, b);
  if (sp.n <= 0 || !sp.ok) return;
  const int t_first = (int)blockIdx.x * 16;         // (signed: n_paged below can be negative)
  const int ti = t_first + (tid >> 4);              // new token of this row
  const int n_paged = sp.nq * R - sp.r0;            // new tokens that go into pages
  if (t_first >= n_paged) return;                   // whole workgroup idle
  const int tc = ti < n_paged ? ti : n_paged - 1;   // whole rows stay active for the exchanges
  const IO* knew = reinterpret_cast<const IO*>(P.k);
  const float nf = token_norm_all_heads<IO, META>(
      knew + (((size_t)b * P.T + (size_t)tc) * Hkv) * D + cg * 8, Hkv, sgn,
      P.c.cfg.rotation == OSCAR_ROTATION_ON);
  if (ti < n_paged) {
    const int pi = sp.r0 + ti;
    const int phys = P.c.block_table[(size_t)b * P.c.max_pages_per_seq + sp.packed_pages + pi / R];
    for (int h = row_lane; h < Hkv; h += 16) {
      META* o = reinterpret_cast<META*>(reinterpret_cast<uint8_t*>(P.c.k_norms) +
                                        ((size_t)phys * Hkv + h) * P.g.k_norms_bytes);
      o[tok_meta_pos(pi % R)] = from_f32<META>(nf);
    }
  }
}

template <typename IO>
int launch_token_norms(const AppendParams& P, hipStream_t st) {
  const dim3 grid((unsigned)((P.T + 15) / 16), (unsigned)P.c.batch);
  if (P.c.cfg.meta_dtype == OSCAR_F16)
    hipLaunchKernelGGL((oscar_token_norm_kernel<IO, __half>), grid, dim3(256), 0, st, P);
  else
    hipLaunchKernelGGL((oscar_token_norm_kernel<IO, float>), grid, dim3(256), 0, st, P);
  return OSCAR_OK;
}

// every instantiation of the encoder for one of the three sets
template <int XF>
int launch_append(const AppendParams& P, dim3 grid, hipStream_t st) {
  switch (P.c.cfg.io_dtype) {
    case OSCAR_F32: return launch_meta<float, XF>(P, grid, st);
    case OSCAR_BF16: return launch_meta<__hip_bfloat16, XF>(P, grid, st);
    case OSCAR_F16: return launch_meta<__half, XF>(P, grid, st);
    default: return OSCAR_ERR_UNSUPPORTED;
  }
}

}  // namespace
