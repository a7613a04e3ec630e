// oscar_quantize_append: Canalized Rotation -> Omni-Token Scaling -> per-channel key
// quantization + per-token value quantization -> bit-packed page write, plus the
// 16-bit residual window (BufferQuantK / BufferQuantV of Algorithm "The OScaR
// algorithm"; key transform of App. "Implementation Details ...", "Overall Design";
// quantizer of Eq. 3-4).
//
// This translation unit is compiled with -ffp-contract=off: the encoder is an
// encoding, and its fp32 operation order is part of the format (codes must not
// depend on whether a multiply-add was fused).
//
// Work decomposition: one workgroup of 256 threads per (sequence, kv head, block of
// R=128 pending tokens).  Thread (slot = tid/16, sub = tid%16) owns channels
// 8*sub..8*sub+7 of token 16*pass+slot for pass = 0..7, so
//   - the 128-point Hadamard butterfly runs 3 stages in registers and 4 stages
//     across the 16 lanes of a token (lane bit s <-> channel bit 3+s),
//   - the token norm is a 16-lane butterfly all-reduce,
//   - per-channel min/max over tokens reduce over passes (registers), over the 4
//     token slots of a wave (lane bits 4,5) and over the 4 waves (LDS),
//   - per-token value min/max reduce over 8 registers and 4|8|16 lanes.
// Codes are staged in LDS as the page image and leave with 16-byte coalesced stores.
#include "oscar_common.h"

namespace {

constexpr int D = OSCAR_D;
constexpr int R = OSCAR_R;
constexpr int VROW_PAD = R + 4;  // LDS row stride (bytes) of the value code bytes

// Staging position of value code (channel c, token t): rows are channels, columns are
// tokens in chunk order (q4 = t%4 major, then k-step, then element), skewed per 32 rows to
// spread LDS banks.
__device__ __forceinline__ int vimg_index(int c, int t) {
  return c * VROW_PAD + (c / 32) * 4 + (t % 4) * 32 + ((t / 4) % 4) * 8 + t / 16;
}

struct AppendParams {
  const void* k;
  const void* v;
  int T;
  const int32_t* new_lens;
  oscar_cache c;
  PageGeom g;
  uint32_t flags;
};

template <typename IO> __device__ __forceinline__ void load8(const IO* p, float (&x)[8]);
template <> __device__ __forceinline__ void load8<float>(const float* p, float (&x)[8]) {
  float4 a = reinterpret_cast<const float4*>(p)[0];
  float4 b = reinterpret_cast<const float4*>(p)[1];
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
  x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
template <> __device__ __forceinline__ void load8<__half>(const __half* p, float (&x)[8]) {
  uint4 r = *reinterpret_cast<const uint4*>(p);
  uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __half2float(__ushort_as_half((unsigned short)(w[i] & 0xffffu)));
    x[2 * i + 1] = __half2float(__ushort_as_half((unsigned short)(w[i] >> 16)));
  }
}
template <> __device__ __forceinline__ void load8<__hip_bfloat16>(const __hip_bfloat16* p,
                                                                  float (&x)[8]) {
  uint4 r = *reinterpret_cast<const uint4*>(p);
  uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __uint_as_float(w[i] << 16);
    x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}

template <typename IO> __device__ __forceinline__ void copy8(IO* dst, const IO* src);
template <> __device__ __forceinline__ void copy8<float>(float* dst, const float* src) {
  reinterpret_cast<float4*>(dst)[0] = reinterpret_cast<const float4*>(src)[0];
  reinterpret_cast<float4*>(dst)[1] = reinterpret_cast<const float4*>(src)[1];
}
template <> __device__ __forceinline__ void copy8<__half>(__half* dst, const __half* src) {
  *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
}
template <>
__device__ __forceinline__ void copy8<__hip_bfloat16>(__hip_bfloat16* dst,
                                                      const __hip_bfloat16* src) {
  *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
}

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

// Key transform of 8 channels of one token held by 16 cooperating lanes:
// K_h = H(k)/sqrt(128), n = ||K_h||_2 rounded to the metadata type, K_u = K_h / n
// rounded to fp16.  Butterfly stage h pairs (i, i|h): lower <- a+b, upper <- a-b.
template <typename META>
__device__ __forceinline__ void key_transform8(float (&x)[8], int sub, float& n_st) {
#pragma unroll
  for (int h = 1; h < 8; h <<= 1) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if ((i & h) == 0) {
        float a = x[i], b = x[i | h];
        x[i] = a + b;
        x[i | h] = a - b;
      }
    }
  }
#pragma unroll
  for (int m = 1; m < 16; m <<= 1) {
    const bool upper = (sub & m) != 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float y = __shfl_xor(x[i], m, 64);
      x[i] = upper ? (y - x[i]) : (x[i] + y);
    }
  }
  const float c = 0.08838834764831845f;  // fp32(1/sqrt(128))
  float t[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    x[i] = x[i] * c;
    t[i] = x[i] * x[i];
  }
  // balanced tree, adjacent pairs first
  float s = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
#pragma unroll
  for (int m = 1; m < 16; m <<= 1) s = s + __shfl_xor(s, m, 64);
  float n = sqrtf(s);
  float nf = round_meta<META>(n);
  float inv = (nf > 0.0f && !isinf(nf)) ? 1.0f / nf : 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = __half2float(__float2half_rn(pin_f32(x[i] * inv)));
  n_st = nf;
}

// Eq. 3-4 parameters of one group, rounded to storage before use.
template <typename META, int BITS>
__device__ __forceinline__ void quant_params(float mn, float mx, float& df, float& rd, float& z) {
  const float qmax = (float)((1 << BITS) - 1);
  float dl = (mx - mn) / qmax;
  df = round_meta<META>(dl);
  if (df == 0.0f) {
    df = round_meta<META>(fabsf(mn));
    if (df == 0.0f || isinf(df)) df = 1.0f;
  }
  rd = 1.0f / df;
  z = round_meta<META>(rintf(-mn * rd));
}

template <int BITS> __device__ __forceinline__ uint32_t quant_code(float x, float rd, float z) {
  const float qmax = (float)((1 << BITS) - 1);
  float c = rintf(x * rd) + z;
  c = fminf(fmaxf(c, 0.0f), qmax);
  return (uint32_t)c;
}

template <typename M> __device__ __forceinline__ void store_meta8(M* dst, const float (&v)[8]);
template <> __device__ __forceinline__ void store_meta8<float>(float* dst, const float (&v)[8]) {
  reinterpret_cast<float4*>(dst)[0] = make_float4(v[0], v[1], v[2], v[3]);
  reinterpret_cast<float4*>(dst)[1] = make_float4(v[4], v[5], v[6], v[7]);
}
template <> __device__ __forceinline__ void store_meta8<__half>(__half* dst, const float (&v)[8]) {
  uint4 o;
  o.x = half_bits(v[0]) | (half_bits(v[1]) << 16);
  o.y = half_bits(v[2]) | (half_bits(v[3]) << 16);
  o.z = half_bits(v[4]) | (half_bits(v[5]) << 16);
  o.w = half_bits(v[6]) | (half_bits(v[7]) << 16);
  *reinterpret_cast<uint4*>(dst) = o;
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

template <typename IO, typename META, int BITS, int KG>
__global__ __launch_bounds__(256) void oscar_append_kernel(AppendParams P) {
  constexpr int NGK = R / KG;        // key groups per page
  constexpr int PPG = KG / 16;       // passes per key group

  __shared__ float s_red[NGK][4][D][2];
  __shared__ __align__(16) uint8_t s_kimg[R * D * BITS / 8];     // key-code page image
  __shared__ __align__(16) uint8_t s_vimg[D * VROW_PAD + 64];    // value codes, one per byte
  __shared__ __align__(16) META s_vmeta[2][4][R];
  __shared__ __align__(16) META s_norm[R];

  const int b = blockIdx.z, kvh = blockIdx.y, blk = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int slot = tid >> 4, sub = tid & 15;
  const int Hkv = P.c.cfg.n_kv_heads;

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

  const IO* knew = reinterpret_cast<const IO*>(P.k);
  const IO* vnew = reinterpret_cast<const IO*>(P.v);
  const size_t res_base = ((size_t)b * Hkv + kvh) * R;
  __half* res_k = reinterpret_cast<__half*>(P.c.res_k) + res_base * D;
  IO* res_v = reinterpret_cast<IO*>(P.c.res_v) + res_base * D;
  META* res_norm = reinterpret_cast<META*>(P.c.res_norm) + res_base;

  // ---- phase 1: gather the block (old residual tokens first, then new tokens) ----
  float u[8][8], vv[8][8], nrm[8];
  if (do_block) {
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int pi = blk * R + p * 16 + slot;  // index among pending tokens
      if (pi < sp.r0) {
        load8<__half>(res_k + (size_t)pi * D + sub * 8, u[p]);
        nrm[p] = to_f32<META>(res_norm[pi]);
        load8<IO>(res_v + (size_t)pi * D + sub * 8, vv[p]);
      } else {
        const size_t ti = (size_t)(pi - sp.r0);
        const size_t off = (((size_t)b * P.T + ti) * Hkv + kvh) * D + sub * 8;
        load8<IO>(knew + off, u[p]);
        load8<IO>(vnew + off, vv[p]);
      }
    }
    // the branch above is uniform per 16-lane token group; transform where needed
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int pi = blk * R + p * 16 + slot;
      float x[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) x[i] = u[p][i];
      float nn;
      key_transform8<META>(x, sub, nn);
      if (pi >= sp.r0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) u[p][i] = x[i];
        nrm[p] = nn;
      }
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
      const size_t off = (((size_t)b * P.T + (size_t)(src0 + ic)) * Hkv + kvh) * D + sub * 8;
      float x[8], nn;
      load8<IO>(knew + off, x);
      key_transform8<META>(x, sub, nn);
      if (i < cnt) {
        const int ds = dst0 + i;
        uint4 o;
        o.x = half_bits(x[0]) | (half_bits(x[1]) << 16);
        o.y = half_bits(x[2]) | (half_bits(x[3]) << 16);
        o.z = half_bits(x[4]) | (half_bits(x[5]) << 16);
        o.w = half_bits(x[6]) | (half_bits(x[7]) << 16);
        *reinterpret_cast<uint4*>(res_k + (size_t)ds * D + sub * 8) = o;
        copy8<IO>(res_v + (size_t)ds * D + sub * 8, vnew + off);
        if (sub == 0) res_norm[ds] = from_f32<META>(nn);
      }
    }
  }
  if (!do_block) break;

  // ---- phase 3: quantize the block held in registers ----
  const int logical_page = sp.packed_pages + blk;
  const int phys = P.c.block_table[(size_t)b * P.c.max_pages_per_seq + logical_page];
  const size_t pg = (size_t)phys * Hkv + kvh;
  uint8_t* o_kcodes = reinterpret_cast<uint8_t*>(P.c.k_codes) + pg * P.g.k_codes_bytes;
  META* o_kmeta = reinterpret_cast<META*>(reinterpret_cast<uint8_t*>(P.c.k_meta) + pg * P.g.k_meta_bytes);
  META* o_knorm = reinterpret_cast<META*>(reinterpret_cast<uint8_t*>(P.c.k_norms) + pg * P.g.k_norms_bytes);
  uint8_t* o_vcodes = reinterpret_cast<uint8_t*>(P.c.v_codes) + pg * P.g.v_codes_bytes;
  META* o_vmeta = reinterpret_cast<META*>(reinterpret_cast<uint8_t*>(P.c.v_meta) + pg * P.g.v_meta_bytes);

  // keys: per-channel min/max over the tokens of each group
#pragma unroll
  for (int gk = 0; gk < NGK; ++gk) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float mn = u[gk * PPG][e], mx = mn;
#pragma unroll
      for (int p = 1; p < PPG; ++p) {
        mn = fminf(mn, u[gk * PPG + p][e]);
        mx = fmaxf(mx, u[gk * PPG + p][e]);
      }
      mn = fminf(mn, __shfl_xor(mn, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mn = fminf(mn, __shfl_xor(mn, 32, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      if (lane < 16) {
        s_red[gk][wave][sub * 8 + e][0] = mn;
        s_red[gk][wave][sub * 8 + e][1] = mx;
      }
    }
  }
  if (sub == 0) {
#pragma unroll
    for (int p = 0; p < 8; ++p) s_norm[tok_meta_pos(p * 16 + slot)] = from_f32<META>(nrm[p]);
  }
  __syncthreads();

#pragma unroll
  for (int gk = 0; gk < NGK; ++gk) {
    float dfa[8], za[8], rda[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float mn = s_red[gk][0][sub * 8 + e][0], mx = s_red[gk][0][sub * 8 + e][1];
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        mn = fminf(mn, s_red[gk][w][sub * 8 + e][0]);
        mx = fmaxf(mx, s_red[gk][w][sub * 8 + e][1]);
      }
      quant_params<META, BITS>(mn, mx, dfa[e], rda[e], za[e]);
    }
    if (slot == 0) {
      // Delta / zero in operand order (see kmeta_pos_of_chan)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int pos = kmeta_pos_of_chan(BITS, sub * 8 + e);
        o_kmeta[(size_t)gk * D + pos] = from_f32<META>(dfa[e]);
        o_kmeta[(size_t)(NGK + gk) * D + pos] = from_f32<META>(za[e]);
      }
    }
#pragma unroll
    for (int p = gk * PPG; p < (gk + 1) * PPG; ++p) {
      uint32_t w = 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) w |= quant_code<BITS>(u[p][e], rda[e], za[e]) << (e * BITS);
      const int tok = p * 16 + slot;
      // chunk (tile = tok/16, n = tok%16, q4 = sub/4); this thread's 8 codes are numbers
      // 8*(sub%4) .. +7 of the chunk
      const int off = chunk_offset(BITS, tok / 16, tok % 16, sub / 4) + (sub % 4) * BITS;
      if (BITS == 2) {
        *reinterpret_cast<uint16_t*>(&s_kimg[off]) = (uint16_t)w;
      } else {
        *reinterpret_cast<uint32_t*>(&s_kimg[off]) = w;
      }
    }
  }

  // values: per-token min/max over each group of v_group channels
  const int lanes_per_vgroup = P.g.v_group / 8;  // 4, 8 or 16
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    float mn = vv[p][0], mx = mn;
#pragma unroll
    for (int e = 1; e < 8; ++e) {
      mn = fminf(mn, vv[p][e]);
      mx = fmaxf(mx, vv[p][e]);
    }
    for (int m = 1; m < lanes_per_vgroup; m <<= 1) {
      mn = fminf(mn, __shfl_xor(mn, m, 64));
      mx = fmaxf(mx, __shfl_xor(mx, m, 64));
    }
    float df, rd, z;
    quant_params<META, BITS>(mn, mx, df, rd, z);
    const int tok = p * 16 + slot;
    if ((sub & (lanes_per_vgroup - 1)) == 0) {
      const int gv = sub / lanes_per_vgroup;
      s_vmeta[0][gv][tok_meta_pos(tok)] = from_f32<META>(df);
      s_vmeta[1][gv][tok_meta_pos(tok)] = from_f32<META>(z);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e)
      s_vimg[vimg_index(sub * 8 + e, tok)] = (uint8_t)quant_code<BITS>(vv[p][e], rd, z);
  }
  __syncthreads();

  // ---- phase 4: coalesced page stores ----
  {
    const uint4* src = reinterpret_cast<const uint4*>(&s_kimg[0]);
    uint4* dst = reinterpret_cast<uint4*>(o_kcodes);
    constexpr int NV = R * D * BITS / 8 / 16;  // uint4 count: 256 (2-bit) or 512 (4-bit)
#pragma unroll
    for (int i = tid; i < NV; i += 256) dst[i] = src[i];
  }
  {
    // thread = (tile pair tp, n, q4): packs the chunks of channels 32*tp+n and 32*tp+16+n
    const int tp = tid >> 6, n = (tid >> 2) & 15, q4 = tid & 3;
    uint32_t outw[2][BITS];  // [channel of the pair][dword of the chunk]
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
      const int c = 32 * tp + 16 * cc + n;
      const uint32_t* row = reinterpret_cast<const uint32_t*>(&s_vimg[vimg_index(c, q4)]);
#pragma unroll
      for (int d = 0; d < BITS; ++d) outw[cc][d] = 0;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        // bytes of elements e = 0..3 and e = 4..7 of k-step kk
        const uint32_t x0 = row[2 * kk], x1 = row[2 * kk + 1];
        if (BITS == 2) {
          const uint32_t ev = (x0 & 3u) | (((x0 >> 16) & 3u) << 2) | ((x1 & 3u) << 4) |
                              (((x1 >> 16) & 3u) << 6);
          const uint32_t od = ((x0 >> 8) & 3u) | (((x0 >> 24) & 3u) << 2) |
                              (((x1 >> 8) & 3u) << 4) | (((x1 >> 24) & 3u) << 6);
          // even elements -> code numbers 4*(kk%2)+r, odd elements -> 8 more
          outw[cc][kk / 2] |= (ev << (8 * (kk % 2))) | (od << (16 + 8 * (kk % 2)));
        } else {
          const uint32_t ev = (x0 & 15u) | (((x0 >> 16) & 15u) << 4) | ((x1 & 15u) << 8) |
                              (((x1 >> 16) & 15u) << 12);
          const uint32_t od = ((x0 >> 8) & 15u) | (((x0 >> 24) & 15u) << 4) |
                              (((x1 >> 8) & 15u) << 8) | (((x1 >> 24) & 15u) << 12);
          outw[cc][kk] = ev | (od << 16);
        }
      }
    }
    uint8_t* dst = o_vcodes + (size_t)tid * 2 * chunk_bytes(BITS);
    if (BITS == 2) {
      *reinterpret_cast<uint4*>(dst) = make_uint4(outw[0][0], outw[0][1], outw[1][0], outw[1][1]);
    } else {
      reinterpret_cast<uint4*>(dst)[0] = make_uint4(outw[0][0], outw[0][1], outw[0][2], outw[0][3]);
      reinterpret_cast<uint4*>(dst)[1] = make_uint4(outw[1][0], outw[1][1], outw[1][2], outw[1][3]);
    }
  }
  {
    // value metadata image: Delta[ngv][R] then zero[ngv][R]
    const int ngv = P.g.ngv;
    const int per_plane = ngv * R;  // elements
    for (int i = tid; i < 2 * per_plane; i += 256) {
      const int plane = i / per_plane, rest = i - plane * per_plane;
      o_vmeta[i] = s_vmeta[plane][rest / R][rest % R];
    }
    if (tid < R) o_knorm[tid] = s_norm[tid];
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

template <typename IO, typename META, int BITS>
int launch_kg(const AppendParams& P, dim3 grid, hipStream_t st) {
  switch (P.g.k_group) {
    case 32: hipLaunchKernelGGL((oscar_append_kernel<IO, META, BITS, 32>), grid, dim3(256), 0, st, P); break;
    case 64: hipLaunchKernelGGL((oscar_append_kernel<IO, META, BITS, 64>), grid, dim3(256), 0, st, P); break;
    case 128: hipLaunchKernelGGL((oscar_append_kernel<IO, META, BITS, 128>), grid, dim3(256), 0, st, P); break;
    default: return OSCAR_ERR_UNSUPPORTED;
  }
  return OSCAR_OK;
}

template <typename IO, typename META>
int launch_bits(const AppendParams& P, dim3 grid, hipStream_t st) {
  if (P.g.bits == 2) return launch_kg<IO, META, 2>(P, grid, st);
  if (P.g.bits == 4) return launch_kg<IO, META, 4>(P, grid, st);
  return OSCAR_ERR_UNSUPPORTED;
}

template <typename IO>
int launch_meta(const AppendParams& P, dim3 grid, hipStream_t st) {
  int rc;
  if (P.c.cfg.meta_dtype == OSCAR_F16) {
    rc = launch_bits<IO, __half>(P, grid, st);
    if (rc == OSCAR_OK && !P.c.tickets)
      hipLaunchKernelGGL((oscar_update_lens_kernel<__half>), dim3((P.c.batch + 63) / 64), dim3(64), 0, st, P);
  } else {
    rc = launch_bits<IO, float>(P, grid, st);
    if (rc == OSCAR_OK && !P.c.tickets)
      hipLaunchKernelGGL((oscar_update_lens_kernel<float>), dim3((P.c.batch + 63) / 64), dim3(64), 0, st, P);
  }
  return rc;
}

}  // namespace

extern "C" int oscar_quantize_append(const void* k, const void* v, int32_t T,
                                     const int32_t* new_lens, oscar_cache* cache,
                                     int32_t max_seq_len_hint, uint32_t flags, void* stream) {
  if (!cache) return OSCAR_ERR_INVALID_ARG;
  int rc = oscar_validate_config(&cache->cfg);
  if (rc != OSCAR_OK) return rc;
  if (T < 0 || cache->batch <= 0 || cache->max_pages_per_seq <= 0 || cache->num_pages <= 0)
    return OSCAR_ERR_INVALID_ARG;
  if (T == 0) return OSCAR_OK;
  if (!k || !v || !cache->k_codes || !cache->k_meta || !cache->k_norms || !cache->v_codes ||
      !cache->v_meta || !cache->res_k || !cache->res_v || !cache->res_norm ||
      !cache->block_table || !cache->seq_lens || !cache->res_lens)
    return OSCAR_ERR_INVALID_ARG;
  if (flags & ~(uint32_t)OSCAR_APPEND_EAGER) return OSCAR_ERR_INVALID_ARG;
  if (max_seq_len_hint >= 0) {
    // pages needed if the longest sequence takes all T tokens (a full residual may stay 16-bit)
    const long long total = (long long)max_seq_len_hint + T;
    const long long pages = (flags & OSCAR_APPEND_EAGER) ? total / R : (total - 1) / R;
    if (pages > cache->max_pages_per_seq) return OSCAR_ERR_CAPACITY;
  }
  AppendParams P;
  P.k = k;
  P.v = v;
  P.T = T;
  P.new_lens = new_lens;
  P.c = *cache;
  P.g = make_geom(cache->cfg.bits, cache->cfg.k_group, cache->cfg.v_group, cache->cfg.meta_dtype);
  P.flags = flags;
  const int nblk = (R + T) / R;  // a sequence completes at most this many blocks
  dim3 grid(nblk, cache->cfg.n_kv_heads, cache->batch);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  switch (cache->cfg.io_dtype) {
    case OSCAR_F32: rc = launch_meta<float>(P, grid, st); break;
    case OSCAR_BF16: rc = launch_meta<__hip_bfloat16>(P, grid, st); break;
    case OSCAR_F16: rc = launch_meta<__half>(P, grid, st); break;
    default: return OSCAR_ERR_UNSUPPORTED;
  }
  if (rc != OSCAR_OK) return rc;
  if (hipGetLastError() != hipSuccess) return OSCAR_ERR_HIP;
  return OSCAR_OK;
}
