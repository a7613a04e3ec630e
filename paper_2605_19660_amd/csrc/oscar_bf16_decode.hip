// 16-bit comparator: split-K decode attention softmax(q K^T) V on an uncompressed,
// un-rotated cache, token-major [batch][tokens][kv heads][128] or head-major
// [batch][kv heads][tokens][128] (the BF16 FlashDecoding-style baseline of the paper's
// efficiency section).  Same split / partial / reduce skeleton as the compressed path,
// 512 bytes per token and kv head.
//
// A 16-lane DPP row owns a token at a time (lane = 8 channels, the query slice of every head
// of the group in registers), walks tokens row, row+16, ... of the split with its own online
// softmax state, four tokens per step and the next four already in flight; logits reduce
// inside the row, nothing is shared until the 16 row states merge through LDS at the end.
// With a head-major cache a wave's four rows read 1 KB of consecutive memory per load.
#include <string.h>

#include "oscar_common.h"

namespace {

__device__ __forceinline__ uint4 load_stream16(const void* p) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}


constexpr int D = OSCAR_D;
constexpr int WS_STRIDE = D + 2;
constexpr int TOK_STEP = 4;   // tokens per row and step

struct PlainParams {
  const void* q;
  const void* k;
  const void* v;
  const int32_t* seq_lens;
  float* ws;
  int batch, S, Hq, Hkv, num_splits;
  int head_major;   // 0: [batch][tokens][kv heads][d], 1: [batch][kv heads][tokens][d]
  float qk_scale_log2;
};

template <typename T> __device__ __forceinline__ float cvt16(uint32_t bits16);
template <> __device__ __forceinline__ float cvt16<__hip_bfloat16>(uint32_t b) {
  return __uint_as_float(b << 16);
}
template <> __device__ __forceinline__ float cvt16<__half>(uint32_t b) {
  return __half2float(__ushort_as_half((unsigned short)b));
}
template <typename T> __device__ __forceinline__ void widen8(const uint4& r, float (&x)[8]) {
  const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = cvt16<T>(w[i] & 0xffffu);
    x[2 * i + 1] = cvt16<T>(w[i] >> 16);
  }
}

template <int CTRL> __device__ __forceinline__ float dpp_get(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
// sum over the 16 lanes of a DPP row; every lane ends with the total
__device__ __forceinline__ float row_sum16(float v) {
  v += dpp_get<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_get<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_get<0x141>(v);  // row_half_mirror
  v += dpp_get<0x140>(v);  // row_mirror
  return v;
}

template <typename T, int GQ>
__global__ __launch_bounds__(256) void oscar_plain_decode_partial_kernel(PlainParams P) {
  __shared__ float s_m[16][GQ], s_l[16][GQ];
  __shared__ __align__(16) float s_o[16][GQ][D];

  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, row = tid >> 4, n = tid & 15;
  const int len = min(P.seq_lens ? P.seq_lens[b] : P.S, P.S);
  // token range of this split, in multiples of 64
  const int per_split = ((len + P.num_splits - 1) / P.num_splits + 63) & ~63;
  const int tok0 = split * per_split, tok1 = min(len, tok0 + per_split);

  // query slices, scaled: channels 8n..8n+7 of every head of the group
  float qf[GQ][8];
#pragma unroll
  for (int h = 0; h < GQ; ++h) {
    const uint4 raw = *reinterpret_cast<const uint4*>(
        reinterpret_cast<const uint16_t*>(P.q) + ((size_t)b * P.Hq + (size_t)kvh * GQ + h) * D + 8 * n);
    widen8<T>(raw, qf[h]);
#pragma unroll
    for (int c = 0; c < 8; ++c) qf[h][c] *= P.qk_scale_log2;
  }
  float m[GQ], l[GQ], o[GQ][8];
#pragma unroll
  for (int h = 0; h < GQ; ++h) {
    m[h] = -INFINITY;
    l[h] = 0.0f;
#pragma unroll
    for (int c = 0; c < 8; ++c) o[h][c] = 0.0f;
  }

  if (tok0 < tok1) {
    const uint8_t* kbase = reinterpret_cast<const uint8_t*>(P.k);
    const uint8_t* vbase = reinterpret_cast<const uint8_t*>(P.v);
    // bytes between consecutive tokens of one kv head, and offset of this stream
    const size_t row_stride = P.head_major ? (size_t)D * 2 : (size_t)P.Hkv * D * 2;
    const size_t seq_off = (P.head_major ? ((size_t)b * P.Hkv + kvh) * P.S * D * 2
                                         : ((size_t)b * P.S * P.Hkv + kvh) * D * 2) + n * 16;
    // this row's tokens: tok0 + row + 16 * i; positions past the end are read from the last
    // valid token and masked
    auto load_step = [&](int t_first, uint4 (&kr)[TOK_STEP], uint4 (&vr)[TOK_STEP]) {
#pragma unroll
      for (int j = 0; j < TOK_STEP; ++j) {
        const int t = min(t_first + 16 * j, tok1 - 1);
        // (read once per launch: non-temporal loads, as in the packed-cache kernel)
        kr[j] = load_stream16(kbase + seq_off + (size_t)t * row_stride);
        vr[j] = load_stream16(vbase + seq_off + (size_t)t * row_stride);
      }
    };
    uint4 kcur[TOK_STEP], vcur[TOK_STEP];
    load_step(tok0 + row, kcur, vcur);
    // uniform trip count for the workgroup (rows past their tokens run masked steps)
    for (int t_first = tok0 + row; t_first - row < tok1; t_first += 16 * TOK_STEP) {
      uint4 knext[TOK_STEP], vnext[TOK_STEP];
      load_step(t_first + 16 * TOK_STEP, knext, vnext);   // clamped: harmless past the end
      float sc[GQ][TOK_STEP];
#pragma unroll
      for (int j = 0; j < TOK_STEP; ++j) {
        float kv[8];
        widen8<T>(kcur[j], kv);
        const bool valid = t_first + 16 * j < tok1;
#pragma unroll
        for (int h = 0; h < GQ; ++h) {
          float acc = qf[h][0] * kv[0];
#pragma unroll
          for (int c = 1; c < 8; ++c) acc = fmaf(qf[h][c], kv[c], acc);
          sc[h][j] = valid ? row_sum16(acc) : -INFINITY;
        }
      }
      float pw[GQ][TOK_STEP];
#pragma unroll
      for (int h = 0; h < GQ; ++h) {
        float m_new = m[h];
#pragma unroll
        for (int j = 0; j < TOK_STEP; ++j) m_new = fmaxf(m_new, sc[h][j]);
        const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m[h] - m_safe);
        m[h] = m_new;
        l[h] *= alpha;
#pragma unroll
        for (int c = 0; c < 8; ++c) o[h][c] *= alpha;
#pragma unroll
        for (int j = 0; j < TOK_STEP; ++j) {
          pw[h][j] = __builtin_amdgcn_exp2f(sc[h][j] - m_safe);
          l[h] += pw[h][j];
        }
      }
#pragma unroll
      for (int j = 0; j < TOK_STEP; ++j) {
        float vv[8];
        widen8<T>(vcur[j], vv);
#pragma unroll
        for (int h = 0; h < GQ; ++h)
#pragma unroll
          for (int c = 0; c < 8; ++c) o[h][c] = fmaf(pw[h][j], vv[c], o[h][c]);
      }
#pragma unroll
      for (int j = 0; j < TOK_STEP; ++j) {
        kcur[j] = knext[j];
        vcur[j] = vnext[j];
      }
    }
  }

  // merge the 16 row states and write the partial record
#pragma unroll
  for (int h = 0; h < GQ; ++h) {
    *reinterpret_cast<float4*>(&s_o[row][h][8 * n]) = make_float4(o[h][0], o[h][1], o[h][2], o[h][3]);
    *reinterpret_cast<float4*>(&s_o[row][h][8 * n + 4]) = make_float4(o[h][4], o[h][5], o[h][6], o[h][7]);
    if (n == 0) {
      s_m[row][h] = m[h];
      s_l[row][h] = l[h];
    }
  }
  __syncthreads();
  for (int i = tid; i < GQ * D; i += 256) {
    const int h = i / D, c = i % D;
    float M = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) M = fmaxf(M, s_m[r][h]);
    float tot = 0.0f, L = 0.0f;
    if (M != -INFINITY) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float w = (s_m[r][h] == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(s_m[r][h] - M);
        tot = fmaf(s_o[r][h][c], w, tot);
        L = fmaf(s_l[r][h], w, L);
      }
    }
    const size_t rec = ((size_t)b * P.Hq + (size_t)kvh * GQ + h) * P.num_splits + split;
    P.ws[rec * WS_STRIDE + c] = tot;
    if (c == 0) {
      P.ws[rec * WS_STRIDE + D] = M;
      P.ws[rec * WS_STRIDE + D + 1] = L;
    }
  }
}

template <typename T>
int launch_plain(const PlainParams& P, int gq, dim3 grid, hipStream_t st) {
  switch (gq) {
#define OSCAR_CASE(G) \
  case G: hipLaunchKernelGGL((oscar_plain_decode_partial_kernel<T, G>), grid, dim3(256), 0, st, P); break;
    OSCAR_CASE(1) OSCAR_CASE(2) OSCAR_CASE(3) OSCAR_CASE(4)
    OSCAR_CASE(5) OSCAR_CASE(6) OSCAR_CASE(7) OSCAR_CASE(8)
#undef OSCAR_CASE
    default: return OSCAR_ERR_UNSUPPORTED;
  }
  return OSCAR_OK;
}

}  // namespace

extern "C" int oscar_bf16_decode_attn(const void* q, const void* k, const void* v,
                                      const int32_t* seq_lens, void* out, int32_t dtype,
                                      int32_t out_dtype, int32_t batch, int32_t kv_stride_tokens,
                                      int32_t kv_layout, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                      float softmax_scale, int32_t max_seq_len_hint,
                                      int32_t num_splits, void* workspace, size_t workspace_bytes,
                                      void* stream) {
  if (!q || !k || !v || !out) return OSCAR_ERR_INVALID_ARG;
  if (batch <= 0 || kv_stride_tokens <= 0 || n_q_heads <= 0 || n_kv_heads <= 0 ||
      n_q_heads % n_kv_heads != 0 || num_splits < 0 || num_splits > 512 || max_seq_len_hint < 0)
    return OSCAR_ERR_INVALID_ARG;
  if (kv_layout != OSCAR_KV_TOKEN_MAJOR && kv_layout != OSCAR_KV_HEAD_MAJOR) return OSCAR_ERR_INVALID_ARG;
  if (dtype != OSCAR_BF16 && dtype != OSCAR_F16) return OSCAR_ERR_UNSUPPORTED;
  if (out_dtype != OSCAR_F32 && out_dtype != dtype) return OSCAR_ERR_INVALID_ARG;
  if (head_dim != OSCAR_D || n_q_heads / n_kv_heads > OSCAR_MAX_GQA) return OSCAR_ERR_UNSUPPORTED;
  oscar_config cfg;
  memset(&cfg, 0, sizeof(cfg));
  cfg.head_dim = head_dim;
  cfg.n_q_heads = n_q_heads;
  cfg.n_kv_heads = n_kv_heads;
  if (num_splits == 0) {
    const int hint = max_seq_len_hint > 0 ? max_seq_len_hint : kv_stride_tokens;
    num_splits = oscar_decode_auto_splits(&cfg, batch, hint);
  }
  const size_t need = oscar_decode_workspace_bytes(&cfg, batch, num_splits);
  if (!workspace || workspace_bytes < need) return OSCAR_ERR_WORKSPACE;
  PlainParams P;
  P.q = q; P.k = k; P.v = v; P.seq_lens = seq_lens;
  P.ws = reinterpret_cast<float*>(workspace);
  P.batch = batch; P.S = kv_stride_tokens; P.Hq = n_q_heads; P.Hkv = n_kv_heads;
  P.num_splits = num_splits;
  P.head_major = (kv_layout == OSCAR_KV_HEAD_MAJOR) ? 1 : 0;
  const float scale = softmax_scale > 0.0f ? softmax_scale : 0.08838834764831845f;
  P.qk_scale_log2 = scale * 1.4426950408889634f;
  dim3 grid(num_splits, n_kv_heads, batch);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const int gq = n_q_heads / n_kv_heads;
  int rc = (dtype == OSCAR_BF16) ? launch_plain<__hip_bfloat16>(P, gq, grid, st)
                                 : launch_plain<__half>(P, gq, grid, st);
  if (rc != OSCAR_OK) return rc;
  oscar_launch_decode_reduce(P.ws, out, num_splits, out_dtype, n_q_heads, batch, st);
  if (hipGetLastError() != hipSuccess) return OSCAR_ERR_HIP;
  return OSCAR_OK;
}
