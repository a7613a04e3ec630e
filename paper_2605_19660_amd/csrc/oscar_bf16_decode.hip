// 16-bit comparator: split-K decode attention softmax(q K^T) V on an uncompressed,
// un-rotated cache, token-major [batch][tokens][kv heads][128] or head-major
// [batch][kv heads][tokens][128] (the BF16 FlashDecoding-style baseline of the paper's
// efficiency section).  Same split / partial / reduce
// skeleton as the compressed path, 512 bytes per token and kv head.
//
// Tile = 64 tokens.  Keys go global -> LDS with 16-byte coalesced loads (padded rows),
// 4 lanes share a token for the dot products; values are read straight from global,
// 32 lanes x 8 bytes per token row, 8 token phases reduced through LDS at the end.
#include <string.h>

#include "oscar_common.h"

namespace {

constexpr int D = OSCAR_D;
constexpr int TILE = 64;
constexpr int KROW = D * 2 + 16;  // padded LDS row, bytes
constexpr int WS_STRIDE = D + 2;

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

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

template <typename T, int GQ>
__global__ __launch_bounds__(256) void oscar_plain_decode_partial_kernel(PlainParams P) {
  __shared__ __align__(16) uint8_t s_k[TILE][KROW];
  __shared__ __align__(16) float s_q[GQ][D];
  __shared__ __align__(16) float s_S[GQ][TILE];
  __shared__ float s_m[GQ], s_l[GQ], s_alpha[GQ];
  __shared__ __align__(16) float s_o[8][GQ][D];

  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int len = min(P.seq_lens ? P.seq_lens[b] : P.S, P.S);
  const int n_tiles = (len + TILE - 1) / TILE;
  const int tps = (n_tiles + P.num_splits - 1) / P.num_splits;
  const int t0 = split * tps, t1 = min(n_tiles, t0 + tps);

  for (int i = tid; i < GQ * D; i += 256) {
    const uint16_t raw = reinterpret_cast<const uint16_t*>(P.q)[((size_t)b * P.Hq + (size_t)kvh * GQ) * D + i];
    s_q[i / D][i % D] = cvt16<T>(raw) * P.qk_scale_log2;
  }
  if (tid < GQ) {
    s_m[tid] = -INFINITY;
    s_l[tid] = 0.0f;
  }
  float o[GQ][4];
#pragma unroll
  for (int h = 0; h < GQ; ++h)
#pragma unroll
    for (int e = 0; e < 4; ++e) o[h][e] = 0.0f;
  __syncthreads();

  const uint8_t* kbase = reinterpret_cast<const uint8_t*>(P.k);
  const uint8_t* vbase = reinterpret_cast<const uint8_t*>(P.v);
  // bytes between consecutive tokens of one kv head, and offset of this stream
  const size_t row_stride = P.head_major ? (size_t)D * 2 : (size_t)P.Hkv * D * 2;
  const size_t seq_off = P.head_major ? ((size_t)b * P.Hkv + kvh) * P.S * D * 2
                                      : ((size_t)b * P.S * P.Hkv + kvh) * D * 2;

  const int tok = tid >> 2, quarter = tid & 3;  // logits: 4 lanes per token
  const int c4 = tid & 31, tg = tid >> 5;       // values: 4 channels per lane, 8 token phases

  for (int tile = t0; tile < t1; ++tile) {
    const int base = tile * TILE;
    // keys -> LDS (1024 x 16 bytes)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * 256;
      const int t = idx >> 4, part = idx & 15;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (base + t < len)
        val = *reinterpret_cast<const uint4*>(kbase + seq_off + (size_t)(base + t) * row_stride + part * 16);
      *reinterpret_cast<uint4*>(&s_k[t][part * 16]) = val;
    }
    // values: issue early, 8 token rows x 8 bytes
    uint2 vraw[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int t = tg + 8 * i;
      vraw[i] = make_uint2(0, 0);
      if (base + t < len)
        vraw[i] = *reinterpret_cast<const uint2*>(vbase + seq_off + (size_t)(base + t) * row_stride + c4 * 8);
    }
    __syncthreads();
    {
      float acc[GQ];
#pragma unroll
      for (int h = 0; h < GQ; ++h) acc[h] = 0.0f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint4 raw = *reinterpret_cast<const uint4*>(&s_k[tok][quarter * 64 + i * 16]);
        const uint32_t wds[4] = {raw.x, raw.y, raw.z, raw.w};
        float kv[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          kv[2 * e] = cvt16<T>(wds[e] & 0xffffu);
          kv[2 * e + 1] = cvt16<T>(wds[e] >> 16);
        }
        const int j = quarter * 32 + i * 8;
#pragma unroll
        for (int h = 0; h < GQ; ++h) {
          const float4 qa = *reinterpret_cast<const float4*>(&s_q[h][j]);
          const float4 qb = *reinterpret_cast<const float4*>(&s_q[h][j + 4]);
          acc[h] = fmaf(qa.x, kv[0], acc[h]);
          acc[h] = fmaf(qa.y, kv[1], acc[h]);
          acc[h] = fmaf(qa.z, kv[2], acc[h]);
          acc[h] = fmaf(qa.w, kv[3], acc[h]);
          acc[h] = fmaf(qb.x, kv[4], acc[h]);
          acc[h] = fmaf(qb.y, kv[5], acc[h]);
          acc[h] = fmaf(qb.z, kv[6], acc[h]);
          acc[h] = fmaf(qb.w, kv[7], acc[h]);
        }
      }
#pragma unroll
      for (int h = 0; h < GQ; ++h) {
        float tot = acc[h] + __shfl_xor(acc[h], 1, 64);
        tot += __shfl_xor(tot, 2, 64);
        if (quarter == 0) s_S[h][tok] = (base + tok < len) ? tot : -INFINITY;
      }
    }
    __syncthreads();
    for (int h = wave; h < GQ; h += 4) {
      const float s0 = s_S[h][lane];
      const float m_old = s_m[h];
      const float m_new = fmaxf(m_old, wave_max(s0));
      const float alpha = exp2f(m_old - m_new);
      const float p0 = exp2f(s0 - m_new);
      const float sum = wave_sum(p0);
      s_S[h][lane] = p0;
      if (lane == 0) {
        s_m[h] = m_new;
        s_l[h] = s_l[h] * alpha + sum;
        s_alpha[h] = alpha;
      }
    }
    __syncthreads();
    {
#pragma unroll
      for (int h = 0; h < GQ; ++h) {
        const float al = s_alpha[h];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[h][e] *= al;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int t = tg + 8 * i;
        const float v0 = cvt16<T>(vraw[i].x & 0xffffu), v1 = cvt16<T>(vraw[i].x >> 16);
        const float v2 = cvt16<T>(vraw[i].y & 0xffffu), v3 = cvt16<T>(vraw[i].y >> 16);
#pragma unroll
        for (int h = 0; h < GQ; ++h) {
          const float p = s_S[h][t];
          o[h][0] = fmaf(p, v0, o[h][0]);
          o[h][1] = fmaf(p, v1, o[h][1]);
          o[h][2] = fmaf(p, v2, o[h][2]);
          o[h][3] = fmaf(p, v3, o[h][3]);
        }
      }
    }
    __syncthreads();
  }

  // reduce the 8 token phases and write the partial record
#pragma unroll
  for (int h = 0; h < GQ; ++h)
    *reinterpret_cast<float4*>(&s_o[tg][h][c4 * 4]) = make_float4(o[h][0], o[h][1], o[h][2], o[h][3]);
  __syncthreads();
  for (int i = tid; i < GQ * D; i += 256) {
    const int h = i / D, c = i % D;
    float tot = 0.0f;
#pragma unroll
    for (int g = 0; g < 8; ++g) tot += s_o[g][h][c];
    const size_t rec = ((size_t)b * P.Hq + (size_t)kvh * GQ + h) * P.num_splits + split;
    P.ws[rec * WS_STRIDE + c] = tot;
  }
  if (tid < GQ) {
    const size_t rec = ((size_t)b * P.Hq + (size_t)kvh * GQ + tid) * P.num_splits + split;
    P.ws[rec * WS_STRIDE + D] = s_m[tid];
    P.ws[rec * WS_STRIDE + D + 1] = s_l[tid];
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
