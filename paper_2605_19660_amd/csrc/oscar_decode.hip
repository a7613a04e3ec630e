// oscar_decode_attn, generic plain-ALU path: split-K partial pass over the packed
// pages + the 16-bit residual, then a log-sum-exp reduce pass.
//
//   logit[h][i] = scale * n_i * sum_j Q_h[h][j] * Delta_k[g(i)][j] * (c_k[i][j] - z_k[g(i)][j])
//   out[h][j]   = sum_i softmax(logit[h])_i * Delta_v[i][G(j)] * (c_v[i][j] - z_v[i][G(j)])
// (App. "Implementation Details ...": logits = (Q_h . dequant(K_u)) * n_k; Algorithm
// "The OScaR algorithm", lines K_all / V_all / Attention; quantizer of Eq. 3-4.)
//
// The scales are folded so the inner loops touch raw integer codes:
//   A[g][h][j] = Q_h[h][j] * Delta_k[g][j]   and   bias[g][h] = sum_j Q_h[h][j] * (Delta_k z_k)[g][j]
//   (float zero-point mode: bias = -sum_j Q_h[h][j] * zero_k[g][j])
// are built once per page, so logit = n_i * (sum_j A * c - bias); on the value side
// w = Delta_v * c + (-Delta_v * z_v) is one fused multiply-add per element.
// One workgroup serves all query heads of a kv head, so every packed byte is read once.
#include <atomic>

#include "oscar_decode_common.h"

namespace {

template <int BITS, int GQ>
__global__ __launch_bounds__(256) void oscar_decode_partial_kernel(DecodeParams P) {
  constexpr int CPW = 32 / BITS;  // codes per 32-bit word
  constexpr int KWORDS = 64 / CPW;  // words per half key row (64 channels)
  constexpr uint32_t CMASK = (1u << BITS) - 1u;

  __shared__ __align__(16) float s_q[GQ][D];
  __shared__ __align__(16) float s_A[4][GQ][D];
  __shared__ float s_bias[4][GQ];
  __shared__ __align__(16) float s_kd[4][D];
  __shared__ __align__(16) float s_kz[4][D];
  __shared__ float s_norm[R];
  __shared__ __align__(16) float2 s_vdz[4][R];  // (Delta_v, -Delta_v * z_v)
  __shared__ __align__(16) float s_S[GQ][R];
  __shared__ float s_m[GQ], s_l[GQ], s_alpha[GQ];

  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int Hkv = P.c.cfg.n_kv_heads, Hq = P.c.cfg.n_q_heads;
  const int ngk = P.g.ngk, ngv = P.g.ngv, mb = P.g.meta_bytes;
  const bool zp_min = P.c.cfg.zp_mode == OSCAR_ZP_MIN;

  const int seq_len = P.c.seq_lens[b];
  const int r = P.c.res_lens[b];
  const int n_pages = (seq_len - r) / R;
  const int pps = (n_pages + P.num_splits - 1) / P.num_splits;
  const int pg0 = split * pps;
  const int pg1 = min(n_pages, pg0 + pps);
  const bool has_res = (split == P.num_splits - 1) && r > 0;

  if (tid < GQ) {
    s_m[tid] = -INFINITY;
    s_l[tid] = 0.0f;
  }
  float o[GQ];
#pragma unroll
  for (int h = 0; h < GQ; ++h) o[h] = 0.0f;

  const bool any_work = (pg0 < pg1) || has_res;
  if (any_work) {
    rotate_queries(s_q, P.q, ((size_t)b * Hq + (size_t)kvh * GQ) * D, P.c.cfg.io_dtype,
                   P.qk_scale_log2, tid, GQ, P.c.cfg.rotation == OSCAR_ROTATION_ON);
  } else {
    __syncthreads();
  }

  const int tok = tid >> 1, half = tid & 1;  // logit phase: (token, channel half)
  const int ch = tid >> 1, th = tid & 1;     // value phase: (channel, token half)

  for (int pg = pg0; pg < pg1; ++pg) {
    const int phys = P.c.block_table[(size_t)b * P.c.max_pages_per_seq + pg];
    const size_t pgi = (size_t)phys * Hkv + kvh;
    const uint8_t* kcodes = reinterpret_cast<const uint8_t*>(P.c.k_codes) + pgi * P.g.k_codes_bytes;
    const uint8_t* kmeta = reinterpret_cast<const uint8_t*>(P.c.k_meta) + pgi * P.g.k_meta_bytes;
    const uint8_t* knorm = reinterpret_cast<const uint8_t*>(P.c.k_norms) + pgi * P.g.k_norms_bytes;
    const uint8_t* vcodes = reinterpret_cast<const uint8_t*>(P.c.v_codes) + pgi * P.g.v_codes_bytes;
    const uint8_t* vmeta = reinterpret_cast<const uint8_t*>(P.c.v_meta) + pgi * P.g.v_meta_bytes;

    // issue the code loads early
    // Two chunks of 32 codes each: channels 64*half .. +63 of this token, and tokens of
    // quarters 2*th, 2*th+1 of this channel (chunk order).
    uint32_t kw[KWORDS], vw[KWORDS];
    {
      constexpr int WPC = KWORDS / 2;  // words per chunk
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const uint32_t* kp = reinterpret_cast<const uint32_t*>(
            kcodes + chunk_offset(BITS, tok / 16, tok % 16, 2 * half + i));
        const uint32_t* vp = reinterpret_cast<const uint32_t*>(
            vcodes + chunk_offset(BITS, ch / 16, ch % 16, 2 * th + i));
#pragma unroll
        for (int w = 0; w < WPC; ++w) {
          kw[i * WPC + w] = kp[w];
          vw[i * WPC + w] = vp[w];
        }
      }
    }
    // (0) metadata -> LDS as fp32, un-permuted (keys by channel, tokens in chunk order)
    for (int i = tid; i < ngk * D; i += 256) {
      const int gk = i / D, pos = kmeta_pos_of_chan(BITS, i % D);
      const float dk = load_meta(kmeta, (size_t)gk * D + pos, mb);
      const float zk = load_meta(kmeta, (size_t)(ngk + gk) * D + pos, mb);
      s_kd[gk][i % D] = dk;
      // what one unit of Q_h on this channel takes off the logit: Delta*z (integer zero-point)
      // or -zero (float zero-point: x = Delta*c + zero)
      s_kz[gk][i % D] = zp_min ? -zk : dk * zk;
    }
    if (tid < R) s_norm[tid] = load_meta(knorm, tok_meta_pos(tid), mb);
    for (int i = tid; i < ngv * R; i += 256) {
      const int gv = i / R, t = i % R;
      const float dv = load_meta(vmeta, (size_t)gv * R + tok_meta_pos(t), mb);
      const float zv = load_meta(vmeta, (size_t)(ngv + gv) * R + tok_meta_pos(t), mb);
      s_vdz[gv][chunk_order(BITS, t)] = make_float2(dv, zp_min ? zv : -dv * zv);
    }
    __syncthreads();
    // (1) A = Q_h * Delta_k, bias = sum_j A * z_k ; pair (group, head) -> one wave
    for (int pr = wave; pr < ngk * GQ; pr += 4) {
      const int gk = pr / GQ, h = pr % GQ;
      const float a0 = s_q[h][lane] * s_kd[gk][lane];
      const float a1 = s_q[h][lane + 64] * s_kd[gk][lane + 64];
      s_A[gk][h][lane] = a0;
      s_A[gk][h][lane + 64] = a1;
      const float part = wave_sum(s_q[h][lane] * s_kz[gk][lane] + s_q[h][lane + 64] * s_kz[gk][lane + 64]);
      if (lane == 0) s_bias[gk][h] = part;
    }
    __syncthreads();
    // (2) logits
    {
      const int gk = tok / P.g.k_group;
      float acc[GQ];
#pragma unroll
      for (int h = 0; h < GQ; ++h) acc[h] = 0.0f;
#pragma unroll
      for (int w = 0; w < KWORDS; ++w) {
#pragma unroll
        for (int e4 = 0; e4 < CPW; e4 += 4) {
          const int j = half * 64 + w * CPW + e4;
          float c[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) c[e] = (float)((kw[w] >> ((e4 + e) * BITS)) & CMASK);
#pragma unroll
          for (int h = 0; h < GQ; ++h) {
            const float4 a = *reinterpret_cast<const float4*>(&s_A[gk][h][j]);
            acc[h] = fmaf(a.x, c[0], acc[h]);
            acc[h] = fmaf(a.y, c[1], acc[h]);
            acc[h] = fmaf(a.z, c[2], acc[h]);
            acc[h] = fmaf(a.w, c[3], acc[h]);
          }
        }
      }
      const float nrm = s_norm[tok];
#pragma unroll
      for (int h = 0; h < GQ; ++h) {
        const float tot = acc[h] + __shfl_xor(acc[h], 1, 64);
        if (half == 0) s_S[h][chunk_order(BITS, tok)] = nrm * (tot - s_bias[gk][h]);
      }
    }
    __syncthreads();
    // (3) online softmax, heads striped over waves
    for (int h = wave; h < GQ; h += 4) {
      const float s0 = s_S[h][lane], s1 = s_S[h][lane + 64];
      const float m_old = s_m[h];
      const float m_new = fmaxf(m_old, wave_max(fmaxf(s0, s1)));
      const float alpha = exp2f(m_old - m_new);
      const float p0 = exp2f(s0 - m_new), p1 = exp2f(s1 - m_new);
      const float sum = wave_sum(p0 + p1);
      s_S[h][lane] = p0;
      s_S[h][lane + 64] = p1;
      if (lane == 0) {
        s_m[h] = m_new;
        s_l[h] = s_l[h] * alpha + sum;
        s_alpha[h] = alpha;
      }
    }
    __syncthreads();
    // (4) o += P * V_hat
    {
      const int gv = ch / P.g.v_group;
#pragma unroll
      for (int h = 0; h < GQ; ++h) o[h] *= s_alpha[h];
#pragma unroll
      for (int w = 0; w < KWORDS; ++w) {
#pragma unroll
        for (int e4 = 0; e4 < CPW; e4 += 4) {
          const int t = th * 64 + w * CPW + e4;
          float wv[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float2 dz = s_vdz[gv][t + e];
            wv[e] = fmaf(dz.x, (float)((vw[w] >> ((e4 + e) * BITS)) & CMASK), dz.y);
          }
#pragma unroll
          for (int h = 0; h < GQ; ++h) {
            const float4 p = *reinterpret_cast<const float4*>(&s_S[h][t]);
            o[h] = fmaf(p.x, wv[0], o[h]);
            o[h] = fmaf(p.y, wv[1], o[h]);
            o[h] = fmaf(p.z, wv[2], o[h]);
            o[h] = fmaf(p.w, wv[3], o[h]);
          }
        }
      }
    }
    __syncthreads();
  }

  if (has_res) {
    // residual tokens: fp16 K_u times stored norm, values in the input precision
    const size_t rb = ((size_t)b * Hkv + kvh) * R;
    const __half* rk = reinterpret_cast<const __half*>(P.c.res_k) + rb * D;
    if (tid < R) s_norm[tid] = tid < r ? load_meta(P.c.res_norm, rb + tid, mb) : 0.0f;
    __syncthreads();
    {
      float acc[GQ];
#pragma unroll
      for (int h = 0; h < GQ; ++h) acc[h] = 0.0f;
      if (tok < r) {
        const uint4* kp = reinterpret_cast<const uint4*>(rk + (size_t)tok * D + half * 64);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint4 raw = kp[i];
          const uint32_t wds[4] = {raw.x, raw.y, raw.z, raw.w};
          float kv[8];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            kv[2 * e] = __half2float(__ushort_as_half((unsigned short)(wds[e] & 0xffffu)));
            kv[2 * e + 1] = __half2float(__ushort_as_half((unsigned short)(wds[e] >> 16)));
          }
          const int j = half * 64 + i * 8;
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
      }
      const float nrm = s_norm[tok];
#pragma unroll
      for (int h = 0; h < GQ; ++h) {
        const float tot = acc[h] + __shfl_xor(acc[h], 1, 64);
        if (half == 0) s_S[h][chunk_order(BITS, tok)] = tok < r ? nrm * tot : -INFINITY;
      }
    }
    __syncthreads();
    for (int h = wave; h < GQ; h += 4) {
      const float s0 = s_S[h][lane], s1 = s_S[h][lane + 64];
      const float m_old = s_m[h];
      const float m_new = fmaxf(m_old, wave_max(fmaxf(s0, s1)));
      const float alpha = exp2f(m_old - m_new);
      const float p0 = exp2f(s0 - m_new), p1 = exp2f(s1 - m_new);
      const float sum = wave_sum(p0 + p1);
      s_S[h][lane] = p0;
      s_S[h][lane + 64] = p1;
      if (lane == 0) {
        s_m[h] = m_new;
        s_l[h] = s_l[h] * alpha + sum;
        s_alpha[h] = alpha;
      }
    }
    __syncthreads();
    {
#pragma unroll
      for (int h = 0; h < GQ; ++h) o[h] *= s_alpha[h];
      const int t_end = min(r, th * 64 + 64);
      // 16 independent loads in flight per batch (positions past the end carry p = 0)
      for (int t0 = th * 64; t0 < t_end; t0 += 16) {
        float wv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i)
          wv[i] = (t0 + i < t_end) ? load_io(P.c.res_v, (rb + t0 + i) * D + ch, P.c.cfg.io_dtype) : 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
          for (int h = 0; h < GQ; ++h)
            o[h] = fmaf(s_S[h][chunk_order(BITS, t0 + i)], wv[i], o[h]);
      }
    }
    __syncthreads();
  }

  // partial record per (b, q head, split)
#pragma unroll
  for (int h = 0; h < GQ; ++h) {
    const float tot = o[h] + __shfl_xor(o[h], 1, 64);
    if (th == 0) {
      const size_t rec = ((size_t)b * Hq + (size_t)kvh * GQ + h) * P.num_splits + split;
      P.ws[rec * WS_STRIDE + ch] = tot;
    }
  }
  if (tid < GQ) {
    const size_t rec = ((size_t)b * Hq + (size_t)kvh * GQ + tid) * P.num_splits + split;
    P.ws[rec * WS_STRIDE + D] = s_m[tid];
    P.ws[rec * WS_STRIDE + D + 1] = s_l[tid];
  }
}

}  // namespace

// Reduce pass shared with the 16-bit comparator: merges split partials
// (o_s, m_s, l_s) with M = max m_s, out = sum o_s 2^(m_s-M) / sum l_s 2^(m_s-M).
// One block of 128 threads per (sequence, query head); the split statistics are fetched
// by one thread each, so no thread walks a chain of dependent loads.
__global__ __launch_bounds__(128) void oscar_decode_reduce_kernel(const float* ws, void* out,
                                                                  int num_splits, int out_dtype) {
  __shared__ float s_w[512];   // weight of each split (num_splits <= 512)
  __shared__ float s_red[4];
  const size_t unit = (size_t)blockIdx.y * gridDim.x + blockIdx.x;  // b * Hq + h
  const int c = threadIdx.x;
  const float* rec = ws + unit * num_splits * WS_STRIDE;
  if (num_splits <= 16) {
    // few splits: every thread fetches all the split statistics (same addresses across the
    // wave) together with its own channel of every partial output, one round of loads and
    // no barrier
    float m[16], l[16], o[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      const bool on = s < num_splits;
      m[s] = on ? rec[(size_t)s * WS_STRIDE + D] : -INFINITY;
      l[s] = on ? rec[(size_t)s * WS_STRIDE + D + 1] : 0.0f;
      o[s] = on ? rec[(size_t)s * WS_STRIDE + c] : 0.0f;
    }
    float M = m[0];
#pragma unroll
    for (int s = 1; s < 16; ++s) M = fmaxf(M, m[s]);
    float L = 0.0f, acc = 0.0f;
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      const float w = (m[s] == -INFINITY) ? 0.0f : exp2f(m[s] - M);
      L = fmaf(l[s], w, L);
      acc = fmaf(o[s], w, acc);
    }
    const float res = L > 0.0f ? acc / L : 0.0f;
    const size_t oi = unit * D + c;
    if (out_dtype == OSCAR_F32) reinterpret_cast<float*>(out)[oi] = res;
    else if (out_dtype == OSCAR_BF16) reinterpret_cast<__hip_bfloat16*>(out)[oi] = __float2bfloat16(res);
    else reinterpret_cast<__half*>(out)[oi] = __float2half_rn(res);
    return;
  }
  // pass 1: M
  float mloc = -INFINITY;
  for (int s = c; s < num_splits; s += 128) mloc = fmaxf(mloc, rec[(size_t)s * WS_STRIDE + D]);
  mloc = wave_max(mloc);
  if ((c & 63) == 0) s_red[c >> 6] = mloc;
  __syncthreads();
  const float M = fmaxf(s_red[0], s_red[1]);
  // pass 2: weights and L
  float lloc = 0.0f;
  for (int s = c; s < num_splits; s += 128) {
    const float m = rec[(size_t)s * WS_STRIDE + D];
    const float w = (m == -INFINITY) ? 0.0f : exp2f(m - M);
    s_w[s] = w;
    lloc += rec[(size_t)s * WS_STRIDE + D + 1] * w;
  }
  lloc = wave_sum(lloc);
  if ((c & 63) == 0) s_red[2 + (c >> 6)] = lloc;
  __syncthreads();
  const float L = s_red[2] + s_red[3];
  // pass 3: weighted sum of the partial outputs, four independent loads in flight
  float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
  int s = 0;
  for (; s + 4 <= num_splits; s += 4) {
    a0 = fmaf(rec[(size_t)(s + 0) * WS_STRIDE + c], s_w[s + 0], a0);
    a1 = fmaf(rec[(size_t)(s + 1) * WS_STRIDE + c], s_w[s + 1], a1);
    a2 = fmaf(rec[(size_t)(s + 2) * WS_STRIDE + c], s_w[s + 2], a2);
    a3 = fmaf(rec[(size_t)(s + 3) * WS_STRIDE + c], s_w[s + 3], a3);
  }
  for (; s < num_splits; ++s) a0 = fmaf(rec[(size_t)s * WS_STRIDE + c], s_w[s], a0);
  const float acc = (a0 + a1) + (a2 + a3);
  const float res = L > 0.0f ? acc / L : 0.0f;
  const size_t oi = unit * D + c;
  if (out_dtype == OSCAR_F32) reinterpret_cast<float*>(out)[oi] = res;
  else if (out_dtype == OSCAR_BF16) reinterpret_cast<__hip_bfloat16*>(out)[oi] = __float2bfloat16(res);
  else reinterpret_cast<__half*>(out)[oi] = __float2half_rn(res);
}

// Host launcher of the reduce pass (also used by the 16-bit comparator).
void oscar_launch_decode_reduce(const float* ws, void* out, int num_splits, int out_dtype,
                                int n_q_heads, int batch, hipStream_t st) {
  hipLaunchKernelGGL(oscar_decode_reduce_kernel, dim3(n_q_heads, batch), dim3(128), 0, st, ws, out,
                     num_splits, out_dtype);
}

namespace {

template <int BITS>
int launch_gq(const DecodeParams& P, int gq, dim3 grid, hipStream_t st, hipEvent_t e0,
              hipEvent_t e1) {
  switch (gq) {
#define OSCAR_CASE(G) \
  case G:                                                                                     \
    if (e0 || e1)                                                                             \
      hipExtLaunchKernelGGL((oscar_decode_partial_kernel<BITS, G>), grid, dim3(256), 0, st,   \
                            e0, e1, 0, P);                                                    \
    else                                                                                      \
      hipLaunchKernelGGL((oscar_decode_partial_kernel<BITS, G>), grid, dim3(256), 0, st, P);  \
    break;
    OSCAR_CASE(1) OSCAR_CASE(2) OSCAR_CASE(3) OSCAR_CASE(4)
    OSCAR_CASE(5) OSCAR_CASE(6) OSCAR_CASE(7) OSCAR_CASE(8)
#undef OSCAR_CASE
    default: return OSCAR_ERR_UNSUPPORTED;
  }
  return OSCAR_OK;
}

}  // namespace

static int check_decode_cache(const oscar_cache* cache) {
  if (!cache) return OSCAR_ERR_INVALID_ARG;
  int rc = oscar_validate_config(&cache->cfg);
  if (rc != OSCAR_OK) return rc;
  if (cache->batch <= 0 || cache->max_pages_per_seq <= 0) return OSCAR_ERR_INVALID_ARG;
  if (!cache->k_codes || !cache->k_meta || !cache->k_norms || !cache->v_codes || !cache->v_meta ||
      !cache->res_k || !cache->res_v || !cache->res_norm || !cache->block_table ||
      !cache->seq_lens || !cache->res_lens)
    return OSCAR_ERR_INVALID_ARG;
  return OSCAR_OK;
}

// out != nullptr (callers pass it for a single split only): the matrix-core kernel writes the
// attention output itself and *wrote_out is set; the generic kernel always writes records.
static int launch_partial(const void* q, const oscar_cache* cache, void* out, int32_t out_dtype,
                          float softmax_scale, int32_t num_splits, void* workspace,
                          size_t workspace_bytes, void* stream, oscar_timer* timer,
                          int* wrote_out = nullptr) {
  int rc = check_decode_cache(cache);
  if (rc != OSCAR_OK) return rc;
  if (!q || num_splits <= 0 || num_splits > 512) return OSCAR_ERR_INVALID_ARG;
  hipEvent_t e0 = timer ? timer->start : nullptr, e1 = timer ? timer->stop : nullptr;
  const size_t need = oscar_decode_workspace_bytes(&cache->cfg, cache->batch, num_splits);
  if (!workspace || workspace_bytes < need) return OSCAR_ERR_WORKSPACE;
  DecodeParams P;
  P.q = q;
  P.out = out;
  P.ws = reinterpret_cast<float*>(workspace);
  P.c = *cache;
  P.g = make_geom(cache->cfg.bits, cache->cfg.k_group, cache->cfg.v_group, cache->cfg.meta_dtype);
  P.num_splits = num_splits;
  const float scale = softmax_scale > 0.0f ? softmax_scale : 0.08838834764831845f;
  P.qk_scale_log2 = scale * 1.4426950408889634f;
  P.out_dtype = out_dtype;
  const int gq = cache->cfg.n_q_heads / cache->cfg.n_kv_heads;
  dim3 grid(num_splits, cache->cfg.n_kv_heads, cache->batch);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (out && num_splits != 1) return OSCAR_ERR_INVALID_ARG;
  if (wrote_out) *wrote_out = 0;
  rc = oscar_launch_decode_mfma(&P, gq, grid, st, e0, e1);
  if (rc == OSCAR_OK && out && wrote_out) *wrote_out = 1;
  if (rc == OSCAR_ERR_UNSUPPORTED) {
    P.out = nullptr;
    rc = (cache->cfg.bits == 2) ? launch_gq<2>(P, gq, grid, st, e0, e1)
                                : launch_gq<4>(P, gq, grid, st, e0, e1);
  }
  if (rc != OSCAR_OK) return rc;
  if (hipGetLastError() != hipSuccess) return OSCAR_ERR_HIP;
  if (timer) timer->armed = 1;
  return OSCAR_OK;
}

extern "C" int oscar_timer_create(oscar_timer** timer) {
  if (!timer) return OSCAR_ERR_INVALID_ARG;
  oscar_timer* t = new (std::nothrow) oscar_timer;
  if (!t) return OSCAR_ERR_HIP;
  t->start = t->stop = nullptr;
  t->armed = 0;
  if (hipEventCreate(&t->start) != hipSuccess || hipEventCreate(&t->stop) != hipSuccess) {
    if (t->start) (void)hipEventDestroy(t->start);
    delete t;
    (void)hipGetLastError();
    return OSCAR_ERR_HIP;
  }
  *timer = t;
  return OSCAR_OK;
}

extern "C" int oscar_timer_destroy(oscar_timer* timer) {
  if (!timer) return OSCAR_OK;
  (void)hipEventDestroy(timer->start);
  (void)hipEventDestroy(timer->stop);
  delete timer;
  return OSCAR_OK;
}

extern "C" int oscar_timer_elapsed_us(oscar_timer* timer, float* us) {
  if (!timer || !us || !timer->armed) return OSCAR_ERR_INVALID_ARG;
  float ms = 0.0f;
  if (hipEventSynchronize(timer->stop) != hipSuccess ||
      hipEventElapsedTime(&ms, timer->start, timer->stop) != hipSuccess) {
    (void)hipGetLastError();
    return OSCAR_ERR_HIP;
  }
  *us = ms * 1000.0f;
  return OSCAR_OK;
}

extern "C" int oscar_decode_attn_partial_timed(const void* q, const oscar_cache* cache,
                                               float softmax_scale, int32_t num_splits,
                                               void* workspace, size_t workspace_bytes,
                                               void* stream, oscar_timer* timer) {
  if (!timer) return OSCAR_ERR_INVALID_ARG;
  return launch_partial(q, cache, nullptr, OSCAR_F32, softmax_scale, num_splits, workspace,
                        workspace_bytes, stream, timer);
}

extern "C" int oscar_decode_attn_partial(const void* q, const oscar_cache* cache,
                                         float softmax_scale, int32_t num_splits,
                                         void* workspace, size_t workspace_bytes, void* stream) {
  return launch_partial(q, cache, nullptr, OSCAR_F32, softmax_scale, num_splits, workspace,
                        workspace_bytes, stream, nullptr);
}

extern "C" int oscar_decode_attn_reduce(const oscar_cache* cache, void* out, int32_t out_dtype,
                                        int32_t num_splits, const void* workspace,
                                        size_t workspace_bytes, void* stream) {
  int rc = check_decode_cache(cache);
  if (rc != OSCAR_OK) return rc;
  if (!out || num_splits <= 0 || num_splits > 512) return OSCAR_ERR_INVALID_ARG;
  if (out_dtype != OSCAR_F32 && out_dtype != cache->cfg.io_dtype) return OSCAR_ERR_INVALID_ARG;
  const size_t need = oscar_decode_workspace_bytes(&cache->cfg, cache->batch, num_splits);
  if (!workspace || workspace_bytes < need) return OSCAR_ERR_WORKSPACE;
  oscar_launch_decode_reduce(reinterpret_cast<const float*>(workspace), out, num_splits, out_dtype,
                             cache->cfg.n_q_heads, cache->batch,
                             reinterpret_cast<hipStream_t>(stream));
  if (hipGetLastError() != hipSuccess) return OSCAR_ERR_HIP;
  return OSCAR_OK;
}

extern "C" int oscar_decode_attn(const void* q, const oscar_cache* cache, void* out,
                                 int32_t out_dtype, float softmax_scale,
                                 int32_t max_seq_len_hint, int32_t num_splits, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  int rc = check_decode_cache(cache);
  if (rc != OSCAR_OK) return rc;
  if (!q || !out || max_seq_len_hint < 0 || num_splits < 0) return OSCAR_ERR_INVALID_ARG;
  if (out_dtype != OSCAR_F32 && out_dtype != cache->cfg.io_dtype) return OSCAR_ERR_INVALID_ARG;
  if (num_splits == 0)
    num_splits = oscar_decode_auto_splits(&cache->cfg, cache->batch, max_seq_len_hint);
  // a single split needs no reduce pass: the matrix-core kernel then writes `out` itself
  int wrote_out = 0;
  rc = launch_partial(q, cache, num_splits == 1 ? out : nullptr, out_dtype, softmax_scale,
                      num_splits, workspace, workspace_bytes, stream, nullptr, &wrote_out);
  if (rc != OSCAR_OK || wrote_out) return rc;
  return oscar_decode_attn_reduce(cache, out, out_dtype, num_splits, workspace, workspace_bytes,
                                  stream);
}

// One decode step as a single call: the new token of every sequence goes through
// oscar_quantize_append (decode rule), then the attention runs over the updated cache.
extern "C" int oscar_decode_step(const void* k_new, const void* v_new, const void* q,
                                 oscar_cache* cache, void* out, int32_t out_dtype,
                                 float softmax_scale, int32_t max_seq_len_hint, int32_t num_splits,
                                 void* workspace, size_t workspace_bytes, void* stream,
                                 oscar_timer* partial_timer) {
  int rc = check_decode_cache(cache);
  if (rc != OSCAR_OK) return rc;
  if (!k_new || !v_new || !q || !out || max_seq_len_hint < 1 || num_splits < 0 || num_splits > 512)
    return OSCAR_ERR_INVALID_ARG;
  if (out_dtype != OSCAR_F32 && out_dtype != cache->cfg.io_dtype) return OSCAR_ERR_INVALID_ARG;
  if (num_splits == 0)
    num_splits = oscar_decode_auto_splits(&cache->cfg, cache->batch, max_seq_len_hint);
  // every argument of the attention is checked before the append is enqueued
  const size_t need = oscar_decode_workspace_bytes(&cache->cfg, cache->batch, num_splits);
  if (!workspace || workspace_bytes < need) return OSCAR_ERR_WORKSPACE;
  rc = oscar_quantize_append(k_new, v_new, 1, nullptr, cache, max_seq_len_hint - 1, 0u, stream);
  if (rc != OSCAR_OK) return rc;
  int wrote_out = 0;
  rc = launch_partial(q, cache, num_splits == 1 ? out : nullptr, out_dtype, softmax_scale,
                      num_splits, workspace, workspace_bytes, stream, partial_timer, &wrote_out);
  if (rc != OSCAR_OK || wrote_out) return rc;
  return oscar_decode_attn_reduce(cache, out, out_dtype, num_splits, workspace, workspace_bytes,
                                  stream);
}

// ---- the entry point that allocates nothing -------------------------------------------------
// Split-K partials live in a fixed array inside the library's device image instead of a caller
// workspace.  In host code the array's name is only a stand-in: its device address is asked of
// the runtime once per device (each GPU holds its own copy) and kept; kernels get that pointer.
static __device__ __align__(256) unsigned char scratch[OSCAR_NOALLOC_SCRATCH_BYTES];

static int noalloc_scratch_of_current_device(void** out) {
  constexpr int kMaxDev = 64;
  static std::atomic<void*> ptr_of[kMaxDev];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) {
    (void)hipGetLastError();
    return OSCAR_ERR_HIP;
  }
  void* p = ptr_of[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return OSCAR_ERR_HIP;
    }
    ptr_of[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return OSCAR_OK;
}

extern "C" int oscar_decode_attn_noalloc(const void* q, const oscar_cache* cache, void* out,
                                         int32_t out_dtype, float softmax_scale,
                                         int32_t max_seq_len_hint, int32_t num_splits,
                                         void* stream) {
  int rc = check_decode_cache(cache);
  if (rc != OSCAR_OK) return rc;
  if (!q || !out || max_seq_len_hint < 0 || num_splits < 0 || num_splits > 512)
    return OSCAR_ERR_INVALID_ARG;
  if (out_dtype != OSCAR_F32 && out_dtype != cache->cfg.io_dtype) return OSCAR_ERR_INVALID_ARG;
  if (num_splits == 0)
    num_splits = oscar_decode_auto_splits(&cache->cfg, cache->batch, max_seq_len_hint);
  const size_t need = oscar_decode_workspace_bytes(&cache->cfg, cache->batch, num_splits);
  if (need == 0 || need > (size_t)OSCAR_NOALLOC_SCRATCH_BYTES) return OSCAR_ERR_WORKSPACE;
  void* ws = nullptr;
  rc = noalloc_scratch_of_current_device(&ws);
  if (rc != OSCAR_OK) return rc;
  // every record of the partials (batch x query head x split) is written by the partial pass
  // before the reduce pass reads it, so nothing of the previous call's contents has to be cleared
  int wrote_out = 0;
  rc = launch_partial(q, cache, num_splits == 1 ? out : nullptr, out_dtype, softmax_scale,
                      num_splits, ws, (size_t)OSCAR_NOALLOC_SCRATCH_BYTES, stream, nullptr,
                      &wrote_out);
  if (rc != OSCAR_OK || wrote_out) return rc;
  return oscar_decode_attn_reduce(cache, out, out_dtype, num_splits, ws,
                                  (size_t)OSCAR_NOALLOC_SCRATCH_BYTES, stream);
}
