// oscar_quantize_append and oscar_rotate entry points; the encoder kernel itself is in
// oscar_append_kernel.h (compiled here for the per-head norm).  -ffp-contract=off.
#include "oscar_append_kernel.h"

namespace {

// largest grid of a multi-block append whose length update rides on the encoder launch
// (oscar_quantize_append)
constexpr size_t kTicketMaxWorkgroups = 1024;

// Stand-alone rotation kernel: 16 vectors of 128 channels per workgroup (one DPP row each).
// NORMALIZE = false: out = H(x)/sqrt(128) in fp32 (queries).
// NORMALIZE = true : norms = ||H(x)/sqrt(128)|| (metadata type), out = fp16 of the quotient
// (keys); `fast` takes the reciprocal square root instruction instead of sqrt + divide.
template <typename IO, typename META, bool NORMALIZE>
__global__ __launch_bounds__(256) void oscar_rotate_kernel(const IO* __restrict__ x, void* out,
                                                           META* norms, long long n_vec, int fast) {
  const int tid = threadIdx.x;
  const int cg = channel_group_of_row_lane(tid & 15);
  uint32_t sgn[4];
#pragma unroll
  for (int st = 0; st < 4; ++st) sgn[st] = ((cg >> st) & 1) ? 0x80000000u : 0u;
  const long long v = (long long)blockIdx.x * 16 + (tid >> 4);
  const long long vc = v < n_vec ? v : n_vec - 1;   // whole rows stay active for the exchanges
  Raw8<IO> raw;
  raw.load(x + (size_t)vc * D + cg * 8);
  float xs[8];
  raw.widen(xs);
  if (!NORMALIZE) {
    rotate8(xs, sgn);
    if (v < n_vec) {
      float4* o = reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + (size_t)v * D + cg * 8);
      o[0] = make_float4(xs[0], xs[1], xs[2], xs[3]);
      o[1] = make_float4(xs[4], xs[5], xs[6], xs[7]);
    }
    return;
  }
  uint4 u;
  float nf;
  if (fast) {
    rotate8(xs, sgn);
    const float s = row_sumsq(xs);
    const float inv = s > 0.0f ? __builtin_amdgcn_rsqf(s) : 0.0f;
    nf = round_meta<META>(s * inv);
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      w[i] = half_bits(pin_f32(xs[2 * i] * inv)) | (half_bits(pin_f32(xs[2 * i + 1] * inv)) << 16);
    u = make_uint4(w[0], w[1], w[2], w[3]);
  } else {
    u = key_transform8<META>(xs, sgn, nf);
  }
  if (v < n_vec) {
    *reinterpret_cast<uint4*>(reinterpret_cast<__half*>(out) + (size_t)v * D + cg * 8) = u;
    if (cg == 0) norms[v] = from_f32<META>(nf);
  }
}

// Matrix-core variant of the rotation (App. "Fused Hadamard-Norm Kernel": H_128 = H_8 (x) H_16,
// the H_16 factor on matrix tiles, the H_8 factor as butterflies).  A vector is read as an
// 8 x 16 matrix X (x[16 a + b]); H_128 x = vec(H_8 X H_16).  One 16x16x16 MFMA computes
// H_16 X^T for two vectors at once: operand A is H_16 (entries +-1, exact in the 16-bit operand
// type), operand B holds the 16 columns (vector, a) with the 16 values of b along the
// contraction; accumulation is fp32.  The accumulator leaves a lane with four consecutive b of
// one (vector, a) -- its output is one 8- or 16-byte store -- and the H_8 factor is three
// butterfly stages across the lanes of a, labelled as everywhere else so that each partner is
// one DPP control.  The summation order differs from the butterfly of the cache path, so
// results agree with it to fp32 rounding, not bit for bit: this variant is an option of
// oscar_rotate, never of oscar_quantize_append.
typedef short short4v __attribute__((ext_vector_type(4)));
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef float float4m __attribute__((ext_vector_type(4)));

template <typename IO> struct MfmaH16;
template <> struct MfmaH16<__hip_bfloat16> {
  // A = H_16[m][4 kg .. 4 kg + 3] as bf16 (+-1), B = the lane's four inputs as they are
  static __device__ __forceinline__ float4m run(uint2 xraw, int m, int kg) {
    short4v h, xb = __builtin_bit_cast(short4v, xraw);
#pragma unroll
    for (int i = 0; i < 4; ++i) h[i] = (short)((__builtin_popcount((4 * kg + i) & m) & 1) ? 0xBF80 : 0x3F80);
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(h, xb, (float4m){0.0f, 0.0f, 0.0f, 0.0f}, 0, 0, 0);
  }
};
template <> struct MfmaH16<__half> {
  static __device__ __forceinline__ float4m run(uint2 xraw, int m, int kg) {
    half4v h, xb = __builtin_bit_cast(half4v, xraw);
#pragma unroll
    for (int i = 0; i < 4; ++i) h[i] = (__builtin_popcount((4 * kg + i) & m) & 1) ? (_Float16)-1.0f : (_Float16)1.0f;
    return __builtin_amdgcn_mfma_f32_16x16x16f16(h, xb, (float4m){0.0f, 0.0f, 0.0f, 0.0f}, 0, 0, 0);
  }
};

// One wave rotates two vectors per step; 4 waves, 8 steps: 64 vectors per workgroup.
template <typename IO, typename META, bool NORMALIZE>
__global__ __launch_bounds__(256) void oscar_rotate_mfma_kernel(const IO* __restrict__ x, void* out,
                                                                META* norms, long long n_vec, int fast) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, kg = lane >> 4;
  // column n of the tile = (vector, a): the row-lane labelling of the butterflies
  const int col = channel_group_of_row_lane(n);
  const int a = col & 7, vl = col >> 3;
  uint32_t sgn[3];
#pragma unroll
  for (int st = 0; st < 3; ++st) sgn[st] = ((a >> st) & 1) ? 0x80000000u : 0u;
  const long long v_base = ((long long)blockIdx.x * 4 + wave) * 16;
  for (int step = 0; step < 8; ++step) {
    const long long v0 = v_base + 2 * step;                 // this step's two vectors
    if (v0 >= n_vec) break;                                  // wave-uniform
    const long long v = v0 + vl;
    const long long vc = v < n_vec ? v : n_vec - 1;          // a vector past the end repeats the last
    // operand B: x[v][16 a + 4 kg .. + 3], 8 bytes per lane
    const uint2 xraw = *reinterpret_cast<const uint2*>(x + (size_t)vc * D + 16 * a + 4 * kg);
    // accumulator: rows 4 kg + i = b, column n: w[i] = (X H_16)[a][4 kg + i] of vector vl
    float4m z = MfmaH16<IO>::run(xraw, n, kg);
    float w[4] = {z[0], z[1], z[2], z[3]};
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = partner<0>(w[i]) + __uint_as_float(__float_as_uint(w[i]) ^ sgn[0]);
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = partner<1>(w[i]) + __uint_as_float(__float_as_uint(w[i]) ^ sgn[1]);
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = partner<2>(w[i]) + __uint_as_float(__float_as_uint(w[i]) ^ sgn[2]);
    const float c = 0.08838834764831845f;  // fp32(1/sqrt(128))
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] *= c;
    const size_t o_idx = (size_t)v * D + 16 * a + 4 * kg;
    if (!NORMALIZE) {
      if (v < n_vec)
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + o_idx) = make_float4(w[0], w[1], w[2], w[3]);
      continue;
    }
    // token norm: sum of squares over the vector's 128 values = 4 registers x 8 lanes of a x 4 groups
    float s = (w[0] * w[0] + w[1] * w[1]) + (w[2] * w[2] + w[3] * w[3]);
    s += partner<0>(s);
    s += partner<1>(s);
    s += partner<2>(s);
    s += __shfl_xor(s, 16, 64);
    s += __shfl_xor(s, 32, 64);
    float inv, nf;
    if (fast) {
      inv = s > 0.0f ? __builtin_amdgcn_rsqf(s) : 0.0f;
      nf = round_meta<META>(s * inv);
    } else {
      nf = round_meta<META>(sqrtf(s));
      inv = (nf > 0.0f && !isinf(nf)) ? 1.0f / nf : 0.0f;
    }
    if (v < n_vec) {
      uint2 pk;
      pk.x = half_bits(pin_f32(w[0] * inv)) | (half_bits(pin_f32(w[1] * inv)) << 16);
      pk.y = half_bits(pin_f32(w[2] * inv)) | (half_bits(pin_f32(w[3] * inv)) << 16);
      *reinterpret_cast<uint2*>(reinterpret_cast<__half*>(out) + o_idx) = pk;
      if (a == 0 && kg == 0) norms[v] = from_f32<META>(nf);
    }
  }
}

template <typename IO>
int launch_rotate_mfma(const void* x, void* out, void* norms, long long n_vec, int meta_dtype,
                       uint32_t flags, hipStream_t st) {
  const dim3 grid((unsigned)((n_vec + 63) / 64));
  const IO* xp = reinterpret_cast<const IO*>(x);
  const int fast = (flags & OSCAR_ROTATE_FAST_RSQRT) ? 1 : 0;
  if (!(flags & OSCAR_ROTATE_NORMALIZE)) {
    hipLaunchKernelGGL((oscar_rotate_mfma_kernel<IO, float, false>), grid, dim3(256), 0, st, xp, out,
                       (float*)nullptr, n_vec, 0);
  } else if (meta_dtype == OSCAR_F16) {
    hipLaunchKernelGGL((oscar_rotate_mfma_kernel<IO, __half, true>), grid, dim3(256), 0, st, xp, out,
                       reinterpret_cast<__half*>(norms), n_vec, fast);
  } else if (meta_dtype == OSCAR_F32) {
    hipLaunchKernelGGL((oscar_rotate_mfma_kernel<IO, float, true>), grid, dim3(256), 0, st, xp, out,
                       reinterpret_cast<float*>(norms), n_vec, fast);
  } else {
    return OSCAR_ERR_UNSUPPORTED;
  }
  return OSCAR_OK;
}

template <typename IO>
int launch_rotate(const void* x, void* out, void* norms, long long n_vec, int meta_dtype,
                  uint32_t flags, hipStream_t st) {
  const dim3 grid((unsigned)((n_vec + 15) / 16));
  const IO* xp = reinterpret_cast<const IO*>(x);
  const int fast = (flags & OSCAR_ROTATE_FAST_RSQRT) ? 1 : 0;
  if (!(flags & OSCAR_ROTATE_NORMALIZE)) {
    hipLaunchKernelGGL((oscar_rotate_kernel<IO, float, false>), grid, dim3(256), 0, st, xp, out,
                       (float*)nullptr, n_vec, 0);
  } else if (meta_dtype == OSCAR_F16) {
    hipLaunchKernelGGL((oscar_rotate_kernel<IO, __half, true>), grid, dim3(256), 0, st, xp, out,
                       reinterpret_cast<__half*>(norms), n_vec, fast);
  } else if (meta_dtype == OSCAR_F32) {
    hipLaunchKernelGGL((oscar_rotate_kernel<IO, float, true>), grid, dim3(256), 0, st, xp, out,
                       reinterpret_cast<float*>(norms), n_vec, fast);
  } else {
    return OSCAR_ERR_UNSUPPORTED;
  }
  return OSCAR_OK;
}

// H along the row axis: thread = (block of 128 rows, column); the 128 values of a column
// sit in registers, all seven butterfly stages are register-to-register, and the lanes of a
// wave read and write consecutive columns.
template <typename IO>
__global__ __launch_bounds__(256) void oscar_rotate_columns_kernel(const IO* __restrict__ w,
                                                                   float* __restrict__ out,
                                                                   long long n_cols) {
  const long long c = (long long)blockIdx.x * 256 + threadIdx.x;
  if (c >= n_cols) return;
  const size_t base = (size_t)blockIdx.y * D * (size_t)n_cols + (size_t)c;
  float x[D];
#pragma unroll
  for (int j = 0; j < D; ++j) x[j] = to_f32<IO>(w[base + (size_t)j * n_cols]);
#pragma unroll
  for (int h = 1; h < D; h <<= 1) {
#pragma unroll
    for (int i = 0; i < D; ++i) {
      if ((i & h) == 0) {
        const float a = x[i], b = x[i | h];
        x[i] = a + b;
        x[i | h] = a - b;
      }
    }
  }
  const float cs = 0.08838834764831845f;  // fp32(1/sqrt(128))
#pragma unroll
  for (int j = 0; j < D; ++j) out[base + (size_t)j * n_cols] = x[j] * cs;
}

}  // namespace

extern "C" int oscar_rotate_columns(const void* w, void* out, int64_t n_rows, int64_t n_cols,
                                    int32_t io_dtype, void* stream) {
  if (!w || !out || n_rows < 0 || n_cols < 0 || n_rows % D != 0) return OSCAR_ERR_INVALID_ARG;
  if (n_rows / D > 65535 || n_cols > ((int64_t)1 << 38)) return OSCAR_ERR_INVALID_ARG;
  if (n_rows == 0 || n_cols == 0) return OSCAR_OK;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const dim3 grid((unsigned)((n_cols + 255) / 256), (unsigned)(n_rows / D));
  float* o = reinterpret_cast<float*>(out);
  switch (io_dtype) {
    case OSCAR_F32:
      hipLaunchKernelGGL((oscar_rotate_columns_kernel<float>), grid, dim3(256), 0, st,
                         reinterpret_cast<const float*>(w), o, (long long)n_cols);
      break;
    case OSCAR_BF16:
      hipLaunchKernelGGL((oscar_rotate_columns_kernel<__hip_bfloat16>), grid, dim3(256), 0, st,
                         reinterpret_cast<const __hip_bfloat16*>(w), o, (long long)n_cols);
      break;
    case OSCAR_F16:
      hipLaunchKernelGGL((oscar_rotate_columns_kernel<__half>), grid, dim3(256), 0, st,
                         reinterpret_cast<const __half*>(w), o, (long long)n_cols);
      break;
    default: return OSCAR_ERR_INVALID_ARG;
  }
  if (hipGetLastError() != hipSuccess) return OSCAR_ERR_HIP;
  return OSCAR_OK;
}

extern "C" int oscar_rotate(const void* x, void* out, void* norms, int64_t n_vec, int32_t io_dtype,
                            int32_t meta_dtype, uint32_t flags, void* stream) {
  if (!x || !out || n_vec < 0) return OSCAR_ERR_INVALID_ARG;
  if (flags & ~(uint32_t)(OSCAR_ROTATE_NORMALIZE | OSCAR_ROTATE_FAST_RSQRT | OSCAR_ROTATE_MATRIX_CORE))
    return OSCAR_ERR_INVALID_ARG;
  if ((flags & OSCAR_ROTATE_FAST_RSQRT) && !(flags & OSCAR_ROTATE_NORMALIZE)) return OSCAR_ERR_INVALID_ARG;
  if ((flags & OSCAR_ROTATE_NORMALIZE) && !norms) return OSCAR_ERR_INVALID_ARG;
  if (n_vec > ((int64_t)1 << 34)) return OSCAR_ERR_INVALID_ARG;
  if (n_vec == 0) return OSCAR_OK;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  int rc;
  if (flags & OSCAR_ROTATE_MATRIX_CORE) {
    // the H_16 factor's entries are exact in the operand type only for 16-bit inputs
    if (io_dtype == OSCAR_BF16) rc = launch_rotate_mfma<__hip_bfloat16>(x, out, norms, n_vec, meta_dtype, flags, st);
    else if (io_dtype == OSCAR_F16) rc = launch_rotate_mfma<__half>(x, out, norms, n_vec, meta_dtype, flags, st);
    else return io_dtype == OSCAR_F32 ? OSCAR_ERR_UNSUPPORTED : OSCAR_ERR_INVALID_ARG;
    if (rc != OSCAR_OK) return rc;
    if (hipGetLastError() != hipSuccess) return OSCAR_ERR_HIP;
    return OSCAR_OK;
  }
  switch (io_dtype) {
    case OSCAR_F32: rc = launch_rotate<float>(x, out, norms, n_vec, meta_dtype, flags, st); break;
    case OSCAR_BF16: rc = launch_rotate<__hip_bfloat16>(x, out, norms, n_vec, meta_dtype, flags, st); break;
    case OSCAR_F16: rc = launch_rotate<__half>(x, out, norms, n_vec, meta_dtype, flags, st); break;
    default: return OSCAR_ERR_INVALID_ARG;
  }
  if (rc != OSCAR_OK) return rc;
  if (hipGetLastError() != hipSuccess) return OSCAR_ERR_HIP;
  return OSCAR_OK;
}

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
  dim3 grid(cache->cfg.n_kv_heads, nblk, cache->batch);
  // The ticket saves a launch, and a workgroup that draws one holds its registers and LDS until
  // the counter's answer is back.  Worth it where a launch is what the call costs (a decode
  // step's one-token append, at any batch size); a multi-block append whose grid runs in many
  // rounds of workgroups updates the lengths with the small second kernel instead.
  if (nblk > 1 && (size_t)grid.x * grid.y * grid.z > kTicketMaxWorkgroups) P.c.tickets = nullptr;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (cache->cfg.norm_scope == OSCAR_NORM_ALL_KV_HEADS)
    rc = oscar_launch_append_all_heads(P, grid, st);
  else if (cache->cfg.rotation == OSCAR_ROTATION_ON && cache->cfg.scale_mode == OSCAR_SCALE_L2)
    rc = launch_append<XF_PUBLISHED>(P, grid, st);
  else
    rc = oscar_launch_append_switched(P, grid, st);
  if (rc != OSCAR_OK) return rc;
  if (hipGetLastError() != hipSuccess) return OSCAR_ERR_HIP;
  return OSCAR_OK;
}
