// Shared host/device helpers of the HIP library: page geometry, element
// conversions and launch-time parameter blocks.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "../../include/oscar.h"

#define OSCAR_D 128   // head dimension built
#define OSCAR_R 128   // page size / residual length built
#define OSCAR_MAX_GQA 8

// ---- page geometry (bytes per page of one kv head) -------------------------
struct PageGeom {
  int bits, k_group, v_group, meta_bytes;
  int ngk, ngv;
  int k_row_bytes;    // one token's key codes
  int v_row_bytes;    // one channel's value codes over the page
  int k_codes_bytes, k_meta_bytes, k_norms_bytes, v_codes_bytes, v_meta_bytes;
  __host__ __device__ int total() const {
    return k_codes_bytes + k_meta_bytes + k_norms_bytes + v_codes_bytes + v_meta_bytes;
  }
};

__host__ __device__ inline PageGeom make_geom(int bits, int k_group, int v_group, int meta_dtype) {
  PageGeom g;
  g.bits = bits;
  g.k_group = k_group;
  g.v_group = v_group;
  g.meta_bytes = (meta_dtype == OSCAR_F32) ? 4 : 2;
  g.ngk = OSCAR_R / k_group;
  g.ngv = OSCAR_D / v_group;
  g.k_row_bytes = OSCAR_D * bits / 8;
  g.v_row_bytes = OSCAR_R * bits / 8;
  g.k_codes_bytes = OSCAR_R * g.k_row_bytes;
  g.k_meta_bytes = 2 * g.ngk * OSCAR_D * g.meta_bytes;
  g.k_norms_bytes = OSCAR_R * g.meta_bytes;
  g.v_codes_bytes = OSCAR_D * g.v_row_bytes;
  g.v_meta_bytes = 2 * g.ngv * OSCAR_R * g.meta_bytes;
  return g;
}

// ---- in-page layouts --------------------------------------------------------
// The packed pools are laid out for the matrix-core decode kernel: a 64-lane wave
// loads one 16x(32 codes) operand tile with one contiguous, fully used access, and a
// lane's bytes are already in the order its MFMA operand registers want.
//
// A "chunk" is the 32 codes one lane owns of a 16 x 128 operand tile: lane (n, q4),
// n = row/column of the tile (0..15), q4 = quarter of the contraction axis (0..3).
// Inside a chunk, code number u (0..31) sits at bit u*bits (little endian) and feeds
// MFMA k-step kk (0..3), vector element e (0..7) with u = slot_index(kk, e): the order
// that falls out of unpacking 16-bit halves of a dword with masks only.
//   keys   : tile = 16 tokens (n = t % 16, T = t / 16); chunk q4 = channels 32*q4 .. 32*q4+31,
//            code u = channel 32*q4 + u.
//   values : tile = 16 channels (n = c % 16, ct = c / 16); chunk q4 = tokens with t % 4 == q4,
//            code slot_index(kk, e) = token 16*e + 4*kk + q4.
// Tiles are stored in pairs so that a lane's two chunks are 16 (2-bit) or 32 (4-bit)
// contiguous bytes: byte offset of chunk (tile, n, q4) =
//   ((tile/2)*64 + n*4 + q4) * 2*CB + (tile%2)*CB,  CB = 4*bits bytes per chunk.
__host__ __device__ constexpr int slot_index(int bits, int kk, int e) {
  return bits == 2 ? 16 * (kk / 2) + 4 * (kk % 2) + e / 2 + 8 * (e % 2)
                   : 8 * kk + e / 2 + 4 * (e % 2);
}
// Weight of a slot after shift-and-mask unpacking: the code lands at bit offset
// slot_bitpos of an fp16 lane's mantissa, i.e. as the number c * 2^slot_bitpos * 2^-24.
// Only offsets 4,6,8 are used for 2-bit codes and 2,6 for 4-bit codes: the MFMA aligns
// products by the operands' nominal exponents, so codes parked far below the top of the
// mantissa (or a wide spread of offsets) cost accumulation precision.
__host__ __device__ constexpr int slot_bitpos(int bits, int kk, int e) {
  if (bits == 2) {
    const int kap = 4 * (kk % 2) + e / 2;  // bit pair inside the 16-bit half
    return 2 * (kap == 0 ? 2 : kap == 1 ? 3 : kap <= 4 ? kap : kap - 3);
  }
  return ((e / 2) % 2) ? 6 : 2;
}
__host__ __device__ constexpr int slot_bitpos_min(int bits) { return bits == 2 ? 4 : 2; }
__host__ __device__ constexpr int chunk_bytes(int bits) { return 4 * bits; }
__host__ __device__ constexpr int chunk_offset(int bits, int tile, int n, int q4) {
  return ((tile / 2) * 64 + n * 4 + q4) * 2 * chunk_bytes(bits) + (tile % 2) * chunk_bytes(bits);
}
// value side: token t -> (q4, code number inside the chunk)
__host__ __device__ constexpr int vtok_q4(int t) { return t % 4; }
__host__ __device__ constexpr int vtok_slot(int bits, int t) {
  return slot_index(bits, (t / 4) % 4, t / 16);
}
// Per-token metadata (token norms, value Delta / zero) is stored in the order the
// logits come out of the QK^T tiles: position (t % 16) * 8 + t / 16.
__host__ __device__ constexpr int tok_meta_pos(int t) { return (t % 16) * 8 + t / 16; }
// Key Delta / zero are stored in operand order: position 32*q4 + 8*kk + e holds channel
// 32*q4 + slot_index(kk, e).
__host__ __device__ constexpr int kmeta_chan_of_pos(int bits, int pos) {
  return 32 * (pos / 32) + slot_index(bits, (pos % 32) / 8, pos % 8);
}
__host__ __device__ constexpr int kmeta_pos_of_chan(int bits, int j) {
  const int q4 = j / 32, u = j % 32;
  int kk = 0, e = 0;
  if (bits == 2) {
    const int d = u / 16, b = (u % 16) / 8, kap = u % 8;
    kk = 2 * d + kap / 4;
    e = 2 * (kap % 4) + b;
  } else {
    const int nu = u % 8;
    kk = u / 8;
    e = 2 * (nu % 4) + nu / 4;
  }
  return 32 * q4 + 8 * kk + e;
}

// ---- element conversions ----------------------------------------------------
template <typename T> __device__ __forceinline__ float to_f32(T x);
template <> __device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f32<__half>(__half x) { return __half2float(x); }
template <> __device__ __forceinline__ float to_f32<__hip_bfloat16>(__hip_bfloat16 x) {
  return __bfloat162float(x);
}

template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ __half from_f32<__half>(float x) { return __float2half_rn(x); }
template <> __device__ __forceinline__ __hip_bfloat16 from_f32<__hip_bfloat16>(float x) {
  return __float2bfloat16(x);
}

// Round a float to the metadata storage type and widen it back.  A value beyond the largest
// finite number of the type is stored as that number (no stored parameter is ever infinite):
// clamping to +-65504 first gives exactly that, since everything in (65504, 65520) rounds down
// to 65504 anyway.  fp32 storage is the identity.
template <typename M> __device__ __forceinline__ float round_meta(float x) {
  return to_f32<M>(from_f32<M>(x));
}
template <> __device__ __forceinline__ float round_meta<__half>(float x) {
  return __half2float(__float2half_rn(__builtin_amdgcn_fmed3f(x, -65504.0f, 65504.0f)));
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Host-side validation shared by the entry points.
int oscar_validate_config(const oscar_config* cfg);

// the pair of events behind the measurement-aid entry points
struct oscar_timer {
  hipEvent_t start, stop;
  int armed;
};

// Reduce pass of split-K decode (defined with the decode kernels).
void oscar_launch_decode_reduce(const float* ws, void* out, int num_splits, int out_dtype,
                                int n_q_heads, int batch, hipStream_t st);

// Matrix-core partial pass (params = the decode parameter block); returns
// OSCAR_ERR_UNSUPPORTED when the configuration must take the generic kernel.
// Resident workgroups per CU of the matrix-core decode kernel for a variant (bits, head slots,
// key groups per page, value groups); the launch bounds and the split heuristic share it.
__host__ __device__ constexpr int oscar_decode_mfma_wgs_per_cu(int bits, int hp, int ngk, int ngv) {
  // (measured, partial pass in us at one / two per CU: (4,1,4,4) 65 / 73 with 13 registers in
  // scratch, (4,2,1,4) 35 / 38, (4,2,2,4) 37 / 43; the other way round (2,2,4,4) 39 / 33,
  // (2,2,2,4) 34 / 30, (4,1,2,4) 62 / 60, (4,1,4,1) 62 / 59, (4,1,4,2) 63 / 61)
  if (hp == 1) return (bits == 4 && ngk == 4 && ngv == 4) ? 1 : 2;
  if (bits == 2) return 2;
  return (ngv == 1 && ngk <= 2) ? 2 : 1;
}
int oscar_launch_decode_mfma(const void* params, int gq, dim3 grid, hipStream_t st,
                             hipEvent_t e0, hipEvent_t e1);

#define OSCAR_HIP_CHECK(expr)                 \
  do {                                        \
    hipError_t e_ = (expr);                   \
    if (e_ != hipSuccess) return OSCAR_ERR_HIP; \
  } while (0)
