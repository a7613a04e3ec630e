// oscar_decode_attn, matrix-core path for gfx950 (v_mfma_f32_16x16x32_f16).
//
// Why matrix cores: at 86 bytes per token and kv head, 70 % of 8 TB/s leaves about 600
// plain-ALU lane operations per token and kv head on 256 CUs; the two GQA-batched
// contractions alone (q K^T and P V, 4..8 query heads per kv head) need 1024..2048 fused
// multiply-adds.  Everything that is a contraction therefore runs on MFMA; unpacking,
// softmax and scale folding stay on the vector ALU.
//
//   logit[h][t] = n_t * ( sum_j (Q_h[h][j] Delta_k[j]) c_k[t][j]  -  sum_j Q_h[h][j] Delta_k[j] z_k[j] )
//   out[h][c]   = sum_t (p[h][t] Delta_v[t][G(c)]) c_v[t][c]  -  sum_t p[h][t] Delta_v[t][G(c)] z_v[t][G(c)]
// (logits of App. "Implementation Details", "Overall Design"; dequantization of Eq. 3-4.)
//
// Exactness devices:
//  * Codes become fp16 operands with one AND per register and no offset: a code parked at
//    bit offset s of an fp16 lane's mantissa (exponent field zero) is the subnormal number
//    c * 2^s * 2^-24, and the MFMA keeps fp16 subnormals.  2^s is divided out of the other
//    operand.  Offsets stay near the top of the mantissa (see slot_bitpos).
//  * The other operand (Q_h*Delta_k, resp. p*Delta_v) is carried as fp16 hi + lo limbs in two
//    rows of the 16-row MFMA tile (rows are otherwise idle for GQA <= 8): hi + lo equals the
//    fp32 product to ~2^-21, the MFMA's products with the codes are exact and accumulation
//    is fp32.  The limbs come from packed fp16 arithmetic on a multiplicand split once
//    (mul_limbs_packed; mul_split_hi_lo is the mixed-precision form it replaced, still built
//    with OSCAR_LIMBS_PACKED = 0).
//  * Zero-points are subtracted analytically in fp32 (the two right-hand sums above).
//
// Work decomposition: grid (split, kv head, sequence); 4 waves per workgroup, every wave
// owns whole pages (no barriers in the page loop) and keeps its own online-softmax state;
// the 4 wave states and the workgroup's slice of the 16-bit residual tokens (plain ALU code,
// the window is dealt to the splits in multiples of 16 tokens) are merged through LDS at
// the end.
// Tile roles: q K^T uses M = query-head limb rows, N = 16 tokens, K = 128 channels;
// P V uses M = query-head limb rows, N = 16 channels, K = 128 tokens.  A lane of the logit
// tile is (token n, head group q4), which is also the lane that owns the 8-token operand
// vector (k-step n/4, quarter n%4) of the P V contraction: probabilities go to LDS as
// 16-byte vectors and come back as MFMA A-operands without any shuffle.
#include <atomic>

#include "oscar_decode_common.h"

// This file is compiled twice: as it stands for the integer zero-point of Eq. 3-4, and through
// oscar_decode_mfma_zpmin.hip with OSCAR_MFMA_ZPMIN = 1 for the float zero-point form; the
// zero-point form is a compile-time constant of the kernel (no branches in the page loop), and
// the two sets of variants compile side by side.
#ifndef OSCAR_MFMA_ZPMIN
#define OSCAR_MFMA_ZPMIN 0
#endif
#include "oscar_rowops.h"

// A prefetch that refills registers in place must not be moved, by the instruction scheduler,
// above the last read of the registers' old contents: the arriving data then lands in other
// registers and is copied home, and the copy waits for a load that was only just issued.
// The fence keeps vector-ALU and vector-memory instructions on their side of it; scalar,
// matrix and LDS instructions may still cross.
#ifndef OSCAR_PREFETCH_FENCE_MASK
#define OSCAR_PREFETCH_FENCE_MASK 0x38C
#endif
#define OSCAR_PREFETCH_FENCE() __builtin_amdgcn_sched_barrier(OSCAR_PREFETCH_FENCE_MASK)

#ifndef OSCAR_DECODE_PRIORITY
#define OSCAR_DECODE_PRIORITY 1
#endif

// Phase time stamps (measurement aid, off in the library proper: build.py --stamps makes a
// second library with them, phase_profile.py runs it).  Lane 0 of every wave of the first and
// the last four workgroups of the grid writes the constant-rate counter (100 MHz, the same on
// every CU) at the phase boundaries below; indices are masked, the array is fixed.
#ifdef OSCAR_DECODE_STAMPS
namespace {
__device__ unsigned long long g_stamps[8][4][32];
}
#define OSCAR_STAMP(i)                                                                  \
  do {                                                                                  \
    if (stamp_on && lane == 0) g_stamps[stamp_slot & 7][wave & 3][(i) & 31] = wall_clock64(); \
  } while (0)
#else
#define OSCAR_STAMP(i)
#endif

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// wave-local LDS hand-off: LDS operations of one wave execute in order; this only stops
// the compiler from moving accesses across the hand-off point.
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Reductions over the 16 lanes of a DPP row (= one head group): xor-1 and xor-2 inside
// quads, then the two mirrors; every lane ends with the same bits.
template <int CTRL> __device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_mov<0xB1>(v));   // quad_perm [1,0,3,2]
  v = fmaxf(v, dpp_mov<0x4E>(v));   // quad_perm [2,3,0,1]
  v = fmaxf(v, dpp_mov<0x141>(v));  // row_half_mirror
  v = fmaxf(v, dpp_mov<0x140>(v));  // row_mirror
  return v;
}
// The same reductions with the permutation folded into the max itself, for the page loop
// (the compiler's form is a move, a canonicalizing max and the max: three instructions a step).
// A DPP operand must not be read in the two issue slots after the register was written: each
// step starts with that wait, which the compiler cannot add inside the block.
#define OSCAR_DPP_MAX_STEPS(OP)                                                              \
  asm volatile("s_nop 1\n\t" OP " %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t" \
               "s_nop 1\n\t" OP " %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t" \
               "s_nop 1\n\t" OP " %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"     \
               "s_nop 1\n\t" OP " %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf"                \
               : "+v"(v))
__device__ __forceinline__ float row16_max_fast(float v) {   // no NaN among the inputs
  OSCAR_DPP_MAX_STEPS("v_max_f32_dpp");
  return v;
}
__device__ __forceinline__ uint32_t row16_max_u32(uint32_t v) {
  OSCAR_DPP_MAX_STEPS("v_max_u32_dpp");
  return v;
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_mov<0xB1>(v);
  v += dpp_mov<0x4E>(v);
  v += dpp_mov<0x141>(v);
  v += dpp_mov<0x140>(v);
  return v;
}

__device__ __forceinline__ void halves_to_f32(const uint4& r, float (&x)[8]) {
  const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __half2float(__ushort_as_half((unsigned short)(w[i] & 0xffffu)));
    x[2 * i + 1] = __half2float(__ushort_as_half((unsigned short)(w[i] >> 16)));
  }
}

// fp16 hi[8] + lo[8] limbs of the exact products x[i] * y[i] (y = 8 packed fp16 values):
// hi = f16(x*y), lo = f16(fma(x, y, -hi)), each a single mixed-precision FMA that reads its
// fp16 sources in place and writes one half of the destination register, so neither the
// multiplier nor the limbs are ever widened, subtracted or packed separately.
// hi + lo equals the product to ~2^-22.
// One block of 16 instructions: a half-register write must not be followed directly by a
// vector instruction that reads the register (the compiler cannot see into the block to
// insert the wait state itself); here every such read comes four instructions after the
// write, and the block ends with a wait state of its own.
__device__ __forceinline__ void mul_split_hi_lo(const float (&x)[8], const uint4& y, uint4& hi,
                                                uint4& lo) {
  uint32_t h0, h1, h2, h3, l0, l1, l2, l3;
  asm volatile("v_fma_mixlo_f16 %0, %8, %16, 0 op_sel_hi:[0,1,0]\n\t"
      "v_fma_mixlo_f16 %1, %10, %17, 0 op_sel_hi:[0,1,0]\n\t"
      "v_fma_mixlo_f16 %2, %12, %18, 0 op_sel_hi:[0,1,0]\n\t"
      "v_fma_mixlo_f16 %3, %14, %19, 0 op_sel_hi:[0,1,0]\n\t"
      "v_fma_mixhi_f16 %0, %9, %16, 0 op_sel:[0,1,0] op_sel_hi:[0,1,0]\n\t"
      "v_fma_mixhi_f16 %1, %11, %17, 0 op_sel:[0,1,0] op_sel_hi:[0,1,0]\n\t"
      "v_fma_mixhi_f16 %2, %13, %18, 0 op_sel:[0,1,0] op_sel_hi:[0,1,0]\n\t"
      "v_fma_mixhi_f16 %3, %15, %19, 0 op_sel:[0,1,0] op_sel_hi:[0,1,0]\n\t"
      "v_fma_mixlo_f16 %4, %8, %16, -%0 op_sel_hi:[0,1,1]\n\t"
      "v_fma_mixlo_f16 %5, %10, %17, -%1 op_sel_hi:[0,1,1]\n\t"
      "v_fma_mixlo_f16 %6, %12, %18, -%2 op_sel_hi:[0,1,1]\n\t"
      "v_fma_mixlo_f16 %7, %14, %19, -%3 op_sel_hi:[0,1,1]\n\t"
      "v_fma_mixhi_f16 %4, %9, %16, -%0 op_sel:[0,1,1] op_sel_hi:[0,1,1]\n\t"
      "v_fma_mixhi_f16 %5, %11, %17, -%1 op_sel:[0,1,1] op_sel_hi:[0,1,1]\n\t"
      "v_fma_mixhi_f16 %6, %13, %18, -%2 op_sel:[0,1,1] op_sel_hi:[0,1,1]\n\t"
      "v_fma_mixhi_f16 %7, %15, %19, -%3 op_sel:[0,1,1] op_sel_hi:[0,1,1]\n\t"
      "s_nop 0"
      : "=&v"(h0), "=&v"(h1), "=&v"(h2), "=&v"(h3), "=&v"(l0), "=&v"(l1), "=&v"(l2), "=&v"(l3)
      : "v"(x[0]), "v"(x[1]), "v"(x[2]), "v"(x[3]), "v"(x[4]), "v"(x[5]), "v"(x[6]), "v"(x[7]),
        "v"(y.x), "v"(y.y), "v"(y.z), "v"(y.w));
  hi = make_uint4(h0, h1, h2, h3);
  lo = make_uint4(l0, l1, l2, l3);
}

// The same limbs from packed fp16 arithmetic, for a multiplicand that serves several
// multipliers (the probabilities of a page against the step sizes of every value group, the
// queries against the step sizes of every page): x is split once into fp16 xh + xl (xl holds
// what the rounding of xh left over: x = xh + xl to 2^-22), and per multiplier
//   hi = xh * y,  e = fma(xh, y, -hi)  (the rounding error of that product, an fp16 number
//   unless it falls below the subnormal range),  lo = fma(xl, y, e)
// -- three packed instructions per two elements where the mixed-precision form takes four of
// twice the issue time.  hi + lo equals the product to ~2^-21.
#ifndef OSCAR_LIMBS_PACKED
#define OSCAR_LIMBS_PACKED 1
#endif
__device__ __forceinline__ void split_to_halves(const float (&x)[8], uint4& xh, uint4& xl) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  uint32_t h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const f32x2 v = {x[2 * i], x[2 * i + 1]};
    const half2v hh = __builtin_convertvector(v, half2v);
    const f32x2 r = {x[2 * i] - (float)hh[0], x[2 * i + 1] - (float)hh[1]};   // exact
    h[i] = __builtin_bit_cast(uint32_t, hh);
    l[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, half2v));
  }
  xh = make_uint4(h[0], h[1], h[2], h[3]);
  xl = make_uint4(l[0], l[1], l[2], l[3]);
}
__device__ __forceinline__ uint4 scale_halves(const uint4& y, half2v k) {
  const uint32_t c[4] = {y.x, y.y, y.z, y.w};
  uint32_t r[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) r[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2v, c[i]) * k);
  return make_uint4(r[0], r[1], r[2], r[3]);
}
__device__ __forceinline__ void mul_limbs_packed(const uint4& xh, const uint4& xl, const uint4& y,
                                                 uint4& hi, uint4& lo) {
  const uint32_t a[4] = {xh.x, xh.y, xh.z, xh.w}, b[4] = {xl.x, xl.y, xl.z, xl.w};
  const uint32_t c[4] = {y.x, y.y, y.z, y.w};
  uint32_t h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const half2v ah = __builtin_bit_cast(half2v, a[i]), al = __builtin_bit_cast(half2v, b[i]);
    const half2v yy = __builtin_bit_cast(half2v, c[i]);
    const half2v p = ah * yy;
    const half2v e = __builtin_elementwise_fma(ah, yy, -p);
    const half2v q = __builtin_elementwise_fma(al, yy, e);
    h[i] = __builtin_bit_cast(uint32_t, p);
    l[i] = __builtin_bit_cast(uint32_t, q);
  }
  hi = make_uint4(h[0], h[1], h[2], h[3]);
  lo = make_uint4(l[0], l[1], l[2], l[3]);
}

// Products of packed fp16 pairs in fp32, and fp16 * fp32, without widening instructions:
// the mixed-precision FMA reads fp16 sources in place.  (The wrong logits that a (32,32)-group
// build once showed with these blocks as plain asm came from an output register placed on the
// destination of a matrix instruction in flight, see keep_tuple; with that fixed they work as
// plain asm too, and stay volatile only because nothing is gained by letting them move.)
__device__ __forceinline__ void mix_mul_pair(uint32_t a, uint32_t b, float& lo, float& hi) {
  asm volatile("v_fma_mix_f32 %0, %1, %2, 0 op_sel_hi:[1,1,0]" : "=v"(lo) : "v"(a), "v"(b));
  asm volatile("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[1,1,0] op_sel_hi:[1,1,0]" : "=v"(hi) : "v"(a), "v"(b));
}
// -(fp16 value), widened: the zero-point term of the float zero-point mode
__device__ __forceinline__ void neg_widen8(const uint4& a, float (&x)[8]) {
  const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = -__half2float(__ushort_as_half((unsigned short)(w[i] & 0xffffu)));
    x[2 * i + 1] = -__half2float(__ushort_as_half((unsigned short)(w[i] >> 16)));
  }
}
__device__ __forceinline__ void mix_mul8(const uint4& a, const uint4& b, float (&x)[8]) {
  mix_mul_pair(a.x, b.x, x[0], x[1]);
  mix_mul_pair(a.y, b.y, x[2], x[3]);
  mix_mul_pair(a.z, b.z, x[4], x[5]);
  mix_mul_pair(a.w, b.w, x[6], x[7]);
}
// x * (fp16 half `hi_half` of packed h)
template <int HI> __device__ __forceinline__ float mix_scale(float x, uint32_t h) {
  float r;
  if (HI) asm volatile("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[0,1,0] op_sel_hi:[0,1,0]" : "=v"(r) : "v"(x), "v"(h));
  else asm volatile("v_fma_mix_f32 %0, %1, %2, 0 op_sel_hi:[0,1,0]" : "=v"(r) : "v"(x), "v"(h));
  return r;
}

// The unpack masks live in vector registers.  Measured on gfx950 with two or more waves per
// SIMD: a v_and_b32 or v_lshrrev_b32 whose operands are vector registers (or a literal) issues in
// about 2.6 clocks per wave, the same instruction with a scalar-register operand in 4.5 -- so the
// masks are kept out of scalar registers (where the compiler puts such loop constants).
template <int BITS> struct Masks {
  uint32_t m0, m1, m2;
  __device__ __forceinline__ void init() {
    m0 = BITS == 2 ? 0x00300030u : 0x003C003Cu;
    m1 = BITS == 2 ? 0x00C000C0u : 0x03C003C0u;
    m2 = 0x03000300u;
    asm volatile("" : "+v"(m0), "+v"(m1));
    if (BITS == 2) asm volatile("" : "+v"(m2));
  }
};

// All four registers of a matrix-instruction result stay allocated up to this point, also the
// ones nobody reads (rows of absent heads).  Without it the register allocator hands such a
// register to the next value while the instruction that will still write it is in flight; for
// its own instructions the compiler then inserts the wait states the hardware asks for, for the
// instructions inside an asm block it cannot -- and the result of a block placed there was
// overwritten when the matrix instruction retired (seen as run-to-run differences of a build
// whose only change was the order of the matrix instructions).
__device__ __forceinline__ void keep_tuple(const float4v& t) { asm volatile("" ::"v"(t)); }

// One 32-code chunk -> the four B-operand vectors (k-steps 0..3) of a 16x16x32 MFMA.
template <int BITS> struct Chunk;
template <> struct Chunk<2> {
  uint32_t w[2];
  __device__ __forceinline__ void operands(u32x4 (&b)[4], const Masks<2>& m) const {
#pragma unroll
    for (int d = 0; d < 2; ++d) {
      // bit pairs 0,1 via << 4 (-> positions 4, 6), pairs 2,3,4 in place, pairs 5,6,7 via >> 6
      const uint32_t x = w[d], y = x >> 6, z = x << 4;
      b[2 * d] = (u32x4){z & m.m0, z & m.m1, x & m.m0, x & m.m1};
      b[2 * d + 1] = (u32x4){x & m.m2, y & m.m0, y & m.m1, y & m.m2};
    }
  }
};
template <> struct Chunk<4> {
  uint32_t w[4];
  __device__ __forceinline__ void operands(u32x4 (&b)[4], const Masks<4>& m) const {
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      // nibbles 0,1 via << 2 (-> bit offsets 2, 6), nibbles 2,3 via >> 6
      const uint32_t x = w[d], y = x >> 6, z = x << 2;
      b[d] = (u32x4){z & m.m0, z & m.m1, y & m.m0, y & m.m1};
    }
  }
};

// Page loads go through raw buffer resources, one per pool.  The resource's base is fixed for
// the whole kernel (pool + kv head * page bytes) and spans one page; the page itself is
// selected by the scalar offset of the load (physical page * kv heads * page bytes), so a new
// page costs a scalar multiply and add per pool instead of a 64-bit address computation.  The
// hardware's range check compares the per-lane offset with (number of records - scalar
// offset), so the record count of a live resource is the end of its page.  The per-lane offset is a loop constant, and a resource of
// zero length turns the prefetch past a wave's last page into loads that return zeros without
// touching memory -- the prefetch needs no branch, so the loaded registers are plain
// loop-carried values (a conditional load made the compiler copy the whole register set, and
// wait for it, at the end of every iteration).  A single wave issues one instruction about
// every five clocks whatever its kind, so scalar bookkeeping in the page loop is not free.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t pool_rsrc(const uint8_t* base, uint32_t page_off,
                                                            int bytes, bool valid) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base), 0,
                                           valid ? (int)(page_off + (uint32_t)bytes) : 0, 0x00020000);
}
// Loads are marked non-temporal (streaming): every byte of the cache is read once per launch,
// and keeping it out of the way of the small kernels around this one took 3 us off a decode
// step on the 32K-context workload (1 us off this kernel).
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, int off, uint32_t soff = 0) {
  return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(r, off, (int)soff, 2));
}

// A lane's two chunks of a tile pair: 16 bytes (2-bit) or 32 bytes (4-bit).
template <int BITS> struct TilePair;
template <> struct TilePair<2> {
  uint4 v;
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int off, uint32_t so) { v = buf_load16(r, off, so); }
  __device__ __forceinline__ Chunk<2> chunk(int i) const {
    Chunk<2> c;
    c.w[0] = i ? v.z : v.x;
    c.w[1] = i ? v.w : v.y;
    return c;
  }
};
template <> struct TilePair<4> {
  uint4 v[2];
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, int off, uint32_t so) {
    v[0] = buf_load16(r, off, so);
    v[1] = buf_load16(r, off + 16, so);
  }
  __device__ __forceinline__ Chunk<4> chunk(int i) const {
    Chunk<4> c;
    c.w[0] = v[i].x; c.w[1] = v[i].y; c.w[2] = v[i].z; c.w[3] = v[i].w;
    return c;
  }
};

// The pools' bases for one kv head and the byte strides between physical pages (wave-uniform).
struct PoolBases {
  const uint8_t *kcodes, *kmeta, *knorm, *vcodes, *vmeta;
  uint32_t s_kcodes, s_kmeta, s_knorm, s_vcodes, s_vmeta;
  __device__ __forceinline__ void make(const DecodeParams& P, int kvh) {
    const uint32_t Hkv = (uint32_t)P.c.cfg.n_kv_heads;
    kcodes = static_cast<const uint8_t*>(P.c.k_codes) + (size_t)kvh * P.g.k_codes_bytes;
    kmeta = static_cast<const uint8_t*>(P.c.k_meta) + (size_t)kvh * P.g.k_meta_bytes;
    knorm = static_cast<const uint8_t*>(P.c.k_norms) + (size_t)kvh * P.g.k_norms_bytes;
    vcodes = static_cast<const uint8_t*>(P.c.v_codes) + (size_t)kvh * P.g.v_codes_bytes;
    vmeta = static_cast<const uint8_t*>(P.c.v_meta) + (size_t)kvh * P.g.v_meta_bytes;
    s_kcodes = Hkv * (uint32_t)P.g.k_codes_bytes;
    s_kmeta = Hkv * (uint32_t)P.g.k_meta_bytes;
    s_knorm = Hkv * (uint32_t)P.g.k_norms_bytes;
    s_vcodes = Hkv * (uint32_t)P.g.v_codes_bytes;
    s_vmeta = Hkv * (uint32_t)P.g.v_meta_bytes;
  }
};
// The five buffer resources of one page and the page's scalar offsets (wave-uniform).
struct PageRsrc {
  __amdgpu_buffer_rsrc_t kcodes, kmeta, knorm, vcodes, vmeta;
  uint32_t o_kcodes, o_kmeta, o_knorm, o_vcodes, o_vmeta;
  __device__ __forceinline__ void make(const PoolBases& B, const DecodeParams& P, uint32_t phys, bool valid) {
    o_kcodes = phys * B.s_kcodes;
    o_kmeta = phys * B.s_kmeta;
    o_knorm = phys * B.s_knorm;
    o_vcodes = phys * B.s_vcodes;
    o_vmeta = phys * B.s_vmeta;
    kcodes = pool_rsrc(B.kcodes, o_kcodes, P.g.k_codes_bytes, valid);
    kmeta = pool_rsrc(B.kmeta, o_kmeta, P.g.k_meta_bytes, valid);
    knorm = pool_rsrc(B.knorm, o_knorm, P.g.k_norms_bytes, valid);
    vcodes = pool_rsrc(B.vcodes, o_vcodes, P.g.v_codes_bytes, valid);
    vmeta = pool_rsrc(B.vmeta, o_vmeta, P.g.v_meta_bytes, valid);
  }
};

// What one wave needs of one page, in registers, single-buffered: every register is
// reloaded for the wave's next page right after its last use for the current one, so each
// load has a whole iteration to arrive and only one copy of a page is ever live.
template <int BITS, int NGK> struct KeyRegs {
  static constexpr int PB = 2 * chunk_bytes(BITS);  // bytes of a lane's tile pair
  TilePair<BITS> kc[4];
  uint4 kd[NGK], kz[NGK];  // key Delta / zero of positions 8n..8n+7 (operand order)
  uint4 nr;                // norms of tokens 16*T+n, T = 0..7
  __device__ __forceinline__ void load_codes(const PageRsrc& r, int tp, int lane) {
    kc[tp].load(r.kcodes, (tp * 64 + (lane & 15) * 4 + (lane >> 4)) * PB, r.o_kcodes);
  }
  __device__ __forceinline__ void load_meta(const PageRsrc& r, int g, int lane) {
    kd[g] = buf_load16(r.kmeta, (g * D + 8 * (lane & 15)) * 2, r.o_kmeta);
    kz[g] = buf_load16(r.kmeta, ((NGK + g) * D + 8 * (lane & 15)) * 2, r.o_kmeta);
  }
  __device__ __forceinline__ void load_norm(const PageRsrc& r, int lane) {
    nr = buf_load16(r.knorm, 8 * (lane & 15) * 2, r.o_knorm);
  }
  __device__ __forceinline__ void load(const PageRsrc& r, int lane) {
#pragma unroll
    for (int tp = 0; tp < 4; ++tp) load_codes(r, tp, lane);
#pragma unroll
    for (int g = 0; g < NGK; ++g) load_meta(r, g, lane);
    load_norm(r, lane);
  }
};
template <int BITS, int NGV> struct ValRegs {
  static constexpr int PB = 2 * chunk_bytes(BITS);
  TilePair<BITS> vc[4];
  uint4 vd[NGV], vz[NGV];  // value Delta / zero of tokens 16*T+n
  __device__ __forceinline__ void load_codes(const PageRsrc& r, int tp, int lane) {
    vc[tp].load(r.vcodes, (tp * 64 + (lane & 15) * 4 + (lane >> 4)) * PB, r.o_vcodes);
  }
  __device__ __forceinline__ void load_delta(const PageRsrc& r, int g, int lane) {
    vd[g] = buf_load16(r.vmeta, (g * R + 8 * (lane & 15)) * 2, r.o_vmeta);
  }
  __device__ __forceinline__ void load_zero(const PageRsrc& r, int g, int lane) {
    vz[g] = buf_load16(r.vmeta, ((NGV + g) * R + 8 * (lane & 15)) * 2, r.o_vmeta);
  }
  __device__ __forceinline__ void load(const PageRsrc& r, int lane) {
#pragma unroll
    for (int tp = 0; tp < 4; ++tp) load_codes(r, tp, lane);
#pragma unroll
    for (int g = 0; g < NGV; ++g) {
      load_delta(r, g, lane);
      load_zero(r, g, lane);
    }
  }
};

// Eight consecutive values of the caller's dtype (a run-time property here), held raw.
// Loads are buffer loads without branches: a branch around a load makes the compiler wait
// for every load in flight where the branches join (the start of this kernel was a chain of
// such waits: each residual token's loads completed, behind the whole first page, before the
// next token's were issued).  fp32 needs 32 bytes; the upper 16 come through a second
// resource that is void for the 16-bit types.
struct IoRsrc {
  __amdgpu_buffer_rsrc_t lo, hi;
  int es;   // bytes per element
  __device__ __forceinline__ void make(const void* base, size_t first_elem, int n_elem, int dt,
                                       bool valid) {
    es = dt == OSCAR_F32 ? 4 : 2;
    uint8_t* p = const_cast<uint8_t*>(static_cast<const uint8_t*>(base)) + first_elem * (size_t)es;
    lo = __builtin_amdgcn_make_buffer_rsrc(p, 0, valid ? n_elem * es : 0, 0x00020000);
    hi = __builtin_amdgcn_make_buffer_rsrc(p, 0, (valid && dt == OSCAR_F32) ? n_elem * es : 0, 0x00020000);
  }
};
struct Raw8rt {
  uint4 a, b;
  // elements elem .. elem+7 of the resource (zeros past its end)
  __device__ __forceinline__ void load(const IoRsrc& r, int elem) {
    a = buf_load16(r.lo, elem * r.es);
    b = buf_load16(r.hi, elem * r.es + 16);
  }
  __device__ __forceinline__ void widen(float (&x)[8], int dt) const {
    if (dt == OSCAR_F32) {
      x[0] = __uint_as_float(a.x); x[1] = __uint_as_float(a.y);
      x[2] = __uint_as_float(a.z); x[3] = __uint_as_float(a.w);
      x[4] = __uint_as_float(b.x); x[5] = __uint_as_float(b.y);
      x[6] = __uint_as_float(b.z); x[7] = __uint_as_float(b.w);
    } else if (dt == OSCAR_BF16) {
      x[0] = __uint_as_float(a.x << 16); x[1] = __uint_as_float(a.x & 0xffff0000u);
      x[2] = __uint_as_float(a.y << 16); x[3] = __uint_as_float(a.y & 0xffff0000u);
      x[4] = __uint_as_float(a.z << 16); x[5] = __uint_as_float(a.z & 0xffff0000u);
      x[6] = __uint_as_float(a.w << 16); x[7] = __uint_as_float(a.w & 0xffff0000u);
    } else {
      halves_to_f32(a, x);
    }
  }
};

// The residual window of one (sequence, kv head) as buffer resources: K_u (fp16), V (caller's
// dtype), token norms (fp16 here: this kernel requires fp16 metadata); void when the wave has
// no residual token.
struct ResRsrc {
  __amdgpu_buffer_rsrc_t k, n;
  IoRsrc v;
  __device__ __forceinline__ void make(const DecodeParams& P, size_t rb, bool valid) {
    uint8_t* kp = const_cast<uint8_t*>(static_cast<const uint8_t*>(P.c.res_k)) + rb * D * 2;
    uint8_t* np = const_cast<uint8_t*>(static_cast<const uint8_t*>(P.c.res_norm)) + rb * 2;
    k = __builtin_amdgcn_make_buffer_rsrc(kp, 0, valid ? R * D * 2 : 0, 0x00020000);
    n = __builtin_amdgcn_make_buffer_rsrc(np, 0, valid ? R * 2 : 0, 0x00020000);
    v.make(P.c.res_v, rb * D, R * D, P.c.cfg.io_dtype, valid);
  }
};

// One residual token's share for a lane: 8 channels (channel group cg) of K_u (fp16) and of
// V (caller's dtype), and the token norm, held raw until the query rotation is done.
// `tok` is the token's slot in the window, clamped by the caller to a slot that exists.
struct ResTok {
  uint4 k;
  Raw8rt v;
  uint32_t nrm;
  __device__ __forceinline__ void load(const ResRsrc& r, int tok, int cg) {
    k = buf_load16(r.k, (tok * D + 8 * cg) * 2);
    v.load(r.v, tok * D + 8 * cg);
    nrm = (uint32_t)(unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r.n, tok * 2, 0, 0);
  }
};
// Step sizes are non-negative fp16 numbers, which order like their bit patterns: packed
// unsigned 16-bit max needs no NaN canonicalization.
typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2v, a),
                                                                __builtin_bit_cast(ushort2v, b)));
}
__device__ __forceinline__ uint4 pk_max4(const uint4& a, const uint4& b) {
  return make_uint4(pk_max_u16(a.x, b.x), pk_max_u16(a.y, b.y), pk_max_u16(a.z, b.z),
                    pk_max_u16(a.w, b.w));
}

// rows of the 16-row operand tile: head h -> hi row 4*(h%4) + 2*(h/4), lo row + 1, so the
// accumulator lane group q4 (rows 4*q4..4*q4+3) owns heads q4 (slot 0) and q4+4 (slot 1).
__device__ __forceinline__ int row_hi(int h) { return 4 * (h & 3) + 2 * (h >> 2); }

// HP = head slots per accumulator lane group: 1 for up to 4 query heads per kv head, 2 for
// 5..8 (twice the per-head registers).  Two workgroups per CU wherever the registers allow it
// with little or no scratch memory (oscar_decode_mfma_wgs_per_cu lists the variants); the
// rest run one workgroup per CU and their overflow lives in accumulation registers
// (measured: 4-bit, G_k = 32 took 188 us with 65 spilled registers at two per CU, 76 us at
// one).
__host__ __device__ constexpr int decode_mfma_wgs_per_cu(int bits, int hp, int ngk, int ngv) {
  return oscar_decode_mfma_wgs_per_cu(bits, hp, ngk, ngv);
}

template <int BITS, int HP, int NGK, int NGV, bool ZPMIN>
__global__ __launch_bounds__(256, decode_mfma_wgs_per_cu(BITS, HP, NGK, NGV))
void oscar_decode_mfma_kernel(DecodeParams P, int gq) {
  constexpr int TPG = 8 / NGK;  // token tiles per key group
  constexpr int CPG = 8 / NGV;  // channel tiles per value group
  constexpr int TABW = D + 8;   // operand table row stride in halves
  // operand tiles unpacked one at a time (instead of in pairs) where the pair's second
  // register set would not fit
  constexpr bool ONE_TILE = (HP == 2) || (NGK == 4);

  // rows padded by 16 bytes: the 16-byte operand reads of lanes n = 0..7 hit 8 different banks
  __shared__ __align__(16) _Float16 s_A[4][16][TABW];   // per wave: (Q_h Delta_k) hi/lo rows
  __shared__ __align__(16) _Float16 s_P[4][16][TABW];   // per wave: (p Delta_v) hi/lo rows
  __shared__ __align__(16) float s_o[4][OSCAR_MAX_GQA][D];  // wave results for the merge
  __shared__ float s_wm[4][OSCAR_MAX_GQA], s_wl[4][OSCAR_MAX_GQA];
  // two head slots: the rotated queries in operand order wait in LDS between pages instead of
  // registers (16 registers that the second slot's softmax state needs)
  __shared__ __align__(16) float4 s_qr[HP == 2 ? 4 : 1][HP == 2 ? 2 : 1][2][HP == 2 ? 64 : 1];

  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63;
  // wave index as a scalar: page numbers and block-table lookups stay on the scalar unit
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, q4 = lane >> 4;
#ifdef OSCAR_DECODE_STAMPS
  const bool stamp_first = kvh == 0 && b == 0 && split < 4;
  const bool stamp_last = kvh == (int)gridDim.y - 1 && b == (int)gridDim.z - 1 && split < 4;
  const bool stamp_on = stamp_first || stamp_last;
  const int stamp_slot = (stamp_last ? 4 : 0) + (split & 3);
#endif
  OSCAR_STAMP(0);   // entry
  // highest priority from the start (it falls in the page loop, see there): the workgroup that
  // reached the CU second should not get its first loads out behind the first one's prologue
  if (OSCAR_DECODE_PRIORITY) __builtin_amdgcn_s_setprio(3);
  const int Hkv = P.c.cfg.n_kv_heads, Hq = P.c.cfg.n_q_heads;
  constexpr bool zp_min = ZPMIN;

  // Pages are dealt round-robin: wave w of split s owns pages 4*s + w + 4*S*k.  The page
  // numbers (and so the block-table addresses) do not depend on the sequence length, which
  // lets the length, table, query and residual loads all start together.
  const int pstride = 4 * P.num_splits;
  const int pg_first = 4 * split + wave;
  const int32_t* table = P.c.block_table + (size_t)b * P.c.max_pages_per_seq;
  // Block-table entries of this wave's pages live in a register, one per lane, 64
  // iterations at a time: the page loop itself issues no dependent lookups.  Entries past
  // the sequence's last page are never used for an access.
  auto load_table = [&](int it0) -> int {
    const int idx = pg_first + pstride * (it0 + lane);
    return idx < P.c.max_pages_per_seq ? table[idx] : 0;
  };
  OSCAR_STAMP(1 + (P.num_splits & 0));   // kernel arguments have arrived
  int tab = load_table(0);
  // queries: DPP row q4 of every wave takes head q4 (and q4 + 4 in the second slot), 8
  // channels (channel group cg) per lane; absent heads read as zeros
  const int cg = channel_group_of_row_lane(n);
  Raw8rt qraw[HP];
  {
    IoRsrc qr_;   // the group's gq query vectors; heads past gq fall off its end and read zeros
    qr_.make(P.q, ((size_t)b * Hq + (size_t)kvh * gq) * D, gq * D, P.c.cfg.io_dtype, true);
#pragma unroll
    for (int s = 0; s < HP; ++s) qraw[s].load(qr_, (q4 + 4 * s) * D + 8 * cg);
  }

  const int seq_len = P.c.seq_lens[b];
  const int r = P.c.res_lens[b];
  const int n_pages = (seq_len - r) / R;
  // Residual slice of this split: rs tokens per split (a multiple of 16), handed out from
  // the last split backwards; inside the workgroup, wave w takes tokens 16*pass + 4*w + j.
  const int rs = 16 * ((((r + 15) >> 4) + P.num_splits - 1) / P.num_splits);
  const int t_lo = min(r, (P.num_splits - 1 - split) * rs);
  const int rcount = min(r, t_lo + rs) - t_lo;
  const bool wave_res = 4 * wave < rcount;

  // ---- first residual pass and first page: issued before anything is computed.  The residual
  // tokens go first: they need no block-table entry, they are few, and the plain-ALU attention
  // over them then runs while the page is still on its way.  Waves without residual tokens skip
  // their loads (a void load still takes its turn in the CU's address unit, and at kernel start
  // all eight waves of a CU queue there). ----
  ResRsrc rres;
  rres.make(P, ((size_t)b * Hkv + kvh) * R, wave_res);
  // slot of the wave's token i of pass p0, clamped to the slice (masked where it is used)
  auto res_slot = [&](int p0, int i) { return t_lo + max(0, min(p0 + 4 * wave + i, rcount - 1)); };
  ResTok rt_first[4];   // the wave's four tokens of the first residual pass
  if (wave_res) {
#pragma unroll
    for (int i = 0; i < 4; ++i) rt_first[i].load(rres, res_slot(0, i), cg);
  }
  PoolBases pools;
  pools.make(P, kvh);
  KeyRegs<BITS, NGK> kr;
  ValRegs<BITS, NGV> vr;
  PageRsrc first;
  first.make(pools, P, (uint32_t)__builtin_amdgcn_readlane(tab, 0), pg_first < n_pages);
  kr.load(first, lane);
  __builtin_amdgcn_sched_barrier(0);
  OSCAR_STAMP(2);   // first page's key-side loads issued

  // this wave's operand tables start as zeros (rows of absent heads stay zero)
  for (int i = lane; i < 16 * TABW / 8; i += 64) {
    reinterpret_cast<uint4*>(&s_A[wave][0][0])[i] = make_uint4(0u, 0u, 0u, 0u);
    reinterpret_cast<uint4*>(&s_P[wave][0][0])[i] = make_uint4(0u, 0u, 0u, 0u);
  }
  // Q_h = H(q)/sqrt(128) * scale*log2(e), every wave for itself (DPP butterflies inside the
  // row, no LDS, no workgroup barrier): qh[s][i] = channel 8*cg + i of head q4 + 4*s
  uint32_t sgn[4];
  butterfly_signs(cg, sgn);
  float qh[HP][8];
#pragma unroll
  for (int s = 0; s < HP; ++s) {
    qraw[s].widen(qh[s], P.c.cfg.io_dtype);
    if (P.c.cfg.rotation == OSCAR_ROTATION_ON) rotate8(qh[s], sgn);
#pragma unroll
    for (int i = 0; i < 8; ++i) qh[s][i] *= P.qk_scale_log2;
  }

  // The first page's value side is asked for only now: all waves of the grid ask for their
  // first page at the same moment, and with the key side of every wave ahead of every value
  // side in the memory system's queues the first logits start earlier (about 1 % on the
  // small-batch workloads, nothing on the others).
  __builtin_amdgcn_sched_barrier(0);
  vr.load(first, lane);
  __builtin_amdgcn_sched_barrier(0);
  OSCAR_STAMP(3);   // queries rotated
  // ---- wave state: online softmax over this wave's pages, seeded by its residual tokens ----
  float m_run[HP], l_run[HP], bv[HP][NGV];
  float4v O[8];
#pragma unroll
  for (int s = 0; s < HP; ++s) {
    m_run[s] = -INFINITY;
    l_run[s] = 0.0f;
#pragma unroll
    for (int g = 0; g < NGV; ++g) bv[s][g] = 0.0f;
  }
#pragma unroll
  for (int ct = 0; ct < 8; ++ct) O[ct] = (float4v){0.0f, 0.0f, 0.0f, 0.0f};
  // accumulator scale: O holds out * 2^-(24 - xv_cur - offset); this start value makes it 1
  int xv_cur = 24 - slot_bitpos_min(BITS);

  // ---- residual tokens: plain-ALU attention over fp16 K_u and raw V, wave-local.  Row q4
  // works for head q4 (+4) on all four tokens of the wave's pass, a lane on its 8 channels:
  // logits are reduced over the 16 lanes of the row, nothing crosses rows.  The result
  // becomes the starting state of the wave's accumulators, so it costs no barrier. ----
  if (wave_res) {
    float mw[HP], lw[HP], ow[HP][8];
#pragma unroll
    for (int s = 0; s < HP; ++s) {
      mw[s] = -INFINITY;
      lw[s] = 0.0f;
#pragma unroll
      for (int c = 0; c < 8; ++c) ow[s][c] = 0.0f;
    }
    // (the raw norms stay opaque until here: converted where they were loaded, they made the
    // wave wait for the loads, and for the whole first page behind them, before the query rotation)
#pragma unroll
    for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(rt_first[i].nrm));
    for (int p0 = 0; p0 + 4 * wave < rcount; p0 += 16) {
      float sc[HP][4], vv[4][8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ResTok rt = rt_first[i];
        if (p0 > 0) rt.load(rres, res_slot(p0, i), cg);
        const bool valid = p0 + 4 * wave + i < rcount;   // wave-uniform
        float kv[8];
        halves_to_f32(rt.k, kv);
        rt.v.widen(vv[i], P.c.cfg.io_dtype);
        const float nrm = __half2float(__ushort_as_half((unsigned short)rt.nrm));
#pragma unroll
        for (int s = 0; s < HP; ++s) {
          float acc = qh[s][0] * kv[0];
#pragma unroll
          for (int c = 1; c < 8; ++c) acc = fmaf(qh[s][c], kv[c], acc);
          sc[s][i] = valid ? nrm * row16_sum(acc) : -INFINITY;
        }
      }
#pragma unroll
      for (int s = 0; s < HP; ++s) {
        // the wave's first token of a pass is valid, so the maximum is finite
        const float m_new = fmaxf(fmaxf(mw[s], fmaxf(sc[s][0], sc[s][1])), fmaxf(sc[s][2], sc[s][3]));
        const float alpha = __builtin_amdgcn_exp2f(mw[s] - m_new);
        mw[s] = m_new;
        lw[s] *= alpha;
#pragma unroll
        for (int c = 0; c < 8; ++c) ow[s][c] *= alpha;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float pw = __builtin_amdgcn_exp2f(sc[s][i] - m_new);
          lw[s] += pw;
#pragma unroll
          for (int c = 0; c < 8; ++c) ow[s][c] = fmaf(pw, vv[i][c], ow[s][c]);
        }
      }
    }
    // hand the result over in accumulator layout through the wave's own slice of s_o
    // (written again only by this wave: for the query hand-off below and at the very end)
#pragma unroll
    for (int s = 0; s < HP; ++s) {
      const int h = q4 + 4 * s;
      if (h < gq) {
        *reinterpret_cast<float4*>(&s_o[wave][h][8 * cg]) = make_float4(ow[s][0], ow[s][1], ow[s][2], ow[s][3]);
        *reinterpret_cast<float4*>(&s_o[wave][h][8 * cg + 4]) = make_float4(ow[s][4], ow[s][5], ow[s][6], ow[s][7]);
      }
    }
    wave_lds_fence();
#pragma unroll
    for (int s = 0; s < HP; ++s) {
      const int h = q4 + 4 * s;
      if (h < gq) {
        m_run[s] = mw[s];
        l_run[s] = (n == 0) ? lw[s] : 0.0f;   // l_run is summed over the 16 lanes at the end
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) O[ct][2 * s] = s_o[wave][h][16 * ct + n];
      }
    }
    wave_lds_fence();
  }
  // rotated queries -> operand order, through the same wave-local slice
#pragma unroll
  for (int s = 0; s < HP; ++s) {
    const int h = q4 + 4 * s;
    if (h < gq) {
      *reinterpret_cast<float4*>(&s_o[wave][h][8 * cg]) = make_float4(qh[s][0], qh[s][1], qh[s][2], qh[s][3]);
      *reinterpret_cast<float4*>(&s_o[wave][h][8 * cg + 4]) = make_float4(qh[s][4], qh[s][5], qh[s][6], qh[s][7]);
    }
  }
  wave_lds_fence();

  // ---- per-lane constants ----
  // writer role for the key operand: positions 8n..8n+7 of heads q4 (+4)
  float qr[HP][8], qs[HP][8], ps[HP];
#if OSCAR_LIMBS_PACKED
  uint4 qsh[HP], qsl[HP];   // qs as fp16 limbs
#endif
#pragma unroll
  for (int s = 0; s < HP; ++s) {
    const int h = q4 + 4 * s;
    float mx = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int chan = 32 * (n >> 2) + slot_index(BITS, n & 3, i);
      qr[s][i] = (h < gq) ? s_o[wave][h][chan] : 0.0f;
      mx = fmaxf(mx, fabsf(qr[s][i]));
    }
    mx = row16_max(mx);
    int ex = 0;
    (void)frexpf(mx, &ex);           // mx < 2^ex
    if (mx == 0.0f) ex = 0;
    // |Q_h| * 2^(xh - bitpos) < 2^14 for every slot, and Delta_k <= 1
    const int xh = 14 + slot_bitpos_min(BITS) - ex;
#pragma unroll
    for (int i = 0; i < 8; ++i) qs[s][i] = ldexpf(qr[s][i], xh - slot_bitpos(BITS, n & 3, i));
    ps[s] = ldexpf(1.0f, 24 - xh);
#if OSCAR_LIMBS_PACKED
    split_to_halves(qs[s], qsh[s], qsl[s]);
#endif
    if constexpr (HP == 2) {
      s_qr[wave][s][0][lane] = make_float4(qr[s][0], qr[s][1], qr[s][2], qr[s][3]);
      s_qr[wave][s][1][lane] = make_float4(qr[s][4], qr[s][5], qr[s][6], qr[s][7]);
    }
  }
  // value side: this lane's tokens 16*T+n feed k-step n/4, element T
  float vsc0[8];
#pragma unroll
  for (int T = 0; T < 8; ++T)
    vsc0[T] = ldexpf(1.0f, slot_bitpos_min(BITS) - slot_bitpos(BITS, n >> 2, T));

  Masks<BITS> masks;
  masks.init();
  OSCAR_STAMP(4);   // prologue done
  _Float16(*A_tab)[TABW] = s_A[wave];
  _Float16(*P_tab)[TABW] = s_P[wave];

  // Issue priority follows what is left to do.  Two workgroups share a CU, so every SIMD holds
  // one wave of each; between waves of equal priority the older one wins every issue slot it
  // can use, and the younger workgroup ran at 40 % of the older one's pace until that one was
  // done, then finished alone, without a partner to hide its stalls behind.  A wave therefore
  // lowers its priority as it gets through its pages (quarter by quarter): whichever wave of a
  // SIMD is behind is served first, and the two finish together.
  const int n_iter = pg_first < n_pages ? (n_pages - pg_first + pstride - 1) / pstride : 0;
  const int prio_step = max(1, (n_iter + 3) >> 2);
  int prio_next = prio_step, prio_level = 0;

  // Iterations come in chunks of 64 so that the table register is only reloaded between
  // chunks; tabn (lane 0) is the first entry of the following chunk.
  for (int it0 = 0; pg_first + pstride * it0 < n_pages; it0 += 64) {
  if (it0 > 0) tab = load_table(it0);
  const int tabn = load_table(it0 + 64);
  const int it_end = min(64, (n_pages - pg_first - pstride * it0 + pstride - 1) / pstride);
  // touch both registers here, so the wait for these two loads sits outside the page loop
  // (inside it, it would also wait for every prefetch in flight)
  asm volatile("" ::"v"(tab), "v"(tabn));
  for (int iti = 0; iti < it_end; ++iti) {
    const int pg = pg_first + pstride * (it0 + iti);
    OSCAR_STAMP(8 + min(it0 + iti, 15));   // top of page iteration 0..15
    if (OSCAR_DECODE_PRIORITY && it0 + iti == prio_next) {
      prio_next += prio_step;
      ++prio_level;
      if (prio_level == 1) __builtin_amdgcn_s_setprio(2);
      else if (prio_level == 2) __builtin_amdgcn_s_setprio(1);
      else __builtin_amdgcn_s_setprio(0);
    }
    const bool has_next = pg + pstride < n_pages;
    // entries past the wave's last page read as 0 (a valid page index) and the load is void
    const int phys = iti < 63 ? __builtin_amdgcn_readlane(tab, iti + 1)
                              : __builtin_amdgcn_readlane(tabn, 0);
    PageRsrc nx;   // the wave's next page
    nx.make(pools, P, (uint32_t)phys, has_next);

    // ---- q K^T ----
    float S[HP][8];
    {
      const uint32_t nt[4] = {kr.nr.x, kr.nr.y, kr.nr.z, kr.nr.w};
#pragma unroll
      for (int g = 0; g < NGK; ++g) {
        // per channel, what one unit of Q_h takes off the logit: Delta*z, or -zero when the
        // zero-point is the float group minimum (x = Delta*c + zero)
        float dz[8];
        if constexpr (zp_min) neg_widen8(kr.kz[g], dz);
        else mix_mul8(kr.kd[g], kr.kz[g], dz);
        float bias[HP];
#pragma unroll
        for (int s = 0; s < HP; ++s) {
          float bp = 0.0f;
          if constexpr (HP == 2) {
            const float4 qa = s_qr[wave][s][0][lane], qb = s_qr[wave][s][1][lane];
            const float qv[8] = {qa.x, qa.y, qa.z, qa.w, qb.x, qb.y, qb.z, qb.w};
#pragma unroll
            for (int i = 0; i < 8; ++i) bp = fmaf(qv[i], dz[i], bp);
          } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) bp = fmaf(qr[s][i], dz[i], bp);
          }
          bias[s] = row16_sum(bp);
          uint4 hi, lo;
#if OSCAR_LIMBS_PACKED
          mul_limbs_packed(qsh[s], qsl[s], kr.kd[g], hi, lo);
#else
          mul_split_hi_lo(qs[s], kr.kd[g], hi, lo);
#endif
          // (rows of heads past the group hold zeros either way: their queries are zero)
          const int h = q4 + 4 * s;
          *reinterpret_cast<uint4*>(&A_tab[row_hi(h)][8 * n]) = hi;
          *reinterpret_cast<uint4*>(&A_tab[row_hi(h) + 1][8 * n]) = lo;
        }
        kr.load_meta(nx, g, lane);
        wave_lds_fence();
        half8 areg[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
          areg[kk] = *reinterpret_cast<const half8*>(&A_tab[n][32 * q4 + 8 * kk]);
        wave_lds_fence();
        // logits of a tile pair: read one pair late, behind the next pair's matrix instructions,
        // so that nothing waits for an accumulator that is still in the matrix pipe
        auto logits = [&](int T, const float4v& a0, const float4v& a1) {
#pragma unroll
          for (int s = 0; s < HP; ++s) {
            // T is even: tokens T, T+1 are the two halves of norm word T/2
            S[s][T] = mix_scale<0>(fmaf(a0[2 * s] + a0[2 * s + 1], ps[s], -bias[s]), nt[T >> 1]);
            S[s][T + 1] = mix_scale<1>(fmaf(a1[2 * s] + a1[2 * s + 1], ps[s], -bias[s]), nt[T >> 1]);
          }
          keep_tuple(a0);
          keep_tuple(a1);
        };
        float4v prev0, prev1;
#pragma unroll
        for (int tt = 0; tt < TPG; tt += 2) {
          // two token tiles at a time: independent accumulators keep the MFMA pipe busy
          const int T = g * TPG + tt;
          float4v acc0 = (float4v){0.0f, 0.0f, 0.0f, 0.0f}, acc1 = acc0;
          if constexpr (!ONE_TILE) {
            u32x4 b0[4], b1[4];
            kr.kc[T >> 1].chunk(0).operands(b0, masks);
            kr.kc[T >> 1].chunk(1).operands(b1, masks);
            OSCAR_PREFETCH_FENCE();
            kr.load_codes(nx, T >> 1, lane);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
              acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                  areg[kk], __builtin_bit_cast(half8, b0[kk]), acc0, 0, 0, 0);
              acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                  areg[kk], __builtin_bit_cast(half8, b1[kk]), acc1, 0, 0, 0);
            }
          } else {
            // one tile at a time: the second head slot needs the registers of the second
            // operand set (the other wave of the SIMD fills the matrix pipe instead)
            u32x4 b0[4];
            kr.kc[T >> 1].chunk(0).operands(b0, masks);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
              acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                  areg[kk], __builtin_bit_cast(half8, b0[kk]), acc0, 0, 0, 0);
            asm volatile("" ::: "memory");
            kr.kc[T >> 1].chunk(1).operands(b0, masks);
            OSCAR_PREFETCH_FENCE();
            kr.load_codes(nx, T >> 1, lane);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
              acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                  areg[kk], __builtin_bit_cast(half8, b0[kk]), acc1, 0, 0, 0);
          }
          if (tt > 0) logits(T - 2, prev0, prev1);
          prev0 = acc0;
          prev1 = acc1;
        }
        logits(g * TPG + TPG - 2, prev0, prev1);
      }
    }
    kr.load_norm(nx, lane);
    if (it0 + iti == 0) OSCAR_STAMP(5);   // first page's logits done

    // ---- online softmax (per head slot; the 16 lanes of a group share a head) ----
    float alpha[HP];
    bool rescale = false;
#pragma unroll
    for (int s = 0; s < HP; ++s) {
      float mx = S[s][0];
#pragma unroll
      for (int T = 1; T < 8; ++T) mx = fmaxf(mx, S[s][T]);
      const float m_new = fmaxf(m_run[s], row16_max_fast(mx));
      alpha[s] = __builtin_amdgcn_exp2f(m_run[s] - m_new);
      rescale |= (m_new != m_run[s]);
      m_run[s] = m_new;
      float sum = 0.0f;
#pragma unroll
      for (int T = 0; T < 8; ++T) {
        S[s][T] = __builtin_amdgcn_exp2f(S[s][T] - m_new);  // S now holds p
        sum += S[s][T];
      }
      l_run[s] = l_run[s] * alpha[s] + sum;
    }

    // ---- scale of the value operand for this page: Delta_v * 2^xv < 2^13 ----
    uint4 dm = vr.vd[0];
#pragma unroll
    for (int g = 1; g < NGV; ++g) dm = pk_max4(dm, vr.vd[g]);
    // Step sizes are non-negative fp16 numbers: the largest has the largest bit pattern, and its
    // exponent field E bounds it by 2^(E - 14) (2^-14 for E = 0: zero or subnormal steps)
    const uint32_t dm2 = pk_max_u16(pk_max_u16(dm.x, dm.y), pk_max_u16(dm.z, dm.w));
    const uint32_t dbits = row16_max_u32(max(dm2 & 0xffffu, dm2 >> 16));  // the 16 lanes of a head group cover all 128 tokens
    const int xv = 27 - (int)(dbits >> 10);
    rescale |= (xv != xv_cur);
    if (__any(rescale)) {
      float f[HP];
#pragma unroll
      for (int s = 0; s < HP; ++s) f[s] = ldexpf(alpha[s], xv - xv_cur);
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
#pragma unroll
        for (int s = 0; s < HP; ++s) {
          O[ct][2 * s] *= f[s];
          O[ct][2 * s + 1] *= f[s];
        }
      }
#pragma unroll
      for (int s = 0; s < HP; ++s)
#pragma unroll
        for (int g = 0; g < NGV; ++g) bv[s][g] *= alpha[s];
    }
    xv_cur = xv;

    // ---- P V, one value group at a time through the wave's LDS table ----
    [[maybe_unused]] const float pscale = ldexpf(1.0f, xv);
    float pc[HP][8];   // p * 2^(xv - slot offset): the value operand before Delta_v
#pragma unroll
    for (int s = 0; s < HP; ++s)
#pragma unroll
      for (int T = 0; T < 8; ++T)
        pc[s][T] = S[s][T] * (vsc0[T] * (OSCAR_LIMBS_PACKED ? 16384.0f : pscale));
#if OSCAR_LIMBS_PACKED
    // The probabilities are split as p * 2^14 (at most 2^14, whatever the page's step sizes
    // are); the rest of the page's power of two goes to the step sizes, whose largest then
    // sits in [2^-2, 2^-1): an exact scaling unless a step size is 2^12 times smaller than
    // the page's largest.
    uint4 pch[HP], pcl[HP];
#pragma unroll
    for (int s = 0; s < HP; ++s) split_to_halves(pc[s], pch[s], pcl[s]);
    const _Float16 ysc = (_Float16)ldexpf(1.0f, xv - 14);
    const half2v ysc2 = {ysc, ysc};
#endif
#pragma unroll
    for (int g = 0; g < NGV; ++g) {
      float dz[8];
      if constexpr (zp_min) neg_widen8(vr.vz[g], dz);
      else mix_mul8(vr.vd[g], vr.vz[g], dz);
#if OSCAR_LIMBS_PACKED
      const uint4 yd = scale_halves(vr.vd[g], ysc2);
#endif
#pragma unroll
      for (int s = 0; s < HP; ++s) {
        float acc_b = 0.0f;
#pragma unroll
        for (int T = 0; T < 8; ++T) acc_b = fmaf(S[s][T], dz[T], acc_b);
        bv[s][g] += acc_b;
        uint4 hi, lo;
#if OSCAR_LIMBS_PACKED
        mul_limbs_packed(pch[s], pcl[s], yd, hi, lo);
#else
        mul_split_hi_lo(pc[s], vr.vd[g], hi, lo);
#endif
        // (heads past the group produce finite values in rows nobody reads back)
        const int h = q4 + 4 * s;
        *reinterpret_cast<uint4*>(&P_tab[row_hi(h)][8 * n]) = hi;
        *reinterpret_cast<uint4*>(&P_tab[row_hi(h) + 1][8 * n]) = lo;
      }
      vr.load_delta(nx, g, lane);
      wave_lds_fence();
      half8 preg[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        preg[kk] = *reinterpret_cast<const half8*>(&P_tab[n][8 * (4 * kk + q4)]);
      wave_lds_fence();
#pragma unroll
      for (int cc = 0; cc < CPG; cc += 2) {
        const int ct = g * CPG + cc;
        if constexpr (!ONE_TILE) {
          u32x4 b0[4], b1[4];
          vr.vc[ct >> 1].chunk(0).operands(b0, masks);
          vr.vc[ct >> 1].chunk(1).operands(b1, masks);
          OSCAR_PREFETCH_FENCE();
          vr.load_codes(nx, ct >> 1, lane);
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            O[ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                preg[kk], __builtin_bit_cast(half8, b0[kk]), O[ct], 0, 0, 0);
            O[ct + 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                preg[kk], __builtin_bit_cast(half8, b1[kk]), O[ct + 1], 0, 0, 0);
          }
        } else {
          u32x4 b0[4];
          vr.vc[ct >> 1].chunk(0).operands(b0, masks);
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
            O[ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                preg[kk], __builtin_bit_cast(half8, b0[kk]), O[ct], 0, 0, 0);
          asm volatile("" ::: "memory");
          vr.vc[ct >> 1].chunk(1).operands(b0, masks);
          OSCAR_PREFETCH_FENCE();
          vr.load_codes(nx, ct >> 1, lane);
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
            O[ct + 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                preg[kk], __builtin_bit_cast(half8, b0[kk]), O[ct + 1], 0, 0, 0);
        }
      }
    }
    // The zero-points of the next page are fetched last, when every temporary of the
    // iteration is dead: fetched where they are consumed (inside the value groups), the
    // compiler parked the arriving registers elsewhere and moved half of each to its home
    // straight away, which made the wave wait for loads it had just issued.
#pragma unroll
    for (int g = 0; g < NGV; ++g) vr.load_zero(nx, g, lane);
  }
  }

#pragma unroll
  for (int ct = 0; ct < 8; ++ct) keep_tuple(O[ct]);
  OSCAR_STAMP(24);   // page loop done
  if (OSCAR_DECODE_PRIORITY) __builtin_amdgcn_s_setprio(0);
  // ---- wave results -> LDS ----
  {
    const float unscale = ldexpf(1.0f, 24 - xv_cur - slot_bitpos_min(BITS));
#pragma unroll
    for (int s = 0; s < HP; ++s) {
      const int h = q4 + 4 * s;
      const float l_tot = row16_sum(l_run[s]);
      float bvt[NGV];
#pragma unroll
      for (int g = 0; g < NGV; ++g) bvt[g] = row16_sum(bv[s][g]);
      if (h < gq) {
#pragma unroll
        for (int ct = 0; ct < 8; ++ct)
          s_o[wave][h][16 * ct + n] = (O[ct][2 * s] + O[ct][2 * s + 1]) * unscale - bvt[ct / CPG];
        if (n == 0) {
          s_wm[wave][h] = m_run[s];
          s_wl[wave][h] = l_tot;
        }
      }
    }
  }

  // ---- merge the 4 wave states and the residual state, write the split's record ----
  OSCAR_STAMP(25);   // wave results in LDS
  __syncthreads();
  OSCAR_STAMP(26);   // all four waves there
  // a thread owns one channel of every second head (the head parity is wave-uniform, so no
  // lane idles); the reads of a head are independent and go out together
  const int ch = tid & (D - 1), hh = __builtin_amdgcn_readfirstlane(tid >> 7);
  // With a single split the record is the result: the host passes the output tensor and
  // launches no reduce pass.  acc / L below are the record's own numbers, divided as the
  // reduce pass divides them, so both routes give the same bits.
  const bool direct = P.out != nullptr;
#pragma unroll
  for (int k = 0; k < OSCAR_MAX_GQA / 2; ++k) {
    const int h = hh + 2 * k;
    if (h < gq) {
      float m[4], o[4];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        m[w] = s_wm[w][h];
        o[w] = s_o[w][h][ch];
      }
      const float M = fmaxf(fmaxf(m[0], m[1]), fmaxf(m[2], m[3]));
      float acc = 0.0f;
      if (M != -INFINITY) {
#pragma unroll
        for (int w = 0; w < 4; ++w)
          if (m[w] != -INFINITY) acc += o[w] * __builtin_amdgcn_exp2f(m[w] - M);
      }
      const size_t unit = (size_t)b * Hq + (size_t)kvh * gq + h;
      if (direct) {
        float L = 0.0f;
        if (M != -INFINITY) {
#pragma unroll
          for (int w = 0; w < 4; ++w)
            if (m[w] != -INFINITY) L += s_wl[w][h] * __builtin_amdgcn_exp2f(m[w] - M);
        }
        const float res = L > 0.0f ? acc / L : 0.0f;
        const size_t oi = unit * D + ch;
        if (P.out_dtype == OSCAR_F32) reinterpret_cast<float*>(P.out)[oi] = res;
        else if (P.out_dtype == OSCAR_BF16) reinterpret_cast<__hip_bfloat16*>(P.out)[oi] = __float2bfloat16(res);
        else reinterpret_cast<__half*>(P.out)[oi] = __float2half_rn(res);
      } else {
        P.ws[(unit * P.num_splits + split) * WS_STRIDE + ch] = acc;
      }
    }
  }
  if (!direct && tid < gq) {
    const int h = tid;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, s_wm[w][h]);
    float L = 0.0f;
    if (M != -INFINITY) {
#pragma unroll
      for (int w = 0; w < 4; ++w)
        if (s_wm[w][h] != -INFINITY) L += s_wl[w][h] * __builtin_amdgcn_exp2f(s_wm[w][h] - M);
    }
    const size_t rec = ((size_t)b * Hq + (size_t)kvh * gq + h) * P.num_splits + split;
    P.ws[rec * WS_STRIDE + D] = M;
    P.ws[rec * WS_STRIDE + D + 1] = L;
  }
  OSCAR_STAMP(27);   // split record written
}

template <int BITS, int HP>
int launch_groups(const DecodeParams& P, int gq, dim3 grid, hipStream_t st, hipEvent_t e0,
                  hipEvent_t e1) {
  const int ngk = P.g.ngk, ngv = P.g.ngv;
  constexpr bool ZPM = OSCAR_MFMA_ZPMIN != 0;
  // the event-carrying launch only when a timer asked for it: the plain launch is what a
  // stream capture records
#define OSCAR_MFMA_CASE(NK, NV)                                                            \
  if (ngk == NK && ngv == NV) {                                                            \
    if (e0 || e1)                                                                          \
      hipExtLaunchKernelGGL((oscar_decode_mfma_kernel<BITS, HP, NK, NV, ZPM>), grid,       \
                            dim3(256), 0, st, e0, e1, 0, P, gq);                           \
    else                                                                                   \
      hipLaunchKernelGGL((oscar_decode_mfma_kernel<BITS, HP, NK, NV, ZPM>), grid,          \
                         dim3(256), 0, st, P, gq);                                         \
    return OSCAR_OK;                                                                       \
  }
  OSCAR_MFMA_CASE(1, 4)
  OSCAR_MFMA_CASE(4, 4)
  OSCAR_MFMA_CASE(1, 1)
  OSCAR_MFMA_CASE(2, 2)
  OSCAR_MFMA_CASE(1, 2)
  OSCAR_MFMA_CASE(2, 1)
  OSCAR_MFMA_CASE(2, 4)
  OSCAR_MFMA_CASE(4, 1)
  OSCAR_MFMA_CASE(4, 2)
#undef OSCAR_MFMA_CASE
  return OSCAR_ERR_UNSUPPORTED;
}

// every variant of this translation unit's zero-point form
int launch_this_form(const DecodeParams& P, int gq, dim3 grid, hipStream_t st, hipEvent_t e0,
                     hipEvent_t e1) {
  if (P.g.bits == 2)
    return gq <= 4 ? launch_groups<2, 1>(P, gq, grid, st, e0, e1) : launch_groups<2, 2>(P, gq, grid, st, e0, e1);
  if (P.g.bits == 4)
    return gq <= 4 ? launch_groups<4, 1>(P, gq, grid, st, e0, e1) : launch_groups<4, 2>(P, gq, grid, st, e0, e1);
  return OSCAR_ERR_UNSUPPORTED;
}

}  // namespace

#if OSCAR_MFMA_ZPMIN

int oscar_launch_decode_mfma_zpmin(const void* params, int gq, dim3 grid, hipStream_t st,
                                   hipEvent_t e0, hipEvent_t e1) {
  return launch_this_form(*reinterpret_cast<const DecodeParams*>(params), gq, grid, st, e0, e1);
}

#else

#ifdef OSCAR_DECODE_STAMPS
// [8 workgroup slots][4 waves][32 stamps] of the last stamped launch (integer zero-point variants)
extern "C" int oscar_debug_read_stamps(void* dst, size_t bytes) {
  if (!dst || bytes != sizeof(g_stamps)) return OSCAR_ERR_INVALID_ARG;
  return hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_stamps), sizeof(g_stamps)) == hipSuccess ? OSCAR_OK : OSCAR_ERR_HIP;
}
#endif

int oscar_launch_decode_mfma_zpmin(const void* params, int gq, dim3 grid, hipStream_t st,
                                   hipEvent_t e0, hipEvent_t e1);

// Test / profiling switch of oscar_debug_force_generic_decode: the only process-wide state of
// the library besides the cached device properties, one relaxed atomic flag read per launch.
static std::atomic<int> g_force_generic{0};

extern "C" int oscar_debug_force_generic_decode(int32_t on) {
  return g_force_generic.exchange(on ? 1 : 0, std::memory_order_relaxed);
}

// Launches the matrix-core partial pass when the configuration is one it is built for
// (fp16 metadata; group sizes 32, 64 or 128 on either side; keys scaled into [-1, 1]; page pools
// below 2 GiB each); OSCAR_ERR_UNSUPPORTED tells the caller to use the generic kernel.
int oscar_launch_decode_mfma(const void* params, int gq, dim3 grid, hipStream_t st,
                             hipEvent_t e0, hipEvent_t e1) {
  const DecodeParams& P = *reinterpret_cast<const DecodeParams*>(params);
  if (P.c.cfg.meta_dtype != OSCAR_F16) return OSCAR_ERR_UNSUPPORTED;
  // the key operand's fixed exponent assumes Delta_k <= 1, which holds when |K_u| <= 1 (L2 or
  // maximum scaling); the un-scaled and mean-absolute-value ablations go to the generic kernel
  if (P.c.cfg.scale_mode != OSCAR_SCALE_L2 && P.c.cfg.scale_mode != OSCAR_SCALE_MAX)
    return OSCAR_ERR_UNSUPPORTED;
  if (g_force_generic.load(std::memory_order_relaxed)) return OSCAR_ERR_UNSUPPORTED;
  // a page is addressed as a 32-bit scalar offset into its pool
  const unsigned long long units = (unsigned long long)P.c.num_pages * (unsigned long long)P.c.cfg.n_kv_heads;
  const int biggest = P.g.k_codes_bytes > P.g.v_meta_bytes ? P.g.k_codes_bytes : P.g.v_meta_bytes;
  if (units * (unsigned long long)biggest > 0x7FFFFFFFull) return OSCAR_ERR_UNSUPPORTED;
  if (P.c.cfg.zp_mode == OSCAR_ZP_MIN) return oscar_launch_decode_mfma_zpmin(params, gq, grid, st, e0, e1);
  return launch_this_form(P, gq, grid, st, e0, e1);
}

#endif
