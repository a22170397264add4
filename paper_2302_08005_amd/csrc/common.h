// Shared device helpers for the gfx950 kernels: bf16 packing, 16-byte vector access, wave
// reductions and the Philox4x32-10 dropout draw.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include <stdint.h>

namespace slapo {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));

typedef uint16_t bf16_t;  // storage of one 16-bit element: bf16, or IEEE half where a kernel is told so (F16 flag)
typedef _Float16 f16_t;   // IEEE half as a type of its own, for the kernels that are templates of the element type
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
enum { DT_BF16 = 0, DT_FP32 = 1, DT_FP16 = 2 };   // element types of the launch interface (the C ABI's values)

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// round-to-nearest-even pack of two floats into one dword (lo = a, hi = b)
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2_t v = {a, b};
  bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
  return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ bf16_t f32_to_bf16(float a) { return (bf16_t)(pack_bf16x2(a, 0.f) & 0xffffu); }

// The two 16-bit formats behind one interface (F16 = IEEE half, else bf16): the hot kernels keep 16-bit data in
// untyped containers (bf16_t storage, bf16x8_t fragments) and only these few operations know the format.
template <bool F16> __device__ __forceinline__ uint32_t pack2(float a, float b) {   // round to nearest even; lo = a
  if constexpr (F16) {
    f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
  } else {
    return pack_bf16x2(a, b);
  }
}
template <bool F16> __device__ __forceinline__ float unpack_lo(uint32_t w) {
  if constexpr (F16) return (float)__builtin_bit_cast(f16x2_t, w)[0];
  else return bf16lo_to_f32(w);
}
template <bool F16> __device__ __forceinline__ float unpack_hi(uint32_t w) {
  if constexpr (F16) return (float)__builtin_bit_cast(f16x2_t, w)[1];
  else return bf16hi_to_f32(w);
}
template <bool F16> __device__ __forceinline__ f32x16_t mfma16(bf16x8_t a, bf16x8_t b, f32x16_t c) {
  if constexpr (F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// acc += a b with the accumulator held in the accumulation registers (AGPRs), written out because the compiler
// picks one MFMA form per function and takes the ordinary registers whenever everything fits into 256 of them.
// Opaque to the compiler's hazard pass: the caller makes sure that a and b were not written by a vector-ALU
// instruction right before (NOPS wait states are emitted in front; LDS reads are tracked through the operand
// registers and waited for by the compiler), that accumulations into one register are at least four MFMAs apart,
// and calls agpr_results_ready() before reading the result with ordinary instructions.
template <bool F16, int NOPS = 1>
__device__ __forceinline__ void mfma16_agpr(f32x16_t& acc, bf16x8_t a, bf16x8_t b) {
  if constexpr (NOPS > 0) {
    if constexpr (F16) asm("s_nop %3\n\tv_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b), "n"(NOPS - 1));
    else asm("s_nop %3\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b), "n"(NOPS - 1));
  } else {
    if constexpr (F16) asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
    else asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
  }
}
// more wait states than any MFMA needs before its result may be read by a non-MFMA instruction
__device__ __forceinline__ void agpr_results_ready() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }

template <bool F16> __device__ __forceinline__ void load8h(const bf16_t* p, float (&v)[8]) {
  const uint4 w = *reinterpret_cast<const uint4*>(p);
  v[0] = unpack_lo<F16>(w.x); v[1] = unpack_hi<F16>(w.x); v[2] = unpack_lo<F16>(w.y); v[3] = unpack_hi<F16>(w.y);
  v[4] = unpack_lo<F16>(w.z); v[5] = unpack_hi<F16>(w.z); v[6] = unpack_lo<F16>(w.w); v[7] = unpack_hi<F16>(w.w);
}
template <bool F16> __device__ __forceinline__ void store8h(bf16_t* p, const float (&v)[8]) {
  uint4 w;
  w.x = pack2<F16>(v[0], v[1]); w.y = pack2<F16>(v[2], v[3]);
  w.z = pack2<F16>(v[4], v[5]); w.w = pack2<F16>(v[6], v[7]);
  *reinterpret_cast<uint4*>(p) = w;
}

// Eight consecutive elements of either storage type <-> eight floats.
__device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
  uint4 w = *reinterpret_cast<const uint4*>(p);
  v[0] = bf16lo_to_f32(w.x); v[1] = bf16hi_to_f32(w.x); v[2] = bf16lo_to_f32(w.y); v[3] = bf16hi_to_f32(w.y);
  v[4] = bf16lo_to_f32(w.z); v[5] = bf16hi_to_f32(w.z); v[6] = bf16lo_to_f32(w.w); v[7] = bf16hi_to_f32(w.w);
}
__device__ __forceinline__ void load8(const f16_t* p, float (&v)[8]) { load8h<true>(reinterpret_cast<const bf16_t*>(p), v); }
__device__ __forceinline__ void store8(f16_t* p, const float (&v)[8]) { store8h<true>(reinterpret_cast<bf16_t*>(p), v); }
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void store8(bf16_t* p, const float (&v)[8]) {
  uint4 w;
  w.x = pack_bf16x2(v[0], v[1]); w.y = pack_bf16x2(v[2], v[3]);
  w.z = pack_bf16x2(v[4], v[5]); w.w = pack_bf16x2(v[6], v[7]);
  *reinterpret_cast<uint4*>(p) = w;
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
// Eight elements kept in their storage form (so that a prefetched row costs few registers) until used.
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> {
  uint4 w;
  __device__ __forceinline__ void load(const bf16_t* p) { w = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void get(float (&v)[8]) const {
    v[0] = bf16lo_to_f32(w.x); v[1] = bf16hi_to_f32(w.x); v[2] = bf16lo_to_f32(w.y); v[3] = bf16hi_to_f32(w.y);
    v[4] = bf16lo_to_f32(w.z); v[5] = bf16hi_to_f32(w.z); v[6] = bf16lo_to_f32(w.w); v[7] = bf16hi_to_f32(w.w);
  }
};
template <> struct Raw8<f16_t> {
  uint4 w;
  __device__ __forceinline__ void load(const f16_t* p) { w = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void get(float (&v)[8]) const {
    v[0] = unpack_lo<true>(w.x); v[1] = unpack_hi<true>(w.x); v[2] = unpack_lo<true>(w.y); v[3] = unpack_hi<true>(w.y);
    v[4] = unpack_lo<true>(w.z); v[5] = unpack_hi<true>(w.z); v[6] = unpack_lo<true>(w.w); v[7] = unpack_hi<true>(w.w);
  }
};
template <> struct Raw8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = *reinterpret_cast<const float4*>(p); b = *reinterpret_cast<const float4*>(p + 4);
  }
  __device__ __forceinline__ void get(float (&v)[8]) const {
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};
__device__ __forceinline__ float to_f32(bf16_t h) { return bf16_to_f32(h); }
__device__ __forceinline__ float to_f32(f16_t h) { return (float)h; }
__device__ __forceinline__ float to_f32(float f) { return f; }
__device__ __forceinline__ void from_f32(bf16_t& d, float f) { d = f32_to_bf16(f); }
__device__ __forceinline__ void from_f32(f16_t& d, float f) { d = (f16_t)f; }
__device__ __forceinline__ void from_f32(float& d, float f) { d = f; }

// One direct 16-byte-per-lane load: lane l of the wavefront fetches base[voffset_l + soffset ..] (bytes; zero
// beyond `bytes`) into LDS at lds + 16 l. A plain function on purpose: the buffer builtins are only known
// to the device pass, and a kernel template that names them directly loses its host-side launch stub.
__device__ __forceinline__ void buffer_load_lds_16(const void* base, unsigned bytes, void* lds, unsigned voffset,
                                                   unsigned soffset) {
  // raw buffer resource: stride 0, size in bytes, untyped 32-bit data format; loop-invariant scalars
  const auto rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)lds, 16, voffset, soffset, 0, 0);
}

// The same load, issued where the compiler does not see it. The compiler orders every LDS read it cannot tell apart
// from a pending direct load behind that load: plain LDS reads pass, but in front of every transposing read
// (ds_read_b64_tr_b16) that follows a direct load it waits for ALL outstanding vector-memory loads, i.e. for the tile
// that was just requested for a later step, which undoes the prefetch. Kernels that mix the two issue their direct
// loads through this form and keep the landing of every tile under their own counter waits (wait_loads_and_lds in
// front of the barrier that hands a tile over), which they need in either form. M0 carries the LDS address; one wait
// state between writing it and the load that reads it.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void buffer_load_lds_16_untracked(const void* base, unsigned bytes, void* lds,
                                                             unsigned voffset, unsigned soffset) {
  typedef int i32x4_t __attribute__((ext_vector_type(4)));
  const unsigned long long a = (unsigned long long)base;
  i32x4_t rsrc;   // the resource words of buffer_load_lds_16
  rsrc[0] = (int)(unsigned)a;
  rsrc[1] = (int)((unsigned)(a >> 32) & 0xffffu);
  rsrc[2] = (int)bytes;
  rsrc[3] = 0x00020000;
  const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)lds;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
               : "memory", "m0");
}
#pragma clang diagnostic pop

// Pipelines of direct loads wait for the oldest tile only: at most N vector-memory loads of this wavefront
// still outstanding (they complete in issue order), LDS operations done; and a barrier that does not bring
// the wait for ALL loads with it, as __syncthreads does.
template <int N>
__device__ __forceinline__ void wait_loads_and_lds() {
  static_assert(N >= 0 && N < 64, "six-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4));
}
__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Sum over the 64 lanes, returned to every lane. Data-parallel-primitive moves (quad permutes, mirrors inside
// rows of 16 lanes, then the row broadcasts) keep the whole reduction in the vector ALU: six dependent adds
// and one lane read instead of six round trips through the LDS crossbar.
__device__ __forceinline__ float wave_sum(float v) {
  auto dpp = [](float x, auto ctrl, auto row_mask) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value,
                                                                   decltype(row_mask)::value, 0xf, true));
  };
  using std::integral_constant;
  v += dpp(v, integral_constant<int, 0xb1>{}, integral_constant<int, 0xf>{});    // quad_perm [1,0,3,2]
  v += dpp(v, integral_constant<int, 0x4e>{}, integral_constant<int, 0xf>{});    // quad_perm [2,3,0,1]
  v += dpp(v, integral_constant<int, 0x141>{}, integral_constant<int, 0xf>{});   // row_half_mirror
  v += dpp(v, integral_constant<int, 0x140>{}, integral_constant<int, 0xf>{});   // row_mirror: every lane holds its row's sum
  v += dpp(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xa>{});   // row_bcast15 into rows 1 and 3
  v += dpp(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xc>{});   // row_bcast31 into rows 2 and 3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Philox4x32-10 block function (Salmon et al., SC'11): counter c[4], key k[2].
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&o)[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // (one 32 x 32 -> 64 bit multiply per product: a high and a low multiply each cost as much as the wide one)
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    c0 = hi1 ^ c1 ^ k0; c1 = lo1; c2 = hi0 ^ c3 ^ k1; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  o[0] = c0; o[1] = c1; o[2] = c2; o[3] = c3;
}

struct DropoutParams {
  uint32_t key0, key1;   // low / high half of the seed
  uint32_t site, layer;  // third and fourth counter word
  uint32_t thr;          // keep iff 16-bit draw >= thr
  float scale;           // 1 / (1 - p)
};

// Keep decisions of the eight elements of block `blk` (= element index >> 3), bit j = element j kept.
__device__ __forceinline__ uint32_t dropout_keep8(const DropoutParams& dp, uint64_t blk) {
  uint32_t o[4];
  philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), dp.site, dp.layer, dp.key0, dp.key1, o);
  uint32_t bits = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint32_t r16 = (o[j >> 1] >> (16 * (j & 1))) & 0xffffu;
    bits |= (r16 >= dp.thr ? 1u : 0u) << j;
  }
  return bits;
}

// Keep decision of the single element e (the plain kernels' per-element form of the same stream).
__device__ __forceinline__ bool dropout_keep1(const DropoutParams& dp, uint64_t e) {
  uint32_t o[4];
  const uint64_t blk = e >> 3;
  philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), dp.site, dp.layer, dp.key0, dp.key1, o);
  const uint32_t j = (uint32_t)e & 7u;
  return ((o[j >> 1] >> (16 * (j & 1))) & 0xffffu) >= dp.thr;
}

}  // namespace slapo
