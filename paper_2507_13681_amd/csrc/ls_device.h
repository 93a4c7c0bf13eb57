// Device-side building blocks shared by the LoopServe kernels (gfx950 only).
//
// The tile products use the 32x32 MFMA shapes of CDNA4.  One "fragment" is the
// 8 contraction-index values a lane feeds into a 32x32x16 product: lane l holds
// row (or column) l % 32 of the operand and the eight k values 8*(l/32) .. +7 of
// the current 16-wide k chunk.  For bf16 that is one v_mfma_f32_32x32x16_bf16;
// for fp32 the same fragment is consumed by eight v_mfma_f32_32x32x2_f32, the
// i-th pairing element i of both lane halves (a permutation of k, applied to
// both operands alike, so the product is unchanged).
//
// Accumulator layout of every 32x32 product D = A * B (A is M x K, B is K x N):
//   lane l, register r (0..15) holds D[8*(r/4) + 4*(l/32) + r%4][l % 32].
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ls {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

struct bf16_t { uint16_t bits; };   // storage type tag for bf16 tensors

template <typename T> struct Frag;
template <> struct Frag<bf16_t> { bf16x8 v; };
template <> struct Frag<float>  { float v[8]; };

template <typename T> struct Elem;
template <> struct Elem<bf16_t> { static constexpr int bytes = 2; static constexpr int per16 = 8; };
template <> struct Elem<float>  { static constexpr int bytes = 4; static constexpr int per16 = 4; };

// acc += A(32 x 16 chunk) * B(16 chunk x 32)
__device__ __forceinline__ void mma(f32x16& acc, const Frag<bf16_t>& a, const Frag<bf16_t>& b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, acc, 0, 0, 0);
}
__device__ __forceinline__ void mma(f32x16& acc, const Frag<float>& a, const Frag<float>& b) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[i], b.v[i], acc, 0, 0, 0);
}

// Load the 8 consecutive elements starting at p (16-byte aligned) as a fragment.
__device__ __forceinline__ void load_frag(Frag<bf16_t>& f, const void* p) {
    f.v = *reinterpret_cast<const bf16x8*>(p);
}
__device__ __forceinline__ void load_frag(Frag<float>& f, const void* p) {
    const f32x4 a = reinterpret_cast<const f32x4*>(p)[0], b = reinterpret_cast<const f32x4*>(p)[1];
    f.v[0] = a.x; f.v[1] = a.y; f.v[2] = a.z; f.v[3] = a.w;
    f.v[4] = b.x; f.v[5] = b.y; f.v[6] = b.z; f.v[7] = b.w;
}
__device__ __forceinline__ void zero_frag(Frag<bf16_t>& f) {
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    f.v = __builtin_bit_cast(bf16x8, z);
}
__device__ __forceinline__ void zero_frag(Frag<float>& f) {
#pragma unroll
    for (int i = 0; i < 8; ++i) f.v[i] = 0.f;
}

// float -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint16_t f2bf(float x) {
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(uint16_t b) {
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}

// Pack 8 probabilities into a fragment (operand of the P*V product).
__device__ __forceinline__ void pack_frag(Frag<bf16_t>& f, const float* p) {
    typedef __attribute__((ext_vector_type(8))) float f32x8;
    const f32x8 x = {p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7]};
    f.v = __builtin_convertvector(x, bf16x8);          // v_cvt_pk_bf16_f32, round to nearest even
}
__device__ __forceinline__ void pack_frag(Frag<float>& f, const float* p) {
#pragma unroll
    for (int i = 0; i < 8; ++i) f.v[i] = p[i];
}

typedef __attribute__((ext_vector_type(4))) short s16x4;

// One wave-wide global -> LDS transfer (global_load_lds_dwordx4): lane l fetches 16 bytes and they land
// at LDS byte address lds + 16 * l; `lds` (and `gbase`) are wave-uniform.  Written as asm statements so
// that the compiler does not count the transfers among the memory operations it tracks: it cannot tell
// which LDS bytes a transfer fills and would make every later LDS read wait for all outstanding
// transfers, serialising a prefetch with the work on the data already there.  A kernel waits for its
// transfers itself (wait_transfers, then a barrier if other waves read the data).  M0 is listed as
// clobbered so that the compiler never keeps a value of its own in M0 across a transfer.
__device__ __forceinline__ void dma16(const unsigned char* gbase, uint32_t voff, uint32_t lds) {   // address = gbase + voff
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(gbase) : "memory", "m0");
}
__device__ __forceinline__ void dma16(const unsigned char* gptr, uint32_t lds) {                    // per-lane address
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds), "v"(gptr) : "memory", "m0");
}
__device__ __forceinline__ void wait_transfers() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for the wave's outstanding global
// loads and stores; a kernel whose waves exchange data through LDS alone need not stall on a store's round trip.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// LDS transpose read of a bf16 tile stored row-major: in a block of 16 lanes, lane s addresses 4
// consecutive 16-bit values and lane L receives value L % 4 of the lanes L/4, L/4+4, L/4+8, L/4+12.
// Two reads (rows r .. and r + 8 ..) give a lane the eight contraction-index values of a fragment.
__device__ __forceinline__ void load_frag_tr(Frag<bf16_t>& f, const unsigned char* lo_addr, const unsigned char* hi_addr) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(lo_addr));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(hi_addr));
    struct U { s16x4 a, b; } u = {lo, hi};
    f.v = __builtin_bit_cast(bf16x8, u);
}

__device__ __forceinline__ float to_float(bf16_t x) { return bf2f(x.bits); }
__device__ __forceinline__ float to_float(float x) { return x; }

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Key row `key` (0..63 inside a tile) sits at this column of the transposed V tile,
// so that the 8 keys one lane half needs for a P*V chunk are contiguous:
// bits 2 and 3 of the key index are swapped.
__device__ __forceinline__ int vt_col(int key) {
    return (key & ~12) | ((key & 8) >> 1) | ((key & 4) << 1);
}

}  // namespace ls
