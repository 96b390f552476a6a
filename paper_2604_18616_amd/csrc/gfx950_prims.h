// Device primitives shared by the gfx950 kernels of this library: vector types, compile-time loops,
// bf16 packing, the direct HBM -> LDS copies and the half-wave exchange.  Device code only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gfx950 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;

#define LDS_PTR(T, p) ((T __attribute__((address_space(3)))*)(p))

template <int V> struct IntC { static constexpr int value = V; };
// compile-time loop: f(IntC<I>{}) for I = BEGIN .. END-1, everything inlined
template <int BEGIN, int END, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (BEGIN < END) {
        f(IntC<BEGIN>{});
        static_for<BEGIN + 1, END>(f);
    }
}

// two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
    f32x2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(unsigned, b);
}

// Asynchronous 16-byte-per-lane copy HBM -> LDS: lane i's 16 bytes at (base + byte_off) land at LDS
// address lds_addr + 16*i (verified on gfx950).  Written as inline asm so that the compiler's
// wait-count pass does not know about the LDS write: given the builtin it puts a full vmcnt(0) wait in
// front of the next LDS read of ANY buffer, which serialises the prefetch.  Completion is awaited
// explicitly (s_waitcnt vmcnt) before the barrier that publishes the tile.  M0 carries the LDS
// address.  It is not in the clobber list: the compiler treats M0 as a reserved register on this
// target (it never keeps a value there across statements, and writes it itself immediately before
// each of its own uses), and it answers a clobber of M0 with a warning that the result is undefined.
__device__ __forceinline__ void dma_to_lds_16B(const void* base, unsigned byte_off, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(byte_off), "s"(base), "s"(lds_addr) : "memory");
}
// The same with the LDS address given as lds_addr + IMM, IMM an assembly-time constant: a kernel keeps
// one scalar base per wavefront instead of one scalar per destination.
template <int IMM>
__device__ __forceinline__ void dma_to_lds_16B(const void* base, unsigned byte_off, unsigned lds_addr) {
    asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(byte_off), "s"(base), "s"(lds_addr), "n"(IMM) : "memory", "scc");
}
// One dword per lane (lane i's 4 bytes land at lds_addr + IMM + 4 i).
template <int IMM>
__device__ __forceinline__ void dma_to_lds_4B(const void* base, unsigned byte_off, unsigned lds_addr) {
    asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :: "v"(byte_off), "s"(base), "s"(lds_addr), "n"(IMM) : "memory", "scc");
}

// The 16-byte copy through a buffer resource: lane i's 16 bytes at (resource base + soff + voff) land at
// lds_addr + 16*i, and a piece that lies past the resource's num_records arrives as zeros (the
// hardware's out-of-range rule for buffer loads, checked on gfx950 with the LDS form of the
// instruction): a partial last tile needs no clamped addresses and no clearing afterwards.
__device__ __forceinline__ i32x4 buffer_resource(const void* base, unsigned bytes) {
    const unsigned long long a = (unsigned long long)base;
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)((unsigned)(a >> 32) & 0xffffu));   // stride 0: a raw buffer
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);                              // num_records, in bytes
    r[3] = 0x00020000;                                                              // 32-bit data format
    return r;
}
__device__ __forceinline__ void dma_buf_to_lds_16B(i32x4 rsrc, unsigned voff, unsigned soff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, %2 offen lds"
                 :: "v"(voff), "s"(rsrc), "s"(soff), "s"(lds_addr) : "memory");
}

// Exchange between lane l and lane l ^ 32.  v_permlane32_swap(a, b) returns
//   r0 = { a[0..31], b[0..31] },  r1 = { a[32..63], b[32..63] }     (verified on gfx950),
// so with b = a, (r0, r1) is (value held by the low-half lane, value held by the high-half lane) in
// every lane.  The two results are copied to scalars before any reinterpretation: a bit cast applied
// directly to a vector element reads element 0.
__device__ __forceinline__ void swap_halves(float x, float& lo, float& hi) {
    const unsigned a = __float_as_uint(x);
    const u32x2 r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    lo = __uint_as_float(r0);
    hi = __uint_as_float(r1);
}
__device__ __forceinline__ float max_across_halves(float x) {
    float lo, hi;
    swap_halves(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float sum_across_halves(float x) {
    float lo, hi;
    swap_halves(x, lo, hi);
    return lo + hi;
}

}  // namespace gfx950
