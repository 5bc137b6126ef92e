// Device helpers shared by the matrix-core kernels (gfx950): vector types, the
// LDS-only barrier, manual vmcnt waits and the global -> LDS 16-byte-per-lane load.
#pragma once

#include <utility>

#include "common.h"

namespace cf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

// Workgroup barrier that orders LDS traffic only: global loads still in flight stay in flight.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

#define CF_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt = imm[15:14]:imm[3:0], expcnt imm[6:4], lgkmcnt imm[11:8])
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

typedef int i32x4_t __attribute__((ext_vector_type(4)));

// Raw buffer descriptor over [base, base+bytes): loads past the end return zeros.
__device__ __forceinline__ i32x4_t make_rsrc(const void* base, int64_t bytes) {
    const int64_t lim = bytes < 0 ? 0 : (bytes > 0xFFFFFFFFll ? 0xFFFFFFFFll : bytes);
    const uint64_t b = reinterpret_cast<uint64_t>(base);
    i32x4_t r;
    r.x = (int)(unsigned)b;
    r.y = (int)(unsigned)((b >> 32) & 0xFFFFu);     // stride 0: raw buffer
    r.z = (int)(unsigned)lim;
    r.w = 0x00020000;
    // the descriptor lives in scalar registers: make the uniformity explicit
    r.x = __builtin_amdgcn_readfirstlane(r.x);
    r.y = __builtin_amdgcn_readfirstlane(r.y);
    r.z = __builtin_amdgcn_readfirstlane(r.z);
    return r;
}

// 16 bytes per lane from global memory straight into LDS: lane l of the wave writes
// LDS bytes [lds_base + 16*l, +16).  Issued as inline assembly so that the compiler
// does not serialise later LDS reads against it; completion is tracked by hand with
// vmcnt (the loads of a wave retire in order).
__device__ __forceinline__ void dma16(unsigned lds_base /*wave-uniform*/, i32x4_t rsrc, unsigned voffset) {
    // both scalar operands are wave-uniform by construction; say so (free when the compiler already knows)
    lds_base = __builtin_amdgcn_readfirstlane(lds_base);
    rsrc.x = __builtin_amdgcn_readfirstlane(rsrc.x);
    rsrc.y = __builtin_amdgcn_readfirstlane(rsrc.y);
    rsrc.z = __builtin_amdgcn_readfirstlane(rsrc.z);
    rsrc.w = __builtin_amdgcn_readfirstlane(rsrc.w);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_base), "v"(voffset), "s"(rsrc)
                 : "memory");
}

// 4 bytes per lane: lane l of the wave writes LDS bytes [lds_base + 4*l, +4).
__device__ __forceinline__ void dma4(unsigned lds_base /*wave-uniform*/, i32x4_t rsrc, unsigned voffset) {
    lds_base = __builtin_amdgcn_readfirstlane(lds_base);
    rsrc.x = __builtin_amdgcn_readfirstlane(rsrc.x);
    rsrc.y = __builtin_amdgcn_readfirstlane(rsrc.y);
    rsrc.z = __builtin_amdgcn_readfirstlane(rsrc.z);
    rsrc.w = __builtin_amdgcn_readfirstlane(rsrc.w);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 :
                 : "s"(lds_base), "v"(voffset), "s"(rsrc)
                 : "memory");
}

// The same with a wave-uniform byte offset added to every lane's address (the instruction's
// scalar offset operand): a loop that walks along a matrix keeps the per-lane offsets fixed
// and advances one scalar.
__device__ __forceinline__ void dma16s(unsigned lds_base /*wave-uniform*/, i32x4_t rsrc, unsigned voffset,
                                       unsigned soffset /*wave-uniform*/) {
    lds_base = __builtin_amdgcn_readfirstlane(lds_base);
    soffset = __builtin_amdgcn_readfirstlane(soffset);
    rsrc.x = __builtin_amdgcn_readfirstlane(rsrc.x);
    rsrc.y = __builtin_amdgcn_readfirstlane(rsrc.y);
    rsrc.z = __builtin_amdgcn_readfirstlane(rsrc.z);
    rsrc.w = __builtin_amdgcn_readfirstlane(rsrc.w);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_base), "v"(voffset), "s"(rsrc), "s"(soffset)
                 : "memory");
}

// The same with the LDS destination as a wave-uniform base plus a compile-time byte offset (one
// scalar add straight into M0) and a compile-time offset on the global address (the instruction's
// 12-bit offset field, which takes part in the descriptor's range check and is ALSO added to the
// LDS destination: lane l writes [lds_base + LDS_IMM + INST_OFF + 16*l, +16)).  With one wave per SIMD
// every scalar or vector ALU instruction between two MFMAs costs issue time, so the load carries
// as few of them as the hardware allows.  All scalar operands must be wave-uniform values.
template <int LDS_IMM, int INST_OFF>
__device__ __forceinline__ void dma16i(unsigned lds_base, i32x4_t rsrc, unsigned voffset, unsigned soffset) {
    static_assert(INST_OFF >= 0 && INST_OFF < 4096, "12-bit instruction offset");
    // say that the scalar operands are uniform (free when the compiler already knows)
    lds_base = __builtin_amdgcn_readfirstlane(lds_base);
    soffset = __builtin_amdgcn_readfirstlane(soffset);
    rsrc.x = __builtin_amdgcn_readfirstlane(rsrc.x);
    rsrc.y = __builtin_amdgcn_readfirstlane(rsrc.y);
    rsrc.z = __builtin_amdgcn_readfirstlane(rsrc.z);
    rsrc.w = __builtin_amdgcn_readfirstlane(rsrc.w);
    asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, %4 offen offset:%5 lds"
                 :
                 : "s"(lds_base), "n"(LDS_IMM), "v"(voffset), "s"(rsrc), "s"(soffset), "n"(INST_OFF)
                 : "memory", "scc");
}

// One 16x16x32 bf16 MFMA (acc += a x b, the accumulator pinned to the AGPR file) with a load of
// the dma16i kind wrapped around it: M0 is written ahead of the MFMA and the load follows it, so
// the MFMA is the wait state that the load needs after the write of M0, and no gap between two
// MFMAs of a stream carries more than one of the load's instructions.
template <int LDS_IMM, int INST_OFF>
__device__ __forceinline__ void mfma16_dma16i(f32x4_t& acc, bf16x8_t a, bf16x8_t b, unsigned lds_base, i32x4_t rsrc,
                                              unsigned voffset, unsigned soffset) {
    static_assert(INST_OFF >= 0 && INST_OFF < 4096, "12-bit instruction offset");
    lds_base = __builtin_amdgcn_readfirstlane(lds_base);
    soffset = __builtin_amdgcn_readfirstlane(soffset);
    rsrc.x = __builtin_amdgcn_readfirstlane(rsrc.x);
    rsrc.y = __builtin_amdgcn_readfirstlane(rsrc.y);
    rsrc.z = __builtin_amdgcn_readfirstlane(rsrc.z);
    rsrc.w = __builtin_amdgcn_readfirstlane(rsrc.w);
    asm volatile("s_add_u32 m0, %3, %4\n\tv_mfma_f32_16x16x32_bf16 %0, %1, %2, %0\n\t"
                 "buffer_load_dwordx4 %5, %6, %7 offen offset:%8 lds"
                 : "+a"(acc)
                 : "v"(a), "v"(b), "s"(lds_base), "n"(LDS_IMM), "v"(voffset), "s"(rsrc), "s"(soffset), "n"(INST_OFF)
                 : "memory", "scc");
}

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{})
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}
template <int V> using ic = std::integral_constant<int, V>;

__device__ __forceinline__ unsigned lds_addr_of(const void* p) {
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

}  // namespace cf
