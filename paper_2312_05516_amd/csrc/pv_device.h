// Internal device-side helpers shared by the kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "pv_plan.h"

namespace pv {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazyLog2 = 8.f;  // the running maximum may lag the true one by this many powers of 2

struct F16 {
    typedef f16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma16(vec8 a, vec8 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x16 mfma32(vec8 a, vec8 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    // The same instruction with its registers pinned: result in ordinary vector registers (the
    // vector ALU reads it next), A operand in vector registers, B operand in accumulation
    // registers (operands that stay put for the whole kernel; named as read-write, though the
    // instruction only reads them, so that the value stays in that register from use to use
    // instead of being parked elsewhere and moved into place).  The compiler does not know what
    // the statement is: whoever reads `d` must keep the instruction's latency in mind (at least
    // two further matrix-core instructions, or the equivalent in s_nop, before a vector-ALU read).
    static __device__ __forceinline__ void mfma32_first(f32x16 &d, u32x4 a, u32x4 &b_acc)
    {
        asm volatile("v_mfma_f32_32x32x16_f16 %0, %2, %1, 0" : "=&v"(d), "+a"(b_acc) : "v"(a));
    }
    // d = a * b + c with c in other registers than d
    static __device__ __forceinline__ void mfma32_from(f32x16 &d, u32x4 a, u32x4 &b_acc, f32x16 c)
    {
        asm volatile("v_mfma_f32_32x32x16_f16 %0, %2, %1, %3"
                     : "=&v"(d), "+a"(b_acc) : "v"(a), "v"(c));
    }
    static __device__ __forceinline__ void mfma32_next(f32x16 &d, u32x4 a, u32x4 &b_acc)
    {
        asm volatile("v_mfma_f32_32x32x16_f16 %0, %2, %1, %0" : "+v"(d), "+a"(b_acc) : "v"(a));
    }
    // the same two with the wait states a vector-ALU write of an operand needs in front: for code
    // outside hand-laid schedules, where the compiler may move operands into place at the last moment
    static __device__ __forceinline__ void mfma32_first_guarded(f32x16 &d, u32x4 a, u32x4 &b_acc)
    {
        asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_f16 %0, %2, %1, 0"
                     : "=&v"(d), "+a"(b_acc) : "v"(a));
    }
    static __device__ __forceinline__ void mfma32_next_guarded(f32x16 &d, u32x4 a, u32x4 &b_acc)
    {
        asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_f16 %0, %2, %1, %0"
                     : "+v"(d), "+a"(b_acc) : "v"(a));
    }
    // two fp32 -> one dword of two 16-bit values (round to nearest even), low half first
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        h2 v = {(_Float16)lo, (_Float16)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
    // acc + low half + high half of a packed pair, in fp32 (one v_dot2 against (1, 1))
    static __device__ __forceinline__ float add_pair(uint32_t packed, float acc)
    {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        const h2 ones = {(_Float16)1.f, (_Float16)1.f};
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, packed), ones, acc, false);
    }
};

struct BF16 {
    typedef bf16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma16(vec8 a, vec8 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x16 mfma32(vec8 a, vec8 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ void mfma32_first(f32x16 &d, u32x4 a, u32x4 &b_acc)
    {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %2, %1, 0" : "=&v"(d), "+a"(b_acc) : "v"(a));
    }
    // d = a * b + c with c in other registers than d
    static __device__ __forceinline__ void mfma32_from(f32x16 &d, u32x4 a, u32x4 &b_acc, f32x16 c)
    {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %2, %1, %3"
                     : "=&v"(d), "+a"(b_acc) : "v"(a), "v"(c));
    }
    static __device__ __forceinline__ void mfma32_next(f32x16 &d, u32x4 a, u32x4 &b_acc)
    {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %2, %1, %0" : "+v"(d), "+a"(b_acc) : "v"(a));
    }
    // the same two with the wait states a vector-ALU write of an operand needs in front: for code
    // outside hand-laid schedules, where the compiler may move operands into place at the last moment
    static __device__ __forceinline__ void mfma32_first_guarded(f32x16 &d, u32x4 a, u32x4 &b_acc)
    {
        asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %2, %1, 0"
                     : "=&v"(d), "+a"(b_acc) : "v"(a));
    }
    static __device__ __forceinline__ void mfma32_next_guarded(f32x16 &d, u32x4 a, u32x4 &b_acc)
    {
        asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %2, %1, %0"
                     : "+v"(d), "+a"(b_acc) : "v"(a));
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        typedef __bf16 b2 __attribute__((ext_vector_type(2)));
        b2 v = {(__bf16)lo, (__bf16)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
    static __device__ __forceinline__ float add_pair(uint32_t packed, float acc)
    {
        typedef __bf16 b2 __attribute__((ext_vector_type(2)));
        const b2 ones = {(__bf16)1.f, (__bf16)1.f};
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(b2, packed), ones, acc, false);
    }
};

template <typename T>
__device__ __forceinline__ typename T::vec8 as_vec8(u32x4 raw)
{
    return __builtin_bit_cast(typename T::vec8, raw);
}

__device__ __forceinline__ u32x4 load16(const void *p)
{
    return *reinterpret_cast<const u32x4 *>(p);
}

// 16-byte load with the streaming (non-temporal) hint: for data that is read once
__device__ __forceinline__ u32x4 load16_stream(const void *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max(a, b, c) in one instruction, for values that are known not to be signalling NaNs (fmaxf on
// values the compiler cannot see through costs an extra canonicalising instruction per input)
__device__ __forceinline__ float max3_raw(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// lane index of the calling thread within its wavefront, wave index made scalar
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63u); }
__device__ __forceinline__ int wave_id()
{
    return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
}

typedef __attribute__((address_space(3))) void *lds_void_ptr;

// Asynchronous 16-byte-per-lane copy from global memory into LDS: lane l of the wavefront writes
// lds_base + 16*l.  Issued as raw instructions so that the compiler's wait-count insertion does
// not serialise it against unrelated LDS reads; completion is awaited explicitly (vmcnt) before the
// barrier that publishes the stage.  lds_base must be wavefront-uniform.  The statement rewrites
// M0.  M0 is a reserved register for this compiler: it never carries a value from one instruction
// to a later one (every instruction that needs M0 gets its own s_mov in front), and it rejects M0
// in a clobber list for that reason, so none is given.
__device__ __forceinline__ void lds_dma16(const void *uniform_base, uint32_t lane_offset,
                                          void *lds_base)
{
    // address = wavefront-uniform 64-bit base (scalar registers) + per-lane 32-bit byte offset
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_void_ptr)lds_base;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(lane_offset), "s"(uniform_base)
                 : "memory");
}

// V part of the KV append, shared by the plain and the rotary-fused append kernels so that the
// bit-exact path exists once.  Thread d (of D) owns head dimension d of one (page, head) tile:
// it gathers that dimension from the `count` (1..8) consecutive new tokens of an append group
// (rows of `vsrc`, `row_stride` elements apart) and stores them at slots slot0 .. slot0+count-1,
// which lie inside one 8-slot run of the V tile.  A full run is one 16-byte store; a partial one
// is written element by element so that the other slots keep their contents.
template <int D>
__device__ __forceinline__ void scatter_v_group(const uint16_t *vsrc, int64_t row_stride,
                                                int count, int slot0, int d, uint16_t *v_tile)
{
    uint16_t vals[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) vals[j] = j < count ? vsrc[j * row_stride + d] : (uint16_t)0;
    uint16_t *vdst = v_tile + ((int64_t)((slot0 >> 3) * D + d) * 8);
    if (count == 8) {
        u32x4 packed;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
            packed[jj] = (uint32_t)vals[2 * jj] | ((uint32_t)vals[2 * jj + 1] << 16);
        *reinterpret_cast<u32x4 *>(vdst) = packed;
    } else {
        const int s0 = slot0 & 7;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (j < count) vdst[s0 + j] = vals[j];
    }
}

// s_waitcnt immediate (gfx9 encoding): wait until at most `vm` vector-memory operations and at most
// `lgkm` LDS / scalar-memory operations are outstanding (15 = do not wait on LDS); the export
// counter is not waited on.
constexpr int waitcnt_imm(int vm, int lgkm)
{
    return (vm & 15) | (7 << 4) | ((lgkm & 15) << 8) | ((vm >> 4) << 14);
}

}  // namespace pv
