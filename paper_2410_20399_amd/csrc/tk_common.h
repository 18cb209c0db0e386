// Device-side building blocks shared by the gfx950 attention kernels.
//
// Lane layouts used throughout (wave64, measured on gfx950):
//   v_mfma_f32_32x32x16_bf16   D[32x32] += A[32x16] * B[16x32]
//     A operand: lane l holds row  (l % 32), k = 8*(l/32) .. 8*(l/32)+7   (8 bf16)
//     B operand: lane l holds col  (l % 32), k = 8*(l/32) .. 8*(l/32)+7   (8 bf16)
//     C/D      : lane l holds col  (l % 32), rows 8*(r/4) + 4*(l/32) + r%4 for r = 0..15
//   ds_read_b64_tr_b16 (16-lane groups): lane j of a group supplies the address of
//     4 consecutive 16-bit elements; viewing the 16 addresses as a 4-row x 16-column block
//     (lane 4*e + c points at row e, columns 4c..4c+3), lane j receives column j, rows 0..3.
//   global_load_lds_dwordx4: lane l's 16 bytes land at (wave-uniform LDS base) + 16*l.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tk {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;

#define TK_LDS __attribute__((address_space(3)))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// s_waitcnt vmcnt(n) with expcnt/lgkmcnt left unconstrained (gfx9 encoding).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// s_waitcnt vmcnt(n) lgkmcnt(0): additionally every LDS read of this wave has returned.  Used before a
// barrier after which another wave's direct-to-LDS load may overwrite what this wave was reading.
template <int N>
__device__ __forceinline__ void wait_vmcnt_lds_done() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt(0x0070 | (N & 15) | ((N >> 4) << 14));
}

// 16 bytes per lane straight from global memory into LDS; lds_wave_base must be wave-uniform.
__device__ __forceinline__ void load_global_to_lds16(const void* gptr, char* lds_wave_base) {
    __builtin_amdgcn_global_load_lds(gptr, (TK_LDS uint32_t*)lds_wave_base, 16, 0, 0);
}

// Same load, issued through inline assembly so that the compiler does not track it: its LDS-DMA
// bookkeeping holds only a handful of loads and otherwise drains EVERY outstanding load before the
// next LDS read.  The caller owns the ordering: wait_vmcnt<> + barrier before anyone reads the data.
__device__ __forceinline__ void load_global_to_lds16_untracked(const void* gptr, const char* lds_wave_base) {
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(TK_LDS const char*)lds_wave_base;
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_addr), "v"(gptr)
                 : "m0", "memory");   // "memory": LDS contents change behind the compiler's back
}

// The same load with the address split into a wave-uniform base (scalar registers) and a 32-bit byte offset per
// lane: no 64-bit vector add per load.
__device__ __forceinline__ void load_global_to_lds16_sbase_untracked(const void* uniform_base, uint32_t lane_byte_off,
                                                                     const char* lds_wave_base) {
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(TK_LDS const char*)lds_wave_base;
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(lane_byte_off), "s"(uniform_base)
                 : "m0", "memory");
}

// The same load by lanes 0..15 only (256 bytes); the other lanes are masked off for the one instruction.
// Call it with every lane active: it restores the execution mask it found.
__device__ __forceinline__ void load_global_to_lds16_lanes16_untracked(const void* gptr, const char* lds_wave_base) {
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(TK_LDS const char*)lds_wave_base;
    uint64_t saved;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, 0xffff\n\ts_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved)
                 : "s"(lds_addr), "v"(gptr)
                 : "m0", "memory");
}

// 4 bytes per lane, same rules: LDS address = wave base + 4 * lane.  For rows of fp32 statistics,
// whose global address is only 4-byte aligned when N is not a multiple of 4.
__device__ __forceinline__ void load_global_to_lds4_untracked(const void* gptr, const char* lds_wave_base) {
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(TK_LDS const char*)lds_wave_base;
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off"
                 :
                 : "s"(lds_addr), "v"(gptr)
                 : "m0", "memory");
}

// 16-byte LDS read as an MFMA operand (8 consecutive-k bf16).
__device__ __forceinline__ bf16x8 lds_read_b128(const char* smem, int byte_off) {
    return *(const bf16x8*)(smem + byte_off);
}

// Transposing LDS read: returns 4 bf16 taken from 4 consecutive ROWS at this lane's column.
__device__ __forceinline__ bf16x4 lds_read_tr16(const char* smem, int byte_off) {
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((TK_LDS s16x4*)(smem + byte_off));
    return __builtin_bit_cast(bf16x4, v);
}

__device__ __forceinline__ bf16x8 concat(bf16x4 a, bf16x4 b) {
    return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Combine a value with the same lane of the other half-wave (lane ^ 32); every lane gets the result.
// permlane32_swap(x, x) returns {x[0..31], x[0..31]} and {x[32..63], x[32..63]}.
__device__ __forceinline__ float half_max(float x) {
    int xi = __builtin_bit_cast(int, x);
    auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    return __builtin_fmaxf(__builtin_bit_cast(float, (int)r[0]), __builtin_bit_cast(float, (int)r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
    int xi = __builtin_bit_cast(int, x);
    auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    return __builtin_bit_cast(float, (int)r[0]) + __builtin_bit_cast(float, (int)r[1]);
}

__device__ __forceinline__ bf16x2 cvt2(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_convertvector(v, bf16x2);
}

__device__ __forceinline__ bf16x8 cvt8(float a0, float a1, float a2, float a3,
                                       float a4, float a5, float a6, float a7) {
    bf16x2 p0 = cvt2(a0, a1), p1 = cvt2(a2, a3), p2 = cvt2(a4, a5), p3 = cvt2(a6, a7);
    bf16x4 q0 = __builtin_shufflevector(p0, p1, 0, 1, 2, 3);
    bf16x4 q1 = __builtin_shufflevector(p2, p3, 0, 1, 2, 3);
    return concat(q0, q1);
}

// Workgroup id -> logical tile id such that each of the 8 XCDs (workgroups are dealt to them
// round-robin) walks a contiguous range of logical ids, so tiles of one head share one L2.
__device__ __forceinline__ int xcd_remap(int wg, int total) {
    return (total % 8 == 0) ? (wg % 8) * (total / 8) + wg / 8 : wg;
}

}  // namespace tk
