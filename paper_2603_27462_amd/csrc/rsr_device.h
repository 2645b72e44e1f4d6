// Device-side building blocks of the RSR multiply kernels (gfx950, wave64): raw LDS
// addressing, DPP scans, and the per-entry gather / tail-store steps written out
// as instructions.  Included by the kernel translation units only.
#pragma once

#include "rsr_internal.h"

namespace rsr {
namespace {

typedef __attribute__((address_space(3))) float lds_f32;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) u32x4 lds_u128;

__device__ __forceinline__ lds_f32 *lds_float(uint32_t addr) {
    return reinterpret_cast<lds_f32 *>(static_cast<uintptr_t>(addr));
}

// ---- cross-lane primitives (DPP; wave64) -------------------------------------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float x) {
    // x + (x moved by the DPP pattern); lanes without a source add 0
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
    return x + __int_as_float(moved);
}

// Inclusive prefix sum over each row of 16 lanes.
__device__ __forceinline__ float row_inclusive_scan(float x) {
    x = dpp_add<0x111, 0xf>(x);  // row_shr:1
    x = dpp_add<0x112, 0xf>(x);  // row_shr:2
    x = dpp_add<0x114, 0xf>(x);  // row_shr:4
    x = dpp_add<0x118, 0xf>(x);  // row_shr:8
    return x;
}

// Inclusive prefix sum over the 64 lanes, in lane order.
__device__ __forceinline__ float wave_inclusive_scan(float x) {
    x = row_inclusive_scan(x);
    x = dpp_add<0x142, 0xa>(x);  // row_bcast:15 into rows 1 and 3
    x = dpp_add<0x143, 0xc>(x);  // row_bcast:31 into rows 2 and 3
    return x;
}

// Signed bit field of `width` bits at bit `at`.
__device__ __forceinline__ float field_as_float(uint32_t word, int at, int width) {
    // (the builtin is declared unsigned: the cast back to int keeps the sign)
    return (float)(int)__builtin_amdgcn_sbfe((int)word, (unsigned)at, (unsigned)width);
}

// ---- the per-entry steps, written out as instructions --------------------------------
// The compiler does not see the LDS operations below, so every consumer is tied
// to them through register operands and the waits are explicit.

// LDS byte address of the element of v an entry names.  HALF = 0: low 16 bits of d.
template <typename VT, int ENC, int HALF>
__device__ __forceinline__ uint32_t entry_addr(uint32_t d) {
    constexpr bool wide = sizeof(VT) == 4;
    if (ENC == kEncSmall) {  // tail<<15 | idx<<1
        if (!wide) return HALF ? ((d >> 16) & 0x7ffeu) : (d & 0x7ffeu);
        return HALF ? ((d >> 15) & 0xfffcu) : ((d & 0x7ffeu) << 1);
    }
    // idx<<1 | tail
    if (!wide) return HALF ? ((d >> 16) & 0xfffeu) : (d & 0xfffeu);
    return HALF ? ((d >> 15) & 0x1fffcu) : ((d & 0xfffeu) << 1);
}

// Gathers eight elements of v as float bits and waits for them, in one instruction block:
// the compiler does not see the LDS operations, and between a read it does not know of and
// the wait for it, it would be free to copy the destination register while the data is still
// on its way.  For bf16 the 16 bits land in the high half of g[i], whose low half is zero
// and stays zero (g is only ever written here).
template <typename VT>
__device__ __forceinline__ void gather8(uint32_t (&g)[8], const uint32_t (&a)[8]) {
    if (sizeof(VT) == 4)
        asm volatile(
            "ds_read_b32 %0, %8\n\t"
            "ds_read_b32 %1, %9\n\t"
            "ds_read_b32 %2, %10\n\t"
            "ds_read_b32 %3, %11\n\t"
            "ds_read_b32 %4, %12\n\t"
            "ds_read_b32 %5, %13\n\t"
            "ds_read_b32 %6, %14\n\t"
            "ds_read_b32 %7, %15\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "+v"(g[0]), "+v"(g[1]), "+v"(g[2]), "+v"(g[3]), "+v"(g[4]), "+v"(g[5]), "+v"(g[6]), "+v"(g[7])
            : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7])
            : "memory");
    else
        asm volatile(
            "ds_read_u16_d16_hi %0, %8\n\t"
            "ds_read_u16_d16_hi %1, %9\n\t"
            "ds_read_u16_d16_hi %2, %10\n\t"
            "ds_read_u16_d16_hi %3, %11\n\t"
            "ds_read_u16_d16_hi %4, %12\n\t"
            "ds_read_u16_d16_hi %5, %13\n\t"
            "ds_read_u16_d16_hi %6, %14\n\t"
            "ds_read_u16_d16_hi %7, %15\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "+v"(g[0]), "+v"(g[1]), "+v"(g[2]), "+v"(g[3]), "+v"(g[4]), "+v"(g[5]), "+v"(g[6]), "+v"(g[7])
            : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7])
            : "memory");
}

// The two entries of dword d: if an entry is a tail, E[ptr] = s, ptr += 4.
// The compare writes the execution mask itself (all 64 lanes are live when this runs:
// the workgroup size is a multiple of 64 and the caller is in wave-uniform control
// flow), and the mask is set back to all ones afterwards.  Big encoding: the tail flag
// is bit 0 / bit 16, moved to the sign by a shift.
__device__ __forceinline__ void tail_store2_big(uint32_t d, float s0, float s1, uint32_t &ptr) {
    uint32_t u;
    asm volatile(
        "v_lshlrev_b32 %[u], 31, %[d]\n\t"
        "v_cmpx_gt_i32 vcc, 0, %[u]\n\t"
        "ds_write_b32 %[p], %[s0]\n\t"
        "v_add_u32 %[p], 4, %[p]\n\t"
        "s_mov_b64 exec, -1\n\t"
        "v_lshlrev_b32 %[u], 15, %[d]\n\t"
        "v_cmpx_gt_i32 vcc, 0, %[u]\n\t"
        "ds_write_b32 %[p], %[s1]\n\t"
        "v_add_u32 %[p], 4, %[p]\n\t"
        "s_mov_b64 exec, -1"
        : [p] "+v"(ptr), [u] "=&v"(u)
        : [d] "v"(d), [s0] "v"(s0), [s1] "v"(s1)
        : "vcc", "memory");
}

// Eight entries (dwords d0..d3) at once, small encoding (the tail flag is the sign of the
// 16-bit entry: a 16-bit compare for the low half, the sign of the dword for the high
// half): the eight tail masks are computed first, as independent instructions, so that the
// part that has to run in order -- set the execution mask, store, advance the pointer --
// is three instructions per entry with a single vector instruction in the dependency chain.
__device__ __forceinline__ void tail_store8_small(uint32_t d0, uint32_t d1, uint32_t d2, uint32_t d3,
                                                  const float (&s)[8], uint32_t &ptr) {
    uint64_t m0, m1, m2, m3, m4, m5, m6, m7;
    asm volatile(
        "v_cmp_gt_i16 %[m0], 0, %[d0]\n\t"
        "v_cmp_gt_i32 %[m1], 0, %[d0]\n\t"
        "v_cmp_gt_i16 %[m2], 0, %[d1]\n\t"
        "v_cmp_gt_i32 %[m3], 0, %[d1]\n\t"
        "v_cmp_gt_i16 %[m4], 0, %[d2]\n\t"
        "v_cmp_gt_i32 %[m5], 0, %[d2]\n\t"
        "v_cmp_gt_i16 %[m6], 0, %[d3]\n\t"
        "v_cmp_gt_i32 %[m7], 0, %[d3]\n\t"
        "s_mov_b64 exec, %[m0]\n\t"
        "ds_write_b32 %[p], %[s0]\n\t"
        "v_add_u32 %[p], 4, %[p]\n\t"
        "s_mov_b64 exec, %[m1]\n\t"
        "ds_write_b32 %[p], %[s1]\n\t"
        "v_add_u32 %[p], 4, %[p]\n\t"
        "s_mov_b64 exec, %[m2]\n\t"
        "ds_write_b32 %[p], %[s2]\n\t"
        "v_add_u32 %[p], 4, %[p]\n\t"
        "s_mov_b64 exec, %[m3]\n\t"
        "ds_write_b32 %[p], %[s3]\n\t"
        "v_add_u32 %[p], 4, %[p]\n\t"
        "s_mov_b64 exec, %[m4]\n\t"
        "ds_write_b32 %[p], %[s4]\n\t"
        "v_add_u32 %[p], 4, %[p]\n\t"
        "s_mov_b64 exec, %[m5]\n\t"
        "ds_write_b32 %[p], %[s5]\n\t"
        "v_add_u32 %[p], 4, %[p]\n\t"
        "s_mov_b64 exec, %[m6]\n\t"
        "ds_write_b32 %[p], %[s6]\n\t"
        "v_add_u32 %[p], 4, %[p]\n\t"
        "s_mov_b64 exec, %[m7]\n\t"
        "ds_write_b32 %[p], %[s7]\n\t"
        "v_add_u32 %[p], 4, %[p]\n\t"
        "s_mov_b64 exec, -1"
        : [p] "+v"(ptr), [m0] "=&s"(m0), [m1] "=&s"(m1), [m2] "=&s"(m2), [m3] "=&s"(m3),
          [m4] "=&s"(m4), [m5] "=&s"(m5), [m6] "=&s"(m6), [m7] "=&s"(m7)
        : [d0] "v"(d0), [d1] "v"(d1), [d2] "v"(d2), [d3] "v"(d3), [s0] "v"(s[0]),
          [s1] "v"(s[1]), [s2] "v"(s[2]), [s3] "v"(s[3]), [s4] "v"(s[4]), [s5] "v"(s[5]),
          [s6] "v"(s[6]), [s7] "v"(s[7])
        : "memory");
}

__device__ __forceinline__ void lds_drain() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

template <typename VT>
__device__ __forceinline__ void lds_store_v(int byte_addr, VT x) {
    *reinterpret_cast<__attribute__((address_space(3))) VT *>(static_cast<uintptr_t>(byte_addr)) = x;
}

}  // namespace
}  // namespace rsr
