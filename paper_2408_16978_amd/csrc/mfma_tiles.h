// Device-side helpers for 64-wide wavefronts and v_mfma_f32_32x32x16_bf16 tiles (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fpdt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// One 32x32x16 bf16 MFMA: acc[32x32] += A[32x16] * B[16x32].
//   A operand: lane l holds A[l%32][8*(l/32) + e], e = 0..7
//   B operand: lane l holds B[8*(l/32) + e][l%32]
//   acc:       lane l, register r holds C[8*(r/4) + 4*(l/32) + r%4][l%32]
__device__ __forceinline__ floatx16 mfma32(bf16x8 a, bf16x8 b, floatx16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Row (0..31) of accumulator register r for this lane.
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// Registers [8*s, 8*s+8) of a 32x32 accumulator, rounded to bf16: the B operand of the
// next MFMA whose contraction runs over the accumulator's rows (TR packing on the A side).
template <int s>
__device__ __forceinline__ bf16x8 pack_half(const floatx16& v)
{
    floatx8 t;
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = v[8 * s + e];
    return __builtin_convertvector(t, bf16x8);
}

// s_waitcnt that waits until at most N vector-memory loads (including direct-to-LDS
// loads) of this wave are still in flight; LDS and export counters are left alone.
// gfx9 encoding: vmcnt = simm16[15:14]:[3:0], expcnt = [6:4], lgkmcnt = [11:8].
template <int N>
__device__ __forceinline__ void wait_vmem_at_most()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}

// Workgroup barrier WITHOUT the memory fence of __syncthreads().  The fence makes a wave wait
// for every vector-memory operation it has in flight, i.e. also for the direct-to-LDS copies
// of tiles that are not needed yet.  The caller waits for exactly what the next tile needs
// (wait_vmem_at_most) and for its own LDS traffic; the empty asm statements keep the compiler
// from moving memory accesses across the barrier.
__device__ __forceinline__ void barrier_no_fence()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): own LDS reads / writes are done
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Direct global -> LDS copy of one 1 KiB fragment by one wave (no VGPR staging): lane l's
// 16 bytes, read from src + 16 l, land at dst + 16 l.  src and dst are wave-uniform.
//
// Issued through inline assembly on purpose.  The compiler's wait-count insertion treats the
// builtin form as an access to both memory and LDS: while one is in flight, every wait for an
// LDS read becomes a wait for ALL LDS reads (no read-ahead under the MFMAs), and LDS reads
// that may alias the copy wait for it.  Hidden from that pass, the copy is tracked by hand:
// callers drain it with wait_vmem_at_most<N>() before the barrier that publishes the tile.
// (Waits the compiler computes for its own vector loads then count too few operations in
// flight, which only makes them stricter.)
//
// copy_address_rule.  A vector-memory instruction that reads its address from scalar registers
// must not follow, within five wait states, a VECTOR instruction that wrote those registers
// (v_readfirstlane_b32 is one).  The compiler keeps that distance for its own instructions; it
// cannot see into inline assembly.  So the copy never reads the caller's registers directly: a
// scalar move takes the address into a register pair of the statement's own first (scalar reads of
// vector-written scalar registers are interlocked by the hardware), and the copy reads that pair.
// The same move is the wait state that the write of M0 needs in front of an LDS-DMA instruction.
__device__ __forceinline__ void frag_to_lds(const u32x4* src_wave_uniform, u32x4* dst_wave_uniform, int lane)
{
    const unsigned lds = __builtin_amdgcn_readfirstlane(
        (unsigned)(uintptr_t)(__attribute__((address_space(3))) void*)dst_wave_uniform);
    const uint64_t a = (uint64_t)(uintptr_t)src_wave_uniform;  // into scalar registers, both halves
    // (readfirstlane returns a signed int: widen each half as unsigned)
    const uint64_t src = ((uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((unsigned)(a >> 32)) << 32) |
                         (uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((unsigned)a);
    uint64_t addr;  // see copy_address_rule below
    asm volatile("s_mov_b32 m0, %1\n\ts_mov_b64 %0, %3\n\tglobal_load_lds_dwordx4 %2, %0"
                 : "=&s"(addr)
                 : "s"(lds), "v"(lane * 16), "s"(src)
                 : "memory");  // m0 is reserved: the compiler sets it right before each use of its own
}

// The same copy with the non-temporal hint: for operands that are read once and must not push
// the tiles other workgroups share out of L2.
__device__ __forceinline__ void frag_to_lds_nt(const u32x4* src_wave_uniform, u32x4* dst_wave_uniform, int lane)
{
    const unsigned lds = __builtin_amdgcn_readfirstlane(
        (unsigned)(uintptr_t)(__attribute__((address_space(3))) void*)dst_wave_uniform);
    const uint64_t a = (uint64_t)(uintptr_t)src_wave_uniform;
    const uint64_t src = ((uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((unsigned)(a >> 32)) << 32) |
                         (uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((unsigned)a);
    uint64_t addr;
    asm volatile("s_mov_b32 m0, %1\n\ts_mov_b64 %0, %3\n\tglobal_load_lds_dwordx4 %2, %0 nt"
                 : "=&s"(addr)
                 : "s"(lds), "v"(lane * 16), "s"(src)
                 : "memory");
}

// The same copy for callers that already hold both addresses in scalar registers (values that
// came out of uniform()): no address arithmetic in vector registers at the point of issue.
// lds_addr is the byte address within LDS, lane16 = 16 * lane.
__device__ __forceinline__ unsigned uniform(unsigned v) { return (unsigned)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ uint64_t uniform(uint64_t v)
{
    return ((uint64_t)uniform((unsigned)(v >> 32)) << 32) | (uint64_t)uniform((unsigned)v);
}
__device__ __forceinline__ unsigned lds_address(const void* p)
{
    return uniform((unsigned)(uintptr_t)(__attribute__((address_space(3))) const void*)p);
}
__device__ __forceinline__ void frag_to_lds_at(uint64_t src_uniform, unsigned lds_addr_uniform, int lane16)
{
    uint64_t addr;
    asm volatile("s_mov_b32 m0, %1\n\ts_mov_b64 %0, %3\n\tglobal_load_lds_dwordx4 %2, %0"
                 : "=&s"(addr)
                 : "s"(lds_addr_uniform), "v"(lane16), "s"(src_uniform)
                 : "memory");
}

// 256 bytes (one dword per lane) global -> LDS the same way: lane l's dword, read from
// src + lane4, lands at lds_addr + 4 l.  lane4 = 4 * lane.
__device__ __forceinline__ void dwords_to_lds_at(uint64_t src_uniform, unsigned lds_addr_uniform, int lane4)
{
    uint64_t addr;
    asm volatile("s_mov_b32 m0, %1\n\ts_mov_b64 %0, %3\n\tglobal_load_lds_dword %2, %0"
                 : "=&s"(addr)
                 : "s"(lds_addr_uniform), "v"(lane4), "s"(src_uniform)
                 : "memory");
}

__device__ __forceinline__ float xor32(float v) { return __shfl_xor(v, 32, 64); }

}  // namespace fpdt
