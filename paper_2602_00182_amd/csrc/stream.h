// Streaming helpers shared by the GEMM kernels: LDS-DMA loads written as assembly, and the wait that
// names how many of a wave's loads may stay in flight.
#pragma once
#include <stdint.h>

#include <hip/hip_runtime.h>

namespace det {

typedef __attribute__((address_space(3))) char lds_char_t;

// One wave instruction: 64 lanes x 16 bytes from global memory straight into the 1 KB LDS block at
// byte address lds_addr (wave-uniform); lane l lands at lds_addr + 16 l.  Written as assembly so
// that the completion wait below can name a count instead of draining every load in flight.
// The source is a wave-uniform base plus a 32-bit byte offset per lane, so that the per-lane part is
// a constant of the kernel and every advance is scalar arithmetic.
__device__ __forceinline__ void dma_block(const void* base, uint32_t lane_off, uint32_t lds_addr)
{
    uint32_t saved_m0;
    asm volatile(
        "s_mov_b32 %0, m0\n\t"
        "s_mov_b32 m0, %1\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %2, %3\n\t"
        "s_mov_b32 m0, %0"
        : "=&s"(saved_m0)
        : "s"(lds_addr), "v"(lane_off), "s"(base)
        : "memory");
}

// A run of such loads with constant strides, three instructions a load: M0 is set once and then
// advanced in place, and the source advances in the per-lane offset.  (Nothing else in this file
// uses M0, and the compiler sets it itself before any instruction of its own that reads it.)
__device__ __forceinline__ void dma_run_begin(uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" ::"s"(lds_addr) : "memory");
}
__device__ __forceinline__ void dma_run_next(const void* base, uint32_t& lane_off, uint32_t src_stride, uint32_t lds_stride)
{
    asm volatile(
        "global_load_lds_dwordx4 %0, %1\n\t"
        "s_add_u32 m0, m0, %3\n\t"
        "v_add_u32 %0, %2, %0"
        : "+v"(lane_off)
        : "s"(base), "s"(src_stride), "s"(lds_stride)
        : "memory", "scc");
}
__device__ __forceinline__ void dma_run(const void* base, uint32_t lane_off, uint32_t src_stride, uint32_t lds_addr,
                                        uint32_t lds_stride, int n)
{
    dma_run_begin(lds_addr);
    for (; n >= 4; n -= 4) {
        dma_run_next(base, lane_off, src_stride, lds_stride);
        dma_run_next(base, lane_off, src_stride, lds_stride);
        dma_run_next(base, lane_off, src_stride, lds_stride);
        dma_run_next(base, lane_off, src_stride, lds_stride);
    }
    for (; n > 0; --n) dma_run_next(base, lane_off, src_stride, lds_stride);
}

// Waits until at most n of this wave's loads are outstanding, then the workgroup barrier.  The load
// counter of the wait instruction has six bits and its largest value, 63, means "do not wait", so 63 and
// anything above fall back to waiting for all loads; a wave must also never let more than 62 loads pile
// up (the host checks the schedule it hands to the kernels for that).  The count is an
// immediate of the wait instruction, so the wait is picked by a computed jump into a table of
// 64 two-instruction entries (8 bytes each): two taken branches where a compare tree takes six.
#define DET_W1(n) "s_waitcnt vmcnt(" #n ")\n\ts_branch .Ldet_wend%=\n\t"
#define DET_W8(a, b, c, d, e, f, g, h) DET_W1(a) DET_W1(b) DET_W1(c) DET_W1(d) DET_W1(e) DET_W1(f) DET_W1(g) DET_W1(h)
__device__ __forceinline__ void wait_loads_then_barrier(int n)
{
    uint32_t off = (uint32_t)(n > 62 ? 0 : n) << 3;
    asm volatile(
        "s_getpc_b64 s[98:99]\n"
        ".Ldet_wbase%=:\n\t"
        "s_add_u32 %0, %0, .Ldet_wtab%=-.Ldet_wbase%=\n\t"
        "s_add_u32 s98, s98, %0\n\t"
        "s_addc_u32 s99, s99, 0\n\t"
        "s_setpc_b64 s[98:99]\n"
        ".Ldet_wtab%=:\n\t"
        DET_W8(0, 1, 2, 3, 4, 5, 6, 7) DET_W8(8, 9, 10, 11, 12, 13, 14, 15)
        DET_W8(16, 17, 18, 19, 20, 21, 22, 23) DET_W8(24, 25, 26, 27, 28, 29, 30, 31)
        DET_W8(32, 33, 34, 35, 36, 37, 38, 39) DET_W8(40, 41, 42, 43, 44, 45, 46, 47)
        DET_W8(48, 49, 50, 51, 52, 53, 54, 55) DET_W8(56, 57, 58, 59, 60, 61, 62, 63)
        ".Ldet_wend%=:\n\t"
        "s_barrier"
        : "+s"(off)
        :
        : "memory", "scc", "s98", "s99");
}
#undef DET_W8
#undef DET_W1

}  // namespace det
