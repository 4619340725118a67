// LDS-direct loads (global memory -> LDS without passing through registers) for gfx950.
//
// Each active lane supplies a 32-bit byte offset from a wave-uniform base pointer; lane i's data lands
// in LDS at lds_base + i * size, whether or not the lanes below it are active.  The loads are written
// as inline assembly so that the compiler's wait-count bookkeeping does not tie them to later LDS
// reads: a stage's loads stay in flight while the previous stage is being multiplied.  The price is
// that completion must be awaited explicitly (lds_dma_wait_all) before the barrier that publishes
// the data.
#ifndef IOLB_LDS_DMA_H
#define IOLB_LDS_DMA_H

#include <hip/hip_runtime.h>

namespace iolb {

typedef __attribute__((address_space(3))) float* lds_float_ptr;

// Byte address of an LDS location (wave-uniform by construction at every call site).
__device__ __forceinline__ unsigned lds_byte_address(const float* p)
{
    return __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lds_float_ptr)p);
}

// 4 bytes per lane from base + offset_bytes.
__device__ __forceinline__ void lds_dma_load_4(const float* base, unsigned offset_bytes, unsigned lds_base_bytes)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :
                 : "v"(offset_bytes), "s"(base), "s"(lds_base_bytes)
                 : "memory", "m0");
}

// 16 bytes per lane from base + offset_bytes; both sides 16-byte aligned.
__device__ __forceinline__ void lds_dma_load_16(const float* base, unsigned offset_bytes, unsigned lds_base_bytes)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(offset_bytes), "s"(base), "s"(lds_base_bytes)
                 : "memory", "m0");
}

// Wait until every load this wave has issued has written its data.  Written with the builtin, not as assembly, so
// that the compiler's own wait-count bookkeeping sees it: after an assembly wait it still believes its earlier
// loads to registers are in flight, and its next wait for them (or before it reuses their registers) then also
// waits for the LDS-direct loads issued in between -- a full memory latency in the middle of a stage.
// s_waitcnt immediate of gfx9: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14]; 0x0F70 = vmcnt(0) only.
__device__ __forceinline__ void lds_dma_wait_all()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);
    asm volatile("" ::: "memory");
}

// Wait until at most N of the wave's loads are still in flight (loads complete in the order they were issued).  The
// registers the awaited loads write are operands, so that no use of them is moved above the wait.  For loads that
// were themselves issued from assembly: the compiler knows of neither.
template <int N, class V>
__device__ __forceinline__ void wait_loads(V& a) { asm volatile("s_waitcnt vmcnt(%1)" : "+v"(a) : "n"(N)); }
template <int N, class V>
__device__ __forceinline__ void wait_loads(V& a, V& b) { asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N)); }
template <int N, class V>
__device__ __forceinline__ void wait_loads(V& a, V& b, V& c, V& d)
{
    asm volatile("s_waitcnt vmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}
// The same without registers to tie: for data that lands in LDS.
template <int N>
__device__ __forceinline__ void wait_loads_lds() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

// Stages `nrows` rows of 4*row4 contiguous floats (row r starts at src + r * pitch floats) into LDS,
// packed row after row from lds_dst.  src, lds_dst and every size are wave-uniform; src, pitch and
// lds_dst are multiples of 4 floats.  Rows beyond the caller's tensor must exist (zero rows are
// provided by the producers).
//   row4 divides 64: one instruction moves 64/row4 whole rows;
//   64 divides row4: a wave moves a row in row4/64 instructions;
//   otherwise: element-wise split with a per-lane division (rare tile widths).
__device__ __forceinline__ void stage_rows(const float* src, int pitch, int row4, int nrows, float* lds_dst,
                                           int wave, int nwaves, int lane)
{
    if (row4 <= 64 && (64 % row4) == 0) {
        const int rows_per_instr = 64 / row4;
        const unsigned voff = 4u * (unsigned)((lane / row4) * pitch + (lane % row4) * 4);
        for (int r0 = wave * rows_per_instr; r0 < nrows; r0 += nwaves * rows_per_instr) {
            if (r0 + lane / row4 < nrows)
                lds_dma_load_16(src + (size_t)r0 * pitch, voff, lds_byte_address(lds_dst + r0 * row4 * 4));
        }
    } else if ((row4 % 64) == 0) {
        const int chunks = row4 / 64;
        const unsigned voff = 16u * (unsigned)lane;
        for (int r = wave; r < nrows; r += nwaves)
            for (int ch = 0; ch < chunks; ++ch)
                lds_dma_load_16(src + (size_t)r * pitch + ch * 256, voff, lds_byte_address(lds_dst + (r * row4 + ch * 64) * 4));
    } else {
        const int total = nrows * row4;
        for (int e0 = wave * 64; e0 < total; e0 += nwaves * 64) {
            const int e = e0 + lane;
            if (e < total) {
                const int r = e / row4, q = e - r * row4;
                lds_dma_load_16(src, 4u * (unsigned)(r * pitch + q * 4), lds_byte_address(lds_dst + e0 * 4));
            }
        }
    }
}

}  // namespace iolb

#endif
