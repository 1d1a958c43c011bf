// Device helpers shared by the fused-block kernels (gfx950): vector types, requantisation bounds, and the
// clamp / shift / pack of one accumulator tile of v_mfma_i32_32x32x32_i8 into matrix-instruction operand bytes.
#pragma once
#include "ee_internal.hpp"

namespace ee {

typedef int v2i_r __attribute__((ext_vector_type(2)));
typedef int v4i_r __attribute__((ext_vector_type(4)));
typedef int v16i_r __attribute__((ext_vector_type(16)));

__device__ __forceinline__ int ir_med3(int v, int lo, int hi)       // lo <= hi: v clamped to [lo, hi]
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
    return r;
}

// Requantisation bounds on the unshifted accumulator: clamp(acc >> s, lo, hi) == clamp(acc, lo * 2^s, (hi + 1) * 2^s - 1) >> s
// (the shift rounds down, so it is monotone); a bound outside int32 clamps nothing, which is then also right.
struct IrClamp { int shift, lo, hi; };
__device__ __forceinline__ IrClamp ir_clamp(int shift, int lo, int hi)
{
    const long long l = (long long)lo << shift, h = (((long long)hi + 1) << shift) - 1;
    return IrClamp{shift, (int)(l < -2147483648LL ? -2147483648LL : l), (int)(h > 2147483647LL ? 2147483647LL : h)};
}

// clamp, shift and pack 16 accumulators (register 4 q + e = channel 8 q + 4 hi + e of the lane's pixel): the shift writes
// its low byte straight into byte e of the packed dword (sub-dword addressing), so a value costs two instructions.  Then
// lanes l and l + 32, which hold channels {0-3, 8-11, 16-19, 24-27} and {4-7, 12-15, 20-23, 28-31} of one pixel, exchange
// halves: afterwards lane l holds channels 0-15 and lane l + 32 channels 16-31, 4 per dword in order.
// FRESH: the accumulators come straight out of a matrix instruction (no other instruction has touched them since).
template <bool FRESH = true>
__device__ __forceinline__ v4i_r ir_requant_pack(const v16i_r& acc, const IrClamp& c)
{
    unsigned d0, d1, d2, d3;
    int t0, t1, t2, t3;
    const int sh = c.shift, lo = c.lo, hi = c.hi;
    // One block of instructions the compiler does not look into, so it keeps its own distances:
    //   * a matrix instruction's result may be read 18 wait states after it was issued at the earliest (the compiler spaces
    //     only instructions it knows): 20 wait states first, unless the accumulators have been through ordinary instructions;
    //   * an instruction that writes part of a register must not be followed at once by one that reads the same
    //     register: the four dwords (and the four temporaries that carry a clamped value to its shift) take turns.
    // %0-%3 packed dwords, %4-%7 temporaries, %8-%23 accumulators, %24 shift, %25 / %26 bounds
#define EE_IR_MED(t, a) "v_med3_i32 " t ", " a ", %25, %26\n\t"
#define EE_IR_SHB(dst, src, sel, unused) "v_ashrrev_i32_sdwa " dst ", %24, " src " dst_sel:" sel " dst_unused:" unused " src0_sel:DWORD src1_sel:DWORD\n\t"
#define EE_IR_ROUND(a0, a1, a2, a3, sel, unused) \
    EE_IR_MED("%4", a0) EE_IR_MED("%5", a1) EE_IR_MED("%6", a2) EE_IR_MED("%7", a3) \
    EE_IR_SHB("%0", "%4", sel, unused) EE_IR_SHB("%1", "%5", sel, unused) EE_IR_SHB("%2", "%6", sel, unused) EE_IR_SHB("%3", "%7", sel, unused)
#define EE_IR_BODY \
        EE_IR_ROUND("%8", "%12", "%16", "%20", "BYTE_0", "UNUSED_PAD") \
        EE_IR_ROUND("%9", "%13", "%17", "%21", "BYTE_1", "UNUSED_PRESERVE") \
        EE_IR_ROUND("%10", "%14", "%18", "%22", "BYTE_2", "UNUSED_PRESERVE") \
        EE_IR_ROUND("%11", "%15", "%19", "%23", "BYTE_3", "UNUSED_PRESERVE") \
        "s_nop 1"
#define EE_IR_OPERANDS \
        : "=&v"(d0), "=&v"(d1), "=&v"(d2), "=&v"(d3), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3) \
        : "v"(acc[0]), "v"(acc[1]), "v"(acc[2]), "v"(acc[3]), "v"(acc[4]), "v"(acc[5]), "v"(acc[6]), "v"(acc[7]), \
          "v"(acc[8]), "v"(acc[9]), "v"(acc[10]), "v"(acc[11]), "v"(acc[12]), "v"(acc[13]), "v"(acc[14]), "v"(acc[15]), \
          "v"(sh), "v"(lo), "v"(hi)
    if constexpr (FRESH) asm("s_nop 15\n\ts_nop 3\n\t" EE_IR_BODY EE_IR_OPERANDS);
    else asm(EE_IR_BODY EE_IR_OPERANDS);
#undef EE_IR_OPERANDS
#undef EE_IR_BODY
#undef EE_IR_ROUND
#undef EE_IR_SHB
#undef EE_IR_MED
    // v_permlane32_swap(a, b): the upper 32 lanes of a change places with the lower 32 lanes of b
    const auto s02 = __builtin_amdgcn_permlane32_swap(d0, d2, false, false);
    const auto s13 = __builtin_amdgcn_permlane32_swap(d1, d3, false, false);
    return v4i_r{(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
}

}  // namespace ee
