// Instantiates the skinny (memory-bound, small M) kernel family.
#include "hgemm_skinny.hpp"

namespace hgemm {

namespace {
#ifndef HGEMM_SKINNY_DEPTH
#define HGEMM_SKINNY_DEPTH 2
#endif
constexpr int kDepth = HGEMM_SKINNY_DEPTH;      // steps of loads a wave keeps in flight (4 KiB each)

template <int WAVES>
void (*kernel_for(int mb, bool fused))(GemmArgs)
{
    switch (mb) {
        case 1: return fused ? skinny_gemm_kernel<1, true, kDepth, WAVES> : skinny_gemm_kernel<1, false, kDepth, WAVES>;
        case 2: return fused ? skinny_gemm_kernel<2, true, kDepth, WAVES> : skinny_gemm_kernel<2, false, kDepth, WAVES>;
        case 4:
            // 16 waves leave a lane 128 registers: two blocks of A at most
            if constexpr (WAVES < 16) return fused ? skinny_gemm_kernel<4, true, kDepth, WAVES> : skinny_gemm_kernel<4, false, kDepth, WAVES>;
            break;
    }
    return nullptr;
}

template <int WAVES>
void (*tn_kernel_for(int mb, bool fused))(GemmArgs)
{
    // loads in flight per lane: 8 steps of 16 bytes of B (and of every 16-row block of A) for one block, 4 for more
    switch (mb) {
        case 1: return fused ? skinny_tn_gemm_kernel<1, true, 8, WAVES> : skinny_tn_gemm_kernel<1, false, 8, WAVES>;
        case 2: return fused ? skinny_tn_gemm_kernel<2, true, 4, WAVES> : skinny_tn_gemm_kernel<2, false, 4, WAVES>;
        case 4:
            if constexpr (WAVES < 16) return fused ? skinny_tn_gemm_kernel<4, true, 4, WAVES> : skinny_tn_gemm_kernel<4, false, 4, WAVES>;
            break;
    }
    return nullptr;
}
}  // namespace

// Kernel for M <= 16 * mb (mb in {1, 2, 4}) and workgroups of 4, 8 or 16 waves, with or without the fused
// reduction, for row-major B (tn = false) or column-major B; null for other values.
void (*skinny_kernel(int mb, bool fused, int waves, bool tn))(GemmArgs)
{
    switch (waves) {
        case 4: return tn ? tn_kernel_for<4>(mb, fused) : kernel_for<4>(mb, fused);
        case 8: return tn ? tn_kernel_for<8>(mb, fused) : kernel_for<8>(mb, fused);
        case 16: return tn ? tn_kernel_for<16>(mb, fused) : kernel_for<16>(mb, fused);
    }
    return nullptr;
}

}  // namespace hgemm
