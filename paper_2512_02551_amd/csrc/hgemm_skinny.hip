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

// Column-major B.  Steps of loads in flight per lane: 16 registers' worth of 16-byte loads shared between the NR / 16
// blocks of B and the MB blocks of A of a step, at least 2, at most 8.  Combinations whose sums would not fit 64 KiB
// of LDS, or whose accumulators and loads would not fit the 128 registers a 16-wave workgroup leaves a lane, do not exist.
template <int WAVES, int MB, int NR>
void (*tn_kernel(bool fused))(GemmArgs)
{
    constexpr int NB = NR / 16;
    constexpr int DEPTH = 16 / (NB + MB) < 2 ? 2 : 16 / (NB + MB) > 8 ? 8 : 16 / (NB + MB);
    if constexpr (WAVES * MB * NB <= 64 && (WAVES < 16 || MB * NB <= 4))
        return fused ? skinny_tn_gemm_kernel<MB, true, DEPTH, WAVES, NR> : skinny_tn_gemm_kernel<MB, false, DEPTH, WAVES, NR>;
    else
        return nullptr;
}

template <int WAVES>
void (*tn_kernel_for(int mb, bool fused, int nr))(GemmArgs)
{
    switch (mb * 100 + nr) {
        case 116: return tn_kernel<WAVES, 1, 16>(fused);
        case 132: return tn_kernel<WAVES, 1, 32>(fused);
        case 164: return tn_kernel<WAVES, 1, 64>(fused);
        case 216: return tn_kernel<WAVES, 2, 16>(fused);
        case 232: return tn_kernel<WAVES, 2, 32>(fused);
        case 264: return tn_kernel<WAVES, 2, 64>(fused);
        case 416: return tn_kernel<WAVES, 4, 16>(fused);
        case 432: return tn_kernel<WAVES, 4, 32>(fused);
        case 464: return tn_kernel<WAVES, 4, 64>(fused);
    }
    return nullptr;
}
}  // namespace

// Kernel for M <= 16 * mb (mb in {1, 2, 4}) and workgroups of 4, 8 or 16 waves, with or without the fused
// reduction, for row-major B (tn_rows = 0) or column-major B with tn_rows = 16, 32 or 64 rows of B per workgroup;
// null for other values.
void (*skinny_kernel(int mb, bool fused, int waves, int tn_rows))(GemmArgs)
{
    switch (waves) {
        case 4: return tn_rows ? tn_kernel_for<4>(mb, fused, tn_rows) : kernel_for<4>(mb, fused);
        case 8: return tn_rows ? tn_kernel_for<8>(mb, fused, tn_rows) : kernel_for<8>(mb, fused);
        case 16: return tn_rows ? tn_kernel_for<16>(mb, fused, tn_rows) : kernel_for<16>(mb, fused);
    }
    return nullptr;
}

}  // namespace hgemm
