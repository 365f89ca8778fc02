// Instantiates the skinny (memory-bound, small M) kernel family.
#include "hgemm_skinny.hpp"

namespace hgemm {

// Kernel for M <= 16 * mb (mb in {1, 2, 4}), with or without the fused reduction; null for other mb.
void (*skinny_kernel(int mb, bool fused))(GemmArgs)
{
    switch (mb) {
        case 1: return fused ? skinny_gemm_kernel<1, true> : skinny_gemm_kernel<1, false>;
        case 2: return fused ? skinny_gemm_kernel<2, true> : skinny_gemm_kernel<2, false>;
        case 4: return fused ? skinny_gemm_kernel<4, true> : skinny_gemm_kernel<4, false>;
    }
    return nullptr;
}

}  // namespace hgemm
