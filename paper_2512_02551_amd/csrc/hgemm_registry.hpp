// Registry of compiled MFMA specialisations, filled by one function per translation unit.
#pragma once
#include <vector>

#include "hgemm_mfma.hpp"

namespace hgemm {

struct MfmaEntry {
    int bm, bn, bk, wm, wn, st, pf;
    int threads, lds_bytes;
    bool deep;                          // deep-staged configuration: only the one-tile-per-workgroup kernels exist
    void (*plain)(GemmArgs);
    void (*splitk)(GemmArgs);
    void (*plain_tn)(GemmArgs);
    void (*splitk_tn)(GemmArgs);
    void (*streamk)(GemmArgs);
    void (*streamk_tn)(GemmArgs);
    void (*splitk_fused)(GemmArgs);
    void (*splitk_fused_tn)(GemmArgs);
    void (*persist)(GemmArgs);          // null when the configuration cannot stage its epilogue in one LDS buffer
    void (*persist_tn)(GemmArgs);
    void (*acc16)(GemmArgs);            // 16-bit accumulator variant (null for the 16-wide matrix-core blocks)
    void (*acc16_tn)(GemmArgs);
    void (*fixup)(GemmArgs);
    int mi = 32;                        // side of the matrix-core output block
};

template <class C, bool TN> inline void (*persist_kernel())(GemmArgs)
{
    if constexpr (C::CAN_PERSIST) return mfma_gemm_kernel<C, MODE_PERSIST, TN>;
    else return nullptr;
}

template <class C, bool TN> inline void (*acc16_kernel())(GemmArgs)
{
    if constexpr (C::MI == 32) return mfma_gemm_kernel<C, MODE_ACC16, TN>;
    else return nullptr;
}

template <class C> inline MfmaEntry make_entry()
{
    if constexpr (C::DEEP) {
        MfmaEntry e{};
        e.bm = C::BM; e.bn = C::BN; e.bk = C::BK; e.wm = C::WAVES_M; e.wn = C::WAVES_N; e.st = C::STAGES; e.pf = C::PF;
        e.threads = C::THREADS; e.lds_bytes = C::LDS_BYTES; e.deep = C::DEEP; e.mi = C::MI;
        e.plain = mfma_gemm_kernel<C, MODE_PLAIN, false>;
        e.plain_tn = mfma_gemm_kernel<C, MODE_PLAIN, true>;
        return e;
    } else {
        MfmaEntry e{C::BM, C::BN, C::BK, C::WAVES_M, C::WAVES_N, C::STAGES, C::PF, C::THREADS, C::LDS_BYTES, false,
                         mfma_gemm_kernel<C, MODE_PLAIN, false>, mfma_gemm_kernel<C, MODE_SPLITK, false>,
                         mfma_gemm_kernel<C, MODE_PLAIN, true>, mfma_gemm_kernel<C, MODE_SPLITK, true>,
                         mfma_gemm_kernel<C, MODE_STREAMK, false>, mfma_gemm_kernel<C, MODE_STREAMK, true>,
                         mfma_gemm_kernel<C, MODE_SPLITK_FUSED, false>, mfma_gemm_kernel<C, MODE_SPLITK_FUSED, true>,
                         persist_kernel<C, false>(), persist_kernel<C, true>(),
                         acc16_kernel<C, false>(), acc16_kernel<C, true>(),
                         streamk_fixup_kernel<C::BM, C::BN, C::BK>};
        e.mi = C::MI;
        return e;
    }
}

void register_chunk_0(std::vector<MfmaEntry>& out);
void register_chunk_1(std::vector<MfmaEntry>& out);
void register_chunk_2(std::vector<MfmaEntry>& out);
void register_chunk_3(std::vector<MfmaEntry>& out);
void register_chunk_4(std::vector<MfmaEntry>& out);
void register_chunk_5(std::vector<MfmaEntry>& out);
void register_chunk_6(std::vector<MfmaEntry>& out);
void register_chunk_7(std::vector<MfmaEntry>& out);

}  // namespace hgemm
