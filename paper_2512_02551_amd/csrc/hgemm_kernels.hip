// Instantiates the MFMA kernels of one chunk of hgemm_configs.inc (compile with -DHGEMM_CHUNK=k).
#include "hgemm_registry.hpp"

#ifndef HGEMM_CHUNK
#error "compile with -DHGEMM_CHUNK=<0..HGEMM_NUM_CHUNKS-1>"
#endif

#define HGEMM_PASTE2(a, b) a##b
#define HGEMM_PASTE(a, b) HGEMM_PASTE2(a, b)

namespace hgemm {

template <int CHUNK, class C> struct MaybeEntry {
    static void add(std::vector<MfmaEntry>&) {}
};
template <class C> struct MaybeEntry<HGEMM_CHUNK, C> {
    static void add(std::vector<MfmaEntry>& out) { out.push_back(make_entry<C>()); }
};

void HGEMM_PASTE(register_chunk_, HGEMM_CHUNK)(std::vector<MfmaEntry>& out)
{
#define HGEMM_CFG(chunk, bm, bn, bk, wm, wn, st, ...) MaybeEntry<chunk, MfmaCfg<bm, bn, bk, wm, wn, st, __VA_ARGS__>>::add(out);
#include "hgemm_configs.inc"
}

}  // namespace hgemm
