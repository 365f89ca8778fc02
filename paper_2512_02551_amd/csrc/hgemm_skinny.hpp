// Memory-bound kernel family for skinny problems (M of a few rows, NN layout): C = A*B is then a
// stream of B through the chip (Section 4.3 of the paper observes that small problems leave the GPU
// under-used; this is the specialisation for them).
//
// What the machine wants for streaming was measured with pure-load probes: many small workgroups,
// every lane with a handful of independent 16-byte loads in flight, row segments of at least 256
// bytes, no long per-workgroup pipeline to fill and drain.  (A 32 MiB matrix is read cold in 6.3-6.7 us
// that way, against 8-12 us for 128-256 workgroups with deep private pipelines.)  So:
//
//   * grid = column strips of 128 (x) by K slabs (y); a workgroup of 4 waves walks its slab in steps
//     of 64 k-rows; one step is 64 x 128 halves = 16 KiB of B, four 16-byte loads per lane straight
//     into registers, issued two steps ahead of use;
//   * the step's block goes through LDS once (swizzled) so that the transposing read can hand the
//     matrix cores 8 consecutive k per lane; v_mfma_f32_16x16x32_f16 with M on a 16-wide side and the
//     operand roles swapped (the instruction computes a tile of C^T), so a lane owns 4 consecutive
//     columns of one row of C; A (a few rows, cache resident) is loaded straight into registers;
//   * K slabs are summed in slab order: either by the split-K reduction launch, or inside the kernel
//     by the workgroup that arrives last at a strip (FUSED), exactly as in the large-tile kernel.
#pragma once
#include "hgemm_mfma.hpp"

namespace hgemm {

constexpr int kSkinnyCols = 128;       // columns per workgroup
constexpr int kSkinnyStep = 64;        // k-rows per step

// MB = 16-row blocks of A a workgroup multiplies with every block of B it loads (M <= 16 * MB).
template <int MB, bool FUSED>
__global__ __launch_bounds__(256) void skinny_gemm_kernel(GemmArgs g)
{
    typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
    __shared__ __attribute__((aligned(1024))) char lds[kSkinnyStep * kSkinnyCols * 2];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int n0 = blockIdx.x * kSkinnyCols;
    const int split = blockIdx.y;
    const int k_lo = split * g.k_per_split;
    const int k_hi = min(g.K, k_lo + g.k_per_split);
    const int steps = (k_hi - k_lo + kSkinnyStep - 1) / kSkinnyStep;

    // Loads go through buffer descriptors: a lane whose row or column is out of range gets an
    // out-of-range offset and reads zeros, so no load sits behind a branch and all of a step's loads
    // are in flight together.
    const unsigned OOB = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rsrcA =
        __builtin_amdgcn_make_buffer_rsrc((void*)g.A, 0, (int)min((long long)g.M * g.lda * 2, 0x7fffffffLL), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcB =
        __builtin_amdgcn_make_buffer_rsrc((void*)g.B, 0, (int)min((long long)g.K * g.ldb * 2, 0x7fffffffLL), 0x00020000);

    // ---- B: thread t loads 16 bytes (8 columns) of rows r, r+16, r+32, r+48 of a step
    const int lc = t & 15, lr = t >> 4;
    const bool col_ok = n0 + 8 * lc < g.N;
    const unsigned b_off = (unsigned)(((k_lo + lr) * g.ldb + n0 + 8 * lc) * 2);
    // LDS: rows of 256 bytes; the 16-byte chunk index is XORed with 4 * (row % 4) so that the four rows
    // a transposing read touches lie in four different quarters of the bank window
    char* wdst = lds + lr * 256 + ((lc ^ ((lr & 3) << 2)) * 16);

    // ---- fragments.  B: within 16 lanes, lane s supplies row s / 4, columns 4 * (s % 4) .. + 3 of the
    // wave's two 16-column blocks.  A: lane holds A[m = lane % 16][8 * (lane / 16) .. + 7].
    const int s16 = lane & 15, grp = lane >> 4;
    int rd_off[2];
#pragma unroll
    for (int cbi = 0; cbi < 2; ++cbi) {
        const int chunk = 2 * (2 * wave + cbi) + ((s16 & 3) >> 1);
        rd_off[cbi] = (8 * grp + (s16 >> 2)) * 256 + ((chunk ^ ((s16 >> 2) << 2)) * 16) + (s16 & 1) * 8;
    }
    unsigned a_off[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = 16 * mb + s16;
        a_off[mb] = m < g.M ? (unsigned)((m * g.lda + k_lo + 8 * grp) * 2) : OOB;
    }

    auto load_b = [&](int step, uint4v (&q)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k = k_lo + step * kSkinnyStep + lr + 16 * j;
            const bool ok = col_ok && k < k_hi;
            q[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrcB, ok ? b_off + (unsigned)((step * kSkinnyStep + 16 * j) * g.ldb * 2) : OOB, 0, 0);
        }
    };
    auto load_a = [&](int step, uint4v (&f)[MB][2]) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int kc = 0; kc < 2; ++kc) {
                const int k = k_lo + step * kSkinnyStep + 32 * kc + 8 * grp;
                const bool ok = a_off[mb] != OOB && k < k_hi;
                f[mb][kc] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, ok ? a_off[mb] + (unsigned)((step * kSkinnyStep + 32 * kc) * 2) : OOB, 0, 0);
            }
    };

    float4v acc[MB][2];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) acc[mb][cbi] = float4v{0.f, 0.f, 0.f, 0.f};

    // two steps of loads in flight: set u holds step s with s % 2 == u (loads past the slab read zeros)
    uint4v bq[2][4];
    uint4v fa[2][MB][2];
    load_b(0, bq[0]);
    load_a(0, fa[0]);
    load_b(1, bq[1]);
    load_a(1, fa[1]);
    for (int base = 0; base < steps; base += 2) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int step = base + u;
            if (step >= steps) break;
            if (step > 0) __syncthreads();                   // every wave is done reading the previous block
#pragma unroll
            for (int j = 0; j < 4; ++j) *(uint4v*)(wdst + j * 16 * 256) = bq[u][j];
            half8 fa_cur[MB][2];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int kc = 0; kc < 2; ++kc) {
                    union { uint4v i; half8 h; } cv;
                    cv.i = fa[u][mb][kc];
                    fa_cur[mb][kc] = cv.h;
                }
            __syncthreads();
            load_b(step + 2, bq[u]);                         // refill this set: two steps ahead
            load_a(step + 2, fa[u]);
#pragma unroll
            for (int kc = 0; kc < 2; ++kc) {
#pragma unroll
                for (int cbi = 0; cbi < 2; ++cbi) {
                    const char* src = lds + kc * 32 * 256 + rd_off[cbi];
                    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)HGEMM_LDS(src));
                    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)HGEMM_LDS(src + 4 * 256));
                    union { struct { short4v lo, hi; } s; half8 h; } cv;
                    cv.s.lo = lo;
                    cv.s.hi = hi;
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        acc[mb][cbi] = __builtin_amdgcn_mfma_f32_16x16x32_f16(cv.h, fa_cur[mb][kc], acc[mb][cbi], 0, 0, 0);
                }
            }
        }
    }

    // ---- epilogue.  acc[mb][cbi][v] = C[16 mb + lane % 16][n0 + 32 wave + 16 cbi + 4 (lane / 16) + v]
    const bool direct = g.splits == 1;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = 16 * mb + s16;
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) {
            const int n = n0 + 32 * wave + 16 * cbi + 4 * grp;
            if (m >= g.M || n >= g.N) continue;
            if (direct) {
                half4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (_Float16)acc[mb][cbi][e];
                *(half4*)(g.C + (size_t)m * g.ldc + n) = o;
            } else {
                float* dst = g.partial + ((size_t)split * g.M + m) * g.N + n;
                if (FUSED) {
                    union { float4v f; unsigned long long u[2]; } w;
                    w.f = acc[mb][cbi];
                    store_agent((unsigned long long*)dst, w.u[0]);
                    store_agent((unsigned long long*)dst + 1, w.u[1]);
                } else {
                    *(float4v*)dst = acc[mb][cbi];
                }
            }
        }
    }
    if (!FUSED || direct) return;

    // Fused reduction over the K slabs of this strip: device-coherent plane stores above, then the
    // workgroup that arrives last re-reads all planes in slab order (the result does not depend on who
    // is last), rounds once and stores.  Nobody waits for anybody.
    __syncthreads();                                          // its release half waits for this wave's stores
    int* flag = (int*)lds;
    if (t == 0) {
        int* ctr = g.counters + blockIdx.x;
        const int arrived = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (arrived == g.splits - 1) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag = arrived;
    }
    __syncthreads();
    if (*flag != g.splits - 1) return;
    sum_split_planes<256, kSkinnyCols / 4>(g, 0, n0, g.M, t);
}

}  // namespace hgemm
