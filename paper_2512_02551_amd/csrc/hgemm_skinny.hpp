// Memory-bound kernel family for skinny problems (M of a few rows, NN layout): C = A*B is then a
// stream of B through the chip (Section 4.3 of the paper observes that small problems leave the GPU
// under-used; this is the specialisation for them).
//
// What the machine wants for streaming was measured with pure-load probes: many small workgroups,
// every lane with a handful of independent 16-byte loads in flight, row segments of at least 256
// bytes, no long per-workgroup pipeline to fill and drain.  (A 32 MiB matrix is read cold in 6.3-6.7 us
// that way, against 8-12 us for 128-256 workgroups with deep private pipelines.)  So:
//
//   * grid = column strips of 128 (x) by K slabs (y); a workgroup of WAVES waves walks its slab in
//     steps of 16 * WAVES k-rows; a wave owns 16 rows of a step (wave w: rows 16 w .. 16 w + 15;
//     16-lane group g of it: rows 4 g .. 4 g + 3) and all 128 columns: four 16-byte loads per lane
//     straight into registers, DEPTH steps of them in flight;
//   * no trip through LDS and no barrier in the main loop.  v_mfma_f32_16x16x16_f16 takes 4
//     consecutive k per lane, which is what a lane has after its four loads (the same 8 columns of 4
//     consecutive rows of B) once the 4 x 8 block of halves it holds is transposed inside its own
//     registers (16 two-input byte selections); M sits on the instruction's other 16-wide side, A (a few
//     rows, cache resident) is loaded straight into registers, 8 bytes per lane and step.  Every
//     product the matrix cores form is a product A[m][k] * B[k][n] of the definition (rows of A
//     beyond M and k-rows beyond the slab are read as zeros and only ever meet each other or rows
//     that are not stored), so non-finite values stay in the elements the definition gives them;
//   * the waves' sums meet once, at the end, through LDS (four waves at a time) and are added in wave
//     order; K slabs are summed in slab order: either by the split-K reduction launch, or inside the
//     kernel by the workgroup that arrives last at a strip (FUSED), exactly as in the large-tile kernel.
//
// (An earlier form staged each 64 x 128 block of B through LDS for a transposing read and
// 16x16x32 instructions, with two barriers per step; this form is 3-30 % faster on every shape tried.)
#pragma once
#include "hgemm_mfma.hpp"

namespace hgemm {

constexpr int kSkinnyCols = 128;       // columns per workgroup

// MB = 16-row blocks of A a workgroup multiplies with every block of B it loads (M <= 16 * MB).
template <int MB, bool FUSED, int DEPTH, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void skinny_gemm_kernel(GemmArgs g)
{
    typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
    typedef unsigned int uint2v __attribute__((ext_vector_type(2)));
    constexpr int STEP = 16 * WAVES;                           // k-rows per step of the workgroup
    constexpr int PITCH = kSkinnyCols + 4;                     // floats per staged row of sums
    static_assert(WAVES % 4 == 0, "the sums meet four waves at a time");
    __shared__ __attribute__((aligned(16))) float red[4 * 16 * PITCH];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int n0 = blockIdx.x * kSkinnyCols;
    const int split = blockIdx.y;
    const int k_lo = split * g.k_per_split;
    const int k_hi = min(g.K, k_lo + g.k_per_split);
    const int steps = (k_hi - k_lo + STEP - 1) / STEP;

    const unsigned OOB = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rsrcA =
        __builtin_amdgcn_make_buffer_rsrc((void*)g.A, 0, (int)min((long long)g.M * g.lda * 2, 0x7fffffffLL), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcB =
        __builtin_amdgcn_make_buffer_rsrc((void*)g.B, 0, (int)min((long long)g.K * g.ldb * 2, 0x7fffffffLL), 0x00020000);

    // lane (grp, c16): rows krow0 + STEP * step + s (s = 0..3) of B, columns n0 + 8 c16 .. + 7;
    // A[16 mb + c16][krow0 + STEP * step .. + 3]
    const int c16 = lane & 15, grp = lane >> 4;
    const int krow0 = k_lo + 16 * wave + 4 * grp;
    const bool col_ok = n0 + 8 * c16 < g.N;
    const unsigned b_off = (unsigned)((krow0 * g.ldb + n0 + 8 * c16) * 2);
    unsigned a_off[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = 16 * mb + c16;
        a_off[mb] = m < g.M ? (unsigned)((m * g.lda + krow0) * 2) : OOB;
    }
    auto load_b = [&](int step, uint4v (&q)[4]) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const bool ok = col_ok && krow0 + step * STEP + s < k_hi;
            q[s] = __builtin_amdgcn_raw_buffer_load_b128(rsrcB, ok ? b_off + (unsigned)((step * STEP + s) * g.ldb * 2) : OOB, 0, 0);
        }
    };
    // K is a multiple of 8 and krow0 of 4: the four k of a lane are in range together or not at all
    auto load_a = [&](int step, uint2v (&f)[MB]) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const bool ok = a_off[mb] != OOB && krow0 + step * STEP < k_hi;
            f[mb] = __builtin_amdgcn_raw_buffer_load_b64(rsrcA, ok ? a_off[mb] + (unsigned)(step * STEP * 2) : OOB, 0, 0);
        }
    };

    float4v acc[MB][8];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[mb][j] = float4v{0.f, 0.f, 0.f, 0.f};

    // set u holds step s with s % DEPTH == u (loads past the slab read zeros)
    uint4v bq[DEPTH][4];
    uint2v fa[DEPTH][MB];
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) {
        load_b(u, bq[u]);
        load_a(u, fa[u]);
    }
    for (int base = 0; base < steps; base += DEPTH) {
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            const int step = base + u;
            if (step >= steps) break;
            // tb[j] = (B[k][n], B[k+1][n], B[k+2][n], B[k+3][n]) for the lane's column n = 8 c16 + j
            uint2v tb[8];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const unsigned x0 = bq[u][0][d], x1 = bq[u][1][d], x2 = bq[u][2][d], x3 = bq[u][3][d];
                tb[2 * d] = uint2v{(x0 & 0xffffu) | (x1 << 16), (x2 & 0xffffu) | (x3 << 16)};
                tb[2 * d + 1] = uint2v{(x0 >> 16) | (x1 & 0xffff0000u), (x2 >> 16) | (x3 & 0xffff0000u)};
            }
            uint2v af[MB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) af[mb] = fa[u][mb];
            load_b(step + DEPTH, bq[u]);                     // refill this set
            load_a(step + DEPTH, fa[u]);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                union { uint2v i; half4 h; } bv;
                bv.i = tb[j];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    union { uint2v i; half4 h; } av;
                    av.i = af[mb];
                    acc[mb][j] = __builtin_amdgcn_mfma_f32_16x16x16f16(bv.h, av.h, acc[mb][j], 0, 0, 0);
                }
            }
        }
    }

    // ---- the waves' sums meet in LDS, one 16-row block of C and four waves at a time.
    // acc[mb][j][r] belongs to C[16 mb + c16][n0 + 32 grp + 8 r + j]
    const bool direct = g.splits == 1;
    float* mine = red + ((wave & 3) * 16 + c16) * PITCH + 32 * grp;
    const bool summing = t < 256;                              // summing role: one row, 8 columns
    const int orow = (t >> 4) & 15, ocol = 8 * (t & 15);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        float4v s0 = float4v{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
        for (int w0 = 0; w0 < WAVES; w0 += 4) {
            if (mb > 0 || w0 > 0) __syncthreads();             // the previous round's sums have been read
            if (wave >= w0 && wave < w0 + 4) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    *(float4v*)(mine + 8 * r) = float4v{acc[mb][0][r], acc[mb][1][r], acc[mb][2][r], acc[mb][3][r]};
                    *(float4v*)(mine + 8 * r + 4) = float4v{acc[mb][4][r], acc[mb][5][r], acc[mb][6][r], acc[mb][7][r]};
                }
            }
            __syncthreads();
            if (summing) {
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float* src = red + (w * 16 + orow) * PITCH + ocol;
                    s0 += *(const float4v*)src;
                    s1 += *(const float4v*)(src + 4);
                }
            }
        }
        const int m = 16 * mb + orow, n = n0 + ocol;
        if (!summing || m >= g.M || n >= g.N) continue;
        if (direct) {
            half8 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o[e] = (_Float16)s0[e];
                o[4 + e] = (_Float16)s1[e];
            }
            *(half8*)(g.C + (size_t)m * g.ldc + n) = o;
        } else {
            float* dst = g.partial + ((size_t)split * g.M + m) * g.N + n;
            if (FUSED) {
                union { float4v f; unsigned long long u[2]; } v0, v1;
                v0.f = s0;
                v1.f = s1;
                store_agent((unsigned long long*)dst, v0.u[0]);
                store_agent((unsigned long long*)dst + 1, v0.u[1]);
                store_agent((unsigned long long*)dst + 2, v1.u[0]);
                store_agent((unsigned long long*)dst + 3, v1.u[1]);
            } else {
                *(float4v*)dst = s0;
                *(float4v*)(dst + 4) = s1;
            }
        }
    }
    if (!FUSED || direct) return;

    // Fused reduction over the K slabs of this strip: device-coherent plane stores above, then the
    // workgroup that arrives last re-reads all planes in slab order (the result does not depend on who
    // is last), rounds once and stores.  Nobody waits for anybody.
    __syncthreads();
    int* flag = (int*)red;
    if (t == 0) {
        int* ctr = g.counters + blockIdx.x;
        const int arrived = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (arrived == g.splits - 1) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag = arrived;
    }
    __syncthreads();
    if (*flag != g.splits - 1) return;
    sum_split_planes<64 * WAVES, kSkinnyCols / 4>(g, 0, n0, g.M, t);
}

// The same family for column-major B (stored N x K, K contiguous: the layout in which frameworks keep the
// weights of a linear layer).  Here nothing needs transposing: v_mfma_f32_16x16x32_f16 takes 8 consecutive k
// per lane, and a 16-byte load of row n of B is exactly that.  A workgroup owns NR = 16, 32 or 64 rows of B (as
// many columns of C), so N / NR workgroups exist before K is split at all; its WAVES waves split the
// workgroup's K range into contiguous parts (every row is read in runs of kilobytes), each wave keeps DEPTH
// steps of loads in flight (NR / 16 KiB of B each), holds 4 accumulator registers per 16 x 16 block of C, and
// the waves' sums meet in LDS at the end and are added in wave order.  Every workgroup reads the rows of A it
// multiplies once per NR rows of B: at NR = 16 and M = 16 that is as many bytes through the L1s again as B
// itself, which is what the wider workgroups are for.  grid.y splits K further (planes, reduction launch or
// FUSED) for short, wide-K problems.
constexpr int kSkinnyTnRows = 16;      // rows of B (columns of C) per workgroup unless a spec asks for more

template <int MB, bool FUSED, int DEPTH, int WAVES, int NR>
__global__ __launch_bounds__(64 * WAVES) void skinny_tn_gemm_kernel(GemmArgs g)
{
    typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
    constexpr int NB = NR / 16;                                // 16-row blocks of B per workgroup
    static_assert(NR % 16 == 0 && WAVES * MB * NB <= 64, "the waves' sums meet in at most 64 KiB of LDS");
    __shared__ __attribute__((aligned(16))) float red[WAVES * MB * NB * 64 * 4];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int n0 = blockIdx.x * NR;
    const int split = blockIdx.y;
    const int k_lo = split * g.k_per_split;
    const int k_hi = min(g.K, k_lo + g.k_per_split);
    const int per_wave = g.k_per_split / WAVES;                // a multiple of 32
    const int kw = k_lo + wave * per_wave;                     // this wave's part of the slab
    const int kw_hi = min(k_hi, kw + per_wave);
    const int steps = kw < kw_hi ? (kw_hi - kw + 31) / 32 : 0;

    const unsigned OOB = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rsrcA =
        __builtin_amdgcn_make_buffer_rsrc((void*)g.A, 0, (int)min((long long)g.M * g.lda * 2, 0x7fffffffLL), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcB =
        __builtin_amdgcn_make_buffer_rsrc((void*)g.B, 0, (int)min((long long)g.N * g.ldb * 2, 0x7fffffffLL), 0x00020000);

    // lane (grp, c16): B rows n0 + 16 nb + c16 and A rows 16 mb + c16, k = kw + 32 step + 8 grp .. + 7 (K is a
    // multiple of 8: the eight k of a lane are in range together or not at all)
    const int c16 = lane & 15, grp = lane >> 4;
    const int k0 = kw + 8 * grp;
    unsigned b_off[NB], a_off[MB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int n = n0 + 16 * nb + c16;
        b_off[nb] = n < g.N ? (unsigned)((n * g.ldb + k0) * 2) : OOB;
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = 16 * mb + c16;
        a_off[mb] = m < g.M ? (unsigned)((m * g.lda + k0) * 2) : OOB;
    }
    auto load_step = [&](int step, uint4v (&b)[NB], uint4v (&a)[MB]) {
        const bool ok = k0 + 32 * step < kw_hi;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
            b[nb] = __builtin_amdgcn_raw_buffer_load_b128(rsrcB, ok && b_off[nb] != OOB ? b_off[nb] + (unsigned)(step * 64) : OOB, 0, 0);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            a[mb] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, ok && a_off[mb] != OOB ? a_off[mb] + (unsigned)(step * 64) : OOB, 0, 0);
    };

    float4v acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = float4v{0.f, 0.f, 0.f, 0.f};

    uint4v bq[DEPTH][NB];
    uint4v fa[DEPTH][MB];
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) load_step(u, bq[u], fa[u]);
    for (int base = 0; base < steps; base += DEPTH) {
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            const int step = base + u;
            if (step >= steps) break;
            union { uint4v i; half8 h; } bv[NB], av[MB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) bv[nb].i = bq[u][nb];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) av[mb].i = fa[u][mb];
            load_step(step + DEPTH, bq[u], fa[u]);           // refill this set
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(bv[nb].h, av[mb].h, acc[mb][nb], 0, 0, 0);
        }
    }

    // ---- the waves' sums meet in LDS.  acc[mb][nb][r] belongs to C[16 mb + c16][n0 + 16 nb + 4 grp + r]
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) *(float4v*)(red + (((wave * MB + mb) * NB + nb) * 64 + lane) * 4) = acc[mb][nb];
    __syncthreads();
    const bool direct = g.splits == 1;
    // block (mb, nb) is summed by wave (mb * NB + nb) % WAVES
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            if ((mb * NB + nb) % WAVES != wave) continue;
            float4v s = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < WAVES; ++w) s += *(const float4v*)(red + (((w * MB + mb) * NB + nb) * 64 + lane) * 4);
            const int m = 16 * mb + c16, n = n0 + 16 * nb + 4 * grp;
            if (m >= g.M || n >= g.N) continue;
            if (direct) {
                half4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (_Float16)s[e];
                *(half4*)(g.C + (size_t)m * g.ldc + n) = o;
            } else {
                float* dst = g.partial + ((size_t)split * g.M + m) * g.N + n;
                if (FUSED) {
                    union { float4v f; unsigned long long u[2]; } v;
                    v.f = s;
                    store_agent((unsigned long long*)dst, v.u[0]);
                    store_agent((unsigned long long*)dst + 1, v.u[1]);
                } else {
                    *(float4v*)dst = s;
                }
            }
        }
    }
    if (!FUSED || direct) return;

    // fused reduction over the K slabs of these columns, as in skinny_gemm_kernel
    __syncthreads();
    int* flag = (int*)red;
    if (t == 0) {
        int* ctr = g.counters + blockIdx.x;
        const int arrived = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (arrived == g.splits - 1) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag = arrived;
    }
    __syncthreads();
    if (*flag != g.splits - 1) return;
    sum_split_planes<64 * WAVES, NR / 4>(g, 0, n0, g.M, t);
}

}  // namespace hgemm
