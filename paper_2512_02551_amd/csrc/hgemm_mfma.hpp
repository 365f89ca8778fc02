// Pipelined MFMA HGEMM kernel for gfx950 (CDNA4), NN layout.
//
// Structure follows the three phases the paper describes for a tiled HGEMM
// (Section 2.1): (1) one BM x BN tile of C per workgroup, cut into 32x32
// matrix-core tiles per wavefront; (2) a main loop that stages BM x BK of A
// and BK x BN of B from global memory into LDS, reads fragments from LDS into
// registers and accumulates in registers over all of K; (3) an epilogue that
// rounds and stores.  The techniques of Section 5.3 appear in their CDNA4
// form:
//   * asynchronous 128-bit global->shared copies   -> buffer_load_dwordx4 ... lds
//     (data goes HBM -> LDS without passing through VGPRs);
//   * multi-stage pipelining (n_stage)             -> STAGES LDS buffers, loads
//     issued STAGES-1 K-tiles ahead of use;
//   * shared-memory swizzle against bank conflicts -> XOR of the 16-byte chunk
//     index with a function of the row, applied on the global side (the LDS
//     side of a direct load is always linear in the lane id);
//   * double-buffered register fragments (5.3.1)   -> frag[2], next k-step read
//     from LDS while the current one feeds the matrix cores, also across the
//     K-tile boundary;
//   * register accumulation                        -> fp32 accumulators live in
//     (Acc)VGPRs for the whole K range;
//   * zero padding to non-divisor tiles (5.2)      -> out-of-range rows/columns
//     are read as zeros by the buffer bounds check or a per-lane predicate and
//     are never stored;
//   * block swizzle (5.3, 6.3)                     -> XCD-aware tile order.
//
// Row-major B is the hard operand: the matrix core wants, per lane, 8
// consecutive k for one column n, while memory has n contiguous.  The LDS
// transposing read ds_read_b64_tr_b16 does the turn: within each group of 16
// lanes, lane s supplies the address of 4 consecutive n at row k0 + s/4,
// column 4*(s%4); lane i receives the four k-values of column i.
//
// The roles of the two MFMA operands are swapped (the instruction computes the
// 32x32 tile of C^T): the "A" operand carries B-fragments, the "B" operand
// A-fragments.  A lane then owns 4 consecutive columns of one row of C, which
// is the contiguous direction of row-major C.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace hgemm {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));

#define HGEMM_LDS(p) ((__attribute__((address_space(3))) void*)(p))

// Division of a tile id by a launch constant without a divide instruction sequence: for 0 <= n < 2^24 and
// d >= 1, floor(n / d) = (((n << 8) * m) >> 32) >> l with l = ceil(log2 d) and m = ceil(2^(24 + l) / d) <= 2^25
// (m * d = 2^(24 + l) + r with 0 <= r < d <= 2^l, so n * m / 2^(24 + l) exceeds n / d by less than 1 / d).
struct FastDiv {
    unsigned m, l;
};
inline FastDiv make_fastdiv(unsigned d)
{
    FastDiv f{0, 0};
    if (d == 0) d = 1;
    while ((1ull << f.l) < d) ++f.l;
    f.m = (unsigned)((((unsigned long long)1 << (24 + f.l)) + d - 1) / d);
    return f;
}
__host__ __device__ inline unsigned fast_div(unsigned n, FastDiv f)
{
    return (unsigned)(((unsigned long long)(n << 8) * f.m) >> 32) >> f.l;
}

struct GemmArgs {
    const _Float16* A;
    const _Float16* B;
    _Float16* C;
    float* partial;      // split-K: [S][M][N] fp32; stream-K: partial tiles; else unused
    int* counters;       // fused split-K: one arrival counter per output tile, zero between launches
    int M, N, K;
    int lda, ldb, ldc;   // elements
    int tiles_m, tiles_n;
    int swizzle;         // group height in tiles for the tile order; 0 = row-major
    // divisors of the tile order, fixed per launch (set_tile_map): tiles_n; one band = group * tiles_n
    // tiles; the rows of a full band; the rows of the last, shorter band
    FastDiv by_tiles_n, by_band, by_rows, by_last_rows;
    int k_per_split;     // K range of one split, a multiple of BK (== K rounded up when not split)
    int splits;
    // stream-K: the first dp_tiles tiles (in tile order) get one workgroup each; the K-tile
    // iterations of the remaining tiles are dealt evenly to sk_workers more workgroups
    int dp_tiles;
    int sk_workers;
    int sk_iters_per_worker;
    int sk_total_iters;  // (tiles - dp_tiles) * ceil(K / BK)
};

// Kernel modes: one full-K tile per workgroup; split-K (grid.y = split) with the reduction in a
// second launch; stream-K; split-K with the reduction fused into the kernel (the workgroup that
// arrives last at a tile sums the planes in split order); persistent (one workgroup per compute unit
// walks tiles wg, wg + grid, ... and never lets its copy pipeline drain: while the last K-tiles of a
// tile are multiplied the first K-tiles of the next one are already being copied, and the epilogue's
// stores complete under the next tile's main loop); 16-bit accumulator (one tile per workgroup, the
// running sums rounded to fp16 after every matrix-core instruction, i.e. after every 16 products: Section 1
// of the paper names fp16 accumulators as a valid choice and Section 2.3.2's exact-match test is built
// for them; the matrix cores of this chip only accumulate in fp32, so the rounding is applied to the
// fp32 accumulator registers and buys no register space).
enum { MODE_PLAIN = 0, MODE_SPLITK = 1, MODE_STREAMK = 2, MODE_SPLITK_FUSED = 3, MODE_PERSIST = 4, MODE_ACC16 = 5 };

// Agent-scope relaxed atomic accesses: the compiler emits loads and stores that are coherent across
// the whole device (the eight XCDs have private, mutually non-coherent L2 caches; plain accesses
// would need a write-back / invalidate of a whole L2 to be seen on another XCD).
__device__ inline void store_agent(unsigned long long* p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline unsigned long long load_agent(const unsigned long long* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The summing half of the fused split-K reduction: the workgroup that arrived last at a tile adds the
// tile's S fp32 planes in split order, rounds once and stores fp16.  A lane owns groups of 4 columns
// (QPR groups per tile row).  The loads are device-coherent and each costs a trip to memory, so a lane
// keeps the loads of 4 column groups x 4 splits in flight at once instead of walking its groups one
// after another; positions and splits out of range are loaded from a valid address and not added, so no
// load sits behind a branch.
template <int THREADS, int QPR>
__device__ __forceinline__ void sum_split_planes(const GemmArgs& g, int m0, int n0, int rows, int t)
{
    constexpr int QU = 4, SU = 4;
    const size_t plane2 = (size_t)g.M * g.N / 2;              // plane size in 8-byte words
    const int items = rows * QPR;
    for (int qb = 0; qb < items; qb += QU * THREADS) {
        const unsigned long long* src[QU];
        _Float16* dst[QU];
        bool ok[QU];
        float4v sum[QU];
#pragma unroll
        for (int j = 0; j < QU; ++j) {
            const int q = qb + j * THREADS + t;
            const int m = m0 + q / QPR, n = n0 + (q % QPR) * 4;
            ok[j] = q < items && n < g.N;
            src[j] = (const unsigned long long*)(g.partial + (ok[j] ? (size_t)m * g.N + n : (size_t)m0 * g.N + n0));
            dst[j] = g.C + (size_t)m * g.ldc + n;
            sum[j] = float4v{0.f, 0.f, 0.f, 0.f};
        }
        for (int s0 = 0; s0 < g.splits; s0 += SU) {
            union { float4v f; unsigned long long u[2]; } v[SU][QU];
#pragma unroll
            for (int u = 0; u < SU; ++u) {
                const size_t off = (size_t)min(s0 + u, g.splits - 1) * plane2;
#pragma unroll
                for (int j = 0; j < QU; ++j) {
                    v[u][j].u[0] = load_agent(src[j] + off);
                    v[u][j].u[1] = load_agent(src[j] + off + 1);
                }
            }
#pragma unroll
            for (int u = 0; u < SU; ++u) {
                if (s0 + u < g.splits) {
#pragma unroll
                    for (int j = 0; j < QU; ++j) sum[j] += v[u][j].f;
                }
            }
        }
#pragma unroll
        for (int j = 0; j < QU; ++j) {
            if (!ok[j]) continue;
            half4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (_Float16)sum[j][e];
            *(half4*)dst[j] = o;
        }
    }
}

// ---------------------------------------------------------------------------
// Tile order.  Hardware deals workgroup ids round-robin to the 8 XCDs, each
// with a private L2.  Step 1 renumbers ids so that, inside every run of 256
// consecutive ids (one workgroup per CU), each XCD owns 32 consecutive logical
// ids.  Step 2 walks the tile grid in bands of `group` tile-rows, column by
// column inside a band, so 32 consecutive logical ids form a compact
// group x (32/group) block that shares A rows and B columns in one L2.
// ---------------------------------------------------------------------------
__host__ __device__ inline int64_t tile_of_workgroup(int64_t wg, int64_t tiles_m, int64_t tiles_n, int64_t group)
{
    const int64_t total = tiles_m * tiles_n;
    const int64_t XCDS = 8, WAVE = 256;
    int64_t logical = wg;
    if (group > 0) {
        const int64_t base = (wg / WAVE) * WAVE;
        const int64_t span = (total - base < WAVE) ? (total - base) : WAVE;   // ids in this run
        const int64_t within = wg - base;
        const int64_t xcd = within % XCDS, seq = within / XCDS;
        const int64_t q = span / XCDS, r = span % XCDS;
        const int64_t start = xcd * q + (xcd < r ? xcd : r);                    // first logical id of this XCD
        logical = base + start + seq;
        // band walk
        const int64_t band_sz = group * tiles_n;
        const int64_t band = logical / band_sz;
        const int64_t first_m = band * group;
        const int64_t rows = (tiles_m - first_m < group) ? (tiles_m - first_m) : group;
        const int64_t in_band = logical - band * band_sz;
        const int64_t tm = first_m + in_band % rows;
        const int64_t tn = in_band / rows;
        return tm * tiles_n + tn;
    }
    return logical;
}

// What the kernels use: the same map in 32-bit arithmetic, straight to tile coordinates, with every
// division by a launch constant replaced by a multiplication (a 3 us kernel otherwise spends a tenth of
// its time on integer divisions before its first load).  Valid while tiles_m * tiles_n < 2^24, which
// the host checks; the host can also compare it with the form above.
inline void set_tile_map(GemmArgs& g)
{
    const unsigned group = (unsigned)(g.swizzle < g.tiles_m ? g.swizzle : g.tiles_m);
    g.by_tiles_n = make_fastdiv((unsigned)g.tiles_n);
    g.by_band = make_fastdiv(group * (unsigned)g.tiles_n);
    g.by_rows = make_fastdiv(group);
    g.by_last_rows = make_fastdiv(group ? (unsigned)g.tiles_m % group : 1u);
}
__host__ __device__ inline void tile_coords(unsigned wg, const GemmArgs& g, unsigned& tm, unsigned& tn)
{
    const unsigned utn = (unsigned)g.tiles_n;
    if (g.swizzle <= 0) {
        tm = fast_div(wg, g.by_tiles_n);
        tn = wg - tm * utn;
        return;
    }
    const unsigned total = (unsigned)g.tiles_m * utn;
    const unsigned base = wg & ~255u;
    const unsigned span = (total - base < 256u) ? (total - base) : 256u;
    const unsigned within = wg - base;
    const unsigned xcd = within & 7u, seq = within >> 3;
    const unsigned q = span >> 3, r = span & 7u;
    const unsigned logical = base + xcd * q + (xcd < r ? xcd : r) + seq;
    const unsigned group = (unsigned)(g.swizzle < g.tiles_m ? g.swizzle : g.tiles_m);
    const unsigned band = fast_div(logical, g.by_band);
    const unsigned first_m = band * group;
    const bool last = (unsigned)g.tiles_m - first_m < group;
    const unsigned rows = last ? (unsigned)g.tiles_m - first_m : group;
    const unsigned in_band = logical - band * group * utn;
    tn = fast_div(in_band, last ? g.by_last_rows : g.by_rows);
    tm = first_m + in_band - tn * rows;
}

// PF = register prefetch distance in k-steps (Sections 5.3.1 and 5.3.2: PF = 1 is the
// double-buffered ping-pong, PF = 3 the multi-step prefetch with four fragment sets).
// MI = side of the matrix-core instruction's output block: 32 (v_mfma_f32_32x32x16_f16, a k-step is 16 k) or
// 16 (v_mfma_f32_16x16x32_f16, a k-step is 32 k).  Per flop the 16-wide instruction moves half as many
// accumulator registers and twice as many operand registers, 20 % fewer in sum; the fragments come out of LDS
// with the same reads either way (a 16-row fragment is 16 rows x 64 bytes instead of 32 rows x 32 bytes).
template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int STAGES_, int PF_ = 1, int MI_ = 32>
struct MfmaCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, STAGES = STAGES_;
    static constexpr int PF = PF_, NSLOT = PF_ + 1;
    static constexpr int NWAVES = WAVES_M * WAVES_N;
    static constexpr int THREADS = 64 * NWAVES;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;       // wave tile
    static constexpr int MI = MI_;
    static constexpr int KSTEP = MI == 32 ? 16 : 32;                   // k per matrix-core instruction
    static constexpr int ACC = MI * MI / 64;                           // accumulator registers per output block
    static constexpr int TM = WTM / MI, TN = WTN / MI;                 // MI x MI output blocks per wave
    static constexpr int KS = BK / KSTEP;                              // k-steps per K-tile
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BK * BN * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
    // one wave-wide direct load moves 64 lanes x 16 B = 1 KiB, linear in LDS
    static constexpr int A_LOADS = A_BYTES / 1024 / NWAVES;            // per wave per K-tile
    static constexpr int B_LOADS = B_BYTES / 1024 / NWAVES;
    static constexpr int LOADS = A_LOADS + B_LOADS;
    static constexpr int A_CPR = BK / 8;                               // 16-byte chunks per A row
    static constexpr int A_RPI = 64 / A_CPR;                           // A rows per wave-load
    static constexpr int A_RP = 256 / (BK * 2);                        // A rows per 256 B of LDS
    static constexpr int B_CPR = BN / 8;
    static constexpr int B_RPI = 64 / B_CPR;                           // B rows per wave-load, when a row divides a wave-load
    // Tile widths that are not powers of two (Section 5.2: the tile need not divide the problem, nor be
    // a power of two): a wave-load then covers a fractional number of B rows and every lane keeps one
    // source offset per load instead of one offset plus a stride.
    static constexpr bool B_RAGGED = 64 % B_CPR != 0;
    // persistent mode stages the epilogue in the one buffer the last K-tile has just vacated
    static constexpr bool CAN_PERSIST = NWAVES * MI_ * (WTN * 2 + 8) <= STAGE_BYTES;
    static_assert(BM % (32 * WAVES_M) == 0 && BN % (32 * WAVES_N) == 0, "wave tile must be a multiple of 32");
    static_assert(MI == 32 || MI == 16, "MI");
    static_assert(BK % KSTEP == 0, "a K-tile holds whole k-steps");
    static_assert(BK == 32 || BK == 64 || BK == 128, "BK");
    // Deep staging: a prefetch distance longer than a K-tile.  BK = 32 (two k-steps per K-tile) with PF = 3: the
    // fragment reads run three k-steps, i.e. up to two K-tiles, ahead of the matrix cores, the four fragment
    // sets cycle once per two K-tiles, and five 32 KiB stages keep four K-tiles of copies in flight -- twice the
    // lead of two 64 KiB stages in the same LDS.  One tile per workgroup only (no split-K, stream-K, persistence).
    // With the 16-wide instruction a K-tile of 32 is a single k-step (KS = 1, PF = 1): the same uniform loop with one
    // k-step per K-tile, two fragment sets, and the reads one K-tile ahead.
    static constexpr bool DEEP = PF > KS || KS == 1;
    static_assert(DEEP ? ((KS == 2 && PF == 3 && STAGES >= 4) || (KS == 1 && PF == 1 && STAGES >= 3))
                       : (KS % NSLOT == 0 && PF >= 1), "the k-steps must cycle through the fragment sets a whole number of times");
    static_assert(A_BYTES % (1024 * NWAVES) == 0 && B_BYTES % (1024 * NWAVES) == 0, "tile must split into wave loads");
    static_assert(BN >= 64 && BN <= 512, "BN");
    static_assert((NWAVES * A_RPI) % 16 == 0, "A swizzle must be periodic in the rows one round of loads covers");
    static_assert(B_RAGGED || (NWAVES * B_RPI) % 4 == 0, "B swizzle periodicity");
    static_assert(BN % 32 == 0, "BN");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    static_assert(LOADS * (STAGES - 1) <= 63, "vmcnt is 6 bits");
};

// XOR applied to the 16-byte chunk index of an A row (rows of BK halves).
template <class C> __device__ inline int swz_a(int row) { return (row / C::A_RP) % C::A_CPR; }
// XOR applied to the chunk index of a B row (rows of BN halves): the four rows
// k..k+3 one transposing read touches must land in four different 64-byte
// quarters of the 256-byte bank window.
// With the 16 x 16 x 32 instruction the first 32 lanes of a transposing read hold two groups of 16 lanes that
// read the same columns at rows k and k + 8 (with 32 x 32 x 16 the two groups read different columns): bit 3 of k
// then moves the row by another 32 bytes, and the two groups meet in different banks.  Only where one offset per
// lane still serves all of a lane's copies, i.e. where the rows of a lane's copies differ by multiples of 16
// (or every copy has an offset of its own, B_RAGGED).
template <class C> __device__ inline int swz_b(int k)
{
    constexpr int PITCH = (C::BN * 2) % 256;      // where consecutive rows start inside the 256-byte bank window
    constexpr bool BIT3 = C::MI == 16 && (PITCH == 0 || PITCH == 128) && (C::B_RAGGED || (C::NWAVES * C::B_RPI) % 16 == 0);
    const int hi = BIT3 ? ((k >> 3) & 1) << 1 : 0;
    if (PITCH == 0) return ((k & 3) << 2) ^ hi;          // BN = 128, 256, 512: all four rows would start at the same place
    if (PITCH == 128) return (((k >> 1) & 1) << 2) ^ hi; // BN = 64, 192: rows k and k+1 already differ, k and k+2 do not
    return 0;                                            // BN = 96, 160: the four rows start in four different quarters
}

typedef int int4v __attribute__((ext_vector_type(4)));

// Raw buffer descriptor (gfx9 layout): 48-bit base, stride 0, byte count, data-format word.
// A load whose byte offset is >= `bytes` returns zero instead of touching memory.
__device__ inline int4v make_rsrc(const void* base, unsigned bytes)
{
    const uint64_t a = (uint64_t)base;
    int4v r;
    // the descriptor lives in scalar registers: say so, whatever the optimiser thinks of its inputs
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)((a >> 32) & 0xffffu));
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}

// One wave-wide asynchronous copy HBM -> LDS: lane i moves 16 bytes from base + voff(i) to
// LDS address lds_addr + 16*i (M0 carries the wave-uniform LDS base; it is an operand of the
// statement, so the compiler loads it and knows it is overwritten).  Issued through inline
// assembly on purpose: the completion of these copies is tracked by hand with vmcnt (see
// wait_vmcnt), and the compiler must not serialise every later LDS read behind them.  The s_nop
// is the wait state the hardware wants between a write of M0 and an LDS-direct load.
__device__ inline void dma16(int4v rsrc, unsigned lds_addr, unsigned voff)
{
    asm volatile("s_nop 0\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds"
                 :
                 : "v"(voff), "s"(rsrc), "{m0}"(__builtin_amdgcn_readfirstlane((int)lds_addr))
                 : "memory");
}

__device__ inline unsigned lds_addr_of(const void* p) { return (unsigned)(uintptr_t)HGEMM_LDS(p); }

template <int N> __device__ inline void wait_vmcnt()
{
    static_assert(N >= 0 && N <= 63, "vmcnt range");
    // gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]; leave exp/lgkm at "no wait"
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// TN = B stored column-major, i.e. as an N x K row-major array (Section 2.2.2): then B tiles are
// staged and read exactly like A tiles (K contiguous), with no transposing read.
// ic<V>{} passes a compile-time integer into a lambda; static_for<N>(f) calls f(ic<0>{}), ..., f(ic<N-1>{}).
// The k-step lambdas take their fragment-set numbers this way, so that the fragment arrays are indexed by
// constants in every instantiation, whatever order the optimiser inlines and unrolls in.
template <int V> using ic = std::integral_constant<int, V>;
template <class F, int... I> __device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>)
{
    (f(ic<I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

template <class C, int MODE, bool TN>
__global__ __launch_bounds__(C::THREADS) void mfma_gemm_kernel(GemmArgs g)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    constexpr bool FUSED = MODE == MODE_SPLITK_FUSED;
    constexpr bool SPLITK = MODE == MODE_SPLITK || FUSED;
    constexpr bool STREAMK = MODE == MODE_STREAMK;
    constexpr bool PERSIST = MODE == MODE_PERSIST;
    constexpr bool ACC16 = MODE == MODE_ACC16;
    constexpr bool DEEP = C::DEEP;
    static_assert(!DEEP || MODE == MODE_PLAIN, "deep-staged configurations run one full-K tile per workgroup");
    constexpr int MI = C::MI;
    static_assert(MI == 32 || !ACC16, "the 16-bit accumulator rounds after every 16 products: 32 x 32 x 16 instructions only");
    constexpr int LG = MI == 32 ? 5 : 4;           // lane / MI = the lane's k-chunk within a k-step
    constexpr int CPK = C::KSTEP / 8;               // 16-byte chunks (8 k) per k-step
    static_assert(!PERSIST || C::CAN_PERSIST, "epilogue staging must fit in one stage");

    // All arguments the set-up reads are pulled into scalar registers here, in one batch of loads:
    // left to itself the compiler fetches some of them later, inside branches, and every such fetch is
    // another round trip to memory in front of the first copy (short kernels are latency chains).
    asm volatile("" :: "s"(g.A), "s"(g.B), "s"(g.C), "s"(g.M), "s"(g.N), "s"(g.K), "s"(g.lda), "s"(g.ldb), "s"(g.ldc),
                 "s"(g.tiles_m), "s"(g.tiles_n), "s"(g.swizzle), "s"(g.k_per_split), "s"(g.splits));
    asm volatile("" :: "s"(g.by_tiles_n.m), "s"(g.by_tiles_n.l), "s"(g.by_band.m), "s"(g.by_band.l), "s"(g.by_rows.m),
                 "s"(g.by_rows.l), "s"(g.by_last_rows.m), "s"(g.by_last_rows.l));

    // Every lambda below has to end up inlined: one that stayed a call would reach the variables it captures
    // through memory, and a buffer descriptor loaded from memory is not in the scalar registers the copies need
    // (the assembler then rejects the copy instruction, so this cannot go unnoticed).  The lambdas are kept small
    // enough for the inliner; forcing it with always_inline, or raising its threshold, inlines before the loops are
    // unrolled and leaves the fragment arrays of some configurations in scratch memory.
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
    const int split = SPLITK ? blockIdx.y : 0;

    // Stream-K bookkeeping (Section 5 of the paper has no counterpart; the scheme is: workgroups
    // [0, dp_tiles) compute one whole tile each, workgroup dp_tiles + w takes the K-tile iterations
    // [w*ipw, (w+1)*ipw) of the remaining tiles, laid end to end).  A worker's range is cut into
    // segments at tile boundaries; a segment that covers a whole tile is stored to C directly, the
    // others go to the workspace as fp32 partial tiles (slot 2w for the worker's first segment,
    // 2w+1 for a later one) and are summed in k order by streamk_fixup_kernel.
    const int kt_per_tile = STREAMK ? (g.K + C::BK - 1) / C::BK : 0;
    int sk_iter = 0, sk_end = 0;
    bool sk_worker = false;
    if (STREAMK && (int)blockIdx.x >= g.dp_tiles) {
        sk_worker = true;
        const int w = (int)blockIdx.x - g.dp_tiles;
        sk_iter = w * g.sk_iters_per_worker;
        sk_end = min(sk_iter + g.sk_iters_per_worker, g.sk_total_iters);
        if (sk_iter >= sk_end) return;
    }
    bool first_segment = true;

  for (;;) {       // one pass per segment; a single pass unless MODE_STREAMK
    int tile_id, k_begin, k_end;
    bool to_partial = SPLITK;
    if (STREAMK && sk_worker) {
        const int t = sk_iter / kt_per_tile;
        const int kt0 = sk_iter - t * kt_per_tile;
        const int kt1 = min(kt_per_tile, kt0 + (sk_end - sk_iter));
        tile_id = g.dp_tiles + t;
        k_begin = kt0 * C::BK;
        k_end = min(g.K, kt1 * C::BK);
        to_partial = !(kt0 == 0 && kt1 == kt_per_tile);
        sk_iter += kt1 - kt0;
    } else {
        tile_id = blockIdx.x;
        k_begin = split * g.k_per_split;
        k_end = min(g.K, k_begin + g.k_per_split);
    }
    const int total_tiles = g.tiles_m * g.tiles_n;
    // (m0, n0): the tile being multiplied and stored.  The copies have a tile of their own (set_load_tile),
    // which in persistent mode runs ahead of it.
    int m0, n0;        // the tile being multiplied and stored
    int lm0, ln0;      // the tile the copies read (the same one, except in persistent mode near the end of a tile)
    auto tile_origin = [&](int id, int& tm0, int& tn0) {
        unsigned tm, tn;
        tile_coords((unsigned)id, g, tm, tn);
        tm0 = (int)tm * C::BM;
        tn0 = (int)tn * C::BN;
    };
    tile_origin(tile_id, m0, n0);
    const int KT = (k_end - k_begin + C::BK - 1) / C::BK;

    const unsigned OOB = 0x80000000u;        // beyond every num_records the host admits
    const int4v rsrcA = make_rsrc(g.A, (unsigned)min((long long)g.M * g.lda * 2, 0x7fffffffLL));
    const int4v rsrcB = make_rsrc(g.B, (unsigned)min((long long)(TN ? g.N : k_end) * g.ldb * 2, 0x7fffffffLL));

    // ---- global -> LDS addressing (per lane, fixed for the whole K loop) ----
    // A: wave-load q = j*NWAVES + wave covers rows [q*A_RPI, (q+1)*A_RPI); lane i writes LDS slot i,
    // i.e. row q*A_RPI + i/A_CPR, physical chunk i%A_CPR, which must hold logical chunk p ^ swz.
    const int a_row = wave * C::A_RPI + lane / C::A_CPR;                 // + j * NWAVES*A_RPI
    const int a_chunk = (lane % C::A_CPR) ^ swz_a<C>(a_row);
    const unsigned a_step = (unsigned)(C::NWAVES * C::A_RPI * g.lda * 2);
    const int a_kcol = k_begin + a_chunk * 8;                             // + kt*BK, compared with k_end
    // B, row-major (NN): wave-load q covers k-rows [q*B_RPI, (q+1)*B_RPI) of the BK x BN tile.
    // B, column-major (TN): the tile is BN x BK with K contiguous and is addressed like the A tile.
    const int b_row = TN ? wave * C::A_RPI + lane / C::A_CPR : wave * C::B_RPI + lane / C::B_CPR;
    const int b_chunk = TN ? (lane % C::A_CPR) ^ swz_a<C>(b_row) : (lane % C::B_CPR) ^ swz_b<C>(b_row);
    // ragged B rows (NN, tile width not a power of two): 16-byte unit q*64 + lane of the tile lies in row
    // unit / B_CPR at physical chunk unit % B_CPR, one offset per wave-load
    constexpr bool RAGGED = !TN && C::B_RAGGED;
    unsigned a_voff0, b_voff0;
    bool b_col_ok;
    unsigned b_voffj[RAGGED ? C::B_LOADS : 1];
    auto set_load_tile = [&](int id) {
        if (id < 0) {                      // no tile: every copy out of range
            a_voff0 = b_voff0 = OOB;
            b_col_ok = true;
            if (RAGGED) {
#pragma unroll
                for (int jb = 0; jb < C::B_LOADS; ++jb) b_voffj[jb] = OOB;
            }
            return;
        }
        if (id == tile_id) { lm0 = m0; ln0 = n0; } else tile_origin(id, lm0, ln0);
        a_voff0 = (unsigned)(((lm0 + a_row) * g.lda + k_begin + a_chunk * 8) * 2);
        b_col_ok = TN ? true : (ln0 + b_chunk * 8) < g.N;
        b_voff0 = TN ? (unsigned)(((ln0 + b_row) * g.ldb + k_begin + b_chunk * 8) * 2)
                     : (b_col_ok ? (unsigned)(((k_begin + b_row) * g.ldb + ln0 + b_chunk * 8) * 2) : OOB);
        if (RAGGED) {
#pragma unroll
            for (int jb = 0; jb < C::B_LOADS; ++jb) {
                const int unit = (jb * C::NWAVES + wave) * 64 + lane;
                const int row = unit / C::B_CPR;
                const int chunk = (unit % C::B_CPR) ^ swz_b<C>(row);
                b_voffj[jb] = (ln0 + chunk * 8) < g.N ? (unsigned)(((k_begin + row) * g.ldb + ln0 + chunk * 8) * 2) : OOB;
            }
        }
    };
    set_load_tile(tile_id);
    const unsigned b_step = TN ? (unsigned)(C::NWAVES * C::A_RPI * g.ldb * 2) : (unsigned)(C::NWAVES * C::B_RPI * g.ldb * 2);
    const unsigned b_kstep = TN ? (unsigned)(C::BK * 2) : (unsigned)(C::BK * g.ldb * 2);
    const int b_kcol = k_begin + b_chunk * 8;                             // TN only: + kt*BK, compared with k_end

    // One wave-load of tile kt: index j < A_LOADS is an A load, the rest are B loads.
    auto dma_one = [&](int kt, int buf, int j) {
        char* sA = lds + buf * C::STAGE_BYTES;
        char* sB = sA + C::A_BYTES;
        if (j < C::A_LOADS) {
            const bool a_ok = (a_kcol + kt * C::BK) < k_end;
            dma16(rsrcA, lds_addr_of(sA + (j * C::NWAVES + wave) * 1024),
                  a_ok ? a_voff0 + (unsigned)(kt * C::BK * 2) + j * a_step : OOB);
        } else {
            const int jb = j - C::A_LOADS;
            if (RAGGED) {
                dma16(rsrcB, lds_addr_of(sB + (jb * C::NWAVES + wave) * 1024),
                      b_voffj[jb] != OOB ? b_voffj[jb] + (unsigned)kt * b_kstep : OOB);
            } else {
                const bool b_ok = TN ? (b_kcol + kt * C::BK) < k_end : b_col_ok;
                dma16(rsrcB, lds_addr_of(sB + (jb * C::NWAVES + wave) * 1024),
                      b_ok ? b_voff0 + (unsigned)kt * b_kstep + jb * b_step : OOB);
            }
        }
    };
    auto load_tile = [&](int kt, int buf) {
#pragma unroll
        for (int j = 0; j < C::LOADS; ++j) dma_one(kt, buf, j);
    };

    // ---- LDS -> register addressing ----------------------------------------
    // A fragment (fed as the MFMA "B" operand): lane holds A[m = l%32][8 consecutive k of half l/32]
    const int fa_row = wm * C::WTM + (lane & (MI - 1));                   // + tm*MI
    const int fa_swz = swz_a<C>(fa_row);
    const int fa_base = fa_row * (C::BK * 2);
    // B fragment (fed as the MFMA "A" operand) through two transposing reads per 8 k-values
    const int fb_krow = 8 * (lane >> LG) + ((lane & 15) >> 2);            // + KSTEP*ks + 4*h
    const int fb_swz = swz_b<C>(fb_krow);                                 // adding KSTEP*ks + 4*h changes none of k&3, bit 1 and bit 3 of k
    const int fb_ncol = wn * C::WTN + (MI == 32 ? 16 * ((lane >> 4) & 1) : 0) + 4 * (lane & 3);   // + tn*MI
    // TN: B fragment read like an A fragment from the BN x BK tile
    const int ft_row = wn * C::WTN + (lane & (MI - 1));                   // + tn*MI
    const int ft_swz = swz_a<C>(ft_row);
    const int ft_base = ft_row * (C::BK * 2);

    half8 fa[C::NSLOT][C::TM];
    half8 fb[C::NSLOT][C::TN];
    typedef typename std::conditional<MI == 32, float16v, float4v>::type acc_t;
    acc_t acc[C::TM][C::TN];          // zeroed at the start of every tile

    // Fragment read number r of a k-step: r < TM reads A fragment r, the rest read B fragment r-TM.
    constexpr int NREADS = C::TM + C::TN;
    constexpr int NMMA = C::TM * C::TN;
    auto read_one = [&](int buf, int ks, int slot, int r) {
        const char* sA = lds + buf * C::STAGE_BYTES;
        const char* sB = sA + C::A_BYTES;
        if (r < C::TM) {
            const int chunk = (CPK * ks + (lane >> LG)) ^ fa_swz;
            fa[slot][r] = *(const half8*)(sA + fa_base + r * MI * (C::BK * 2) + chunk * 16);
        } else if (TN) {
            const int tn = r - C::TM;
            const int chunk = (CPK * ks + (lane >> LG)) ^ ft_swz;
            fb[slot][tn] = *(const half8*)(sB + ft_base + tn * MI * (C::BK * 2) + chunk * 16);
        } else {
            const int tn = r - C::TM;
            const int n = fb_ncol + tn * MI;
            const int off = ((n >> 3) ^ fb_swz) * 16 + (n & 7) * 2;
            short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) short4v*)HGEMM_LDS(sB + (C::KSTEP * ks + fb_krow) * (C::BN * 2) + off));
            short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) short4v*)HGEMM_LDS(sB + (C::KSTEP * ks + 4 + fb_krow) * (C::BN * 2) + off));
            union { struct { short4v lo, hi; } s; half8 h; } u;
            u.s.lo = lo;
            u.s.hi = hi;
            fb[slot][tn] = u.h;
        }
    };
    auto read_frags = [&](int buf, int ks, int slot) {
#pragma unroll
        for (int r = 0; r < NREADS; ++r) read_one(buf, ks, slot, r);
    };
    // Order of the output blocks within a k-step.  With prefetch distance 1 the fragments of this k-step were read
    // during the previous one, A fragments first and B fragments last: walking the blocks column by column uses the
    // B fragment that arrived last, last (its read is then most of a k-step old), instead of after a handful of
    // instructions -- which is what one wave per SIMD needs, having no second wave to cover a late fragment.  With
    // longer prefetch distances every fragment is old enough and the order is row by row.
    auto mma_one = [&](int slot, int i) {
        const int tm = C::PF == 1 ? i % C::TM : i / C::TN, tn = C::PF == 1 ? i / C::TM : i % C::TN;
        if constexpr (MI == 32) acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[slot][tn], fa[slot][tm], acc[tm][tn], 0, 0, 0);
        else acc[tm][tn] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fb[slot][tn], fa[slot][tm], acc[tm][tn], 0, 0, 0);
    };
    // 16-bit accumulator: the running sums are fp16 values between matrix-core instructions (round to nearest
    // even, overflow to infinity).  Every accumulator block takes exactly one instruction per k-step, so the
    // rounding is applied to all of them at the end of the k-step.
    auto round_accumulators = [&]() {
#pragma unroll
        for (int tm = 0; tm < C::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < C::TN; ++tn)
#pragma unroll
                for (int e = 0; e < C::ACC; ++e) acc[tm][tn][e] = (float)(_Float16)acc[tm][tn][e];
    };

    using std::integral_constant;
    // One k-step with a pinned instruction order: matrix-core instruction i is followed by its
    // share of the side work (fragment reads for the k-step PF steps ahead, and after the barrier
    // of a tile the global->LDS copies of a later tile), so that the side work issues in the shadow
    // of the matrix cores instead of in a burst in front of them (the staggered prefetch of
    // Section 5.3.4, taken to instruction granularity).
    // Copies [dma_lo, dma_hi) of tile dma_kt go to buffer dma_buf.
    // Everything that selects a register or an instruction slot is a compile-time value (tags), so the fragment and
    // accumulator arrays are indexed by constants in every instantiation, whatever the optimiser inlines or unrolls.
    // (A k-step of more than 32 matrix-core instructions is issued in two halves: one lambda with all of them is too
    // large for the inliner, and a lambda that stays a call reaches the buffer descriptors through memory.)
    auto kstep_part = [&](auto i0_tag, auto i1_tag, auto slot_tag, int rbuf, int rks, auto rslot_tag, auto do_reads_tag, int dma_kt, int dma_buf,
                          auto dma_lo_tag, auto dma_hi_tag) {
        constexpr int i0 = decltype(i0_tag)::value, i1 = decltype(i1_tag)::value;
        constexpr int slot = decltype(slot_tag)::value, rslot = decltype(rslot_tag)::value;
        constexpr int dma_lo = decltype(dma_lo_tag)::value, dma_hi = decltype(dma_hi_tag)::value;
        constexpr int nreads = decltype(do_reads_tag)::value ? NREADS : 0;
        constexpr int nside = nreads + (dma_hi - dma_lo);
        static_for<i1 - i0>([&](auto ii) {
            constexpr int i = i0 + decltype(ii)::value;
            mma_one(slot, i);
            // side ops [lo, hi) go after MFMA i: spread nside ops evenly over the NMMA slots
            constexpr int lo = (i * nside) / NMMA, hi = ((i + 1) * nside) / NMMA;
            static_for<hi - lo>([&](auto tt) {
                constexpr int t = lo + decltype(tt)::value;
                // fragment reads first (they are needed soonest), then the copies
                if constexpr (t < nreads) read_one(rbuf, rks, rslot, t);
                else dma_one(dma_kt, dma_buf, dma_lo + t - nreads);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    auto kstep = [&](auto slot, int rbuf, int rks, auto rslot, auto do_reads, int dma_kt, int dma_buf, auto dma_lo, auto dma_hi) {
        if constexpr (NMMA > 32) {
            kstep_part(ic<0>{}, ic<NMMA / 2>{}, slot, rbuf, rks, rslot, do_reads, dma_kt, dma_buf, dma_lo, dma_hi);
            kstep_part(ic<NMMA / 2>{}, ic<NMMA>{}, slot, rbuf, rks, rslot, do_reads, dma_kt, dma_buf, dma_lo, dma_hi);
        } else {
            kstep_part(ic<0>{}, ic<NMMA>{}, slot, rbuf, rks, rslot, do_reads, dma_kt, dma_buf, dma_lo, dma_hi);
        }
    };

    // One K-tile.  Tile kt lives in LDS buffer kt % STAGES.  The k-step that runs at position ks
    // reads the fragments of position ks + PF; the barrier sits in front of the first k-step whose
    // reads fall into the next tile (ks == KS - PF): by then every wave holds all its fragments of
    // tile kt in registers, so after the barrier buffer kt % STAGES is free for tile kt+STAGES, and
    // tile kt+1 (copies issued STAGES-1 tiles earlier) is complete and visible to all waves.
    // WAIT = number of copies that may still be in flight at the barrier; HAS_NEXT = a next tile
    // exists; DMA = K-tile dma_kt (of the copies' tile) is copied into the vacated buffer after the barrier.
    auto tile_body = [&](int dma_kt, int buf, int nbuf, auto wait_tag, auto has_next_tag, auto dma_tag) {
        constexpr int WAIT = decltype(wait_tag)::value;
        constexpr bool HAS_NEXT = decltype(has_next_tag)::value;
        constexpr bool DMA = decltype(dma_tag)::value;
        static_for<C::KS>([&](auto ks_tag) {
            constexpr int ks = decltype(ks_tag)::value;
            constexpr bool after = ks >= C::KS - C::PF;        // this step runs behind the barrier
            if (ks == C::KS - C::PF && HAS_NEXT) {
                wait_vmcnt<WAIT>();
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            }
            constexpr int t = ks + C::PF;
            constexpr bool in_next = t >= C::KS;
            constexpr int j = ks - (C::KS - C::PF);             // index among the post-barrier steps
            constexpr int dlo = (DMA && after) ? (j * C::LOADS) / C::PF : 0;
            constexpr int dhi = (DMA && after) ? ((j + 1) * C::LOADS) / C::PF : 0;
            kstep(ic<ks % C::NSLOT>{}, in_next ? nbuf : buf, in_next ? t - C::KS : t, ic<t % C::NSLOT>{},
                  std::bool_constant<(in_next ? HAS_NEXT : true)>{}, dma_kt, buf, ic<dlo>{}, ic<dhi>{});
            if (ACC16) {
                round_accumulators();
                __builtin_amdgcn_sched_barrier(0);
            }
        });
    };

    // ---- main loop ----------------------------------------------------------
    int buf = 0;                      // LDS buffer of the K-tile being multiplied
    bool has_next = false;            // persistent mode: this workgroup has another tile after this one
    if (!DEEP && KT > 0) {
#pragma unroll
        for (int s = 0; s < C::STAGES; ++s)
            if (s < KT) load_tile(s, s);
        // tile 0 must have landed: at most the later prologue tiles may still be in flight
        if (KT >= C::STAGES) wait_vmcnt<(C::STAGES - 1) * C::LOADS>(); else wait_vmcnt<0>();
        asm volatile("s_barrier" ::: "memory");
#pragma unroll
        for (int ks = 0; ks < (DEEP ? 0 : C::PF); ++ks) read_frags(0, ks, ks);
        __builtin_amdgcn_sched_barrier(0);
    }
  for (;;) {       // one pass per tile of this workgroup; a single pass unless MODE_PERSIST
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
#pragma unroll
            for (int v = 0; v < C::ACC; ++v) acc[i][j][v] = 0.f;
    if constexpr (DEEP) {
        // Deep-staged main loop.  The reads lead the matrix cores by three k-steps; "the read tile" is the K-tile
        // the reads are in.  When the reads move on to the next K-tile: that tile must have landed (all copies but
        // those of the STAGES - 2 younger tiles), every wave must be done reading the tile they leave (its buffer
        // is refilled next), one barrier covers both.  Every pass issues the same number of copies -- K-tiles
        // past the end are copied out of range, which moves zeros -- so the waits are compile-time constants, and
        // an odd number of K-tiles is rounded up with a tile of zeros so that the fragment sets cycle evenly.
        constexpr int S = C::STAGES, L = C::LOADS;
        static_assert((S - 1) * L <= 63, "vmcnt range");
        int rt = 0, rb = 0;                  // read tile and its buffer
        int dkt = 0, dbuf = 0;               // the refill in progress: K-tile dkt into buffer dbuf
        auto enter_next_tile = [&]() {
            wait_vmcnt<(S - 2) * L>();
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            dkt = rt + S;
            dbuf = rb;
            rt += 1;
            rb = (rb + 1 == S) ? 0 : rb + 1;
        };
#pragma unroll
        for (int s0 = 0; s0 < S; ++s0) load_tile(s0, s0);
        wait_vmcnt<(S - 1) * L>();
        asm volatile("s_barrier" ::: "memory");
        read_frags(0, 0, 0);
      if constexpr (C::KS == 1) {
        // One k-step per K-tile: a pass multiplies the fragments of K-tile t (set t % 2), reads those of K-tile t + 1
        // into the other set and refills the buffer K-tile t has left with K-tile t + STAGES.
        __builtin_amdgcn_sched_barrier(0);
        const int KT2 = (KT + 1) & ~1;
        for (int t2 = 0; t2 < KT2; t2 += 2) {
            enter_next_tile();
            kstep(ic<0>{}, rb, 0, ic<1>{}, std::true_type{}, dkt, dbuf, ic<0>{}, ic<L>{});
            enter_next_tile();
            kstep(ic<1>{}, rb, 0, ic<0>{}, std::true_type{}, dkt, dbuf, ic<0>{}, ic<L>{});
        }
        wait_vmcnt<0>();                     // copies still in flight would land in the epilogue's staging area
      } else {
        read_frags(0, 1, 1);
        enter_next_tile();
#pragma unroll
        for (int j = 0; j < L / 2; ++j) dma_one(dkt, dbuf, j);     // K-tile S into the buffer K-tile 0 has left, first half
        read_frags(rb, 0, 2);
        __builtin_amdgcn_sched_barrier(0);
        const int KT2 = (KT + 1) & ~1;
        // One pass = two K-tiles = four k-steps; k-step u multiplies fragment set u and reads the k-step three
        // ahead into set (u + 3) % 4.  A refill is issued in two halves: behind the barrier, and in the k-step after.
        for (int t2 = 0; t2 < KT2; t2 += 2) {
            kstep(ic<0>{}, rb, 1, ic<3>{}, std::true_type{}, dkt, dbuf, ic<L / 2>{}, ic<L>{});
            enter_next_tile();
            kstep(ic<1>{}, rb, 0, ic<0>{}, std::true_type{}, dkt, dbuf, ic<0>{}, ic<L / 2>{});
            kstep(ic<2>{}, rb, 1, ic<1>{}, std::true_type{}, dkt, dbuf, ic<L / 2>{}, ic<L>{});
            enter_next_tile();
            kstep(ic<3>{}, rb, 0, ic<2>{}, std::true_type{}, dkt, dbuf, ic<0>{}, ic<L / 2>{});
        }
        wait_vmcnt<0>();                     // copies still in flight would land in the epilogue's staging area
      }
    } else if (KT > 0) {
        constexpr int STEADY = (C::STAGES - 2) * C::LOADS;
        int kt = 0;
        if (PERSIST) {
            // One loop over all K-tiles but the last, every pass with copies behind its barrier.  While
            // this tile still has K-tiles to copy the copies are its own; from K-tile KT - STAGES on they
            // belong to this workgroup's next tile (the pipeline does not drain).  On the workgroup's
            // final tile those passes issue copies that are all out of range: they move nothing, and the
            // loop keeps one shape and one count of copies in flight.  (The host admits persistent plans
            // only when KT >= STAGES.)
            has_next = tile_id + (int)gridDim.x < total_tiles;
            for (; kt + 1 < KT; ++kt) {
                const int nbuf = (buf + 1 == C::STAGES) ? 0 : buf + 1;
                if (kt + C::STAGES == KT) set_load_tile(has_next ? tile_id + (int)gridDim.x : -1);
                tile_body(kt + C::STAGES < KT ? kt + C::STAGES : kt + C::STAGES - KT, buf, nbuf, integral_constant<int, STEADY>{},
                          integral_constant<bool, true>{}, integral_constant<bool, true>{});
                buf = nbuf;
            }
        } else {
            // steady state: a later tile exists to be copied and a next tile exists to be read
            for (; kt + C::STAGES < KT; ++kt) {
                const int nbuf = (buf + 1 == C::STAGES) ? 0 : buf + 1;
                tile_body(kt + C::STAGES, buf, nbuf, integral_constant<int, STEADY>{}, integral_constant<bool, true>{},
                          integral_constant<bool, true>{});
                buf = nbuf;
            }
            // drain: no more copies to issue
            for (; kt + 1 < KT; ++kt) {
                const int nbuf = (buf + 1 == C::STAGES) ? 0 : buf + 1;
                tile_body(0, buf, nbuf, integral_constant<int, 0>{}, integral_constant<bool, true>{}, integral_constant<bool, false>{});
                buf = nbuf;
            }
        }
        // last K-tile: nothing more to copy or to read ahead (persistent mode: the epilogue stages in its buffer)
        tile_body(0, buf, buf, integral_constant<int, 0>{}, integral_constant<bool, false>{}, integral_constant<bool, false>{});
    }

    // ---- epilogue ------------------------------------------------------------
    // acc[tm][tn][v]: row m = m0 + wm*WTM + tm*MI + l%MI, columns n = n0 + wn*WTN + tn*MI + 8*(v/4) + 4*(l/MI) + v%4
    // (MI = 16: v < 4, one group of 4 consecutive columns per block)
    const int row_t = wm * C::WTM + (lane & (MI - 1));     // tile-local
    const int col_t = wn * C::WTN + 4 * (lane >> LG);
    constexpr int VG = C::ACC / 4;                         // groups of 4 consecutive columns a lane holds per output block
    if (!to_partial) {
        // fp32 -> fp16 (round to nearest even), then through LDS so that a lane stores 16 contiguous
        // bytes and a wave whole row segments (Section 5.3.3: registers -> shared -> global with wide
        // copies).  Each wave turns its own 32 x WTN slab in a private LDS region, one slab per tm.
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // all waves are done with the operand buffers
        constexpr int ROWB = C::WTN * 2 + 8;      // +8 bytes: the 32 rows a half-wave writes hit 32 different banks pairs
        constexpr int CPR = C::WTN / 8;           // 16-byte chunks per slab row
        // persistent mode: only the buffer of the last K-tile is free (the others hold the next tile's first K-tiles)
        char* stage = lds + (PERSIST ? buf * C::STAGE_BYTES : 0) + wave * (MI * ROWB);
        static_assert(C::NWAVES * MI * ROWB <= C::LDS_BYTES, "epilogue staging must fit in the operand buffers");
        static_assert(MI * CPR >= 64, "a slab holds at least one 16-byte chunk per lane");
#pragma unroll
        for (int tm = 0; tm < C::TM; ++tm) {
#pragma unroll
            for (int tn = 0; tn < C::TN; ++tn) {
#pragma unroll
                for (int vg = 0; vg < VG; ++vg) {
                    half4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (_Float16)acc[tm][tn][vg * 4 + e];
                    *(half4*)(stage + (lane & (MI - 1)) * ROWB + (tn * MI + vg * 8 + 4 * (lane >> LG)) * 2) = o;
                }
            }
#pragma unroll
            for (int j = 0; j < (MI * CPR) / 64; ++j) {
                const int idx = j * 64 + lane;
                const int r = idx / CPR, ch = idx % CPR;
                const half4 lo = *(const half4*)(stage + r * ROWB + ch * 16);
                const half4 hi = *(const half4*)(stage + r * ROWB + ch * 16 + 8);
                const int m = m0 + wm * C::WTM + tm * MI + r;
                const int n = n0 + wn * C::WTN + ch * 8;
                if (m < g.M && n < g.N) {
                    half8 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) { v[e] = lo[e]; v[4 + e] = hi[e]; }
                    *(half8*)(g.C + (size_t)m * g.ldc + n) = v;
                }
            }
        }
    } else {
        // fp32 partial sums (split-K plane or stream-K partial tile): 16-byte stores straight from registers
        float* sk_slot = nullptr;
        if (STREAMK)
            sk_slot = g.partial + ((size_t)2 * ((int)blockIdx.x - g.dp_tiles) + (first_segment ? 0 : 1)) * (size_t)(C::BM * C::BN);
#pragma unroll
        for (int tm = 0; tm < C::TM; ++tm) {
            const int m = m0 + row_t + tm * MI;
#pragma unroll
            for (int tn = 0; tn < C::TN; ++tn) {
#pragma unroll
                for (int vg = 0; vg < VG; ++vg) {
                    const int n = n0 + col_t + tn * MI + vg * 8;
                    float4v o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = acc[tm][tn][vg * 4 + e];
                    if (STREAMK) {
                        *(float4v*)(sk_slot + (row_t + tm * MI) * C::BN + col_t + tn * MI + vg * 8) = o;
                    } else if (m < g.M && n < g.N) {
                        float* dst = g.partial + ((size_t)split * g.M + m) * g.N + n;
                        if (FUSED) {
                            // device-coherent stores: the summing workgroup may sit on another XCD
                            union { float4v f; unsigned long long u[2]; } w;
                            w.f = o;
                            store_agent((unsigned long long*)dst, w.u[0]);
                            store_agent((unsigned long long*)dst + 1, w.u[1]);
                        } else {
                            *(float4v*)dst = o;
                        }
                    }
                }
            }
        }
        if (FUSED) {
            // Fused reduction.  Every workgroup of a tile stores its fp32 plane with device-coherent
            // stores, waits until they are performed (the release half of the barrier waits for all of
            // the wave's outstanding stores), then counts itself in.  The workgroup that finds all
            // others already counted -- whichever split it is -- re-reads the S planes in split order,
            // so the sum does not depend on arrival order, rounds once and stores the tile of C.
            // Nobody waits for anybody: a workgroup that is not last simply exits.
            __syncthreads();
            int* flag = (int*)lds;
            if (threadIdx.x == 0) {
                int* ctr = g.counters + tile_id;
                const int arrived = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (arrived == g.splits - 1) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // clean for the next launch
                *flag = arrived;
            }
            __syncthreads();
            if (*flag != g.splits - 1) return;
            sum_split_planes<C::THREADS, C::BN / 4>(g, m0, n0, min(C::BM, g.M - m0), (int)threadIdx.x);
        }
    }
    if (PERSIST && !has_next) wait_vmcnt<0>();        // the final tile's out-of-range copies
    if (!(PERSIST && has_next)) break;
    // ---- persistent mode: on to this workgroup's next tile -----------------------------------
    // The copies of its K-tiles 0 .. STAGES-2 are in flight or landed.  K-tile STAGES-1 goes into the
    // buffer the epilogue has just staged in, once every wave has read its staging area back; then
    // K-tile 0 must have landed (the epilogue's stores count in vmcnt too, which only makes the wait
    // longer) and the first fragments are read, as in the prologue.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    load_tile(C::STAGES - 1, buf);
    buf = (buf + 1 == C::STAGES) ? 0 : buf + 1;
    wait_vmcnt<(C::STAGES - 1) * C::LOADS>();
    asm volatile("s_barrier" ::: "memory");
#pragma unroll
    for (int ks = 0; ks < C::PF; ++ks) read_frags(buf, ks, ks);
    __builtin_amdgcn_sched_barrier(0);
    tile_id += (int)gridDim.x;
    m0 = lm0;          // the copies already belong to this tile
    n0 = ln0;
  }
    if (!(STREAMK && sk_worker) || sk_iter >= sk_end) break;
    first_segment = false;
    // the next segment's copies reuse the LDS buffers: every wave must be done reading them
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  }
}

// Stream-K second pass: grid.x = tiles that stream-K workers shared, grid.y = slices of a tile.  Sums the fp32
// partial tiles of the workers that touched the tile, in increasing k (= increasing worker)
// order, rounds once to fp16 and stores the in-range part of the tile.
template <int BM, int BN, int BK>
__global__ __launch_bounds__(256) void streamk_fixup_kernel(GemmArgs g)
{
    const int kt_per_tile = (g.K + BK - 1) / BK;
    const int t = blockIdx.x;                                   // index among the stream-K tiles
    const int it0 = t * kt_per_tile, it1 = it0 + kt_per_tile;   // this tile's iteration range
    const int ipw = g.sk_iters_per_worker;
    const int w_first = it0 / ipw, w_last = (it1 - 1) / ipw;
    if (w_first == w_last) {
        // a single worker saw the whole tile: it stored C itself unless it saw only part of it
        const int wb = w_first * ipw, we = min(wb + ipw, g.sk_total_iters);
        if (wb <= it0 && we >= it1) return;
    }
    unsigned tm, tn;
    tile_coords((unsigned)(g.dp_tiles + t), g, tm, tn);
    const int m0 = (int)tm * BM;
    const int n0 = (int)tn * BN;
    // blockIdx.y picks a slice of 1024 groups of 4 consecutive columns
    for (int q = blockIdx.y * 1024 + threadIdx.x; q < min((int)(blockIdx.y + 1) * 1024, BM * BN / 4); q += 256) {
        const int r = q / (BN / 4), c = (q % (BN / 4)) * 4;
        if (m0 + r >= g.M || n0 + c >= g.N) continue;
        float4v sum = {0.f, 0.f, 0.f, 0.f};
        for (int w = w_first; w <= w_last; ++w) {
            const int wb = w * ipw;
            const int s0 = max(wb, it0);
            const int slot = 2 * w + (s0 == wb ? 0 : 1);
            sum += *(const float4v*)(g.partial + (size_t)slot * (BM * BN) + r * BN + c);
        }
        half4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (_Float16)sum[e];
        *(half4*)(g.C + (size_t)(m0 + r) * g.ldc + n0 + c) = o;
    }
}

}  // namespace hgemm
