// Host side of the C ABI declared in include/hgemm.h: plan construction (spec
// parsing, dispatch table lookup, plan-time cost model), launch, and helpers.
#include "../../include/hgemm.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "hgemm_aux.hpp"
#include "hgemm_mfma.hpp"
#include "hgemm_registry.hpp"
#include "hgemm_skinny.hpp"

namespace hgemm {

// ---------------------------------------------------------------------------
// Kernel registry: every compiled MFMA specialisation (hgemm_configs.inc), gathered from the
// translation units that instantiate them.
// ---------------------------------------------------------------------------
static const std::vector<MfmaEntry>& registry()
{
    static const std::vector<MfmaEntry> r = [] {
        std::vector<MfmaEntry> v;
        register_chunk_0(v); register_chunk_1(v); register_chunk_2(v); register_chunk_3(v);
        register_chunk_4(v); register_chunk_5(v); register_chunk_6(v); register_chunk_7(v);
        return v;
    }();
    return r;
}

void (*skinny_kernel(int mb, bool fused, int waves, int tn_rows))(GemmArgs);      // hgemm_skinny.hip

constexpr int64_t kSkinnyMaxM = 64;

enum Family { FAM_GENERIC = 0, FAM_MFMA = 1, FAM_SKINNY = 2 };

struct Spec {
    Family fam = FAM_GENERIC;
    int bm = 0, bn = 0, bk = 0, wm = 0, wn = 0, st = 0;
    int pf = 1;     // register prefetch distance in k-steps
    int sk = 1;     // split-K factor
    int gm = 8;     // tile-order group height; 0 = row-major
    int tb = 0;     // 1 = transpose row-major B into the workspace first, then run the K-contiguous (TN) kernel
    int sm = 0;     // 1 = stream-K: whole waves of tiles data-parallel, the rest shared by K-tile iterations
    int fr = 0;     // 1 = split-K with the reduction fused into the kernel (last-arriving workgroup sums in split order)
    int ps = 0;     // 1 = persistent: one workgroup per compute unit walks the tiles without draining its copy pipeline
    int ac = 32;    // accumulator width: 32 = fp32 over all of K; 16 = rounded to fp16 after every 16 products
    int mi = 32;    // matrix-core output block: 32 = v_mfma_f32_32x32x16_f16, 16 = v_mfma_f32_16x16x32_f16
    int wv = 4;     // skinny family: waves per workgroup (4, 8 or 16), each taking 16 k-rows of a step
    int nr = 16;    // skinny family, column-major B: rows of B (columns of C) per workgroup (16, 32 or 64)
};

// k-rows a workgroup of the skinny family takes per step (K slabs are whole numbers of steps) and the columns of C
// it owns: row-major B 16 rows per wave and 128 columns, column-major B 32 k per wave and 16 columns
static int64_t skinny_step(const Spec& s, bool tn = false) { return (tn ? 32 : 16) * s.wv; }
static int64_t skinny_cols(const Spec& s, bool tn) { return tn ? s.nr : kSkinnyCols; }

static std::string spec_to_string(const Spec& s)
{
    char buf[160];
    if (s.fam == FAM_GENERIC) return "generic";
    if (s.fam == FAM_SKINNY) {
        snprintf(buf, sizeof buf, "skinny,sk=%d%s", s.sk, s.fr ? ",fr=1" : "");
        if (s.wv != 4) snprintf(buf + strlen(buf), sizeof buf - strlen(buf), ",wv=%d", s.wv);
        if (s.nr != 16) snprintf(buf + strlen(buf), sizeof buf - strlen(buf), ",nr=%d", s.nr);
        return buf;
    }
    snprintf(buf, sizeof buf, "mfma,bm=%d,bn=%d,bk=%d,wm=%d,wn=%d,st=%d,pf=%d,sk=%d,gm=%d%s", s.bm, s.bn, s.bk, s.wm, s.wn,
             s.st, s.pf, s.sk, s.gm, s.tb ? ",tb=1" : "");
    if (s.sm) strncat(buf, ",sm=1", sizeof buf - strlen(buf) - 1);
    if (s.fr) strncat(buf, ",fr=1", sizeof buf - strlen(buf) - 1);
    if (s.ps) strncat(buf, ",ps=1", sizeof buf - strlen(buf) - 1);
    if (s.ac == 16) strncat(buf, ",ac=16", sizeof buf - strlen(buf) - 1);
    if (s.mi == 16) strncat(buf, ",mi=16", sizeof buf - strlen(buf) - 1);
    return buf;
}

static bool parse_spec(const char* text, Spec* out)
{
    if (!text) return false;
    std::string s(text);
    size_t pos = s.find(',');
    std::string fam = s.substr(0, pos);
    Spec sp;
    if (fam == "generic") {
        sp.fam = FAM_GENERIC;
    } else if (fam == "mfma") {
        sp.fam = FAM_MFMA;
    } else if (fam == "skinny") {
        sp.fam = FAM_SKINNY;
    } else {
        return false;
    }
    while (pos != std::string::npos) {
        size_t next = s.find(',', pos + 1);
        std::string kv = s.substr(pos + 1, next == std::string::npos ? std::string::npos : next - pos - 1);
        pos = next;
        size_t eq = kv.find('=');
        if (eq == std::string::npos || eq == 0 || eq + 1 >= kv.size()) return false;
        std::string key = kv.substr(0, eq);
        char* end = nullptr;
        long v = strtol(kv.c_str() + eq + 1, &end, 10);
        if (*end != '\0' || v < 0 || v > (1 << 20)) return false;
        if (key == "bm") sp.bm = (int)v;
        else if (key == "bn") sp.bn = (int)v;
        else if (key == "bk") sp.bk = (int)v;
        else if (key == "wm") sp.wm = (int)v;
        else if (key == "wn") sp.wn = (int)v;
        else if (key == "st") sp.st = (int)v;
        else if (key == "pf") sp.pf = (int)v;
        else if (key == "sk") sp.sk = (int)v;
        else if (key == "gm") sp.gm = (int)v;
        else if (key == "tb") sp.tb = (int)v;
        else if (key == "sm") sp.sm = (int)v;
        else if (key == "fr") sp.fr = (int)v;
        else if (key == "ps") sp.ps = (int)v;
        else if (key == "ac") sp.ac = (int)v;
        else if (key == "mi") sp.mi = (int)v;
        else if (key == "wv") sp.wv = (int)v;
        else if (key == "nr") sp.nr = (int)v;
        else if (key == "pad") { /* reported by hgemm_plan_describe; padding follows from the shape, not from the spec */ }
        else return false;
    }
    if (sp.sk < 1 || sp.tb > 1 || sp.sm > 1 || sp.fr > 1 || sp.ps > 1 || (sp.sm && sp.sk > 1) || (sp.ps && (sp.sk > 1 || sp.sm)))
        return false;
    // the 16-bit accumulator is a running sum over all of K in k order: one tile per workgroup, no splitting of K
    if ((sp.ac != 32 && sp.ac != 16) || (sp.ac == 16 && (sp.fam != FAM_MFMA || sp.sk > 1 || sp.sm || sp.ps || sp.fr))) return false;
    if (sp.mi != 32 && sp.mi != 16) return false;
    if ((sp.wv != 4 && sp.wv != 8 && sp.wv != 16) || (sp.wv != 4 && sp.fam != FAM_SKINNY)) return false;
    if ((sp.nr != 16 && sp.nr != 32 && sp.nr != 64) || (sp.nr != 16 && sp.fam != FAM_SKINNY)) return false;
    *out = sp;
    return true;
}

static const MfmaEntry* find_entry(const Spec& s)
{
    for (const MfmaEntry& e : registry())
        if (e.bm == s.bm && e.bn == s.bn && e.bk == s.bk && e.wm == s.wm && e.wn == s.wn && e.st == s.st && e.pf == s.pf && e.mi == s.mi) return &e;
    return nullptr;
}

}  // namespace hgemm

using namespace hgemm;

struct hgemm_plan_s {
    int64_t M, N, K;
    hgemm_layouts_t lay;        // with packed leading dimensions resolved
    Spec spec;
    const MfmaEntry* entry;     // null for the generic and skinny families
    void (*skinny)(GemmArgs);   // the skinny family's kernel, else null
    GemmArgs args;              // pointers filled in at run time
    void* workspace;            // [transposed B (when spec.tb)] [split-K / stream-K partial sums]
    size_t workspace_bytes;
    size_t partial_offset;      // byte offset of the partial sums inside the workspace
    bool tn_kernel;             // the MFMA kernel reads B with K contiguous
    int device;
    // Zero padding (Section 5.2) for problems whose N, K or leading dimensions are not multiples of 8:
    // M, N, K, lay above then describe packed, zero-filled copies in the workspace whose N and K are
    // rounded up to 8, and the fields below keep the caller's problem.
    bool padded;
    int64_t uM, uN, uK;
    hgemm_layouts_t ulay;
    size_t a_off, b_off, c_off; // byte offsets of the padded copies of A, B and C inside the workspace
    size_t bt_off;              // byte offset of the transposed copy of B (spec.tb)
    bool static_ws;             // the workspace is this device's static scratch array, not an allocation
    // Operands beyond the reach of the kernels' 32-bit buffer offsets (2 GiB per operand): the problem runs
    // as a grid of row blocks of A and C by column panels of B and C, each an ordinary plan of its own on
    // offset pointers.  A row-major B of that size cannot be cut into panels that way (a panel still spans
    // all K rows), so it is first copied, transposed, into the workspace (N x K, K contiguous), whose
    // panels of rows are contiguous.
    bool blocked = false;
    bool blocked_bt = false;            // B is row-major and goes through the transposed copy
    int64_t block_m = 0, block_n = 0;   // rows and columns per block
    hgemm_layouts_t block_lay;          // layouts the blocks' plans were made for
    hgemm_plan_s* sub[2][2] = {{nullptr, nullptr}, {nullptr, nullptr}};   // [last, shorter row block][last, narrower panel]
};

// ---------------------------------------------------------------------------
// Static scratch for hgemm_run_static(): callers that may not allocate (code under HIP graph
// capture, tight serving loops) get their split-K planes, stream-K partial tiles and padded operand
// copies from this array instead of a hipMalloc'ed workspace.  Every GPU the library runs on holds
// its own copy at its own address until the process ends.  In host code the array's name is only a
// stand-in for the symbol: the device address comes from hipGetSymbolAddress(), once per device.
// ---------------------------------------------------------------------------
constexpr size_t kScratchBytes = (size_t)HGEMM_STATIC_SCRATCH_BYTES;
constexpr size_t kCounterBytes = 64 * 1024;      // arrival counters of fused split-K plans: up to 16384 tiles
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on device `dev` (which must be the current device), or null.
void* scratch_ptr_for(int dev)
{
    if (dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

bool fast_path_ok(int64_t M, int64_t N, int64_t K, const hgemm_layouts_t& l)
{
    if (N % 8 || K % 8 || l.lda % 8 || l.ldb % 8 || l.ldc % 8) return false;
    // buffer offsets are 32-bit and bit 31 marks "out of range": keep every operand, including
    // the rows a padded tile may address, below 2 GiB
    const int64_t lim = (int64_t)1 << 31;
    const int64_t b_rows = (l.b == HGEMM_ROW_MAJOR) ? K : N;
    if ((M + 512) * l.lda * 2 >= lim || (b_rows + 512) * l.ldb * 2 >= lim || M * l.ldc * 2 >= ((int64_t)1 << 33)) return false;
    if ((N + 512) * K * 2 >= lim) return false;      // also the transposed copy of B, should a plan ask for one
    if (M >= (1 << 24) || N >= (1 << 24) || K >= (1 << 24)) return false;
    return true;
}

// Compute units of the current device, asked once per process.  Host-only callers on a machine
// without a GPU (the planner's helpers are usable there) get the MI355X figure.
int64_t cu_count()
{
    static const int64_t n = [] {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
            return (int64_t)prop.multiProcessorCount;
        (void)hipGetLastError();
        return (int64_t)256;
    }();
    return n;
}
constexpr int64_t kLdsPerCU = 160 * 1024;
constexpr double kCacheResidentBytes = 192.0 * 1024 * 1024;

// Last-resort rules, used only when neither the table nor the cost model yields a kernel this
// build holds.  They follow the trends of
// Section 6 (tile height/width grow with M/N; more stages for long K) with MI355X numbers:
// 256 CUs want >= 256 workgroups, so small problems take smaller tiles or split K.
Spec heuristic(int64_t M, int64_t N, int64_t K)
{
    Spec s;
    s.fam = FAM_MFMA;
    s.gm = 8;
    auto tiles = [&](int bm, int bn) { return ((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
    const int64_t CUS = cu_count();
    if (M <= 32) {
        s.bm = 32; s.bn = 128; s.bk = 64; s.wm = 1; s.wn = 4; s.st = 4;
    } else if (M <= 64) {
        s.bm = 64; s.bn = 128; s.bk = 64; s.wm = 2; s.wn = 2; s.st = 4;
    } else if (tiles(256, 256) >= CUS) {
        s.bm = 256; s.bn = 256; s.bk = 64; s.wm = 2; s.wn = 2; s.st = 2;
    } else if (tiles(128, 128) >= CUS || M * N >= (int64_t)2048 * 2048) {
        s.bm = 128; s.bn = 128; s.bk = 64; s.wm = 2; s.wn = 2; s.st = 4;
    } else {
        s.bm = 64; s.bn = 64; s.bk = 64; s.wm = 2; s.wn = 2; s.st = 4;
        if (M >= 128 && N >= 128 && tiles(128, 128) * 4 >= CUS) { s.bm = 128; s.bn = 128; }
    }
    // split K when the grid leaves most CUs idle and K is long enough to share
    const int64_t t = tiles(s.bm, s.bn);
    s.sk = 1;
    if (t < CUS && K >= 1024) {
        int64_t want = (2 * CUS + t - 1) / t;                 // aim at about two workgroups per CU
        int64_t max_by_k = K / (4 * s.bk);                    // at least four K-tiles per split
        s.sk = (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, max_by_k), 64));
    }
    return s;
}

#include "dispatch_table.inc"
#include "dispatch_table_tn.inc"

// The measured row for a shape: with column-major B the table tuned in that layout first, then (as for
// row-major B) the table tuned with row-major B, whose tile sizes and split factors carry over.
bool table_lookup(int64_t M, int64_t N, int64_t K, bool b_col_major, Spec* out)
{
    if (b_col_major)
        for (size_t i = 0; i < sizeof(kDispatchTableTN) / sizeof(kDispatchTableTN[0]); ++i) {
            const DispatchRow& r = kDispatchTableTN[i];
            if (r.m == M && r.n == N && r.k == K && r.spec[0] != '\0' && parse_spec(r.spec, out)) return true;
        }
    for (size_t i = 0; i < sizeof(kDispatchTable) / sizeof(kDispatchTable[0]); ++i) {
        const DispatchRow& r = kDispatchTable[i];
        if (r.m == M && r.n == N && r.k == K) {
            // a row of the NN table serves a column-major B only if it names the large-tile family (the streaming
            // family decomposes the two layouts differently: slab and wave counts do not carry over)
            return r.spec[0] != '\0' && parse_spec(r.spec, out) && !(b_col_major && out->fam != FAM_MFMA);
        }
    }
    return false;
}

// ---------------------------------------------------------------------------
// Plan-time cost model for shapes the table does not hold.  Section 6 of the paper reads trends off
// its per-shape winners; here the dependence on (M, N, K) is an explicit model of one launch --
// matrix-core and copy time per K-tile, prologue/epilogue per workgroup, rounds over the compute
// units, whole-problem memory time, the second pass of split-K -- with constants fitted to measured
// times of all candidates on random shapes (plan_model.py holds the same formula and the fit).
// ---------------------------------------------------------------------------
struct PlanModel {
#define PLAN_MODEL_CONST(name, value) double name = value;
#include "plan_model.inc"
#undef PLAN_MODEL_CONST
};
const PlanModel kModel;

constexpr double kPadMinMacs = 1024.0 * 1024;     // below this many multiply-adds an unaligned problem stays on the generic kernel

// Split count finish_plan() will actually use: ranges are whole K-tiles, empty splits are dropped.
int64_t effective_splits(int64_t ktiles, int64_t sk)
{
    sk = std::min<int64_t>(sk, std::max<int64_t>(ktiles, 1));
    if (sk < 1) sk = 1;
    const int64_t per = (ktiles + sk - 1) / sk;
    return std::max<int64_t>(1, (ktiles + per - 1) / std::max<int64_t>(per, 1));
}

// Split factors worth considering for a configuration with `t` tiles and `ktiles` K-tiles.
std::vector<int> split_candidates(int64_t t, int64_t ktiles)
{
    std::vector<int> sks = {1};
    const int64_t kCUs = cu_count();
    if (t < 2 * kCUs) {
        for (int sk : {2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64}) {
            if (ktiles / sk < 2) break;
            if (t * sk > 8 * kCUs) break;
            sks.push_back(sk);
        }
    }
    return sks;
}

// Tiles far taller or wider than the problem only waste matrix-core work.
bool tile_fits_problem(const MfmaEntry& e, int64_t M, int64_t N)
{
    if (e.bm >= 2 * M && e.bm > 32) return false;
    if (e.bn >= 2 * N && e.bn > 64) return false;
    return true;
}

// Predicted microseconds of one call (plain or split-K kernel, default tile order).
double predict_us(int64_t Mi, int64_t Ni, int64_t Ki, int bm, int bn, int bk, int wm, int wn, int st, int pf, int64_t ski)
{
    const PlanModel& g = kModel;
    const int64_t kCUs = cu_count();
    const double M = (double)Mi, N = (double)Ni, K = (double)Ki;
    const int nw = wm * wn;
    const double tiles = (double)(((Mi + bm - 1) / bm) * ((Ni + bn - 1) / bn));
    const double kt = (double)((Ki + bk - 1) / bk);
    const double sk = (double)ski;
    const int64_t lds = (int64_t)st * (bm + bn) * bk * 2;
    const int tm = bm / wm / 32, tn = bn / wn / 32;
    const int regs = tm * tn * 16 + (pf + 1) * (tm + tn) * 4 + 40;       // accumulators + fragment sets + addressing
    const int wps = std::max(1, std::min(8, 512 / std::max(regs, 64)));  // waves per SIMD the register file admits
    const double occ = (double)std::max<int64_t>(1, std::min<int64_t>(kLdsPerCU / lds, nw <= wps * 4 ? (wps * 4) / nw : 1));

    const double wgs = tiles * sk;
    const double kt_wg = std::ceil(kt / sk);
    const double w = std::ceil(wgs / (double)kCUs);
    const double co = std::min(occ, w);
    const double rounds = std::ceil(w / co);
    const double flop = 2.0 * M * N * K;
    const double big = std::min(2.0, std::max(0.0, std::log10(std::max(flop, 1.0)) - 10.0)) / 2.0;
    double t_mfma = 2.0 * bm * bn * bk / g.F * (1.0 + g.c1 * (double)(tm + tn) / (double)(tm * tn)) * (1.0 + g.cp * big);
    if (pf == 1) t_mfma *= g.q1;
    if (bm == 32) t_mfma *= g.m32;
    if (bk == 128) t_mfma *= g.k128; else if (bk == 32) t_mfma *= g.k32;
    const double stage = (double)(bm + bn) * bk * 2.0;
    const double bytes_in = 2.0 * (M * K + K * N);
    const double bytes_c = 2.0 * M * N;
    const double part = ski > 1 ? sk * M * N * 4.0 : 0.0;
    const bool resident = bytes_in + bytes_c < kCacheResidentBytes;
    const double miss = std::min(1.0, bytes_in / (wgs * kt_wg * stage));
    const double lat = g.L + miss * (resident ? 0.0 : g.Lh);
    double peak = g.BW * (nw == 2 ? g.a2 : nw == 8 ? g.a8 : nw == 16 ? g.a16 : 1.0);
    peak *= (bn == 64 ? g.b64 : bn == 256 ? g.b256 : 1.0);
    const double inflight = (double)std::max(st - 1, 1) * stage * co;
    const double bw = std::min(peak, inflight / lat) / co;
    const double t_copy = stage / bw;
    const double t_kt = std::max(t_mfma * co, t_copy) + g.ov * std::min(t_mfma * co, t_copy) + g.tk;        // ns
    const double pro = g.Tpro;
    const double epi = g.e0 + (ski > 1 ? bm * bn * 4.0 / g.BWp : bm * bn * 2.0 / g.BWepi) * 1e-3;
    const double cu_time = rounds * (kt_wg * t_kt * 1e-3 + pro + epi);
    const double tot_inflight = std::min(wgs, (double)kCUs * occ) * (double)std::max(st - 1, 1) * stage;
    const double bw_read = (resident && part + bytes_in + bytes_c < kCacheResidentBytes)
                               ? g.BWs
                               : std::min(g.BWh * (bn == 64 ? g.h64 : bn == 128 ? g.h128 : 1.0), tot_inflight / g.Lhb);
    const double writes = ski > 1 ? part : bytes_c;
    const double tiles_m = (double)((Mi + bm - 1) / bm);
    const double hbm_bytes = resident ? bytes_in : 2.0 * M * K + 2.0 * K * N * (1.0 + g.rr * (std::min(tiles_m, 8.0) - 1.0));
    const double t_main = std::max(cu_time, hbm_bytes / bw_read * 1e-3) + writes / (co <= 1.0 ? g.BWw1 : g.BWw2) * 1e-3;
    const double t_red = ski > 1 ? g.Tr0 + g.Tr1 * std::ceil(sk / 8.0) + (part + bytes_c) / g.BWr * 1e-3 : 0.0;
    return g.T0 + t_main + t_red;
}

// Predicted microseconds of one call of a skinny-family kernel: a launch floor, the chip-wide streaming
// time of B at a rate that grows with the number of workgroups in flight, the partial-plane traffic,
// and the reduction (a second launch, or the tail of the fused form).
struct SkinnyModel {
    // fitted (soft-L1 on log time, rms 0.095) to 107 measured (shape, slabs, fused) points of the register-transposing
    // kernel: M = 1, 16 on the C3 weights with every slab count, M = 1 .. 64 on weights of 112-448 MiB
    double t0 = 4.2;          // us: launch, first bytes and the waves' meeting at the end
    double bw = 6770.0;       // bytes/ns: chip-wide streaming rate with enough workgroups
    double wg_bw = 37.7;      // bytes/ns one workgroup sustains (its two steps of loads in flight)
    double round = 1.44;      // us of fill and drain per round of resident workgroups (3 per compute unit)
    double part_bw = 8750.0;  // bytes/ns for writing and re-reading fp32 planes
    double red2 = 1.93;       // us: second launch of the two-kernel reduction
    double red1 = 1.57;       // us: tail of the fused reduction
    double red1_per_mb = 5.0; // us more per MiB of planes when they are stored device-coherently
    double per_block = 0.28;  // relative cost of every further 16-row block of A (registers: fewer resident waves)
};
const SkinnyModel kSkinny;

double predict_skinny_us(int64_t M, int64_t N, int64_t K, int64_t sk, bool fused)
{
    const SkinnyModel& g = kSkinny;
    const double strips = (double)((N + kSkinnyCols - 1) / kSkinnyCols);
    const double wgs = strips * (double)sk;
    const double rate = std::min(g.bw, g.wg_bw * wgs);
    const double planes = sk > 1 ? (double)sk * M * N * 4.0 : 0.0;
    const double mblocks = M <= 16 ? 1.0 : M <= 32 ? 2.0 : 4.0;
    double t = g.t0 + 2.0 * (double)K * N / rate * 1e-3 * (1.0 + g.per_block * (mblocks - 1.0)) + std::ceil(wgs / (3.0 * (double)cu_count())) * g.round +
               2.0 * planes / g.part_bw * 1e-3;
    if (sk > 1) t += fused ? g.red1 + g.red1_per_mb * planes / 1048576.0 : g.red2;
    return t;
}

// The cheapest compiled configuration and split factor under the model.
// Split-K with the reduction fused into the kernel against the two-launch form, as measured on skinny
// shapes: the second launch (its dispatch gap and its own round trip) goes away, the planes are stored
// device-coherently (slower per byte) and the last workgroup's re-read is a serial tail.
double fused_delta_us(int64_t M, int64_t N, int64_t sk)
{
    const double planes_mib = (double)sk * (double)M * (double)N * 4.0 / 1048576.0;
    return -0.8 + 1.6 * planes_mib;
}

// Slab counts worth considering for the skinny family (distinct after rounding to whole steps of a
// four-wave workgroup, 64 rows).
std::vector<int> skinny_split_candidates(int64_t N, int64_t K)
{
    const int64_t ksteps = (K + 63) / 64, strips = (N + kSkinnyCols - 1) / kSkinnyCols;
    std::vector<int> out;
    int64_t last = 0;
    for (int sk : {1, 2, 4, 8, 16, 32, 64, 128}) {
        const int64_t eff = effective_splits(ksteps, sk);
        if (eff == last || strips * eff > 64 * cu_count()) continue;
        last = eff;
        out.push_back((int)eff);
    }
    return out;
}

bool model_choice(int64_t M, int64_t N, int64_t K, Spec* out, bool b_row_major = true)
{
    double best = 1e300;
    bool found = false;
    if (b_row_major && M <= kSkinnyMaxM) {
        for (int sk : skinny_split_candidates(N, K)) {
            for (int fr = 0; fr <= (sk > 1 ? 1 : 0); ++fr) {
                const double us = predict_skinny_us(M, N, K, sk, fr != 0);
                if (us < best) {
                    best = us;
                    found = true;
                    Spec s;
                    s.fam = FAM_SKINNY; s.sk = (int)sk; s.fr = fr;
                    *out = s;
                }
            }
        }
    }
    // The large-tile model below was fitted to timings with the operands warm in the last-level cache wherever
    // they fit it, the streaming family's to operands streamed from HBM; the two are not comparable for a few
    // rows of A against weights that no cache holds (256 MiB and more).  Measured from HBM at M <= 32 the
    // streaming family is the faster one there (8 and 32 x 28672 x 8192: 81 / 94 us against 128 for the large-tile
    // pick; 8192 x 28672: 77 / 87 against 116; 4 x 16384 x 16384: 87 us, 77 % of the HBM rate); for weights of
    // 128-160 MiB the two families are level at M = 1 and the 32-row tiles ahead from M = 16 on (32 x 10240 x 8192:
    // 36 us against 51), so those stay with the model.
    if (found && M <= 32 && 2.0 * (double)K * (double)N >= 256.0 * 1048576.0) return true;
    for (const MfmaEntry& e : registry()) {
        if (e.deep || e.mi != 32) continue;          // the cost model was not fitted to these kernels: the tuner's business
        if (!tile_fits_problem(e, M, N)) continue;
        const int64_t t = ((M + e.bm - 1) / e.bm) * ((N + e.bn - 1) / e.bn);
        const int64_t ktiles = (K + e.bk - 1) / e.bk;
        for (int sk0 : split_candidates(t, ktiles)) {
            const int64_t sk = effective_splits(ktiles, sk0);
            double us = predict_us(M, N, K, e.bm, e.bn, e.bk, e.wm, e.wn, e.st, e.pf, sk);
            const bool fuse = sk > 1 && fused_delta_us(M, N, sk) < 0.0 && (int64_t)t * (int64_t)sizeof(int) <= (int64_t)kCounterBytes;
            if (fuse) us += fused_delta_us(M, N, sk);
            if (us < best) {
                best = us;
                found = true;
                Spec s;
                s.fam = FAM_MFMA; s.bm = e.bm; s.bn = e.bn; s.bk = e.bk; s.wm = e.wm; s.wn = e.wn; s.st = e.st; s.pf = e.pf;
                s.sk = (int)sk; s.gm = 8; s.fr = fuse ? 1 : 0;
                *out = s;
            }
        }
    }
    return found;
}

// Large problems the table does not hold: the tuned choice of the nearest shape that it does hold.
// The cost model was fitted before the 16x16x32 kernels existed and never picks them, and on problems
// of many tiles a neighbour's winner carries over (25 off-table shapes of at least 10^11 flop: the
// neighbour's kernel is faster than the model's on 21, 4.7 % in the geometric mean) -- except where the
// neighbour's tile fills the last round of workgroups much worse than the model's pick does (3000 x
// 6144 x 4096: 288 tiles of 256 x 256 against 512 of 192 x 192, 18 % slower), which is what the
// comparison of the two fill ratios below rules out (with it: 20 of 136 shapes change, those 7.5 %
// faster in the geometric mean, none slower by more than 0.3 %).  Distance = sum over M, N, K of
// |log2 ratio|, at most 1.5.
double last_round_fill(const Spec& s, int64_t M, int64_t N)
{
    if (s.fam != FAM_MFMA || s.bm <= 0 || s.bn <= 0) return 0.0;
    const int64_t cus = cu_count();
    const int64_t t = ((M + s.bm - 1) / s.bm) * ((N + s.bn - 1) / s.bn) * std::max(1, s.sk);
    return (double)t / (double)(((t + cus - 1) / cus) * cus);
}

bool neighbour_choice(int64_t M, int64_t N, int64_t K, bool b_col_major, const Spec& model, Spec* out)
{
    if (2.0 * (double)M * (double)N * (double)K < 3e10 || std::min(M, N) < 512 || model.fam != FAM_MFMA) return false;
    const DispatchRow* rows = b_col_major ? kDispatchTableTN : kDispatchTable;
    const size_t count = b_col_major ? sizeof(kDispatchTableTN) / sizeof(kDispatchTableTN[0]) : sizeof(kDispatchTable) / sizeof(kDispatchTable[0]);
    auto lg = [](int64_t v) { return std::log2((double)std::max<int64_t>(v, 1)); };
    double best = 1.5;
    const DispatchRow* pick = nullptr;
    for (size_t i = 0; i < count; ++i) {
        const DispatchRow& r = rows[i];
        if (r.m <= 0 || r.spec[0] == '\0') continue;
        const double d = std::fabs(lg(M) - lg(r.m)) + std::fabs(lg(N) - lg(r.n)) + std::fabs(lg(K) - lg(r.k));
        if (d <= best) { best = d; pick = &r; }
    }
    Spec near;
    if (!pick || !parse_spec(pick->spec, &near) || near.fam != FAM_MFMA || near.tb) return false;
    const MfmaEntry* e = find_entry(near);
    if (!e || !tile_fits_problem(*e, M, N)) return false;
    if (last_round_fill(near, M, N) < last_round_fill(model, M, N) - 0.1) return false;
    *out = near;
    return true;
}

// Gives the plan its workspace of p->workspace_bytes (static scratch or an allocation), points the
// partial-sum and counter arguments into it and clears the counters of an allocated one.
hgemm_status_t acquire_workspace(hgemm_plan_s* p, size_t partial_bytes, size_t ctr_bytes)
{
    GemmArgs& a = p->args;
    if (p->workspace_bytes && p->static_ws) {
        if (p->workspace_bytes > kScratchBytes) { p->workspace_bytes = 0; return HGEMM_ERR_WORKSPACE; }
        p->workspace = scratch_ptr_for(p->device);
        if (!p->workspace) { p->workspace_bytes = 0; return HGEMM_ERR_LAUNCH; }
        if (partial_bytes) a.partial = (float*)((char*)p->workspace + p->partial_offset);
        if (ctr_bytes) a.counters = (int*)p->workspace;          // static arrays start out zero
    } else if (p->workspace_bytes) {
        if (hipMalloc(&p->workspace, p->workspace_bytes) != hipSuccess) {
            (void)hipGetLastError();
            p->workspace = nullptr;
            p->workspace_bytes = 0;
            return HGEMM_ERR_ALLOC;
        }
        if (partial_bytes) a.partial = (float*)((char*)p->workspace + p->partial_offset);
        if (ctr_bytes) {
            if (hipMemset(p->workspace, 0, ctr_bytes) != hipSuccess) {
                (void)hipGetLastError();
                (void)hipFree(p->workspace);
                p->workspace = nullptr;
                p->workspace_bytes = 0;
                return HGEMM_ERR_ALLOC;
            }
            a.counters = (int*)p->workspace;
        }
    }
    return HGEMM_OK;
}

hgemm_status_t finish_plan(hgemm_plan_s* p)
{
    const int64_t M = p->M, N = p->N, K = p->K;
    Spec& s = p->spec;
    p->entry = nullptr;
    p->workspace = nullptr;
    p->workspace_bytes = 0;
    p->partial_offset = 0;
    p->tn_kernel = false;
    memset(&p->args, 0, sizeof p->args);
    p->skinny = nullptr;
    if (s.fam == FAM_GENERIC) return HGEMM_OK;
    if (s.fam == FAM_SKINNY) {
        // strips of columns x K slabs of whole steps; partial planes as for split-K
        if (!fast_path_ok(M, N, K, p->lay) || M <= 0 || N <= 0 || K <= 0 || M > kSkinnyMaxM) return HGEMM_ERR_UNSUPPORTED;
        const bool tn = p->lay.b == HGEMM_COL_MAJOR;
        p->tn_kernel = tn;
        const int mb = M <= 16 ? 1 : M <= 32 ? 2 : 4;
        const int64_t step = skinny_step(s, tn);
        const int64_t ksteps = (K + step - 1) / step;
        const int64_t sk = effective_splits(ksteps, s.sk);
        if (sk > 65535) return HGEMM_ERR_UNSUPPORTED;
        s.sk = (int)sk;
        if (sk == 1) s.fr = 0;
        if (!tn && s.nr != 16) return HGEMM_ERR_UNSUPPORTED;
        const int64_t strips = (N + skinny_cols(s, tn) - 1) / skinny_cols(s, tn);
        if (s.fr && strips * (int64_t)sizeof(int) > (int64_t)kCounterBytes) return HGEMM_ERR_UNSUPPORTED;
        p->skinny = skinny_kernel(mb, s.fr != 0, s.wv, tn ? s.nr : 0);
        if (!p->skinny) return HGEMM_ERR_UNSUPPORTED;
        GemmArgs& a = p->args;
        a.M = (int)M; a.N = (int)N; a.K = (int)K;
        a.lda = (int)p->lay.lda; a.ldb = (int)p->lay.ldb; a.ldc = (int)p->lay.ldc;
        a.tiles_m = 1; a.tiles_n = (int)strips;
        a.splits = (int)sk;
        a.k_per_split = (int)(((ksteps + sk - 1) / sk) * step);
        // workspace: [counters] [padded copies of A, B, C (plans on zero-padded operands)] [planes]
        auto up256s = [](size_t b) { return ((b + 255) / 256) * 256; };
        size_t pad_bytes = 0;
        p->a_off = p->b_off = p->c_off = 0;
        if (p->padded) {
            p->b_off = up256s((size_t)M * (size_t)K * 2);
            p->c_off = p->b_off + up256s((size_t)K * (size_t)N * 2);
            pad_bytes = p->c_off + up256s((size_t)M * (size_t)N * 2);
        }
        const size_t partial_bytes = sk > 1 ? up256s((size_t)sk * (size_t)M * (size_t)N * sizeof(float)) : 0;
        const size_t ctr_bytes = (s.fr || (p->static_ws && pad_bytes + partial_bytes > 0)) ? kCounterBytes : 0;
        p->a_off += ctr_bytes; p->b_off += ctr_bytes; p->c_off += ctr_bytes;
        p->bt_off = ctr_bytes + pad_bytes;
        p->partial_offset = ctr_bytes + pad_bytes;
        p->workspace_bytes = ctr_bytes + pad_bytes + partial_bytes;
        return acquire_workspace(p, partial_bytes, ctr_bytes);
    }
    const MfmaEntry* e = find_entry(s);
    if (!e) return HGEMM_ERR_UNSUPPORTED;
    if (!fast_path_ok(M, N, K, p->lay)) return HGEMM_ERR_UNSUPPORTED;
    if (s.tb && p->lay.b != HGEMM_ROW_MAJOR) return HGEMM_ERR_UNSUPPORTED;
    p->tn_kernel = s.tb || p->lay.b == HGEMM_COL_MAJOR;
    p->entry = e;
    // deep-staged configurations exist for one full-K tile per workgroup only; the 16-bit accumulator for 32-wide blocks only
    if (e->deep && (s.sk > 1 || s.sm || s.ps || s.fr || s.ac == 16)) return HGEMM_ERR_UNSUPPORTED;
    if (s.ac == 16 && !e->acc16) return HGEMM_ERR_UNSUPPORTED;
    // dynamic LDS beyond 64 KiB has to be requested per kernel function
    {
        void (*const kernels[])(GemmArgs) = {e->plain, e->splitk, e->plain_tn, e->splitk_tn, e->streamk, e->streamk_tn, e->splitk_fused,
                                             e->splitk_fused_tn, e->persist, e->persist_tn, e->acc16, e->acc16_tn};
        bool ok = true;
        for (auto k : kernels)
            if (k && hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize, e->lds_bytes) != hipSuccess) ok = false;
        if (!ok) {
            (void)hipGetLastError();
            return HGEMM_ERR_LAUNCH;
        }
    }
    GemmArgs& a = p->args;
    a.M = (int)M; a.N = (int)N; a.K = (int)K;
    a.lda = (int)p->lay.lda; a.ldb = s.tb ? (int)K : (int)p->lay.ldb; a.ldc = (int)p->lay.ldc;
    a.tiles_m = (int)((M + e->bm - 1) / e->bm);
    a.tiles_n = (int)((N + e->bn - 1) / e->bn);
    if ((int64_t)a.tiles_m * a.tiles_n >= ((int64_t)1 << 24)) return HGEMM_ERR_UNSUPPORTED;      // tile_coords()
    // with a handful of tiles the order cannot matter: spare the kernel the arithmetic of the map
    a.swizzle = (int64_t)a.tiles_m * a.tiles_n <= 16 ? 0 : s.gm;
    set_tile_map(a);
    // split K into ranges that are multiples of BK; drop splits that would be empty
    int64_t ktiles = (K + e->bk - 1) / e->bk;
    const int64_t sk = effective_splits(ktiles, s.sk);
    const int64_t per = (ktiles + sk - 1) / sk;
    if (sk > 65535) return HGEMM_ERR_UNSUPPORTED;
    s.sk = (int)sk;
    if (sk == 1) s.fr = 0;                              // nothing to reduce
    if (s.ps) {
        if (!e->persist) return HGEMM_ERR_UNSUPPORTED;
        // persistent walking needs more tiles than compute units and a K long enough to keep the pipeline full
        if ((int64_t)a.tiles_m * a.tiles_n <= cu_count() || ktiles < e->st || sk > 1) s.ps = 0;
    }
    a.splits = (int)sk;
    a.k_per_split = (int)(per * e->bk);
    // stream-K geometry
    a.dp_tiles = a.tiles_m * a.tiles_n;
    a.sk_workers = 0;
    a.sk_iters_per_worker = 1;
    a.sk_total_iters = 0;
    if (s.sm) {
        const int64_t G = cu_count();
        const int64_t tiles = (int64_t)a.tiles_m * a.tiles_n;
        const int64_t dp = (tiles / G) * G;
        if (dp == tiles) {
            s.sm = 0;                                   // whole waves only: nothing to stream
        } else {
            const int64_t total = (tiles - dp) * ktiles;
            const int64_t ipw = (total + G - 1) / G;
            a.dp_tiles = (int)dp;
            a.sk_iters_per_worker = (int)ipw;
            a.sk_total_iters = (int)total;
            a.sk_workers = (int)((total + ipw - 1) / ipw);
        }
    }
    auto up256 = [](size_t b) { return ((b + 255) / 256) * 256; };
    size_t pad_bytes = 0;
    p->a_off = p->b_off = p->c_off = 0;
    if (p->padded) {
        p->a_off = 0;
        p->b_off = up256((size_t)M * (size_t)K * 2);
        p->c_off = p->b_off + up256((size_t)K * (size_t)N * 2);
        pad_bytes = p->c_off + up256((size_t)M * (size_t)N * 2);
    }
    size_t bt_bytes = s.tb ? up256((size_t)N * (size_t)K * 2) : 0;
    size_t partial_bytes = sk > 1 ? (size_t)sk * (size_t)M * (size_t)N * sizeof(float) : 0;
    if (s.sm) partial_bytes = (size_t)2 * a.sk_workers * e->bm * e->bn * sizeof(float);
    partial_bytes = up256(partial_bytes);
    // fused split-K: one arrival counter per tile in front of everything else.  Counters are zero
    // whenever no launch is in flight (the last arriver resets its own), so their place is fixed:
    // the first kCounterBytes of the workspace, whatever the rest of it holds.
    // (In the static scratch every plan keeps clear of that region, so it stays zero for the fused ones.)
    const size_t ctr_bytes = (s.fr || (p->static_ws && pad_bytes + bt_bytes + partial_bytes > 0)) ? kCounterBytes : 0;
    if (s.fr && (size_t)a.tiles_m * a.tiles_n * sizeof(int) > kCounterBytes) return HGEMM_ERR_UNSUPPORTED;
    p->a_off += ctr_bytes; p->b_off += ctr_bytes; p->c_off += ctr_bytes;
    p->bt_off = ctr_bytes + pad_bytes;
    p->partial_offset = ctr_bytes + pad_bytes + bt_bytes;
    p->workspace_bytes = ctr_bytes + pad_bytes + bt_bytes + partial_bytes;
    return acquire_workspace(p, partial_bytes, ctr_bytes);
}

// True when device `dev` is a gfx950; the answer is kept per device (hipGetDeviceProperties is slow).
bool device_is_gfx950(int dev)
{
    static std::mutex m;
    static signed char known[kMaxDevices] = {0};       // 0 = not asked yet, 1 = yes, -1 = no
    if (dev < 0 || dev >= kMaxDevices) return false;
    std::lock_guard<std::mutex> lock(m);
    if (known[dev] == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return false; }
        known[dev] = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : -1;
    }
    return known[dev] == 1;
}

// Fills *p (caller's storage) with a runnable plan.  static_ws: the workspace is the device's static
// scratch array and nothing is allocated; otherwise the workspace is hipMalloc'ed and owned by the plan.
// The specialisation the planner tries first for an aligned problem of less than 2 GiB per operand, and where
// it comes from: the layout's dispatch table (packed leading dimensions only), else the cost model, whose pick a
// large problem trades for the kernel tuned for the nearest shape of the table (neighbour_choice); `fallback` is
// the model's pick in that last case, should the neighbour's kernel refuse the shape.
const char* choose_spec(int64_t M, int64_t N, int64_t K, const hgemm_layouts_t& l, bool padded, Spec* first, Spec* fallback)
{
    const bool tn = l.b == HGEMM_COL_MAJOR;
    const bool packed = l.lda == K && l.ldc == N && l.ldb == (tn ? K : N);
    const char* source = "table";
    if (!table_lookup(M, N, K, tn, first) || !packed) {
        source = "model";
        if (!model_choice(M, N, K, first, !tn)) {
            *first = heuristic(M, N, K);
            source = "rules";
        }
        *fallback = *first;
        if (neighbour_choice(M, N, K, tn, *fallback, first)) return "neighbour";
    }
    if (tn || padded) first->tb = 0;      // B already has K contiguous / is copied once already
    *fallback = *first;
    return source;
}

hgemm_status_t init_blocked(hgemm_plan_s* p);

hgemm_status_t init_plan(hgemm_plan_s* p, int64_t M, int64_t N, int64_t K, const hgemm_layouts_t* layouts, const char* spec_text,
                         bool static_ws)
{
    if (M < 0 || N < 0 || K < 0) return HGEMM_ERR_INVALID_ARG;
    hgemm_layouts_t l;
    if (layouts) {
        l = *layouts;
    } else {
        l.a = l.b = l.c = HGEMM_ROW_MAJOR;
        l.lda = l.ldb = l.ldc = 0;
    }
    if ((l.a != HGEMM_ROW_MAJOR && l.a != HGEMM_COL_MAJOR) || (l.b != HGEMM_ROW_MAJOR && l.b != HGEMM_COL_MAJOR) ||
        (l.c != HGEMM_ROW_MAJOR && l.c != HGEMM_COL_MAJOR))
        return HGEMM_ERR_INVALID_ARG;
    if (l.a != HGEMM_ROW_MAJOR || l.c != HGEMM_ROW_MAJOR) return HGEMM_ERR_UNSUPPORTED;
    if (l.lda < 0 || l.ldb < 0 || l.ldc < 0) return HGEMM_ERR_INVALID_ARG;
    if (l.lda == 0) l.lda = K;
    if (l.ldb == 0) l.ldb = (l.b == HGEMM_ROW_MAJOR) ? N : K;
    if (l.ldc == 0) l.ldc = N;
    if (l.lda < K || l.ldc < N || l.ldb < ((l.b == HGEMM_ROW_MAJOR) ? N : K)) return HGEMM_ERR_INVALID_ARG;

    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return HGEMM_ERR_ARCH; }
    if (!device_is_gfx950(dev)) return HGEMM_ERR_ARCH;

    p->M = M; p->N = N; p->K = K; p->lay = l; p->device = dev;
    p->padded = false;
    p->static_ws = static_ws;
    p->uM = M; p->uN = N; p->uK = K; p->ulay = l;
    p->a_off = p->b_off = p->c_off = p->bt_off = 0;

    hgemm_status_t st;
    if (spec_text) {
        if (!parse_spec(spec_text, &p->spec)) return HGEMM_ERR_INVALID_ARG;
        st = finish_plan(p);
    } else {
        bool fast = fast_path_ok(M, N, K, l) && M > 0 && N > 0 && K > 0;
        if (!fast && M > 0 && N > 0 && K > 0 && (double)M * (double)N * (double)K >= kPadMinMacs) {
            // N, K or a leading dimension is not a multiple of 8.  Above a size where the one-thread-per-
            // element kernel would take longer than four extra launches, run the matrix-core kernel on
            // packed copies whose N and K are rounded up to 8 and zero-filled (the paper's zero padding,
            // Section 5.2, applied to the dimensions the 16-byte copies need aligned).
            const int64_t Kp = (K + 7) / 8 * 8, Np = (N + 7) / 8 * 8;
            hgemm_layouts_t lp = l;
            lp.lda = Kp;
            lp.ldb = (l.b == HGEMM_ROW_MAJOR) ? Np : Kp;
            lp.ldc = Np;
            if (fast_path_ok(M, Np, Kp, lp)) {
                p->padded = true;
                p->N = N = Np;
                p->K = K = Kp;
                p->lay = l = lp;
                fast = true;
            }
        }
        const bool dims_aligned = !(N % 8 || K % 8 || l.lda % 8 || l.ldb % 8 || l.ldc % 8) && M < (1 << 24) && N < (1 << 24) && K < (1 << 24);
        if (!fast && !static_ws && M > 0 && N > 0 && K > 0 && dims_aligned && init_blocked(p) == HGEMM_OK) return HGEMM_OK;
        if (!fast) {
            p->spec = Spec();
            st = finish_plan(p);
        } else {
            Spec fallback;
            if (!strcmp(choose_spec(M, N, K, l, p->padded, &p->spec, &fallback), "neighbour")) {
                if (finish_plan(p) == HGEMM_OK) return HGEMM_OK;
                p->spec = fallback;
                if (l.b == HGEMM_COL_MAJOR || p->padded) p->spec.tb = 0;
            }
            st = finish_plan(p);
            if (st == HGEMM_ERR_UNSUPPORTED) {
                // a table row naming a kernel this build lacks, or a row of the NN table, consulted for a
                // column-major B, that names the streaming family (row-major B only): the cost model decides
                if (!model_choice(M, N, K, &p->spec, l.b == HGEMM_ROW_MAJOR)) p->spec = heuristic(M, N, K);
                if (l.b == HGEMM_COL_MAJOR || p->padded) p->spec.tb = 0;
                st = finish_plan(p);
                if (st == HGEMM_ERR_UNSUPPORTED) {
                    p->spec = heuristic(M, N, K);
                    st = finish_plan(p);
                }
            }
            if (st != HGEMM_OK && st != HGEMM_ERR_WORKSPACE && p->padded) {   // e.g. no memory for the padded copies: the generic kernel needs none
                p->padded = false;
                p->M = p->uM; p->N = p->uN; p->K = p->uK; p->lay = p->ulay;
                p->spec = Spec();
                st = finish_plan(p);
            }
        }
    }
    return st;
}

void destroy_blocks(hgemm_plan_s* p)
{
    for (auto& row : p->sub)
        for (hgemm_plan_s*& q : row) {
            if (!q) continue;
            if (q->workspace && !q->static_ws && hipFree(q->workspace) != hipSuccess) (void)hipGetLastError();
            delete q;
            q = nullptr;
        }
    p->blocked = false;
}

// Plans a problem whose dimensions are aligned but whose operands reach 2 GiB as a grid of blocks (see
// hgemm_plan_s).  On failure the plan is left as it was, for the generic kernel.
// Block sizes for a problem whose dimensions are aligned but whose operands reach 2 GiB: rows per block of A and
// C, columns per panel of B and C (equal sizes, multiples of 256), whether a row-major B has to go through a
// transposed copy, and the layouts the blocks are planned for.  False when no such split exists.
bool block_sizes(int64_t M, int64_t N, int64_t K, const hgemm_layouts_t& l, int64_t* rows, int64_t* cols, bool* transposed, hgemm_layouts_t* block_lay)
{
    const int64_t lim = (int64_t)1 << 31;
    auto down256 = [](int64_t v) { return v / 256 * 256; };
    int64_t bm = std::min<int64_t>(M, std::min(down256((lim - 1) / (l.lda * 2) - 512), down256((((int64_t)1 << 33) - 1) / (l.ldc * 2))));
    if (bm <= 0) return false;
    hgemm_layouts_t sl = l;
    // can the matrix-core kernels address B as it lies?  (asked of a block of 256 rows)
    bool bt = false;
    if (l.b == HGEMM_ROW_MAJOR && !fast_path_ok(std::min<int64_t>(bm, 256), N, K, l)) {
        if ((K + 63) / 64 > 65535) return false;          // grid of the transposing copy
        bt = true;
        sl.b = HGEMM_COL_MAJOR;
        sl.ldb = K;
    }
    int64_t bn = N;
    if (sl.b == HGEMM_COL_MAJOR) {
        bn = std::min<int64_t>(N, down256((lim - 1) / (sl.ldb * 2) - 512));
        if (bn <= 0) return false;
    }
    // blocks of equal size (a multiple of 256) rather than full ones and a sliver
    auto even = [](int64_t total, int64_t most) {
        const int64_t parts = (total + most - 1) / most;
        return std::min(most, ((total + parts - 1) / parts + 255) / 256 * 256);
    };
    if (bm < M) bm = even(M, bm);
    if (bn < N) bn = even(N, bn);
    if (!fast_path_ok(bm, bn, K, sl)) return false;
    *rows = bm;
    *cols = bn;
    *transposed = bt;
    *block_lay = sl;
    return true;
}

hgemm_status_t init_blocked(hgemm_plan_s* p)
{
    const int64_t M = p->M, N = p->N, K = p->K;
    int64_t bm = 0, bn = 0;
    bool bt = false;
    hgemm_layouts_t sl;
    if (!block_sizes(M, N, K, p->lay, &bm, &bn, &bt, &sl)) return HGEMM_ERR_UNSUPPORTED;
    p->blocked_bt = bt;
    p->block_m = bm;
    p->block_n = bn;
    p->block_lay = sl;
    const int64_t rows[2] = {M >= bm ? bm : 0, M % bm}, cols[2] = {N >= bn ? bn : 0, N % bn};
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) {
            if (rows[i] == 0 || cols[j] == 0) continue;
            hgemm_plan_s* q = new (std::nothrow) hgemm_plan_s();
            hgemm_status_t st = q ? init_plan(q, rows[i], cols[j], K, &sl, nullptr, false) : HGEMM_ERR_ALLOC;
            if (st == HGEMM_OK && q->blocked) st = HGEMM_ERR_UNSUPPORTED;
            if (st != HGEMM_OK) {
                if (q) {
                    destroy_blocks(q);
                    if (q->workspace && hipFree(q->workspace) != hipSuccess) (void)hipGetLastError();
                    delete q;
                }
                destroy_blocks(p);
                return st;
            }
            p->sub[i][j] = q;
        }
    p->spec = Spec();
    p->entry = nullptr;
    p->skinny = nullptr;
    p->workspace = nullptr;
    p->workspace_bytes = 0;
    if (bt) {
        const size_t bytes = (size_t)N * (size_t)K * 2;
        if (hipMalloc(&p->workspace, bytes) != hipSuccess) {
            (void)hipGetLastError();
            p->workspace = nullptr;
            destroy_blocks(p);
            return HGEMM_ERR_ALLOC;
        }
        p->workspace_bytes = bytes;
    }
    p->blocked = true;
    return HGEMM_OK;
}

hgemm_status_t make_plan(hgemm_plan_t* out, int64_t M, int64_t N, int64_t K, const hgemm_layouts_t* layouts,
                         const char* spec_text)
{
    if (!out) return HGEMM_ERR_INVALID_ARG;
    hgemm_plan_s* p = new (std::nothrow) hgemm_plan_s();
    if (!p) return HGEMM_ERR_ALLOC;
    const hgemm_status_t st = init_plan(p, M, N, K, layouts, spec_text, false);
    if (st != HGEMM_OK) { delete p; return st; }
    *out = p;
    return HGEMM_OK;
}

}  // namespace

extern "C" {

hgemm_status_t hgemm_plan(hgemm_plan_t* out, int64_t M, int64_t N, int64_t K, const hgemm_layouts_t* layouts)
{
    return make_plan(out, M, N, K, layouts, nullptr);
}

hgemm_status_t hgemm_plan_override(hgemm_plan_t* out, int64_t M, int64_t N, int64_t K, const hgemm_layouts_t* layouts,
                                   const char* spec)
{
    if (!spec) return HGEMM_ERR_INVALID_ARG;
    return make_plan(out, M, N, K, layouts, spec);
}

hgemm_status_t hgemm_plan_choice(int64_t M, int64_t N, int64_t K, const hgemm_layouts_t* layouts, char* buf, size_t n)
{
    if (!buf || n == 0 || M < 0 || N < 0 || K < 0) return HGEMM_ERR_INVALID_ARG;
    hgemm_layouts_t l;
    if (layouts) l = *layouts; else { l.a = l.b = l.c = HGEMM_ROW_MAJOR; l.lda = l.ldb = l.ldc = 0; }
    if ((l.b != HGEMM_ROW_MAJOR && l.b != HGEMM_COL_MAJOR) || l.lda < 0 || l.ldb < 0 || l.ldc < 0) return HGEMM_ERR_INVALID_ARG;
    if (l.a != HGEMM_ROW_MAJOR || l.c != HGEMM_ROW_MAJOR) return HGEMM_ERR_UNSUPPORTED;
    if (l.lda == 0) l.lda = K;
    if (l.ldb == 0) l.ldb = (l.b == HGEMM_ROW_MAJOR) ? N : K;
    if (l.ldc == 0) l.ldc = N;
    if (l.lda < K || l.ldc < N || l.ldb < ((l.b == HGEMM_ROW_MAJOR) ? N : K)) return HGEMM_ERR_INVALID_ARG;
    std::string out;
    const bool nonempty = M > 0 && N > 0 && K > 0;
    bool fast = nonempty && fast_path_ok(M, N, K, l);
    bool padded = false;
    if (!fast && nonempty && (double)M * (double)N * (double)K >= kPadMinMacs) {
        const int64_t Kp = (K + 7) / 8 * 8, Np = (N + 7) / 8 * 8;
        hgemm_layouts_t lp = l;
        lp.lda = Kp;
        lp.ldb = (l.b == HGEMM_ROW_MAJOR) ? Np : Kp;
        lp.ldc = Np;
        if (fast_path_ok(M, Np, Kp, lp)) { padded = fast = true; N = Np; K = Kp; l = lp; }
    }
    int64_t rows = 0, cols = 0;
    bool bt = false;
    hgemm_layouts_t bl;
    const bool dims_aligned = !(N % 8 || K % 8 || l.lda % 8 || l.ldb % 8 || l.ldc % 8) && M < (1 << 24) && N < (1 << 24) && K < (1 << 24);
    if (!nonempty) {
        out = "empty";
    } else if (!fast && dims_aligned && block_sizes(M, N, K, l, &rows, &cols, &bt, &bl)) {
        char head[96];
        snprintf(head, sizeof head, "blocks,rows=%lld,cols=%lld%s", (long long)rows, (long long)cols, bt ? ",bt=1" : "");
        out = head;
    } else if (!fast) {
        out = "generic";
    } else {
        Spec first, fallback;
        const char* source = choose_spec(M, N, K, l, padded, &first, &fallback);
        out = std::string(source) + ": " + spec_to_string(first) + (padded ? ",pad=1" : "");
    }
    if (out.size() + 1 > n) { buf[0] = '\0'; return HGEMM_ERR_INVALID_ARG; }
    memcpy(buf, out.c_str(), out.size() + 1);
    return HGEMM_OK;
}

static hgemm_status_t run_plan(const hgemm_plan_s* plan, const void* A, const void* B, void* C, void* hip_stream)
{
    const int64_t M = plan->M, N = plan->N, K = plan->K;
    if (M == 0 || N == 0) return HGEMM_OK;
    if (!C) return HGEMM_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (K == 0) {
        const int wide = (((uintptr_t)C & 15) == 0 && plan->lay.ldc % 8 == 0) ? 1 : 0;
        hipLaunchKernelGGL(zero_c_kernel, dim3((unsigned)((N + 2047) / 2048), (unsigned)std::min<int64_t>(M, 16384)), dim3(256), 0, stream,
                           (_Float16*)C, M, N, plan->lay.ldc, wide);
        return hipGetLastError() == hipSuccess ? HGEMM_OK : HGEMM_ERR_LAUNCH;
    }
    if (!A || !B) return HGEMM_ERR_INVALID_ARG;

    if (plan->blocked) {
        const _Float16* Bp = (const _Float16*)B;
        if (plan->blocked_bt) {
            hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)((N + 63) / 64), (unsigned)((K + 63) / 64)), dim3(256), 0, stream,
                               (const _Float16*)B, (_Float16*)plan->workspace, (int)K, (int)N, (int)plan->lay.ldb);
            if (hipGetLastError() != hipSuccess) return HGEMM_ERR_LAUNCH;
            Bp = (const _Float16*)plan->workspace;
        }
        const bool panels = plan->block_lay.b == HGEMM_COL_MAJOR;          // else every block takes all of B
        for (int64_t m0 = 0; m0 < M; m0 += plan->block_m)
            for (int64_t n0 = 0; n0 < N; n0 += plan->block_n) {
                const hgemm_plan_s* q = plan->sub[M - m0 < plan->block_m ? 1 : 0][N - n0 < plan->block_n ? 1 : 0];
                if (!q) return HGEMM_ERR_INVALID_ARG;
                const hgemm_status_t st = run_plan(q, (const _Float16*)A + m0 * plan->lay.lda, panels ? Bp + n0 * plan->block_lay.ldb : Bp,
                                                   (_Float16*)C + m0 * plan->lay.ldc + n0, hip_stream);
                if (st != HGEMM_OK) return st;
            }
        return HGEMM_OK;
    }

    void* const user_C = C;
    if (plan->padded) {
        // zero-filled packed copies of A and B; the kernels below then see an aligned problem
        char* ws = (char*)plan->workspace;
        const hgemm_layouts_t& ul = plan->ulay;
        auto copy = [&](const void* src, int64_t src_ld, int64_t src_rows, int64_t src_cols, void* dst, int64_t dst_ld, int64_t dst_rows,
                        int64_t dst_cols) {
            const dim3 grid((unsigned)((dst_cols + kCopyColsPerBlock - 1) / kCopyColsPerBlock),
                            (unsigned)std::min<int64_t>((dst_rows + kCopyRowsPerBlock - 1) / kCopyRowsPerBlock, 32768));
            hipLaunchKernelGGL(copy2d_kernel<true>, grid, dim3(256), 0, stream, (const _Float16*)src, src_ld, src_rows, src_cols,
                               (_Float16*)dst, dst_ld, dst_rows, dst_cols);
        };
        copy(A, ul.lda, plan->uM, plan->uK, ws + plan->a_off, K, M, K);
        if (ul.b == HGEMM_ROW_MAJOR) copy(B, ul.ldb, plan->uK, plan->uN, ws + plan->b_off, N, K, N);
        else copy(B, ul.ldb, plan->uN, plan->uK, ws + plan->b_off, K, N, K);
        if (hipGetLastError() != hipSuccess) return HGEMM_ERR_LAUNCH;
        A = ws + plan->a_off;
        B = ws + plan->b_off;
        C = ws + plan->c_off;
    }
    // the padded output goes back to the caller's C (its N columns, its leading dimension)
    auto finish = [&]() -> hgemm_status_t {
        if (hipGetLastError() != hipSuccess) return HGEMM_ERR_LAUNCH;
        if (plan->padded) {
            const dim3 grid((unsigned)((plan->uN + kCopyColsPerBlock - 1) / kCopyColsPerBlock),
                            (unsigned)std::min<int64_t>((plan->uM + kCopyRowsPerBlock - 1) / kCopyRowsPerBlock, 32768));
            hipLaunchKernelGGL(copy2d_kernel<false>, grid, dim3(256), 0, stream, (const _Float16*)C, N, M, N, (_Float16*)user_C,
                               plan->ulay.ldc, plan->uM, plan->uN);
            if (hipGetLastError() != hipSuccess) return HGEMM_ERR_LAUNCH;
        }
        return HGEMM_OK;
    };

    const bool aligned = ((((uintptr_t)A) | ((uintptr_t)B) | ((uintptr_t)C)) & 15) == 0;
    if (plan->spec.fam == FAM_GENERIC || !aligned) {
        if (N > (int64_t)64 * 0x7fffffff || (M + 3) / 4 > 65535) {
            // grid.y limit: fold rows into several launches
            for (int64_t mb = 0; mb < M; mb += 4 * 65535) {
                const int64_t rows = std::min<int64_t>(M - mb, 4 * 65535);
                hipLaunchKernelGGL(generic_gemm_kernel, dim3((unsigned)((N + 63) / 64), (unsigned)((rows + 3) / 4)), dim3(256), 0,
                                   stream, (const _Float16*)A + mb * plan->lay.lda, (const _Float16*)B,
                                   (_Float16*)C + mb * plan->lay.ldc, rows, N, K, plan->lay.lda, plan->lay.ldb, plan->lay.ldc,
                                   plan->lay.b == HGEMM_COL_MAJOR ? 1 : 0);
            }
        } else {
            hipLaunchKernelGGL(generic_gemm_kernel, dim3((unsigned)((N + 63) / 64), (unsigned)((M + 3) / 4)), dim3(256), 0, stream,
                               (const _Float16*)A, (const _Float16*)B, (_Float16*)C, M, N, K, plan->lay.lda, plan->lay.ldb,
                               plan->lay.ldc, plan->lay.b == HGEMM_COL_MAJOR ? 1 : 0);
        }
        return finish();
    }

    GemmArgs a = plan->args;
    a.A = (const _Float16*)A;
    a.B = (const _Float16*)B;
    a.C = (_Float16*)C;
    if (plan->skinny) {
        hipLaunchKernelGGL(plan->skinny, dim3((unsigned)a.tiles_n, (unsigned)a.splits), dim3(64u * (unsigned)plan->spec.wv), 0, stream, a);
        if (a.splits > 1 && !plan->spec.fr) {
            if (hipGetLastError() != hipSuccess) return HGEMM_ERR_LAUNCH;
            const int64_t quads = M * (N / 4);
            const int blocks = (int)std::min<int64_t>((quads + 255) / 256, 2048);
            hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks), dim3(256), 0, stream,
                               (const float*)((const char*)plan->workspace + plan->partial_offset), (_Float16*)C, (int)M, (int)N,
                               (int)plan->lay.ldc, a.splits);
        }
        return finish();
    }
    const MfmaEntry* e = plan->entry;
    const unsigned wgs = (unsigned)(a.tiles_m * a.tiles_n);
    if (plan->spec.tb) {
        // B (K x N, row-major) -> workspace (N x K, row-major), then the K-contiguous kernel
        hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)((N + 63) / 64), (unsigned)((K + 63) / 64)), dim3(256), 0, stream,
                           (const _Float16*)B, (_Float16*)((char*)plan->workspace + plan->bt_off), (int)K, (int)N, (int)plan->lay.ldb);
        if (hipGetLastError() != hipSuccess) return HGEMM_ERR_LAUNCH;
        a.B = (const _Float16*)((char*)plan->workspace + plan->bt_off);
    }
    if (plan->spec.sm) {
        hipLaunchKernelGGL(plan->tn_kernel ? e->streamk_tn : e->streamk, dim3((unsigned)(a.dp_tiles + a.sk_workers)), dim3(e->threads),
                           e->lds_bytes, stream, a);
        if (hipGetLastError() != hipSuccess) return HGEMM_ERR_LAUNCH;
        hipLaunchKernelGGL(e->fixup, dim3(wgs - (unsigned)a.dp_tiles, (unsigned)((e->bm * e->bn / 4 + 1023) / 1024)), dim3(256), 0,
                           stream, a);
    } else if (plan->spec.ps) {
        hipLaunchKernelGGL(plan->tn_kernel ? e->persist_tn : e->persist, dim3((unsigned)std::min<int64_t>(wgs, cu_count())), dim3(e->threads),
                           e->lds_bytes, stream, a);
    } else if (a.splits > 1 && plan->spec.fr) {
        hipLaunchKernelGGL(plan->tn_kernel ? e->splitk_fused_tn : e->splitk_fused, dim3(wgs, (unsigned)a.splits), dim3(e->threads),
                           e->lds_bytes, stream, a);
    } else if (a.splits > 1) {
        hipLaunchKernelGGL(plan->tn_kernel ? e->splitk_tn : e->splitk, dim3(wgs, (unsigned)a.splits), dim3(e->threads), e->lds_bytes,
                           stream, a);
        if (hipGetLastError() != hipSuccess) return HGEMM_ERR_LAUNCH;
        const int64_t quads = M * (N / 4);
        const int blocks = (int)std::min<int64_t>((quads + 255) / 256, 2048);
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks), dim3(256), 0, stream,
                           (const float*)((const char*)plan->workspace + plan->partial_offset), (_Float16*)C, (int)M, (int)N,
                           (int)plan->lay.ldc, a.splits);
    } else if (plan->spec.ac == 16) {
        hipLaunchKernelGGL(plan->tn_kernel ? e->acc16_tn : e->acc16, dim3(wgs), dim3(e->threads), e->lds_bytes, stream, a);
    } else {
        hipLaunchKernelGGL(plan->tn_kernel ? e->plain_tn : e->plain, dim3(wgs), dim3(e->threads), e->lds_bytes, stream, a);
    }
    return finish();
}

hgemm_status_t hgemm_run(hgemm_plan_t plan, const void* A, const void* B, void* C, void* hip_stream)
{
    if (!plan) return HGEMM_ERR_INVALID_ARG;
    return run_plan(plan, A, B, C, hip_stream);
}

hgemm_status_t hgemm_run_many(hgemm_plan_t plan, int64_t count, int64_t sets, int64_t first, const void* const* A,
                              const void* const* B, void* const* C, void* hip_stream)
{
    if (!plan || count < 0 || sets < 1 || first < 0 || first >= sets || !A || !B || !C) return HGEMM_ERR_INVALID_ARG;
    int64_t set = first;
    for (int64_t i = 0; i < count; ++i) {
        const hgemm_status_t st = run_plan(plan, A[set], B[set], C[set], hip_stream);
        if (st != HGEMM_OK) return st;
        if (++set == sets) set = 0;
    }
    return HGEMM_OK;
}

hgemm_status_t hgemm_run_static(int64_t M, int64_t N, int64_t K, const hgemm_layouts_t* layouts, const void* A, const void* B,
                                void* C, void* hip_stream)
{
    hgemm_plan_s plan;                       // lives on this call's stack; its workspace is the static scratch
    const hgemm_status_t st = init_plan(&plan, M, N, K, layouts, nullptr, true);
    if (st != HGEMM_OK) return st;
    return run_plan(&plan, A, B, C, hip_stream);
}

hgemm_status_t hgemm_destroy(hgemm_plan_t plan)
{
    if (!plan) return HGEMM_OK;
    destroy_blocks(plan);
    if (plan->workspace && !plan->static_ws) {
        if (hipFree(plan->workspace) != hipSuccess) (void)hipGetLastError();
    }
    delete plan;
    return HGEMM_OK;
}

const char* hgemm_status_string(hgemm_status_t status)
{
    switch (status) {
        case HGEMM_OK: return "ok";
        case HGEMM_ERR_INVALID_ARG: return "invalid argument";
        case HGEMM_ERR_UNSUPPORTED: return "unsupported layout, alignment or specialisation";
        case HGEMM_ERR_ALLOC: return "allocation failed";
        case HGEMM_ERR_LAUNCH: return "kernel launch failed";
        case HGEMM_ERR_ARCH: return "device is not gfx950";
        case HGEMM_ERR_WORKSPACE: return "problem needs more scratch than the static buffer holds";
    }
    return "unknown status";
}

hgemm_status_t hgemm_plan_describe(hgemm_plan_t plan, char* buf, size_t n)
{
    if (!plan || !buf || n == 0) return HGEMM_ERR_INVALID_ARG;
    std::string s;
    if (plan->blocked) {
        char head[96];
        snprintf(head, sizeof head, "blocks,rows=%lld,cols=%lld%s: ", (long long)plan->block_m, (long long)plan->block_n, plan->blocked_bt ? ",bt=1" : "");
        const hgemm_plan_s* q = plan->sub[0][0] ? plan->sub[0][0] : plan->sub[1][0] ? plan->sub[1][0] : plan->sub[0][1] ? plan->sub[0][1] : plan->sub[1][1];
        s = std::string(head) + (q ? spec_to_string(q->spec) : std::string("?"));
    } else {
        s = spec_to_string(plan->spec) + (plan->padded ? ",pad=1" : "");
    }
    if (s.size() + 1 > n) { buf[0] = '\0'; return HGEMM_ERR_INVALID_ARG; }
    memcpy(buf, s.c_str(), s.size() + 1);
    return HGEMM_OK;
}

size_t hgemm_plan_workspace_bytes(hgemm_plan_t plan)
{
    if (!plan) return 0;
    size_t bytes = plan->workspace_bytes;
    for (const auto& row : plan->sub)
        for (const hgemm_plan_s* q : row)
            if (q) bytes += q->workspace_bytes;
    return bytes;
}

hgemm_status_t hgemm_plan_launch_info(hgemm_plan_t plan, int64_t* workgroups, int64_t* lds_bytes, int64_t* threads)
{
    if (!plan) return HGEMM_ERR_INVALID_ARG;
    if (plan->blocked) {                     // the figures of the most frequent kind of block
        for (const auto& row : plan->sub)
            for (hgemm_plan_s* q : row)
                if (q) return hgemm_plan_launch_info(q, workgroups, lds_bytes, threads);
        return HGEMM_ERR_INVALID_ARG;
    }
    int64_t wg, lds, th;
    if (plan->skinny) {
        wg = (int64_t)plan->args.tiles_n * plan->args.splits;
        lds = plan->tn_kernel ? plan->spec.wv * (plan->M <= 16 ? 1 : plan->M <= 32 ? 2 : 4) * (plan->spec.nr / 16) * 1024 : 4 * 16 * (kSkinnyCols + 4) * 4;
        th = 64 * plan->spec.wv;
    } else if (plan->entry) {
        wg = plan->spec.sm ? (int64_t)plan->args.dp_tiles + plan->args.sk_workers
                           : (int64_t)plan->args.tiles_m * plan->args.tiles_n * plan->args.splits;
        if (plan->spec.ps) wg = std::min<int64_t>(wg, cu_count());
        lds = plan->entry->lds_bytes;
        th = plan->entry->threads;
    } else {
        wg = ((plan->N + 63) / 64) * ((plan->M + 3) / 4);
        lds = 0;
        th = 256;
    }
    if (workgroups) *workgroups = wg;
    if (lds_bytes) *lds_bytes = lds;
    if (threads) *threads = th;
    return HGEMM_OK;
}

const char* hgemm_spec_help(void)
{
    // built once, inside the initialiser of a function-local static (thread-safe since C++11)
    static const std::string text = [] {
        std::string t =
            "generic\n"
            "    one thread per element, any shape, alignment and layout\n"
            "skinny,sk=SPLITS[,fr=1][,wv=WAVES][,nr=ROWS]\n"
            "    memory-bound kernel for M <= 64 rows of A (row-major B): workgroups of wv = 4 (default), 8 or 16 waves\n"
            "    take 128 columns and a K slab each and stream it in steps of 16 * wv rows; a wave takes 16 rows of a\n"
            "    step, transposes its 4 x 8 blocks in registers for 16x16x16 matrix-core instructions (M on a 16-wide\n"
            "    side; no LDS and no barrier in the main loop), the waves' sums meet once at the end; slabs are summed in\n"
            "    slab order by the split-K reduction launch or, with fr = 1, by the workgroup that arrives last.\n"
            "    Column-major B (K contiguous): a workgroup takes nr = 16 (default), 32 or 64 rows of B (columns of C), its waves split its K\n"
            "    range into contiguous parts of whole 32-k steps, 16-byte loads are the operands of 16x16x32 instructions\n"
            "    as they come; sk splits K further across workgroups\n"
            "mfma,bm=BM,bn=BN,bk=BK,wm=WM,wn=WN,st=STAGES[,pf=PREFETCH][,sk=SPLITS][,gm=GROUP][,tb=1][,sm=1][,fr=1][,ps=1][,ac=16][,mi=16]\n"
            "    pipelined 32x32x16 MFMA kernel; BMxBN tile per workgroup, WMxWN wavefronts, STAGES LDS buffers,\n"
            "    pf = register prefetch distance in k-steps (1 = ping-pong, 3 = four fragment sets),\n"
            "    sk = split-K factor (fp32 partials + ordered reduction), gm = tile-order group height (0 = row-major),\n"
            "    tb = 1: copy row-major B transposed into the workspace first and run the K-contiguous kernel,\n"
            "    fr = 1: with sk > 1, the reduction is fused into the kernel: every workgroup stores its fp32 plane, the one\n"
            "            that arrives last at a tile sums the planes in split order (same bits as the two-launch form)\n"
            "    ps = 1: persistent: one workgroup per compute unit walks tiles wg, wg + grid, ...; the copies of the next\n"
            "            tile's first K-tiles start under the last K-tiles of the current one\n"
            "    sm = 1: stream-K (whole waves of tiles one per workgroup, the remaining tiles' K iterations dealt\n"
            "            evenly to one more workgroup per CU, fp32 partial tiles summed in k order by a second kernel)\n"
            "    ac = 16: 16-bit accumulator: the running sums are rounded to fp16 after every matrix-core instruction\n"
            "            (16 products); explicit specs only, with sk = 1 and without sm, ps, fr; never chosen by hgemm_plan,\n"
            "            which always accumulates in fp32 over all of K\n"
            "    pad = 1 in a description: N, K or a leading dimension is not a multiple of 8 and the kernel runs on\n"
            "            zero-padded packed copies held in the plan's workspace (decided by hgemm_plan from the shape)\n"
            "    compiled (bm,bn,bk,wm,wn,st,pf):";
        for (const MfmaEntry& e : registry()) {
            if (e.deep || e.mi != 32) continue;
            char b[64];
            snprintf(b, sizeof b, " (%d,%d,%d,%d,%d,%d,%d)", e.bm, e.bn, e.bk, e.wm, e.wn, e.st, e.pf);
            t += b;
        }
        t += "\n"
             "    deep-staged, pf longer than a K-tile (bk = 32, pf = 3: fragment reads run up to two K-tiles ahead, st stages of\n"
             "    32 k each keep st - 1 K-tiles of copies in flight); one full-K tile per workgroup only: sk = 1, no sm, ps, fr, ac\n"
             "    deep (bm,bn,bk,wm,wn,st,pf):";
        for (const MfmaEntry& e : registry()) {
            if (!e.deep || e.mi != 32) continue;
            char b[64];
            snprintf(b, sizeof b, " (%d,%d,%d,%d,%d,%d,%d)", e.bm, e.bn, e.bk, e.wm, e.wn, e.st, e.pf);
            t += b;
        }
        t += "\n"
             "    mi = 16: v_mfma_f32_16x16x32_f16 instead of v_mfma_f32_32x32x16_f16 (a k-step is then 32 k); one full-K tile per\n"
             "    workgroup only, like the deep-staged ones\n"
             "    mi16 (bm,bn,bk,wm,wn,st,pf):";
        for (const MfmaEntry& e : registry()) {
            if (e.mi != 16) continue;
            char b[64];
            snprintf(b, sizeof b, " (%d,%d,%d,%d,%d,%d,%d)", e.bm, e.bn, e.bk, e.wm, e.wn, e.st, e.pf);
            t += b;
        }
        t += "\n";
        return t;
    }();
    return text.c_str();
}

hgemm_status_t hgemm_candidates(int64_t M, int64_t N, int64_t K, const hgemm_layouts_t* layouts, char* buf, size_t n)
{
    if (!buf || n == 0 || M < 0 || N < 0 || K < 0) return HGEMM_ERR_INVALID_ARG;
    hgemm_layouts_t l;
    if (layouts) l = *layouts; else { l.a = l.b = l.c = HGEMM_ROW_MAJOR; l.lda = l.ldb = l.ldc = 0; }
    if (l.lda == 0) l.lda = K;
    if (l.ldb == 0) l.ldb = (l.b == HGEMM_ROW_MAJOR) ? N : K;
    if (l.ldc == 0) l.ldc = N;
    std::string out;
    if (!fast_path_ok(M, N, K, l) || M == 0 || N == 0 || K == 0) {
        out = "generic\n";
    } else {
        const int64_t CUS = cu_count();
        if (l.b == HGEMM_ROW_MAJOR && M <= kSkinnyMaxM) {       // few rows: the streaming family competes
            for (int eff : skinny_split_candidates(N, K)) {
                for (int fr = 0; fr <= ((eff > 1 && fused_delta_us(M, N, eff) < 1.0) ? 1 : 0); ++fr) {
                    for (int wv : {4, 8, 16}) {
                        if (wv == 16 && M > 32) continue;
                        Spec s;
                        s.fam = FAM_SKINNY; s.sk = (int)eff; s.fr = fr; s.wv = wv;
                        if (effective_splits((K + skinny_step(s) - 1) / skinny_step(s), eff) != eff) continue;
                        out += spec_to_string(s);
                        out += "\n";
                    }
                }
            }
        }
        if (l.b == HGEMM_COL_MAJOR && M <= kSkinnyMaxM) {       // the streaming family for K-contiguous B: N / 16 workgroups before any split
            const int mblocks = M <= 16 ? 1 : M <= 32 ? 2 : 4;
            for (int nr : {16, 32, 64})
                for (int wv : {4, 8, 16}) {
                    const int blocks = mblocks * (nr / 16);
                    if (wv * blocks > 64 || (wv == 16 && blocks > 4)) continue;       // kernels that do not exist
                    if (nr > 16 && (N + nr - 1) / nr < CUS / 2) continue;             // too few workgroups to be worth timing
                    int64_t last = 0;
                    for (int sk : {1, 2, 4, 8, 16}) {
                        Spec s;
                        s.fam = FAM_SKINNY; s.wv = wv; s.nr = nr;
                        const int64_t eff = effective_splits((K + skinny_step(s, true) - 1) / skinny_step(s, true), sk);
                        if (eff == last || ((N + nr - 1) / nr) * eff > 64 * CUS) continue;
                        last = eff;
                        for (int fr = 0; fr <= (eff > 1 ? 1 : 0); ++fr) {
                            s.sk = (int)eff; s.fr = fr;
                            out += spec_to_string(s);
                            out += "\n";
                        }
                    }
                }
        }
        for (const MfmaEntry& e : registry()) {
            if (!tile_fits_problem(e, M, N)) continue;
            const int64_t t = ((M + e.bm - 1) / e.bm) * ((N + e.bn - 1) / e.bn);
            const int64_t ktiles = (K + e.bk - 1) / e.bk;
            if (e.deep) {                                       // one full-K tile per workgroup; worth timing once the chip is full
                if (t < CUS / 2 || ktiles < 2 * e.st) continue;
                for (int gm : {8, 0, 4, 16}) {
                    if (gm != 8 && (t < 2 * CUS)) continue;
                    Spec s;
                    s.fam = FAM_MFMA; s.bm = e.bm; s.bn = e.bn; s.bk = e.bk; s.wm = e.wm; s.wn = e.wn; s.st = e.st; s.pf = e.pf; s.mi = e.mi; s.sk = 1; s.gm = gm;
                    out += spec_to_string(s);
                    out += "\n";
                }
                continue;
            }
            const std::vector<int> sks = split_candidates(t, ktiles);
            if (t % CUS != 0 && ktiles >= 4 && e.bm >= 64 && e.bn >= 64) {
                Spec s;
                s.fam = FAM_MFMA; s.bm = e.bm; s.bn = e.bn; s.bk = e.bk; s.wm = e.wm; s.wn = e.wn; s.st = e.st; s.pf = e.pf; s.mi = e.mi; s.sk = 1; s.gm = 8; s.sm = 1;
                out += spec_to_string(s);
                out += "\n";
            }
            for (int sk : sks) {
                for (int gm : {8, 0, 4, 16}) {
                    if (gm != 8 && (t < 2 * CUS)) continue;      // order matters only when tiles outnumber CUs
                    Spec s;
                    s.fam = FAM_MFMA; s.bm = e.bm; s.bn = e.bn; s.bk = e.bk; s.wm = e.wm; s.wn = e.wn; s.st = e.st; s.pf = e.pf; s.mi = e.mi; s.sk = sk; s.gm = gm;
                    out += spec_to_string(s);
                    out += "\n";
                    if (sk == 1 && gm == 8 && e.persist && t > CUS && ktiles >= e.st) {      // the same tiles walked by persistent workgroups
                        s.ps = 1;
                        out += spec_to_string(s);
                        out += "\n";
                        s.ps = 0;
                    }
                    if (sk > 1 && gm == 8 && fused_delta_us(M, N, sk) < 1.0) {   // the same split with the reduction fused into the kernel
                        s.fr = 1;
                        out += spec_to_string(s);
                        out += "\n";
                        s.fr = 0;
                    }
                    // row-major B, tall problem: paying one transposing copy of B can be cheaper than
                    // transposing reads in every workgroup
                    if (l.b == HGEMM_ROW_MAJOR && gm == 8 && M >= 1024 && e.bm >= 128 && e.bn >= 128) {
                        s.tb = 1;
                        out += spec_to_string(s);
                        out += "\n";
                    }
                }
            }
        }
    }
    if (out.size() + 1 > n) { buf[0] = '\0'; return HGEMM_ERR_INVALID_ARG; }
    memcpy(buf, out.c_str(), out.size() + 1);
    return HGEMM_OK;
}

hgemm_status_t hgemm_predict_us(int64_t M, int64_t N, int64_t K, const char* spec, double* us)
{
    if (!spec || !us || M <= 0 || N <= 0 || K <= 0) return HGEMM_ERR_INVALID_ARG;
    Spec s;
    if (!parse_spec(spec, &s)) return HGEMM_ERR_INVALID_ARG;
    if (s.fam == FAM_SKINNY) {
        if (M > kSkinnyMaxM) return HGEMM_ERR_UNSUPPORTED;
        const int64_t eff = effective_splits((K + skinny_step(s) - 1) / skinny_step(s), s.sk);
        *us = predict_skinny_us(M, N, K, eff, s.fr != 0 && eff > 1);
        return HGEMM_OK;
    }
    if (s.fam != FAM_MFMA || s.sm || s.tb || s.ps || s.ac == 16 || !find_entry(s)) return HGEMM_ERR_UNSUPPORTED;
    const int64_t eff = effective_splits((K + s.bk - 1) / s.bk, s.sk);
    *us = predict_us(M, N, K, s.bm, s.bn, s.bk, s.wm, s.wn, s.st, s.pf, eff);
    if (s.fr && eff > 1) *us += fused_delta_us(M, N, eff);
    return HGEMM_OK;
}

int64_t hgemm_tiles(int64_t dim, int64_t tile) { return (dim < 0 || tile <= 0) ? -1 : (dim + tile - 1) / tile; }
int64_t hgemm_padded(int64_t dim, int64_t tile) { return (dim < 0 || tile <= 0) ? -1 : ((dim + tile - 1) / tile) * tile; }

int64_t hgemm_tile_of_workgroup(int64_t wg, int64_t tiles_m, int64_t tiles_n, int64_t swizzle)
{
    if (tiles_m <= 0 || tiles_n <= 0 || wg < 0 || wg >= tiles_m * tiles_n || swizzle < 0) return -1;
    const int64_t tile = tile_of_workgroup(wg, tiles_m, tiles_n, swizzle);
    // the kernels use the multiplication form of the same map: report a disagreement instead of hiding it
    if (tiles_m * tiles_n < ((int64_t)1 << 24)) {
        GemmArgs a{};
        a.tiles_m = (int)tiles_m;
        a.tiles_n = (int)tiles_n;
        a.swizzle = (int)std::min<int64_t>(swizzle, tiles_m);
        set_tile_map(a);
        unsigned tm = 0, tn = 0;
        tile_coords((unsigned)wg, a, tm, tn);
        if ((int64_t)tm * tiles_n + tn != tile) return -2;
    }
    return tile;
}

hgemm_status_t hgemm_calibrate_mfma(int64_t iters, void* hip_stream, double* ms, double* flop)
{
    if (!ms || !flop || iters <= 0 || iters > (1 << 24)) return HGEMM_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return HGEMM_ERR_ARCH; }
    float* out = nullptr;
    if (hipMalloc(&out, 4) != hipSuccess) { (void)hipGetLastError(); return HGEMM_ERR_ALLOC; }
    hipEvent_t e0, e1;
    hipEventCreate(&e0);
    hipEventCreate(&e1);
    const int blocks = prop.multiProcessorCount * 2;
    hipLaunchKernelGGL(calib_mfma_kernel, dim3(blocks), dim3(256), 0, stream, out, (int)iters);   // warm-up
    hipEventRecord(e0, stream);
    hipLaunchKernelGGL(calib_mfma_kernel, dim3(blocks), dim3(256), 0, stream, out, (int)iters);
    hipEventRecord(e1, stream);
    hipError_t err = hipEventSynchronize(e1);
    float t = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&t, e0, e1);
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    hipFree(out);
    if (err != hipSuccess) { (void)hipGetLastError(); return HGEMM_ERR_LAUNCH; }
    *ms = t;
    *flop = (double)blocks * 4.0 * (double)iters * 4.0 * 32768.0;    // 4 waves x 4 MFMAs of 32*32*16*2 flop
    return HGEMM_OK;
}

hgemm_status_t hgemm_calibrate_hbm_read(const void* src, size_t bytes, void* hip_stream, double* ms)
{
    if (!src || !ms || bytes < 16 || (((uintptr_t)src) & 15)) return HGEMM_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return HGEMM_ERR_ARCH; }
    uint32_t* out = nullptr;
    if (hipMalloc(&out, 4) != hipSuccess) { (void)hipGetLastError(); return HGEMM_ERR_ALLOC; }
    hipEvent_t e0, e1;
    hipEventCreate(&e0);
    hipEventCreate(&e1);
    const int blocks = prop.multiProcessorCount * 8;
    hipEventRecord(e0, stream);
    hipLaunchKernelGGL(calib_read_kernel, dim3(blocks), dim3(256), 0, stream, (const uint4*)src, bytes / 16, out);
    hipEventRecord(e1, stream);
    hipError_t err = hipEventSynchronize(e1);
    float t = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&t, e0, e1);
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    hipFree(out);
    if (err != hipSuccess) { (void)hipGetLastError(); return HGEMM_ERR_LAUNCH; }
    *ms = t;
    return HGEMM_OK;
}

}  // extern "C"
