// C ABI of the gfx950 GEMM library: argument checks, variant selection
// (the tuning/execution parameters of the paper's Section 3.1), launches.
#include "../../include/peak_gemm.h"

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include <dlfcn.h>

#include <mutex>
#include <string>

#include "gemm_device.h"
#include "skinny_device.h"
#include "variant.h"

namespace peak {

constexpr int LDS_LIMIT = 160 * 1024; // bytes per workgroup on gfx950

// The variant table: the groups of the other translation units, joined in a fixed order.
static const std::vector<Variant> &variants()
{
    static const std::vector<Variant> table = [] {
        std::vector<Variant> t;
        const VariantGroup groups[] = {variants_general(), variants_bf16_nt(), variants_f16_nt(), variants_bf16_nn(),
                                       variants_f16_nn(),  variants_f32(),     variants_ta(),     variants_skinny(),
                                       variants_mf16()};
        for (const VariantGroup &g : groups) t.insert(t.end(), g.rows, g.rows + g.count);
        return t;
    }();
    return table;
}
#define g_variants (variants())
#define NUM_VARIANTS ((int)variants().size())

// Compute units of the device the plans are made for: PEAK_GEMM_NUM_CU, else the
// current device's count, else (no device visible) that of the MI355X.
static int num_cu()
{
    static const int n = [] {
        if (const char *e = getenv("PEAK_GEMM_NUM_CU")) {
            const int v = atoi(e);
            if (v >= 1 && v <= 4096) return v;
        }
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            return v;
        (void)hipGetLastError();
        return 256;
    }();
    return n;
}

}  // namespace peak

using namespace peak;

// Grid and K split of one variant for the plan's problem.
struct Geometry {
    int variant;          // index into the variant table, -1: nothing to launch
    int tiles_m, tiles_n, split, ktiles_total, ktiles_per_slice, group_m, rot_m, rot_n;
    int sk_tiles;         // hybrid stream-K: tiles of the last, partial round that are cut into `split` K slices; 0: off
    size_t ws_bytes;
};

struct peak_gemm_plan {
    peak_gemm_desc_t d;
    Geometry g;           // the selected variant
    Geometry alt;         // register-staged stand-in for runs whose A or B base is not 16-byte aligned
                          // (variant -1 when the selected variant has no alignment needs)
    size_t ws_bytes;      // the larger of the two workspaces
};

static int esize_of(int dt) { return dt == PEAK_DT_F32 ? 4 : 2; }

static bool variant_fits(const Variant &v, const peak_gemm_desc_t &d)
{
    if (v.dt != d.dtype) return false;
    if (v.lds > LDS_LIMIT) return false;
    // layouts: kernel's A_T means A does not run along K, i.e. transA == 1;
    // kernel's B_T means B stored K x N, i.e. transB == 0
    const int a_t = d.transA ? 1 : 0, b_t = d.transB ? 0 : 1;
    if (v.a_t != a_t || v.b_t != b_t) return false;
    if (v.kind != KIND_TILED && d.M > v.max_m) return false;
    if (v.direct) {
        const int es = esize_of(d.dtype);
        const bool a_along_k = !v.a_t, b_along_k = !v.b_t;      // copied in 16-byte chunks along K
        if (v.kind == KIND_TILED) {
            // K may stop inside the last K tile: at a 16-byte chunk boundary for an operand that
            // runs along K, anywhere for one staged as [k][.] rows
            if ((a_along_k || b_along_k) && (d.K * es) % 16 != 0) return false;
            if (v.tr && (d.N * es) % 16 != 0) return false;
            if (v.atr && (d.M * es) % 16 != 0) return false;
        } else if (d.K % v.bk != 0 || d.K < v.bk) {
            return false;
        }
        if ((d.lda * es) % 16 != 0 || (d.ldb * es) % 16 != 0) return false;
        // a workgroup's operand panel is addressed with 32-bit byte offsets
        const int64_t lim = (int64_t)1 << 31;
        if (v.atr ? ((d.K - 1) * d.lda + d.M) * es >= lim : a_along_k && ((int64_t)(v.bm - 1) * d.lda + d.K) * es >= lim) return false;
        if (v.tr ? ((d.K - 1) * d.ldb + d.N) * es >= lim : b_along_k && ((int64_t)(v.bn - 1) * d.ldb + d.K) * es >= lim) return false;
    }
    return true;
}

static int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Estimated time of a tiled variant, in units of "one 32x32xBK-row MFMA group":
// rounds of workgroups over the CUs times the work of one tile.  Used only to
// rank variants; the measured sweep decides the constants.
static double tiled_cost(const Variant &v, const peak_gemm_desc_t &d, int split)
{
    const int64_t tiles = cdiv(d.M, v.bm) * cdiv(d.N, v.bn) * split;
    const int64_t rounds = cdiv(tiles, num_cu());
    const double ktiles = (double)cdiv(cdiv(d.K, v.bk), split);
    // one unit = one multiply-add at the 16-bit MFMA rate; an fp32 one takes 16 of them (2500 vs 157 TFLOP/s)
    const double tile_work = (double)v.bm * v.bn * v.bk * ktiles * (v.dt == DT_F32 ? 16.0 : 1.0);
    // small tiles pay more LDS/L2 traffic per flop; direct loads overlap better.
    // The constants come from the measured sweeps on the graded shapes.
    double eff = 1.0;
    if (v.dt == DT_F32) {                               // fp32 MFMA is slow enough that tile size hardly matters
        if (v.bm * v.bn >= 256 * 256) eff = 0.90;       // 128x128 per wave: a quarter of the LDS traffic of 64x64 wave tiles
        else if (v.bm * v.bn >= 256 * 128) eff = 0.86;
        else if (v.bm * v.bn >= 128 * 128) eff = 0.95;
        else if (v.bm * v.bn >= 128 * 64) eff = 0.8;    // as good per multiply-add as 128x128 while few workgroups run
        else eff = 0.5;
    } else {
        if (v.bm * v.bn >= 256 * 256) eff = 1.0;
        else if (v.bm * v.bn >= 256 * 128) eff = 0.85;
        else if (v.bm * v.bn >= 128 * 128) eff = 0.85;   // 64 KB of LDS: two workgroups share a CU
        else if (v.bm * v.bn >= 128 * 64 && v.direct) eff = 0.7;   // 48 KB: three; ahead while the tiles are few
        else eff = 0.3;
    }
    if (!v.direct) eff *= 0.7;
    if (v.tr) eff *= v.dt == DT_F32 ? 1.10 : 1.03;      // B staged directly: no register transposition, no masked loads
    if (v.lds > 140 * 1024 && v.ns == 2 && !v.tr) eff *= 1.02;   // third A stage, A's loads spread over the step (+2 % measured; nothing with [k][n] B)
    if (v.nt == 256 && v.bm == 256 && v.bn == 256 && v.lds > 140 * 1024) eff *= 1.02;   // one wave per SIMD on top of that
    if (v.mf16) eff *= 1.10;                            // 16x16x32 MFMA: same cycles, higher clock (+10 % measured)
    if (v.atr) eff *= 1.5;                              // likewise A; the alternative is the register-staged general tile
    if (v.dt == DT_F32 && v.ns == 3) eff *= 0.97;
    const double fixed = 12.0e6;                    // prologue + epilogue of one tile, same units
    // K slices write and re-read fp32 partials: about 9 units per element and slice when they go
    // through HBM, half of that while the workspace stays in the last-level cache
    const double ws_bytes = 4.0 * (double)split * (double)d.M * (double)d.N;
    // ... plus the launch of the reduction kernel (about 3 us)
    const double reduce = split > 1 ? (ws_bytes <= 64.0e6 ? 4.5 : 9.0) * (double)split * (double)d.M * (double)d.N + 8.0e6 : 0.0;
    return rounds * (tile_work / eff + fixed) + reduce;
}

static int choose_split(const Variant &v, const peak_gemm_desc_t &d)
{
    const int64_t tiles = cdiv(d.M, v.bm) * cdiv(d.N, v.bn);
    const int64_t ktiles = cdiv(d.K, v.bk);
    if (tiles > num_cu() / 2 || ktiles < 4) return 1;
    int best = 1;
    double best_cost = tiled_cost(v, d, 1);
    for (int s = 2; s <= 16; ++s) {
        if (ktiles / s < 2) break;
        const double c = tiled_cost(v, d, s);
        if (c < best_cost * 0.95) { best_cost = c; best = s; }
    }
    return best;
}

// Hybrid stream-K (the paper's Split-K of Section 4.1, Table 2, applied to the last round only):
// with T tiles on P compute units the last round holds T mod P tiles and leaves the other units
// idle for a whole tile's time.  Those tiles are cut into S = floor(P / (T mod P)) K slices each,
// so the round takes a slice's time plus the ordered sum of the partial tiles.  Returns S (0: not
// applicable or not worth it by the cost model); *sk_tiles receives T mod P.
static int streamk_split(const Variant &v, const peak_gemm_desc_t &d, int *sk_tiles)
{
    *sk_tiles = 0;
    if (!v.mf16) return 0;                                   // built into the 16x16x32 kernels only
    const int64_t tiles = cdiv(d.M, v.bm) * cdiv(d.N, v.bn), P = num_cu();
    const int64_t rem = tiles % P, ktiles = cdiv(d.K, v.bk);
    if (tiles < P || rem == 0) return 0;
    int64_t S = P / rem;
    if (S > ktiles / 4) S = ktiles / 4;                      // at least four K tiles per slice
    if (S > 255) S = 255;
    if (S < 2) return 0;
    *sk_tiles = (int)rem;
    return (int)S;
}

// cost-model estimate, in the units of tiled_cost: is the cut round cheaper than a whole one?
static bool streamk_pays(const Variant &v, const peak_gemm_desc_t &d, int S, int sk_tiles)
{
    const double tile = (double)v.bm * v.bn * v.bk * (double)cdiv(d.K, v.bk);
    const double fixed = 12.0e6;
    const double partials = (double)S * sk_tiles * v.bm * v.bn;
    const double cut = tile / S + fixed + (4.0 * partials <= 64.0e6 ? 4.5 : 9.0) * partials + 8.0e6;
    return cut < 0.9 * (tile + fixed);
}

// streamk: 1 take hybrid stream-K wherever it applies, -1 never, 0 let the cost model decide
static void plan_geometry(Geometry *p, const peak_gemm_desc_t &d, int variant, int forced_split, int streamk = 0)
{
    const Variant &v = g_variants[variant];
    p->variant = variant;
    p->sk_tiles = 0;
    p->tiles_m = (int)cdiv(d.M, v.bm);
    p->tiles_n = (int)cdiv(d.N, v.bn);
    p->ktiles_total = (int)cdiv(d.K, v.bk);
    int split = forced_split > 0 ? forced_split
              : v.kind == KIND_SKINNY     ? skinny_split(d.N, d.K, v.bn, v.bk)
              : v.kind == KIND_SKINNY_REG ? skinny_reg_split(d.N, d.K)
                                          : choose_split(v, d);
    if (split > p->ktiles_total) split = p->ktiles_total;
    if (split < 1) split = 1;
    p->ktiles_per_slice = (int)cdiv(p->ktiles_total, split);
    p->split = (int)cdiv(p->ktiles_total, p->ktiles_per_slice);   // no empty slices
    p->group_m = p->tiles_m >= 8 ? 8 : (p->tiles_m > 0 ? p->tiles_m : 1);
    p->rot_m = 0;                                           // K rotation off for the tiled kernels: measured no gain on the graded shapes
    p->rot_n = v.kind == KIND_SKINNY ? 5 : 0;               // streaming kernel: neighbouring workgroups start five K tiles apart
                                                            // (bf16 16x16384x16384: 5.3 TB/s without, 6.0 with 1, 6.2 with 5 or 13)
    if (const char *e = getenv("PEAK_GEMM_GROUP_M")) {      // tuning knob: tile rows per band
        const int g = atoi(e);
        if (g >= 1 && g <= 64) p->group_m = g < p->tiles_m ? g : (p->tiles_m > 0 ? p->tiles_m : 1);
    }
    if (const char *e = getenv("PEAK_GEMM_ROT")) {          // tuning knob: "rot_m,rot_n"
        int a = 0, b = 0;
        if (sscanf(e, "%d,%d", &a, &b) == 2 && a >= 0 && b >= 0) { p->rot_m = a; p->rot_n = b; }
    }
    p->ws_bytes = p->split > 1 ? (size_t)p->split * (size_t)d.M * (size_t)d.N * sizeof(float) : 0;
    // hybrid stream-K where nothing forces a K split: PEAK_GEMM_STREAMK_ON / _OFF decide, else the cost model
    if (forced_split <= 0 && p->split == 1 && streamk >= 0) {
        int sk_tiles = 0;
        const int S = streamk_split(v, d, &sk_tiles);
        if (S >= 2 && (streamk > 0 || streamk_pays(v, d, S, sk_tiles))) {
            p->ktiles_per_slice = (int)cdiv(p->ktiles_total, S);
            p->split = (int)cdiv(p->ktiles_total, p->ktiles_per_slice);
            p->sk_tiles = sk_tiles;
            p->ws_bytes = (size_t)p->split * (size_t)sk_tiles * (size_t)v.bm * v.bn * sizeof(float);
        }
    }
}

// The selector's own choice among the variants that fit (cost model); with
// `staged_only`, among those that take any operand alignment.
static int select_variant(const peak_gemm_desc_t &d, bool staged_only)
{
    double best = 0.0;
    int pick = -1, second_stream = -1;
    for (int i = 0; i < NUM_VARIANTS; ++i) {
        const Variant &v = g_variants[i];
        if (v.sweep_only || (staged_only && v.direct) || !variant_fits(v, d)) continue;
        if (v.kind != KIND_TILED) {
            // a streaming kernel wins whenever it applies
            if (v.stream_rank == 2) return i;
            if (v.stream_rank == 1 && second_stream < 0) second_stream = i;
            continue;
        }
        const double c = tiled_cost(v, d, choose_split(v, d));
        if (pick < 0 || c < best) { pick = i; best = c; }
    }
    return second_stream >= 0 ? second_stream : pick;
}

// Selector table from an offline sweep: exact shape -> variant and K split.
struct TuneEntry {
    int dt, ta, tb;
    int64_t M, N, K;
    int variant, split;
};
static std::vector<TuneEntry> g_tuning;
static bool g_tuning_env_done = false;

static int variant_by_name(const char *name)
{
    for (int i = 0; i < NUM_VARIANTS; ++i)
        if (strcmp(g_variants[i].name, name) == 0) return i;
    return -1;
}

static int load_tuning_file(const char *path)
{
    FILE *f = fopen(path, "r");
    if (!f) return -1;
    std::vector<TuneEntry> table;
    char line[512];
    bool ok = true;
    while (ok && fgets(line, sizeof line, f)) {
        char *hash = strchr(line, '#');
        if (hash) *hash = 0;
        char dt[16], name[128];
        TuneEntry e;
        long long M, N, K;
        const int n = sscanf(line, "%15s %d %d %lld %lld %lld %127s %d", dt, &e.ta, &e.tb, &M, &N, &K, name, &e.split);
        if (n <= 0) continue;                               // blank or comment line
        e.dt = strcmp(dt, "f32") == 0 ? PEAK_DT_F32 : strcmp(dt, "f16") == 0 ? PEAK_DT_F16 : strcmp(dt, "bf16") == 0 ? PEAK_DT_BF16 : -1;
        e.variant = n >= 7 ? variant_by_name(name) : -1;
        e.M = M; e.N = N; e.K = K;
        ok = n == 8 && e.dt >= 0 && e.variant >= 0 && (e.ta | 1) == 1 && (e.tb | 1) == 1 && M > 0 && N > 0 && K > 0 &&
             e.split >= 0 && e.split <= 255 && g_variants[e.variant].dt == e.dt;
        if (ok) table.push_back(e);
    }
    fclose(f);
    if (!ok) return -1;
    g_tuning.swap(table);
    return (int)g_tuning.size();
}

// The table that ships with the library: peak_gemm_tuning.txt beside the shared object.
static std::string shipped_table_path()
{
    Dl_info info;
    if (!dladdr((const void *)&peak_gemm_variant_count, &info) || !info.dli_fname) return std::string();
    std::string path(info.dli_fname);
    const size_t slash = path.rfind('/');
    path = slash == std::string::npos ? std::string() : path.substr(0, slash + 1);
    return path + "peak_gemm_tuning.txt";
}

static const TuneEntry *tuned(const peak_gemm_desc_t &d)
{
    if (!g_tuning_env_done) {
        g_tuning_env_done = true;
        // PEAK_GEMM_TUNING names another table; set to the empty string it turns the shipped one off
        if (const char *e = getenv("PEAK_GEMM_TUNING")) {
            if (*e) load_tuning_file(e);
        } else {
            const std::string path = shipped_table_path();
            if (!path.empty()) load_tuning_file(path.c_str());
        }
    }
    for (const TuneEntry &e : g_tuning)
        if (e.dt == (int)d.dtype && e.ta == d.transA && e.tb == d.transB && e.M == d.M && e.N == d.N && e.K == d.K &&
            variant_fits(g_variants[e.variant], d))
            return &e;
    return nullptr;
}

extern "C" {

int peak_gemm_load_tuning(const char *path)
{
    g_tuning_env_done = true;                               // an explicit call overrides the environment
    if (!path) {
        g_tuning.clear();
        return 0;
    }
    return load_tuning_file(path);
}

const char *peak_status_string(peak_status_t s)
{
    switch (s) {
    case PEAK_OK: return "ok";
    case PEAK_ERR_INVALID_ARG: return "invalid argument";
    case PEAK_ERR_UNSUPPORTED: return "no kernel variant supports this problem";
    case PEAK_ERR_WORKSPACE: return "workspace missing or too small";
    case PEAK_ERR_HIP: return "HIP runtime error at launch";
    case PEAK_ERR_ALLOC: return "host allocation failed";
    }
    return "unknown status";
}

int peak_gemm_variant_count(void) { return NUM_VARIANTS; }

const char *peak_gemm_variant_name(int id)
{
    if (id < 0 || id >= NUM_VARIANTS) return nullptr;
    return g_variants[id].name;
}

peak_status_t peak_gemm_create(const peak_gemm_desc_t *desc, peak_gemm_plan_t **out_plan)
{
    if (out_plan) *out_plan = nullptr;
    if (!desc || !out_plan) return PEAK_ERR_INVALID_ARG;
    const peak_gemm_desc_t &d = *desc;
    if (d.M < 0 || d.N < 0 || d.K < 0) return PEAK_ERR_INVALID_ARG;
    if (d.dtype != PEAK_DT_F32 && d.dtype != PEAK_DT_F16 && d.dtype != PEAK_DT_BF16) return PEAK_ERR_INVALID_ARG;
    if ((d.transA != 0 && d.transA != 1) || (d.transB != 0 && d.transB != 1)) return PEAK_ERR_INVALID_ARG;
    if (d.flags & ~(0xFFFFu | PEAK_GEMM_C_F32 | PEAK_GEMM_STREAMK_ON | PEAK_GEMM_STREAMK_OFF)) return PEAK_ERR_INVALID_ARG;
    if ((d.flags & PEAK_GEMM_STREAMK_ON) && (d.flags & PEAK_GEMM_STREAMK_OFF)) return PEAK_ERR_INVALID_ARG;
    const int64_t min_lda = d.transA ? d.M : d.K, min_ldb = d.transB ? d.K : d.N;
    if (d.lda < (min_lda > 1 ? min_lda : 1) || d.ldb < (min_ldb > 1 ? min_ldb : 1) || d.ldc < (d.N > 1 ? d.N : 1))
        return PEAK_ERR_INVALID_ARG;
    // index arithmetic is 64-bit, but tile counts and the grid are 32-bit
    if (d.M > (int64_t)1 << 30 || d.N > (int64_t)1 << 30 || d.K > (int64_t)1 << 30) return PEAK_ERR_UNSUPPORTED;

    peak_gemm_plan *p = new (std::nothrow) peak_gemm_plan;
    if (!p) return PEAK_ERR_ALLOC;
    memset(p, 0, sizeof *p);
    p->d = d;
    p->g.variant = p->alt.variant = -1;
    p->g.split = p->alt.split = 1;

    const int forced = (int)(d.flags & 0xFF) - 1;
    const int forced_split = (int)((d.flags >> 8) & 0xFF);

    if (d.M == 0 || d.N == 0 || d.K == 0) {           // nothing to multiply; run() scales C or does nothing
        if (forced >= 0 && (forced >= NUM_VARIANTS || g_variants[forced].dt != d.dtype)) {
            delete p;
            return PEAK_ERR_UNSUPPORTED;
        }
        *out_plan = p;
        return PEAK_OK;
    }

    int pick = -1;
    int table_split = 0;
    if (forced >= 0) {
        if (forced >= NUM_VARIANTS || !variant_fits(g_variants[forced], d)) {
            delete p;
            return PEAK_ERR_UNSUPPORTED;
        }
        pick = forced;
    } else if (const TuneEntry *t = tuned(d)) {
        pick = t->variant;
        table_split = t->split > 0 ? t->split : -1;
    } else {
        pick = select_variant(d, false);
        if (pick < 0) {
            delete p;
            return PEAK_ERR_UNSUPPORTED;
        }
    }
    // a table entry with split 0 stands for hybrid stream-K
    int streamk = (d.flags & PEAK_GEMM_STREAMK_ON) ? 1 : (d.flags & PEAK_GEMM_STREAMK_OFF) ? -1 : 0;
    if (forced_split <= 0 && streamk == 0 && table_split < 0) streamk = 1;
    plan_geometry(&p->g, d, pick, forced_split > 0 ? forced_split : (table_split > 0 ? table_split : 0), streamk);
    // Leading dimensions are known here, base addresses only at run time: a variant that copies
    // 16-byte chunks gets a register-staged stand-in for runs whose A or B base is off that alignment
    if (g_variants[pick].direct) {
        const int alt = select_variant(d, true);
        if (alt >= 0) plan_geometry(&p->alt, d, alt, forced_split);
    }
    p->ws_bytes = p->g.ws_bytes > p->alt.ws_bytes ? p->g.ws_bytes : p->alt.ws_bytes;
    const int64_t grid = (int64_t)p->g.tiles_m * p->g.tiles_n * p->g.split;   // (an upper bound for a stream-K plan)
    const int64_t grid_alt = p->alt.variant < 0 ? 0 : (int64_t)p->alt.tiles_m * p->alt.tiles_n * p->alt.split;
    if (grid > 0x7FFFFFFF || grid_alt > 0x7FFFFFFF) {
        delete p;
        return PEAK_ERR_UNSUPPORTED;
    }
    *out_plan = p;
    return PEAK_OK;
}

size_t peak_gemm_workspace_bytes(const peak_gemm_plan_t *plan) { return plan ? plan->ws_bytes : 0; }

// workgroups of the GEMM launch
static int64_t grid_blocks(const Geometry &g)
{
    const int64_t tiles = (int64_t)g.tiles_m * g.tiles_n;
    return g.sk_tiles ? tiles - g.sk_tiles + (int64_t)g.sk_tiles * g.split : tiles * g.split;
}

int peak_gemm_plan_info(const peak_gemm_plan_t *p, char *buf, size_t n)
{
    if (!p) return snprintf(buf, n, "null plan");
    if (p->g.variant < 0)
        return snprintf(buf, n, "variant=none (degenerate size) M=%lld N=%lld K=%lld", (long long)p->d.M,
                        (long long)p->d.N, (long long)p->d.K);
    const Geometry &g = p->g;
    const Variant &v = g_variants[g.variant];
    return snprintf(buf, n,
                    "variant=%d:%s tile=%dx%dx%d threads=%d stages=%d lds=%d split=%d ktiles/slice=%d "
                    "grid=%lld (tiles %dx%d) group_m=%d workspace=%zu unaligned=%s streamk=%d",
                    g.variant, v.name, v.bm, v.bn, v.bk, v.nt, v.ns, v.lds, g.split, g.ktiles_per_slice,
                    (long long)grid_blocks(g), g.tiles_m, g.tiles_n, g.group_m, p->ws_bytes,
                    p->alt.variant >= 0 ? g_variants[p->alt.variant].name : "same", g.sk_tiles);
}

static peak_status_t run_plan(peak_gemm_plan_t *p, float alpha, const void *A, const void *B, float beta, void *C,
                              const Hook &hook, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!p) return PEAK_ERR_INVALID_ARG;
    const peak_gemm_desc_t &d = p->d;
    if (d.M == 0 || d.N == 0) return PEAK_OK;
    if (!C) return PEAK_ERR_INVALID_ARG;
    const int es = esize_of(d.dtype);
    const int c_dt = (d.flags & PEAK_GEMM_C_F32) ? PEAK_DT_F32 : d.dtype;      // storage type of C
    const int es_c = esize_of(c_dt);
    if ((uintptr_t)C % es_c) return PEAK_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;

    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.A = A; a.B = B; a.C = C; a.ws = nullptr;
    a.M = d.M; a.N = d.N; a.K = d.K;
    a.lda = d.lda; a.ldb = d.ldb; a.ldc = d.ldc;
    a.alpha = alpha; a.beta = beta;
    a.hook = hook;
    a.split = 1;
    if ((uintptr_t)C % (4 * es_c) == 0 && (d.ldc * es_c) % (4 * es_c) == 0) a.flags |= GF_C_VEC;
    if ((uintptr_t)C % 16 == 0 && (d.ldc * es_c) % 16 == 0) a.flags |= GF_C_VEC16;
    if (c_dt != d.dtype) a.flags |= GF_C_F32;

    const bool no_product = (d.K == 0 || alpha == 0.0f);
    if (no_product) {
        if (beta == 1.0f && !(hook.bias_kind | hook.act)) return PEAK_OK;
        const int64_t blocks = cdiv(d.M * d.N, 256);
        if (blocks > 0x7FFFFFFF) return PEAK_ERR_UNSUPPORTED;
        dim3 grid((unsigned)blocks);
        if (c_dt == PEAK_DT_F32) hipLaunchKernelGGL(scale_c_kernel<DT_F32>, grid, dim3(256), 0, stream, a);
        else if (c_dt == PEAK_DT_F16) hipLaunchKernelGGL(scale_c_kernel<DT_F16>, grid, dim3(256), 0, stream, a);
        else hipLaunchKernelGGL(scale_c_kernel<DT_BF16>, grid, dim3(256), 0, stream, a);
        return hipGetLastError() == hipSuccess ? PEAK_OK : PEAK_ERR_HIP;
    }

    if (!A || !B) return PEAK_ERR_INVALID_ARG;
    if ((uintptr_t)A % es || (uintptr_t)B % es) return PEAK_ERR_INVALID_ARG;
    if (p->g.variant < 0) return PEAK_ERR_UNSUPPORTED;

    const bool a_al = (uintptr_t)A % 16 == 0 && (d.lda * es) % 16 == 0;
    const bool b_al = (uintptr_t)B % 16 == 0 && (d.ldb * es) % 16 == 0;
    if (a_al) a.flags |= GF_A_VEC;
    if (b_al) a.flags |= GF_B_VEC;
    // the selected variant, or its stand-in when it copies 16-byte chunks and a base is off that alignment
    const Geometry *g = &p->g;
    if (g_variants[g->variant].direct && !(a_al && b_al)) {
        if (p->alt.variant < 0) return PEAK_ERR_UNSUPPORTED;
        g = &p->alt;
    }
    const Variant &v = g_variants[g->variant];

    if (g->split > 1) {
        if (!workspace || workspace_bytes < g->ws_bytes) return PEAK_ERR_WORKSPACE;
        if ((uintptr_t)workspace % 256) return PEAK_ERR_INVALID_ARG;
        a.ws = (float *)workspace;
        if (d.N % 4 == 0) a.flags |= GF_WS_VEC;
    }
#ifdef PEAK_TRACE
    // diagnostic build: an unsplit run writes 64 bytes of time stamps per wave into the workspace, if one that large is given
    if (g->split == 1 && workspace && workspace_bytes >= (size_t)g->tiles_m * g->tiles_n * (v.nt / 64) * 64) a.ws = (float *)workspace;
#endif
    a.tiles_m = g->tiles_m; a.tiles_n = g->tiles_n;
    a.split = g->split;
    a.ktiles_per_slice = g->ktiles_per_slice;
    a.ktiles_total = g->ktiles_total;
    a.group_m = g->group_m;
    a.rot_m = g->rot_m;
    a.rot_n = g->rot_n;
    a.sk_tiles = g->sk_tiles;

    int64_t nblocks = grid_blocks(*g);
    if (v.kind == KIND_SKINNY_REG) nblocks = cdiv((int64_t)g->tiles_n * g->split, v.nt / 64);   // one wave per row group and slice
    dim3 grid((unsigned)nblocks);
    if (v.launch(a, grid, stream) != hipSuccess) return PEAK_ERR_HIP;

    if (g->sk_tiles) {
        // the cut tiles: ordered sum of their slices (the 16x16x32 kernels' tile is 256 x 256)
        dim3 rgrid(256 * (256 / 4) / 256, (unsigned)g->sk_tiles);
        if (c_dt == PEAK_DT_F32 || d.dtype == PEAK_DT_BF16)
            hipLaunchKernelGGL((streamk_reduce_kernel<DT_BF16, 256, 256>), rgrid, dim3(256), 0, stream, a);
        else
            hipLaunchKernelGGL((streamk_reduce_kernel<DT_F16, 256, 256>), rgrid, dim3(256), 0, stream, a);
        if (hipGetLastError() != hipSuccess) return PEAK_ERR_HIP;
    } else if (g->split > 1) {
        const int64_t quads = d.M * cdiv(d.N, 4);
        dim3 rgrid((unsigned)cdiv(quads, 256));
        if (c_dt == PEAK_DT_F32) hipLaunchKernelGGL(splitk_reduce_kernel<DT_F32>, rgrid, dim3(256), 0, stream, a);
        else if (c_dt == PEAK_DT_F16) hipLaunchKernelGGL(splitk_reduce_kernel<DT_F16>, rgrid, dim3(256), 0, stream, a);
        else hipLaunchKernelGGL(splitk_reduce_kernel<DT_BF16>, rgrid, dim3(256), 0, stream, a);
        if (hipGetLastError() != hipSuccess) return PEAK_ERR_HIP;
    }
    return PEAK_OK;
}

peak_status_t peak_gemm_run(peak_gemm_plan_t *plan, float alpha, const void *A, const void *B, float beta, void *C,
                            void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return run_plan(plan, alpha, A, B, beta, C, Hook{nullptr, BIAS_NONE, ACT_NONE}, workspace, workspace_bytes, hip_stream);
}

peak_status_t peak_gemm_run_fused(peak_gemm_plan_t *plan, float alpha, const void *A, const void *B, float beta, void *C,
                                  const peak_gemm_epilogue_t *epilogue,
                                  void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Hook hook{nullptr, BIAS_NONE, ACT_NONE};
    if (epilogue) {
        static_assert(PEAK_BIAS_PER_COLUMN == BIAS_PER_COLUMN && PEAK_BIAS_PER_ROW == BIAS_PER_ROW &&
                      PEAK_ACT_RELU == ACT_RELU && PEAK_ACT_GELU_TANH == ACT_GELU_TANH, "interface and kernel enums agree");
        if (epilogue->bias_kind < PEAK_BIAS_NONE || epilogue->bias_kind > PEAK_BIAS_PER_ROW) return PEAK_ERR_INVALID_ARG;
        if (epilogue->act < PEAK_ACT_NONE || epilogue->act > PEAK_ACT_GELU_TANH) return PEAK_ERR_INVALID_ARG;
        if (epilogue->bias_kind != PEAK_BIAS_NONE) {
            if (!epilogue->bias || (uintptr_t)epilogue->bias % sizeof(float)) return PEAK_ERR_INVALID_ARG;
            hook.bias = (const float *)epilogue->bias;
        }
        hook.bias_kind = epilogue->bias_kind;
        hook.act = epilogue->act;
    }
    return run_plan(plan, alpha, A, B, beta, C, hook, workspace, workspace_bytes, hip_stream);
}

// Workspace of peak_gemm_run_static: one array per GPU, part of the loaded code
// object, held until the process ends.  In host code the array's name only
// stands for the symbol; its address on a device comes from hipGetSymbolAddress
// with that device current.
static __device__ __align__(256) unsigned char scratch[PEAK_GEMM_STATIC_WORKSPACE_BYTES];

constexpr int MAX_DEVICES = 64;
static void *g_scratch_ptr[MAX_DEVICES];          // per device; nullptr until looked up
static std::mutex g_scratch_mutex;

peak_status_t peak_gemm_run_static(peak_gemm_plan_t *plan, float alpha, const void *A, const void *B, float beta,
                                   void *C, void *hip_stream)
{
    if (!plan) return PEAK_ERR_INVALID_ARG;
    if (plan->ws_bytes > (size_t)PEAK_GEMM_STATIC_WORKSPACE_BYTES) return PEAK_ERR_WORKSPACE;
    void *ws = nullptr;
    if (plan->ws_bytes > 0) {
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return PEAK_ERR_HIP;
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void *ptr = nullptr;
            if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
                (void)hipGetLastError();
                return PEAK_ERR_HIP;
            }
            g_scratch_ptr[dev] = ptr;
        }
        ws = g_scratch_ptr[dev];
    }
    // Every element of the partials that the reduction reads is written by the slices of
    // this very call, so nothing of an earlier call's contents needs clearing.
    return run_plan(plan, alpha, A, B, beta, C, Hook{nullptr, BIAS_NONE, ACT_NONE}, ws,
                    ws ? (size_t)PEAK_GEMM_STATIC_WORKSPACE_BYTES : 0, hip_stream);
}

peak_status_t peak_gemm_destroy(peak_gemm_plan_t *plan)
{
    delete plan;
    return PEAK_OK;
}

}  // extern "C"
