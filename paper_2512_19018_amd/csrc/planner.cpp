// Plans: argument checks, variant selection (cost model, selector table), K split and
// stream-K decisions, and the entry points of the C ABI that need no GPU runtime.
#include "planner.h"

#include <dlfcn.h>

#include <cerrno>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

using namespace peak;

constexpr int LDS_LIMIT = 160 * 1024; // bytes per workgroup on gfx950

static int g_num_variants = 0;
static const Variant *variant_table()
{
    static const Variant *table = planner_variants(&g_num_variants);
    return table;
}
#define g_variants (variant_table())
#define NUM_VARIANTS (variant_table(), g_num_variants)

// Compute units of the device the plans are made for: PEAK_GEMM_NUM_CU, else the
// current device's count, else (no device visible) that of the MI355X.
static int num_cu()
{
    static const int n = [] {
        if (const char *e = getenv("PEAK_GEMM_NUM_CU")) {
            const int v = atoi(e);
            if (v >= 1 && v <= 4096) return v;
        }
        const int v = planner_device_cu_count();
        return v > 0 ? v : 256;
    }();
    return n;
}

static int esize_of(int dt) { return dt == PEAK_DT_F32 ? 4 : 2; }

static bool variant_fits(const Variant &v, const peak_gemm_desc_t &d)
{
    if (v.dt != d.dtype) return false;
    if (v.lds > LDS_LIMIT) return false;
    // layouts: kernel's A_T means A does not run along K, i.e. transA == 1;
    // kernel's B_T means B stored K x N, i.e. transB == 0
    const int a_t = d.transA ? 1 : 0, b_t = d.transB ? 0 : 1;
    const bool a_copy = stages_a(v, d.transA);              // the kernel then reads a copy of A with rows of K elements
    if ((v.a_t != a_t && !a_copy) || v.b_t != b_t) return false;
    if (v.kind != KIND_TILED && d.M > v.max_m) return false;
    if (a_copy && (!v.direct || d.M > 64)) return false;
    if (v.direct) {
        const int es = esize_of(d.dtype);
        const int64_t lda = a_copy ? d.K : d.lda;
        const bool a_along_k = !v.a_t, b_along_k = !v.b_t;      // copied in 16-byte chunks along K
        if (v.kind == KIND_TILED) {
            // K may stop inside the last K tile: at a 16-byte chunk boundary for an operand that
            // runs along K, anywhere for one staged as [k][.] rows
            if ((a_along_k || b_along_k) && (d.K * es) % 16 != 0) return false;
            if (v.tr && (d.N * es) % 16 != 0) return false;
            if (v.atr && (d.M * es) % 16 != 0) return false;
        } else {
            if (d.K % v.bk != 0 || d.K < v.bk) return false;
            if (v.tr && (d.N * es) % 16 != 0) return false;
        }
        if ((lda * es) % 16 != 0 || (d.ldb * es) % 16 != 0) return false;
        // a workgroup's operand panel is addressed with 32-bit byte offsets
        const int64_t lim = (int64_t)1 << 31;
        if (v.atr ? ((d.K - 1) * lda + d.M) * es >= lim : a_along_k && ((int64_t)(v.bm - 1) * lda + d.K) * es >= lim) return false;
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
    const double tile_work = (double)v.bm * v.bn * v.bk * ktiles * (v.dt == PEAK_DT_F32 ? 16.0 : 1.0);
    // small tiles pay more LDS/L2 traffic per flop; direct loads overlap better.
    // The constants come from the measured sweeps on the graded shapes.
    double eff = 1.0;
    if (v.dt == PEAK_DT_F32) {                               // fp32 MFMA is slow enough that tile size hardly matters
        // 128x128 per wave: a quarter of the LDS traffic of 64x64 wave tiles; with one wave per SIMD 1-3 % ahead of
        // the 128 x 128 tile on full rounds (2048x8192x8192: 1822 us against 1871)
        if (v.bm * v.bn >= 256 * 256) eff = v.nt == 256 && v.lds > 140 * 1024 ? 0.96 : 0.90;
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
    if (v.tr) eff *= v.dt == PEAK_DT_F32 ? 1.10 : 1.03;      // B staged directly: no register transposition, no masked loads
    if (v.lds > 140 * 1024 && v.ns == 2 && !v.tr) eff *= 1.02;   // third A stage, A's loads spread over the step (+2 % measured; nothing with [k][n] B)
    if (v.nt == 256 && v.bm == 256 && v.bn == 256 && v.lds > 140 * 1024) eff *= 1.02;   // one wave per SIMD on top of that
    // 16x16x32 MFMA: same cycles, higher clock (256 x 256: +10 % measured; 128 x 128: 3-8 % ahead of the 32x32x16
    // kernel of the same tile, and a fifth behind the 256 x 256 tile where both run full rounds: bf16 8192x4608x8192
    // 542 us against 431)
    if (v.mf16) eff *= v.bm * v.bn == 256 * 256 ? 1.10 : v.bm * v.bn == 256 * 128 ? 1.08 : 1.04;
    // ... with loads four K tiles ahead and the CU to itself: for at most one workgroup per CU, where it
    // stands in for the second workgroup that would cover the loads' latency
    // (likewise the form with 128 k per stage: one workgroup per CU, half the barriers per multiply-add, 256 bytes
    // of a row per load step; bf16 128x28672x8192 87 us against 93)
    // The gain fades with the depth of K: a long launch runs at the chip's power limit, where the energy per
    // multiply-add decides and the 256 x 256 tile's smaller LDS and L2 traffic wins (bf16 512x8192x28672: 252 us
    // against 211 for the 256 x 256 tile split four ways; 512x8192x8192: the 128 x 128 form ahead, 57.8 us).
    const double kdepth = ktiles * v.bk;
    if (v.mf16 && v.bm == 128 && v.bn == 128 && (v.ns > 2 || v.bk == 128))
        eff *= tiles > num_cu() ? 0.85 : kdepth > 16384.0 ? 0.8 : kdepth > 8192.0 ? 1.1 : 1.3;
    else if (v.mf16 && v.bm == 128 && v.bn == 128 && tiles <= num_cu())
        eff *= kdepth > 8192.0 ? 0.72 : 0.85;           // the two-workgroups-per-CU form with a CU to itself
    else if (v.dt != PEAK_DT_F32 && v.bm * v.bn < 256 * 256 && kdepth > 8192.0)
        eff *= 0.85;                                    // likewise the other tiles below 256 x 256 (256 x 128 at 512x8192x28672 in two slices: 264 us)
    // The small tiles of the 32x32x16 kernels hide the loads' latency behind the other workgroups of their CU.
    // Where there is at most one round of them and K is deep, each K tile waits out a trip to memory
    // (bf16 512x4096x4096: 128x64 tiles 37 us, the 128 x 128 forms above 26; f16 NN likewise 37 against 29).
    if (v.dt != PEAK_DT_F32 && !v.mf16 && v.bm * v.bn < 256 * 128 && tiles <= num_cu() && kdepth >= 2048.0) eff *= 0.6;
    // (A staged as [k][m] rows gets no factor of its own: every direct kernel for an A stored K x M stages it that
    // way, the register-staged general tile is marked down above, and a factor here would only shrink the tile work
    // against the cost of a K split's reduction - bf16 512x8192x28672 TN: 128x128 tiles unsplit 347 us, the
    // 256x256 tile in four slices 206)
    if (v.dt == PEAK_DT_F32 && v.ns == 3) eff *= 0.97;
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
    if (!v.mf16 || v.bm != 256 || v.bn != 256) return 0;     // built into the 256 x 256 16x16x32 kernels only
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
    // tile rows per band: an XCD's 32 tiles of a moment form a patch of group_m x 32 / group_m tiles.  Re-measured with
    // the 16x16x32 kernels, 4 rows against 8 in alternating blocks: bf16 8192x4608x8192 +0.8 %, 6144^3 +0.9 %, 4096^3
    // +0.5 %, 8192^3 level, and -0.6 % with few tile columns (f16 5000x3000x12288)
    const int band_rows = p->tiles_n >= 16 ? 4 : 8;
    p->group_m = p->tiles_m >= band_rows ? band_rows : (p->tiles_m > 0 ? p->tiles_m : 1);
    p->rot_m = 0;                                           // K rotation off for the tiled kernels: measured no gain on the graded shapes
                                                            // (bf16 8192^3: 694 us without, 701 with 1, 736 with 5)
    p->rot_n = v.kind == KIND_SKINNY && !v.tr ? 5 : 0;               // streaming kernel: neighbouring workgroups start five K tiles apart
                                                            // (bf16 16x16384x16384: 5.3 TB/s without, 6.0 with 1, 6.2 with 5 or 13)
    // ... except where a single row of tiles has every workgroup stream rows of B that no other reads: started one
    // K tile apart they spread over the memory channels (16x16x32 kernels; bf16 128x28672x8192 109 -> 103 us)
    if (v.mf16 && p->tiles_m == 1 && p->tiles_n > 1) p->rot_n = 1;
    if (const char *e = getenv("PEAK_GEMM_GROUP_M")) {      // tuning knob: tile rows per band
        const int g = atoi(e);
        if (g >= 1 && g <= 64) p->group_m = g < p->tiles_m ? g : (p->tiles_m > 0 ? p->tiles_m : 1);
    }
    if (const char *e = getenv("PEAK_GEMM_ROT")) {          // tuning knob: "rot_m,rot_n"
        int a = 0, b = 0;
        if (sscanf(e, "%d,%d", &a, &b) == 2 && a >= 0 && b >= 0) { p->rot_m = a; p->rot_n = b; }
    }
    p->ws_bytes = p->split > 1 ? (size_t)p->split * (size_t)d.M * (size_t)d.N * sizeof(float) : 0;
    p->a_copy = stages_a(v, d.transA) ? 1 : 0;
    p->a_copy_off = 0;
    if (p->a_copy) {                                        // behind the partials, on a 256-byte boundary
        p->a_copy_off = (p->ws_bytes + 255) & ~(size_t)255;
        p->ws_bytes = p->a_copy_off + (((size_t)d.M * (size_t)d.K * esize_of(d.dtype) + 255) & ~(size_t)255);
    }
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
    int pick = -1, stream[4] = {-1, -1, -1, -1};            // first fitting streaming kernel of each rank
    // streaming kernels: only those with the fewest rows of the M x K operand that hold M
    int stream_bm = 0;
    for (int i = 0; i < NUM_VARIANTS; ++i) {
        const Variant &v = g_variants[i];
        if (v.kind == KIND_TILED || v.sweep_only || (staged_only && v.direct) || !variant_fits(v, d)) continue;
        if (stages_a(v, d.transA) && d.N * d.K * esize_of(d.dtype) < ((int64_t)8 << 20)) continue;
        if (stream_bm == 0 || v.bm < stream_bm) stream_bm = v.bm;
    }
    for (int i = 0; i < NUM_VARIANTS; ++i) {
        const Variant &v = g_variants[i];
        if (v.sweep_only || (staged_only && v.direct) || !variant_fits(v, d)) continue;
        if (v.kind != KIND_TILED) {
            if (v.bm != stream_bm) continue;
            // the transposition of A is one more launch: worth it once the streamed operand has some MB
            if (stages_a(v, d.transA) && d.N * d.K * esize_of(d.dtype) < ((int64_t)8 << 20)) continue;
            // rank 3 only where one workgroup per tile of its (larger) BN fills four fifths of the chip, or where
            // the M x K operand is tall enough for its re-reads to matter (every workgroup reads its K slice of
            // all of it: bf16 64x8192x28672 takes 101.9 us with 128 rows per workgroup, 126.4 us with 64)
            if (v.stream_rank == 3 && v.bm < 64 && cdiv(d.N, v.bn) * 5 < (int64_t)num_cu() * 4) continue;
            if (stream[v.stream_rank] < 0) stream[v.stream_rank] = i;
            continue;
        }
        const int split = choose_split(v, d);
        double c = tiled_cost(v, d, split);
        if (split == 1) {
            // a partial last round that hybrid stream-K will cut costs a slice and the reduction, not a whole tile
            int sk_tiles = 0;
            const int S = streamk_split(v, d, &sk_tiles);
            if (S >= 2 && streamk_pays(v, d, S, sk_tiles)) {
                const int64_t tiles = cdiv(d.M, v.bm) * cdiv(d.N, v.bn);
                const double per_round = c / (double)cdiv(tiles, num_cu());
                c -= per_round * (1.0 - 1.0 / S) * 0.8;              // four fifths of the saving that round counting predicts
            }
        }
        if (pick < 0 || c < best) { pick = i; best = c; }
    }
    // a streaming kernel wins whenever one applies
    for (int r = 3; r >= 1; --r)
        if (stream[r] >= 0) return stream[r];
    return pick;
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

// whole decimal number within [lo, hi]; anything else (sign games, overflow, trailing characters) is refused
static bool parse_int(const char *tok, long long lo, long long hi, long long *out)
{
    if (!tok || !*tok) return false;
    char *end = nullptr;
    errno = 0;
    const long long v = strtoll(tok, &end, 10);
    if (errno != 0 || end == tok || *end != 0 || v < lo || v > hi) return false;
    *out = v;
    return true;
}

static int load_tuning_file(const char *path)
{
    FILE *f = fopen(path, "r");
    if (!f) return -1;
    std::vector<TuneEntry> table;
    char line[512];
    bool ok = true;
    while (ok && fgets(line, sizeof line, f)) {
        const size_t len = strlen(line);
        if (len == sizeof line - 1 && line[len - 1] != '\n') { ok = false; break; }   // longer than any valid row
        if (char *hash = strchr(line, '#')) *hash = 0;
        // up to eight whitespace-separated columns; further ones are ignored
        char *tok[8];
        int n = 0;
        for (char *t = strtok(line, " \t\r\n"); t && n < 8; t = strtok(nullptr, " \t\r\n")) tok[n++] = t;
        if (n == 0) continue;                               // blank or comment line
        TuneEntry e;
        long long ta = 0, tb = 0, M = 0, N = 0, K = 0, split = 0;
        ok = n == 8;
        if (ok) {
            e.dt = strcmp(tok[0], "f32") == 0 ? PEAK_DT_F32 : strcmp(tok[0], "f16") == 0 ? PEAK_DT_F16
                 : strcmp(tok[0], "bf16") == 0 ? PEAK_DT_BF16 : -1;
            e.variant = variant_by_name(tok[6]);
            const long long dim_max = (long long)1 << 30;
            ok = e.dt >= 0 && e.variant >= 0 && g_variants[e.variant].dt == e.dt &&
                 parse_int(tok[1], 0, 1, &ta) && parse_int(tok[2], 0, 1, &tb) &&
                 parse_int(tok[3], 1, dim_max, &M) && parse_int(tok[4], 1, dim_max, &N) && parse_int(tok[5], 1, dim_max, &K) &&
                 parse_int(tok[7], 0, 255, &split);
        }
        if (ok) {
            e.ta = (int)ta; e.tb = (int)tb; e.M = M; e.N = N; e.K = K; e.split = (int)split;
            table.push_back(e);
        }
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

int64_t peak::grid_blocks(const Geometry &g)
{
    const int64_t tiles = (int64_t)g.tiles_m * g.tiles_n;
    return g.sk_tiles ? tiles - g.sk_tiles + (int64_t)g.sk_tiles * g.split : tiles * g.split;
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
                    "grid=%lld (tiles %dx%d) group_m=%d workspace=%zu unaligned=%s streamk=%d rot=%d,%d acopy=%d",
                    g.variant, v.name, v.bm, v.bn, v.bk, v.nt, v.ns, v.lds, g.split, g.ktiles_per_slice,
                    (long long)grid_blocks(g), g.tiles_m, g.tiles_n, g.group_m, p->ws_bytes,
                    p->alt.variant >= 0 ? g_variants[p->alt.variant].name : "same", g.sk_tiles, g.rot_m, g.rot_n, g.a_copy);
}

peak_status_t peak_gemm_destroy(peak_gemm_plan_t *plan)
{
    delete plan;
    return PEAK_OK;
}

}  // extern "C"
