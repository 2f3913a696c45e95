// Host-only driver for the sanitizer test: the library's planner (csrc/planner.cpp) built with
// the host compiler under AddressSanitizer and UndefinedBehaviorSanitizer, with a stand-in
// variant table (same row type, kinds and flags as the real one; no kernels behind it).
// Walks descriptors of every kind through peak_gemm_create / plan_info / destroy and feeds
// the selector-table parser well-formed, malformed and hostile files.  Exit status 0 = clean.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../paper_2512_19018_amd/csrc/planner.h"

namespace peak {

static int no_launch(const GemmArgs &, unsigned, void *) { return 1; }

// name, kind, dt, a_t, b_t, direct, bm, bn, bk, nt, ns, lds, max_m, launch, tr, atr, sweep_only, stream_rank, mf16
static const Variant g_rows[] = {
    {"f32_r128x128_nn", KIND_TILED, 0, 0, 1, 0, 128, 128, 32, 256, 2, 65536, 0, &no_launch, 0, 0, 0, 0, 0},
    {"f32_r128x128_nt", KIND_TILED, 0, 0, 0, 0, 128, 128, 32, 256, 2, 65536, 0, &no_launch, 0, 0, 0, 0, 0},
    {"f32_r64x64_tn", KIND_TILED, 0, 1, 1, 0, 64, 64, 32, 256, 2, 32768, 0, &no_launch, 0, 0, 0, 0, 0},
    {"f32_r64x64_tt", KIND_TILED, 0, 1, 0, 0, 64, 64, 32, 256, 2, 32768, 0, &no_launch, 0, 0, 0, 0, 0},
    {"f32_t256x256w4a3_nn", KIND_TILED, 0, 0, 1, 1, 256, 256, 32, 256, 2, 163840, 0, &no_launch, 1, 0, 0, 0, 0},
    {"bf16_r128x128_nt", KIND_TILED, 2, 0, 0, 0, 128, 128, 64, 256, 2, 65536, 0, &no_launch, 0, 0, 0, 0, 0},
    {"bf16_r64x64_nn", KIND_TILED, 2, 0, 1, 0, 64, 64, 64, 256, 2, 32768, 0, &no_launch, 0, 0, 0, 0, 0},
    {"bf16_r64x64_tn", KIND_TILED, 2, 1, 1, 0, 64, 64, 64, 256, 2, 32768, 0, &no_launch, 0, 0, 0, 0, 0},
    {"bf16_r64x64_tt", KIND_TILED, 2, 1, 0, 0, 64, 64, 64, 256, 2, 32768, 0, &no_launch, 0, 0, 0, 0, 0},
    {"bf16_d128x128w4_nt", KIND_TILED, 2, 0, 0, 1, 128, 128, 64, 256, 2, 65536, 0, &no_launch, 0, 0, 0, 0, 0},
    {"bf16_d256x256w8k32s5_nt", KIND_TILED, 2, 0, 0, 1, 256, 256, 32, 512, 5, 163840, 0, &no_launch, 0, 0, 1, 0, 0},
    {"bf16_m256x256w4a3_nt", KIND_TILED, 2, 0, 0, 1, 256, 256, 64, 256, 2, 163840, 0, &no_launch, 0, 0, 0, 0, 1},
    {"bf16_m256x256w4a3_nn", KIND_TILED, 2, 0, 1, 1, 256, 256, 64, 256, 2, 163840, 0, &no_launch, 1, 0, 0, 0, 1},
    {"bf16_m256x256w4a3_tn", KIND_TILED, 2, 1, 1, 1, 256, 256, 64, 256, 2, 163840, 0, &no_launch, 1, 1, 0, 0, 1},
    {"bf16_too_much_lds_nt", KIND_TILED, 2, 0, 0, 1, 256, 256, 64, 256, 3, 200000, 0, &no_launch, 0, 0, 0, 0, 0},
    {"f16_r128x128_nt", KIND_TILED, 1, 0, 0, 0, 128, 128, 64, 256, 2, 65536, 0, &no_launch, 0, 0, 0, 0, 0},
    {"f16_r128x128_nn", KIND_TILED, 1, 0, 1, 0, 128, 128, 64, 256, 2, 65536, 0, &no_launch, 0, 0, 0, 0, 0},
    {"bf16_skinny16s3_nt", KIND_SKINNY, 2, 0, 0, 1, 16, 64, 128, 256, 3, 61440, 16, &no_launch, 0, 0, 0, 2, 0},
    {"bf16_skinny128k256s2_nt", KIND_SKINNY, 2, 0, 0, 1, 16, 128, 256, 512, 2, 147456, 16, &no_launch, 0, 0, 0, 3, 0},
    {"bf16_skinnyreg_d8_nt", KIND_SKINNY_REG, 2, 0, 0, 1, 16, 16, 64, 256, 8, 0, 16, &no_launch, 0, 0, 0, 1, 0},
};

const Variant *planner_variants(int *count)
{
    *count = (int)(sizeof(g_rows) / sizeof(g_rows[0]));
    return g_rows;
}

int planner_device_cu_count() { return 0; }   // no device: the planner falls back to 256

}  // namespace peak

static int failures = 0;
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed line %d: %s\n", __LINE__, #c); ++failures; } } while (0)

static void write_file(const std::string &path, const std::string &text)
{
    FILE *f = fopen(path.c_str(), "wb");
    if (!f) { perror(path.c_str()); exit(3); }
    fwrite(text.data(), 1, text.size(), f);
    fclose(f);
}

int main(int argc, char **argv)
{
    const std::string dir = argc > 1 ? argv[1] : "/tmp";
    const int nvar = peak_gemm_variant_count();
    CHECK(nvar == 20);
    CHECK(peak_gemm_variant_name(-1) == nullptr && peak_gemm_variant_name(nvar) == nullptr);
    for (int s = -2; s < 9; ++s) CHECK(peak_status_string((peak_status_t)s) != nullptr);

    // descriptors: sizes around tile edges, degenerate, huge; all dtypes, layouts; forced variants and splits; flag bits
    const int64_t sizes[] = {0, 1, 7, 16, 63, 64, 65, 255, 256, 257, 1000, 4096, 4608, 8192, 16384, (int64_t)1 << 30, ((int64_t)1 << 30) + 1};
    const uint32_t flag_sets[] = {0, PEAK_GEMM_C_F32, PEAK_GEMM_STREAMK_ON, PEAK_GEMM_STREAMK_OFF, PEAK_GEMM_STREAMK_ON | PEAK_GEMM_STREAMK_OFF,
                                  0x80000000u, 0x100000u};
    long plans = 0;
    unsigned rng = 12345;
    auto next = [&]() { rng = rng * 1664525u + 1013904223u; return rng >> 8; };
    for (int dt = -1; dt <= 3; ++dt)
        for (int ta = 0; ta <= 1; ++ta)
            for (int tb = 0; tb <= 1; ++tb)
                for (int it = 0; it < 400; ++it) {
                    peak_gemm_desc_t d;
                    memset(&d, 0, sizeof d);
                    d.M = sizes[next() % 17]; d.N = sizes[next() % 17]; d.K = sizes[next() % 17];
                    if (it % 50 == 0) d.M = -1;
                    d.transA = ta; d.transB = tb; d.dtype = dt;
                    const int64_t min_lda = ta ? d.M : d.K, min_ldb = tb ? d.K : d.N;
                    const int pad = (int)(next() % 4) * (int)(next() % 9);
                    d.lda = (min_lda > 1 ? min_lda : 1) + pad;
                    d.ldb = (min_ldb > 1 ? min_ldb : 1) + (int)(next() % 3) * 8;
                    d.ldc = (d.N > 1 ? d.N : 1) + (int)(next() % 2) * 4;
                    if (it % 37 == 0) d.lda = 0;
                    uint32_t flags = flag_sets[next() % 7];
                    if (next() % 3 == 0) flags |= (next() % (nvar + 3)) + 1;            // forced variant, some out of range
                    if (next() % 3 == 0) flags |= (next() % 256) << 8;                  // forced split
                    d.flags = flags;
                    peak_gemm_plan_t *plan = (peak_gemm_plan_t *)0x1;
                    const peak_status_t st = peak_gemm_create(&d, &plan);
                    if (st != PEAK_OK) { CHECK(plan == nullptr); continue; }
                    CHECK(plan != nullptr);
                    ++plans;
                    char small[16], big[1024];
                    const int need = peak_gemm_plan_info(plan, big, sizeof big);
                    CHECK(need > 0 && need < (int)sizeof big && (int)strlen(big) == need);
                    CHECK(peak_gemm_plan_info(plan, small, sizeof small) == need && strlen(small) == sizeof small - 1);
                    CHECK(peak_gemm_plan_info(plan, small, 0) == need);
                    (void)peak_gemm_workspace_bytes(plan);
                    CHECK(peak_gemm_destroy(plan) == PEAK_OK);
                }
    CHECK(plans > 1000);
    peak_gemm_plan_t *plan = nullptr;
    CHECK(peak_gemm_create(nullptr, &plan) == PEAK_ERR_INVALID_ARG);
    peak_gemm_desc_t d0;
    memset(&d0, 0, sizeof d0);
    CHECK(peak_gemm_create(&d0, nullptr) == PEAK_ERR_INVALID_ARG);
    CHECK(peak_gemm_destroy(nullptr) == PEAK_OK && peak_gemm_workspace_bytes(nullptr) == 0);
    char buf[64];
    CHECK(peak_gemm_plan_info(nullptr, buf, sizeof buf) > 0);

    // selector tables
    const std::string good = dir + "/table_good.txt", bad = dir + "/table_bad.txt";
    write_file(good, "# comment only line\n\nbf16 0 1 8192 8192 8192 bf16_m256x256w4a3_nt 1   # 700 us\n"
                     "bf16 0 1 8192 4608 8192 bf16_m256x256w4a3_nt 0\nf32 0 0 4096 4096 4096 f32_t256x256w4a3_nn 1 trailing columns are ignored\n"
                     "bf16 0 1 16 16384 16384 bf16_skinny16s3_nt 1");
    CHECK(peak_gemm_load_tuning(good.c_str()) == 4);
    peak_gemm_desc_t d;
    memset(&d, 0, sizeof d);
    d.M = 8192; d.N = 4608; d.K = 8192; d.lda = 8192; d.ldb = 8192; d.ldc = 4608; d.transB = 1; d.dtype = PEAK_DT_BF16;
    CHECK(peak_gemm_create(&d, &plan) == PEAK_OK);
    char info[1024];
    peak_gemm_plan_info(plan, info, sizeof info);
    CHECK(strstr(info, "streamk=64") != nullptr);                                 // split 0 in the table = stream-K on
    peak_gemm_destroy(plan);
    const char *hostile[] = {
        "bf16 0 1 8192 8192 8192 no_such_variant 1\n",
        "bf16 0 1 8192 8192 8192 f32_t256x256w4a3_nn 1\n",                       // dtype of the variant differs
        "bf16 0 1 8192 8192 8192 bf16_m256x256w4a3_nt\n",                        // column missing
        "bf16 2 1 8192 8192 8192 bf16_m256x256w4a3_nt 1\n",
        "bf16 0 1 -5 8192 8192 bf16_m256x256w4a3_nt 1\n",
        "bf16 0 1 8192 8192 8192 bf16_m256x256w4a3_nt 999\n",
        "bf16 0 1 99999999999999999999999999 8192 8192 bf16_m256x256w4a3_nt 1\n",
        "quux 0 1 8 8 8 bf16_m256x256w4a3_nt 1\n",
        "bf16 0 1 8192 8192 8192 AAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAAA 1\n",
    };
    for (const char *h : hostile) {
        write_file(bad, h);
        CHECK(peak_gemm_load_tuning(bad.c_str()) == -1);
    }
    // a line far beyond the parser's buffer, and raw bytes
    write_file(bad, std::string(5000, 'x') + " 0 1 8 8 8 bf16_m256x256w4a3_nt 1\n");
    CHECK(peak_gemm_load_tuning(bad.c_str()) == -1);
    std::string junk;
    for (int i = 0; i < 4096; ++i) junk.push_back((char)(next() & 0xFF));
    write_file(bad, junk);
    (void)peak_gemm_load_tuning(bad.c_str());                                     // any verdict, no bad access
    CHECK(peak_gemm_load_tuning((dir + "/does_not_exist.txt").c_str()) == -1);
    CHECK(peak_gemm_load_tuning(good.c_str()) == 4);                              // still usable afterwards
    CHECK(peak_gemm_load_tuning(nullptr) == 0);

    if (failures) { fprintf(stderr, "%d checks failed\n", failures); return 1; }
    printf("planner sanitizer run clean: %ld plans made and destroyed\n", plans);
    return 0;
}
