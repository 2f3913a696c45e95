// Host side of the library that needs no GPU runtime: the kernel variant table's
// row type, plans, and the selector (the tuning and execution parameters of the
// paper's Section 3.1; the table from the sweep of Section 3.3).  Plain C++, so
// that it also builds with the host compiler alone (the sanitizer test does).
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "../../include/peak_gemm.h"

namespace peak {

struct GemmArgs;

// enqueues the variant's kernel on `stream` (a hipStream_t) with `grid` workgroups; 0 on success
typedef int (*launch_fn)(const GemmArgs &, unsigned grid, void *stream);

enum Kind { KIND_TILED = 0, KIND_SKINNY = 1, KIND_SKINNY_REG = 2 };

struct Variant {
    const char *name;
    int kind;
    int dt;
    int a_t, b_t;        // operand layouts the kernel was built for (1: stored K rows x M/N)
    int direct;          // needs 16-byte aligned operand bases and rows (tiled: K a whole number of 16-byte chunks; skinny: K % BK == 0)
    int bm, bn, bk, nt, ns, lds;
    int max_m;           // skinny kernels: largest M
    launch_fn launch;
    int tr;              // B (K x N) goes to LDS untransposed ([k][n] rows)
    int atr;             // A (K x M) goes to LDS untransposed ([k][m] rows)
    int sweep_only;      // 1: reachable through the force bits only (kept for sweeps); the selector skips it
    int stream_rank;     // streaming (skinny) kernels: 3 = taken when its workgroups fill the chip without a K split,
                         // 2 = the usual choice, 1 = the fallback for other K, 0 = sweeps only
    int mf16;            // built on the 16x16x32 MFMA (holds a higher clock under the chip's power limit)
};

struct VariantGroup {
    const Variant *rows;
    int count;
};

// The library's variant table and the compute-unit count of the current device (<= 0: no
// device visible).  Defined beside the kernels (peak_gemm.hip); a host-only build supplies its own.
const Variant *planner_variants(int *count);
int planner_device_cu_count();

// Grid and K split of one variant for the plan's problem.
struct Geometry {
    int variant;          // index into the variant table, -1: nothing to launch
    int tiles_m, tiles_n, split, ktiles_total, ktiles_per_slice, group_m, rot_m, rot_n;
    int sk_tiles;         // hybrid stream-K: tiles of the last, partial round that are cut into `split` K slices; 0: off
    int a_copy;           // streaming kernel on an A stored K x M: A is first written out along K (M rows of K
                          // elements) at a_copy_off of the workspace, and the kernel reads that
    size_t a_copy_off;
    size_t ws_bytes;
};

// A streaming kernel built for A along K also serves an A stored K x M (at most 64 columns): the run
// transposes A into the workspace first, a few MB against the K x N operand the kernel then streams.
static inline bool stages_a(const Variant &v, int transA) { return v.kind == KIND_SKINNY && !v.a_t && transA; }

// workgroups of the GEMM launch
int64_t grid_blocks(const Geometry &g);

// Number of K slices: one workgroup per CU is enough once it streams (measured:
// splitting further only adds the reduction pass), at least 4 stages each.  Workgroups on
// four fifths of the CUs already count as enough (bf16 16x28672x8192 with 128 rows per
// workgroup: 224 workgroups unsplit 74.9 us, 448 in two slices 87.1 us).
static inline int skinny_split(int64_t N, int64_t K, int bn, int kstep)
{
    const int64_t tiles_n = (N + bn - 1) / bn;
    const int64_t ktiles = (K + kstep - 1) / kstep;
    int64_t s = (256 + tiles_n / 4) / tiles_n;
    if (s > ktiles / 4) s = ktiles / 4;
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    return (int)s;
}

// K slices for the register-streaming kernel: aim at >= 8 waves per CU
static inline int skinny_reg_split(int64_t N, int64_t K)
{
    const int64_t groups = (N + 15) / 16;
    const int64_t iters = K / 64;
    int64_t s = (2048 + groups - 1) / groups;
    if (s > iters / 16) s = iters / 16;
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    return (int)s;
}

}  // namespace peak

struct peak_gemm_plan {
    peak_gemm_desc_t d;
    peak::Geometry g;           // the selected variant
    peak::Geometry alt;         // register-staged stand-in for runs whose A or B base is not 16-byte aligned
                          // (variant -1 when the selected variant has no alignment needs)
    size_t ws_bytes;      // the larger of the two workspaces
};
