// Device side of the C ABI: the variant table joined from its translation units, the launches,
// the small kernels' instantiations, and the entry point with a workspace of its own.
#include "../../include/peak_gemm.h"

#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <vector>

#include "gemm_device.h"
#include "skinny_device.h"
#include "variant.h"

namespace peak {

// The variant table: the groups of the other translation units, joined in a fixed order.
static const std::vector<Variant> &variants()
{
    static const std::vector<Variant> table = [] {
        std::vector<Variant> t;
        const VariantGroup groups[] = {variants_general(), variants_bf16_nt(), variants_f16_nt(), variants_bf16_nn(),
                                       variants_f16_nn(),  variants_f32(),     variants_ta(),     variants_skinny(),
                                       variants_mf16(),    variants_mf16s(),   variants_mf16d(),   variants_mf16r(),
                                       variants_mf16k()};
        for (const VariantGroup &g : groups) t.insert(t.end(), g.rows, g.rows + g.count);
        return t;
    }();
    return table;
}

const Variant *planner_variants(int *count)
{
    *count = (int)variants().size();
    return variants().data();
}

int planner_device_cu_count()
{
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
        return v;
    (void)hipGetLastError();
    return 0;
}

}  // namespace peak

using namespace peak;
#define g_variants (variants())

// A stored K x M (at most 64 columns) written out as M rows of K elements, for the streaming kernels,
// which read their small operand along K.  One workgroup turns 64 k-rows around in LDS: reads run along
// the rows of A, writes along K.
template <class T>
__global__ __launch_bounds__(256) void stage_a_kernel(const T *A, int64_t lda, T *dst, int M, int64_t K)
{
    __shared__ T tile[64][65];
    const int64_t k0 = (int64_t)blockIdx.x * 64;
    for (int idx = threadIdx.x; idx < 64 * M; idx += 256) {
        const int k = idx / M, m = idx % M;
        if (k0 + k < K) tile[k][m] = A[(k0 + k) * lda + m];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < 64 * M; idx += 256) {
        const int m = idx / 64, k = idx % 64;
        if (k0 + k < K) dst[(int64_t)m * K + k0 + k] = tile[k][m];
    }
}

static int esize_of(int dt) { return dt == PEAK_DT_F32 ? 4 : 2; }
static int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

extern "C" {

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

    // (a plan that stages A reads its own aligned copy, whatever the base and rows of A)
    bool a_al = (uintptr_t)A % 16 == 0 && (d.lda * es) % 16 == 0;
    const bool b_al = (uintptr_t)B % 16 == 0 && (d.ldb * es) % 16 == 0;
    // the selected variant, or its stand-in when it copies 16-byte chunks and a base is off that alignment
    const Geometry *g = &p->g;
    if (g_variants[g->variant].direct && !((a_al || g->a_copy) && b_al)) {
        if (p->alt.variant < 0) return PEAK_ERR_UNSUPPORTED;
        g = &p->alt;
    }
    const Variant &v = g_variants[g->variant];

    if (g->split > 1 || g->a_copy) {
        if (!workspace || workspace_bytes < g->ws_bytes) return PEAK_ERR_WORKSPACE;
        if ((uintptr_t)workspace % 256) return PEAK_ERR_INVALID_ARG;
    }
    if (g->split > 1) {
        a.ws = (float *)workspace;
        if (d.N % 4 == 0) a.flags |= GF_WS_VEC;
    }
    if (g->a_copy) {
        if (d.M > 64) return PEAK_ERR_UNSUPPORTED;          // (the planner admits no such plan)
        void *copy = (char *)workspace + g->a_copy_off;
        dim3 sgrid((unsigned)cdiv(d.K, 64));
        if (es == 4) hipLaunchKernelGGL(stage_a_kernel<uint32_t>, sgrid, dim3(256), 0, stream, (const uint32_t *)A, d.lda, (uint32_t *)copy, (int)d.M, d.K);
        else hipLaunchKernelGGL(stage_a_kernel<uint16_t>, sgrid, dim3(256), 0, stream, (const uint16_t *)A, d.lda, (uint16_t *)copy, (int)d.M, d.K);
        if (hipGetLastError() != hipSuccess) return PEAK_ERR_HIP;
        a.A = copy;
        a.lda = d.K;
        a_al = true;
    }
    if (a_al) a.flags |= GF_A_VEC;
    if (b_al) a.flags |= GF_B_VEC;
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
    if (v.launch(a, (unsigned)nblocks, (void *)stream) != 0) return PEAK_ERR_HIP;

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

}  // extern "C"
