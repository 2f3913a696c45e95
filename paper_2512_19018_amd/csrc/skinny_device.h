// Streaming kernel for skinny products (M <= 16, both operands running along K
// in memory): the N x K operand is read from HBM exactly once and that read is
// the whole cost, so the kernel is built around keeping many direct-to-LDS
// loads in flight per CU, not around the matrix cores (one 16x16x32 MFMA per
// 32 k still does the arithmetic).  K is cut into slices (the paper's Split-K,
// Section 4.1 Table 2) so that enough workgroups stream at once; the fp32
// partials are summed in slice order by splitk_reduce_kernel.
#pragma once

#include "gemm_device.h"
#include "planner.h"

namespace peak {

template <int DT_, int BN_, int KSTEP_, int NS_>
struct SkinnyCfg {
    static constexpr int DT = DT_;
    static_assert(DT_ != DT_F32, "16-bit storage only");
    static constexpr int ESZ = 2, EPC = 8;
    static constexpr int BM = 16, BN = BN_, KSTEP = KSTEP_, NS = NS_;
    static constexpr int RB = KSTEP_ * ESZ;               // bytes per tile row and stage
    static constexpr int CPR = RB / 16;                   // 16-byte chunks per tile row
    static constexpr int NW = BN_ / 16;                   // one wave per 16 rows of the N x K operand
    static constexpr int NT = NW * 64;
    static constexpr int A_BYTES = BM * RB, B_BYTES = BN_ * RB;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = STAGE_BYTES * NS_;
    static constexpr int ROWS_PER_INST = 64 / CPR;        // a wave load fills 1024 contiguous LDS bytes
    static constexpr int A_INST = BM / ROWS_PER_INST, B_INST = BN_ / ROWS_PER_INST;
    static_assert(CPR % 16 == 0 && CPR <= 64, "row of 256, 512 or 1024 bytes");
    static_assert(A_INST % NW == 0 || NW % A_INST == 0, "A loads split evenly");
    static_assert(B_INST % NW == 0, "B loads split evenly");
    static constexpr int B_PER_WAVE = B_INST / NW;
    // every wave issues the same number of loads per stage: its share of B, and
    // one A instruction (waves beyond A_INST repeat an A instruction of another
    // wave, writing the same bytes to the same place)
    static constexpr int A_PER_WAVE = A_INST >= NW ? A_INST / NW : 1;
    static constexpr int DLOADS = A_PER_WAVE + B_PER_WAVE;
};

// chunk c of tile row r sits at position c ^ (r & 15) (in units of 16 bytes,
// within the aligned group of 16 chunks c belongs to)
PEAK_DEV int skinny_pos(int r, int c) { return c ^ (r & 15); }

template <class C>
__global__ __launch_bounds__(C::NT) void skinny_kernel(const GemmArgs p)
{
    __shared__ __attribute__((aligned(1024))) char lds[C::LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tn = blockIdx.x % p.tiles_n, slice = blockIdx.x / p.tiles_n;
    const int64_t n0 = (int64_t)tn * C::BN;

    const int kt_begin = slice * p.ktiles_per_slice;
    int kt_end = kt_begin + p.ktiles_per_slice;
    if (kt_end > p.ktiles_total) kt_end = p.ktiles_total;
    const int KT = kt_end - kt_begin;
    const int64_t kbase = (int64_t)kt_begin * C::KSTEP;

    // sources of this lane's direct loads at the slice's first k
    const char *ga[C::A_PER_WAVE];
    const char *gb[C::B_PER_WAVE];
    int ja[C::A_PER_WAVE], jb[C::B_PER_WAVE];
#pragma unroll
    for (int i = 0; i < C::A_PER_WAVE; ++i) {
        const int j = (wave + C::NW * i) % C::A_INST;
        const int row = j * C::ROWS_PER_INST + lane / C::CPR, pos = lane % C::CPR;
        const int c = (pos & ~15) | skinny_pos(row, pos & 15);
        int64_t gr = row;
        if (gr > p.M - 1) gr = p.M - 1;
        ga[i] = (const char *)p.A + (gr * p.lda + kbase + (int64_t)c * C::EPC) * C::ESZ;
        ja[i] = j;
    }
#pragma unroll
    for (int i = 0; i < C::B_PER_WAVE; ++i) {
        const int j = wave + C::NW * i;
        const int row = j * C::ROWS_PER_INST + lane / C::CPR, pos = lane % C::CPR;
        const int c = (pos & ~15) | skinny_pos(row, pos & 15);
        int64_t gr = n0 + row;
        if (gr > p.N - 1) gr = p.N - 1;
        gb[i] = (const char *)p.B + (gr * p.ldb + kbase + (int64_t)c * C::EPC) * C::ESZ;
        jb[i] = j;
    }
    // K rotation: workgroup tn walks its K tiles starting at tile tn * rot_n (mod KT) and wraps
    // around.  Left alone, all workgroups read the same k range at the same time from rows that
    // lie a power of two apart, which concentrates the requests of the whole chip on a few
    // memory channels; started at different tiles they spread over all of them.  Only the
    // order of the sum over k changes.
    const int rot = (int)(((int64_t)tn * p.rot_n) % KT);
    auto issue = [&](int kt, int stage) {
        int kc = (kt < KT ? kt : KT - 1) + rot;          // past the end: refetch the last tile into a free stage
        if (kc >= KT) kc -= KT;
        char *st = lds + stage * C::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < C::A_PER_WAVE; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(ga[i] + (int64_t)kc * C::RB),
                                             (__attribute__((address_space(3))) void *)(st + ja[i] * 1024), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < C::B_PER_WAVE; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gb[i] + (int64_t)kc * C::RB),
                                             (__attribute__((address_space(3))) void *)(st + C::A_BYTES + jb[i] * 1024), 16, 0, 0);
    };

    // fragment addresses: lane reads tile row (lane % 16), chunk 4*kg + lane/16
    const int r16 = lane & 15, q = lane >> 4;
    const int a_row = r16 * C::RB;
    const int b_row = C::A_BYTES + (wave * 16 + r16) * C::RB;
    const int a_sw = r16, b_sw = (wave * 16 + r16) & 15;       // both equal r16; kept apart for clarity

    typedef float f32x4v __attribute__((ext_vector_type(4)));
    f32x4v acc = {0.0f, 0.0f, 0.0f, 0.0f};

    constexpr int P = C::NS - 1;
#pragma unroll
    for (int s = 0; s < P; ++s) issue(s, s);

    for (int kt0 = 0; kt0 < KT; kt0 += C::NS) {
#pragma unroll
        for (int s = 0; s < C::NS; ++s) {
            const int kt = kt0 + s;
            if (kt < KT) {
                wait_vmcnt<(P - 1) * C::DLOADS>();
                lds_barrier();
                issue(kt + P, (s + P) % C::NS);
                const char *st = lds + s * C::STAGE_BYTES;
#pragma unroll
                for (int kg = 0; kg < C::KSTEP / 32; ++kg) {
                    const int c = kg * 4 + q;
                    const u32x4 af = *(const u32x4 *)(st + a_row + (((c & ~15) | ((c & 15) ^ a_sw)) << 4));
                    const u32x4 bf = *(const u32x4 *)(st + b_row + (((c & ~15) | ((c & 15) ^ b_sw)) << 4));
                    if (C::DT == DT_BF16)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, bf),
                                                                      __builtin_bit_cast(bf16x8, af), acc, 0, 0, 0);
                    else
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, bf),
                                                                     __builtin_bit_cast(f16x8, af), acc, 0, 0, 0);
                }
            }
        }
    }
    wait_vmcnt<0>();        // the refetches past the end must land before this workgroup's LDS is given away

    // acc[v] <-> m = lane % 16, n = n0 + wave*16 + 4*(lane/16) + v
    const int64_t m = r16;
    const int64_t n = n0 + wave * 16 + q * 4;
    const int64_t left = p.N - n;
    if (m < p.M && left > 0) {
        const int nvalid = left >= 4 ? 4 : (int)left;
        const float x[4] = {acc[0], acc[1], acc[2], acc[3]};
        if (p.split > 1)
            store4<DT_F32>(p.ws + (int64_t)slice * p.M * p.N, m * p.N + n, x, 1.0f, 0.0f, p.flags & GF_WS_VEC, nvalid);
        else {
            if (p.flags & GF_C_F32)
                store4<DT_F32>(p.C, m * p.ldc + n, x, p.alpha, p.beta, p.flags & GF_C_VEC, nvalid, p.hook, m, n);
            else
                store4<C::DT>(p.C, m * p.ldc + n, x, p.alpha, p.beta, p.flags & GF_C_VEC, nvalid, p.hook, m, n);
        }
    }
}


// ---------------------------------------------------------------------------
// Register-streaming skinny kernel: no LDS, no barriers.  One wave owns 16 rows
// of the N x K operand over one K slice and streams them straight from global
// memory into MFMA operand registers, DEPTH iterations (of 64 k) ahead; the
// matching 16 x 64 pieces of the M x K operand come the same way and are shared
// between the waves of a CU by the L1 cache.  Every byte of the big operand is
// read once, by one wave, in row order.
//   lane l:  operand row l % 16,  k = k0 + 8*(l/16) .. +7   (first MFMA of the iteration)
//                                 k = k0 + 32 + 8*(l/16) .. +7   (second MFMA)
//   acc[v] <-> m = l % 16,  n = 16*rowgroup + 4*(l/16) + v
// ---------------------------------------------------------------------------
template <int DT_, int DEPTH_, int WAVES_>
struct SkinnyRegCfg {
    static constexpr int DT = DT_;
    static_assert(DT_ != DT_F32, "16-bit storage only");
    static constexpr int DEPTH = DEPTH_, NW = WAVES_, NT = WAVES_ * 64;
    static constexpr int KIT = 64;                      // k per iteration
    static constexpr int LDS_BYTES = 0;
};

template <class C>
__global__ __launch_bounds__(C::NT) void skinny_reg_kernel(const GemmArgs p)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int groups = p.tiles_n;                       // row groups of 16 along N
    const int64_t w = (int64_t)blockIdx.x * C::NW + wave;
    if (w >= (int64_t)groups * p.split) return;         // whole wave leaves; there are no barriers
    const int g = (int)(w % groups), slice = (int)(w / groups);
    const int r16 = lane & 15, q = lane >> 4;

    const int it_begin = slice * p.ktiles_per_slice;
    int it_end = it_begin + p.ktiles_per_slice;
    if (it_end > p.ktiles_total) it_end = p.ktiles_total;
    const int NIT = it_end - it_begin;                  // >= 1

    int64_t brow = (int64_t)g * 16 + r16;
    if (brow > p.N - 1) brow = p.N - 1;                 // duplicates of a valid row; never stored
    int64_t arow = r16;
    if (arow > p.M - 1) arow = p.M - 1;
    const char *bp = (const char *)p.B + (brow * p.ldb + (int64_t)it_begin * C::KIT + q * 8) * 2;
    const char *ap = (const char *)p.A + (arow * p.lda + (int64_t)it_begin * C::KIT + q * 8) * 2;

    u32x4 b_lo[C::DEPTH], b_hi[C::DEPTH], a_lo[C::DEPTH], a_hi[C::DEPTH];
    auto load_it = [&](int it, int slot) {
        const int ic = it < NIT ? it : NIT - 1;         // past the end: reload the last iteration, unused
        const int64_t off = (int64_t)ic * (C::KIT * 2);
        b_lo[slot] = *(const u32x4 *)(bp + off);
        b_hi[slot] = *(const u32x4 *)(bp + off + 64);
        a_lo[slot] = *(const u32x4 *)(ap + off);
        a_hi[slot] = *(const u32x4 *)(ap + off + 64);
    };
    typedef float f32x4v __attribute__((ext_vector_type(4)));
    f32x4v acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
    auto mma = [&](f32x4v &acc, const u32x4 &bf, const u32x4 &af) {
        if (C::DT == DT_BF16)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, bf), __builtin_bit_cast(bf16x8, af), acc, 0, 0, 0);
        else
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, bf), __builtin_bit_cast(f16x8, af), acc, 0, 0, 0);
    };

#pragma unroll
    for (int d = 0; d < C::DEPTH; ++d) load_it(d, d);
    for (int it0 = 0; it0 < NIT; it0 += C::DEPTH) {
#pragma unroll
        for (int d = 0; d < C::DEPTH; ++d) {
            const int it = it0 + d;
            if (it < NIT) {
                mma(acc0, b_lo[d], a_lo[d]);
                mma(acc1, b_hi[d], a_hi[d]);
                load_it(it + C::DEPTH, d);
            }
        }
    }

    const int64_t m = r16;
    const int64_t n = (int64_t)g * 16 + q * 4;
    const int64_t left = p.N - n;
    if (m < p.M && left > 0) {
        const int nvalid = left >= 4 ? 4 : (int)left;
        const float x[4] = {acc0[0] + acc1[0], acc0[1] + acc1[1], acc0[2] + acc1[2], acc0[3] + acc1[3]};
        if (p.split > 1)
            store4<DT_F32>(p.ws + (int64_t)slice * p.M * p.N, m * p.N + n, x, 1.0f, 0.0f, p.flags & GF_WS_VEC, nvalid);
        else {
            if (p.flags & GF_C_F32)
                store4<DT_F32>(p.C, m * p.ldc + n, x, p.alpha, p.beta, p.flags & GF_C_VEC, nvalid, p.hook, m, n);
            else
                store4<C::DT>(p.C, m * p.ldc + n, x, p.alpha, p.beta, p.flags & GF_C_VEC, nvalid, p.hook, m, n);
        }
    }
}

}  // namespace peak
