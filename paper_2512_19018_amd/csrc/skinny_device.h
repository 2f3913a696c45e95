// Streaming kernel for skinny products (M <= 64, both operands running along K
// in memory): the N x K operand is read from HBM exactly once and that read is
// the whole cost, so the kernel is built around keeping many direct-to-LDS
// loads in flight per CU, not around the matrix cores (one 16x16 MFMA per
// 16 rows of either operand and 32 k - 16 k in fp32 - still does the arithmetic).
// K is cut into slices (the paper's Split-K,
// Section 4.1 Table 2) so that enough workgroups stream at once; the fp32
// partials are summed in slice order by splitk_reduce_kernel.
#pragma once

#include "gemm_device.h"
#include "planner.h"

namespace peak {

// MBLK: 16-row blocks of the M x K operand (M <= 16 * MBLK); each wave multiplies all of them
// with its 16 rows of the other operand.
// KW: waves per 16 rows of the N x K operand.  With 2, the two take the even and the odd rounds of
// fragment reads of every stage and their sums are added in LDS at the end (even rounds first): where
// the MFMAs are the bound (fp32 with several blocks) a SIMD then has a second wave to issue from while
// the first waits for its fragments.
// PIPE: the loop is software-pipelined across the stage's barrier (see the kernel).
template <int DT_, int BN_, int KSTEP_, int NS_, int MBLK_ = 1, int KW_ = 1, int PIPE_ = 0>
struct SkinnyCfg {
    static constexpr int DT = DT_;
    static constexpr bool PIPE = PIPE_ != 0;
    static constexpr int ESZ = DT_ == DT_F32 ? 4 : 2, EPC = 16 / ESZ;
    static constexpr int MBLK = MBLK_, KW = KW_;
    static constexpr int KMMA = 4 * EPC;                  // k per round of fragment reads: 4 chunks of 16 bytes
    static constexpr int BM = 16 * MBLK_, BN = BN_, KSTEP = KSTEP_, NS = NS_;
    static constexpr int RB = KSTEP_ * ESZ;               // bytes per tile row and stage
    static constexpr int CPR = RB / 16;                   // 16-byte chunks per tile row
    static constexpr int NWC = BN_ / 16;                  // wave columns: one per 16 rows of the N x K operand
    static constexpr int NW = NWC * KW_;
    static constexpr int NT = NW * 64;
    static_assert(KW_ == 1 || (KW_ == 2 && (KSTEP_ / KMMA) % 2 == 0), "one or two waves per 16 rows; an even number of rounds per stage");
    static_assert(KW_ == 1 || NWC * MBLK_ * 1024 <= (BM + BN_) * RB, "the odd waves' sums fit the first stage");
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
    const int wcol = C::KW == 1 ? wave : wave % C::NWC;        // which 16 rows of the N x K operand
    const int kpar = C::KW == 1 ? 0 : wave / C::NWC;           // which rounds of a stage: kg = KW * i + kpar
    const int a_row = r16 * C::RB;
    const int b_row = C::A_BYTES + (wcol * 16 + r16) * C::RB;
    const int a_sw = r16, b_sw = (wcol * 16 + r16) & 15;       // both equal r16; kept apart for clarity

    typedef float f32x4v __attribute__((ext_vector_type(4)));
    f32x4v acc[C::MBLK];
#pragma unroll
    for (int mb = 0; mb < C::MBLK; ++mb) acc[mb] = f32x4v{0.0f, 0.0f, 0.0f, 0.0f};

    if constexpr (C::PIPE) {
        // Where the MFMAs are the bound, the stage's barrier must not drain the matrix pipe: the fragments of a
        // stage's last round are read before the barrier, and that round's MFMAs are issued after it, one between
        // each two of what the barrier releases - the loads that refill this very stage (every wave has its last
        // fragments in registers, so the stage is free) and the reads of the next stage's first fragments.
        constexpr int G = C::KSTEP / C::KMMA / C::KW;       // rounds per stage and wave
        static_assert(G % 2 == 0, "two fragment sets take turns: an even number of rounds per stage");
        constexpr int NFR = 1 + C::MBLK;                     // fragment reads per round
        constexpr int NMF = C::DT == DT_F32 ? 4 * C::MBLK : C::MBLK;   // MFMAs per round
        u32x4 bfr[2], afr[2][C::MBLK];
        auto read_one = [&](const char *st, int kg, int f, u32x4 &bf, u32x4 (&af)[C::MBLK]) {
            const int c = (kg * C::KW + kpar) * 4 + q;
            if (f == 0) bf = *(const u32x4 *)(st + b_row + (((c & ~15) | ((c & 15) ^ b_sw)) << 4));
            else af[f - 1] = *(const u32x4 *)(st + a_row + (f - 1) * 16 * C::RB + (((c & ~15) | ((c & 15) ^ a_sw)) << 4));
        };
        auto mfma_one = [&](int j, const u32x4 &bf, const u32x4 (&af)[C::MBLK]) {
            if constexpr (C::DT == DT_F32) {
                const int e = j / C::MBLK, mb = j % C::MBLK;          // the blocks take turns
                const uint32_t be = bf[e], ae = af[mb][e];
                acc[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(__builtin_bit_cast(float, be), __builtin_bit_cast(float, ae), acc[mb], 0, 0, 0);
            } else if constexpr (C::DT == DT_BF16) {
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, bf), __builtin_bit_cast(bf16x8, af[j]), acc[j], 0, 0, 0);
            } else {
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, bf), __builtin_bit_cast(f16x8, af[j]), acc[j], 0, 0, 0);
            }
        };
        auto issue_one = [&](int kc, int stage, int i) {
            char *st = lds + stage * C::STAGE_BYTES;
            if (i < C::A_PER_WAVE)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(ga[i] + (int64_t)kc * C::RB),
                                                 (__attribute__((address_space(3))) void *)(st + ja[i] * 1024), 16, 0, 0);
            else
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gb[i - C::A_PER_WAVE] + (int64_t)kc * C::RB),
                                                 (__attribute__((address_space(3))) void *)(st + C::A_BYTES + jb[i - C::A_PER_WAVE] * 1024), 16, 0, 0);
        };
#pragma unroll
        for (int s = 0; s < C::NS; ++s) issue(s, s);       // every stage of the ring
        wait_vmcnt<(C::NS - 1) * C::DLOADS>();
        lds_barrier();
#pragma unroll
        for (int f = 0; f < NFR; ++f) read_one(lds, 0, f, bfr[0], afr[0]);
        for (int kt0 = 0; kt0 < KT; kt0 += C::NS) {
#pragma unroll
            for (int s = 0; s < C::NS; ++s) {
                const int kt = kt0 + s;
                if (kt < KT) {
                    const char *st = lds + s * C::STAGE_BYTES;
#pragma unroll
                    for (int kg = 0; kg + 1 < G; ++kg) {
                        // the next round's fragments behind this round's first MFMAs, so that nothing waits for them
                        constexpr int NS1 = NMF > NFR ? NMF : NFR;
                        __builtin_amdgcn_sched_barrier(0);       // (... or lift one above the wait for this round's)
#pragma unroll
                        for (int j = 0; j < NS1; ++j) {
                            if (j < NMF) mfma_one(j, bfr[kg & 1], afr[kg & 1]);
                            if (j < NFR) {
                                read_one(st, kg + 1, j, bfr[(kg + 1) & 1], afr[(kg + 1) & 1]);
                                __builtin_amdgcn_sched_barrier(0);   // (the compiler would sink the reads to the round's end)
                            }
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);       // (this round's MFMAs stay ahead of the barrier: they cover its reads)
                    wait_vmcnt<(C::NS - 2) * C::DLOADS>();   // tile kt + 1 has landed (this wave's part)
                    lds_barrier();                           // ... everybody's, and nobody reads this stage any more
                    int kc = (kt + C::NS < KT ? kt + C::NS : KT - 1) + rot;   // past the end: refetch the last tile
                    if (kc >= KT) kc -= KT;
                    const char *stn = lds + ((s + 1) % C::NS) * C::STAGE_BYTES;
                    constexpr int NSLOT = NMF > C::DLOADS + NFR ? NMF : C::DLOADS + NFR;
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < NSLOT; ++j) {
                        if (j < NMF) mfma_one(j, bfr[(G - 1) & 1], afr[(G - 1) & 1]);
                        if (j < NFR) read_one(stn, 0, j, bfr[0], afr[0]);
                        else if (j - NFR < C::DLOADS) issue_one(kc, s, j - NFR);
                        if (j < NFR + C::DLOADS) __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        }
    } else {
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
                for (int kg = 0; kg < C::KSTEP / C::KMMA / C::KW; ++kg) {
                    const int c = (kg * C::KW + kpar) * 4 + q;
                    const u32x4 bf = *(const u32x4 *)(st + b_row + (((c & ~15) | ((c & 15) ^ b_sw)) << 4));
                    u32x4 af[C::MBLK];
#pragma unroll
                    for (int mb = 0; mb < C::MBLK; ++mb)
                        af[mb] = *(const u32x4 *)(st + a_row + mb * 16 * C::RB + (((c & ~15) | ((c & 15) ^ a_sw)) << 4));
                    if constexpr (C::DT == DT_F32) {
                        // fp32: the chunk holds 4 k per lane; MFMA e takes element e of both chunks, so its four k
                        // are 16 * kg + 4 * (lane / 16) + e over the four lane groups.  The blocks take turns, so
                        // that an MFMA does not follow the one whose result it adds to.
#pragma unroll
                        for (int e = 0; e < 4; ++e)
#pragma unroll
                            for (int mb = 0; mb < C::MBLK; ++mb) {
                                const uint32_t be = bf[e], ae = af[mb][e];      // (a bit cast straight from the vector's element takes element 0)
                                acc[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(__builtin_bit_cast(float, be),
                                                                               __builtin_bit_cast(float, ae), acc[mb], 0, 0, 0);
                            }
                    } else {
#pragma unroll
                        for (int mb = 0; mb < C::MBLK; ++mb) {
                            if constexpr (C::DT == DT_BF16)
                                acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, bf),
                                                                                  __builtin_bit_cast(bf16x8, af[mb]), acc[mb], 0, 0, 0);
                            else
                                acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, bf),
                                                                                 __builtin_bit_cast(f16x8, af[mb]), acc[mb], 0, 0, 0);
                        }
                    }
                }
            }
        }
    }
    }
    wait_vmcnt<0>();        // the refetches past the end must land before this workgroup's LDS is given away

    if constexpr (C::KW == 2) {
        // the odd rounds' sums go through LDS to the wave that holds the even rounds' and stores
        lds_barrier();                                      // every wave is through its last stage, no load is under way
        f32x4v *red = (f32x4v *)lds + (wcol * C::MBLK) * 64 + lane;
        if (kpar == 1) {
#pragma unroll
            for (int mb = 0; mb < C::MBLK; ++mb) red[mb * 64] = acc[mb];
        }
        lds_barrier();
        if (kpar == 1) return;
#pragma unroll
        for (int mb = 0; mb < C::MBLK; ++mb) acc[mb] += red[mb * 64];
    }

    // acc[mb][v] <-> m = 16*mb + lane % 16, n = n0 + wcol*16 + 4*(lane/16) + v
    const int64_t n = n0 + wcol * 16 + q * 4;
    const int64_t left = p.N - n;
#pragma unroll
    for (int mb = 0; mb < C::MBLK; ++mb) {
        const int64_t m = mb * 16 + r16;
        if (m < p.M && left > 0) {
            const int nvalid = left >= 4 ? 4 : (int)left;
            const float x[4] = {acc[mb][0], acc[mb][1], acc[mb][2], acc[mb][3]};
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

// ---------------------------------------------------------------------------
// Streaming kernel for skinny products whose N-side operand is stored K x N
// (B with transB = 0; A runs along K): the same idea, with the big operand kept
// in LDS as [k][n] rows of 512 bytes.  A workgroup owns 512 bytes of every k-row
// (256 columns in 16 bits, 128 in fp32) over one K slice; a stage is 128 bytes of
// K per row of A (64 k in 16 bits, 32 in fp32).  All workgroups walk the same
// k-rows at the same time, which are contiguous in memory across the workgroups,
// so the requests spread over the memory channels without a rotation.
//   16 bits: the N-side fragments of the 16x16x32 MFMA come from transposing reads
//            (ds_read_b64_tr_b16), with the tile's chunks placed as in the 16x16x32 tiled kernels.
//   fp32:    16x16x4 MFMA; a lane needs one element of a k-row, read as such; chunk c of
//            k-row k sits at c ^ 4 * ((k >> 2) & 3), so the four k-rows of one read fall
//            into four different groups of 16 banks.
// ---------------------------------------------------------------------------
template <int DT_, int NS_, int MBLK_, int NW_ = 8>
struct SkinnyKnCfg {
    static constexpr int DT = DT_;
    static constexpr int ESZ = DT_ == DT_F32 ? 4 : 2, EPC = 16 / ESZ;
    static constexpr int MBLK = MBLK_, NS = NS_, NW = NW_, NT = NW_ * 64;
    static constexpr int RB = 128;                        // bytes of K per stage row of A
    static constexpr int CPR = RB / 16;
    static constexpr int BK = RB / ESZ, KSTEP = BK;       // k per stage
    static constexpr int ROWB = 512;                      // bytes per k-row of the N-side tile
    static constexpr int BM = 16 * MBLK_, BN = ROWB / ESZ;
    static constexpr int NBW = BN / 16 / NW_;             // 16-column blocks per wave
    static_assert(NBW >= 1 && NBW * 16 * NW_ == BN, "whole blocks per wave");
    static constexpr int A_BYTES = BM * RB, B_BYTES = BK * ROWB;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = STAGE_BYTES * NS_;
    static constexpr int A_INST = BM * CPR / 64;          // 1024-byte wave loads per stage of A
    static_assert(A_INST % NW_ == 0 || NW_ % A_INST == 0, "A loads split evenly");
    static constexpr int A_PER_WAVE = A_INST >= NW_ ? A_INST / NW_ : 1;   // waves beyond A_INST repeat one of another wave
    // chunk c of A's tile row r sits at c ^ swizzle(r): a fragment read's step takes 8 rows at chunk c and the
    // same rows at chunk c + 2; bits 0 and 2 separate the rows of one parity, bit 1 is left to the chunk
    static __device__ __forceinline__ int swizzle(int r) { return ((r >> 1) & 1) | (((r >> 2) & 1) << 2); }
    static __device__ __forceinline__ int kn_swizzle(int k)
    {
        if constexpr (DT_ == DT_F32) return 4 * ((k >> 2) & 3);
        else return (4 * (k & 3)) ^ (2 * (((k >> 3) ^ (k >> 4)) & 1));
    }
};

template <class C>
__global__ __launch_bounds__(C::NT) void skinny_kn_kernel(const GemmArgs p)
{
    __shared__ __attribute__((aligned(1024))) char lds[C::LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tn = blockIdx.x % p.tiles_n, slice = blockIdx.x / p.tiles_n;
    const int64_t n0 = (int64_t)tn * C::BN;
    const int r16 = lane & 15, q = lane >> 4;

    const int kt_begin = slice * p.ktiles_per_slice;
    int kt_end = kt_begin + p.ktiles_per_slice;
    if (kt_end > p.ktiles_total) kt_end = p.ktiles_total;
    const int KT = kt_end - kt_begin;
    const int64_t kbase = (int64_t)kt_begin * C::KSTEP;

    // A: this lane's direct loads at the slice's first k
    const char *ga[C::A_PER_WAVE];
    int ja[C::A_PER_WAVE];
#pragma unroll
    for (int i = 0; i < C::A_PER_WAVE; ++i) {
        const int j = (wave + C::NW * i) % C::A_INST;
        const int row = j * (64 / C::CPR) + lane / C::CPR, pos = lane % C::CPR;
        const int c = pos ^ C::swizzle(row);
        int64_t gr = row;
        if (gr > p.M - 1) gr = p.M - 1;
        ga[i] = (const char *)p.A + (gr * p.lda + kbase + (int64_t)c * C::EPC) * C::ESZ;
        ja[i] = j;
    }
    LoaderDirectKN<C, C::BN, true> nB;
    nB.init(p.B, p.ldb, n0, p.N, kbase, p.K, C::BK, wave, lane);
    constexpr int LB = LoaderDirectKN<C, C::BN, true>::PER_WAVE;
    static_assert(LoaderDirectKN<C, C::BN, true>::NINST % C::NW == 0, "every wave issues the same number of loads");
    constexpr int DLOADS = C::A_PER_WAVE + LB;

    auto issue = [&](int kt, int stage) {
        const int kc = kt < KT ? kt : KT - 1;             // past the end: refetch the last tile into a free stage
        char *st = lds + stage * C::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < C::A_PER_WAVE; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(ga[i] + (int64_t)kc * C::RB),
                                             (__attribute__((address_space(3))) void *)(st + ja[i] * 1024), 16, 0, 0);
        nB.template issue_at<0, 1, false>(st + C::A_BYTES, nB.soffset_of(kc), false, wave);
    };

    // fragment addresses within a stage
    //   A: lane reads tile row 16 mb + lane % 16, chunk 4 g + lane / 16 of k-group g (a quarter of the stage's K)
    const int a_addr0 = r16 * C::RB + ((q ^ C::swizzle(r16)) << 4);          // g = 0; g = 1 flips chunk bit 2
    const int a_addr1 = r16 * C::RB + (((4 + q) ^ C::swizzle(r16)) << 4);
    //   N side, 16 bits: see the 16x16x32 tiled kernels (k-rows 8 q + r16 / 4 and four rows on, 4 columns per lane)
    //   N side, fp32: element (k-row 16 g + 4 q + e, column block's lane % 16)
    int b_addr[C::NBW];
#pragma unroll
    for (int i = 0; i < C::NBW; ++i) {
        if constexpr (C::DT == DT_F32) {
            const int col = (wave * C::NBW + i) * 16 + r16;
            b_addr[i] = C::A_BYTES + (4 * q) * C::ROWB + (((col >> 2) ^ C::kn_swizzle(4 * q)) << 4) + (col & 3) * 4;
        } else {
            const int krow = 8 * q + (r16 >> 2);
            const int col = (wave * C::NBW + i) * 16 + 4 * (r16 & 3);
            b_addr[i] = C::A_BYTES + krow * C::ROWB + (((col >> 3) ^ C::kn_swizzle(krow)) << 4) + (r16 & 1) * 8;
        }
    }
    const uint32_t lds_b0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;

    typedef float f32x4v __attribute__((ext_vector_type(4)));
    f32x4v acc[C::MBLK][C::NBW];
#pragma unroll
    for (int mb = 0; mb < C::MBLK; ++mb)
#pragma unroll
        for (int i = 0; i < C::NBW; ++i) acc[mb][i] = f32x4v{0.0f, 0.0f, 0.0f, 0.0f};

    constexpr int P = C::NS - 1;
#pragma unroll
    for (int s = 0; s < P; ++s) issue(s, s);

    for (int kt0 = 0; kt0 < KT; kt0 += C::NS) {
        static_for<C::NS>([&](auto sc) {
            constexpr int s = decltype(sc)::value;
            const int kt = kt0 + s;
            if (kt < KT) {
                wait_vmcnt<(P - 1) * DLOADS>();
                lds_barrier();
                issue(kt + P, (s + P) % C::NS);
                const char *st = lds + s * C::STAGE_BYTES;
                u32x4 af[2][C::MBLK];
#pragma unroll
                for (int mb = 0; mb < C::MBLK; ++mb) {
                    af[0][mb] = *(const u32x4 *)(st + a_addr0 + mb * 16 * C::RB);
                    af[1][mb] = *(const u32x4 *)(st + a_addr1 + mb * 16 * C::RB);
                }
                if constexpr (C::DT == DT_F32) {
                    float bv[2][4][C::NBW];
#pragma unroll
                    for (int g = 0; g < 2; ++g)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
#pragma unroll
                            for (int i = 0; i < C::NBW; ++i) bv[g][e][i] = *(const float *)(st + b_addr[i] + (16 * g + e) * C::ROWB);
#pragma unroll
                    for (int g = 0; g < 2; ++g)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
#pragma unroll
                            for (int i = 0; i < C::NBW; ++i)
#pragma unroll
                                for (int mb = 0; mb < C::MBLK; ++mb) {
                                    const uint32_t ae = af[g][mb][e];
                                    acc[mb][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(bv[g][e][i], __builtin_bit_cast(float, ae),
                                                                                      acc[mb][i], 0, 0, 0);
                                }
                } else {
                    // the transposing reads go out as assembly (the compiler would put a wait for every outstanding
                    // direct-to-LDS load in front of them); one wait for everything asked of LDS hands them over
                    u32x2 lo[2][C::NBW], hi[2][C::NBW];
                    static_for<2>([&](auto gc) {
                        constexpr int g = decltype(gc)::value;
                        static_for<C::NBW>([&](auto ic) {
                            constexpr int i = decltype(ic)::value;
                            constexpr int off = g * 32 * C::ROWB;               // (the immediate holds 16 bits: the stage goes into the address)
                            const uint32_t a0 = lds_b0 + b_addr[i] + s * C::STAGE_BYTES;
                            u32x2 &l = lo[g][i], &h = hi[g][i];
                            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(l) : "v"(a0), "n"(off) : "memory");
                            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(h) : "v"(a0), "n"(off + 4 * C::ROWB) : "memory");
                        });
                    });
                    __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));
#pragma unroll
                    for (int g = 0; g < 2; ++g)
#pragma unroll
                        for (int i = 0; i < C::NBW; ++i) {
                            u32x2 &l = lo[g][i], &h = hi[g][i];
                            asm volatile("" : "+v"(l), "+v"(h));
                            const u32x4 bf = u32x4{l[0], l[1], h[0], h[1]};
#pragma unroll
                            for (int mb = 0; mb < C::MBLK; ++mb) {
                                if constexpr (C::DT == DT_BF16)
                                    acc[mb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, bf),
                                                                                         __builtin_bit_cast(bf16x8, af[g][mb]), acc[mb][i], 0, 0, 0);
                                else
                                    acc[mb][i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, bf),
                                                                                        __builtin_bit_cast(f16x8, af[g][mb]), acc[mb][i], 0, 0, 0);
                            }
                        }
                }
            }
        });
    }
    wait_vmcnt<0>();        // the refetches past the end must land before this workgroup's LDS is given away

    // acc[mb][i][v] <-> m = 16 mb + lane % 16, n = n0 + 16 (wave NBW + i) + 4 (lane / 16) + v
#pragma unroll
    for (int mb = 0; mb < C::MBLK; ++mb)
#pragma unroll
        for (int i = 0; i < C::NBW; ++i) {
            const int64_t m = mb * 16 + r16;
            const int64_t n = n0 + (wave * C::NBW + i) * 16 + q * 4;
            const int64_t left = p.N - n;
            if (m < p.M && left > 0) {
                const int nvalid = left >= 4 ? 4 : (int)left;
                const float x[4] = {acc[mb][i][0], acc[mb][i][1], acc[mb][i][2], acc[mb][i][3]};
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
}

}  // namespace peak
