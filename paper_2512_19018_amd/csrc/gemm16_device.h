// Tiled kernel built on the 16x16x32 MFMA (v_mfma_f32_16x16x32_{bf16,f16}) for
// 16-bit operands that both run along K in memory: 256x256 workgroup tile, four
// waves (one per SIMD) with a 128x128 wave tile each, i.e. 8 x 8 blocks of 16x16
// whose 256 accumulator registers sit in the accumulation half of the register
// file.  Measured on MI355X, the chip is power limited under a matrix load and
// this instruction does the same multiply-adds for less power than 32x32x16: an
// MFMA-only loop sustains about 14 % more with it, and a GEMM built on it holds a
// correspondingly higher clock at the same number of cycles.
//
// In the paper's vocabulary (Section 2.2, Section 4.1 Table 2) this is the
// Tensor-Core / Tensor-Tiling step taken with another tile of the matrix unit;
// staging (Pipelining: three A stages and two B stages of 64 k, filled by
// direct-to-LDS buffer loads), the XOR placement of 16-byte chunks (Offset), the
// tile order (Block-Swizzle), Split-K slices and the epilogue are those of
// gemm_kernel.
#pragma once

#include "gemm_device.h"

namespace peak {

typedef float f32x4v __attribute__((ext_vector_type(4)));

template <int DT_>
struct Cfg16 {
    static_assert(DT_ == DT_F16 || DT_ == DT_BF16, "16-bit storage");
    static constexpr int DT = DT_;
    static constexpr int ESZ = 2, EPC = 8;
    static constexpr int BM = 256, BN = 256, RB = 128, CPR = 8, BK = 64;
    static constexpr int WAVES_M = 2, WAVES_N = 2, NW = 4, NT = 256;
    static constexpr int WTM = 128, WTN = 128;
    static constexpr int MB = WTM / 16, NB = WTN / 16;      // 16x16 blocks per wave tile
    static constexpr int KS = BK / 32;                      // MFMA k-steps per K tile
    static constexpr int NSA = 3, NSB = 2;
    static constexpr int A_BYTES = BM * RB, B_BYTES = BN * RB;
    static constexpr int LDS_BYTES = A_BYTES * NSA + B_BYTES * NSB;
    // Chunk c of tile row r sits at chunk position c ^ swizzle(r).  The swizzle depends on
    // r % 16 only, so the fragments of rows r, r + 16, r + 32, ... lie a constant 2 KB apart
    // and one address register serves all of them through the read's immediate offset.
    // A fragment read takes rows r0 .. r0 + 15 at one logical chunk: even rows share one half
    // of the 256-byte bank period, odd rows the other, and within a half the eight rows get
    // eight different chunk positions.
    static __device__ __forceinline__ int swizzle(int r) { return (r & 7) ^ ((r >> 3) & 1); }
};

template <class C>
__global__ __launch_bounds__(C::NT) void gemm16_kernel(const GemmArgs p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the kernel's symbol
    __shared__ __attribute__((aligned(1024))) char lds[C::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
    const int r16 = lane & 15, q = lane >> 4;

    const int tiles = p.tiles_m * p.tiles_n;
    const int bid = blockIdx.x;
    const int slice = __builtin_amdgcn_readfirstlane(bid / tiles);
    int tm, tn;
    tile_of_block(bid - slice * tiles, p.tiles_m, p.tiles_n, p.group_m, tm, tn);
    const int64_t m0 = (int64_t)tm * C::BM, n0 = (int64_t)tn * C::BN;

    const int kt_begin = slice * p.ktiles_per_slice;
    int kt_end = kt_begin + p.ktiles_per_slice;
    if (kt_end > p.ktiles_total) kt_end = p.ktiles_total;
    const int KT = __builtin_amdgcn_readfirstlane(kt_end - kt_begin);   // >= 1 by construction of the plan
    const int64_t kbase = (int64_t)kt_begin * C::BK;

    // acc[mb][nb][v] <-> m = 16 * mb + lane % 16,  n = 16 * nb + 4 * (lane / 16) + v   (within the wave tile):
    // the B tile's rows feed the instruction's row operand and the A tile's rows its column
    // operand, so a lane holds 4 consecutive n of one m
    f32x4v acc[C::MB][C::NB];
#pragma unroll
    for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) acc[mb][nb] = f32x4v{0.0f, 0.0f, 0.0f, 0.0f};

    // fragment of k-step ks: lane reads row (lane % 16) of its block, chunk 4 * ks + lane / 16
    // (8 k).  One address per operand and k-step; blocks and stages go into the immediate.
    int a_base[C::KS], b_base[C::KS];
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
        const int ra = wm * C::WTM + r16, rb = wn * C::WTN + r16;
        a_base[ks] = ra * C::RB + (((4 * ks + q) ^ C::swizzle(ra)) << 4);
        b_base[ks] = C::NSA * C::A_BYTES + rb * C::RB + (((4 * ks + q) ^ C::swizzle(rb)) << 4);
    }
    auto read_a = [&](auto stagec, auto ksc, auto ic) -> u32x4 {
        constexpr int off = decltype(stagec)::value * C::A_BYTES + decltype(ic)::value * 16 * C::RB;
        return *(const u32x4 *)(lds + a_base[decltype(ksc)::value] + off);
    };
    auto read_b = [&](auto stagec, auto ksc, auto ic) -> u32x4 {
        constexpr int off = decltype(stagec)::value * C::B_BYTES + decltype(ic)::value * 16 * C::RB;
        return *(const u32x4 *)(lds + b_base[decltype(ksc)::value] + off);
    };

    LoaderDirect<C, C::BM> dA;
    LoaderDirect<C, C::BN> dB;
    constexpr int LA = LoaderDirect<C, C::BM>::PER_WAVE, LB = LoaderDirect<C, C::BN>::PER_WAVE;
    static_assert(LoaderDirect<C, C::BM>::NINST % C::NW == 0 && LoaderDirect<C, C::BN>::NINST % C::NW == 0,
                  "every wave issues the same number of loads");
    const int tail_k = __builtin_amdgcn_readfirstlane((int)(p.K - (int64_t)(p.ktiles_total - 1) * C::BK));
    const int tail_tile = tail_k < C::BK ? p.ktiles_total - 1 - kt_begin : -1;   // relative to the slice
    dA.init(p.A, p.lda, m0, p.M, kbase, p.K, tail_k, wave, lane);
    dB.init(p.B, p.ldb, n0, p.N, kbase, p.K, tail_k, wave, lane);
    auto a_stage = [&](int s) { return lds + s * C::A_BYTES; };
    auto b_stage = [&](int s) { return lds + C::NSA * C::A_BYTES + s * C::B_BYTES; };
    // Loads of tile kt, part PART of the wave's LA (LB) instructions.  Past the end the last
    // tile is fetched again into a free stage, so the count in flight stays what the waits assume.
    auto issue_a = [&](int kt, int sa, auto part) {
        const int kr = kt < KT ? kt : KT - 1;
        dA.template issue<decltype(part)::value, LA>(a_stage(sa), kr, kr == tail_tile, wave);
    };
    auto issue_b = [&](int kt, int sb, auto part) {
        const int kr = kt < KT ? kt : KT - 1;
        dB.template issue<decltype(part)::value, LB>(b_stage(sb), kr, kr == tail_tile, wave);
    };

    // Main loop.  One wave per SIMD: nothing else hides this wave's stalls, so the order of
    // instructions is fixed by hand, one slot per MFMA (16 cycles): the MFMA, then at most one
    // fragment read of the next k-step or one load.
    //   k-step 0 of tile kt:  fragments of k-step 1;  first half of A's loads of tile kt+2
    //                         (its stage was released by the barrier of tile kt-1)
    //   k-step 1 of tile kt:  wait for own loads of tile kt+1, barrier (tile kt+1 complete, tile kt
    //                         read by everyone);  fragments of tile kt+1, k-step 0;  B's loads of
    //                         tile kt+2 into the stage tile kt has just left, rest of A's loads
    constexpr int NM = C::MB * C::NB;                        // MFMAs per k-step
    constexpr int NFR = C::MB + C::NB;                       // fragments per k-step
    static_assert(C::KS == 2 && LA % 2 == 0 && 2 * NFR <= NM, "slot plan below");
    u32x4 af[2][C::MB], bf[2][C::NB];
    // fragment f of a k-step in the order the MFMAs first need them: B0, A0 .. A7, B1 .. B7
    auto fetch_one = [&](auto sac, auto sbc, auto ksc, auto fc) {
        constexpr int f = decltype(fc)::value, set = decltype(ksc)::value;
        if constexpr (f == 0) bf[set][0] = read_b(sbc, ksc, IC<0>{});
        else if constexpr (f <= C::MB) af[set][f - 1] = read_a(sac, ksc, IC<f - 1>{});
        else bf[set][f - C::MB] = read_b(sbc, ksc, IC<f - C::MB>{});
    };
    auto mfma_one = [&](auto setc, auto jc) {
        constexpr int set = decltype(setc)::value, j = decltype(jc)::value;
        constexpr int nb = j / C::MB, mb = j % C::MB;
        f32x4v &c = acc[mb][nb];
        const u32x4 &b = bf[set][nb], &a = af[set][mb];
        if constexpr (C::DT == DT_BF16)
            asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(b), "v"(a));
        else
            asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(b), "v"(a));
    };
    static_for<NM>([&](auto jc) {                             // accumulators into AGPRs now
        constexpr int j = decltype(jc)::value;
        f32x4v &c = acc[j % C::MB][j / C::MB];
        asm volatile("" : "+a"(c));
    });
    asm volatile("s_nop 7\n\ts_nop 7" ::: "memory");

    constexpr int PENDING = LA / 2;                          // loads of the tile under way at its barrier
    static_for<LA>([&](auto pc) { issue_a(0, 0, pc); });
    static_for<LB>([&](auto pc) { issue_b(0, 0, pc); });
    wait_vmcnt<0>();
    lds_barrier();
    static_for<LB>([&](auto pc) { issue_b(1, 1, pc); });
    static_for<LA>([&](auto pc) { issue_a(1, 1, pc); });
    static_for<NFR>([&](auto fc) { fetch_one(IC<0>{}, IC<0>{}, IC<0>{}, fc); });
    constexpr int U = 6;                                     // tiles per trip: both stage indices static
    for (int kt0 = 0; kt0 < KT; kt0 += U) {
        static_for<U>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            constexpr int s = u % 2, sa = u % 3, sa1 = (sa + 1) % 3, sa2 = (sa + 2) % 3;
            const int kt = kt0 + u;
            if (kt < KT) {
                // k-step 0
                __builtin_amdgcn_sched_barrier(0);
                static_for<NM>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    mfma_one(IC<0>{}, jc);
                    if constexpr (j % 2 == 0 && j / 2 < NFR) fetch_one(IC<sa>{}, IC<s>{}, IC<1>{}, IC<j / 2>{});
                    if constexpr (j % 16 == 1 && j / 16 < LA / 2) issue_a(kt + 2, sa2, IC<j / 16>{});
                    __builtin_amdgcn_sched_barrier(0);
                });
                // k-step 1
                wait_vmcnt<PENDING>();                       // own loads of tile kt+1
                lds_barrier();                               // tile kt+1 complete, tile kt read
                __builtin_amdgcn_sched_barrier(0);
                static_for<NM>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    mfma_one(IC<1>{}, jc);
                    if constexpr (j % 2 == 0 && j / 2 < NFR) fetch_one(IC<sa1>{}, IC<1 - s>{}, IC<0>{}, IC<j / 2>{});
                    if constexpr (j % 4 == 1 && j / 4 < LB) issue_b(kt + 2, s, IC<j / 4>{});
                    if constexpr (j % 8 == 3 && j / 8 >= 4 && j / 8 - 4 < LA / 2) issue_a(kt + 2, sa2, IC<LA / 2 + j / 8 - 4>{});
                    __builtin_amdgcn_sched_barrier(0);
                });
            }
        });
    }
    // 16x16x32 MFMA: 4 passes of 4 cycles; an accumulator may be read 10 wait states after the issue
    asm volatile("s_nop 15" ::: "memory");
    static_for<NM>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        f32x4v &c = acc[j % C::MB][j / C::MB];
        asm volatile("" : "+a"(c));
    });
    wait_vmcnt<0>();    // refetches past the end must land before this workgroup's LDS is given away

    // Epilogue: slab s = rows 32 s .. 32 s + 31 of the wave tile = blocks 2 s and 2 s + 1.
    auto write_slab = [&](int sl, char *scr) {
        constexpr int SROW = C::WTN * 4 + 16;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb)
                *(f32x4v *)(scr + (16 * h + r16) * SROW + (nb * 16 + 4 * q) * 4) = acc[2 * sl + h][nb];
    };
    auto write16 = [&](int sl, char *scr16) {
        constexpr int SROW16 = C::WTN * 2 + 16;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb) {
                float x[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // out of the accumulation registers here, group by group
                    const float aj = acc[2 * sl + h][nb][j];
                    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x[j]) : "a"(aj));
                    x[j] *= p.alpha;
                }
                union { u32x2 u; _Float16 hh[4]; __bf16 bb[4]; } pk;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (C::DT == DT_F16) pk.hh[j] = (_Float16)x[j];
                    else pk.bb[j] = (__bf16)x[j];
                }
                const int grp = (nb * 4 + q) ^ h;            // 4-column group, swapped pairwise in rows 16..31
                *(u32x2 *)(scr16 + (16 * h + r16) * SROW16 + grp * 8) = pk.u;
            }
    };
    epilogue_slabs<C, C::WTM / 32>(p, lds, wave, lane, wm, wn, m0, n0, slice, write_slab, write16);
#endif
}

}  // namespace peak
