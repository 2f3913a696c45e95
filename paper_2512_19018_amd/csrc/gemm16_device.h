// Tiled kernel built on the 16x16x32 MFMA (v_mfma_f32_16x16x32_{bf16,f16}) for
// 16-bit operands in any of the four layouts: 256x256 workgroup tile, four
// waves (one per SIMD) with a 128x128 wave tile each, i.e. 8 x 8 blocks of 16x16
// whose 256 accumulator registers sit in the accumulation half of the register
// file; or, for mid-size problems, a 128x128 tile with 64x64 per wave, two
// workgroups to a CU or one that loads four K tiles ahead.  Measured on MI355X, the chip is power limited under a matrix load and
// this instruction does the same multiply-adds for less power than 32x32x16: an
// MFMA-only loop sustains about 14 % more with it, and a GEMM built on it holds a
// correspondingly higher clock at the same number of cycles.
//
// In the paper's vocabulary (Section 2.2, Section 4.1 Table 2) this is the
// Tensor-Core / Tensor-Tiling step taken with another tile of the matrix unit;
// staging (Pipelining: PF + 1 stages of A and PF of B, 64 k each, filled by
// direct-to-LDS buffer loads PF K tiles ahead), the XOR placement of 16-byte chunks (Offset), the
// tile order (Block-Swizzle), Split-K slices and the epilogue are those of
// gemm_kernel.  An operand that does not run along K in memory (A stored K x M,
// B stored K x N) is staged as it lies, [k][m] or [k][n] rows, and its fragments
// come back through the transposing LDS read (the paper's Transpose, done by the
// LDS hardware on the way out instead of in registers on the way in).
#pragma once

#include "gemm_device.h"

namespace peak {

typedef float f32x4v __attribute__((ext_vector_type(4)));

constexpr int A_BYTES_OF(int tile, int bk = 64) { return tile * bk * 2; }    // one stage of one operand: tile rows x BK k x 2 bytes

// TILE: 256 (the large problems: one workgroup per CU, one wave per SIMD, 128x128 per wave) or
// 128 (mid-size problems: 64x64 per wave, 80 KB of LDS and half the registers, so two workgroups
// share a CU and cover each other's waits)
// PF: prefetch distance in K tiles (the loads of tile kt + PF go out during tile kt): PF + 1 stages of A,
// PF of B.  2 for the large tile, whose K tile takes 2048 cycles of MFMAs; 4 for the small tile when a
// workgroup has its CU to itself (512 cycles per K tile cover a fraction of a load's latency: measured 532
// cycles of waiting per K tile at bf16 2048^3 with a distance of 2)
// TILE_N: columns of the tile when it is not square (256 x 128: problems that fill the chip with neither
// the 256 x 256 nor the 128 x 128 tile, and whose wave tile of 128 x 64 still spares the LDS)
// BK: k per stage, 64 or 128.  128 (the 128 x 128 tile only: 3 + 2 stages of 32 KB) halves the barriers and waits
// per multiply-add and takes 256 bytes of a row from memory at a time instead of 128.
template <int DT_, bool A_KM_ = false, bool B_KN_ = false, int TILE_ = 256, int PF_ = 2, int TILE_N_ = TILE_, int BK_ = 64>
struct Cfg16 {
    static_assert(DT_ == DT_F16 || DT_ == DT_BF16, "16-bit storage");
    static_assert((TILE_ == 256 || TILE_ == 128) && (TILE_N_ == 256 || TILE_N_ == 128), "workgroup tile");
    static constexpr int DT = DT_;
    static constexpr bool A_KM = A_KM_;                      // A stored K x M: staged as [k][m] rows
    static constexpr bool B_KN = B_KN_;                      // B stored K x N: staged as [k][n] rows
    static constexpr int ESZ = 2, EPC = 8;
    static_assert(BK_ == 64 || BK_ == 128, "k per stage");
    static constexpr int BM = TILE_, BN = TILE_N_, RB = BK_ * 2, CPR = RB / 16, BK = BK_;
    static constexpr int WAVES_M = 2, WAVES_N = 2, NW = 4, NT = 256;
    static constexpr int PF = PF_;
    static constexpr int WAVES_PER_EU = PF_ == 2 && TILE_ == 128 && TILE_N_ == 128 && BK_ == 64 ? 2 : 1;   // workgroups per CU the register budget is cut for
    static constexpr int WTM = BM / 2, WTN = BN / 2;
    static constexpr int MB = WTM / 16, NB = WTN / 16;      // 16x16 blocks per wave tile
    static constexpr int KS = BK / 32;                      // MFMA k-steps per K tile
    static constexpr int NSA = PF_ + 1, NSB = PF_;
    static_assert(PF_ >= 2 && A_BYTES_OF(TILE_, BK_) * NSA + A_BYTES_OF(TILE_N_, BK_) * NSB <= 160 * 1024, "stages fit the LDS");
    static constexpr int A_BYTES = BM * RB, B_BYTES = BN * RB;
    static constexpr int LDS_BYTES = A_BYTES * NSA + B_BYTES * NSB;
    // Chunk c of tile row r sits at chunk position c ^ swizzle(r).  The swizzle depends on
    // r % 16 only, so the fragments of rows r, r + 16, r + 32, ... lie a constant 2 KB apart
    // and one address register serves all of them through the read's immediate offset.
    // A fragment read has lane l on row r0 + l % 16, logical chunk c0 + l / 16.  The LDS takes
    // a 16-byte read in four steps of 16 lanes, lanes 8 i .. 8 i + 7 together with lanes
    // 32 + 8 i .. 32 + 8 i + 7 (measured: a swizzle that is conflict-free for 16 consecutive
    // lanes but not for these groups showed a bank conflict on every read): eight consecutive
    // rows, each at chunks c and c + 2.  Rows two apart share the banks of one half of the
    // 256-byte bank period, so the four rows of a half must be given four chunk positions
    // whose partners under "^ 2" are four others: bit 1 of the swizzle is the same for the
    // eight rows of a group (and differs between the two groups of a block, which keeps
    // sixteen consecutive lanes conflict-free as well), bits 0 and 2 count the row pairs.
    // With 256-byte rows (BK = 128) all rows start in the same bank and a step's 8 rows x 2 chunks must take all
    // 16 positions of a row: bits 0, 2 and 3 count the rows of a group, bit 1 again tells the two groups apart.
    static __device__ __forceinline__ int swizzle(int r)
    {
        if constexpr (BK_ == 64) return ((r >> 1) & 1) | (((r >> 2) & 1) << 2) | (((r >> 3) & 1) << 1);
        else return (r & 1) | (((r >> 1) & 1) << 2) | (((r >> 2) & 1) << 3) | (((r >> 3) & 1) << 1);
    }
    // Tiles kept as [k][x] rows (512 bytes each, so all rows start in the same bank): chunk c of
    // row k sits at c ^ kn_swizzle(k).  A transposing read has its four groups of 16 lanes on
    // k-rows 8 q .. 8 q + 3 (q = lane / 16), 32 bytes of each.  4 * (k & 3) sends the four rows of
    // a group to four different 64-byte bank groups; the second term moves the rows of groups
    // q = 1 and q = 2 into the other 32-byte half, so that whichever two groups the LDS takes in
    // one step (0 with 1 and 2 with 3, or 0 with 2 and 1 with 3) miss each other.
    static __device__ __forceinline__ int kn_swizzle(int k) { return (4 * (k & 3)) ^ (2 * (((k >> 3) ^ (k >> 4)) & 1)); }
};

// Slot plan of the main loop: which fragment read (0 .. 15 of the next k-step), which of A's
// loads (first half in k-step 0, second half in k-step 1, after the tile's barrier) and which
// of B's loads (k-step 1) follows MFMA j of a k-step; -1: none.  A read after every other MFMA
// of the first half, loads in between and after.  Measured at bf16 8192^3 against this plan
// (1503 TFLOP/s in that run): reads after each of the first 16 MFMAs and the loads after them
// 1371, all loads in the second half of the k-step 1410, one load after every 8th MFMA
// throughout the same within 0.3 %.
// The 128 x 128 tile has 16 MFMAs and 8 fragments per k-step: the reads follow the first 8 MFMAs
// (so the last has returned when the k-step ends), the loads the other 8, evenly spaced.
constexpr int slot_pick(bool hit, int idx, int count) { return hit && idx >= 0 && idx < count ? idx : -1; }
constexpr int slot_read_of(int j, int nm, int nfr) { return nm >= 4 * nfr ? slot_pick(j % 2 == 0, j / 2, nfr) : slot_pick(true, j, nfr); }
// position t of n loads spread over the slots behind the reads (the small tile's plan)
constexpr int slot_late(int j, int nm, int nfr, int n) { return j >= nfr && n > 0 && (j - nfr) % ((nm - nfr) / n) == 0 ? (j - nfr) / ((nm - nfr) / n) : -1; }
constexpr int slot_a0_of(int j, int n, int nm, int nfr) { return nm >= 4 * nfr ? slot_pick(j % 16 == 1, j / 16, n) : slot_pick(true, slot_late(j, nm, nfr, n), n); }
constexpr int slot_b1_of(int j, int n, int nm, int nfr, int na1)
{
    return nm >= 4 * nfr ? slot_pick(j % 4 == 1, j / 4, n) : slot_pick(true, slot_late(j, nm, nfr, n + na1), n);
}
constexpr int slot_a1_of(int j, int n, int nm, int nfr, int nb1)
{
    return nm >= 4 * nfr ? slot_pick(j % 8 == 3 && j / 8 >= 4, j / 8 - 4, n) : slot_pick(true, slot_late(j, nm, nfr, n + nb1) - nb1, n);
}

// every fragment and every load of a K tile has exactly one slot, no slot holds a read and a load, and the
// loads of k-step 1 come before the slot that works out the next tile's offsets (nm - 2)
constexpr bool slot_plan_ok(int nm, int nfr, int la, int lb)
{
    const int la0 = la / 2, la1 = la - la0;
    int reads = 0, a0 = 0, b1 = 0, a1 = 0;
    for (int j = 0; j < nm; ++j) {
        const int r = slot_read_of(j, nm, nfr), x = slot_a0_of(j, la0, nm, nfr);
        const int y = slot_b1_of(j, lb, nm, nfr, la1), z = slot_a1_of(j, la1, nm, nfr, lb);
        if (r >= 0 && (x >= 0 || y >= 0 || z >= 0)) return false;
        if (y >= 0 && z >= 0) return false;
        if ((y >= 0 || z >= 0) && j >= nm - 2) return false;
        if (r >= 0) { if (r != reads) return false; ++reads; }
        if (x >= 0) { if (x != a0) return false; ++a0; }
        if (y >= 0) { if (y != b1) return false; ++b1; }
        if (z >= 0) { if (z != a1) return false; ++a1; }
    }
    return reads == nfr && a0 == la0 && b1 == lb && a1 == la1;
}
static_assert(slot_plan_ok(64, 16, 8, 8), "slot plan of the 256 x 256 tile");
static_assert(slot_plan_ok(16, 8, 4, 4), "slot plan of the 128 x 128 tile");
static_assert(slot_plan_ok(32, 12, 8, 4), "slot plan of the 256 x 128 tile");

// MAY_TAIL false: K is a whole number of K tiles (the host picks the instantiation).  No load
// then needs the per-lane offsets of a tile that K ends inside, and the select between the
// two sets of offsets, one vector instruction per load, is left out: a 16-cycle MFMA slot has
// room for three other instructions.
template <class C, bool MAY_TAIL>
__global__ __launch_bounds__(C::NT, C::WAVES_PER_EU) void gemm16_kernel(const GemmArgs p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the kernel's symbol
    __shared__ __attribute__((aligned(1024))) char lds[C::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
    const int r16 = lane & 15, q = lane >> 4;
#ifdef PEAK_TRACE
    // Diagnostic build only: per wave, shader-clock time stamps of the kernel's phases and the
    // cycles spent at the K loop's waits, written to the workspace.
    const uint64_t tr_start = __builtin_amdgcn_s_memtime();
    uint64_t tr_loop0 = 0, tr_loop1 = 0, tr_w0 = 0, tr_w1 = 0, tr_wait_sum = 0, tr_wait_max = 0;
#endif

    // Which tile, which K slice.  Split-K: slice s of tile t is workgroup s * tiles + t.  Hybrid
    // stream-K: the first tiles - sk_tiles workgroups take one tile each over the whole of K;
    // the rest (the last, partial round of workgroups) share the remaining sk_tiles tiles,
    // `split` K slices each, so that the round ends after a slice instead of a tile.
    const int tiles = p.tiles_m * p.tiles_n;
    const int bid = blockIdx.x;
    const int whole = tiles - p.sk_tiles;                   // stream-K: tiles that are not cut
    int slice, tile, sk_pos = -1;
    if (p.sk_tiles == 0) {
        slice = __builtin_amdgcn_readfirstlane(bid / tiles);
        tile = bid - slice * tiles;
    } else if (bid < whole) {
        slice = -1;                                         // the whole of K
        tile = bid;
    } else {
        slice = __builtin_amdgcn_readfirstlane((bid - whole) / p.sk_tiles);
        sk_pos = (bid - whole) - slice * p.sk_tiles;
        tile = whole + sk_pos;
    }
    int tm, tn;
    tile_of_block(tile, p.tiles_m, p.tiles_n, p.group_m, tm, tn);
    const int64_t m0 = (int64_t)tm * C::BM, n0 = (int64_t)tn * C::BN;

    const int kt_begin = slice < 0 ? 0 : slice * p.ktiles_per_slice;
    int kt_end = slice < 0 ? p.ktiles_total : kt_begin + p.ktiles_per_slice;
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

    // Fragment of k-step ks for an operand staged along K: lane reads row (lane % 16) of its
    // block, chunk 4 * ks + lane / 16 (8 k).  One address per operand and k-step; blocks and
    // stages go into the read's immediate offset.
    int a_base[C::KS], b_base[C::KS];
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
        const int ra = wm * C::WTM + r16, rb = wn * C::WTN + r16;
        a_base[ks] = ra * C::RB + (((4 * ks + q) ^ C::swizzle(ra)) << 4);
        b_base[ks] = C::NSA * C::A_BYTES + rb * C::RB + (((4 * ks + q) ^ C::swizzle(rb)) << 4);
    }
    // Operand staged as [k][x] rows (x = m or n; 512 bytes per k-row, chunk c of row k at
    // c ^ kn_swizzle(k)): the transposing read works on groups of 16 lanes, which together
    // point at 4 k-rows x 16 x (lane i of the group at k-row i / 4, columns 4 * (i % 4) .. + 3)
    // and each get the 4 k of one x.  Group lane / 16 takes k-rows 8 * (lane / 16) .. + 3, a
    // second read 4 rows on takes the other half of the lane's 8 k.  One address per block
    // (the swizzle does not commute with the block's column offset); k-step (32 rows), the
    // second read (4 rows) and the stage go into the immediate.
    int a_kx[C::A_KM ? C::MB : 1], a_kx2[C::A_KM ? C::MB : 1], b_kx[C::B_KN ? C::NB : 1];
    {
        const int krow = 8 * q + (r16 >> 2);
        if constexpr (C::A_KM) {
#pragma unroll
            for (int i = 0; i < C::MB; ++i) {
                const int col = wm * C::WTM + i * 16 + 4 * (r16 & 3);
                a_kx[i] = krow * (C::BM * C::ESZ) + (((col >> 3) ^ C::kn_swizzle(krow)) << 4) + (r16 & 1) * 8;
                a_kx2[i] = a_kx[i] + 2 * C::A_BYTES;
            }
        }
        if constexpr (C::B_KN) {
#pragma unroll
            for (int i = 0; i < C::NB; ++i) {
                const int col = wn * C::WTN + i * 16 + 4 * (r16 & 3);
                b_kx[i] = C::NSA * C::A_BYTES + krow * (C::BN * C::ESZ) + (((col >> 3) ^ C::kn_swizzle(krow)) << 4) + (r16 & 1) * 8;
            }
        }
    }
    const uint32_t lds_b0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    u32x4 af[2][C::MB], bf[2][C::NB];
    // halves of the fragments read with the transposing read, which goes out as assembly: the
    // compiler's wait-count pass would put a wait for every outstanding direct-to-LDS load in
    // front of it (it takes them to alias).  They are handed over by settle() at the start of the
    // k-step that uses them, after a wait for everything the wave has asked of LDS.
    u32x2 al[2][C::A_KM ? C::MB : 1], ah[2][C::A_KM ? C::MB : 1], bl[2][C::B_KN ? C::NB : 1], bh[2][C::B_KN ? C::NB : 1];
    auto read_a = [&](auto stagec, auto ksc, auto ic, auto setc) {
        constexpr int stage = decltype(stagec)::value, ks = decltype(ksc)::value, i = decltype(ic)::value, set = decltype(setc)::value;
        if constexpr (C::A_KM) {
            // (the immediate holds 16 bits: the third stage goes through an address of its own)
            constexpr int off = (stage % 2) * C::A_BYTES + ks * 32 * (C::BM * C::ESZ);
            constexpr int pair = stage / 2;                  // stages beyond the third: added at run time
            const uint32_t a0 = lds_b0 + (pair == 0 ? a_kx[i] : pair == 1 ? a_kx2[i] : a_kx[i] + pair * 2 * C::A_BYTES);
            u32x2 &lo = al[set][i], &hi = ah[set][i];
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(a0), "n"(off) : "memory");
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(a0), "n"(off + 4 * C::BM * C::ESZ) : "memory");
        } else {
            constexpr int off = stage * C::A_BYTES + i * 16 * C::RB;
            af[set][i] = *(const u32x4 *)(lds + a_base[ks] + off);
        }
    };
    auto read_b = [&](auto stagec, auto ksc, auto ic, auto setc) {
        constexpr int stage = decltype(stagec)::value, ks = decltype(ksc)::value, i = decltype(ic)::value, set = decltype(setc)::value;
        if constexpr (C::B_KN) {
            constexpr int off = stage * C::B_BYTES + ks * 32 * (C::BN * C::ESZ);
            const uint32_t a0 = lds_b0 + b_kx[i];
            u32x2 &lo = bl[set][i], &hi = bh[set][i];
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(a0), "n"(off) : "memory");
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(a0), "n"(off + 4 * C::BN * C::ESZ) : "memory");
        } else {
            constexpr int off = stage * C::B_BYTES + i * 16 * C::RB;
            bf[set][i] = *(const u32x4 *)(lds + b_base[ks] + off);
        }
    };
    // the assembly-read halves of `set` have arrived: hand them to the compiler
    auto settle = [&](auto setc) {
        constexpr int set = decltype(setc)::value;
        if constexpr (C::A_KM || C::B_KN) {
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));
            if constexpr (C::A_KM) {
#pragma unroll
                for (int i = 0; i < C::MB; ++i) {
                    u32x2 &lo = al[set][i], &hi = ah[set][i];
                    asm volatile("" : "+v"(lo), "+v"(hi));
                    af[set][i] = u32x4{lo[0], lo[1], hi[0], hi[1]};
                }
            }
            if constexpr (C::B_KN) {
#pragma unroll
                for (int i = 0; i < C::NB; ++i) {
                    u32x2 &lo = bl[set][i], &hi = bh[set][i];
                    asm volatile("" : "+v"(lo), "+v"(hi));
                    bf[set][i] = u32x4{lo[0], lo[1], hi[0], hi[1]};
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    LoaderDirect<C, C::BM> dA;
    LoaderDirect<C, C::BN> dB;
    LoaderDirectKN<C, C::BM> nA;
    LoaderDirectKN<C, C::BN> nB;
    constexpr int LA = C::A_KM ? LoaderDirectKN<C, C::BM>::PER_WAVE : LoaderDirect<C, C::BM>::PER_WAVE;
    constexpr int LB = C::B_KN ? LoaderDirectKN<C, C::BN>::PER_WAVE : LoaderDirect<C, C::BN>::PER_WAVE;
    static_assert((C::A_KM ? LoaderDirectKN<C, C::BM>::NINST : LoaderDirect<C, C::BM>::NINST) % C::NW == 0 &&
                  (C::B_KN ? LoaderDirectKN<C, C::BN>::NINST : LoaderDirect<C, C::BN>::NINST) % C::NW == 0,
                  "every wave issues the same number of loads");
    const int tail_k = __builtin_amdgcn_readfirstlane((int)(p.K - (int64_t)(p.ktiles_total - 1) * C::BK));
    const int tail_tile = tail_k < C::BK ? p.ktiles_total - 1 - kt_begin : -1;   // relative to the slice
    if constexpr (C::A_KM) nA.init(p.A, p.lda, m0, p.M, kbase, p.K, tail_k, wave, lane);
    else dA.init(p.A, p.lda, m0, p.M, kbase, p.K, tail_k, wave, lane);
    if constexpr (C::B_KN) nB.init(p.B, p.ldb, n0, p.N, kbase, p.K, tail_k, wave, lane);
    else dB.init(p.B, p.ldb, n0, p.N, kbase, p.K, tail_k, wave, lane);
    auto a_stage = [&](int s) { return lds + s * C::A_BYTES; };
    auto b_stage = [&](int s) { return lds + C::NSA * C::A_BYTES + s * C::B_BYTES; };
    // Loads of the tile whose scalar offsets and tail flag are in (soa, sob, tl), part PART of the
    // wave's LA (LB) instructions.  The three are worked out a tile ahead, in a slot of the
    // schedule that holds nothing else (next_offsets).  Past the end the last tile is fetched
    // again into a free stage, so the count in flight stays what the waits assume.
    int soa = 0, sob = 0;
    bool tl = false;
    // K rotation: this workgroup walks its K tiles starting at tile `rot` and wraps round (only the order
    // of the sum over k changes).  Off (0) unless the plan asks for it: where every tile streams rows of its
    // own from HBM, workgroups that all read the same k range at once load few memory channels at a time.
    const int rot = __builtin_amdgcn_readfirstlane((int)(((int64_t)tn * p.rot_n + (int64_t)tm * p.rot_m) % KT));
    auto next_offsets = [&](int kt) {
        int kr = (kt < KT ? kt : KT - 1) + rot;
        if (kr >= KT) kr -= KT;
        soa = C::A_KM ? nA.soffset_of(kr) : dA.soffset_of(kr);
        sob = C::B_KN ? nB.soffset_of(kr) : dB.soffset_of(kr);
        tl = kr == tail_tile;
    };
    auto issue_a = [&](int sa, auto part, auto may_tail) {
        constexpr bool MT = decltype(may_tail)::value != 0;
        if constexpr (C::A_KM) nA.template issue_at<decltype(part)::value, LA, MT>(a_stage(sa), soa, tl, wave);
        else dA.template issue_at<decltype(part)::value, LA, MT>(a_stage(sa), soa, tl, wave);
    };
    auto issue_b = [&](int sb, auto part, auto may_tail) {
        constexpr bool MT = decltype(may_tail)::value != 0;
        if constexpr (C::B_KN) nB.template issue_at<decltype(part)::value, LB, MT>(b_stage(sb), sob, tl, wave);
        else dB.template issue_at<decltype(part)::value, LB, MT>(b_stage(sb), sob, tl, wave);
    };

    // In the loop a load goes out as assembly, in two parts around an MFMA: the LDS address into m0
    // before it, the load after it.  Issued as one builtin, both parts land behind the MFMA, and the
    // compiler, which does not count the MFMA's assembly as an instruction, puts the wait state that
    // m0 needs between them: four instructions in a 16-cycle slot that has room for three
    // (measured per 256 x 256 x 64 step with and without the loop's loads: 5 cycles per load).
    auto m0_a = [&](int sa, auto part) {
        const uint32_t dst = lds_b0 + sa * C::A_BYTES + (wave + C::NW * decltype(part)::value) * 1024;
        asm volatile("s_mov_b32 m0, %0" : : "s"(dst) : "m0");
    };
    auto m0_b = [&](int sb, auto part) {
        const uint32_t dst = lds_b0 + C::NSA * C::A_BYTES + sb * C::B_BYTES + (wave + C::NW * decltype(part)::value) * 1024;
        asm volatile("s_mov_b32 m0, %0" : : "s"(dst) : "m0");
    };
    auto ld_a = [&](auto part, auto may_tail) {
        constexpr int i = decltype(part)::value;
        constexpr bool MT = decltype(may_tail)::value != 0;
        if constexpr (C::A_KM) {
            const int vo = MT && tl ? nA.voff_tail[i] : nA.voff[i], so = soa;
            const __amdgpu_buffer_rsrc_t rs = nA.rsrc;
            asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds" : : "v"(vo), "s"(rs), "s"(so) : "memory");
        } else {
            const int vo = MT && tl ? dA.voff_tail[i] : dA.voff[i], so = soa;
            const __amdgpu_buffer_rsrc_t rs = dA.rsrc;
            asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds" : : "v"(vo), "s"(rs), "s"(so) : "memory");
        }
    };
    auto ld_b = [&](auto part, auto may_tail) {
        constexpr int i = decltype(part)::value;
        constexpr bool MT = decltype(may_tail)::value != 0;
        if constexpr (C::B_KN) {
            const int vo = MT && tl ? nB.voff_tail[i] : nB.voff[i], so = sob;
            const __amdgpu_buffer_rsrc_t rs = nB.rsrc;
            asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds" : : "v"(vo), "s"(rs), "s"(so) : "memory");
        } else {
            const int vo = MT && tl ? dB.voff_tail[i] : dB.voff[i], so = sob;
            const __amdgpu_buffer_rsrc_t rs = dB.rsrc;
            asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds" : : "v"(vo), "s"(rs), "s"(so) : "memory");
        }
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
    static_assert(LA % 2 == 0 && 2 * NFR <= NM, "slot plan below");
    static_assert(C::KS == 4 || (C::KS == 2 && slot_plan_ok(NM, NFR, LA, LB)), "two k-steps per K tile: the slot plan below");
    static_assert(C::KS == 2 || (C::KS == 4 && C::PF == 2 && NM == 16 && NFR == 8 && LA == 8 && LB == 8), "four k-steps: 128 x 128 tile");
    // fragment f of a k-step in the order the MFMAs first need them: B0, A0 .. A7, B1 .. B7
    auto fetch_one_set = [&](auto sac, auto sbc, auto ksc, auto setc, auto fc) {
        constexpr int f = decltype(fc)::value;
        if constexpr (f == 0) read_b(sbc, ksc, IC<0>{}, setc);
        else if constexpr (f <= C::MB) read_a(sac, ksc, IC<f - 1>{}, setc);
        else read_b(sbc, ksc, IC<f - C::MB>{}, setc);
    };
    auto fetch_one = [&](auto sac, auto sbc, auto ksc, auto fc) { fetch_one_set(sac, sbc, ksc, ksc, fc); };   // two k-steps: set = k-step
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
    constexpr int LA0 = LA / 2;                              // A's loads that go out in k-step 0
    // loads that may still be under way at a tile's barrier: those of the tiles after the next one
    constexpr int PENDING = (C::PF - 2) * (LA + LB) + LA0;
    static_assert(PENDING < 64, "fits the wait's counter");
    auto slot_read = [](int j) constexpr { return slot_read_of(j, NM, NFR); };
    auto slot_a0 = [](int j) constexpr { return slot_a0_of(j, LA0, NM, NFR); };
    auto slot_b1 = [](int j) constexpr { return slot_b1_of(j, LB, NM, NFR, LA - LA0); };
    auto slot_a1 = [](int j) constexpr { return slot_a1_of(j, LA - LA0, NM, NFR, LB); };
    constexpr int PF = C::PF;
    next_offsets(0);
    static_for<LA>([&](auto pc) { issue_a(0, pc, IC<1>{}); });
    static_for<LB>([&](auto pc) { issue_b(0, pc, IC<1>{}); });
    static_for<NM>([&](auto jc) {                             // accumulators into AGPRs now
        constexpr int j = decltype(jc)::value;
        f32x4v &c = acc[j % C::MB][j / C::MB];
        asm volatile("" : "+a"(c));
    });
    if constexpr (PF == 2) {
        wait_vmcnt<0>();
        lds_barrier();
        next_offsets(1);
        static_for<LB>([&](auto pc) { issue_b(1, pc, IC<1>{}); });
        static_for<LA>([&](auto pc) { issue_a(1, pc, IC<1>{}); });
    } else {
        // tiles 1 .. PF-1 right behind tile 0; only tile 0 has to have landed
        static_for<PF - 1>([&](auto tc) {
            constexpr int t = decltype(tc)::value + 1;
            next_offsets(t);
            static_for<LB>([&](auto pc) { issue_b(t, pc, IC<1>{}); });
            static_for<LA>([&](auto pc) { issue_a(t, pc, IC<1>{}); });
        });
        wait_vmcnt<(PF - 1) * (LA + LB)>();
        lds_barrier();
    }
    next_offsets(PF);
    asm volatile("s_nop 7\n\ts_nop 7" ::: "memory");
    static_for<NFR>([&](auto fc) { fetch_one(IC<0>{}, IC<0>{}, IC<0>{}, fc); });
#ifdef PEAK_TRACE
    tr_loop0 = __builtin_amdgcn_s_memtime();
#endif
    if constexpr (C::KS == 4) {
        // Four k-steps of 16 MFMAs per K tile (BK = 128).  Fragments of the next k-step follow the first eight
        // MFMAs of each; A's eight loads of tile kt+2 are spread over the slots behind them in k-steps 0 to 2
        // (its stage is free since the barrier of tile kt-1), the tile's barrier stands before k-step 3, and B's
        // eight loads follow it.  The loads' offsets are worked out at the start of the tile.
        constexpr auto may_tail = IC<MAY_TAIL ? 1 : 0>{};
        constexpr int U = C::NSA * C::NSB;
        for (int kt0 = 0; kt0 < KT; kt0 += U) {
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                constexpr int s = u % C::NSB, s1 = (u + 1) % C::NSB, sa = u % C::NSA, sa1 = (sa + 1) % C::NSA, sa2 = (sa + C::PF) % C::NSA;
                const int kt = kt0 + u;
                if (kt < KT) {
                    static_for<4>([&](auto ksc) {
                        constexpr int ks = decltype(ksc)::value, cur = ks & 1, nxt = cur ^ 1;
                        if constexpr (ks == 3) {
                            wait_vmcnt<LA>();                    // own loads of tile kt+1 (A's of tile kt+2 may be under way)
                            lds_barrier();                       // tile kt+1 complete, tile kt read
                        }
                        settle(IC<cur>{});
                        __builtin_amdgcn_sched_barrier(0);
                        static_for<NM>([&](auto jc) {
                            constexpr int j = decltype(jc)::value;
                            // which load follows MFMA j: A part 3 ks + (j - 8) / 2 in k-steps 0 to 2, B part j - 8 in k-step 3
                            constexpr int pa = ks < 3 && j >= 8 && j % 2 == 0 && 3 * ks + (j - 8) / 2 < LA && (j - 8) / 2 < 3 ? 3 * ks + (j - 8) / 2 : -1;
                            constexpr int pb = ks == 3 && j >= 8 ? j - 8 : -1;
                            if constexpr (ks == 0 && j == 0) next_offsets(kt + C::PF);
                            if constexpr (pa >= 0) m0_a(sa2, IC<(pa >= 0 ? pa : 0)>{});
                            if constexpr (pb >= 0) m0_b(s, IC<(pb >= 0 ? pb : 0)>{});
                            mfma_one(IC<cur>{}, jc);
                            if constexpr (j < NFR) {
                                if constexpr (ks < 3) fetch_one_set(IC<sa>{}, IC<s>{}, IC<(ks + 1) % 4>{}, IC<nxt>{}, jc);
                                else fetch_one_set(IC<sa1>{}, IC<s1>{}, IC<0>{}, IC<nxt>{}, jc);
                            }
                            if constexpr (pa >= 0) ld_a(IC<(pa >= 0 ? pa : 0)>{}, may_tail);
                            if constexpr (pb >= 0) ld_b(IC<(pb >= 0 ? pb : 0)>{}, may_tail);
                            __builtin_amdgcn_sched_barrier(0);
                        });
                    });
                }
            });
        }
    } else {
        constexpr auto may_tail = IC<MAY_TAIL ? 1 : 0>{};
        constexpr int U = C::NSA * C::NSB;                   // tiles per trip: both stage indices static (NSA and NSB differ by one)
        for (int kt0 = 0; kt0 < KT; kt0 += U) {
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                // stages of tile kt (B: s, A: sa), of tile kt+1 (s1, sa1) and of the tile whose loads go out now (B: s again, A: sa2)
                constexpr int s = u % C::NSB, s1 = (u + 1) % C::NSB, sa = u % C::NSA, sa1 = (sa + 1) % C::NSA, sa2 = (sa + C::PF) % C::NSA;
                const int kt = kt0 + u;
                if (kt < KT) {
                    // k-step 0
                    settle(IC<0>{});
#ifdef PEAK_TRACE
                    {
                        const uint64_t dw = tr_w1 - tr_w0;   // the wait of the tile before: stamps long since returned
                        tr_wait_sum += dw;
                        tr_wait_max = dw > tr_wait_max ? dw : tr_wait_max;
                    }
#endif
                    __builtin_amdgcn_sched_barrier(0);
                    static_for<NM>([&](auto jc) {
                        constexpr int j = decltype(jc)::value;
                        if constexpr (slot_a0(j) >= 0) m0_a(sa2, IC<(slot_a0(j) >= 0 ? slot_a0(j) : 0)>{});
                        mfma_one(IC<0>{}, jc);
                        if constexpr (slot_read(j) >= 0) fetch_one(IC<sa>{}, IC<s>{}, IC<1>{}, IC<(slot_read(j) >= 0 ? slot_read(j) : 0)>{});
                        if constexpr (slot_a0(j) >= 0) ld_a(IC<(slot_a0(j) >= 0 ? slot_a0(j) : 0)>{}, may_tail);
                        __builtin_amdgcn_sched_barrier(0);
                    });
                    // k-step 1
#ifdef PEAK_TRACE
                    tr_w0 = __builtin_amdgcn_s_memtime();
#endif
                    wait_vmcnt<PENDING>();                   // own loads of tile kt+1
                    lds_barrier();                           // tile kt+1 complete, tile kt read
#ifdef PEAK_TRACE
                    tr_w1 = __builtin_amdgcn_s_memtime();
#endif
                    settle(IC<1>{});
                    __builtin_amdgcn_sched_barrier(0);
                    static_for<NM>([&](auto jc) {
                        constexpr int j = decltype(jc)::value;
                        if constexpr (slot_b1(j) >= 0) m0_b(s, IC<(slot_b1(j) >= 0 ? slot_b1(j) : 0)>{});
                        if constexpr (slot_a1(j) >= 0) m0_a(sa2, IC<(LA0 + (slot_a1(j) >= 0 ? slot_a1(j) : 0)) % LA>{});
                        mfma_one(IC<1>{}, jc);
                        if constexpr (slot_read(j) >= 0) fetch_one(IC<sa1>{}, IC<s1>{}, IC<0>{}, IC<(slot_read(j) >= 0 ? slot_read(j) : 0)>{});
                        if constexpr (slot_b1(j) >= 0) ld_b(IC<(slot_b1(j) >= 0 ? slot_b1(j) : 0)>{}, may_tail);
                        if constexpr (slot_a1(j) >= 0) ld_a(IC<(LA0 + (slot_a1(j) >= 0 ? slot_a1(j) : 0)) % LA>{}, may_tail);
                        if constexpr (j == NM - 2) next_offsets(kt + 1 + C::PF);   // for the loads the next tile issues
                        __builtin_amdgcn_sched_barrier(0);
                    });
                }
            });
        }
    }
    settle(IC<0>{});    // reads issued as assembly feed nothing here, but must have returned before their registers are reused
    // 16x16x32 MFMA: 4 passes of 4 cycles; an accumulator may be read 10 wait states after the issue
    asm volatile("s_nop 15" ::: "memory");
#ifdef PEAK_TRACE
    tr_loop1 = __builtin_amdgcn_s_memtime();
#endif
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
    PartialOut po = splitk_out(p, slice < 0 ? 0 : slice);
    if (p.sk_tiles != 0) {
        po = PartialOut{nullptr, 0, 0, 0, false};
        if (slice >= 0)     // partial tile, stored densely: [slice][position among the cut tiles][BM][BN]
            po = PartialOut{p.ws + ((int64_t)slice * p.sk_tiles + sk_pos) * (C::BM * C::BN), C::BN, m0, n0, true};
    }
    epilogue_slabs<C, C::WTM / 32>(p, lds, wave, lane, wm, wn, m0, n0, po, write_slab, write16);
#ifdef PEAK_TRACE
    if (p.split == 1 && p.ws && lane == 0) {
        const uint64_t tr_end = __builtin_amdgcn_s_memtime();
        uint32_t hwid, xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hwid));
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        uint64_t *dst = (uint64_t *)p.ws + ((size_t)blockIdx.x * C::NW + wave) * 8;
        dst[0] = tr_start; dst[1] = tr_loop0; dst[2] = tr_loop1; dst[3] = tr_end;
        dst[4] = tr_wait_sum; dst[5] = tr_wait_max; dst[6] = (uint64_t)hwid | ((uint64_t)xcc << 32); dst[7] = (uint64_t)p.ktiles_total;
    }
#endif
#endif
}

}  // namespace peak
