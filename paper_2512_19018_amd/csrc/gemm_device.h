// Device side of the gfx950 GEMM: workgroup tile -> LDS staging ring -> MFMA
// register tiles -> epilogue.  One kernel template, instantiated per dtype,
// tile shape and operand layout.
//
// Vocabulary follows Section 2.2 of the paper ("Matrix Multiplication"):
//   thread-block tile  t_m x t_n (x t_k)  ->  BM x BN x BK, one workgroup
//   warp tile          w_m x w_n          ->  WTM x WTN, one 64-lane wavefront,
//                                             a grid of 32x32 MFMA blocks
// and the transformations of Section 4.1 (Table 2 and the sequences of Table
// 3): Tensor-Core/Tensor-Tiling -> MFMA blocks per wave, Transpose -> the
// transposing store of operands that do not run along K in memory, Offset ->
// the XOR swizzle of 16-byte chunks (in place of padding), Pipelining /
// Register-Staging -> the LDS ring filled by direct-to-LDS loads or through
// registers, Block-Swizzle -> the XCD-aware tile order, Split-K -> K slices
// with an ordered fp32 reduction.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace peak {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

enum { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2 };

// flags in GemmArgs::flags
enum {
    GF_A_VEC = 1,      // A base and row stride are 16-byte aligned
    GF_B_VEC = 2,      // B likewise
    GF_C_VEC = 4,      // C rows allow 4-element vector access
    GF_WS_VEC = 8,     // workspace rows (N floats) allow 16-byte access
    GF_C_VEC16 = 16,   // C base and row stride are 16-byte aligned
    GF_C_F32 = 32      // C is stored as fp32 although A and B are 16-bit
};

// Fused output step: v <- act(v + bias), applied to alpha*acc + beta*C in fp32
// before the one rounding to the storage type.
enum { BIAS_NONE = 0, BIAS_PER_COLUMN = 1, BIAS_PER_ROW = 2 };
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU_TANH = 2 };
struct Hook {
    const float *bias;        // device, fp32: N values (per column) or M values (per row)
    int32_t bias_kind;
    int32_t act;
};

struct GemmArgs {
    const void *A;
    const void *B;
    void *C;
    float *ws;                // split > 1: fp32 partials [split][M][N]
    int64_t M, N, K;
    int64_t lda, ldb, ldc;    // elements
    float alpha, beta;
    int32_t tiles_m, tiles_n;
    int32_t split;            // number of K slices
    int32_t ktiles_per_slice; // BK-tiles per slice (last slice may be shorter)
    int32_t ktiles_total;     // ceil(K / BK)
    int32_t group_m;          // tile rows per band of the tile order
    int32_t rot_m, rot_n;     // K rotation per tile row / tile column within an XCD's patch of tiles
    int32_t sk_tiles;         // hybrid stream-K: the last sk_tiles tiles of the tile order are cut into `split` K slices
                              // (fp32 partials [slice][tile][BM][BN] in ws), all others take the whole of K; 0: off
    uint32_t flags;
    Hook hook;
};

#define PEAK_DEV static __device__ __forceinline__
#define PEAK_DEVM __device__ __forceinline__

// compile-time integer and loop (for template arguments inside lambdas)
template <int V>
struct IC { static constexpr int value = V; };
template <int N, int I = 0, class F>
PEAK_DEV void static_for(F &&f)
{
    if constexpr (I < N) {
        f(IC<I>{});
        static_for<N, I + 1>(f);
    }
}

// s_waitcnt immediate (gfx9 encoding): vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8.
constexpr int waitcnt_imm(int vmcnt, int lgkmcnt) { return ((vmcnt >> 4) & 3) << 14 | (vmcnt & 15) | 0x70 | (lgkmcnt & 15) << 8; }

PEAK_DEV void lds_barrier()
{
    // LDS traffic of this wave done, then workgroup barrier.  Outstanding
    // global loads are left in flight on purpose (no fence: a fence would wait
    // for them).  The empty asm statements keep the compiler from moving LDS
    // accesses across; the wait is a builtin so that the compiler's own
    // wait-count bookkeeping sees it.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <int N>
PEAK_DEV void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(N, 15));
    asm volatile("" ::: "memory");
}

// ---------------------------------------------------------------------------
// Tile geometry.  A tile row holds RB bytes of K (BK elements) cut into 16-byte
// chunks; chunk c of row r sits at chunk position c ^ swz(r), which keeps both
// the row-wise 16-byte stores and the 32-rows-same-chunk fragment reads free of
// bank conflicts.
// ---------------------------------------------------------------------------
template <int CPR>
PEAK_DEV int swz(int r)
{
    if (CPR == 8) return (r ^ (r >> 3)) & 7;
    return ((r >> 1) ^ (r >> 3)) & 3;          // CPR == 4: two rows share 128 bytes
}

template <int DT_, int BM_, int BN_, int RB_, int WAVES_M_, int WAVES_N_, int NS_,
          bool A_T_, bool B_T_, bool DIRECT_, int AX_ = 0, bool TR_ = false, bool PP_ = false, bool ATR_ = false, bool AG_ = false>
struct Cfg {
    static constexpr int DT = DT_;
    static constexpr int ESZ = DT_ == DT_F32 ? 4 : 2;
    static constexpr int EPC = 16 / ESZ;              // elements per 16-byte chunk
    static constexpr int BM = BM_, BN = BN_, RB = RB_;
    static constexpr int CPR = RB_ / 16;              // chunks per tile row
    static constexpr int BK = RB_ / ESZ;              // t_k
    static constexpr int KG = CPR / 2;                // 32-row MFMA groups per tile row
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int NW = WAVES_M_ * WAVES_N_;
    static constexpr int NT = NW * 64;
    static constexpr int WTM = BM_ / WAVES_M_, WTN = BN_ / WAVES_N_;
    static constexpr int MI = WTM / 32, NI = WTN / 32;
    static constexpr int NS = NS_;
    static constexpr bool A_T = A_T_;                 // A stored K rows x M (does not run along K)
    static constexpr bool B_T = B_T_;                 // B stored K rows x N (does not run along K)
    static constexpr bool DIRECT = DIRECT_;           // K-running operands go global -> LDS directly
    // B stored K x N: copied global -> LDS directly as [k][n] rows, no register
    // staging.  16-bit fragments come back through the transposing LDS read
    // (ds_read_b64_tr_b16); fp32 needs no transposition at all (one float per lane
    // and MFMA, 32 lanes along a row)
    static constexpr bool B_TR = TR_;
    // the same for A stored K x M: [k][m] rows in LDS, read with the transposing read
    static constexpr bool A_TR = ATR_;
    static_assert(!ATR_ || (DIRECT_ && A_T_ && RB_ == 128 && AX_ == 0 && !PP_), "A kept as [k][m] rows in LDS: A stored K x M, direct");
    static_assert(!TR_ || (DIRECT_ && B_T_ && (!A_T_ || ATR_) && RB_ == 128), "B kept as [k][n] rows in LDS: B stored K x N, direct");
    // the chunk swizzle of the 16-bit [k][n] and [k][m] rows moves a chunk by up to 12 places within its row
    static_assert(DT_ == DT_F32 || ((!TR_ || BN_ >= 128) && (!ATR_ || BM_ >= 128)), "16-bit rows kept as [k][n] need at least 16 chunks");
    static constexpr int A_BYTES = BM_ * RB_;
    static constexpr int B_BYTES = BN_ * RB_;
    // chunk c of tile row r sits at chunk position c ^ swizzle(r)
    static __device__ __forceinline__ int swizzle(int r) { return swz<RB_ / 16>(r); }
    // ... and chunk c of row k of a 16-bit tile kept as [k][n] (or [k][m]) rows at c ^ kn_swizzle(k)
    static __device__ __forceinline__ int kn_swizzle(int k) { return 4 * (k & 3); }
    // LDS: NSA stages of the A tile, then NSB stages of the B tile.  AX extra A
    // stages let A's loads run one more step ahead than B's when LDS cannot hold
    // another full stage of both (asymmetric ring, prefetch loops only).
    static constexpr int NSA = NS_ + AX_, NSB = NS_;
    static constexpr int LDS_BYTES = A_BYTES * NSA + B_BYTES * NSB;
    static constexpr bool PIPE = NS_ >= 4 && AX_ == 0 && !PP_;   // run-ahead main loop (see gemm_kernel); with 3 stages the
                                                         // two-phase loop keeps loads two steps ahead instead
    // Alternating main loop: the two waves of a SIMD take turns, one reading
    // fragments and issuing loads while the other multiplies (see gemm_kernel)
    static constexpr bool PP = PP_;
    // One wave per SIMD with a 128x128 wave tile: the 256 accumulator registers must sit in
    // the accumulation half of the register file.  The compiler does not manage that (it
    // keeps part of them in ordinary registers and spills), so for this shape the MFMAs of
    // the main loop are written as assembly with the accumulators constrained to AGPRs.
    // AG: the same hand-scheduled loop for fp32 with 64x64 wave tiles (128x128 tile, four waves).  Left to the
    // compiler that loop kept the matrix cores busy 81 % of the time at fp32 2048^3, against 92 % for the
    // hand-scheduled 256x256 tile.
    static constexpr bool ACC_AGPR = (WAVES_M_ * WAVES_N_ == 4 && (BM_ / WAVES_M_) * (BN_ / WAVES_N_) == 128 * 128) || AG_;
    static_assert(!AG_ || (DT_ == DT_F32 && WAVES_M_ * WAVES_N_ == 4 && BM_ / WAVES_M_ == 64 && BN_ / WAVES_N_ == 64),
                  "hand-scheduled loop on request: fp32, four waves, 64x64 wave tiles");
    static_assert(!PP_ || (NS_ >= 2 && AX_ == 0 && DIRECT_ && !A_T_ && (!B_T_ || TR_) && WAVES_M_ * WAVES_N_ == 8),
                  "alternating loop: 8 waves, both operands direct");
    static_assert(AX_ == 0 || (AX_ == 1 && NS_ == 2 && RB_ == 128 && DIRECT_ && !A_T_ && (!B_T_ || TR_)),
                  "one extra A stage: two stages of B, both operands direct");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is a grid of 32x32 MFMA blocks");
    static_assert(RB_ == 128 || RB_ == 64, "tile row is 64 or 128 bytes");
    static_assert((BM_ * CPR) % 64 == 0 && (BN_ * CPR) % 64 == 0, "whole wave loads");
};

// ---------------------------------------------------------------------------
// Register-staged tile loads.
// ---------------------------------------------------------------------------
template <int DT>
PEAK_DEV u32x4 load_chunk_elems(const void *base, int64_t idx0, int64_t stride, int nvalid)
{
    // nvalid leading elements of the chunk come from memory (element idx0 + e*stride), the rest are zero.
    constexpr int EPC = DT == DT_F32 ? 4 : 8;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (DT == DT_F32) {
        const uint32_t *p = (const uint32_t *)base;
#pragma unroll
        for (int e = 0; e < EPC; ++e)
            if (e < nvalid) v[e] = p[idx0 + e * stride];
    } else {
        const uint16_t *p = (const uint16_t *)base;
#pragma unroll
        for (int e = 0; e < EPC; ++e)
            if (e < nvalid) v[e >> 1] |= (uint32_t)p[idx0 + e * stride] << ((e & 1) * 16);
    }
    return v;
}

// Operand that runs along K in memory: rows x K, row stride ld.
template <class C, int ROWS>
struct LoaderK {
    static constexpr int NCH = (ROWS * C::CPR + C::NT - 1) / C::NT;
    u32x4 v[NCH];

    PEAK_DEVM void load(const void *base, int64_t ld, int64_t row0, int64_t nrows, int64_t k0, int64_t kend,
                       bool vec, int tid)
    {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int idx = tid + C::NT * i;
            const int row = idx / C::CPR, c = idx % C::CPR;
            u32x4 val = {0u, 0u, 0u, 0u};
            if (ROWS * C::CPR % C::NT == 0 || idx < ROWS * C::CPR) {
                int64_t gr = row0 + row;
                if (gr > nrows - 1) gr = nrows - 1;          // duplicate of a valid row; its results are never stored
                const int64_t k = k0 + (int64_t)c * C::EPC;
                const int64_t left = kend - k;
                if (vec && left >= C::EPC) {
                    val = *(const u32x4 *)((const char *)base + (gr * ld + k) * C::ESZ);
                } else if (left > 0) {
                    val = load_chunk_elems<C::DT>(base, gr * ld + k, 1, left < C::EPC ? (int)left : C::EPC);
                }
            }
            v[i] = val;
        }
    }

    PEAK_DEVM void store(char *lds_tile, int tid) const
    {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int idx = tid + C::NT * i;
            const int row = idx / C::CPR, c = idx % C::CPR;
            if (ROWS * C::CPR % C::NT == 0 || idx < ROWS * C::CPR)
                *(u32x4 *)(lds_tile + row * C::RB + ((c ^ swz<C::CPR>(row)) << 4)) = v[i];
        }
    }
};

// Operand stored K rows x `rows` (runs along M or N in memory).  Each thread
// takes an EPC(k) x EPC(rows) block, transposes it in registers and stores EPC
// chunks, one per tile row.
template <class C, int ROWS>
struct LoaderT {
    static constexpr int E = C::EPC;
    static constexpr int RBLK = ROWS / E;                         // blocks along the tile rows
    static constexpr int NBLK = RBLK * C::CPR;
    static constexpr int NB = (NBLK + C::NT - 1) / C::NT;
    u32x4 v[NB][E];                                               // [block][k within chunk] -> E row-elements

    PEAK_DEVM void load(const void *base, int64_t ld, int64_t row0, int64_t nrows, int64_t k0, int64_t kend,
                       bool vec, int tid)
    {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int id = tid + C::NT * b;
            const int rb = id % RBLK, c = id / RBLK;
            const int64_t r = row0 + (int64_t)rb * E;             // first tile row of the block, as a global row/col index
#pragma unroll
            for (int kk = 0; kk < E; ++kk) {
                u32x4 val = {0u, 0u, 0u, 0u};
                const int64_t k = k0 + (int64_t)c * E + kk;
                if ((NBLK % C::NT == 0 || id < NBLK) && k < kend) {
                    const int64_t left = nrows - r;
                    if (vec && left >= E) {
                        val = *(const u32x4 *)((const char *)base + (k * ld + r) * C::ESZ);
                    } else if (left > 0) {
                        val = load_chunk_elems<C::DT>(base, k * ld + r, 1, left < E ? (int)left : E);
                    }
                }
                v[b][kk] = val;
            }
        }
    }

    PEAK_DEVM void store(char *lds_tile, int tid) const
    {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int id = tid + C::NT * b;
            const int rb = id % RBLK, c = id / RBLK;
            if (NBLK % C::NT == 0 || id < NBLK) {
#pragma unroll
                for (int i = 0; i < E; ++i) {
                    u32x4 o;
                    if (C::DT == DT_F32) {
                        o[0] = v[b][0][i]; o[1] = v[b][1][i]; o[2] = v[b][2][i]; o[3] = v[b][3][i];
                    } else {
                        // 16-bit: element i of k-row kk is half (i & 1) of dword (i >> 1)
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            const uint32_t lo = v[b][2 * d][i >> 1], hi = v[b][2 * d + 1][i >> 1];
                            o[d] = (i & 1) ? ((lo >> 16) | (hi & 0xFFFF0000u)) : ((lo & 0xFFFFu) | (hi << 16));
                        }
                    }
                    const int row = rb * E + i;
                    *(u32x4 *)(lds_tile + row * C::RB + ((c ^ swz<C::CPR>(row)) << 4)) = o;
                }
            }
        }
    }
};

// Direct global -> LDS copy of an operand that runs along K, with buffer loads
// (buffer_load_dwordx4 ... lds).  One wave instruction fills 1024 contiguous LDS
// bytes (64 / CPR tile rows); which global chunk a lane fetches is chosen so that
// the swizzled layout comes out.  The buffer descriptor covers exactly this
// workgroup's panel, so a lane can never touch memory outside the operand; the
// step along K goes into the scalar offset.
// A per-lane offset no descriptor of ours reaches (panels stay below 2^31 bytes):
// a buffer load with it is out of range and delivers zeros.
constexpr int OOB_VOFFSET = 0x7FFFFF00;

template <class C, int ROWS>
struct LoaderDirect {
    static constexpr int NINST = ROWS * C::CPR / 64;              // wave instructions per tile
    static constexpr int PER_WAVE = (NINST + C::NW - 1) / C::NW;
    __amdgpu_buffer_rsrc_t rsrc;
    int voff[PER_WAVE];                                           // this lane's byte offset in the panel, per instruction
    int voff_tail[PER_WAVE];                                      // the same for the last K tile: out of range where the chunk lies past K

    // tail_k: number of valid k in the matrix's last K tile (BK when K is a multiple of BK)
    PEAK_DEVM void init(const void *base, int64_t ld, int64_t row0, int64_t nrows, int64_t k0, int64_t K, int tail_k, int wave, int lane)
    {
        int64_t rows_here = nrows - row0;                         // >= 1
        if (rows_here > ROWS) rows_here = ROWS;
        const uint64_t panel = (uint64_t)((const char *)base + (row0 * ld + k0) * C::ESZ);
        const int64_t bytes = ((rows_here - 1) * ld + (K - k0)) * C::ESZ;   // < 2^31, checked when the plan is made
        // the descriptor is the same for every lane: say so, or it may end up in vector registers
        const uint64_t panel_u = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(panel >> 32)) << 32) |
                                 (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)panel);
        rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)panel_u, 0, __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000);
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const int j = wave + C::NW * i;
            int row = j * (64 / C::CPR) + lane / C::CPR;
            const int pos = lane % C::CPR;
            const int c = pos ^ C::swizzle(row);
            if (row > rows_here - 1) row = (int)rows_here - 1;    // duplicate of a valid row; its results are never stored
            voff[i] = (int)((row * ld + (int64_t)c * C::EPC) * C::ESZ);
            voff_tail[i] = c * C::EPC >= tail_k ? OOB_VOFFSET : voff[i];
        }
    }

    // ktile: tile index relative to k0.  Issues this wave's instructions i with
    // i % NPARTS == PART, so that a tile's loads can be spread over a step.
    // tail: this is the matrix's last K tile and K stops inside it; chunks past K
    // are fetched with an offset beyond the descriptor's range, which stores zeros.
    template <int PART, int NPARTS>
    PEAK_DEVM void issue(char *lds_tile, int ktile, bool tail, int wave) const
    {
        issue_at<PART, NPARTS, true>(lds_tile, soffset_of(ktile), tail, wave);
    }

    // byte offset of K tile `ktile` (relative to k0) within the panel: the loads' scalar offset
    PEAK_DEVM int soffset_of(int ktile) const { return ktile * C::RB; }

    // ... with the scalar offset worked out by the caller (ahead of time, away from the loads);
    // MAY_TAIL false: the caller knows that K ends on a tile boundary and spares the select
    template <int PART, int NPARTS, bool MAY_TAIL>
    PEAK_DEVM void issue_at(char *lds_tile, int soffset, bool tail, int wave) const
    {
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const int j = wave + C::NW * i;
            if (i % NPARTS == PART && (NINST % C::NW == 0 || j < NINST)) {
                const int vo = MAY_TAIL && tail ? voff_tail[i] : voff[i];   // one select on a uniform condition
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void *)(lds_tile + j * 1024),
                                                         16, vo, soffset, 0, 0);
            }
        }
    }
};

// Direct global -> LDS copy of an operand stored K x N (B with transB = 0; the
// same serves A stored K x M, with M for N and COLS = BM).  The LDS tile keeps
// that orientation: BK rows of COLS elements.  16-byte chunk c of
// row k sits at chunk position c ^ (4 * (k & 3)): a transposing fragment read
// takes 4 k-rows x 64 bytes per 32 lanes, the rows are a multiple of 256 bytes
// apart, and the XOR moves each of the four rows to its own 64-byte group of
// banks (measured: with 2 * (k & 3) a quarter of the LDS cycles were bank
// conflicts, rows k and k+1 sharing a group).  N is a whole
// number of chunks; a chunk that would start at or past column N fetches the
// row's last valid chunk instead (it only feeds columns of C that are never
// stored), so every access stays inside the matrix.
// SWZ: chunk positions go through C::kn_swizzle (the tiled fp32 kernels read their [k][n] tile row-wise
// and leave it out)
template <class C, int COLS, bool SWZ = (C::DT != DT_F32)>
struct LoaderDirectKN {
    static constexpr int ROWB = COLS * C::ESZ;                    // bytes per k-row of the tile
    static constexpr int CPRN = ROWB / 16;
    static constexpr int RPI = 1024 / ROWB;                       // k-rows per wave instruction
    static constexpr int NINST = C::BK / RPI;
    static constexpr int PER_WAVE = (NINST + C::NW - 1) / C::NW;
    static_assert(1024 % ROWB == 0 && C::BK % RPI == 0, "whole rows per instruction");
    __amdgpu_buffer_rsrc_t rsrc;
    int voff[PER_WAVE];
    int voff_tail[PER_WAVE];                                      // for the last K tile: out of range where the k-row lies past K
    int step_bytes;                                               // BK rows of the stored matrix

    PEAK_DEVM void init(const void *base, int64_t ld, int64_t n0, int64_t N, int64_t k0, int64_t K, int tail_k, int wave, int lane)
    {
        const uint64_t panel = (uint64_t)((const char *)base + (k0 * ld + n0) * C::ESZ);
        const int64_t bytes = ((K - k0 - 1) * ld + (N - n0)) * C::ESZ;       // < 2^31, checked when the plan is made
        const uint64_t panel_u = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(panel >> 32)) << 32) |
                                 (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)panel);
        rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)panel_u, 0, __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000);
        step_bytes = __builtin_amdgcn_readfirstlane((int)(C::BK * ld * C::ESZ));
        const int last_chunk = (int)((N - n0) / C::EPC) - 1;                  // >= 0: N and n0 are multiples of EPC
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const int j = wave + C::NW * i;
            const int row = j * RPI + lane / CPRN;
            const int pos = lane % CPRN;
            int c = pos;
            if constexpr (SWZ) c = pos ^ C::kn_swizzle(row);
            if (c > last_chunk) c = last_chunk;
            voff[i] = (int)((row * ld + (int64_t)c * C::EPC) * C::ESZ);
            voff_tail[i] = row >= tail_k ? OOB_VOFFSET : voff[i];
        }
    }

    template <int PART, int NPARTS>
    PEAK_DEVM void issue(char *lds_tile, int ktile, bool tail, int wave) const
    {
        issue_at<PART, NPARTS, true>(lds_tile, soffset_of(ktile), tail, wave);
    }

    PEAK_DEVM int soffset_of(int ktile) const { return ktile * step_bytes; }

    template <int PART, int NPARTS, bool MAY_TAIL>
    PEAK_DEVM void issue_at(char *lds_tile, int soffset, bool tail, int wave) const
    {
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const int j = wave + C::NW * i;
            if (i % NPARTS == PART && (NINST % C::NW == 0 || j < NINST)) {
                const int vo = MAY_TAIL && tail ? voff_tail[i] : voff[i];
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void *)(lds_tile + j * 1024),
                                                         16, vo, soffset, 0, 0);
            }
        }
    }
};

// ---------------------------------------------------------------------------
// MFMA on one 16-byte fragment pair.  The roles are swapped on purpose: the B
// tile's rows (n) feed the instruction's row operand and the A tile's rows (m)
// its column operand, so a lane ends up holding 4 consecutive n of one m and
// the epilogue can store vectors along a row of C.
//   acc[v] <-> m = lane % 32,  n = 8*(v/4) + 4*(lane/32) + v%4     (within the 32x32 block)
// ---------------------------------------------------------------------------
template <int DT>
PEAK_DEV void mfma_frag(f32x16 &acc, const u32x4 &bfrag, const u32x4 &afrag)
{
    if (DT == DT_BF16) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bfrag),
                                                      __builtin_bit_cast(bf16x8, afrag), acc, 0, 0, 0);
    } else if (DT == DT_F16) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, bfrag),
                                                     __builtin_bit_cast(f16x8, afrag), acc, 0, 0, 0);
    } else {
        // fp32: the chunk holds 4 k values per lane half; step s multiplies k = 4*half + s of both operands
        const f32x4 bq = __builtin_bit_cast(f32x4, bfrag), aq = __builtin_bit_cast(f32x4, afrag);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(bq[0], aq[0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(bq[1], aq[1], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(bq[2], aq[2], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(bq[3], aq[3], acc, 0, 0, 0);
    }
}

template <int DT>
PEAK_DEV float elem_to_float(const void *p, int64_t idx)
{
    if (DT == DT_F32) return ((const float *)p)[idx];
    if (DT == DT_F16) return (float)((const _Float16 *)p)[idx];
    return (float)((const __bf16 *)p)[idx];
}

template <int DT>
PEAK_DEV void float_to_elem(void *p, int64_t idx, float x)
{
    if (DT == DT_F32) ((float *)p)[idx] = x;
    else if (DT == DT_F16) ((_Float16 *)p)[idx] = (_Float16)x;       // round to nearest even
    else ((__bf16 *)p)[idx] = (__bf16)x;                             // round to nearest even
}

// The fused output step on NE values: v <- act(v + b).
// (The choices are made outside the element loops, which then unroll.)
template <int NE>
PEAK_DEV void hook_apply(int act, bool has_bias, float (&v)[NE], const float (&b)[NE])
{
    if (has_bias) {
#pragma unroll
        for (int e = 0; e < NE; ++e) v[e] += b[e];
    }
    if (act == ACT_RELU) {
#pragma unroll
        for (int e = 0; e < NE; ++e) v[e] = v[e] > 0.0f ? v[e] : 0.0f;
    } else if (act == ACT_GELU_TANH) {
        // v/2 * (1 + tanh(u)) = v / (1 + exp(-2u)),  u = sqrt(2/pi) * (v + 0.044715 v^3);
        // -2u*log2(e) = v * (c1 + c3 v^2), one hardware exp2 and one hardware reciprocal (1 ulp each)
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const float t = v[e] * (-2.302208198f + -0.1029432396f * v[e] * v[e]);
            v[e] = v[e] * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t));
        }
    }
}

PEAK_DEV bool hook_active(const Hook &h) { return (h.bias_kind | h.act) != 0; }

// Bias of nvalid (1..4) consecutive outputs of row m, from column n on.
PEAK_DEV void hook_bias4(const Hook &h, int64_t m, int64_t n, int nvalid, float (&b)[4])
{
    b[0] = b[1] = b[2] = b[3] = 0.0f;
    if (h.bias_kind == BIAS_PER_COLUMN) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (e < nvalid) b[e] = h.bias[n + e];
    } else if (h.bias_kind == BIAS_PER_ROW) {
        b[0] = b[1] = b[2] = b[3] = h.bias[m];
    }
}

// Stores nvalid (1..4) consecutive elements of one row of C, rounded once:
// C[idx + e] = act(alpha * x[e] + beta * C[idx + e] + b[e]); the fused step (act, b)
// only with `hooked`.
template <int DT>
PEAK_DEV void store4(void *C, int64_t idx, const float x[4], float alpha, float beta, bool vec, int nvalid,
                     bool hooked, int act, bool has_bias, const float (&b)[4])
{
    if (vec && nvalid == 4) {
        float o[4] = {alpha * x[0], alpha * x[1], alpha * x[2], alpha * x[3]};
        if (DT == DT_F32) {
            if (beta != 0.0f) {
                const f32x4 c = *(const f32x4 *)((const float *)C + idx);
                o[0] += beta * c[0]; o[1] += beta * c[1]; o[2] += beta * c[2]; o[3] += beta * c[3];
            }
            if (hooked) hook_apply(act, has_bias, o, b);
            const f32x4 ov = {o[0], o[1], o[2], o[3]};
            *(f32x4 *)((float *)C + idx) = ov;
        } else {
            if (beta != 0.0f) {
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] += beta * elem_to_float<DT>(C, idx + e);
            }
            if (hooked) hook_apply(act, has_bias, o, b);
            union { u32x2 u; _Float16 h[4]; __bf16 b[4]; } pk;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (DT == DT_F16) pk.h[e] = (_Float16)o[e];
                else pk.b[e] = (__bf16)o[e];
            }
            *(u32x2 *)((uint16_t *)C + idx) = pk.u;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (e < nvalid) {
                float o1[1] = {alpha * x[e]};
                if (beta != 0.0f) o1[0] += beta * elem_to_float<DT>(C, idx + e);
                const float b1[1] = {b[e]};
                if (hooked) hook_apply(act, has_bias, o1, b1);
                float_to_elem<DT>(C, idx + e, o1[0]);
            }
        }
    }
}

// ... without a fused step (split-K partials)
template <int DT>
PEAK_DEV void store4(void *C, int64_t idx, const float x[4], float alpha, float beta, bool vec, int nvalid)
{
    const float none[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    store4<DT>(C, idx, x, alpha, beta, vec, nvalid, false, ACT_NONE, false, none);
}

// ... with the fused step of `hk` for row m, columns n.. (fetches the bias itself)
template <int DT>
PEAK_DEV void store4(void *C, int64_t idx, const float x[4], float alpha, float beta, bool vec, int nvalid,
                     const Hook hk, int64_t m, int64_t n)
{
    float b[4];
    hook_bias4(hk, m, n, nvalid, b);
    store4<DT>(C, idx, x, alpha, beta, vec, nvalid, hook_active(hk), hk.act, hk.bias_kind != BIAS_NONE, b);
}

// Tile order (the paper's Block-Swizzle, made XCD-aware): consecutive workgroup
// ids go round-robin to the 8 XCDs, each with its own L2.  Give every XCD a
// contiguous run of the band-ordered tile list, so the tiles an XCD works on at
// one time share A row panels and B column panels in that L2.
PEAK_DEV void tile_of_block(int t, int tiles_m, int tiles_n, int group_m, int &tm, int &tn)
{
    const int total = tiles_m * tiles_n;
    const int xcd = t & 7, idx = t >> 3;
    const int base = total >> 3, rem = total & 7;
    const int L = xcd * base + (xcd < rem ? xcd : rem) + idx;
    const int band = group_m * tiles_n;
    const int g = L / band;
    const int first = g * group_m;
    const int gsz = (tiles_m - first) < group_m ? (tiles_m - first) : group_m;
    const int w = L - g * band;
    tm = first + w % gsz;
    tn = w / gsz;
}

// ---------------------------------------------------------------------------
// Epilogue shared by the tiled kernels.  Each wave turns its wave tile around in
// LDS, one slab of 32 rows at a time, so that a store instruction writes whole
// row segments of C.  How the accumulators of a slab get into LDS depends on the
// MFMA block shape and is the caller's part:
//   write_slab(s, scr)    raw fp32 accumulators of slab s to scr[row * SROW + 4 * col], SROW = WTN * 4 + 16
//   write16(s, scr16)     (16-bit kernels) alpha * acc rounded to the storage type, 8 bytes per 4-column
//                         group g = col / 4 at scr16[row * SROW16 + 8 * (g ^ (row >> 4))], SROW16 = WTN * 2 + 16
// ---------------------------------------------------------------------------
// Where a workgroup that holds a K slice puts its fp32 partial tile: element (m, n) of C goes to
// base[(m - m_org) * ld + (n - n_org)].  base == nullptr: the workgroup holds the whole of K
// and writes C itself.
struct PartialOut {
    float *base;
    int64_t ld, m_org, n_org;
    bool vec;                 // rows allow 16-byte access
};

// Split-K: slice s of every tile goes to its own M x N plane of the workspace.
PEAK_DEV PartialOut splitk_out(const GemmArgs &p, int slice)
{
    if (p.split <= 1) return PartialOut{nullptr, 0, 0, 0, false};
    return PartialOut{p.ws + (int64_t)slice * p.M * p.N, p.N, 0, 0, (p.flags & GF_WS_VEC) != 0};
}

template <class C, int SLABS, class WriteSlab, class Write16>
PEAK_DEV void epilogue_slabs(const GemmArgs &p, char *lds, int wave, int lane, int wm, int wn, int64_t m0, int64_t n0,
                             const PartialOut &po, WriteSlab &&write_slab, Write16 &&write16)
{
    const bool c_vec = p.flags & GF_C_VEC, ws_vec = po.vec;
    float *wsl = po.base;
    const bool interior = m0 + C::BM <= p.M && n0 + C::BN <= p.N;      // whole tile inside C: no masks
    // Each wave turns its 32-row slabs around in LDS (fp32, padded rows) so that a
    // store instruction writes whole row segments of the wave tile (16 bytes per
    // lane, WTN elements per row) instead of 32 scattered 8-byte pieces.  Interior
    // tiles with 16-byte aligned C rows store vectors; edge tiles, unaligned rows and
    // split-K partials leave through the same turnaround with masked stores, so the
    // accumulators have one way out and never wait in ordinary registers.
    constexpr int SROW = C::WTN * 4 + 16;                              // scratch row stride, bytes
    static_assert(32 * SROW * C::NW <= C::LDS_BYTES, "the staging buffers are large enough for the turnaround");
    {
        lds_barrier();                                                 // nobody still reads the last stage
        char *scr = lds + wave * (32 * SROW);
        constexpr int OUT_ROW = C::WTN * C::ESZ;                       // bytes of one output row of the wave tile
        constexpr int LPR = OUT_ROW / 16;                              // lanes per row on the way out
        constexpr int RPI = 64 / LPR;                                  // rows per store instruction
        static_assert(OUT_ROW % 16 == 0 && 64 % LPR == 0 && 32 % RPI == 0, "wave tile rows split into 16-byte pieces");
        const int orow = lane / LPR, ocol = (lane % LPR) * (16 / C::ESZ);   // row within the group, first column (elements)
        // fused step: a lane stores the same columns of every row, so their bias is fetched once
        const bool hooked = !wsl && hook_active(p.hook), has_bias = p.hook.bias_kind != BIAS_NONE;
        const bool c_f32 = C::DT != DT_F32 && (p.flags & GF_C_F32);    // fp32 C of a 16-bit kernel: masked readout
        constexpr int EPL = 16 / C::ESZ;                               // elements per lane and row
        float bcol[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) bcol[e] = 0.0f;
        if (hooked && p.hook.bias_kind == BIAS_PER_COLUMN) {
            const int64_t n = n0 + wn * C::WTN + ocol;
#pragma unroll
            for (int e = 0; e < EPL; ++e)
                if (n + e < p.N) bcol[e] = p.hook.bias[n + e];
        }
        // Plain runs of the 16-bit kernels on interior tiles (beta == 0, no fused step): the slab
        // goes through LDS already scaled and rounded, 8 bytes per lane and 4-column group, which
        // halves the LDS traffic of the turnaround; the way back is a 16-byte read and the store.
        // Rows r and r + 16 would meet in the same banks (row stride = 4 banks mod 64), so the
        // 8-byte groups of rows 16..31 swap places pairwise; the reader swaps them back.
        if constexpr (C::DT != DT_F32) {
            if (interior && !wsl && (p.flags & GF_C_VEC16) && !c_f32 && p.beta == 0.0f && !hooked) {
                constexpr int SROW16 = C::WTN * 2 + 16;
                constexpr int G = 32 / RPI;
                char *scr16 = lds + wave * (32 * SROW16);
                write16(0, scr16);
#pragma unroll
                for (int mi = 0; mi < SLABS; ++mi) {
                    u32x4 v[G];
#pragma unroll
                    for (int g = 0; g < G; ++g)
                        v[g] = *(const u32x4 *)(scr16 + (g * RPI + orow) * SROW16 + ocol * 2);
                    if (mi + 1 < SLABS) write16(mi + 1, scr16);      // in-order LDS: lands after the reads above
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const int64_t m = m0 + wm * C::WTM + mi * 32 + g * RPI + orow;
                        const int64_t n = n0 + wn * C::WTN + ocol;
                        const u32x4 o = (((g * RPI) >> 4) & 1) ? u32x4{v[g][2], v[g][3], v[g][0], v[g][1]} : v[g];
                        *(u32x4 *)((uint16_t *)p.C + m * p.ldc + n) = o;
                    }
                }
                return;
            }
        }
        // A wave's LDS instructions execute in the order issued, so the next slab may be
        // written into the same scratch as soon as this slab's reads are issued: the writes
        // then run while this slab is converted and stored.
        write_slab(0, scr);
#pragma unroll
        for (int mi = 0; mi < SLABS; ++mi) {
            float brow = 0.0f;                                         // per-row bias of slab row (lane % 32)
            if (hooked && p.hook.bias_kind == BIAS_PER_ROW) {
                const int64_t m = m0 + wm * C::WTM + mi * 32 + (lane & 31);
                if (m < p.M) brow = p.hook.bias[m];
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);         // one slab's accumulators out of the accumulation registers at a time
            // 16-byte stores need aligned rows; on edge tiles also that no lane's column group
            // straddles N (then a group is either stored whole or not at all)
            const bool vec_ok = !wsl && (p.flags & GF_C_VEC16) && !c_f32 && (interior || p.N % EPL == 0);
            if (!vec_ok) {
                // masked 4-element stores
#pragma unroll 1
                for (int g = 0; g < 32 / RPI; ++g) {
                    const int row = g * RPI + orow;
                    const int64_t m = m0 + wm * C::WTM + mi * 32 + row;
                    const int64_t n = n0 + wn * C::WTN + ocol;
                    const char *src = scr + row * SROW + ocol * 4;
                    const float br = __shfl(brow, row);                // (every lane takes part)
                    if (m < p.M) {
#pragma unroll
                        for (int q = 0; q < 4 / C::ESZ; ++q) {         // 4 elements at a time
                            const int64_t nn = n + q * 4, left = p.N - nn;
                            if (left > 0) {
                                const int nvalid = left >= 4 ? 4 : (int)left;
                                const f32x4 t = *(const f32x4 *)(src + q * 16);
                                const float x[4] = {t[0], t[1], t[2], t[3]};
                                if (wsl) store4<DT_F32>(wsl, (m - po.m_org) * po.ld + (nn - po.n_org), x, 1.0f, 0.0f, ws_vec, nvalid);
                                else {
                                    const bool per_row = p.hook.bias_kind == BIAS_PER_ROW;
                                    const float b[4] = {per_row ? br : bcol[q * 4 + 0], per_row ? br : bcol[q * 4 + 1],
                                                        per_row ? br : bcol[q * 4 + 2], per_row ? br : bcol[q * 4 + 3]};
                                    if (c_f32)
                                        store4<DT_F32>(p.C, m * p.ldc + nn, x, p.alpha, p.beta, c_vec, nvalid,
                                                       hooked, p.hook.act, has_bias, b);
                                    else
                                        store4<C::DT>(p.C, m * p.ldc + nn, x, p.alpha, p.beta, c_vec, nvalid,
                                                      hooked, p.hook.act, has_bias, b);
                                }
                            }
                        }
                    }
                }
                if (mi + 1 < SLABS) write_slab(mi + 1, scr);
            } else {
                // All rows of the slab are fetched from LDS first, so that one LDS latency is
                // paid per slab and not per row; PLAIN (interior, beta == 0, no fused step) is straight-line.
                auto vector_readout = [&](auto plain_c) {
                    constexpr bool PLAIN = decltype(plain_c)::value != 0;
                    constexpr int G = 32 / RPI;
                    // beta != 0: the slab's C_in is asked for first, all rows at once, so that its way
                    // from memory overlaps the LDS turnaround instead of following it row by row
                    u32x4 cin[G];
                    const bool need_c = !PLAIN && p.beta != 0.0f;
                    if (need_c) {
#pragma unroll
                        for (int g = 0; g < G; ++g) {
                            const int64_t m = m0 + wm * C::WTM + mi * 32 + g * RPI + orow;
                            const int64_t n = n0 + wn * C::WTN + ocol;
                            cin[g] = u32x4{0u, 0u, 0u, 0u};
                            if (interior || (m < p.M && n + EPL <= p.N))
                                cin[g] = *(const u32x4 *)((const char *)p.C + (m * p.ldc + n) * C::ESZ);
                        }
                    }
                    f32x4 lo[G], hi[G];
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const char *src = scr + (g * RPI + orow) * SROW + ocol * 4;
                        lo[g] = *(const f32x4 *)src;
                        if constexpr (C::DT != DT_F32) hi[g] = *(const f32x4 *)(src + 16);
                    }
                    // per-row bias of the rows this lane stores, handed round (every lane takes part)
                    // before the next slab's writes queue up behind the shuffles
                    float brs[G];
                    const bool per_row = !PLAIN && hooked && p.hook.bias_kind == BIAS_PER_ROW;
                    if (per_row) {
#pragma unroll
                        for (int g = 0; g < G; ++g) brs[g] = __shfl(brow, g * RPI + orow);
                    }
                    if (mi + 1 < SLABS) write_slab(mi + 1, scr);
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const int row = g * RPI + orow;
                        const int64_t m = m0 + wm * C::WTM + mi * 32 + row;
                        const int64_t n = n0 + wn * C::WTN + ocol;
                        float b[EPL];                                  // this row's bias, if any
                        if (!PLAIN && !interior && !(m < p.M && n + EPL <= p.N)) continue;
                        if (!PLAIN && hooked) {
#pragma unroll
                            for (int e = 0; e < EPL; ++e) b[e] = per_row ? brs[g] : bcol[e];
                        }
                        if constexpr (C::DT == DT_F32) {
                            f32x4 o = lo[g];
                            o[0] *= p.alpha; o[1] *= p.alpha; o[2] *= p.alpha; o[3] *= p.alpha;
                            float *dst = (float *)p.C + m * p.ldc + n;
                            if (need_c) {
                                const f32x4 c = __builtin_bit_cast(f32x4, cin[g]);
                                o[0] += p.beta * c[0]; o[1] += p.beta * c[1]; o[2] += p.beta * c[2]; o[3] += p.beta * c[3];
                            }
                            if (!PLAIN && hooked) {
                                float oh[4] = {o[0], o[1], o[2], o[3]};
                                hook_apply(p.hook.act, has_bias, oh, b);
                                o[0] = oh[0]; o[1] = oh[1]; o[2] = oh[2]; o[3] = oh[3];
                            }
                            *(f32x4 *)dst = o;
                        } else {
                            float o[8] = {p.alpha * lo[g][0], p.alpha * lo[g][1], p.alpha * lo[g][2], p.alpha * lo[g][3],
                                          p.alpha * hi[g][0], p.alpha * hi[g][1], p.alpha * hi[g][2], p.alpha * hi[g][3]};
                            uint16_t *dst = (uint16_t *)p.C + m * p.ldc + n;
                            union { u32x4 u; _Float16 h[8]; __bf16 b[8]; } pk;
                            if (need_c) {
                                pk.u = cin[g];
#pragma unroll
                                for (int e = 0; e < 8; ++e) o[e] += p.beta * (C::DT == DT_F16 ? (float)pk.h[e] : (float)pk.b[e]);
                            }
                            if (!PLAIN && hooked) hook_apply(p.hook.act, has_bias, o, b);
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                if (C::DT == DT_F16) pk.h[e] = (_Float16)o[e];
                                else pk.b[e] = (__bf16)o[e];
                            }
                            *(u32x4 *)dst = pk.u;
                        }
                    }
                };
                if (p.beta == 0.0f && !hooked && interior) vector_readout(IC<1>{});
                else vector_readout(IC<0>{});
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// ---------------------------------------------------------------------------
// The GEMM kernel.
// ---------------------------------------------------------------------------
template <class C>
__global__ __launch_bounds__(C::NT) void gemm_kernel(const GemmArgs p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the kernel's symbol; the body uses device-only builtins
    __shared__ __attribute__((aligned(1024))) char lds[C::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
#ifdef PEAK_TRACE
    // Diagnostic build only: per wave, shader-clock time stamps of the kernel's phases and the
    // cycles spent at the K loop's waits, written to the workspace (see trace_store below).
    const uint64_t tr_start = __builtin_amdgcn_s_memtime();
    uint64_t tr_loop0 = 0, tr_loop1 = 0, tr_w0 = 0, tr_w1 = 0, tr_wait_sum = 0, tr_wait_max = 0;
    auto trace_store = [&]() {
        if (p.split == 1 && p.ws && lane == 0) {
            const uint64_t tr_end = __builtin_amdgcn_s_memtime();
            uint32_t hwid, xcc;
            asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hwid));
            asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
            uint64_t *dst = (uint64_t *)p.ws + ((size_t)blockIdx.x * C::NW + wave) * 8;
            dst[0] = tr_start; dst[1] = tr_loop0; dst[2] = tr_loop1; dst[3] = tr_end;
            dst[4] = tr_wait_sum; dst[5] = tr_wait_max; dst[6] = (uint64_t)hwid | ((uint64_t)xcc << 32); dst[7] = (uint64_t)p.ktiles_total;
        }
    };
#endif
    const int r32 = lane & 31, half = lane >> 5;

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
    const int64_t kend = p.K;                               // zero fill beyond K (only the last slice can reach it)

    const bool a_vec = p.flags & GF_A_VEC, b_vec = p.flags & GF_B_VEC;

    f32x16 acc[C::MI][C::NI];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    // per-lane fragment addresses within a stage (chunk 2*kg + half of row r sits at (2*kg) ^ x, x below)
    int a_addr[C::MI], b_addr[C::NI];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi) {
        const int r = wm * C::WTM + mi * 32 + r32;
        a_addr[mi] = r * C::RB + ((half ^ swz<C::CPR>(r)) << 4);
        if (C::A_TR && C::DT == DT_F32) {
            a_addr[mi] = (4 * half) * (C::BM * 4) + r * 4;
        } else if (C::A_TR) {
            const int i16 = lane & 15, g16 = (lane & 31) >> 4;
            const int krow = half * 8 + (i16 >> 2);
            const int mcol = wm * C::WTM + mi * 32 + 16 * g16 + 4 * (i16 & 3);
            a_addr[mi] = krow * (C::BM * C::ESZ) + (((mcol >> 3) ^ (4 * (krow & 3))) << 4) + (i16 & 1) * 8;
        }
    }
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) {
        const int r = wn * C::WTN + ni * 32 + r32;
        // (the B region's offset is part of the address, so that the stage offset left over
        // for the read instruction fits its 16-bit immediate field)
        b_addr[ni] = C::NSA * C::A_BYTES + r * C::RB + ((half ^ swz<C::CPR>(r)) << 4);
        if (C::B_TR && C::DT == DT_F32) {
            // [k][n] rows of floats: lane reads row 8*kg + 4*half + step, column n
            b_addr[ni] = C::NSA * C::A_BYTES + (4 * half) * (C::BN * 4) + r * 4;
        } else if (C::B_TR) {
            // transposing read: the 16 lanes of a group cover 4 k-rows x 16 n; lane i of the group
            // points at k-row i/4, columns 4*(i%4) .. +3 of its group's 16
            const int i16 = lane & 15, g16 = (lane & 31) >> 4;
            const int krow = half * 8 + (i16 >> 2);
            const int ncol = wn * C::WTN + ni * 32 + 16 * g16 + 4 * (i16 & 3);
            b_addr[ni] = C::NSA * C::A_BYTES + krow * (C::BN * C::ESZ) + (((ncol >> 3) ^ (4 * (krow & 3))) << 4) + (i16 & 1) * 8;
        }
    }
    // fragment of A for k-group kg: 8 k per lane (the [k][m] forms mirror read_b below)
    auto read_a = [&](const char *sta, int mi, int kg) -> u32x4 {
        if (C::A_TR && C::DT == DT_F32) {
            const char *q0 = sta + a_addr[mi] + (8 * kg) * (C::BM * 4);
            return u32x4{*(const uint32_t *)q0, *(const uint32_t *)(q0 + C::BM * 4), *(const uint32_t *)(q0 + 2 * C::BM * 4),
                         *(const uint32_t *)(q0 + 3 * C::BM * 4)};
        }
        if (C::A_TR) {
            typedef short s16x4 __attribute__((ext_vector_type(4)));
            const char *q0 = sta + a_addr[mi] + (16 * kg) * (C::BM * C::ESZ);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)q0);
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(q0 + 4 * (C::BM * C::ESZ)));
            const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
            return u32x4{l2[0], l2[1], h2[0], h2[1]};
        }
        return *(const u32x4 *)(sta + (a_addr[mi] ^ (kg << 5)));
    };
    // fragment of B for k-group kg: 8 k per lane
    auto read_b = [&](const char *stb, int ni, int kg) -> u32x4 {
        if (C::B_TR && C::DT == DT_F32) {
            const char *q0 = stb + b_addr[ni] + (8 * kg) * (C::BN * 4);
            return u32x4{*(const uint32_t *)q0, *(const uint32_t *)(q0 + C::BN * 4), *(const uint32_t *)(q0 + 2 * C::BN * 4),
                         *(const uint32_t *)(q0 + 3 * C::BN * 4)};
        }
        if (C::B_TR) {
            typedef short s16x4 __attribute__((ext_vector_type(4)));
            const char *q0 = stb + b_addr[ni] + (16 * kg) * (C::BN * C::ESZ);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)q0);
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(q0 + 4 * (C::BN * C::ESZ)));
            const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
            return u32x4{l2[0], l2[1], h2[0], h2[1]};
        }
        return *(const u32x4 *)(stb + (b_addr[ni] ^ (kg << 5)));
    };

    // operand loaders
    constexpr bool A_DIRECT = C::DIRECT && (!C::A_T || C::A_TR), B_DIRECT = C::DIRECT && (!C::B_T || C::B_TR);
    LoaderDirect<C, C::BM> dA;
    LoaderDirect<C, C::BN> dB;
    LoaderDirectKN<C, C::BM> nA;
    LoaderDirectKN<C, C::BN> nB;
    LoaderK<C, C::BM> kA;
    LoaderK<C, C::BN> kB;
    LoaderT<C, C::BM> tA;
    LoaderT<C, C::BN> tB;
    // loads per thread and tile that stay in flight across iterations
    constexpr int LA = !A_DIRECT ? 0 : (C::A_TR ? LoaderDirectKN<C, C::BM>::PER_WAVE : LoaderDirect<C, C::BM>::PER_WAVE);
    constexpr int LB = !B_DIRECT ? 0 : (C::B_TR ? LoaderDirectKN<C, C::BN>::PER_WAVE : LoaderDirect<C, C::BN>::PER_WAVE);
    constexpr int DLOADS = LA + LB;
    constexpr int P = C::NS - 1;                            // prefetch distance of the direct loads
    static_assert(!A_DIRECT || (C::A_TR ? LoaderDirectKN<C, C::BM>::NINST : LoaderDirect<C, C::BM>::NINST) % C::NW == 0, "every wave issues the same number of loads");
    static_assert(!B_DIRECT || (C::B_TR ? LoaderDirectKN<C, C::BN>::NINST : LoaderDirect<C, C::BN>::NINST) % C::NW == 0, "every wave issues the same number of loads");

    // valid k in the matrix's last K tile; only the slice that holds that tile can see a short one
    const int tail_k = __builtin_amdgcn_readfirstlane((int)(p.K - (int64_t)(p.ktiles_total - 1) * C::BK));
    const int tail_tile = tail_k < C::BK ? p.ktiles_total - 1 - kt_begin : -1;   // relative to the slice
    if (A_DIRECT && !C::A_TR) dA.init(p.A, p.lda, m0, p.M, kbase, p.K, tail_k, wave, lane);
    if (A_DIRECT && C::A_TR) nA.init(p.A, p.lda, m0, p.M, kbase, p.K, tail_k, wave, lane);
    if (B_DIRECT && !C::B_TR) dB.init(p.B, p.ldb, n0, p.N, kbase, p.K, tail_k, wave, lane);
    if (B_DIRECT && C::B_TR) nB.init(p.B, p.ldb, n0, p.N, kbase, p.K, tail_k, wave, lane);

    auto a_stage = [&](int s) { return lds + s * C::A_BYTES; };
    auto b_stage = [&](int s) { return lds + C::NSA * C::A_BYTES + s * C::B_BYTES; };   // for the loaders
    auto b_frag_base = [&](int s) { return lds + s * C::B_BYTES; };                     // for read_b (b_addr holds the rest)

    // K rotation: this workgroup walks its K tiles starting at tile `rot` and
    // wraps around.  Workgroups that share an A or B panel in one XCD's L2 start
    // at different tiles, so one of them touches a chunk first and the others,
    // a step or two later, find it in L2 instead of all waiting on the same miss.
    const int rot = __builtin_amdgcn_readfirstlane(((tm & 7) * p.rot_m + (tn & 3) * p.rot_n) % KT);
    auto rotated = [&](int kt) {
        const int kr = kt + rot;
        return kr >= KT ? kr - KT : kr;
    };
    auto load_regs = [&](int kt) {                          // kt relative to the slice
        const int64_t k0 = kbase + (int64_t)rotated(kt) * C::BK;
        if (!A_DIRECT) {
            if (C::A_T) tA.load(p.A, p.lda, m0, p.M, k0, kend, a_vec, tid);
            else        kA.load(p.A, p.lda, m0, p.M, k0, kend, a_vec, tid);
        }
        if (!B_DIRECT) {
            if (C::B_T) tB.load(p.B, p.ldb, n0, p.N, k0, kend, b_vec, tid);
            else        kB.load(p.B, p.ldb, n0, p.N, k0, kend, b_vec, tid);
        }
    };
    auto store_regs = [&](int sa, int sb) {
        if (!A_DIRECT) {
            if (C::A_T) tA.store(a_stage(sa), tid); else kA.store(a_stage(sa), tid);
        }
        if (!B_DIRECT) {
            if (C::B_T) tB.store(b_stage(sb), tid); else kB.store(b_stage(sb), tid);
        }
    };
    // Direct loads of tile kt, part PART of NPARTS (the parts of a tile can be
    // issued between groups of MFMAs).  Past the end the last tile is fetched again
    // into a free stage, so the number of loads in flight stays what the waits assume.
    auto issue_a = [&](int kt, int sa, auto part, auto nparts) {
        constexpr int PART = decltype(part)::value, NPARTS = decltype(nparts)::value;
        const int kr = rotated(kt < KT ? kt : KT - 1);
        if (A_DIRECT && !C::A_TR) dA.template issue<PART, NPARTS>(a_stage(sa), kr, kr == tail_tile, wave);
        if (A_DIRECT && C::A_TR) nA.template issue<PART, NPARTS>(a_stage(sa), kr, kr == tail_tile, wave);
    };
    auto issue_b = [&](int kt, int sb, auto part, auto nparts) {
        constexpr int PART = decltype(part)::value, NPARTS = decltype(nparts)::value;
        const int kr = rotated(kt < KT ? kt : KT - 1);
        if (B_DIRECT && !C::B_TR) dB.template issue<PART, NPARTS>(b_stage(sb), kr, kr == tail_tile, wave);
        if (B_DIRECT && C::B_TR) nB.template issue<PART, NPARTS>(b_stage(sb), kr, kr == tail_tile, wave);
    };
    auto issue_direct_all = [&](int kt, int stage) {
        issue_a(kt, stage, IC<0>{}, IC<1>{});
        issue_b(kt, stage, IC<0>{}, IC<1>{});
    };
    auto mfma_half = [&](const u32x4 *af, const u32x4 *bf, auto half_c) {
        constexpr int H = decltype(half_c)::value;
        constexpr int MH = C::MI > 1 ? C::MI / 2 : 1;
        constexpr int M_LO = C::MI > 1 ? H * MH : 0, M_HI = C::MI > 1 ? (H + 1) * MH : (H == 0 ? 1 : 0);
        if (C::DT == DT_F32) {
            // k step outermost: consecutive MFMAs go to different accumulators instead of
            // four in a row waiting on the same one
#pragma unroll
            for (int st = 0; st < 4; ++st)
#pragma unroll
                for (int mi = M_LO; mi < M_HI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < C::NI; ++ni) {
                        const f32x4 bq = __builtin_bit_cast(f32x4, bf[ni]), aq = __builtin_bit_cast(f32x4, af[mi]);
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(bq[st], aq[st], acc[mi][ni], 0, 0, 0);
                    }
        } else {
#pragma unroll
            for (int mi = M_LO; mi < M_HI; ++mi)
#pragma unroll
                for (int ni = 0; ni < C::NI; ++ni) mfma_frag<C::DT>(acc[mi][ni], bf[ni], af[mi]);
        }
    };
    // two-phase step: all k-groups of one stage
    auto compute = [&](int sa, int sb) {
        const char *sta = a_stage(sa), *stb = b_frag_base(sb);
#pragma unroll
        for (int kg = 0; kg < C::KG; ++kg) {
            u32x4 af[C::MI], bf[C::NI];
#pragma unroll
            for (int mi = 0; mi < C::MI; ++mi) af[mi] = read_a(sta, mi, kg);
#pragma unroll
            for (int ni = 0; ni < C::NI; ++ni) bf[ni] = read_b(stb, ni, kg);
            mfma_half(af, bf, IC<0>{});
            mfma_half(af, bf, IC<1>{});
            __builtin_amdgcn_sched_barrier(0);          // one k-group's fragments live at a time
        }
    };

    constexpr bool ALL_DIRECT = A_DIRECT && B_DIRECT;
    constexpr bool PREFETCH2 = ALL_DIRECT && C::NS == 2 && C::KG % 2 == 0 && !C::PP;
    if (C::PP) {
        // Alternating scheme.  Waves w and w+4 share a SIMD.  A K tile is worked off two
        // k-groups at a time; for each such part a wave first reads its fragments from
        // LDS (and, in a tile's first part, issues its share of the loads of a later
        // tile), then runs the part's MFMAs from registers.  The second group of four waves runs one
        // phase behind the first, so on every SIMD one wave is multiplying while the
        // other one is reading; a barrier ends every phase.
        // With two parts per tile:
        //   phase        4t      4t+1     4t+2     4t+3
        //   waves 0-3  read t.0  mul t.0  read t.1  mul t.1
        //   waves 4-7  mul t-1.1 read t.0 mul t.0   read t.1
        // Tile t's stage is free once its last read phase (4t+3) has ended.
        constexpr int HK = 2;                                       // k-groups per phase
        constexpr int UPT = C::KG / HK;                             // phase pairs per K tile
        const int grp = __builtin_amdgcn_readfirstlane(wave >> 2);
        u32x4 af[HK][C::MI], bf[HK][C::NI];
        auto fetch_half = [&](int stage, int h) {
            const char *sta = a_stage(stage), *stb = b_frag_base(stage);
#pragma unroll
            for (int kk = 0; kk < HK; ++kk) {
#pragma unroll
                for (int ni = 0; ni < C::NI; ++ni) bf[kk][ni] = read_b(stb, ni, h * HK + kk);
#pragma unroll
                for (int mi = 0; mi < C::MI; ++mi) af[kk][mi] = read_a(sta, mi, h * HK + kk);
            }
        };
        auto multiply_half = [&]() {
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int kk = 0; kk < HK; ++kk) {
                mfma_half(af[kk], bf[kk], IC<0>{});
                mfma_half(af[kk], bf[kk], IC<1>{});
            }
            __builtin_amdgcn_s_setprio(0);
        };
        auto end_phase = [&]() {
            __builtin_amdgcn_sched_barrier(0);
            lds_barrier();
            __builtin_amdgcn_sched_barrier(0);
        };
        // With NS stages the loads of tile t+NS-1 go out in the first read phase of
        // tile t (its stage held tile t-1, whose last read phase has just ended), and
        // before the barrier that precedes the first read of tile t+1 every wave has
        // waited until at most NS-2 of its tiles are still in flight.  Past the end
        // the last tile is fetched again, so that the count stays what the waits assume.
        constexpr int INFLIGHT = (C::NS - 2) * DLOADS;
#pragma unroll
        for (int s = 0; s < C::NS - 1; ++s) issue_direct_all(s, s);
        wait_vmcnt<INFLIGHT>();                                     // tile 0
        lds_barrier();
        if (grp == 1) end_phase();                                  // the second group starts one phase late
        for (int kt0 = 0; kt0 < KT; kt0 += C::NS) {
            static_for<C::NS>([&](auto sc) {
                constexpr int s = decltype(sc)::value;
                const int kt = kt0 + s;
                if (kt < KT) {
                    static_for<UPT>([&](auto hc) {
                        constexpr int h = decltype(hc)::value;
                        if (h == 0) issue_direct_all(kt + C::NS - 1, (s + C::NS - 1) % C::NS);
                        fetch_half(s, h);
                        if (h == UPT - 1 && grp == 1) wait_vmcnt<INFLIGHT>();
                        end_phase();
                        multiply_half();
                        if (h == UPT - 1 && grp == 0) wait_vmcnt<INFLIGHT>();
                        end_phase();
                    });
                }
            });
        }
        if (grp == 0) end_phase();                                  // the first group finishes one phase early
    } else if constexpr (PREFETCH2 && C::ACC_AGPR && !C::A_TR) {
        // One wave per SIMD.  Same scheme as the prefetch loop below (fragments one k-group
        // ahead, the tile's barrier before its last k-group, loads of tile kt+2 after it), but
        // nothing else runs on the SIMD while this wave issues its LDS reads and loads, so
        // the instruction order is fixed by hand: after each MFMA at most one fragment read
        // of the next k-group and at most one load.  The MFMAs are assembly (accumulators in
        // AGPRs); the compiler does not know their latencies, so the wait states that the
        // hardware needs between the zeroing of the accumulators and the first MFMA, and
        // between the last MFMA and the first read of an accumulator, are put in by hand.
        constexpr int NM = C::MI * C::NI, NFR = C::MI + C::NI;
        // (fp32: a slot is four MFMAs of 64 cycles and takes two loads where the tile has fewer slots than loads)
        constexpr int LPS = C::DT == DT_F32 && DLOADS > NM ? 2 : 1;     // loads per slot
        static_assert(NFR <= NM && DLOADS <= LPS * NM && C::MI == C::NI, "one read and one load (fp32: two) per MFMA slot");
        u32x4 af[2][C::MI], bf[2][C::NI];
        // B kept as [k][n] rows: its transposing reads go out as assembly (the compiler would put a
        // wait for all loads in front of each, see the loop below) into bl/bh and are handed over
        // at the start of the next k-group, when everything asked of LDS has arrived
        constexpr bool TRA = C::B_TR && C::DT != DT_F32;        // (fp32 [k][n] rows need no transposition: plain reads)
        u32x2 bl[2][C::NI], bh[2][C::NI];
        const uint32_t lds_b0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
        auto fetch_one = [&](int stage_a, int stage, int kg, auto setc, auto fc) {
            constexpr int set = decltype(setc)::value, f = decltype(fc)::value;
            // B0 A0 B1 A1 ...: the order in which the MFMAs below first need them
            if constexpr (f % 2 == 1) {
                af[set][f / 2] = read_a(a_stage(stage_a), f / 2, kg);
            } else if constexpr (TRA) {
                const uint32_t a0 = lds_b0 + stage * C::B_BYTES + b_addr[f / 2] + (16 * kg) * (C::BN * C::ESZ);
                u32x2 &lo = bl[set][f / 2], &hi = bh[set][f / 2];
                asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(a0) : "memory");
                asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(a0), "n"(4 * C::BN * C::ESZ) : "memory");
            } else {
                bf[set][f / 2] = read_b(b_frag_base(stage), f / 2, kg);
            }
        };
        auto settle = [&](auto setc) {
            constexpr int set = decltype(setc)::value;
            if constexpr (TRA) {
                __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));
#pragma unroll
                for (int i = 0; i < C::NI; ++i) {
                    u32x2 &lo = bl[set][i], &hi = bh[set][i];
                    asm volatile("" : "+v"(lo), "+v"(hi));
                    bf[set][i] = u32x4{lo[0], lo[1], hi[0], hi[1]};
                }
            }
        };
        auto mfma_one = [&](auto setc, auto ic) {
            constexpr int set = decltype(setc)::value, i = decltype(ic)::value;
            constexpr int mi = i / C::NI, ni = i % C::NI;
            f32x16 &c = acc[mi][ni];
            const u32x4 &b = bf[set][ni], &a = af[set][mi];
            if constexpr (C::DT == DT_BF16) {
                asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(b), "v"(a));
            } else if constexpr (C::DT == DT_F16) {
                asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(c) : "v"(b), "v"(a));
            } else {
                // fp32: a fragment holds 4 k per lane, one 32x32x2 MFMA each.  Slot i takes k step
                // i / 4 of four blocks, so that consecutive MFMAs write different accumulators and an
                // accumulator comes round again only 16 MFMAs later (the compiler, which would put the
                // wait states between dependent MFMAs, does not see inside these statements).
                // With four blocks in all (64x64 wave tile) a slot is one k step of all of them.
                static_assert(C::MI * C::NI == 16 || C::MI * C::NI == 4, "four blocks per slot");
                constexpr int SPK = C::MI * C::NI / 4;                   // slots per k step
                constexpr int st = i / SPK;
                static_for<4>([&](auto bc) {
                    constexpr int blk = (i % SPK) * 4 + decltype(bc)::value;
                    f32x16 &cc = acc[blk / C::NI][blk % C::NI];
                    const float bv = __builtin_bit_cast(f32x4, bf[set][blk % C::NI])[st];
                    const float av = __builtin_bit_cast(f32x4, af[set][blk / C::NI])[st];
                    asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, %2, %0" : "+a"(cc) : "v"(bv), "v"(av));
                });
            }
        };
        auto load_one = [&](int t, int stage, auto jc) {
            constexpr int j = decltype(jc)::value;
            if constexpr (j < LA) issue_a(t, stage, IC<j>{}, IC<LA>{});
            else issue_b(t, stage, IC<j - LA>{}, IC<LB>{});
        };
        static_for<C::MI * C::NI>([&](auto ic) {                        // accumulators into AGPRs now
            constexpr int i = decltype(ic)::value;
            f32x16 &c = acc[i / C::NI][i % C::NI];
            asm volatile("" : "+a"(c));
        });
        asm volatile("s_nop 7\n\ts_nop 7" ::: "memory");
        // With a third A stage, A's loads of tile kt+2 are spread over the whole of step kt
        // (APK per k-group) and have more than a step to land; B's follow the barrier, one
        // every other MFMA.  Without it all loads of tile kt+2 follow the barrier.
        constexpr bool AXP = C::NSA == 3;
        constexpr int APK = AXP ? LA / C::KG : 0;                       // A loads per k-group
        static_assert(!AXP || (LA % C::KG == 0 && APK >= 1), "A's loads divide over the k-groups");
        constexpr int U = AXP ? 6 : 2;
        constexpr int PENDING = AXP ? (C::KG - 1) * APK : 0;            // loads of the step under way at its barrier
        issue_direct_all(0, 0);
        wait_vmcnt<0>();
        lds_barrier();
#ifdef PEAK_TRACE
        tr_loop0 = __builtin_amdgcn_s_memtime();
#endif
        issue_b(1, 1, IC<0>{}, IC<1>{});
        issue_a(1, 1, IC<0>{}, IC<1>{});
        static_for<NFR>([&](auto fc) { fetch_one(0, 0, 0, IC<0>{}, fc); });
        for (int kt0 = 0; kt0 < KT; kt0 += U) {
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                constexpr int s = u % 2, sa = AXP ? u % 3 : s;
                constexpr int sa1 = AXP ? (sa + 1) % 3 : 1 - s, sa2 = AXP ? (sa + 2) % 3 : s;   // A stages of tiles kt+1, kt+2
                const int kt = kt0 + u;
                if (kt < KT) {
                    static_for<C::KG>([&](auto kgc) {
                        constexpr int kg = decltype(kgc)::value;
                        constexpr bool LAST = kg + 1 == C::KG;
                        constexpr int cur = kg & 1, nxt = cur ^ 1;
                        if constexpr (LAST) {
#ifdef PEAK_TRACE
                            tr_w0 = __builtin_amdgcn_s_memtime();
#endif
                            wait_vmcnt<PENDING>();                      // own loads of tile kt+1
                            lds_barrier();                              // tile kt+1 complete, tile kt read
#ifdef PEAK_TRACE
                            tr_w1 = __builtin_amdgcn_s_memtime();
#endif
                        }
                        settle(IC<cur>{});
#ifdef PEAK_TRACE
                        if constexpr (kg == 1) {
                            // the stamps of the step before: long since returned (the fragments this
                            // k-group needs were asked for after them and are waited for here anyway)
                            const uint64_t dw = tr_w1 - tr_w0;
                            tr_wait_sum += dw;
                            tr_wait_max = dw > tr_wait_max ? dw : tr_wait_max;
                        }
#endif
                        __builtin_amdgcn_sched_barrier(0);
                        static_for<NM>([&](auto ic) {
                            constexpr int i = decltype(ic)::value;
                            mfma_one(IC<cur>{}, ic);
                            if constexpr (i < NFR) {
                                if constexpr (LAST) fetch_one(sa1, 1 - s, 0, IC<nxt>{}, ic);
                                else fetch_one(sa, s, kg + 1, IC<nxt>{}, ic);
                            }
                            if constexpr (AXP) {
                                // A: load number kg*APK + q of tile kt+2 after MFMA q*(NM/APK) + 1
                                static_for<APK>([&](auto qc) {
                                    constexpr int q = decltype(qc)::value;
                                    if constexpr (i == q * (NM / APK) + 1) issue_a(kt + 2, sa2, IC<kg * APK + q>{}, IC<LA>{});
                                });
                                // B: after the barrier, one after every other MFMA (half of them a k-group
                                // later instead: no gain)
                                if constexpr (LAST && i % 2 == 0 && i / 2 < LB) issue_b(kt + 2, s, IC<i / 2>{}, IC<LB>{});
                            } else {
                                if constexpr (LAST && LPS * i < DLOADS) load_one(kt + 2, s, IC<LPS * i>{});
                                if constexpr (LAST && LPS == 2 && LPS * i + 1 < DLOADS) load_one(kt + 2, s, IC<(LPS * i + 1 < DLOADS ? LPS * i + 1 : 0)>{});
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        });
                    });
                }
            });
        }
        settle(IC<0>{});      // the last k-group's reads feed nothing, but must have returned before their registers are reused
        // 32x32x16 MFMA: 8 passes of 4 cycles; an accumulator may be read 18 wait states after the issue
        // (32x32x2 fp32: 16 passes)
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        if constexpr (C::DT == DT_F32) asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#ifdef PEAK_TRACE
        tr_loop1 = __builtin_amdgcn_s_memtime();
#endif
        static_for<C::MI * C::NI>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            f32x16 &c = acc[i / C::NI][i % C::NI];
            asm volatile("" : "+a"(c));
        });
    } else if (PREFETCH2) {
        // Two stages, fragments one k-group ahead.  The barrier of a tile sits before
        // its last k-group: by then every wave has read all of the tile (the last
        // k-group's fragments were fetched one k-group earlier) and has waited for its
        // own loads of the next tile.  So after it the tile's stage can be refilled
        // (tile kt+2, a whole step before it is needed) and the next tile's first
        // fragments can be fetched, and the MFMA stream never waits on LDS.
        u32x4 af[2][C::MI], bf[2][C::NI];
        // The compiler's wait-count pass puts s_waitcnt vmcnt(0) in front of every
        // transposing LDS read that follows a direct-to-LDS load (it takes them to alias),
        // which would expose the whole load latency once per tile.  So the transposing
        // reads of this loop are issued as assembly, into the halves bl/bh, and their
        // completion is waited for by hand: at the start of each k-group everything the
        // wave has asked of LDS (the fragments fetched one k-group earlier) has arrived.
        // In-order return of LDS data keeps the compiler's own lgkmcnt waits for the A
        // fragments valid with the extra reads in between (they can only over-wait).
        constexpr bool TR_ASM = C::B_TR && C::DT != DT_F32, ATR_ASM = C::A_TR && C::DT != DT_F32;
        u32x2 bl[2][C::NI], bh[2][C::NI], al[2][C::MI], ah[2][C::MI];
        const uint32_t lds_b0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
        auto fetch = [&](int stage_a, int stage, int kg, int set) {
            const char *sta = a_stage(stage_a), *stb = b_frag_base(stage);
#pragma unroll
            for (int i = 0; i < (C::MI > C::NI ? C::MI : C::NI); ++i) {
                if (i < C::NI) {
                    if constexpr (TR_ASM) {
                        const uint32_t a0 = lds_b0 + stage * C::B_BYTES + b_addr[i] + (16 * kg) * (C::BN * C::ESZ);
                        asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(bl[set][i]) : "v"(a0) : "memory");
                        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(bh[set][i]) : "v"(a0), "n"(4 * C::BN * C::ESZ) : "memory");
                    } else {
                        bf[set][i] = read_b(stb, i, kg);
                    }
                }
                if (i < C::MI) {
                    if constexpr (ATR_ASM) {
                        const uint32_t a0 = lds_b0 + stage_a * C::A_BYTES + a_addr[i] + (16 * kg) * (C::BM * C::ESZ);
                        asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(al[set][i]) : "v"(a0) : "memory");
                        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(ah[set][i]) : "v"(a0), "n"(4 * C::BM * C::ESZ) : "memory");
                    } else {
                        af[set][i] = read_a(sta, i, kg);
                    }
                }
            }
        };
        // the assembly-read fragments of `set` have arrived (see above): hand them to the compiler
        auto settle = [&](auto setc) {
            constexpr int set = decltype(setc)::value;
            if constexpr (TR_ASM || ATR_ASM) {
                __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));
                if constexpr (TR_ASM) {
#pragma unroll
                    for (int i = 0; i < C::NI; ++i) {
                        asm volatile("" : "+v"(bl[set][i]), "+v"(bh[set][i]));
                        bf[set][i] = u32x4{bl[set][i][0], bl[set][i][1], bh[set][i][0], bh[set][i][1]};
                    }
                }
                if constexpr (ATR_ASM) {
#pragma unroll
                    for (int i = 0; i < C::MI; ++i) {
                        asm volatile("" : "+v"(al[set][i]), "+v"(ah[set][i]));
                        af[set][i] = u32x4{al[set][i][0], al[set][i][1], ah[set][i][0], ah[set][i][1]};
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // With two waves per SIMD (waves w and w+4), the second wave issues its loads one
        // k-group after the first: a wave can sit at its load instructions for a while
        // when the CU's load queue is full, and this way the other wave of the SIMD is
        // multiplying meanwhile instead of sitting there as well.
        constexpr bool STAGGER = C::NW == 8 && C::KG >= 3 && C::DT != DT_F32;   // (fp32: measured slightly worse)
        const int grp = __builtin_amdgcn_readfirstlane(wave >> 2);
        // Three A stages (asymmetric ring): the stage of A tile kt+2 is free a whole step
        // before B's, so its loads go out one per k-group through step kt and have more
        // than a step to land; only B's loads leave in a burst after the barrier.
        constexpr bool AXP = PREFETCH2 && C::NSA == 3;
        static_assert(!AXP || (LA == C::KG && C::NSB == 2), "one A load per wave and k-group");
        constexpr int U = AXP ? 6 : 2;                               // tiles per trip: both stage indices static
        constexpr int BPARTS = 1;                                    // B's loads in one burst (half of them a k-group later: no gain)
        constexpr int PENDING = AXP ? C::KG - 1 : 0;                 // loads of the step under way at its barrier
        issue_direct_all(0, 0);
        wait_vmcnt<0>();
        lds_barrier();
        if (AXP) {
            issue_b(1, 1, IC<0>{}, IC<BPARTS>{});
            issue_a(1, 1, IC<0>{}, IC<1>{});
        } else if (!STAGGER || grp == 0) {
            issue_direct_all(1, 1);
        }
        fetch(0, 0, 0, 0);
        for (int kt0 = 0; kt0 < KT; kt0 += U) {
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                constexpr int s = u % 2, sa = AXP ? u % 3 : s;       // stages of tile kt: B's and A's
                const int kt = kt0 + u;
                if (kt < KT) {
                    static_for<C::KG>([&](auto kgc) {
                        constexpr int kg = decltype(kgc)::value;
                        constexpr bool LAST = kg + 1 == C::KG;
                        if constexpr (LAST) {
                            wait_vmcnt<PENDING>();                      // own loads of tile kt+1
                            lds_barrier();                              // tile kt+1 complete, tile kt read
                            settle(IC<(kg & 1)>{});
                            if constexpr (AXP) {
                                issue_b(kt + 2, s, IC<0>{}, IC<BPARTS>{});
                                issue_a(kt + 2, (sa + 2) % 3, kgc, IC<C::KG>{});
                            } else if (!STAGGER || grp == 0) {
                                issue_direct_all(kt + 2, s);
                            }
                            fetch(AXP ? (sa + 1) % 3 : 1 - s, 1 - s, 0, 0);
                        } else {
                            settle(IC<(kg & 1)>{});
                            if constexpr (AXP) {
                                if constexpr (kg == 0 && BPARTS == 2) issue_b(kt + 1, 1 - s, IC<1>{}, IC<2>{});
                                issue_a(kt + 2, (sa + 2) % 3, kgc, IC<C::KG>{});
                            } else if constexpr (kg == 0) {
                                if (STAGGER && grp == 1) issue_direct_all(kt + 1, 1 - s);
                            }
                            fetch(sa, s, kg + 1, (kg + 1) & 1);
                        }
                        mfma_half(af[kg & 1], bf[kg & 1], IC<0>{});
                        mfma_half(af[kg & 1], bf[kg & 1], IC<1>{});
                        constexpr int NMFMA = C::MI * C::NI * (C::DT == DT_F32 ? 4 : 1);
                        constexpr int NDS = (ATR_ASM ? 0 : C::MI * (!C::A_TR ? 1 : 4)) + (TR_ASM ? 0 : C::NI * (!C::B_TR ? 1 : 4));
                        constexpr int NVM = AXP ? (LAST ? LB + 1 : 1) : (LAST ? DLOADS : 0);
                        constexpr int PER = C::DT == DT_F32 ? 4 : 1;       // MFMAs per slot
                        static_for<NMFMA / PER>([&](auto ic) {
                            constexpr int i = decltype(ic)::value;
                            __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);
                            if constexpr (i < NDS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                            else if constexpr (i - NDS < NVM) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                        });
                        __builtin_amdgcn_sched_barrier(0);
                    });
                }
            });
        }
        // The last k-group fetched fragments of a tile that does not exist.  Reads issued as
        // assembly must still be waited for and their registers kept until then: the compiler
        // takes the unused results for dead, and an LDS read that returns after its registers
        // were given to something else (an address of the epilogue, say) would overwrite it.
        settle(IC<0>{});
    } else if (!C::PIPE) {
        // Two-phase scheme: at the barrier of step kt tile kt is complete; its
        // fragments are read after the barrier.
        if (DLOADS > 0) {
#pragma unroll
            for (int s = 0; s < P; ++s) issue_direct_all(s, s);
        }
        if (!ALL_DIRECT) {
            load_regs(0);
            store_regs(0, 0);
        }
        for (int kt0 = 0; kt0 < KT; kt0 += C::NS) {
#pragma unroll
            for (int s = 0; s < C::NS; ++s) {
                const int kt = kt0 + s;
                if (kt < KT) {
                    if (DLOADS > 0) wait_vmcnt<(P - 1) * DLOADS>();     // tile kt has landed (this wave's part)
                    lds_barrier();                                      // everyone's part; stage (kt-1) % NS is free
                    if (!ALL_DIRECT && kt + 1 < KT) load_regs(kt + 1);
                    // with one stage in flight the loads go out at once: each gets the whole step to land
                    if (DLOADS > 0) issue_direct_all(kt + P, (s + P) % C::NS);
                    compute(s, s);
                    if (!ALL_DIRECT && kt + 1 < KT) store_regs((s + 1) % C::NS, (s + 1) % C::NS);
                }
            }
        }
    } else {
        // Run-ahead scheme (NS >= 4): at the barrier of step j tiles <= j+1 are
        // complete, so the fragments of the next tile's first k-group are fetched
        // before that barrier and the MFMA stream never waits on LDS behind it.
        //   step j:  registers <- tile j+2 ; direct loads of tile j+NS-1 -> stage (j-1) % NS ;
        //            per k-group: fetch the next fragments, then MFMAs on the current ones ;
        //            registers -> stage (j+2) % NS ; wait for own direct loads of tile j+2 ; barrier
        static_assert(!C::PIPE || (C::NS >= 4 && C::KG % 2 == 0), "run-ahead needs 4 stages and an even number of k-groups");
        constexpr int PN = C::PIPE ? C::NS : 4;
        if (DLOADS > 0) {
#pragma unroll
            for (int s = 0; s < PN - 1; ++s) issue_direct_all(s, s);
        }
        if (!ALL_DIRECT) {
            load_regs(0);
            store_regs(0, 0);
            if (KT > 1) {
                load_regs(1);
                store_regs(1, 1);
            }
        }
        u32x4 af[2][C::MI], bf[2][C::NI];
        auto fetch = [&](int stage, int kg, int set) {
            // in the order the MFMAs of the next k-group consume them
            const char *sta = a_stage(stage), *stb = b_frag_base(stage);
#pragma unroll
            for (int i = 0; i < (C::MI > C::NI ? C::MI : C::NI); ++i) {
                if (i < C::NI) bf[set][i] = read_b(stb, i, kg);
                if (i < C::MI) af[set][i] = read_a(sta, i, kg);
            }
        };
        // tiles 0 and 1 complete; first fragments
        if (DLOADS > 0) wait_vmcnt<(PN - 3) * DLOADS>();
        lds_barrier();
        fetch(0, 0, 0);
        for (int j0 = 0; j0 < KT; j0 += PN) {
#pragma unroll
            for (int s = 0; s < PN; ++s) {
                const int j = j0 + s;
                if (j < KT) {
                    if (!ALL_DIRECT && j + 2 < KT) load_regs(j + 2);
                    static_for<C::KG>([&](auto kgc) {
                        constexpr int kg = decltype(kgc)::value;
                        // next fragments: same tile, or the first k-group of tile j+1 (past the
                        // end this reads a stage nobody uses; the values are dropped)
                        if (kg + 1 < C::KG) fetch(s, kg + 1, (kg + 1) & 1);
                        else fetch((s + 1) % PN, 0, 0);
                        // this k-group's share of the loads of tile j+NS-1
                        issue_a(j + PN - 1, (s + PN - 1) % PN, kgc, IC<C::KG>{});
                        issue_b(j + PN - 1, (s + PN - 1) % PN, kgc, IC<C::KG>{});
                        mfma_half(af[kg & 1], bf[kg & 1], IC<0>{});
                        mfma_half(af[kg & 1], bf[kg & 1], IC<1>{});
                        // Issue order inside the k-group: one LDS read or one global load after each
                        // MFMA.  A run of memory instructions leaves the matrix pipe idle when the
                        // other wave of the SIMD is in the same phase (or there is no other wave);
                        // spread out, they issue in the shadow of the MFMA before them.
                        constexpr int NMFMA = C::MI * C::NI * (C::DT == DT_F32 ? 4 : 1);
                        constexpr int NDS = C::MI + C::NI * (!C::B_TR ? 1 : (C::DT == DT_F32 ? 4 : 2));
                        constexpr int NVM = (LA + C::KG - 1 - kg) / C::KG + (LB + C::KG - 1 - kg) / C::KG;
                        constexpr int PER = C::DT == DT_F32 ? 4 : 1;       // MFMAs per slot
                        static_for<NMFMA / PER>([&](auto ic) {
                            constexpr int i = decltype(ic)::value;
                            __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);
                            if constexpr (i < NDS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                            else if constexpr (i - NDS < NVM) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                        });
                        __builtin_amdgcn_sched_barrier(0);
                    });
                    if (!ALL_DIRECT && j + 2 < KT) store_regs((s + 2) % PN, (s + 2) % PN);
                    if (DLOADS > 0) wait_vmcnt<(PN - 3) * DLOADS>();    // own loads of tile j+2 have landed
                    lds_barrier();                                      // tiles <= j+2 complete; stage j % NS is free
                }
            }
        }
    }

    if (DLOADS > 0) wait_vmcnt<0>();    // refetches past the end must land before this workgroup's LDS is given away

    // epilogue: the accumulators of slab mi (32 rows of the wave tile) go to LDS ...
    // (raw accumulators: alpha is applied on the way back, so that accumulators held in
    // AGPRs can go to LDS without passing through the ordinary registers)
    auto write_slab = [&](int mi, char *scr) {
        constexpr int SROW = C::WTN * 4 + 16;
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                f32x4 v = {acc[mi][ni][vq * 4 + 0], acc[mi][ni][vq * 4 + 1], acc[mi][ni][vq * 4 + 2], acc[mi][ni][vq * 4 + 3]};
                *(f32x4 *)(scr + r32 * SROW + (ni * 32 + vq * 8 + half * 4) * 4) = v;
            }
    };
    // ... or, for plain runs of the 16-bit kernels, already scaled and rounded
    auto write16 = [&](int mi, char *scr16) {
        constexpr int SROW16 = C::WTN * 2 + 16;
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                float x[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if constexpr (C::ACC_AGPR) {
                        // copied out of the accumulation registers here, group by group (left to
                        // itself the compiler copies all of them ahead of the branch and spills)
                        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x[j]) : "a"(acc[mi][ni][vq * 4 + j]));
                    } else {
                        x[j] = acc[mi][ni][vq * 4 + j];
                    }
                    x[j] *= p.alpha;
                }
                union { u32x2 u; _Float16 h[4]; __bf16 b[4]; } pk;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (C::DT == DT_F16) pk.h[j] = (_Float16)x[j];
                    else pk.b[j] = (__bf16)x[j];
                }
                const int grp = (ni * 8 + vq * 2 + half) ^ (r32 >> 4);
                *(u32x2 *)(scr16 + r32 * SROW16 + grp * 8) = pk.u;
            }
    };
    epilogue_slabs<C, C::MI>(p, lds, wave, lane, wm, wn, m0, n0, splitk_out(p, slice), write_slab, write16);
#ifdef PEAK_TRACE
    trace_store();
#endif
#endif
}

// ---------------------------------------------------------------------------
// Split-K, second step: C = alpha * (sum over slices, in slice order) + beta*C.
// One thread per 4 consecutive outputs of a row.
// ---------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const GemmArgs p)
{
    const int64_t quads_per_row = (p.N + 3) / 4;
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= p.M * quads_per_row) return;
    const int64_t m = q / quads_per_row, n = (q % quads_per_row) * 4;
    const int nvalid = p.N - n >= 4 ? 4 : (int)(p.N - n);
    const bool ws_vec = p.flags & GF_WS_VEC;
    float x[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int s = 0; s < p.split; ++s) {
        const float *w = p.ws + ((int64_t)s * p.M + m) * p.N + n;
        if (ws_vec && nvalid == 4) {
            const f32x4 t = *(const f32x4 *)w;
            x[0] += t[0]; x[1] += t[1]; x[2] += t[2]; x[3] += t[3];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (e < nvalid) x[e] += w[e];
        }
    }
    store4<DT>(p.C, m * p.ldc + n, x, p.alpha, p.beta, p.flags & GF_C_VEC, nvalid, p.hook, m, n);
}

// Hybrid stream-K, second step: the tiles that were cut along K are summed over their slices,
// in slice order, and stored like any other tile.  One thread per 4 consecutive outputs of a
// tile row; blockIdx.y is the tile's position among the cut tiles.
template <int DT, int BM, int BN>
__global__ __launch_bounds__(256) void streamk_reduce_kernel(const GemmArgs p)
{
    const int r = blockIdx.y;
    const int q = blockIdx.x * 256 + threadIdx.x;                 // 4-column group within the tile
    if (q >= BM * (BN / 4)) return;
    int tm, tn;
    tile_of_block(p.tiles_m * p.tiles_n - p.sk_tiles + r, p.tiles_m, p.tiles_n, p.group_m, tm, tn);
    const int row = q / (BN / 4), col = (q % (BN / 4)) * 4;
    const int64_t m = (int64_t)tm * BM + row, n = (int64_t)tn * BN + col;
    if (m >= p.M || n >= p.N) return;
    const int nvalid = p.N - n >= 4 ? 4 : (int)(p.N - n);
    float x[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int s = 0; s < p.split; ++s) {
        const f32x4 t = *(const f32x4 *)(p.ws + ((int64_t)s * p.sk_tiles + r) * (BM * BN) + row * BN + col);
        x[0] += t[0]; x[1] += t[1]; x[2] += t[2]; x[3] += t[3];
    }
    if (p.flags & GF_C_F32) store4<DT_F32>(p.C, m * p.ldc + n, x, p.alpha, p.beta, p.flags & GF_C_VEC, nvalid, p.hook, m, n);
    else store4<DT>(p.C, m * p.ldc + n, x, p.alpha, p.beta, p.flags & GF_C_VEC, nvalid, p.hook, m, n);
}

// C = hook(beta * C) (alpha == 0 or K == 0).  beta == 0 writes without reading.
template <int DT>
__global__ __launch_bounds__(256) void scale_c_kernel(const GemmArgs p)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= p.M * p.N) return;
    const int64_t m = e / p.N, n = e % p.N;
    float o = 0.0f;
    if (p.beta != 0.0f) o = p.beta * elem_to_float<DT>(p.C, m * p.ldc + n);
    if (hook_active(p.hook)) {
        float o1[1] = {o}, b4[4];
        hook_bias4(p.hook, m, n, 1, b4);
        const float b1[1] = {b4[0]};
        hook_apply(p.hook.act, p.hook.bias_kind != BIAS_NONE, o1, b1);
        o = o1[0];
    }
    float_to_elem<DT>(p.C, m * p.ldc + n, o);
}

}  // namespace peak
