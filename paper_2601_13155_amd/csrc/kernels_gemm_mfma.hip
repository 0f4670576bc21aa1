// bf16 matrix-core GEMM for gfx950:  C[M,N] = A[M,K] * B[N,K]^T, fp32 accumulation.
//
// Serves the dense contractions of the SPTS layer: K / Q / V / O projections, the gathered SwiGLU
// FFN and the low-rank proxy.  Both operands are K-contiguous, so MFMA fragments are plain 16-byte
// LDS reads with no transposition.
//
//  * 256x256 output tile per workgroup, 8 wavefronts (4x2), each owning 64x128 = 2x4 MFMA
//    32x32x16 blocks: 128 fp32 accumulators per lane, 8 MFMAs per 6 fragment reads, two wavefronts
//    per SIMD so that one wavefront's LDS reads, waits and barriers hide behind the other's MFMAs.
//  * K is consumed in slabs of 64 (32 when K is not a multiple of 64, or when a second A operand
//    is staged).  Slabs travel global memory -> LDS directly (global_load_lds_dwordx4: no VGPR
//    staging, no ds_write instructions) into a ring of 2 LDS stages of 64 KB (4 stages of 32 KB for
//    slabs of 32, 3 with a second A operand): the loads of the next slab(s) are in flight while the
//    current one is multiplied.  The wavefront counts its own outstanding slab loads with
//    s_waitcnt vmcnt(n) and one workgroup barrier per slab publishes a landed slab and frees the
//    stage consumed before it.
//  * The address of a load is a wavefront-uniform base in SGPRs, advanced along K by scalar adds, plus
//    a 32-bit per-lane offset fixed for the whole tile, and the steady state is unrolled over the ring
//    so that LDS stage offsets are immediates: the loop holds no vector address arithmetic (vector
//    instructions barely overlap with MFMAs on this chip: interleaved 1:1 they take 0.75 of the sum).
//  * A direct-to-LDS load puts lane i's 16 bytes at base + 16*i, so the XOR swizzle that makes the
//    16-lane b128 fragment reads bank-conflict free is applied on the global side: lane i fetches
//    the chunk that belongs at position i.
//  * Fragment reads of the next k-step are issued between the MFMAs of the current one
//    (sched_group_barrier pins the interleaving); the barrier sits a few MFMAs into the second
//    k-step so that the matrix pipe stays fed while wavefronts meet.
//  * Slab-major operands.  With row-major operands and slabs of 32 a load instruction takes 64 bytes of each of 16
//    rows, so every 128-byte line is requested twice (by the loads of two consecutive slabs) and the kernel is bound
//    by L2 requests (measured: whole-line loads of the same data are 8-9 % faster, per operand).  An operand stored
//    [K/32][rows][32] (64 bytes per row and slab, neighbouring rows adjacent) makes the same 16 rows 1 KB of whole
//    lines; only the addresses differ (row pitch 64 bytes, slab pitch rows * 64 bytes), the LDS image and the order
//    of the products do not.  B: slab-major weight copies (b_slab); A: activations that another kernel of this library
//    wrote slab-major (a_slab; the SiLU and store epilogues and the split-K finish write such a C on request, c_slab).
//    Calls with slab operands run the 32-wide, 4-stage instantiation whatever K is.
//  * Rows of A may be gathered through an index list (the active-token gather of Eq. (skip) is
//    folded into the A loads: a row is 2*K contiguous bytes, so nothing is lost in coalescing),
//    rows of C may be scattered through one (the residual update X[T] += ...).
//  * The MFMA is issued as D^T = B * A^T so that a lane ends up with 4 consecutive output columns
//    of one row: lane-local rotary / SiLU-mul pairing, in-lane row sums, 8-byte packed pieces.
//  * The finished bf16 tile is staged through LDS (the operand ring is free by then) and leaves in
//    whole rows, 16 bytes per lane: stores straight from the fragment layout reach memory as 16-byte
//    pieces of 32 different rows per instruction, which cost a short-K GEMM a quarter of its time.
//  * Workgroup ids are remapped so that each of the 8 XCDs (own L2 each) walks a contiguous range
//    of tiles in groups of 4 row panels: concurrently running tiles share A and B panels in L2.
//  * One workgroup fits a CU, so tiles run in rounds of 256.  When the last round is partly filled
//    its tiles are split over K (tail split-K): several workgroups each take a share of K, write
//    fp32 partial tiles, and a small second kernel sums them and applies the epilogue.  A GEMM with
//    fewer than 256 tiles is the special case without whole rounds.
//  * The plain-store epilogue can take its B rows from two matrices (columns [0, N/2) from B0,
//    [N/2, N) from B1): the two down-projections of the proxy run as one launch.
//
// Epilogues: plain store (+ optional transposed copy for V), rotary embedding (pairs (j, j+d/2) sit
// in the same lane because an N block pair is d/2 apart), SiLU(gate)*up with gate and up columns
// interleaved per wavefront, residual add into scattered rows, per-row partial sums of squares.
#include "spts_internal.h"

namespace spts {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 256, BN = 256;
#ifndef SPTS_GEMM_UNROLL_RING
#define SPTS_GEMM_UNROLL_RING 1
#endif

// K slab geometry.  A tile row holds BK bf16 = CPR 16-byte chunks; chunk c of row `row` is stored at
// chunk position c ^ ((row / RP) % CPR) (RP = rows per 256 bytes), so the 16 lanes of a b128
// fragment read (16 consecutive rows, same chunk) cover all 64 LDS banks exactly once.
template <int BK> struct Slab {
    static constexpr int ROW_BYTES = BK * 2;
    static constexpr int CPR = BK / 8;
    static constexpr int RP = 256 / ROW_BYTES;
    static constexpr int TILE_BYTES = 256 * ROW_BYTES;
    static constexpr int ROWS_PER_LOAD = 64 / CPR;   // tile rows moved by one direct-to-LDS load
    __device__ static inline int swz(int row) { return (row / RP) % CPR; }
    __device__ static inline int off(int row, int c) { return row * ROW_BYTES + ((c ^ swz(row)) << 4); }
};

__device__ inline uint32_t pack_bf16x2(float a, float b) { return cvt_pk_bf16(a, b); }
// SiLU with the hardware exponential and reciprocal (about 1 ulp each in fp32; the result is rounded to
// bf16): an IEEE division would cost ten more instructions per element, which shows in the short-K
// proxy GEMM whose epilogue is a quarter of the tile time
__device__ inline float silu_f(float g) {
    return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
}

// tile number -> (row tile, column tile): grouped raster, GM row tiles per group, rows fastest inside
// a group, so that workgroups running together share A and B tiles in L2
__device__ __forceinline__ void tile_of(int id, int nM, int nN, int& tm, int& tn) {
    constexpr int GM = 4;
    const int group = id / (GM * nN);
    const int first_m = group * GM;
    const int gsz = (nM - first_m) < GM ? (nM - first_m) : GM;
    const int in_g = id % (GM * nN);
    tm = first_m + in_g % gsz;
    tn = in_g / gsz;
}

// NW wavefronts per workgroup: 4 (2x2 wavefronts of 128x128, one per SIMD) or 8 (4x2 wavefronts of
// 64x128, two per SIMD: a wavefront's memory instructions, waits and barriers hide behind the other's
// MFMAs at the price of 50 % more LDS fragment traffic).
template <int EPI, int BK, bool DUAL_A, int NW>
__global__ void __launch_bounds__(NW * 64) gemm_mfma_kernel(GemmArgs a, int nM, int nN, int nfull, int nunits) {
    using S = Slab<BK>;
    constexpr int MI = 16 / NW;                   // 32-row blocks per wavefront (4 or 2)
    constexpr int WROWS = 32 * MI;                // output rows per wavefront
    constexpr int LROWS = 256 / NW;               // operand tile rows each wavefront loads
    constexpr bool DUAL = (EPI == EPI_SILU_MUL);
    constexpr bool SEG = (EPI == EPI_ROPE_STORE);   // two products side by side: rotary columns, then stored columns
    constexpr bool CAN_SPLIT = (EPI == EPI_STORE || EPI == EPI_RESIDUAL || EPI == EPI_ROPE || SEG);
    constexpr int TILE_BYTES = S::TILE_BYTES;
    constexpr int NOPS = DUAL_A ? 3 : 2;          // operand tiles per stage (A, B[, A1])
    constexpr int NST = BK == 64 ? 2 : (DUAL_A ? 3 : 4);   // LDS ring stages
    constexpr int STAGE = TILE_BYTES * NOPS;
    constexpr int LPO = LROWS / S::ROWS_PER_LOAD; // loads per wavefront per operand tile
    constexpr int PER = LPO * NOPS;               // direct-to-LDS loads per wavefront per slab
    constexpr int KSTEPS = BK / 16;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // ---- work unit.  Workgroup b runs on XCD b % 8 as that XCD's (b / 8)-th workgroup.  Every XCD
    //      takes a contiguous range of whole tiles first, then a contiguous range of split units
    //      (a split unit = one K share of one of the tiles behind the first nfull), so that all
    //      XCDs run out of whole tiles at the same time.
    const int xcd = (int)(blockIdx.x % 8), pos = (int)(blockIdx.x / 8);
    const int pf = (nfull + 7) / 8;
    int id, split = 0, ksplit = 1;
    if (pos < pf) {
        id = xcd * pf + pos;
        if (id >= nfull) return;
    } else {
        if (!CAN_SPLIT) return;
        const int u = xcd * ((nunits + 7) / 8) + (pos - pf);
        if (u >= nunits) return;
        ksplit = a.ksplit;
        id = nfull + u / ksplit;
        split = u % ksplit;
    }
    const bool partial = CAN_SPLIT && ksplit > 1;
    int tm, tn;
    tile_of(id, nM, nN, tm, tn);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int64_t row0 = (int64_t)tm * BM;
    constexpr int OUT_COLS = DUAL ? 128 : 256;   // output columns covered by one tile
    const int col0 = tn * OUT_COLS;

    // ---- direct-to-LDS assignment: wavefront w moves tile rows [64w, 64w+64) of every operand, 16
    //      (BK=32) or 8 (BK=64) rows = 1 KB per load; lane -> (row, LDS chunk position), and fetches
    //      the global chunk that the swizzle maps to that LDS position.
    // A load's address is a wavefront-uniform base (SGPR pair, advanced along K with scalar adds) plus a
    // 32-bit per-lane byte offset that never changes: no vector instructions for addresses in the loop.
    // Bases: A rows from row0 on (or the whole gather source when rows come through an index list, whose
    // byte size must then fit 32 bits); the B rows this wavefront moves.
    // Slab-major operands (32-wide slabs): a row of a slab is 64 bytes and consecutive rows are adjacent, so the row
    // pitch is 64 bytes and one slab further on is rows * 64 bytes.
    const bool a_slab = BK == 32 && a.a_slab, b_slab = BK == 32 && a.b_slab;
    const int64_t a_pitch = a_slab ? 64 : a.lda * 2, b_pitch = b_slab ? 64 : a.ldb * 2;      // bytes between rows
    const bool second = SEG && col0 >= a.n_split;   // this tile belongs to the second product (B1 -> C2)
    const int64_t a_kstep = a_slab ? a.M * 64 : BK * 2;                                              // bytes per slab
    const int64_t b_kstep = b_slab ? (second ? a.b_rows1 : a.b_rows) * 64 : BK * 2;
    uint32_t oa[LPO], ob[LPO];
    const char* abase = (const char*)a.A + (a.a_idx ? (int64_t)0 : row0 * a_pitch);
    const char* a1base = DUAL_A ? (const char*)a.A1 + (a.a_idx ? (int64_t)0 : row0 * a_pitch) : abase;
    const char* bbase;
    {
        const int rw = wave * LROWS;   // first B tile row of this wavefront
        if (DUAL) bbase = rw < 128 ? (const char*)a.B0 + (int64_t)(col0 + rw) * b_pitch
                                   : (const char*)a.B1 + (int64_t)(col0 + rw - 128) * b_pitch;
        else if (SEG) bbase = second ? (const char*)a.B1 + (int64_t)(col0 - a.n_split + rw) * b_pitch
                                     : (const char*)a.B0 + (int64_t)(col0 + rw) * b_pitch;
        else if (a.B1 && col0 >= a.N / 2) bbase = (const char*)a.B1 + (int64_t)(col0 - a.N / 2 + rw) * b_pitch;
        else bbase = (const char*)a.B0 + (int64_t)(col0 + rw) * b_pitch;
    }
#pragma unroll
    for (int q = 0; q < LPO; ++q) {
        const int rl = q * S::ROWS_PER_LOAD + lane / S::CPR;   // row inside the wavefront's share
        const int r = wave * LROWS + rl;
        const int c = (lane % S::CPR) ^ S::swz(r);
        int64_t grow = row0 + r;
        if (grow >= a.M) grow = a.M - 1;  // clamp: duplicates of the last row are never stored
        const int64_t srow = a.a_idx ? (int64_t)a.a_idx[grow] : grow - row0;
        oa[q] = (uint32_t)(srow * a_pitch + c * 16);
        ob[q] = (uint32_t)((int64_t)rl * b_pitch + c * 16);
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const uint32_t lds_w = lds0 + wave * (LROWS * S::ROW_BYTES);   // this wavefront's rows inside an operand tile
    // load number u (0 .. PER-1) of slab kt_: operand u % NOPS, 16-row group u / NOPS
#define SPTS_DMA_ONE(kt_, u)                                                                   \
    {                                                                                          \
        const uint32_t sb_ = lds_w + ((kt_) % NST) * STAGE + ((u) / NOPS) * 1024;              \
        const int64_t ks_ = kbeg + (kt_);                                                      \
        if ((u) % NOPS == 0) dma16s(oa[(u) / NOPS], abase + ks_ * a_kstep, sb_);               \
        else if ((u) % NOPS == 1) dma16s(ob[(u) / NOPS], bbase + ks_ * b_kstep, sb_ + TILE_BYTES); \
        else dma16s(oa[(u) / NOPS], a1base + ks_ * a_kstep, sb_ + 2 * TILE_BYTES);             \
    }
#define SPTS_DMA_SLAB(kt_)                                                                     \
    { _Pragma("unroll") for (int u_ = 0; u_ < PER; ++u_) SPTS_DMA_ONE(kt_, u_) }

    f32x16 acc[MI][4];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // B tile row of this wavefront's N block j
    auto brow = [&](int j) { return DUAL ? (j >> 1) * 128 + wn * 64 + (j & 1) * 32 : wn * 128 + j * 32; };

    bf16x8 af[2][MI], bfr[2][4], af1[2][DUAL_A ? MI : 1];
#define SPTS_LOAD_FRAGS(buf, stage, ks)                                                                      \
    {                                                                                                        \
        const char* sA_ = smem + (stage) * STAGE;                                                            \
        const char* sB_ = sA_ + TILE_BYTES;                                                                  \
        const int c_ = (ks) * 2 + lh;                                                                        \
        _Pragma("unroll") for (int i = 0; i < MI; ++i) {                                                     \
            af[buf][i] = *reinterpret_cast<const bf16x8*>(sA_ + S::off(wm * WROWS + i * 32 + l32, c_));    \
            if (DUAL_A)                                                                                      \
                af1[buf][i] = *reinterpret_cast<const bf16x8*>(sB_ + TILE_BYTES + S::off(wm * WROWS + i * 32 + l32, c_)); \
        }                                                                                                    \
        _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                        \
            bfr[buf][j] = *reinterpret_cast<const bf16x8*>(sB_ + S::off(brow(j) + l32, c_));               \
    }
#define SPTS_MFMA(buf, i, j)                                                                                 \
    {                                                                                                        \
        if (DUAL_A && (j) >= 2)                                                                              \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[buf][j], af1[buf][i], acc[i][j], 0, 0, 0); \
        else                                                                                                 \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[buf][j], af[buf][i], acc[i][j], 0, 0, 0);  \
    }
    constexpr int NREADS = (DUAL_A ? 2 * MI : MI) + 4;   // fragment reads per k-step
    constexpr int NM = 4 * MI;                            // MFMAs per k-step
    constexpr int HS = NM / 2;                            // MFMA slots per half k-step

    // K slabs of this workgroup: all of them, or the split's share (the first nk_all % ksplit splits
    // take one slab more)
    const int nk_all = a.K / BK;
    const int nk = nk_all / ksplit + (split < nk_all % ksplit ? 1 : 0);
    const int kbeg = split * (nk_all / ksplit) + (split < nk_all % ksplit ? split : nk_all % ksplit);
    // ---- prologue: slabs 0 .. NST-2 are put in flight, slab 0 must have landed
    {
        const int npre = nk < NST - 1 ? nk : NST - 1;
        for (int t = 0; t < npre; ++t) SPTS_DMA_SLAB(t)
        if (npre == NST - 1) { SPTS_WAIT_VMCNT((NST - 2) * PER); } else { SPTS_WAIT_VMCNT(0); }   // slab 0 landed
    }
    __syncthreads();
    SPTS_LOAD_FRAGS(0, 0, 0)

    // One K slab = KSTEPS k-steps of 16 MFMAs per wavefront.  Every memory instruction sits in the
    // shadow of an MFMA (an MFMA occupies the matrix pipe for 32 cycles while the wavefront may
    // issue other work):
    //   k-step s < KSTEPS-1: MFMA 1-8 are each followed by one fragment read of k-step s+1,
    //                        MFMA 9-16 by one direct-to-LDS load of slab kt+NST-1 (ISSUE);
    //   last k-step: 4 MFMAs, then wait for this wavefront's share of slab kt+1 and meet the
    //                workgroup (slab kt+1 is published, stage kt%NST is free for the next iteration),
    //                then 12 MFMAs, the first 8 each followed by a fragment read of slab kt+1.
    // ISSUE / NEXT are literal constants at every expansion.
    // HS MFMA slots, one fragment read after each (two after the first NREADS-HS of them)
#define SPTS_INTERLEAVE_READS                                                                                \
    _Pragma("unroll") for (int g_ = 0; g_ < NREADS - HS; ++g_) {                                             \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                   \
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                                                   \
    }                                                                                                        \
    _Pragma("unroll") for (int g_ = NREADS - HS; g_ < HS; ++g_) {                                            \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                   \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                   \
    }
#define SPTS_SLAB(kt_, ISSUE, NEXT, WAITN)                                                                   \
    {                                                                                                        \
        const int st_ = (kt_) % NST;                                                                         \
        _Pragma("unroll") for (int ks = 0; ks + 1 < KSTEPS; ++ks) {                                          \
            const int fb = ks & 1;                                                                           \
            SPTS_LOAD_FRAGS(fb ^ 1, st_, ks + 1)                                                             \
            _Pragma("unroll") for (int m_ = 0; m_ < HS; ++m_) SPTS_MFMA(fb, m_ / 4, m_ % 4)                  \
            SPTS_INTERLEAVE_READS                                                                            \
            __builtin_amdgcn_sched_barrier(0);                                                               \
            _Pragma("unroll") for (int m_ = HS; m_ < NM; ++m_) {                                             \
                SPTS_MFMA(fb, m_ / 4, m_ % 4)                                                                \
                if (ISSUE) {                                                                                 \
                    const int u_ = ks * HS + m_ - HS;                                                        \
                    __builtin_amdgcn_sched_barrier(0);                                                       \
                    if (u_ < PER) SPTS_DMA_ONE((kt_) + NST - 1, (u_ < PER ? u_ : 0))                         \
                    if (KSTEPS == 2 && u_ + HS < PER) SPTS_DMA_ONE((kt_) + NST - 1, (u_ + HS < PER ? u_ + HS : 0)) \
                    __builtin_amdgcn_sched_barrier(0);                                                       \
                }                                                                                            \
            }                                                                                                \
        }                                                                                                    \
        {                                                                                                    \
            constexpr int fb = (KSTEPS - 1) & 1;                                                             \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) SPTS_MFMA(fb, 0, j)                                \
            if (NEXT) { SPTS_WAIT_VMCNT(WAITN); }                                                            \
            __syncthreads();                                                                                 \
            if (NEXT) { SPTS_LOAD_FRAGS(fb ^ 1, ((kt_) + 1) % NST, 0) }                                      \
            _Pragma("unroll") for (int i = 1; i < MI; ++i)                                                   \
                _Pragma("unroll") for (int j = 0; j < 4; ++j) SPTS_MFMA(fb, i, j)                            \
            if (NEXT) {                                                                                      \
                _Pragma("unroll") for (int g_ = 0; g_ < NM - 4; ++g_) {                                      \
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                       \
                    __builtin_amdgcn_sched_group_barrier(0x100, (NREADS + NM - 5) / (NM - 4), 0);            \
                }                                                                                            \
            }                                                                                                \
            __builtin_amdgcn_sched_barrier(0);                                                               \
        }                                                                                                    \
    }

    int kt = 0;
    // steady state: slab kt+NST-1 exists; after its loads are issued the slabs behind kt+1 in flight
    // are kt+2 .. kt+NST-1.  First in groups of NST slabs, where the ring stage of every slab is a
    // compile-time constant and the LDS addresses of the fragment reads need no arithmetic in the loop.
    if (SPTS_GEMM_UNROLL_RING && (NST & (NST - 1)) == 0) {
        int kb = 0;
        for (; kb * NST + 2 * NST - 2 < nk; ++kb) {
            _Pragma("unroll") for (int u = 0; u < NST; ++u) SPTS_SLAB(kb * NST + u, true, true, (NST - 2) * PER)
        }
        kt = kb * NST;
    }
    for (; kt + NST - 1 < nk; ++kt) SPTS_SLAB(kt, true, true, (NST - 2) * PER)
    // drain: nothing left to issue; wait for everything that is still in flight
    for (; kt + 1 < nk; ++kt) SPTS_SLAB(kt, false, true, 0)
    SPTS_SLAB(kt, false, false, 0)

    // ---- epilogue.  acc[i][j][r]: row = row0 + wm*WROWS + i*32 + l32,
    //      column (inside N block j) = 8*(r/4) + 4*lh + r%4  -> 4 consecutive columns per r/4.
    bf16_t* Cb = (bf16_t*)a.C;
    if (partial) {
        // raw fp32 accumulators in fragment order: every store instruction of a wavefront writes 1 KB
        float* P = a.part32 + ((int64_t)(id - nfull) * ksplit + split) * (BM * 256);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    *reinterpret_cast<f32x4*>(P + ((((wave * MI + i) * 4 + j) * 4 + q) * 64 + lane) * 4) = v;
                }
        return;
    }
    if (EPI == EPI_SUMSQ) {
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) s += acc[i][j][r] * acc[i][j][r];
            s += __shfl_xor(s, 32);
            int64_t grow = row0 + wm * WROWS + i * 32 + l32;
            if (lh == 0 && grow < a.M) a.part[grow * a.part_ld + tn * 2 + wn] = s;
        }
        return;
    }
    // The finished values are packed to bf16 and staged through LDS (the operand ring is free now) so that
    // the tile leaves in whole rows: a lane owns 4 consecutive columns of 16 different rows per N block,
    // and stores straight from the fragment layout would reach memory as 16-byte pieces of 32 rows per
    // instruction.  Staged row tr keeps 16-byte chunk c at chunk position c ^ (tr % NCH): the 32 lanes of a
    // fragment write (32 rows, same chunk) and the row-wise reads are both spread over all banks.
    constexpr int NCH = OUT_COLS / 8;            // 16-byte chunks per staged row
    constexpr int ROWB = OUT_COLS * 2;           // bytes per staged row
    const int colshift = second ? a.n_split : 0; // the second product's outputs count their columns from n_split
    if (second) Cb = (bf16_t*)a.C2;
    const int64_t ldo = second ? a.ldc2 : a.ldc;
    auto stage = [&](int tr, int tc, uint2 o) {
        *reinterpret_cast<uint2*>(smem + tr * ROWB + ((((tc >> 3) ^ tr) & (NCH - 1)) << 4) + ((tc & 4) << 1)) = o;
    };
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int tr = wm * WROWS + i * 32 + l32;
        const int64_t grow = row0 + tr;
        const bool rok = grow < a.M;
        const int64_t growc = rok ? grow : a.M - 1;
        const int64_t crow = a.c_idx ? (int64_t)a.c_idx[growc] : growc;
        if (EPI == EPI_STORE || (SEG && second)) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int cb = col0 - colshift + wn * 128 + j * 32 + 4 * lh;   // column of this product's output
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 o;
                    o.x = pack_bf16x2(acc[i][j][4 * q], acc[i][j][4 * q + 1]);
                    o.y = pack_bf16x2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                    stage(tr, cb - (col0 - colshift) + 8 * q, o);
                    if (a.Ct && grow < a.ldct) {
                        bf16_t* ct = (bf16_t*)a.Ct;
                        const uint16_t e[4] = {(uint16_t)(o.x & 0xffff), (uint16_t)(o.x >> 16), (uint16_t)(o.y & 0xffff), (uint16_t)(o.y >> 16)};
#pragma unroll
                        for (int t = 0; t < 4; ++t) ct[(int64_t)(cb + 8 * q + t) * a.ldct + vt_key_slot(grow)].v = e[t];
                    }
                }
            }
        } else if (EPI == EPI_RESIDUAL) {
            // the old values are read in the fragment layout (rows past M read the last row; they are not
            // stored): one rounding of old + acc, as without the staging
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int cb = col0 + wn * 128 + j * 32 + 4 * lh;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint2 old = *reinterpret_cast<const uint2*>(Cb + crow * a.ldc + cb + 8 * q);
                    float x0 = __uint_as_float(old.x << 16), x1 = __uint_as_float(old.x & 0xffff0000u);
                    float x2 = __uint_as_float(old.y << 16), x3 = __uint_as_float(old.y & 0xffff0000u);
                    uint2 o;
                    o.x = pack_bf16x2(x0 + acc[i][j][4 * q], x1 + acc[i][j][4 * q + 1]);
                    o.y = pack_bf16x2(x2 + acc[i][j][4 * q + 2], x3 + acc[i][j][4 * q + 3]);
                    stage(tr, cb - col0 + 8 * q, o);
                }
            }
        } else if (EPI == EPI_SILU_MUL) {
            {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int cb = col0 + wn * 64 + j * 32 + 4 * lh;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float h0 = silu_f(acc[i][j][4 * q]) * acc[i][j + 2][4 * q];
                        float h1 = silu_f(acc[i][j][4 * q + 1]) * acc[i][j + 2][4 * q + 1];
                        float h2 = silu_f(acc[i][j][4 * q + 2]) * acc[i][j + 2][4 * q + 2];
                        float h3 = silu_f(acc[i][j][4 * q + 3]) * acc[i][j + 2][4 * q + 3];
                        uint2 o; o.x = pack_bf16x2(h0, h1); o.y = pack_bf16x2(h2, h3);
                        stage(tr, cb - col0 + 8 * q, o);
                    }
                }
            }
        } else if (EPI == EPI_ROPE || SEG) {
            {
                const int64_t trow = a.rope_idx ? (int64_t)a.rope_idx[growc] : growc;
                const int half = a.head_dim >> 1;
                const float2* tab = a.rope + trow * half;
                const float rs = a.rope_scale != 0.f ? a.rope_scale : 1.f;
                if (half == 64) {
                    // wavefront = one head of 128 columns: blocks (0,2) and (1,3) are d/2 apart
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int jj = j * 32 + 4 * lh;
                        const int cb = col0 + wn * 128 + jj;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            float lo[4], hi[4];
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                float2 cs = tab[jj + 8 * q + t];
                                float x1 = acc[i][j][4 * q + t], x2 = acc[i][j + 2][4 * q + t];
                                lo[t] = (x1 * cs.x - x2 * cs.y) * rs;
                                hi[t] = (x2 * cs.x + x1 * cs.y) * rs;
                            }
                            uint2 o1, o2;
                            o1.x = pack_bf16x2(lo[0], lo[1]); o1.y = pack_bf16x2(lo[2], lo[3]);
                            o2.x = pack_bf16x2(hi[0], hi[1]); o2.y = pack_bf16x2(hi[2], hi[3]);
                            stage(tr, cb - col0 + 8 * q, o1);
                            stage(tr, cb - col0 + 64 + 8 * q, o2);
                        }
                    }
                } else {
                    // d = 64: two heads per wavefront; blocks (0,1) and (2,3) are d/2 = 32 apart
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        const int jj = 4 * lh;
                        const int cb = col0 + wn * 128 + hh * 64 + jj;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            float lo[4], hi[4];
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                float2 cs = tab[jj + 8 * q + t];
                                float x1 = acc[i][2 * hh][4 * q + t], x2 = acc[i][2 * hh + 1][4 * q + t];
                                lo[t] = (x1 * cs.x - x2 * cs.y) * rs;
                                hi[t] = (x2 * cs.x + x1 * cs.y) * rs;
                            }
                            uint2 o1, o2;
                            o1.x = pack_bf16x2(lo[0], lo[1]); o1.y = pack_bf16x2(lo[2], lo[3]);
                            o2.x = pack_bf16x2(hi[0], hi[1]); o2.y = pack_bf16x2(hi[2], hi[3]);
                            stage(tr, cb - col0 + 8 * q, o1);
                            stage(tr, cb - col0 + 32 + 8 * q, o2);
                        }
                    }
                }
            }
        }
    }
    // ---- the staged tile leaves row by row: NCH consecutive lanes write one row's OUT_COLS columns as
    //      16-byte pieces (whole 128-byte lines), rows through the scatter list when there is one
    __syncthreads();
    if ((EPI == EPI_SILU_MUL || EPI == EPI_STORE) && a.c_slab) {
        // slab-major output: slab sl of the tile is 256 rows x 64 bytes, contiguous over the rows; 4 lanes per row
        constexpr int RPS = NW * 64 / 4;         // rows per pass
        const int oc4 = tid & 3, r_in = tid >> 2;
#pragma unroll
        for (int sl = 0; sl < OUT_COLS / 32; ++sl)
#pragma unroll
            for (int p = 0; p < 256 / RPS; ++p) {
                const int tr = p * RPS + r_in;
                const int64_t grow = row0 + tr;
                if (grow < a.M) {
                    const u32x4 v = *reinterpret_cast<const u32x4*>(smem + tr * ROWB + ((((sl * 4 + oc4) ^ tr) & (NCH - 1)) << 4));
                    *reinterpret_cast<u32x4*>(Cb + (((int64_t)(col0 >> 5) + sl) * a.M + grow) * 32 + oc4 * 8) = v;
                }
            }
        return;
    }
    constexpr int RPP = NW * 64 / NCH;           // rows per pass of the workgroup
    const int oc = tid % NCH, orow = tid / NCH;
#pragma unroll 4
    for (int p = 0; p < 256 / RPP; ++p) {
        const int tr = p * RPP + orow;
        const int64_t grow = row0 + tr;
        if (grow < a.M) {
            const int64_t crow = a.c_idx ? (int64_t)a.c_idx[grow] : grow;
            const u32x4 v = *reinterpret_cast<const u32x4*>(smem + tr * ROWB + (((oc ^ tr) & (NCH - 1)) << 4));
            *reinterpret_cast<u32x4*>(Cb + crow * ldo + (col0 - colshift) + oc * 8) = v;
        }
    }
}

int gemm_sumsq_blocks(int32_t N, bool mfma) { return mfma ? (N + 127) / 128 : (N + 63) / 64; }

static inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool gemm_mfma_supported(const GemmArgs& a) {
    if (a.c_is_f32) return false;
    const bool dual = a.epi == EPI_SILU_MUL;
    const int ncols = dual ? 128 : 256;
    if (a.M <= 0 || a.N <= 0 || a.N % ncols != 0) return false;
    if (a.K < 32 || a.K % 32 != 0) return false;
    if (a.lda % 8 != 0 || a.ldb % 8 != 0) return false;
    // slab-major operands: served by the 32-wide-slab instantiations; A not gathered
    const bool seg = a.epi == EPI_ROPE_STORE;
    if ((a.a_slab || a.b_slab) && a.epi != EPI_SILU_MUL && a.epi != EPI_RESIDUAL && a.epi != EPI_STORE && a.epi != EPI_ROPE && !seg) return false;
    if (seg) {
        if (a.n_split <= 0 || a.n_split >= a.N || a.n_split % 256 != 0 || a.c_idx || a.c_slab) return false;
        if (!a.B1 || !al16(a.B1) || !a.C2 || !al16(a.C2) || a.ldc2 % 8 != 0) return false;
        if (a.b_slab && (a.b_rows < a.n_split || a.b_rows1 < a.N - a.n_split)) return false;
    }
    if (a.a_slab && a.a_idx) return false;
    if (a.b_slab && !seg && a.b_rows < (a.epi == EPI_STORE && a.B1 ? a.N / 2 : a.N)) return false;   // rows of each B matrix
    if (a.c_slab && ((a.epi != EPI_SILU_MUL && a.epi != EPI_STORE) || a.c_idx || a.Ct)) return false;
    if (!al16(a.A) || !al16(a.B0) || (a.A1 && !al16(a.A1)) || (dual && !al16(a.B1))) return false;
    if (a.epi != EPI_SUMSQ) {
        if (a.ldc % 8 != 0 || !al16(a.C)) return false;
    }
    if ((a.epi == EPI_ROPE || seg) && a.head_dim != 128 && a.head_dim != 64) return false;
    if (a.Ct && a.epi != EPI_STORE && !seg) return false;
    if (a.epi == EPI_STORE && a.B1 && (a.N % 512 != 0 || !al16(a.B1))) return false;
    if (a.ksplit > 1) {
        if (!a.part32 || !al16(a.part32) || (a.epi != EPI_STORE && a.epi != EPI_RESIDUAL && a.epi != EPI_ROPE && !seg)) return false;
        if (a.K / 64 < a.ksplit || a.nfull < 0 || a.nfull > (a.M + BM - 1) / BM * (a.N / 256)) return false;
    }
    if (a.M > (int64_t)1 << 30) return false;
    // 32-bit byte offsets from the load bases: the gather source as a whole, 256 rows of A or B otherwise
    if (a.a_idx && (a.a_rows <= 0 || a.a_rows * a.lda * 2 >= ((int64_t)1 << 32))) return false;
    if (256 * a.lda * 2 >= ((int64_t)1 << 32) || 256 * a.ldb * 2 >= ((int64_t)1 << 32)) return false;
    return true;
}

template <int EPI, int BK, bool DUAL_A, int NW>
static hipError_t launch_t(const GemmArgs& a, hipStream_t s) {
    const int ncols = EPI == EPI_SILU_MUL ? 128 : 256;
    const int nM = (int)((a.M + BM - 1) / BM), nN = a.N / ncols;
    const int tiles = nM * nN;
    const bool split = a.ksplit > 1;
    const int nfull = split ? a.nfull : tiles;
    const int nunits = split ? (tiles - nfull) * a.ksplit : 0;
    const int grid = 8 * ((nfull + 7) / 8 + (nunits + 7) / 8);
    const size_t lds = (size_t)Slab<BK>::TILE_BYTES * (DUAL_A ? 3 : 2) * (BK == 64 ? 2 : (DUAL_A ? 3 : 4));
    {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&gemm_mfma_kernel<EPI, BK, DUAL_A, NW>), (int)lds);
        if (e != hipSuccess) return e;
    }
    gemm_mfma_kernel<EPI, BK, DUAL_A, NW><<<dim3(grid), dim3(NW * 64), lds, s>>>(a, nM, nN, nfull, nunits);
    return hipGetLastError();
}

// ---- tail split-K second pass: one thread per accumulator-fragment quad (4 consecutive columns of one
//      row) of a split tile; sums the splits in split order and applies the epilogue exactly as the
//      single-pass kernel does.  For EPI_ROPE a thread owns the quad and its partner d/2 columns on.
template <int NW>
__global__ void __launch_bounds__(256) splitk_finish_kernel(GemmArgs a, int nM, int nN, int nfull) {
    constexpr int MI = 16 / NW, WROWS = 32 * MI;
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int rt = (int)(g >> 14);                 // split tile (16384 quads per tile)
    const int v = (int)(g & 16383);
    const int lane = v & 63, q = (v >> 6) & 3, j = (v >> 8) & 3, wi = v >> 10;
    const int wave = wi / MI, i = wi % MI;
    const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, lh = lane >> 5;
    int tm, tn;
    tile_of(nfull + rt, nM, nN, tm, tn);
    const int64_t grow = (int64_t)tm * BM + wm * WROWS + i * 32 + l32;
    const int col0 = tn * 256;
    const float* P = a.part32 + (int64_t)rt * a.ksplit * (BM * 256);
    auto quad = [&](int jj) {
        const float* p = P + ((((wave * MI + i) * 4 + jj) * 4 + q) * 64 + lane) * 4;
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
        for (int sp = 0; sp < a.ksplit; ++sp) s += *reinterpret_cast<const f32x4*>(p + (int64_t)sp * (BM * 256));
        return s;
    };
    const bool rok = grow < a.M;
    const int64_t growc = rok ? grow : a.M - 1;
    const int64_t crow = a.c_idx ? (int64_t)a.c_idx[growc] : growc;
    bf16_t* Cb = (bf16_t*)a.C;
    // two products in one launch: a tile is either a rotary tile of the first or a stored tile of the second
    int epi = a.epi, colshift = 0;
    int64_t ldo = a.ldc;
    if (epi == EPI_ROPE_STORE) {
        if (col0 >= a.n_split) { epi = EPI_STORE; colshift = a.n_split; Cb = (bf16_t*)a.C2; ldo = a.ldc2; }
        else epi = EPI_ROPE;
    }
    if (epi == EPI_STORE) {
        const f32x4 s = quad(j);
        const int col = col0 - colshift + wn * 128 + j * 32 + 4 * lh + 8 * q;
        u32x2 o = {pack_bf16x2(s.x, s.y), pack_bf16x2(s.z, s.w)};
        if (rok) {
            if (a.c_slab) *reinterpret_cast<u32x2*>(Cb + ((int64_t)(col >> 5) * a.M + grow) * 32 + (col & 31)) = o;   // slab-major C
            else *reinterpret_cast<u32x2*>(Cb + crow * ldo + col) = o;
        }
        if (a.Ct && grow < a.ldct) {
            bf16_t* ct = (bf16_t*)a.Ct;
            const uint16_t e[4] = {(uint16_t)(o.x & 0xffff), (uint16_t)(o.x >> 16), (uint16_t)(o.y & 0xffff), (uint16_t)(o.y >> 16)};
#pragma unroll
            for (int t = 0; t < 4; ++t) ct[(int64_t)(col + t) * a.ldct + vt_key_slot(grow)].v = e[t];
        }
    } else if (epi == EPI_RESIDUAL) {
        if (!rok) return;
        const f32x4 s = quad(j);
        const int col = col0 + wn * 128 + j * 32 + 4 * lh + 8 * q;
        u32x2* p = reinterpret_cast<u32x2*>(Cb + crow * a.ldc + col);
        const u32x2 old = *p;
        u32x2 o;
        o.x = pack_bf16x2(__uint_as_float(old.x << 16) + s.x, __uint_as_float(old.x & 0xffff0000u) + s.y);
        o.y = pack_bf16x2(__uint_as_float(old.y << 16) + s.z, __uint_as_float(old.y & 0xffff0000u) + s.w);
        *p = o;
    } else {   // EPI_ROPE
        if (!rok) return;
        const int half = a.head_dim >> 1;
        int j1, j2, jj;   // accumulator blocks of the quad and of its partner; column inside the half head
        if (half == 64) { if (j >= 2) return; j1 = j; j2 = j + 2; jj = j * 32 + 4 * lh + 8 * q; }
        else { if (j & 1) return; j1 = j; j2 = j + 1; jj = 4 * lh + 8 * q; }
        const f32x4 x1 = quad(j1), x2 = quad(j2);
        const int64_t trow = a.rope_idx ? (int64_t)a.rope_idx[grow] : grow;
        const float2* tab = a.rope + trow * half + jj;
        const float rs = a.rope_scale != 0.f ? a.rope_scale : 1.f;
        float lo[4], hi[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float2 cs = tab[t];
            lo[t] = (x1[t] * cs.x - x2[t] * cs.y) * rs;
            hi[t] = (x2[t] * cs.x + x1[t] * cs.y) * rs;
        }
        const int col = col0 + wn * 128 + (half == 64 ? 0 : (j >> 1) * 64) + jj;
        u32x2 o1 = {pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3])};
        u32x2 o2 = {pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3])};
        *reinterpret_cast<u32x2*>(Cb + crow * a.ldc + col) = o1;
        *reinterpret_cast<u32x2*>(Cb + crow * a.ldc + col + half) = o2;
    }
}

// Cost model behind the split plan (one workgroup per CU, 256 CUs): a whole tile takes
// t_tile = 2*256*256*K flops at the sustained per-CU rate; the tail of `rem` tiles costs one t_tile
// unsplit, or ceil(rem*ks/256)/ks of it plus the partial-tile traffic (rem*ks tiles of 256 KB, written
// and read back) plus one more launch when split ks ways.
int gemm_pick_split(int64_t M, int32_t N, int32_t K, int epi, int32_t* nfull) {
    *nfull = 0;
    if (epi != EPI_STORE && epi != EPI_RESIDUAL && epi != EPI_ROPE && epi != EPI_ROPE_STORE) return 1;
    if (N % 256 != 0 || M <= 0) return 1;
    const int64_t tiles = ((M + BM - 1) / BM) * (N / 256);
    const int rem = (int)(tiles % 256);
    if (rem == 0) return 1;
    const double t_tile = 2.0 * 256 * 256 * K / 4.2e12;
    double best = t_tile;
    int best_ks = 1;
    for (int ks = 2; ks <= 8; ++ks) {
        if (K / ks < 512) break;
        const int rounds = (rem * ks + 255) / 256;
        const double t = t_tile * rounds / ks + (double)rem * ks * 262144.0 * 2.0 / 4.0e12 + 6e-6;
        if (t < best * 0.97) { best = t; best_ks = ks; }
    }
    *nfull = (int32_t)(tiles - rem);
    return best_ks;
}

// wavefronts per workgroup used by launch_gemm_mfma (4 or 8)
#ifndef SPTS_GEMM_NW
#define SPTS_GEMM_NW 8
#endif

hipError_t launch_gemm_mfma(const GemmArgs& a, hipStream_t s) {
    constexpr int NW = SPTS_GEMM_NW;
    const bool slab = a.a_slab || a.b_slab;   // slab-major operands exist for 32-wide slabs only
    hipError_t e;
    switch (a.epi) {
        case EPI_STORE: e = (a.K % 64 == 0 && !slab ? launch_t<EPI_STORE, 64, false, NW>(a, s) : launch_t<EPI_STORE, 32, false, NW>(a, s)); break;
        case EPI_RESIDUAL: e = (a.K % 64 == 0 && !slab ? launch_t<EPI_RESIDUAL, 64, false, NW>(a, s) : launch_t<EPI_RESIDUAL, 32, false, NW>(a, s)); break;
        case EPI_SUMSQ: e = (a.K % 64 == 0 ? launch_t<EPI_SUMSQ, 64, false, NW>(a, s) : launch_t<EPI_SUMSQ, 32, false, NW>(a, s)); break;
        case EPI_ROPE: e = (a.K % 64 == 0 && !slab ? launch_t<EPI_ROPE, 64, false, NW>(a, s) : launch_t<EPI_ROPE, 32, false, NW>(a, s)); break;
        case EPI_ROPE_STORE: e = (a.K % 64 == 0 && !slab ? launch_t<EPI_ROPE_STORE, 64, false, NW>(a, s) : launch_t<EPI_ROPE_STORE, 32, false, NW>(a, s)); break;
        case EPI_SILU_MUL:
            if (a.A1) e = launch_t<EPI_SILU_MUL, 32, true, NW>(a, s);
            else e = launch_t<EPI_SILU_MUL, 32, false, NW>(a, s);   // 4 stages of 32 measured 2 % faster here than 2 of 64
            break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess || a.ksplit <= 1) return e;
    const int nM = (int)((a.M + BM - 1) / BM), nN = a.N / 256;
    const int64_t quads = (int64_t)(nM * nN - a.nfull) * 16384;
    if (quads <= 0) return hipSuccess;
    splitk_finish_kernel<NW><<<dim3((unsigned)(quads / 256)), dim3(256), 0, s>>>(a, nM, nN, a.nfull);
    return hipGetLastError();
}

}  // namespace spts
