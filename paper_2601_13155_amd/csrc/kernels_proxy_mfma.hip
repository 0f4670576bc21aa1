// Hidden layer of the low-rank proxy FFN on the matrix cores (Eq. (proxy_ffn)):
//   h[n, c] = silu( t_g[n, :] . Vg[c, :] ) * ( t_u[n, :] . Vu[c, :] ),   t_g = x Ug, t_u = x Uu  (K = r = 256)
// for all N candidates and all Dlow channels.  As a GEMM this is the least favourable shape of the layer: K is only 256,
// so a 256 x 128 output tile has 8 slabs between its prologue and an epilogue whose SiLU arithmetic (two
// quarter-rate transcendentals per element) takes about as much vector time as the 8 slabs take matrix time, one after
// the other.  This kernel turns the loops around:
//  * A wavefront owns 32 rows and keeps their t_g / t_u fragments in registers for its whole life (B operand of
//    h^T = V t^T: 16 k-steps x 2 x 4 registers = 128); a workgroup = 8 wavefronts = 256 rows.
//  * The workgroup streams its share of the channels in tiles of 32 (Vg and Vu rows, 32 KB per tile for r = 256) through a
//    4-stage direct-to-LDS ring shared by the 8 wavefronts (tiles are published in pairs: one barrier per two tiles); per
//    tile a wavefront issues 32 MFMAs (one LDS fragment each).
//  * Two accumulator sets alternate: while the matrix pipe works on tile c, the vector ALU takes SiLU(gate) * up of tile
//    c - 1, packs it to bf16 and stores it -- written as 16 steps of two MFMAs + one element's arithmetic, fenced for the
//    scheduler, so the two kinds of work are offered to the SIMD side by side.
//  * The rows of a weight tile are put into LDS with the two middle quads of every 16 swapped (vt_key_slot): the
//    accumulator layout of the 32x32 MFMA then gives a lane 2 x 8 consecutive channels, and one exchange between the lane
//    halves (v_permlane32_swap) makes that 16 consecutive channels = 32 contiguous bytes of its row, stored as two 16-byte
//    pieces; the wavefront's 32 rows x 64 bytes are one contiguous 2 KB of the slab-major output.  (Passing the tile
//    through LDS to store whole 1 KB runs per instruction measured 4 % slower: the round trip sits at the end of a tile.)
//  * Output: h slab-major [Dlow/32][N][32], the layout the following projection GEMM reads as whole lines.
//  * Grid: (row tiles of 256) x (channel shares); the share count is chosen so that the workgroups fill whole rounds of the
//    256 CUs.  Workgroups of one XCD take neighbouring ids, i.e. mostly the same channel share: its weights stay in that L2.
// Same products in the same k order as the GEMM path and the same SiLU: results are bit-identical to it.
#include "spts_internal.h"

namespace spts {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PH_NSTG = 4;          // ring stages (tiles of 32 channels)
constexpr int PH_WAVES = 8;

__device__ inline float ph_silu(float g) {
    return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
}

template <int KS>   // k-steps of 16: r = 16 * KS
__global__ void __launch_bounds__(PH_WAVES * 64) proxy_hidden_kernel(ProxyHiddenArgs a, int RT, int SC) {
    constexpr int NSL = KS / 2;                   // 32-wide K slabs
    constexpr int MAT_BYTES = NSL * 2048;         // one matrix's tile: [NSL][32 channels][64 bytes]
    constexpr int STAGE = 2 * MAT_BYTES;          // Vg tile + Vu tile
    constexpr int LOADS = 2 * NSL * 2;            // 1 KB loads per tile
    constexpr int LPW = LOADS / PH_WAVES;         // per wavefront
    constexpr int EPS = 16 / KS;                  // elements of the previous tile finished per k-step
    static_assert(KS == 16, "r = 256");
    extern __shared__ __attribute__((aligned(16))) char smem[];   // the ring: PH_NSTG stages of (Vg tile, Vu tile)

    // ---- work unit: (row tile, channel share); ids of one XCD are consecutive
    const int total = RT * SC;
    const int per = (total + 7) / 8;
    const int id = (int)(blockIdx.x % 8) * per + (int)(blockIdx.x / 8);
    if (id >= total) return;
    const int sc = id / RT, rt = id % RT;
    const int TT = a.Dlow / 32;
    const int tile_begin = (int)((int64_t)sc * TT / SC), tile_end = (int)((int64_t)(sc + 1) * TT / SC);
    const int ntiles = tile_end - tile_begin;
    if (ntiles <= 0) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;
    const int64_t row0w = (int64_t)rt * 256 + wave * 32;

    // ---- direct-to-LDS loads of a weight tile: load q = (matrix X, slab s, 16-row half hf); lane -> (LDS row, chunk position)
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    uint32_t goff[2];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
        const int m = hf * 16 + (lane >> 2);                 // LDS row of the tile
        const int ch = (int)vt_key_slot(m);                  // channel (inside the tile) that belongs there
        const int c = (lane & 3) ^ ((m >> 2) & 3);           // global chunk for this LDS chunk position
        goff[hf] = (uint32_t)(ch * 64 + c * 16);
    }
    const char* Wg = (const char*)a.Vg_s;
    const char* Wu = (const char*)a.Vu_s;
#define SPTS_PH_DMA(tl_)                                                                                      \
    {                                                                                                         \
        const int tile_ = tile_begin + (tl_);                                                                 \
        const uint32_t st_ = lds0 + (uint32_t)(((tl_) % PH_NSTG) * STAGE);                                    \
        _Pragma("unroll") for (int u_ = 0; u_ < LPW; ++u_) {                                                  \
            const int q_ = wave * LPW + u_;                                                                   \
            const int X_ = q_ / (2 * NSL), s_ = (q_ % (2 * NSL)) >> 1, hf_ = q_ & 1;                          \
            const char* src_ = (X_ ? Wu : Wg) + ((int64_t)s_ * a.Dlow + (int64_t)tile_ * 32) * 64;            \
            dma16s(goff[hf_], src_, st_ + (uint32_t)(X_ * MAT_BYTES + s_ * 2048 + hf_ * 1024));               \
        }                                                                                                     \
    }

    // ---- prologue: the first four tiles in flight, then this wavefront's rows of t into registers
    {
        const int npre = ntiles < PH_NSTG ? ntiles : PH_NSTG;
        for (int t = 0; t < npre; ++t) SPTS_PH_DMA(t)
    }
    bf16x8 tg[KS], tu[KS];
    {
        int64_t row = row0w + l32;
        if (row >= a.N) row = a.N - 1;
        const char* pg = (const char*)a.tg + row * a.t_row_pitch + lh * 16;
        const char* pu = (const char*)a.tu + row * a.t_row_pitch + lh * 16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int64_t o = (int64_t)(ks >> 1) * a.t_slab_pitch + (ks & 1) * 32;
            tg[ks] = *reinterpret_cast<const bf16x8*>(pg + o);
            tu[ks] = *reinterpret_cast<const bf16x8*>(pu + o);
        }
    }
    // fragment read offsets inside a matrix tile for the two k-steps of a slab
    uint32_t foff[2];
#pragma unroll
    for (int par = 0; par < 2; ++par) foff[par] = (uint32_t)(l32 * 64 + (((2 * par + lh) ^ ((l32 >> 2) & 3)) << 4));
    char* hp = (char*)a.hp;
    const int64_t out_off = (row0w + l32) * 64 + lh * 32;   // the lane's 32 bytes inside a slab of the output
    const bool row_ok = row0w + l32 < a.N;

    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 Ga = zero16, Ua = zero16, Gb = zero16, Ub = zero16;

    // One tile: 2*KS MFMAs into (GC, UC) from the ring stage of tile tl_, interleaved with the arithmetic of the previous
    // tile's accumulators (GP, UP), whose packed result is stored at the end (two 16-byte pieces per lane).
    constexpr int FD = 3;   // fragment reads run FD k-steps ahead (2 and 4 measure the same)
#define SPTS_PH_FRAG(X_, ks_) (*reinterpret_cast<const bf16x8*>(sT_ + (X_) * MAT_BYTES + ((ks_) >> 1) * 2048 + foff[(ks_) & 1]))
#define SPTS_PH_TILE(tl_, GC, UC, GP, UP)                                                                      \
    {                                                                                                         \
        const char* sT_ = smem + ((tl_) % PH_NSTG) * STAGE;                                                   \
        const bool prev_ = (tl_) > 0;                                                                         \
        bf16x8 fg_[FD + 1], fu_[FD + 1];                                                                      \
        _Pragma("unroll") for (int i_ = 0; i_ < FD; ++i_) { fg_[i_] = SPTS_PH_FRAG(0, i_); fu_[i_] = SPTS_PH_FRAG(1, i_); } \
        float h_[16];                                                                                         \
        _Pragma("unroll") for (int i_ = 0; i_ < KS; ++i_) {                                                   \
            if (i_ + FD < KS) { fg_[(i_ + FD) % (FD + 1)] = SPTS_PH_FRAG(0, i_ + FD); fu_[(i_ + FD) % (FD + 1)] = SPTS_PH_FRAG(1, i_ + FD); } \
            GC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fg_[i_ % (FD + 1)], tg[i_], i_ == 0 ? zero16 : GC, 0, 0, 0); \
            UC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fu_[i_ % (FD + 1)], tu[i_], i_ == 0 ? zero16 : UC, 0, 0, 0); \
            _Pragma("unroll") for (int e_ = i_ * EPS; e_ < (i_ + 1) * EPS; ++e_) h_[e_] = ph_silu(GP[e_]) * UP[e_]; \
            __builtin_amdgcn_sched_barrier(0);                                                                \
        }                                                                                                     \
        if (prev_) {                                                                                          \
            u32x4 x_, y_;                                                                                     \
            _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_) {                                                \
                const uint32_t lo_ = cvt_pk_bf16(h_[2 * j_], h_[2 * j_ + 1]);                                 \
                const uint32_t hi_ = cvt_pk_bf16(h_[8 + 2 * j_], h_[8 + 2 * j_ + 1]);                         \
                const auto sw_ = __builtin_amdgcn_permlane32_swap(lo_, hi_, false, false);                    \
                x_[j_] = sw_[0]; y_[j_] = sw_[1];                                                             \
            }                                                                                                 \
            char* dst_ = hp + (int64_t)(tile_begin + (tl_) - 1) * a.N * 64 + out_off;                         \
            if (row_ok) { *reinterpret_cast<u32x4*>(dst_) = x_; *reinterpret_cast<u32x4*>(dst_ + 16) = y_; }  \
        }                                                                                                     \
    }

    // Everything in flight lands here (the t fragments included): the compiler does not see the direct-to-LDS loads, so
    // a wait it would place later for its own loads must find none outstanding.
    SPTS_WAIT_VMCNT(0);
    __syncthreads();
    // Tiles are taken in pairs: one wait + one workgroup barrier publishes tiles tl and tl + 1 (their loads were issued
    // right after the previous barrier) and frees the two stages the previous pair was read from, which the loads of
    // tiles tl + 2 and tl + 3 then refill.  The only operations a wavefront issued after those loads are the previous pair's
    // four output stores (two per tile), so "all but the newest 4" covers the loads -- provided the stores were really
    // issued: a wavefront whose rows reach past N may skip some (no active lane), so it waits for everything instead.
    const bool full_wave = row0w + 32 <= a.N;
    for (int tl = 0; tl < ntiles; tl += 2) {
        if (tl > 0) {
            if (full_wave) { SPTS_WAIT_VMCNT(4); } else { SPTS_WAIT_VMCNT(0); }
            __syncthreads();
            if (tl + 2 < ntiles) SPTS_PH_DMA(tl + 2)
            if (tl + 3 < ntiles) SPTS_PH_DMA(tl + 3)
        }
        SPTS_PH_TILE(tl, Ga, Ua, Gb, Ub)
        if (tl + 1 < ntiles) SPTS_PH_TILE(tl + 1, Gb, Ub, Ga, Ua)
    }
    // the last tile's accumulators: a slot without MFMAs
    {
        const bool odd = (ntiles & 1) != 0;   // last tile index is even -> it used (Ga, Ua)
        float h[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) h[e] = odd ? ph_silu(Ga[e]) * Ua[e] : ph_silu(Gb[e]) * Ub[e];
        u32x4 x, y;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t lo = cvt_pk_bf16(h[2 * j], h[2 * j + 1]);
            const uint32_t hi = cvt_pk_bf16(h[8 + 2 * j], h[8 + 2 * j + 1]);
            const auto sw2 = __builtin_amdgcn_permlane32_swap(lo, hi, false, false);
            x[j] = sw2[0]; y[j] = sw2[1];
        }
        char* dst = hp + (int64_t)(tile_end - 1) * a.N * 64 + out_off;
        if (row_ok) { *reinterpret_cast<u32x4*>(dst) = x; *reinterpret_cast<u32x4*>(dst + 16) = y; }
    }
}

bool proxy_hidden_supported(const ProxyHiddenArgs& a) {
    if (a.r != 256) return false;   // the rank every configuration uses; other ranks take the GEMM path
    if (a.N <= 0 || a.N >= ((int64_t)1 << 31) || a.Dlow <= 0 || a.Dlow % 32 != 0) return false;
    if (!a.Vg_s || !a.Vu_s || !a.tg || !a.tu || !a.hp) return false;
    auto al = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    if (!al(a.Vg_s) || !al(a.Vu_s) || !al(a.tg) || !al(a.tu) || !al(a.hp)) return false;
    if (a.t_row_pitch % 16 != 0 || a.t_slab_pitch % 16 != 0) return false;
    return true;
}

// channel shares per row tile: the smallest count (each share at least 8 tiles of 32 channels) whose workgroups fill
// whole rounds of the 256 CUs to within 3 % of the best
static int pick_shares(int RT, int TT) {
    int best = 1;
    double best_eff = 0.0;
    for (int sc = 1; sc <= 64 && TT / sc >= 8; ++sc) {
        const int64_t wg = (int64_t)RT * sc;
        const int64_t rounds = (wg + 255) / 256;
        const double eff = (double)wg / (double)(rounds * 256);
        if (eff > best_eff * 1.03) { best_eff = eff; best = sc; }
    }
    return best;
}

hipError_t launch_proxy_hidden(const ProxyHiddenArgs& a, hipStream_t s) {
    const int RT = (int)((a.N + 255) / 256), TT = a.Dlow / 32;
    const int SC = pick_shares(RT, TT);
    const int total = RT * SC;
    const int grid = (total + 7) / 8 * 8;
    const int ks = a.r / 16;
    const size_t lds = (size_t)PH_NSTG * 2 * (ks / 2) * 2048;
    if (ks != 16) return hipErrorInvalidValue;
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&proxy_hidden_kernel<16>), (int)lds);
    if (e != hipSuccess) return e;
    proxy_hidden_kernel<16><<<dim3(grid), dim3(PH_WAVES * 64), lds, s>>>(a, RT, SC);
    return hipGetLastError();
}

}  // namespace spts
