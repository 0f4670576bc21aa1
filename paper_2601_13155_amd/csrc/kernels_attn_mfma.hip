// Flash-style causal GQA prefill attention on the matrix cores (bf16 in, fp32 softmax/accumulate).
//
// out[i, h, :] = softmax_j( q[i,h].k[j,g(h)] / sqrt(d)  for kpos[j] <= qpos[i] ) . v[j, g(h), :]
// The query set and the key set carry their own ascending absolute positions, so the same kernel
// serves the reduced attention over the active tokens of Alg. 1 (queries = keys = active set), the
// dense branch, and queries = active / keys = all candidates.
//
// Layout of the computation (gfx950, wave64, MFMA 32x32x16 bf16):
//  * S^T = K Q^T is computed instead of S: the MFMA result then has one query per lane column, so
//    the row sum of the softmax is an in-lane reduction plus one exchange with lane^32 at the end,
//    and the probabilities already sit in the operand layout of the second product.
//  * O^T += V^T P^T takes V^T tiles (keys contiguous) as the A operand.  The value projection
//    writes that transposed copy with the keys of every 16-group in the order the probability
//    fragments come out of the matrix core (vt_key_slot), so a value fragment is one 16-byte read.
//  * One workgroup = 8 wavefronts x 32 queries, two wavefronts per SIMD; the wavefronts belong to 4, 2 or 1 heads of one
//    kv-head group (as many as divide the group: 64, 128 or 256 queries of each), which multiply the same K / V^T tiles,
//    so a tile loaded once serves all of them (+3.5 % at 13K keys with 4 heads against 1).  Two wavefronts per SIMD, so
//    one wavefront's softmax arithmetic and LDS latencies hide behind the other's MFMAs (4 wavefronts
//    x 64 queries halve the LDS traffic but leave every LDS round trip exposed: 540 vs 820 TFLOP/s with the
//    earlier softmax).
//    K / V^T tiles of 64 keys travel global memory -> LDS directly (global_load_lds_dwordx4, swizzle
//    applied on the global side) into a ring of 5 stages (all 160 KB): tile t+3 is in flight while the
//    keys of tiles t and t+1 and the values of tiles t-1 and t are multiplied; one barrier per tile.
//  * Software pipeline inside the wavefront at 32-key block granularity: a slot holds the QK^T MFMAs of
//    block b+1, the PV MFMAs of block b-1 and the softmax arithmetic of block b (three independent
//    register sets), written as 16 steps of one MFMA + one fragment read (a few steps ahead) + a share
//    of the softmax.  A wavefront issues in order, so vector instructions only run in the shadow of an
//    MFMA when they sit right behind it in the instruction stream (measured on this chip: a 1:1 mix of
//    MFMA time and vector time takes 0.75 of their sum when interleaved, their sum when not).
//    With the textbook online softmax (scale folded into an FMA, running maximum per block, rescale when it moved)
//    the vector ALU was as busy as the matrix pipe (57 % / 56 % of the cycles, counters) and the two overlapped for
//    only half of that; the softmax here is cut to one exponential per logit and one conversion + one dot product
//    per pair (see the slot below): q arrives pre-scaled, the MFMA starts from minus a reference maximum that
//    moves only when a block overflows it by a wide margin, the row sum is a bf16 dot product with (1, 1).
//    816 -> ~970 TFLOP/s at 13107 x 13107, 32 heads.  What is left is issue-bound rather than bound by one unit:
//    timing variants without the softmax, without the fragment reads, without the tile loads or without the barrier
//    each gain 4-12 %, and all of them together reach 1450 TFLOP/s (MFMAs only, at the clock the chip then holds).
//  * Key tiles beyond the last visible position are never visited; tiles that are entirely visible
//    to a wavefront skip the mask; a wavefront whose queries see nothing of a tile skips its work.
//  * Work items are laid out (kv head, query tile descending, head in group) and split over the 8 XCDs so that the heads
//    that share a KV head run on the same XCD's L2, longest tiles first: contiguously when there are at least 8 kv heads,
//    dealt out in turn to the XCDs of a head's group when there are fewer (so that every XCD gets long and short tiles).
#include "spts_internal.h"

namespace spts {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int BKV = 64;
constexpr int ATT_NST = 5;
constexpr float ATT_TAU = 8.0f;        // a query's reference maximum moves to a block's maximum that is this far above it (log2 units)
constexpr float ATT_SUM_MAX = 4096.0f; // a lane asks for the check when its 16 probabilities of a block sum to more (16 * 2^ATT_TAU)

template <int D> struct AttnLds {
    static constexpr int K_BYTES = BKV * D * 2;
    static constexpr int V_BYTES = D * BKV * 2;
    static constexpr int STAGE = K_BYTES + V_BYTES;
    static constexpr int CPRK = D / 8;            // 16-byte chunks per K row
    static constexpr int RPK = 256 / (2 * D);     // K rows per 256 bytes
    static constexpr int K_ROWS_PER_LOAD = 64 / CPRK;
    // per wavefront, NW wavefronts: BKV/NW K rows and D/NW V^T rows each (8 V^T rows per load)
    template <int NW> static constexpr int k_loads() { return (BKV / NW) / K_ROWS_PER_LOAD; }
    template <int NW> static constexpr int v_loads() { return (D / NW) / 8; }
    __device__ static inline int kswz(int row) { return (row / RPK) % CPRK; }
    __device__ static inline int koff(int row, int c) { return row * (2 * D) + ((c ^ kswz(row)) << 4); }
    // V^T tile: row = value column (128 bytes = 8 chunks of 16 bytes = 8 keys each)
    __device__ static inline int vswz(int row) { return (row >> 1) & 7; }
    __device__ static inline int voff(int row, int c) { return row * (BKV * 2) + ((c ^ vswz(row)) << 4); }
};

__device__ inline uint32_t pk2(float a, float b) { return cvt_pk_bf16(a, b); }

// HPW heads of one kv-head group per workgroup (NW / HPW wavefronts x 32 queries each): they multiply the same K / V^T
// tiles, so a tile that is loaded once serves HPW heads.
template <int D, int HPW, int NW>
__global__ void __launch_bounds__(NW * 64) attn_mfma_kernel(AttnArgs a, int nQ, int total, int xpg, float qmul) {
    using L = AttnLds<D>;
    constexpr int QB = 1;                // 32-query blocks per wavefront
    constexpr int WPH = NW / HPW;        // wavefronts per head
    constexpr int BQ = WPH * QB * 32;    // queries (of each of its heads) per workgroup
    static_assert(NW % HPW == 0, "whole wavefronts per head");
    constexpr int KS = D / 16;   // k-steps of the QK^T product
    constexpr int DB = D / 32;   // 32-column blocks of the output
    constexpr int K_LOADS = L::template k_loads<NW>();
    constexpr int V_LOADS = L::template v_loads<NW>();
    constexpr int PER = K_LOADS + V_LOADS;
    constexpr int NSTEP = KS + 2 * DB;   // MFMAs per pipeline slot: QK^T of one block + PV of another
#ifndef SPTS_ATT_FD
#define SPTS_ATT_FD 3
#endif
    constexpr int FD = SPTS_ATT_FD;      // fragment reads run FD steps ahead of the MFMA that consumes them
    static_assert(NSTEP == 16 || NSTEP == 8, "the pipeline slot is written for these two head sizes");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // Work item = (kv head g, query tile, HPW heads of the group), the items of a kv head ordered longest tile first.
    // Workgroup b runs on XCD b % 8 as that XCD's (b / 8)-th workgroup.  With at least 8 kv heads every XCD takes a
    // contiguous range of items (whole kv heads when Hkv % 8 == 0).  With fewer kv heads (xpg = 8 / Hkv XCDs per head) a
    // contiguous range would give one XCD of the group the long tiles and another the short ones (a causal tile's work
    // grows with its index), so the items of a head are dealt out to its XCDs in turn.
    const int grp = a.H / a.Hkv;
    const int ngh = grp / HPW;           // head sets per kv head (the host picks an HPW that divides the group)
    int g, item;
    if (xpg > 1) {
        const int xcd = (int)(blockIdx.x % 8), pos = (int)(blockIdx.x / 8);
        g = xcd / xpg;
        item = pos * xpg + xcd % xpg;
        if (item >= nQ * ngh) return;
    } else {
        const int per = (total + 7) / 8;
        const int id = (int)(blockIdx.x % 8) * per + (int)(blockIdx.x / 8);
        if (id >= total) return;
        g = id / (ngh * nQ);
        item = id % (ngh * nQ);
    }
    const int qtile = nQ - 1 - item / ngh;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;
    const int h = g * grp + (item % ngh) * HPW + wave / WPH;   // this wavefront's head
    const int64_t q0 = (int64_t)qtile * BQ;
    const int64_t q0w = q0 + (wave % WPH) * (QB * 32);

    // ---- visible key ranges.  Positions are strictly ascending, so "keys visible to position p" is a
    //      prefix; its length is an upper bound search (or the index itself when both sets coincide).
    const bool same_set = a.qpos == a.kpos;
    auto visible_count = [&](int64_t qi) -> int64_t {
        if (same_set) return qi + 1;
        const int p = a.qpos[qi];
        int64_t lo = 0, hi = a.Mk;
        while (lo < hi) {
            int64_t mid = (lo + hi) >> 1;
            if (a.kpos[mid] <= p) lo = mid + 1; else hi = mid;
        }
        return lo;
    };
    const int64_t q_last = (q0 + BQ < a.Mq ? q0 + BQ : a.Mq) - 1;
    const int n_tiles = (int)((visible_count(q_last) + BKV - 1) / BKV);            // workgroup
    const int64_t qw_first = q0w < a.Mq ? q0w : a.Mq - 1;
    int64_t qw_last = (q0w + QB * 32 < a.Mq ? q0w + QB * 32 : a.Mq) - 1;
    if (qw_last < qw_first) qw_last = qw_first;
    const int nbw = (int)((visible_count(qw_last) + 31) / 32);     // 32-key blocks this wavefront works on
    const int nbfull = (int)(visible_count(qw_first) / 32);        // blocks it sees entirely (no mask)

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds q[query = l32][16*ks + 8*lh .. +7]
    bf16x8 qf[QB][KS];
    int qpos_l[QB];
    const bf16_t* Q = (const bf16_t*)a.q;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int64_t qi = q0w + qb * 32 + l32;
        if (qi >= a.Mq) qi = a.Mq - 1;
        qpos_l[qb] = a.qpos[qi];
        const bf16_t* qr = Q + (qi * a.H + h) * (int64_t)D + 8 * lh;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = *reinterpret_cast<const bf16x8*>(qr + 16 * ks);
        // q normally arrives carrying log2(e)/sqrt(d) (qmul == 1); otherwise the rest of the factor is folded in here
        if (qmul != 1.0f) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                u32x4 raw = __builtin_bit_cast(u32x4, qf[qb][ks]);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    raw[j] = pk2(__uint_as_float(raw[j] << 16) * qmul, __uint_as_float(raw[j] & 0xffff0000u) * qmul);
                qf[qb][ks] = __builtin_bit_cast(bf16x8, raw);
            }
        }
    }

    // ---- direct-to-LDS tile loads.  Wavefront w moves K rows [64/NW*w, 64/NW*(w+1)) and V^T rows
    //      [D/NW*w, D/NW*(w+1)); a lane fetches the chunk that the swizzle maps to its LDS position.
    const bf16_t* Kg = (const bf16_t*)a.k;
    const bf16_t* Vt = (const bf16_t*)a.vt;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    // A lane's byte offset from the tile's first key (K) / first key column of the kv head's V^T rows is the same for
    // every tile; the tile's base is wavefront-uniform and advances in scalar registers.
    int krow[K_LOADS], kchunk[K_LOADS];
    uint32_t koffv[K_LOADS], voffv[V_LOADS];
#pragma unroll
    for (int q = 0; q < K_LOADS; ++q) {
        krow[q] = wave * (BKV / NW) + q * L::K_ROWS_PER_LOAD + lane / L::CPRK;
        kchunk[q] = (lane % L::CPRK) ^ L::kswz(krow[q]);
        koffv[q] = (uint32_t)((krow[q] * a.Hkv * D + kchunk[q] * 8) * 2);
    }
#pragma unroll
    for (int q = 0; q < V_LOADS; ++q) {
        const int row = wave * (D / NW) + q * 8 + (lane >> 3);
        const int c = (lane & 7) ^ L::vswz(row);
        voffv[q] = (uint32_t)(((int64_t)row * a.ldvt + c * 8) * 2);   // < 2^32: checked on the host
    }
    const bf16_t* Vg = Vt + (int64_t)g * D * a.ldvt;
#define SPTS_ATT_DMA(t_)                                                                                   \
    {                                                                                                      \
        const int64_t key0_ = (int64_t)(t_) * BKV;                                                         \
        const uint32_t sb_ = lds0 + ((t_) % ATT_NST) * L::STAGE;                                           \
        if (key0_ + BKV <= a.Mk) {                                                                         \
            const bf16_t* kb_ = Kg + (key0_ * a.Hkv + g) * (int64_t)D;                                     \
            _Pragma("unroll") for (int q = 0; q < K_LOADS; ++q)                                            \
                dma16s(koffv[q], kb_, sb_ + wave * (BKV / NW * 2 * D) + q * 1024);                         \
        } else {   /* last, partial tile: rows past the end re-read the last key (masked later) */         \
            _Pragma("unroll") for (int q = 0; q < K_LOADS; ++q) {                                          \
                int64_t key_ = key0_ + krow[q];                                                            \
                if (key_ >= a.Mk) key_ = a.Mk - 1;                                                         \
                dma16(Kg + (key_ * a.Hkv + g) * (int64_t)D + kchunk[q] * 8,                                \
                      sb_ + wave * (BKV / NW * 2 * D) + q * 1024);                                         \
            }                                                                                              \
        }                                                                                                  \
        _Pragma("unroll") for (int q = 0; q < V_LOADS; ++q)                                                \
            dma16s(voffv[q], Vg + key0_, sb_ + L::K_BYTES + wave * (D / NW * BKV * 2) + q * 1024);         \
    }

    f32x16 o[DB][QB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][qb][r] = 0.f;
    float l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) l_run[qb] = 0.f;
    // minus the reference maximum of the lane's query, 16 times: the C operand that starts a block's S^T product, so the
    // logits leave the matrix core already relative to it
    f32x16 cinit = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 sa[QB], sb[QB];   // S^T of two consecutive 32-key blocks (one being produced, one in the softmax)
    bf16x8 pfa[QB][2], pfb[QB][2];   // probabilities of two consecutive blocks (one being produced, one multiplied)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {   // slot 0 multiplies an all-zero "block -1"
            const u32x4 z_ = {0u, 0u, 0u, 0u};
            pfa[qb][hf] = __builtin_bit_cast(bf16x8, z_);
            pfb[qb][hf] = __builtin_bit_cast(bf16x8, z_);
        }
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const bf16x2 ones2 = {(__bf16)1.0f, (__bf16)1.0f};

    // S^T block: 32 keys (block kb_ of the tile in `stage_`) x QB*32 queries
#define SPTS_ATT_QK(SDST, stage_, kb_)                                                                     \
    {                                                                                                      \
        const char* sK_ = smem + (stage_) * L::STAGE;                                                      \
        _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                                \
            const bf16x8 kf_ = *reinterpret_cast<const bf16x8*>(sK_ + L::koff((kb_) * 32 + l32, 2 * ks + lh)); \
            _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)                                              \
                SDST[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf_, qf[qb][ks], ks == 0 ? zero16 : SDST[qb], 0, 0, 0); \
        }                                                                                                  \
    }
    // mask of a block that this wavefront does not see entirely (diagonal blocks, tail block)
#define SPTS_ATT_MASK(SSRC, b_)                                                                            \
    {                                                                                                      \
        const int64_t key0_ = (int64_t)(b_) * 32;                                                          \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                   \
            const int64_t key_ = key0_ + 8 * (r >> 2) + 4 * lh + (r & 3);                                  \
            const int kpl_ = a.kpos[key_ < a.Mk ? key_ : a.Mk - 1];   /* unconditional, in-bounds load */  \
            const int kp_ = key_ < a.Mk ? kpl_ : 0x7fffffff;                                               \
            _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)                                              \
                SSRC[qb][r] = kp_ > qpos_l[qb] ? -INFINITY : SSRC[qb][r];                                  \
        }                                                                                                  \
    }
    // Slot b_ of the wavefront's pipeline (block = 2*tile + kb).  Three independent instruction streams
    // share it: the QK^T MFMAs of block b_+1, the PV MFMAs of block b_-1 and the softmax arithmetic of
    // block b_.  The matrix pipe and the vector ALU work side by side only when a wavefront offers both
    // kinds of work at once (it issues in order: behind a run of MFMAs it can only wait for the pipe), so
    // the slot is written as NSTEP steps of one MFMA + one fragment read (FD steps ahead) + a share of
    // the softmax, fenced off from each other for the scheduler.
    // The vector ALU is the scarcer unit here (counters: both units busy ~57 % of the time with the classic online
    // softmax), so the softmax is kept to the instructions that cannot be avoided -- per logit one exponential, per
    // pair of logits one conversion and one dot product with (1, 1) for the row sum:
    //  * q carries log2(e)/sqrt(d) and every S^T product starts from minus the query's reference maximum (cinit): the
    //    MFMA delivers the exponent itself.
    //  * No maximum is taken in the common path.  The reference is the maximum of block 0 and afterwards moves only
    //    when a lane's sum of 16 probabilities exceeds ATT_SUM_MAX (some logit is then more than ATT_TAU above the
    //    reference; an overflowed exponential makes the sum infinite and is caught the same way).  The softmax does not
    //    depend on the reference, and probabilities up to ATT_SUM_MAX are far inside the range of the fp32 sums and
    //    the bf16 operands.
    //  * A move is the rare path, taken by the whole wavefront when any lane asks: block maximum per query, the
    //    block's logits shifted and its probabilities recomputed, the accumulator and the row sum (blocks < b_, whose
    //    MFMAs were issued above) rescaled, the S^T of block b_+1 (started from the old reference) shifted and cinit
    //    refreshed.
    // Slot 0 multiplies an all-zero block -1; the slot after a wavefront's last block (live_ false) only multiplies
    // that block's probabilities: its QK^T product and softmax run on stale data and leave the reference and the row
    // sum untouched.
#define SPTS_ATT_FRAG(s_)                                                                                  \
    ((s_) < KS ? *reinterpret_cast<const bf16x8*>(sQ_ + L::koff(kbq_ * 32 + l32, 2 * ((s_) % KS) + lh))    \
               : *reinterpret_cast<const bf16x8*>(sP_ + L::voff((((s_) - KS) % DB) * 32 + l32,             \
                                                              2 * (2 * kbp_ + ((s_) - KS) / DB) + lh)))
#define SPTS_ATT_PAIR(c_)                                                                                  \
    {                                                                                                      \
        const uint32_t w_ = pk2(p_[2 * (c_)], p_[2 * (c_) + 1]);   /* a scalar: bit_cast of a vector element reads element 0 */ \
        pk_[(c_) >> 2][(c_) & 3] = w_;                                                                     \
        sum_ = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w_), ones2, sum_, false);        \
    }
#define SPTS_ATT_BLOCK(b_, SC, SN, PC, PP)                                                                 \
    if ((b_) <= nbw) {                                                                                     \
        const bool live_ = (b_) < nbw;                                                                     \
        if (live_ && (b_) >= nbfull) SPTS_ATT_MASK(SC, b_)                                                 \
        const int bn_ = (b_) + 1, bp_ = (b_) >= 1 ? (b_) - 1 : 0;                                          \
        const char* sQ_ = smem + ((bn_ >> 1) % ATT_NST) * L::STAGE;                                        \
        const char* sP_ = smem + ((bp_ >> 1) % ATT_NST) * L::STAGE + L::K_BYTES;                           \
        const int kbq_ = bn_ & 1, kbp_ = bp_ & 1;                                                          \
        bf16x8 fr_[FD + 1];                                                                                \
        _Pragma("unroll") for (int i_ = 0; i_ < FD; ++i_) fr_[i_] = SPTS_ATT_FRAG(i_);                     \
        float p_[16], sum_ = 0.f;                                                                          \
        u32x4 pk_[2];                                                                                      \
        _Pragma("unroll") for (int i_ = 0; i_ < NSTEP; ++i_) {                                             \
            if (i_ + FD < NSTEP) fr_[(i_ + FD) % (FD + 1)] = SPTS_ATT_FRAG(i_ + FD);                       \
            if (i_ < KS)                                                                                   \
                SN[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr_[i_ % (FD + 1)], qf[0][i_ % KS], i_ == 0 ? cinit : SN[0], 0, 0, 0); \
            else                                                                                           \
                o[(i_ - KS) % DB][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr_[i_ % (FD + 1)], PP[0][(i_ - KS) / DB], \
                                                                               o[(i_ - KS) % DB][0], 0, 0, 0); \
            constexpr int EPS_ = 16 / NSTEP;   /* exponentials per step: 1 or 2 */                         \
            _Pragma("unroll") for (int e = i_ * EPS_; e < (i_ + 1) * EPS_; ++e) p_[e] = __builtin_amdgcn_exp2f(SC[0][e]); \
            if (EPS_ == 2) SPTS_ATT_PAIR(i_)                                                               \
            else if (i_ & 1) SPTS_ATT_PAIR(i_ >> 1)                                                        \
            __builtin_amdgcn_sched_barrier(0);                                                             \
        }                                                                                                  \
        /* a use of the probabilities in this basic block: without it the exponentials are sunk past */   \
        /* the branch below, out of reach of the MFMAs they are meant to overlap                      */   \
        asm volatile("" ::"v"(pk_[0]), "v"(pk_[1]), "v"(sum_));                                            \
        const bool ask_ = live_ && ((b_) == 0 || !(sum_ <= ATT_SUM_MAX));                                  \
        if (__ballot(ask_) != 0) {                                                                         \
            asm volatile("");   /* keeps this a branch */                                                  \
            float mx_ = -INFINITY;                                                                         \
            _Pragma("unroll") for (int r = 0; r < 16; ++r) mx_ = fmaxf(mx_, SC[0][r]);                     \
            const auto sw_ = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx_), __float_as_uint(mx_), false, false); \
            mx_ = fmaxf(__uint_as_float(sw_[0]), __uint_as_float(sw_[1]));                                 \
            const bool need_ = live_ && mx_ > ((b_) == 0 ? -INFINITY : ATT_TAU);                           \
            const float pend_ = need_ ? mx_ : 0.f;                                                         \
            sum_ = 0.f;                                                                                    \
            _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                               \
                SC[0][r] -= pend_;                                                                         \
                p_[r] = __builtin_amdgcn_exp2f(SC[0][r]);                                                  \
            }                                                                                              \
            _Pragma("unroll") for (int c = 0; c < 8; ++c) SPTS_ATT_PAIR(c)                                 \
            if ((b_) > 0) {   /* in slot 0 both are still zero, and 2^-pend_ may not be finite */           \
                const float alpha_ = __builtin_amdgcn_exp2f(-pend_);                                       \
                l_run[0] *= alpha_;                                                                        \
                _Pragma("unroll") for (int db = 0; db < DB; ++db)                                          \
                    _Pragma("unroll") for (int r = 0; r < 16; ++r) o[db][0][r] *= alpha_;                  \
            }                                                                                              \
            _Pragma("unroll") for (int r = 0; r < 16; ++r) { SN[0][r] -= pend_; cinit[r] -= pend_; }       \
        }                                                                                                  \
        PC[0][0] = __builtin_bit_cast(bf16x8, pk_[0]);                                                     \
        PC[0][1] = __builtin_bit_cast(bf16x8, pk_[1]);                                                     \
        l_run[0] += live_ ? sum_ : 0.f;                                                                    \
    }

    // ---- prologue: tiles 0..2 in flight, tile 0 landed, S^T of block 0
    if (n_tiles > 0) SPTS_ATT_DMA(0)
    if (n_tiles > 1) SPTS_ATT_DMA(1)
    if (n_tiles > 2) SPTS_ATT_DMA(2)
    // Everything in flight must land here, the query fragments included: the compiler does not see the
    // direct-to-LDS loads, so a wait it places inside the loop for one of its own earlier loads (vmcnt
    // counts both kinds) would drain the ring on every block.  After an explicit vmcnt(0) it has none left.
    SPTS_WAIT_VMCNT(0);
    __syncthreads();
    if (nbw > 0) SPTS_ATT_QK(sa, 0, 0)
    for (int t = 0; t < n_tiles; ++t) {
        // publish tile t+1 (its keys are multiplied during this step), then refill the ring: stage
        // (t+3)%5 held tile t-2, which nobody reads any more after this barrier (the values of tile t-1
        // are still multiplied in this step)
        if (t + 1 < n_tiles) {
            if (t + 2 < n_tiles) { SPTS_WAIT_VMCNT(PER); } else { SPTS_WAIT_VMCNT(0); }
        }
        __syncthreads();
        if (t + 3 < n_tiles) SPTS_ATT_DMA(t + 3)
        SPTS_ATT_BLOCK(2 * t, sa, sb, pfa, pfb)
        SPTS_ATT_BLOCK(2 * t + 1, sb, sa, pfb, pfa)
    }
    // the slot after the last block of a wavefront that worked through the last tile
    if (n_tiles > 0) SPTS_ATT_BLOCK(2 * n_tiles, sa, sb, pfa, pfb)

    // ---- normalise and store.  A lane holds 4 consecutive value columns of its query per r/4, i.e. a store from the
    //      fragment layout would carry 16-byte pieces of 32 rows per instruction; the wavefront's 32 x D tile goes
    //      through LDS instead (the ring is free once every wavefront is past its last fragment read; a wavefront
    //      uses its own 32 * D * 2 bytes) and leaves as whole lines.  Chunk c (16 bytes) of row r sits at c ^ (r % NCH).
    static_assert(QB == 1, "one 32-query block per wavefront");
    constexpr int NCH = D / 8;                       // 16-byte chunks per row
    bf16_t* O = (bf16_t*)a.out;
    __syncthreads();
    char* stg = smem + (size_t)wave * (32 * D * 2);
    {
        const float l = l_run[0] + __shfl_xor(l_run[0], 32);
        const float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                u32x2 w = {pk2(o[db][0][4 * q4] * inv, o[db][0][4 * q4 + 1] * inv),
                           pk2(o[db][0][4 * q4 + 2] * inv, o[db][0][4 * q4 + 3] * inv)};
                *reinterpret_cast<u32x2*>(stg + l32 * (D * 2) + ((((db * 4 + q4) ^ l32) & (NCH - 1)) << 4) + lh * 8) = w;
            }
    }
    __syncthreads();
    if (a.out_slab) {
        // slab h*D/32 + sl holds 32 columns of every row: 4 lanes per row, 16 rows = 1 KB contiguous per instruction
        const int c4 = lane & 3;
#pragma unroll
        for (int sl = 0; sl < DB; ++sl)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int r = p * 16 + (lane >> 2);
                const int64_t qi = q0w + r;
                if (qi < a.Mq) {
                    const u32x4 v = *reinterpret_cast<const u32x4*>(stg + r * (D * 2) + ((((sl * 4 + c4) ^ r) & (NCH - 1)) << 4));
                    *reinterpret_cast<u32x4*>(O + (((int64_t)h * DB + sl) * a.Mq + qi) * 32 + c4 * 8) = v;
                }
            }
    } else {
        // row-major: NCH lanes per row write this head's D columns of it
        constexpr int RPP = 64 / NCH;                // rows per pass
        const int c = lane % NCH;
#pragma unroll
        for (int p = 0; p < 32 / RPP; ++p) {
            const int r = p * RPP + lane / NCH;
            const int64_t qi = q0w + r;
            if (qi < a.Mq) {
                const u32x4 v = *reinterpret_cast<const u32x4*>(stg + r * (D * 2) + (((c ^ r) & (NCH - 1)) << 4));
                *reinterpret_cast<u32x4*>(O + (qi * a.H + h) * (int64_t)D + c * 8) = v;
            }
        }
    }
}

float attention_mfma_q_scale(int d) { return 1.4426950408889634f / sqrtf((float)d); }

bool attention_mfma_supported(const AttnArgs& a) {
    if (a.d != 128 && a.d != 64) return false;
    if (a.Mq <= 0 || a.Mk <= 0 || a.H % a.Hkv != 0) return false;
    if (!a.vt || a.ldvt % BKV != 0 || a.ldvt < (a.Mk + BKV - 1) / BKV * BKV) return false;
    if (a.ldvt * (int64_t)a.d * 2 >= ((int64_t)1 << 32)) return false;   // a lane's offset inside a kv head's V^T rows is 32-bit
    auto al = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    return al(a.q) && al(a.k) && al(a.vt) && al(a.out);
}

template <int D, int HPW, int NW>
static hipError_t launch_attn_t(const AttnArgs& a, hipStream_t s) {
    constexpr int BQ = NW / HPW * 32;
    const int nQ = (int)((a.Mq + BQ - 1) / BQ);
    const int grp = a.H / a.Hkv;
    const int ngh = grp / HPW;
    const int total = nQ * a.Hkv * ngh;
    // XCDs per kv head when the kv heads are fewer than the XCDs and divide them; 1 = contiguous split of all items
    const int xpg = (a.Hkv < 8 && 8 % a.Hkv == 0) ? 8 / a.Hkv : 1;
    const int grid = xpg > 1 ? 8 * ((nQ * ngh + xpg - 1) / xpg) : (total + 7) / 8 * 8;
    const size_t lds = (size_t)AttnLds<D>::STAGE * ATT_NST;
    {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&attn_mfma_kernel<D, HPW, NW>), (int)lds);
        if (e != hipSuccess) return e;
    }
    const float want = attention_mfma_q_scale(D);
    const float qmul = (a.q_scale != 0.f) ? want / a.q_scale : want;   // exactly 1 when the producer applied `want`
    attn_mfma_kernel<D, HPW, NW><<<dim3(grid), dim3(NW * 64), lds, s>>>(a, nQ, total, xpg, qmul);
    return hipGetLastError();
}

#ifndef SPTS_ATT_HPW_MAX
#define SPTS_ATT_HPW_MAX 4
#endif

template <int D>
static hipError_t launch_attn_d(const AttnArgs& a, hipStream_t s) {
    // as many heads of a kv-head group per workgroup as divide the group (4, 2 or 1)
    const int grp = a.H / a.Hkv;
    if (SPTS_ATT_HPW_MAX >= 4 && grp % 4 == 0) return launch_attn_t<D, 4, 8>(a, s);
    if (SPTS_ATT_HPW_MAX >= 2 && grp % 2 == 0) return launch_attn_t<D, 2, 8>(a, s);
    return launch_attn_t<D, 1, 8>(a, s);
}

hipError_t launch_attention_mfma(const AttnArgs& a, hipStream_t s) {
    if (a.d == 128) return launch_attn_d<128>(a, s);
    return launch_attn_d<64>(a, s);
}

}  // namespace spts
