// Flash-style causal GQA prefill attention on the matrix cores (bf16 in, fp32 softmax/accumulate).
//
// out[i, h, :] = softmax_j( q[i,h].k[j,g(h)] / sqrt(d)  for kpos[j] <= qpos[i] ) . v[j, g(h), :]
// The query set and the key set carry their own ascending absolute positions, so the same kernel
// serves the reduced attention over the active tokens of Alg. 1 (queries = keys = active set), the
// dense branch, and queries = active / keys = all candidates.
//
// Layout of the computation (gfx950, wave64, MFMA 32x32x16 bf16):
//  * S^T = K Q^T is computed instead of S: the MFMA result then has one query per lane column, so
//    the row maximum / row sum of the online softmax are in-lane reductions plus one exchange with
//    lane^32, and the probabilities already sit in the operand layout of the second product.
//  * O^T += V^T P^T takes V^T tiles (keys contiguous) as the A operand: the value projection writes
//    that transposed copy, so no transposition happens here.  The key index permutation implied by
//    the accumulator layout is applied to the V^T fragment addresses (a sum over keys is order-free).
//  * One workgroup = 4 wavefronts x (QB*32) queries of one head; K / V^T tiles of 64 keys are shared
//    through LDS (XOR-swizzled, conflict-free fragment reads), global->register prefetch of the next
//    tile overlaps the MFMAs, two LDS stages, one barrier per tile.
//  * Key tiles beyond the last visible position are never visited (binary search on kpos); tiles
//    that are entirely visible skip the mask; a wavefront whose queries see nothing of a tile skips
//    its MFMAs.
//  * Work ids are laid out (kv head, query tile descending, head in group) and split contiguously
//    over the 8 XCDs: the heads that share a KV head run on the same XCD's L2, longest tiles first.
#include "spts_internal.h"

namespace spts {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BKV = 64;

template <int D> struct AttnLds {
    static constexpr int K_BYTES = BKV * D * 2;
    static constexpr int V_BYTES = D * BKV * 2;
    static constexpr int STAGE = K_BYTES + V_BYTES + BKV * 4;
    static constexpr int CPRK = D / 8;            // 16-byte chunks per K row
    static constexpr int RPK = 256 / (2 * D);     // K rows per 256 bytes
    __device__ static inline int koff(int row, int c) { return row * (2 * D) + ((c ^ ((row / RPK) % CPRK)) << 4); }
    // V^T tile: row = value column, 16 chunks of 8 bytes (4 keys)
    __device__ static inline int voff(int row, int c8) { return row * (BKV * 2) + ((c8 ^ ((row >> 1) & 15)) << 3); }
};

__device__ inline uint32_t pk2(float a, float b) { return cvt_pk_bf16(a, b); }

template <int D, int QB>
__global__ void __launch_bounds__(256) attn_mfma_kernel(AttnArgs a, int nQ, int total, float scale_log2e) {
    using L = AttnLds<D>;
    constexpr int BQ = 4 * QB * 32;
    constexpr int KS = D / 16;   // k-steps of the QK^T product
    constexpr int DB = D / 32;   // 32-column blocks of the output
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int per = (total + 7) / 8;
    const int id = (int)(blockIdx.x % 8) * per + (int)(blockIdx.x / 8);
    if (id >= total) return;
    const int grp = a.H / a.Hkv;
    const int hg = id % grp;
    const int qtile = nQ - 1 - (id / grp) % nQ;
    const int g = id / (grp * nQ);
    const int h = g * grp + hg;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int64_t q0 = (int64_t)qtile * BQ;
    const int64_t q0w = q0 + wave * (QB * 32);

    // ---- visible key range of this workgroup / wavefront
    const int64_t q_last = (q0 + BQ < a.Mq ? q0 + BQ : a.Mq) - 1;
    const int qpos_max = a.qpos[q_last];
    int64_t lo = 0, hi = a.Mk;  // first index with kpos > qpos_max
    while (lo < hi) {
        int64_t mid = (lo + hi) >> 1;
        if (a.kpos[mid] <= qpos_max) lo = mid + 1; else hi = mid;
    }
    const int n_tiles = (int)((lo + BKV - 1) / BKV);
    const int64_t qw_first = q0w < a.Mq ? q0w : a.Mq - 1;
    const int64_t qw_last = (q0w + QB * 32 < a.Mq ? q0w + QB * 32 : a.Mq) - 1;
    const int qmin_w = a.qpos[qw_first];
    const int qmax_w = a.qpos[qw_last > qw_first ? qw_last : qw_first];

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
    }

    // ---- global -> register staging of one K tile and one V^T tile
    constexpr int KCH = BKV * L::CPRK / 256;   // 16-byte chunks per thread (K)
    constexpr int VCH = D * 8 / 256;           // 16-byte chunks per thread (V^T)
    const int kc = tid % L::CPRK, kr = tid / L::CPRK;
    const int vc = tid % 8, vr = tid / 8;
    const bf16_t* Kg = (const bf16_t*)a.k;
    const bf16_t* Vt = (const bf16_t*)a.vt;
    u32x4 rk[KCH], rv[VCH];
    int rpos = 0;
    auto load_tile = [&](int t) {
        const int64_t key0 = (int64_t)t * BKV;
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            int64_t key = key0 + kr + (256 / L::CPRK) * i;
            if (key >= a.Mk) key = a.Mk - 1;
            rk[i] = *reinterpret_cast<const u32x4*>(Kg + (key * a.Hkv + g) * (int64_t)D + kc * 8);
        }
#pragma unroll
        for (int i = 0; i < VCH; ++i) {
            int row = vr + 32 * i;
            rv[i] = *reinterpret_cast<const u32x4*>(Vt + ((int64_t)g * D + row) * a.ldvt + key0 + vc * 8);
        }
        if (tid < BKV) { int64_t key = key0 + tid; rpos = key < a.Mk ? a.kpos[key] : 0x7fffffff; }
    };
    auto store_tile = [&](int stage) {
        char* sK = smem + stage * L::STAGE;
        char* sV = sK + L::K_BYTES;
        int* sP = reinterpret_cast<int*>(sV + L::V_BYTES);
#pragma unroll
        for (int i = 0; i < KCH; ++i) *reinterpret_cast<u32x4*>(sK + L::koff(kr + (256 / L::CPRK) * i, kc)) = rk[i];
#pragma unroll
        for (int i = 0; i < VCH; ++i) {
            int row = vr + 32 * i;
            *reinterpret_cast<u32x2*>(sV + L::voff(row, 2 * vc)) = u32x2{rv[i].x, rv[i].y};
            *reinterpret_cast<u32x2*>(sV + L::voff(row, 2 * vc + 1)) = u32x2{rv[i].z, rv[i].w};
        }
        if (tid < BKV) sP[tid] = rpos;
    };

    f32x16 o[DB][QB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][qb][r] = 0.f;
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.f; }

    if (n_tiles > 0) { load_tile(0); store_tile(0); }
    __syncthreads();
    for (int t = 0; t < n_tiles; ++t) {
        if (t + 1 < n_tiles) load_tile(t + 1);
        const char* sK = smem + (t & 1) * L::STAGE;
        const char* sV = sK + L::K_BYTES;
        const int* sP = reinterpret_cast<const int*>(sV + L::V_BYTES);
        const int kfirst = sP[0], klast = sP[BKV - 1];
        if (kfirst <= qmax_w) {   // wavefront-uniform: some query of this wavefront sees this tile
            // ---- S^T = K Q^T   (2 key blocks x QB query blocks)
            f32x16 s[2][QB];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[kb][qb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    bf16x8 kf = *reinterpret_cast<const bf16x8*>(sK + L::koff(kb * 32 + l32, 2 * ks + lh));
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        s[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][ks], s[kb][qb], 0, 0, 0);
                }
            }
            // ---- mask (only on tiles that are not entirely visible to this wavefront); logits stay
            //      unscaled: the softmax scale is folded into the exponent's FMA
            const bool need_mask = klast > qmin_w;
            if (need_mask) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const int4 kp = *reinterpret_cast<const int4*>(sP + kb * 32 + 8 * q4 + 4 * lh);
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb) {
                            const int qp = qpos_l[qb];
                            if (kp.x > qp) s[kb][qb][4 * q4] = -INFINITY;
                            if (kp.y > qp) s[kb][qb][4 * q4 + 1] = -INFINITY;
                            if (kp.z > qp) s[kb][qb][4 * q4 + 2] = -INFINITY;
                            if (kp.w > qp) s[kb][qb][4 * q4 + 3] = -INFINITY;
                        }
                    }
            }
            // ---- online softmax per query (lane column; lanes l and l^32 share a query)
            bf16x8 pf[QB][4];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                float mx = -INFINITY;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][qb][r]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_old = m_run[qb];
                const float m_new = fmaxf(m_old, mx);
                const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
                const float msc = m_use * scale_log2e;
                m_run[qb] = m_new;
                float sum = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf) {
                        float p[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][qb][8 * hf + e], scale_log2e, -msc));
                            sum += p[e];
                        }
                        u32x4 packed = {pk2(p[0], p[1]), pk2(p[2], p[3]), pk2(p[4], p[5]), pk2(p[6], p[7])};
                        pf[qb][2 * kb + hf] = __builtin_bit_cast(bf16x8, packed);
                    }
                // the running maximum rarely moves after the first tiles: rescale only when some lane needs it
                if (__ballot(m_new != m_old) != 0) {
                    const float alpha = __builtin_amdgcn_exp2f((m_old - m_use) * scale_log2e);
                    l_run[qb] *= alpha;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o[db][qb][r] *= alpha;
                }
                l_run[qb] += sum;
            }
            // ---- O^T += V^T P^T
#pragma unroll
            for (int st = 0; st < 4; ++st) {
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    u32x2 v0 = *reinterpret_cast<const u32x2*>(sV + L::voff(db * 32 + l32, 4 * st + lh));
                    u32x2 v1 = *reinterpret_cast<const u32x2*>(sV + L::voff(db * 32 + l32, 4 * st + 2 + lh));
                    u32x4 vv = {v0.x, v0.y, v1.x, v1.y};
                    bf16x8 vf = __builtin_bit_cast(bf16x8, vv);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qb][st], o[db][qb], 0, 0, 0);
                }
            }
        }
        if (t + 1 < n_tiles) store_tile((t + 1) & 1);
        __syncthreads();
    }

    // ---- normalise and store: lane holds 4 consecutive value columns of its query per r/4
    bf16_t* O = (bf16_t*)a.out;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        float l = l_run[qb] + __shfl_xor(l_run[qb], 32);
        float inv = l > 0.f ? 1.0f / l : 0.f;
        int64_t qi = q0w + qb * 32 + l32;
        if (qi < a.Mq) {
            bf16_t* orow = O + (qi * a.H + h) * (int64_t)D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    uint2 w;
                    w.x = pk2(o[db][qb][4 * q4] * inv, o[db][qb][4 * q4 + 1] * inv);
                    w.y = pk2(o[db][qb][4 * q4 + 2] * inv, o[db][qb][4 * q4 + 3] * inv);
                    *reinterpret_cast<uint2*>(orow + db * 32 + 8 * q4 + 4 * lh) = w;
                }
        }
    }
}

bool attention_mfma_supported(const AttnArgs& a) {
    if (a.d != 128 && a.d != 64) return false;
    if (a.Mq <= 0 || a.Mk <= 0 || a.H % a.Hkv != 0) return false;
    if (!a.vt || a.ldvt % BKV != 0 || a.ldvt < (a.Mk + BKV - 1) / BKV * BKV) return false;
    auto al = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    return al(a.q) && al(a.k) && al(a.vt) && al(a.out);
}

template <int D, int QB>
static hipError_t launch_attn_t(const AttnArgs& a, hipStream_t s) {
    constexpr int BQ = 4 * QB * 32;
    const int nQ = (int)((a.Mq + BQ - 1) / BQ);
    const int total = nQ * a.H;
    const int grid = (total + 7) / 8 * 8;
    const size_t lds = (size_t)AttnLds<D>::STAGE * 2;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_kernel<D, QB>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
    attn_mfma_kernel<D, QB><<<dim3(grid), dim3(256), lds, s>>>(a, nQ, total, scale_log2e);
    return hipGetLastError();
}

hipError_t launch_attention_mfma(const AttnArgs& a, hipStream_t s) {
    if (a.d == 128) return launch_attn_t<128, 2>(a, s);
    return launch_attn_t<64, 2>(a, s);
}

}  // namespace spts
