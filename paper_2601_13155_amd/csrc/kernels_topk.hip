// TopK(S, k): the k largest scores under (score descending, index ascending), written in ascending
// index order (Sec. 3.2 TopK; Eq. (ffn_selection); Eq. (stage_prune)).
//
// Design for gfx950: N <= 2^17..2^20 fp32 scores are 0.5-4 MB, i.e. L2-resident and latency-bound, so
// one workgroup of 1024 lanes (16 wavefronts) owns the whole problem and never leaves the CU:
//   1. MSB-first radix select on order-preserving 32-bit keys, 4 passes of 8 bits, with a 256-bin
//      LDS histogram per pass (integer LDS atomics: order-independent, hence deterministic) -> the
//      exact key T of the k-th largest element, the number of keys above it, and how many keys equal
//      to T are still needed (those are taken lowest index first: the tie rule).
//   2. Ordered stream compaction without a per-chunk workgroup barrier: every wavefront owns one
//      contiguous slice; a first sweep counts its (greater, equal) elements with ballots, a 16-entry
//      LDS prefix gives each wavefront its output offsets, a second sweep ranks every element inside
//      the wavefront with ballot + mbcnt (lane prefix popcount) and writes
//      out[gt_before + min(eq_before, need_eq)].
#include "spts_internal.h"

namespace spts {

constexpr int TOPK_THREADS = 1024;
constexpr int TOPK_WAVES = TOPK_THREADS / 64;

__device__ inline uint32_t order_key(float f) {
    f = f + 0.0f;  // -0.0 -> +0.0
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ inline uint32_t load_key(const float* __restrict__ s, int64_t i, int64_t N, int protect_last) {
    uint32_t key = order_key(s[i]);
    if (protect_last && i == N - 1) key = 0xFFFFFFFFu;
    return key;
}

__device__ inline int lane_prefix_popc(uint64_t mask) {
    // number of set bits below this lane
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

__global__ void __launch_bounds__(TOPK_THREADS) topk_kernel(const float* __restrict__ scores, int64_t N, int64_t k,
                                                            int protect_last, int32_t* __restrict__ idx_out) {
    __shared__ int hist[256];
    __shared__ uint32_t sh_prefix;     // key bits decided so far
    __shared__ int64_t sh_need;        // how many elements are still to be taken inside the current bucket
    __shared__ int64_t wave_gt[TOPK_WAVES], wave_eq[TOPK_WAVES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;

    if (tid == 0) { sh_prefix = 0; sh_need = k; }
    uint32_t prefix = 0;
    int64_t need = k;

    // ---- 1. radix select
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        const uint32_t hi_mask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int64_t i = tid; i < N; i += TOPK_THREADS) {
            uint32_t key = load_key(scores, i, N, protect_last);
            if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 0xFF], 1);
        }
        __syncthreads();
        if (wave == 0) {
            // bins in descending order: lane l owns bins 255-4l .. 252-4l
            int c0 = hist[255 - 4 * lane], c1 = hist[254 - 4 * lane], c2 = hist[253 - 4 * lane], c3 = hist[252 - 4 * lane];
            int64_t tot = (int64_t)c0 + c1 + c2 + c3;
            int64_t incl = tot;
            for (int off = 1; off < 64; off <<= 1) {
                int64_t o = __shfl_up(incl, off);
                if (lane >= off) incl += o;
            }
            int64_t excl = incl - tot;  // elements in bins above this lane's bins
            if (excl < need && need <= incl) {
                int64_t rem = need - excl;
                int bin;
                if (rem <= c0) { bin = 255 - 4 * lane; }
                else if (rem <= (int64_t)c0 + c1) { bin = 254 - 4 * lane; rem -= c0; }
                else if (rem <= (int64_t)c0 + c1 + c2) { bin = 253 - 4 * lane; rem -= (int64_t)c0 + c1; }
                else { bin = 252 - 4 * lane; rem -= (int64_t)c0 + c1 + c2; }
                sh_prefix = prefix | ((uint32_t)bin << shift);
                sh_need = rem;
            }
        }
        __syncthreads();
        prefix = sh_prefix;
        need = sh_need;
    }
    const uint32_t T = prefix;     // key of the k-th largest element
    const int64_t need_eq = need;  // elements equal to T to take (lowest indices first), >= 1

    // ---- 2. ordered compaction, one contiguous slice per wavefront (slice length multiple of 64)
    int64_t per_wave = ((N + TOPK_WAVES - 1) / TOPK_WAVES + 63) / 64 * 64;
    int64_t lo = (int64_t)wave * per_wave;
    int64_t hi = lo + per_wave < N ? lo + per_wave : N;
    int64_t cgt = 0, ceq = 0;
    for (int64_t base = lo; base < hi; base += 64) {
        int64_t i = base + lane;
        bool gt = false, eq = false;
        if (i < hi) { uint32_t key = load_key(scores, i, N, protect_last); gt = key > T; eq = key == T; }
        cgt += __popcll(__ballot(gt));
        ceq += __popcll(__ballot(eq));
    }
    if (lane == 0) { wave_gt[wave] = cgt; wave_eq[wave] = ceq; }
    __syncthreads();
    int64_t gt_before = 0, eq_before = 0;
    for (int w = 0; w < wave; ++w) { gt_before += wave_gt[w]; eq_before += wave_eq[w]; }
    for (int64_t base = lo; base < hi; base += 64) {
        int64_t i = base + lane;
        bool gt = false, eq = false;
        if (i < hi) { uint32_t key = load_key(scores, i, N, protect_last); gt = key > T; eq = key == T; }
        uint64_t mgt = __ballot(gt), meq = __ballot(eq);
        int64_t my_gt = gt_before + lane_prefix_popc(mgt);
        int64_t my_eq = eq_before + lane_prefix_popc(meq);
        if (gt || (eq && my_eq < need_eq)) {
            int64_t o = my_gt + (my_eq < need_eq ? my_eq : need_eq);
            idx_out[o] = (int32_t)i;
        }
        gt_before += __popcll(mgt);
        eq_before += __popcll(meq);
    }
}

hipError_t launch_topk(const float* scores, int64_t N, int64_t k, int protect_last, int32_t* idx_out, int32_t* scratch,
                       hipStream_t s) {
    (void)scratch;
    if (k <= 0 || N <= 0) return hipSuccess;
    topk_kernel<<<dim3(1), dim3(TOPK_THREADS), 0, s>>>(scores, N, k, protect_last, idx_out);
    return hipGetLastError();
}

}  // namespace spts
