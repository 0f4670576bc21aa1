// TopK(S, k): the k largest scores under (score descending, index ascending), written in ascending
// index order (Sec. 3.2 TopK; Eq. (ffn_selection); Eq. (stage_prune)).
//
// Design for gfx950: N <= 2^17..2^20 fp32 scores are 0.5-4 MB, i.e. L2-resident and latency-bound, so
// one workgroup of 1024 lanes (16 wavefronts) owns the whole problem and never leaves the CU:
//   1. MSB-first radix select on order-preserving 32-bit keys, 4 passes of 8 bits, with a 256-bin
//      LDS histogram per pass (integer LDS atomics: order-independent, hence deterministic) -> the
//      exact key T of the k-th largest element, the number of keys above it, and how many keys equal
//      to T are still needed (those are taken lowest index first: the tie rule).
//      Scores of one layer are probabilities of similar magnitude, so almost all keys share their
//      top bits and fall into one or two bins: lanes whose bin equals that of the wavefront's first
//      active lane are counted with one ballot and a single atomic instead of 64 serialised ones.
//   2. Ordered stream compaction without a per-chunk workgroup barrier: every wavefront owns one
//      contiguous slice; a first sweep counts its (greater, equal) elements with ballots, a 16-entry
//      LDS prefix gives each wavefront its output offsets, a second sweep ranks every element inside
//      the wavefront with ballot + mbcnt (lane prefix popcount) and writes
//      out[gt_before + min(eq_before, need_eq)].
// Up to 32768 scores the keys are read once and stay in registers (KPT per lane, wavefront w holding
// the contiguous slice [64*KPT*w, 64*KPT*(w+1))); longer inputs re-read the scores in every sweep.
// Shortcut for step 1 (register-resident and long-row kernels): one pass builds an 8192-bin histogram
// of the top 13 key bits, the keys of the bin that holds the k-th largest go to LDS and the remaining
// 19 bits are resolved there; the four 8-bit passes over all keys remain as the route for rows whose
// threshold bin does not fit (heavily tied scores).  Both routes yield the same exact threshold.
#include "spts_internal.h"

#include <mutex>

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

// hist[bin] += 1 for every active lane.  Lanes that share the bin of the first active lane are
// counted by that lane alone (one atomic for the whole group); the others add for themselves.
__device__ inline void hist_add(int* hist, bool active, int bin) {
    const uint64_t act = __ballot(active);
    if (act == 0) return;
    const int first = __builtin_ctzll(act);
    const int lead = __builtin_amdgcn_readlane(bin, first);
    const bool same = active && bin == lead;
    const uint64_t m = __ballot(same);
    const int lane = threadIdx.x & 63;
    if (lane == first) atomicAdd(&hist[lead], (int)__popcll(m));
    else if (active && !same) atomicAdd(&hist[bin], 1);
}

// wavefront 0: from the 256-bin histogram and the rank `need` still wanted, the bin that holds the
// need-th largest element of the current bucket; updates (prefix, need) in LDS
__device__ inline void pick_bin(const int* hist, int lane, int shift, uint32_t prefix, int64_t need, uint32_t* sh_prefix,
                                int64_t* sh_need) {
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
        *sh_prefix = prefix | ((uint32_t)bin << shift);
        *sh_need = rem;
    }
}

// ---- the threshold bin resolved in LDS (used by the register-resident and the long-row kernels) -------------------
// A first histogram over the keys' top 13 bits (sign, exponent, four mantissa bits: a bin is 4.4 % wide in value) finds the
// bin of the k-th largest key; every wavefront then copies the low 19 bits of ITS keys of that bin into its own LDS
// region, and three radix passes over those few keys (8 + 8 + 3 bits) give the exact threshold, the number of keys equal
// to it that are still wanted, and each wavefront's (greater, equal) counts.  A wavefront whose share of the bin does not
// fit its region (heavily tied scores) makes the caller fall back to 8-bit passes over all keys.
constexpr int T13_BINS = 8192;
constexpr int T13_LOW = 19;
constexpr int T13_CW = 768;                                              // keys per wavefront region
constexpr int T13_LDS_BYTES = T13_BINS * 4 + TOPK_WAVES * T13_CW * 4;    // 80 KB: two workgroups per CU

// all 1024 lanes: from the 8192-bin histogram the bin that holds the k-th largest key (-> *sh_bin) and the rank wanted
// inside it (-> *sh_need); ends with a barrier
__device__ inline void t13_pick(const int* h13, int64_t k, int* wave_tot, int* sh_bin, int64_t* sh_need) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int BPT = T13_BINS / TOPK_THREADS;   // bins per lane, descending
    int c[BPT], tot = 0;
#pragma unroll
    for (int q = 0; q < BPT; ++q) { c[q] = h13[T13_BINS - 1 - BPT * tid - q]; tot += c[q]; }
    int incl = tot;
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int64_t excl = incl - tot;
    for (int w = 0; w < wave; ++w) excl += wave_tot[w];
    if (excl < k && k <= excl + tot) {
        int64_t rem = k - excl;
        int q = 0;
#pragma unroll
        for (int t = 0; t < BPT - 1; ++t)
            if (q == t && rem > c[t]) { rem -= c[t]; q = t + 1; }
        *sh_bin = T13_BINS - 1 - BPT * tid - q;
        *sh_need = rem;
    }
    __syncthreads();
}

// all 1024 lanes: cand[0 .. cnt) = low 19 bits of this wavefront's keys of the bin, `need` = rank wanted inside the bin.
// Returns the low 19 bits of the threshold; *need_eq = keys equal to it still wanted; *g / *e = this wavefront's
// candidates above / equal to it.
__device__ inline uint32_t t13_resolve(const uint32_t* cand, int cnt, int64_t need, int* hist, uint32_t* sh_prefix,
                                       int64_t* sh_need, int* need_eq, int* g, int* e) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t prefix = 0;
    const int cnt64 = (cnt + 63) & ~63;
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 11 : pass == 1 ? 3 : 0;
        const uint32_t dmask = pass == 2 ? 0x7u : 0xFFu;
        const uint32_t hi_mask = pass == 0 ? 0u : pass == 1 ? 0x7F800u : 0x7FFF8u;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int j = lane; j < cnt64; j += 64) {
            const uint32_t c = j < cnt ? cand[j] : 0u;
            hist_add(hist, j < cnt && (c & hi_mask) == prefix, (int)((c >> shift) & dmask));
        }
        __syncthreads();
        if (wave == 0) pick_bin(hist, lane, shift, prefix, need, sh_prefix, sh_need);
        __syncthreads();
        prefix = *sh_prefix;
        need = *sh_need;
    }
    *need_eq = (int)need;
    int gg = 0, ee = 0;
    for (int j = lane; j < cnt64; j += 64) {
        const uint32_t c = j < cnt ? cand[j] : 0u;
        gg += (int)__popcll(__ballot(j < cnt && c > prefix));
        ee += (int)__popcll(__ballot(j < cnt && c == prefix));
    }
    *g = gg; *e = ee;
    return prefix;
}

// Register-resident variant: N <= 1024 * KPT.  Lane keeps keys[j] = key of element lo + 64*j + lane,
// lo = 64*KPT*wave; slots at or beyond N hold key 0 and are never written out.
template <int KPT>
__global__ void __launch_bounds__(TOPK_THREADS) topk_reg_kernel(const float* __restrict__ scores, int64_t N, int64_t k,
                                                                int protect_last, int32_t* __restrict__ idx_out, TopkSegments seg) {
    extern __shared__ __attribute__((aligned(16))) char lsm[];
    int* h13 = reinterpret_cast<int*>(lsm);                                                   // [T13_BINS]
    uint32_t (*cand)[T13_CW] = reinterpret_cast<uint32_t (*)[T13_CW]>(lsm + T13_BINS * 4);   // [TOPK_WAVES][T13_CW]
    __shared__ int hist[256];
    __shared__ uint32_t sh_prefix;
    __shared__ int64_t sh_need;
    __shared__ int wave_gt[TOPK_WAVES], wave_eq[TOPK_WAVES], wave_tot[TOPK_WAVES];
    __shared__ int sh_bin, sh_over;

    // one independent problem per workgroup: equal rows, or the segment the descriptors give it
    if (seg.offsets) {
        const int64_t b0 = seg.offsets[blockIdx.x];
        N = seg.offsets[blockIdx.x + 1] - b0;
        k = seg.k[blockIdx.x];
        scores += b0;
        idx_out += seg.out_offsets[blockIdx.x];
        if (k > N) k = N;
        if (k <= 0 || N <= 0) return;
    } else {
        scores += (int64_t)blockIdx.x * N;
        idx_out += (int64_t)blockIdx.x * k;
    }
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lo = wave * (64 * KPT);

    uint32_t keys[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const int64_t i = lo + 64 * j + lane;
        keys[j] = i < N ? load_key(scores, i, N, protect_last) : 0u;
    }

    // one pass over the keys for their top 13 bits, the rest of the threshold from the bin's keys in LDS
    uint32_t T = 0;
    int need_eq = 0;
    for (int i = tid; i < T13_BINS; i += TOPK_THREADS) h13[i] = 0;
    if (tid == 0) { sh_over = 0; sh_bin = 0; sh_need = k; }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < KPT; ++j) hist_add(h13, lo + 64 * j + lane < N, (int)(keys[j] >> T13_LOW));
    __syncthreads();
    t13_pick(h13, k, wave_tot, &sh_bin, &sh_need);
    const uint32_t bin = (uint32_t)sh_bin;
    int cnt = 0, cgt = 0;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const bool valid = lo + 64 * j + lane < N;
        const uint32_t top = keys[j] >> T13_LOW;
        cgt += (int)__popcll(__ballot(valid && top > bin));
        const bool in = valid && top == bin;
        const uint64_t m = __ballot(in);
        const int at = cnt + lane_prefix_popc(m);
        if (in && at < T13_CW) cand[wave][at] = keys[j] & ((1u << T13_LOW) - 1u);
        cnt += (int)__popcll(m);
    }
    if (lane == 0 && cnt > T13_CW) sh_over = 1;
    __syncthreads();
    if (sh_over == 0) {
        int g, e;
        const uint32_t low = t13_resolve(cand[wave], cnt, sh_need, hist, &sh_prefix, &sh_need, &need_eq, &g, &e);
        T = (bin << T13_LOW) | low;
        if (lane == 0) { wave_gt[wave] = cgt + g; wave_eq[wave] = e; }
    } else {
        // heavily tied keys: four 8-bit passes over the registers
        if (tid == 0) { sh_prefix = 0; sh_need = k; }
        uint32_t prefix = 0;
        int64_t need = k;
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            const uint32_t hi_mask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
#pragma unroll
            for (int j = 0; j < KPT; ++j) {
                const bool valid = lo + 64 * j + lane < N;
                hist_add(hist, valid && (keys[j] & hi_mask) == prefix, (int)((keys[j] >> shift) & 0xFF));
            }
            __syncthreads();
            if (wave == 0) pick_bin(hist, lane, shift, prefix, need, &sh_prefix, &sh_need);
            __syncthreads();
            prefix = sh_prefix;
            need = sh_need;
        }
        T = prefix;
        need_eq = (int)need;
        int ceq = 0;
        cgt = 0;
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const bool valid = lo + 64 * j + lane < N;
            cgt += (int)__popcll(__ballot(valid && keys[j] > T));
            ceq += (int)__popcll(__ballot(valid && keys[j] == T));
        }
        if (lane == 0) { wave_gt[wave] = cgt; wave_eq[wave] = ceq; }
    }
    __syncthreads();
    int gt_before = 0, eq_before = 0;
    for (int w = 0; w < wave; ++w) { gt_before += wave_gt[w]; eq_before += wave_eq[w]; }
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const int i = lo + 64 * j + lane;
        const bool valid = i < N;
        const bool gt = valid && keys[j] > T, eq = valid && keys[j] == T;
        const uint64_t mgt = __ballot(gt), meq = __ballot(eq);
        const int my_gt = gt_before + lane_prefix_popc(mgt);
        const int my_eq = eq_before + lane_prefix_popc(meq);
        if (gt || (eq && my_eq < need_eq)) idx_out[my_gt + (my_eq < need_eq ? my_eq : need_eq)] = i;
        gt_before += (int)__popcll(mgt);
        eq_before += (int)__popcll(meq);
    }
}

__global__ void __launch_bounds__(TOPK_THREADS) topk_kernel(const float* __restrict__ scores, int64_t N, int64_t k,
                                                            int protect_last, int32_t* __restrict__ idx_out, TopkSegments seg) {
    __shared__ int hist[256];
    __shared__ uint32_t sh_prefix;     // key bits decided so far
    __shared__ int64_t sh_need;        // how many elements are still to be taken inside the current bucket
    __shared__ int64_t wave_gt[TOPK_WAVES], wave_eq[TOPK_WAVES];

    // one independent problem per workgroup: equal rows, or the segment the descriptors give it
    if (seg.offsets) {
        const int64_t b0 = seg.offsets[blockIdx.x];
        N = seg.offsets[blockIdx.x + 1] - b0;
        k = seg.k[blockIdx.x];
        scores += b0;
        idx_out += seg.out_offsets[blockIdx.x];
        if (k > N) k = N;
        if (k <= 0 || N <= 0) return;
    } else {
        scores += (int64_t)blockIdx.x * N;
        idx_out += (int64_t)blockIdx.x * k;
    }
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
        // every lane runs the same number of rounds (hist_add uses wavefront-wide ballots)
        for (int64_t base = 0; base < N; base += TOPK_THREADS) {
            const int64_t i = base + tid;
            uint32_t key = i < N ? load_key(scores, i, N, protect_last) : 0u;
            hist_add(hist, i < N && (key & hi_mask) == prefix, (int)((key >> shift) & 0xFF));
        }
        __syncthreads();
        if (wave == 0) pick_bin(hist, lane, shift, prefix, need, &sh_prefix, &sh_need);
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

// Long rows of a batch (N > 32768, N % 4 == 0, equal rows): one workgroup per row as above, but written for streaming.
// Every wavefront owns one contiguous slice in all sweeps and reads it as 16-byte loads, four per lane in flight (64 KB per
// workgroup).
// Three sweeps over the row in the usual case: (1) an 8192-bin histogram of the keys' top 13 bits (sign, exponent, four
// mantissa bits) finds the bin of the k-th largest key; (2) every wavefront copies the low 19 bits of its keys of that bin
// into its own LDS region and counts the keys of higher bins -- scores of one layer spread over several octaves, so the
// bin (4.4 % wide in value) holds a few percent of the row --, the remaining 19 bits are then resolved by three radix passes
// over LDS, which also leave each wavefront's (greater, equal) counts; (3) the ordered compaction.  If a wavefront's
// keys of the bin do not fit its region (heavily tied scores), the kernel falls back to four 8-bit passes over the row with
// histograms private to the wavefront, six sweeps in all; both routes end in the same exact (threshold, rank) pair.
typedef float f32x4v __attribute__((ext_vector_type(4)));
constexpr int LONG_U = 4;                       // 16-byte loads in flight per lane
constexpr int LONG_STEP = 64 * 4 * LONG_U;      // scores a wavefront takes per iteration

__global__ void __launch_bounds__(TOPK_THREADS) topk_long_kernel(const float* __restrict__ scores, int64_t N, int64_t k,
                                                                 int protect_last, int32_t* __restrict__ idx_out) {
    extern __shared__ __attribute__((aligned(16))) char lsm[];
    int* h13 = reinterpret_cast<int*>(lsm);                                                     // [T13_BINS]
    uint32_t (*cand)[T13_CW] = reinterpret_cast<uint32_t (*)[T13_CW]>(lsm + T13_BINS * 4);     // [TOPK_WAVES][T13_CW]
    int (*whist)[256] = reinterpret_cast<int (*)[256]>(lsm + T13_BINS * 4);                     // fallback only, same bytes
    __shared__ int hist[256];
    __shared__ uint32_t sh_prefix;
    __shared__ int64_t sh_need;
    __shared__ int wave_gt[TOPK_WAVES], wave_eq[TOPK_WAVES], wave_tot[TOPK_WAVES];
    __shared__ int sh_b12, sh_over;
    scores += (int64_t)blockIdx.x * N;
    idx_out += (int64_t)blockIdx.x * k;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = (int)N;
    const int per_wave = ((n + TOPK_WAVES - 1) / TOPK_WAVES + LONG_STEP - 1) / LONG_STEP * LONG_STEP;
    const int lo = wave * per_wave;
    const int hi = lo + per_wave < n ? lo + per_wave : n;   // n % 4 == 0, so a 16-byte load that starts below hi ends below it
    const uint32_t last_key_at = protect_last ? (uint32_t)(n - 1) : 0xFFFFFFFFu;

    // one iteration of a sweep over the wavefront's slice: the keys of load u, element e (index i0 + e) go to BODY
#define SPTS_LONG_SWEEP(BODY)                                                                              \
    for (int base = lo; base < hi; base += LONG_STEP) {                                                    \
        f32x4v v[LONG_U];                                                                                  \
        _Pragma("unroll") for (int u = 0; u < LONG_U; ++u) {                                               \
            const int i0 = base + u * 256 + lane * 4;                                                      \
            v[u] = i0 < hi ? *reinterpret_cast<const f32x4v*>(scores + i0) : f32x4v{0.f, 0.f, 0.f, 0.f};   \
        }                                                                                                  \
        _Pragma("unroll") for (int u = 0; u < LONG_U; ++u) {                                               \
            const int i0 = base + u * 256 + lane * 4;                                                      \
            const bool valid = i0 < hi;                                                                    \
            _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                                \
                uint32_t key = order_key(v[u][e]);                                                         \
                if ((uint32_t)(i0 + e) == last_key_at) key = 0xFFFFFFFFu;                                  \
                BODY                                                                                       \
            }                                                                                              \
        }                                                                                                  \
    }

    uint32_t T = 0;
    int need_eq = 0;
    // ---- sweep 1: top 13 bits
    for (int i = tid; i < T13_BINS; i += TOPK_THREADS) h13[i] = 0;
    if (tid == 0) { sh_over = 0; sh_b12 = 0; sh_need = k; }
    __syncthreads();
    SPTS_LONG_SWEEP({ hist_add(h13, valid, (int)(key >> T13_LOW)); })
    __syncthreads();
    t13_pick(h13, k, wave_tot, &sh_b12, &sh_need);
    const uint32_t b12 = (uint32_t)sh_b12;
    int64_t need = sh_need;
    // ---- sweep 2: the wavefront's keys of that bin into its LDS region (low 19 bits), keys of higher bins counted
    int cnt = 0, cgt = 0;
    SPTS_LONG_SWEEP({
        const uint32_t top = key >> T13_LOW;
        cgt += (int)__popcll(__ballot(valid && top > b12));
        const bool in = valid && top == b12;
        const uint64_t m = __ballot(in);
        const int at = cnt + lane_prefix_popc(m);
        if (in && at < T13_CW) cand[wave][at] = key & ((1u << T13_LOW) - 1u);
        cnt += (int)__popcll(m);
    })
    if (lane == 0 && cnt > T13_CW) sh_over = 1;
    __syncthreads();
    if (sh_over == 0) {
        int g, e;
        const uint32_t low = t13_resolve(cand[wave], cnt, need, hist, &sh_prefix, &sh_need, &need_eq, &g, &e);
        T = (b12 << T13_LOW) | low;
        if (lane == 0) { wave_gt[wave] = cgt + g; wave_eq[wave] = e; }
    } else {
        // ---- fallback: four 8-bit passes over the row
        __syncthreads();   // every wavefront has read sh_over before the regions are reused as histograms
        if (tid == 0) { sh_prefix = 0; sh_need = k; }
        uint32_t prefix = 0;
        need = k;
        cgt = 0;   // last pass: keys of this wavefront's slice whose decided 24 bits exceed the prefix
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            const uint32_t hi_mask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
            for (int i = lane; i < 256; i += 64) whist[wave][i] = 0;
            __syncthreads();
            SPTS_LONG_SWEEP({
                hist_add(whist[wave], valid && (key & hi_mask) == prefix, (int)((key >> shift) & 0xFF));
                if (pass == 3) cgt += (int)__popcll(__ballot(valid && (key & hi_mask) > prefix));
            })
            __syncthreads();
            if (tid < 256) {
                int t = 0;
#pragma unroll
                for (int w = 0; w < TOPK_WAVES; ++w) t += whist[w][tid];
                hist[tid] = t;
            }
            __syncthreads();
            if (wave == 0) pick_bin(hist, lane, shift, prefix, need, &sh_prefix, &sh_need);
            __syncthreads();
            prefix = sh_prefix;
            need = sh_need;
        }
        T = prefix;
        need_eq = (int)need;
        // this wavefront's keys above T / equal to T, from its own last-digit histogram
        const int digit = (int)(T & 0xFFu);
        int above = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int b = lane * 4 + q;
            above += b > digit ? whist[wave][b] : 0;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) above += __shfl_xor(above, off);
        if (lane == 0) { wave_gt[wave] = above + cgt; wave_eq[wave] = whist[wave][digit]; }
    }
    __syncthreads();
    int gt_before = 0, eq_before = 0;
    for (int w = 0; w < wave; ++w) { gt_before += wave_gt[w]; eq_before += wave_eq[w]; }
    // ordered compaction of the slice: index order inside an iteration is (load u, lane, element e)
    for (int base = lo; base < hi; base += LONG_STEP) {
        f32x4v v[LONG_U];
#pragma unroll
        for (int u = 0; u < LONG_U; ++u) {
            const int i0 = base + u * 256 + lane * 4;
            v[u] = i0 < hi ? *reinterpret_cast<const f32x4v*>(scores + i0) : f32x4v{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < LONG_U; ++u) {
            const int i0 = base + u * 256 + lane * 4;
            const bool valid = i0 < hi;
            bool gt[4], eq[4];
            int lower_gt = 0, lower_eq = 0, tot_gt = 0, tot_eq = 0;   // selected keys of lower lanes / of the whole wavefront, this load
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint32_t key = order_key(v[u][e]);
                if ((uint32_t)(i0 + e) == last_key_at) key = 0xFFFFFFFFu;
                gt[e] = valid && key > T;
                eq[e] = valid && key == T;
                const uint64_t mg = __ballot(gt[e]), me = __ballot(eq[e]);
                lower_gt += lane_prefix_popc(mg); lower_eq += lane_prefix_popc(me);
                tot_gt += (int)__popcll(mg); tot_eq += (int)__popcll(me);
            }
            int my_gt = gt_before + lower_gt, my_eq = eq_before + lower_eq;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (gt[e] || (eq[e] && my_eq < need_eq)) idx_out[my_gt + (my_eq < need_eq ? my_eq : need_eq)] = i0 + e;
                my_gt += gt[e] ? 1 : 0;
                my_eq += eq[e] ? 1 : 0;
            }
            gt_before += tot_gt;
            eq_before += tot_eq;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// One problem spread over the chip (N up to TOPK_MULTI_MAX_N): the same radix select, but every 8-bit
// pass is its own launch of G workgroups, and no workgroup ever communicates with another one inside
// a launch: no atomics, no fences, no counters, nothing to clear between calls.  Workgroup g owns the
// contiguous slice [g * 1024 * KPT, (g + 1) * 1024 * KPT) (keys in registers for the duration of a
// launch), counts its share of the current digit into a private LDS histogram and stores those 256
// counters as row g of a table in the scratch.  The NEXT launch starts with every workgroup adding
// up the G rows for itself (G * 1 KB from L2, sixteen 16-byte loads in flight per lane) and picking
// the bin -- all workgroups reach the same (prefix, need) because the sums are integers -- before it
// counts the next digit into the other of two tables.  The fifth launch picks the last digit, turns
// the last table into its own output offsets (keys above the threshold and keys equal to it in the
// slices before its own) and writes its piece of the ascending index list.
struct TopkMultiScratch {
    int32_t rows[2][TOPK_MULTI_MAX_WG][256];   // histogram rows of the even / odd passes
    int32_t gt_hi[TOPK_MULTI_MAX_WG];          // last pass: keys of the slice whose decided 24 bits exceed the prefix
    uint32_t prefix[4]; int32_t need[4];       // state after pass p (written by workgroup 0 of launch p + 1)
};
static_assert(sizeof(TopkMultiScratch) <= TOPK_MULTI_SCRATCH_BYTES, "scratch size constant too small");

typedef int i32x4 __attribute__((ext_vector_type(4)));

// hist[0..256) = column sums of the G rows of `table`; all 1024 lanes take part, ends with a barrier
__device__ inline void topk_sum_rows(const int32_t (*table)[256], int G, int (*part)[256], int* hist) {
    const int tid = threadIdx.x;
    const int c4 = (tid & 63) * 4;
    i32x4 sum = {0, 0, 0, 0};
    for (int r = tid >> 6; r < G; r += 16) sum += *(const i32x4*)&table[r][c4];
    *(i32x4*)&part[tid >> 6][c4] = sum;
    __syncthreads();
    if (tid < 256) {
        int t = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q) t += part[q][tid];
        hist[tid] = t;
    }
    __syncthreads();
}

template <int KPT>
__global__ void __launch_bounds__(TOPK_THREADS) topk_multi_hist_kernel(const float* __restrict__ scores, int N, int k,
                                                                       int protect_last, TopkMultiScratch* scr, int pass) {
    __shared__ int hist[256];
    __shared__ __attribute__((aligned(16))) int part[16][256];
    __shared__ uint32_t sh_prefix;
    __shared__ int64_t sh_need;
    __shared__ int wave_cnt[TOPK_WAVES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x, G = gridDim.x;
    const int lo = g * (1024 * KPT) + wave * (64 * KPT);
    uint32_t keys[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const int i = lo + 64 * j + lane;
        keys[j] = i < N ? load_key(scores, i, N, protect_last) : 0u;
    }
    // state after the previous pass: the bin choice the previous launch's table implies
    uint32_t prefix = 0u;
    int64_t need = k;
    if (pass > 0) {
        if (pass > 1) { prefix = scr->prefix[pass - 2]; need = scr->need[pass - 2]; }
        if (tid == 0) { sh_prefix = prefix; sh_need = need; }
        topk_sum_rows(scr->rows[(pass - 1) & 1], G, part, hist);
        if (wave == 0) pick_bin(hist, lane, 24 - 8 * (pass - 1), prefix, need, &sh_prefix, &sh_need);
        __syncthreads();
        prefix = sh_prefix;
        need = sh_need;
        if (g == 0 && tid == 0) { scr->prefix[pass - 1] = prefix; scr->need[pass - 1] = (int32_t)need; }
    }
    const int shift = 24 - 8 * pass;
    const uint32_t hi_mask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
    __syncthreads();
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    int cgt = 0;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const bool valid = lo + 64 * j + lane < N;
        hist_add(hist, valid && (keys[j] & hi_mask) == prefix, (int)((keys[j] >> shift) & 0xFF));
        if (pass == 3) cgt += (int)__popcll(__ballot(valid && (keys[j] & hi_mask) > prefix));
    }
    if (lane == 0) wave_cnt[wave] = cgt;
    __syncthreads();
    if (tid < 256) scr->rows[pass & 1][g][tid] = hist[tid];
    if (tid == 0 && pass == 3) {
        int t = 0;
        for (int w = 0; w < TOPK_WAVES; ++w) t += wave_cnt[w];
        scr->gt_hi[g] = t;
    }
}

template <int KPT>
__global__ void __launch_bounds__(TOPK_THREADS) topk_multi_write_kernel(const float* __restrict__ scores, int N, int protect_last,
                                                                        const TopkMultiScratch* scr, int32_t* __restrict__ idx_out) {
    __shared__ int hist[256];
    __shared__ __attribute__((aligned(16))) int part[16][256];
    __shared__ uint32_t sh_prefix;
    __shared__ int64_t sh_need;
    __shared__ int wave_gt[TOPK_WAVES], wave_eq[TOPK_WAVES];
    __shared__ int red_gt[TOPK_WAVES], red_eq[TOPK_WAVES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x, G = gridDim.x;
    const int lo = g * (1024 * KPT) + wave * (64 * KPT);
    uint32_t keys[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const int i = lo + 64 * j + lane;
        keys[j] = i < N ? load_key(scores, i, N, protect_last) : 0u;
    }
    // the last digit: threshold key T and the number of keys equal to T still to be taken
    const int32_t (*table)[256] = scr->rows[1];
    {
        const uint32_t prefix = scr->prefix[2];
        const int64_t need = scr->need[2];
        if (tid == 0) { sh_prefix = prefix; sh_need = need; }
        topk_sum_rows(table, G, part, hist);
        if (wave == 0) pick_bin(hist, lane, 0, prefix, need, &sh_prefix, &sh_need);
        __syncthreads();
    }
    const uint32_t T = sh_prefix;
    const int need_eq = (int)sh_need;
    const int digit = (int)(T & 0xFFu);
    // keys above T / equal to T in the slices before this one: eight lanes per row of the table, each 32 consecutive
    // bins (eight 16-byte loads), rows at or beyond g contribute nothing
    int row_gt = 0, row_eq = 0;
    {
        const int r = tid >> 3, sub = tid & 7;
        if (r < g) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int b = sub * 32 + q * 4;
                const i32x4 v = *(const i32x4*)&table[r][b];
                row_gt += (b > digit ? v[0] : 0) + (b + 1 > digit ? v[1] : 0) + (b + 2 > digit ? v[2] : 0) + (b + 3 > digit ? v[3] : 0);
            }
            if (sub == 0) { row_gt += scr->gt_hi[r]; row_eq = table[r][digit]; }
        }
    }
    int cgt = 0, ceq = 0;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const bool valid = lo + 64 * j + lane < N;
        cgt += (int)__popcll(__ballot(valid && keys[j] > T));
        ceq += (int)__popcll(__ballot(valid && keys[j] == T));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { row_gt += __shfl_xor(row_gt, off); row_eq += __shfl_xor(row_eq, off); }
    if (lane == 0) { wave_gt[wave] = cgt; wave_eq[wave] = ceq; red_gt[wave] = row_gt; red_eq[wave] = row_eq; }
    __syncthreads();
    int gt_before = 0, eq_before = 0;
    for (int w = 0; w < TOPK_WAVES; ++w) { gt_before += red_gt[w]; eq_before += red_eq[w]; }
    for (int w = 0; w < wave; ++w) { gt_before += wave_gt[w]; eq_before += wave_eq[w]; }
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const int i = lo + 64 * j + lane;
        const bool valid = i < N;
        const bool gt = valid && keys[j] > T, eq = valid && keys[j] == T;
        const uint64_t mgt = __ballot(gt), meq = __ballot(eq);
        const int my_gt = gt_before + lane_prefix_popc(mgt);
        const int my_eq = eq_before + lane_prefix_popc(meq);
        if (gt || (eq && my_eq < need_eq)) idx_out[my_gt + (my_eq < need_eq ? my_eq : need_eq)] = i;
        gt_before += (int)__popcll(mgt);
        eq_before += (int)__popcll(meq);
    }
}

template <int KPT>
static hipError_t topk_multi_launch(const float* scores, int N, int k, int protect_last, int32_t* idx_out,
                                    TopkMultiScratch* scr, hipStream_t s) {
    const int G = (N + 1024 * KPT - 1) / (1024 * KPT);
    for (int pass = 0; pass < 4; ++pass)
        topk_multi_hist_kernel<KPT><<<dim3(G), dim3(TOPK_THREADS), 0, s>>>(scores, N, k, protect_last, scr, pass);
    topk_multi_write_kernel<KPT><<<dim3(G), dim3(TOPK_THREADS), 0, s>>>(scores, N, protect_last, scr, idx_out);
    return hipGetLastError();
}

// Scratch of the no-allocation entry point: one array per GPU, in the code object's own device memory.  Nothing in it
// has to start at zero: every word a call reads was written earlier in the same call.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[TOPK_MULTI_SCRATCH_BYTES];

hipError_t topk_static_scratch(void** out) {
    // In host code the array's name is only a handle for the runtime: the address a kernel can use comes from
    // hipGetSymbolAddress, once per device (every GPU holds its own copy at its own address).
    constexpr int MAX_DEV = 64;
    static std::mutex mtx;
    static void* dev_ptr[MAX_DEV] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEV) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mtx);
    if (!dev_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        dev_ptr[dev] = p;
    }
    *out = dev_ptr[dev];
    return hipSuccess;
}

hipError_t launch_topk_multi(const float* scores, int64_t N, int64_t k, int protect_last, int32_t* idx_out, void* scratch,
                             hipStream_t s) {
    if (k <= 0 || N <= 0) return hipSuccess;
    if (N > TOPK_MULTI_MAX_N || k > N || !scratch) return hipErrorInvalidValue;
    TopkMultiScratch* scr = (TopkMultiScratch*)scratch;
    // slices of 4096 keys (32 workgroups at N = 131072: every workgroup re-adds all rows of the table, so a small
    // grid keeps that cheap); longer rows take 8192 so that the grid stays within the table
    if (N <= (int64_t)TOPK_MULTI_MAX_WG * 4096) return topk_multi_launch<4>(scores, (int)N, (int)k, protect_last, idx_out, scr, s);
    return topk_multi_launch<8>(scores, (int)N, (int)k, protect_last, idx_out, scr, s);
}

// ---------------------------------------------------------------------------------------------
// Mean of the k largest |values| of every row of a [rows, T] matrix (Eq. (channel_importance): the
// importance of an FFN channel is the mean of the top-rho fraction of its saliencies over the
// calibration tokens; rows = channels).  Same radix select as above on the keys of |v| (exact
// k-th value and how many copies of it count), then a sum of everything above it in a fixed order
// (per lane, shuffle tree, wavefronts in order): deterministic.  One workgroup per row; the row is
// re-read in every sweep and stays in L2 meanwhile.
template <typename T>
__global__ void __launch_bounds__(TOPK_THREADS) topk_mean_kernel(const T* __restrict__ vals, int64_t ld, int64_t n, int64_t k,
                                                                 float* __restrict__ out) {
    __shared__ int hist[256];
    __shared__ uint32_t sh_prefix;
    __shared__ int64_t sh_need;
    __shared__ float wsum[TOPK_WAVES];
    const T* row = vals + (int64_t)blockIdx.x * ld;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { sh_prefix = 0; sh_need = k; }
    uint32_t prefix = 0;
    int64_t need = k;
    // bf16 values widen to keys whose low 16 bits are zero: two 8-bit passes decide the whole key
    constexpr int NPASS = sizeof(T) == 2 ? 2 : 4;
    for (int pass = 0; pass < NPASS; ++pass) {
        const int shift = 24 - 8 * pass;
        const uint32_t hi_mask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int64_t base = 0; base < n; base += TOPK_THREADS) {
            const int64_t i = base + tid;
            const uint32_t key = i < n ? order_key(fabsf(to_f32(row[i]))) : 0u;
            hist_add(hist, i < n && (key & hi_mask) == prefix, (int)((key >> shift) & 0xFF));
        }
        __syncthreads();
        if (wave == 0) pick_bin(hist, lane, shift, prefix, need, &sh_prefix, &sh_need);
        __syncthreads();
        prefix = sh_prefix;
        need = sh_need;
    }
    const uint32_t Tk = prefix;       // key of the k-th largest |value|
    float s = 0.f, tval = 0.f;
    for (int64_t base = 0; base < n; base += TOPK_THREADS) {
        const int64_t i = base + tid;
        if (i < n) {
            const float v = fabsf(to_f32(row[i]));
            const uint32_t key = order_key(v);
            if (key > Tk) s += v;
            if (key == Tk) tval = v;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { s += __shfl_xor(s, off); tval = fmaxf(tval, __shfl_xor(tval, off)); }
    __shared__ float wt[TOPK_WAVES];
    if (lane == 0) { wsum[wave] = s; wt[wave] = tval; }
    __syncthreads();
    if (tid == 0) {
        float tot = 0.f, tv = 0.f;
        for (int w = 0; w < TOPK_WAVES; ++w) { tot += wsum[w]; tv = fmaxf(tv, wt[w]); }
        out[blockIdx.x] = (tot + (float)need * tv) / (float)k;
    }
}

hipError_t launch_topk_mean(const void* vals, int64_t ld, int64_t rows, int64_t n, int64_t k, float* out, bool bf16,
                            hipStream_t s) {
    if (rows <= 0 || n <= 0 || k <= 0) return hipSuccess;
    const dim3 g((unsigned)rows), b(TOPK_THREADS);
    if (bf16) topk_mean_kernel<bf16_t><<<g, b, 0, s>>>((const bf16_t*)vals, ld, n, k, out);
    else topk_mean_kernel<float><<<g, b, 0, s>>>((const float*)vals, ld, n, k, out);
    return hipGetLastError();
}

hipError_t launch_topk(const float* scores, int64_t N, int64_t k, int protect_last, int32_t* idx_out, int batch,
                       hipStream_t s, TopkSegments seg) {
    // with segments N is the longest segment (it picks the kernel variant) and k is ignored
    if ((k <= 0 && !seg.offsets) || N <= 0 || batch <= 0) return hipSuccess;
    const dim3 g((unsigned)batch), b(TOPK_THREADS);
    if (N <= 1024 * 32) {
        hipError_t e;
        if (N <= 1024 * 8) {
            if ((e = ensure_dynamic_lds(reinterpret_cast<const void*>(&topk_reg_kernel<8>), T13_LDS_BYTES)) != hipSuccess) return e;
            topk_reg_kernel<8><<<g, b, T13_LDS_BYTES, s>>>(scores, N, k, protect_last, idx_out, seg);
        } else if (N <= 1024 * 16) {
            if ((e = ensure_dynamic_lds(reinterpret_cast<const void*>(&topk_reg_kernel<16>), T13_LDS_BYTES)) != hipSuccess) return e;
            topk_reg_kernel<16><<<g, b, T13_LDS_BYTES, s>>>(scores, N, k, protect_last, idx_out, seg);
        } else {
            if ((e = ensure_dynamic_lds(reinterpret_cast<const void*>(&topk_reg_kernel<32>), T13_LDS_BYTES)) != hipSuccess) return e;
            topk_reg_kernel<32><<<g, b, T13_LDS_BYTES, s>>>(scores, N, k, protect_last, idx_out, seg);
        }
    }
    else if (!seg.offsets && N % 4 == 0 && N < ((int64_t)1 << 30)) {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&topk_long_kernel), T13_LDS_BYTES);
        if (e != hipSuccess) return e;
        topk_long_kernel<<<g, b, T13_LDS_BYTES, s>>>(scores, N, k, protect_last, idx_out);
    }
    else topk_kernel<<<g, b, 0, s>>>(scores, N, k, protect_last, idx_out, seg);
    return hipGetLastError();
}

}  // namespace spts
