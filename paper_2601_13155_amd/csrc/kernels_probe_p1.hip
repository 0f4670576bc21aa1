// PAP probe with a single probe row (P = 1: Eq. (mha_importance) exactly as printed, the paper's
// default): S[n] = 1/H * sum_h softmax_n( q_h . k[n, g(h)] / sqrt(d) )[n], q = the last candidate's
// rotary query, which sees every candidate.
//
// One query per head makes this a scan of K at memory speed, not a matrix product:
//   pass 1  grid (key chunks, KV heads): LPK lanes hold one key row in 16-byte pieces, the H/Hkv
//           queries of the KV head sit in registers; every key's logits (scaled to base 2) go to
//           logit[h][n] (fp32 scratch) and each lane group keeps a running (max, sum-exp) per
//           head; groups and wavefronts merge in a fixed order -> stats_part[chunk][h]
//   pass 2  one wavefront per head: (M_h, 1/L_h) over the chunks
//   pass 3  S[n] = 1/H * sum_h exp2(logit[h][n] - M_h) / L_h, heads in order (deterministic)
// K is read once (N*Hkv*d elements); the logits cost 8*H*N bytes of L2-resident traffic.
#include "spts_internal.h"
#include "spts_lanes.h"

namespace spts {

constexpr int P1_CHUNK = 128;      // keys per workgroup (many short workgroups: the scan is latency-bound per wavefront)
constexpr int P1_GRP_MAX = 8;      // query heads per KV head, at most

// scratch floats the single-row probe needs: logits [H][Np] + stats_part [nchunks][H][2] + stats [H][2]
size_t probe_p1_scratch_floats(int64_t N, int H) {
    const int64_t Np = (N + 255) / 256 * 256;
    const int64_t nchunks = (N + P1_CHUNK - 1) / P1_CHUNK;
    return (size_t)(H * Np + (nchunks + 1) * H * 2 + 64);
}

template <typename T, int D>
__global__ void __launch_bounds__(256) probe_p1_logits_kernel(const T* __restrict__ q, const T* __restrict__ K, int64_t N,
                                                              int64_t Np, int H, int Hkv, float scale_log2e,
                                                              float* __restrict__ logit, float* __restrict__ stats_part) {
    constexpr int EPC = 16 / (int)sizeof(T);
    constexpr int LPK = D / EPC;
    constexpr int KPW = 64 / LPK;
    __shared__ float sm[4][P1_GRP_MAX][2];
    const int chunk = blockIdx.x, g = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % LPK, kslot = lane / LPK;
    const int grp = H / Hkv;
    const int64_t m_begin = (int64_t)chunk * P1_CHUNK;
    const int64_t m_end = m_begin + P1_CHUNK < N ? m_begin + P1_CHUNK : N;

    u32x4 qv[P1_GRP_MAX];
#pragma unroll
    for (int hg = 0; hg < P1_GRP_MAX; ++hg) {
        const int h = g * grp + (hg < grp ? hg : 0);
        qv[hg] = *reinterpret_cast<const u32x4*>(q + (int64_t)h * D + sub * EPC);
    }
    float mrun[P1_GRP_MAX], lrun[P1_GRP_MAX];
#pragma unroll
    for (int hg = 0; hg < P1_GRP_MAX; ++hg) { mrun[hg] = -INFINITY; lrun[hg] = 0.f; }

    const T* Kg = K + (int64_t)g * D + sub * EPC;
    const int64_t rstride = (int64_t)Hkv * D;
    int64_t m = m_begin + wave * KPW + kslot;
    u32x4 kv = {0, 0, 0, 0};
    if (m_begin < m_end) kv = *reinterpret_cast<const u32x4*>(Kg + (m < m_end ? m : m_end - 1) * rstride);
    for (int64_t m0 = m_begin + wave * KPW; m0 < m_end; m0 += 4 * KPW, m += 4 * KPW) {
        const bool valid = m < m_end;
        const int64_t mn_ = m + 4 * KPW;
        const u32x4 kvn = *reinterpret_cast<const u32x4*>(Kg + (mn_ < m_end ? mn_ : m_end - 1) * rstride);
#pragma unroll
        for (int hg = 0; hg < P1_GRP_MAX; ++hg) {
            if (hg < grp) {
                float s = group_sum<LPK>(dot16(kv, qv[hg], 0.f, T{})) * scale_log2e;
                if (valid && sub == 0) logit[(int64_t)(g * grp + hg) * Np + m] = s;
                s = valid ? s : -INFINITY;
                const float mn = fmaxf(mrun[hg], s);
                const float mu = mn == -INFINITY ? 0.f : mn;
                lrun[hg] = lrun[hg] * __builtin_amdgcn_exp2f(mrun[hg] - mu) + __builtin_amdgcn_exp2f(s - mu);
                mrun[hg] = mn;
            }
        }
        kv = kvn;
    }
    // merge lane groups (lanes with equal `sub`), then wavefronts
#pragma unroll
    for (int hg = 0; hg < P1_GRP_MAX; ++hg) {
        if (hg < grp) {
#pragma unroll
            for (int off = LPK; off < 64; off <<= 1) {
                const float mo = __shfl_xor(mrun[hg], off), lo = __shfl_xor(lrun[hg], off);
                const float mn = fmaxf(mrun[hg], mo);
                const float mu = mn == -INFINITY ? 0.f : mn;
                lrun[hg] = lrun[hg] * __builtin_amdgcn_exp2f(mrun[hg] - mu) + lo * __builtin_amdgcn_exp2f(mo - mu);
                mrun[hg] = mn;
            }
            if (lane == 0) { sm[wave][hg][0] = mrun[hg]; sm[wave][hg][1] = lrun[hg]; }
        }
    }
    __syncthreads();
    if (tid < grp) {
        float mn = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mn = fmaxf(mn, sm[w][tid][0]);
        const float mu = mn == -INFINITY ? 0.f : mn;
        float l = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) l += sm[w][tid][1] * __builtin_amdgcn_exp2f(sm[w][tid][0] - mu);
        float* o = stats_part + ((int64_t)chunk * H + g * grp + tid) * 2;
        o[0] = mn;
        o[1] = l;
    }
}

// stats[h] = (M_h, 1/L_h): one wavefront per head, lanes over the chunks, fixed shuffle tree
__global__ void __launch_bounds__(256) probe_p1_combine_kernel(const float* __restrict__ stats_part, int nchunks, int H,
                                                               float* __restrict__ stats) {
    const int lane = threadIdx.x & 63;
    const int h = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (h >= H) return;
    float M = -INFINITY;
    for (int c = lane; c < nchunks; c += 64) M = fmaxf(M, stats_part[((int64_t)c * H + h) * 2]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    float L = 0.f;
    for (int c = lane; c < nchunks; c += 64) {
        const float* s = stats_part + ((int64_t)c * H + h) * 2;
        if (s[0] != -INFINITY) L += s[1] * __builtin_amdgcn_exp2f(s[0] - M);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) L += __shfl_xor(L, off);
    if (lane == 0) { stats[2 * h] = M; stats[2 * h + 1] = L > 0.f ? 1.0f / L : 0.f; }
}

__global__ void __launch_bounds__(256) probe_p1_scores_kernel(const float* __restrict__ logit, const float* __restrict__ stats,
                                                              int64_t N, int64_t Np, int H, float* __restrict__ S) {
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    float acc = 0.f;
    for (int h = 0; h < H; ++h) acc += __builtin_amdgcn_exp2f(logit[(int64_t)h * Np + n] - stats[2 * h]) * stats[2 * h + 1];
    S[n] = acc / (float)H;
}

bool probe_p1_supported(const ProbeArgs& a) {
    if (a.P != 1 || a.N <= 0 || a.Hkv <= 0 || a.H % a.Hkv != 0 || a.H / a.Hkv > P1_GRP_MAX) return false;
    if (a.d != 16 && a.d != 32 && a.d != 64 && a.d != 128) return false;
    auto al = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    return al(a.qp) && al(a.k);
}

template <typename T>
static hipError_t launch_probe_p1_t(const ProbeArgs& a, float* scratch, hipStream_t s) {
    const int64_t Np = (a.N + 255) / 256 * 256;
    const int nchunks = (int)((a.N + P1_CHUNK - 1) / P1_CHUNK);
    float* logit = scratch;
    float* stats_part = logit + (size_t)a.H * Np;
    float* stats = stats_part + (size_t)nchunks * a.H * 2;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)a.d) / (a.q_scale != 0.f ? a.q_scale : 1.0f);   // qp may arrive pre-scaled
    const dim3 g((unsigned)nchunks, (unsigned)a.Hkv), b(256);
    const T* q = (const T*)a.qp;
    const T* K = (const T*)a.k;
    switch (a.d) {
        case 128: probe_p1_logits_kernel<T, 128><<<g, b, 0, s>>>(q, K, a.N, Np, a.H, a.Hkv, scale_log2e, logit, stats_part); break;
        case 64: probe_p1_logits_kernel<T, 64><<<g, b, 0, s>>>(q, K, a.N, Np, a.H, a.Hkv, scale_log2e, logit, stats_part); break;
        case 32: probe_p1_logits_kernel<T, 32><<<g, b, 0, s>>>(q, K, a.N, Np, a.H, a.Hkv, scale_log2e, logit, stats_part); break;
        case 16: probe_p1_logits_kernel<T, 16><<<g, b, 0, s>>>(q, K, a.N, Np, a.H, a.Hkv, scale_log2e, logit, stats_part); break;
        default: return hipErrorInvalidValue;
    }
    probe_p1_combine_kernel<<<dim3((unsigned)((a.H + 3) / 4)), b, 0, s>>>(stats_part, nchunks, a.H, stats);
    probe_p1_scores_kernel<<<dim3((unsigned)((a.N + 255) / 256)), b, 0, s>>>(logit, stats, a.N, Np, a.H, a.S);
    return hipGetLastError();
}

// scratch: probe_p1_scratch_floats(N, H) floats
hipError_t launch_probe_p1(const ProbeArgs& a, float* scratch, bool bf16, hipStream_t s) {
    return bf16 ? launch_probe_p1_t<bf16_t>(a, scratch, s) : launch_probe_p1_t<float>(a, scratch, s);
}

}  // namespace spts
