// Shape-agnostic causal GQA attention and PAP probe scoring with fp32 arithmetic.  These serve the
// fp32 configuration and head dimensions / dtypes the matrix-core kernels do not take.
#include "spts_internal.h"

namespace spts {

constexpr int MAX_D = 256;

// ---------------------------------------------------------------- attention
// One wavefront per (query row, head).  Keys are visited in chunks of 64 (one key per lane for the
// logits, one output column group per lane for the value sum) with an online softmax.
template <typename T>
__global__ void __launch_bounds__(64) attention_generic_kernel(AttnArgs a) {
    __shared__ float qs[MAX_D];
    __shared__ float ps[64];
    const int64_t i = blockIdx.x;
    const int h = blockIdx.y;
    const int g = h / (a.H / a.Hkv);
    const int lane = threadIdx.x;
    const int d = a.d;
    const T* q = (const T*)a.q + (i * a.H + h) * (int64_t)d;
    const T* K = (const T*)a.k;
    const T* V = (const T*)a.v;
    const float scale = 1.0f / sqrtf((float)d) / (a.q_scale != 0.f ? a.q_scale : 1.0f);   // q may arrive pre-scaled
    for (int j = lane; j < d; j += 64) qs[j] = to_f32(q[j]);
    __syncthreads();
    const int qp = a.qpos[i];

    float m = -INFINITY, l = 0.f;
    float acc[MAX_D / 64] = {};
    for (int64_t j0 = 0; j0 < a.Mk; j0 += 64) {
        if (a.kpos[j0] > qp) break;  // ascending positions: nothing visible from here on
        int64_t j = j0 + lane;
        float logit = -INFINITY;
        if (j < a.Mk && a.kpos[j] <= qp) {
            const T* kr = K + (j * a.Hkv + g) * (int64_t)d;
            float s = 0.f;
            for (int c = 0; c < d; ++c) s = fmaf(qs[c], to_f32(kr[c]), s);
            logit = s * scale;
        }
        float cm = logit;
        for (int off = 32; off > 0; off >>= 1) cm = fmaxf(cm, __shfl_xor(cm, off));
        float m_new = fmaxf(m, cm);  // finite: the chunk's first key is visible
        float p = (logit == -INFINITY) ? 0.f : expf(logit - m_new);
        float csum = p;
        for (int off = 32; off > 0; off >>= 1) csum += __shfl_xor(csum, off);
        float alpha = (m == -INFINITY) ? 0.f : expf(m - m_new);
        l = l * alpha + csum;
        m = m_new;
        ps[lane] = p;
        __syncthreads();
        int64_t nk = a.Mk - j0 < 64 ? a.Mk - j0 : 64;
#pragma unroll
        for (int t = 0; t < MAX_D / 64; ++t) {
            int c = lane + 64 * t;
            if (c < d) {
                float s = acc[t] * alpha;
                for (int64_t jj = 0; jj < nk; ++jj) s = fmaf(ps[jj], to_f32(V[((j0 + jj) * a.Hkv + g) * (int64_t)d + c]), s);
                acc[t] = s;
            }
        }
        __syncthreads();
    }
    T* o = (T*)a.out + (i * a.H + h) * (int64_t)d;
    float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
    for (int t = 0; t < MAX_D / 64; ++t) {
        int c = lane + 64 * t;
        if (c < d) o[c] = from_f32<T>(acc[t] * inv);
    }
}

hipError_t launch_attention_generic(const AttnArgs& a, bool bf16, hipStream_t s) {
    if (a.Mq == 0) return hipSuccess;
    dim3 grid((unsigned)a.Mq, (unsigned)a.H), block(64);
    if (bf16) attention_generic_kernel<bf16_t><<<grid, block, 0, s>>>(a);
    else attention_generic_kernel<float><<<grid, block, 0, s>>>(a);
    return hipGetLastError();
}

// ---------------------------------------------------------------- probe (Eq. (mha_importance))
// Pass 1: one workgroup per probe row (p, h): max and sum of exp over the visible candidates.
template <typename T>
__global__ void __launch_bounds__(256) probe_stats_generic_kernel(ProbeArgs a) {
    __shared__ float qs[MAX_D];
    __shared__ float red[4];
    const int p = blockIdx.x / a.H, h = blockIdx.x % a.H;
    const int g = h / (a.H / a.Hkv);
    const int d = a.d;
    const T* q = (const T*)a.qp + ((int64_t)p * a.H + h) * d;
    const T* K = (const T*)a.k;
    const float scale = 1.0f / sqrtf((float)d) / (a.q_scale != 0.f ? a.q_scale : 1.0f);   // q may arrive pre-scaled
    for (int j = threadIdx.x; j < d; j += 256) qs[j] = to_f32(q[j]);
    __syncthreads();
    const int64_t nvis = a.N - a.P + p + 1;  // candidates 0 .. N-P+p
    float m = -INFINITY;
    for (int64_t n = threadIdx.x; n < nvis; n += 256) {
        const T* kr = K + (n * a.Hkv + g) * (int64_t)d;
        float s = 0.f;
        for (int c = 0; c < d; ++c) s = fmaf(qs[c], to_f32(kr[c]), s);
        m = fmaxf(m, s * scale);
    }
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float l = 0.f;
    for (int64_t n = threadIdx.x; n < nvis; n += 256) {
        const T* kr = K + (n * a.Hkv + g) * (int64_t)d;
        float s = 0.f;
        for (int c = 0; c < d; ++c) s = fmaf(qs[c], to_f32(kr[c]), s);
        l += expf(s * scale - m);
    }
    for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = l;
    __syncthreads();
    if (threadIdx.x == 0) {
        a.stats[2 * blockIdx.x] = m;
        a.stats[2 * blockIdx.x + 1] = red[0] + red[1] + red[2] + red[3];
    }
}

// Pass 2: one lane per candidate, rows visited in a fixed order (deterministic sum).
template <typename T>
__global__ void __launch_bounds__(256) probe_accum_generic_kernel(ProbeArgs a) {
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= a.N) return;
    const int d = a.d;
    const T* K = (const T*)a.k;
    const T* Q = (const T*)a.qp;
    const float scale = 1.0f / sqrtf((float)d) / (a.q_scale != 0.f ? a.q_scale : 1.0f);   // q may arrive pre-scaled
    const int grp = a.H / a.Hkv;
    float acc = 0.f;
    for (int p = 0; p < a.P; ++p) {
        if (n > a.N - a.P + p) continue;
        for (int h = 0; h < a.H; ++h) {
            const T* kr = K + (n * a.Hkv + h / grp) * (int64_t)d;
            const T* q = Q + ((int64_t)p * a.H + h) * d;
            float s = 0.f;
            for (int c = 0; c < d; ++c) s = fmaf(to_f32(q[c]), to_f32(kr[c]), s);
            float m = a.stats[2 * (p * a.H + h)], l = a.stats[2 * (p * a.H + h) + 1];
            acc += expf(s * scale - m) / l;
        }
    }
    a.S[n] = acc / (float)(a.P * a.H);
}

hipError_t launch_probe_generic(const ProbeArgs& a, bool bf16, hipStream_t s) {
    if (a.N == 0) return hipSuccess;
    dim3 g1((unsigned)(a.P * a.H)), g2((unsigned)((a.N + 255) / 256)), b(256);
    if (bf16) {
        probe_stats_generic_kernel<bf16_t><<<g1, b, 0, s>>>(a);
        probe_accum_generic_kernel<bf16_t><<<g2, b, 0, s>>>(a);
    } else {
        probe_stats_generic_kernel<float><<<g1, b, 0, s>>>(a);
        probe_accum_generic_kernel<float><<<g2, b, 0, s>>>(a);
    }
    return hipGetLastError();
}

}  // namespace spts
