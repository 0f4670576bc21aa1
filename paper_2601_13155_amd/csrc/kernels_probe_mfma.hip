// PAP probe scoring on the matrix cores (Eq. (mha_importance) with a probe window of P rows):
//   S[n] = 1/(P*H) * sum over probe rows (p, h) of softmax_n( qp[p,h].k[n,g(h)] / sqrt(d) )[n],
// probe row p being candidate N-P+p, which sees candidates 0..N-P+p.
//
// A softmax needs the full-row denominator before any probability can be averaged over rows, so
// K is streamed twice:
//   pass 1  per (kv head g, chunk of 256 keys): running (max, sum-exp) of every probe row of that
//           head group over the chunk  ->  stats_part[chunk][g][row]
//   combine per (g, row): global max M and 1/sum over the chunks
//   pass 2  per (g, chunk): logits again, p = exp2(s - M) / L summed over the rows of the group
//           ->  part[g][n];   final: S[n] = sum_g part[g][n] / (P*H)   (fixed order: deterministic)
// The R = P*H/Hkv probe rows of one KV head form a dense [R x d] operand that stays in registers
// (32*RB rows per wavefront); K tiles of 64 keys go through LDS (swizzled, shared by the 4
// wavefronts).  Pass 1 computes S^T = K Q^T (one probe row per lane column: row max in-lane),
// pass 2 computes S = Q K^T (one key per lane column: the sum over rows is in-lane).
#include "spts_internal.h"

namespace spts {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PKV = 64;          // keys per tile
constexpr int CHUNK_TILES = 4;   // tiles per workgroup
constexpr int CHUNK = PKV * CHUNK_TILES;

template <int D> struct ProbeLds {
    static constexpr int CPRK = D / 8;
    static constexpr int RPK = 256 / (2 * D);
    static constexpr int K_BYTES = PKV * D * 2;
    __device__ static inline int koff(int row, int c) { return row * (2 * D) + ((c ^ ((row / RPK) % CPRK)) << 4); }
};

// stats_part: [nchunks][Hkv][Rp][2]; stats: [Hkv][Rp][2] (M, 1/L); part: [Hkv][Np]
// NWV wavefronts per workgroup, 32 * RB probe rows each.  Two wavefronts per SIMD are asked of the register allocator
// where the rows fit (RB <= 2; left alone it used 270 registers for pass 2 and ran one).
template <int D, int RB, int PASS, int NWV>
__global__ void __launch_bounds__(64 * NWV) __attribute__((amdgpu_waves_per_eu((PASS == 2 && RB <= 2) ? 2 : 1, 8))) probe_mfma_kernel(ProbeArgs a, int Rp, int64_t Np, float qmul,
                                                         float* __restrict__ stats_part, const float* __restrict__ stats) {
    using L = ProbeLds<D>;
    constexpr int KS = D / 16;
    __shared__ __attribute__((aligned(16))) char sK[2][L::K_BYTES];
    constexpr int NT = 64 * NWV;
    __shared__ float sRed[NWV][PKV];

    const int chunk = blockIdx.x, g = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int grp = a.H / a.Hkv;
    const int R = a.P * grp;
    const int64_t key_begin = (int64_t)chunk * CHUNK;
    const int64_t key_end = key_begin + CHUNK < a.N ? key_begin + CHUNK : a.N;
    const int n_tiles = (int)((key_end - key_begin + PKV - 1) / PKV);

    // ---- probe-row fragments: row rr = p * grp + hg  <->  qp[p, g*grp + hg, :]
    bf16x8 qf[RB][KS];
    int vis_last[RB];   // last candidate index visible to the lane's row in block rb (pass 1 layout)
    const bf16_t* Q = (const bf16_t*)a.qp;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        int rr = wave * 32 * RB + rb * 32 + l32;
        int rc = rr < R ? rr : R - 1;
        int p = rc / grp, hg = rc % grp;
        vis_last[rb] = rr < R ? (int)(a.N - a.P + p) : -1;
        const bf16_t* qr = Q + ((int64_t)p * a.H + g * grp + hg) * D + 8 * lh;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[rb][ks] = *reinterpret_cast<const bf16x8*>(qr + 16 * ks);
        // qp normally arrives carrying log2(e)/sqrt(d) (qmul == 1): the logits leave the matrix core as exponents of 2;
        // otherwise the rest of the factor is folded in here (a second bf16 rounding)
        if (qmul != 1.0f) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                u32x4 raw = __builtin_bit_cast(u32x4, qf[rb][ks]);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    raw[j] = cvt_pk_bf16(__uint_as_float(raw[j] << 16) * qmul, __uint_as_float(raw[j] & 0xffff0000u) * qmul);
                qf[rb][ks] = __builtin_bit_cast(bf16x8, raw);
            }
        }
    }
    // pass 2: the lane's 16 rows per block keep their exponent offset log2(1/L) - M in registers, laid out as the C operand
    // that starts a block's product: the MFMA then delivers log2 of the probability itself (padded rows and empty rows:
    // offset -inf, probability 0)
    f32x16 coff[PASS == 2 ? RB : 1];
    // ... and, for the tiles that reach into the probe window, (window row p of the register's probe row) + 1, two per
    // register: candidate N - P + j is hidden from the row when j >= p + 1 (0 for padded rows, whose offset is -inf anyway)
    uint32_t pvis[PASS == 2 ? RB : 1][8];
    if (PASS == 2) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rr = wave * 32 * RB + rb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                const float2 st = *reinterpret_cast<const float2*>(stats + ((int64_t)g * Rp + rr) * 2);
                coff[rb][r] = st.y > 0.f ? __builtin_amdgcn_logf(st.y) - st.x : -INFINITY;
                const uint32_t enc = rr < R ? (uint32_t)(rr / grp + 1) : 0u;
                if (r & 1) pvis[rb][r >> 1] |= enc << 16; else pvis[rb][r >> 1] = enc;
            }
    }

    constexpr int KCH = PKV * L::CPRK / NT;
    static_assert(KCH >= 1, "a key tile gives every thread at least one 16-byte chunk");
    const int kc = tid % L::CPRK, kr = tid / L::CPRK;
    const bf16_t* Kg = (const bf16_t*)a.k;
    u32x4 rk[KCH];
    auto load_tile = [&](int t) {
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            int64_t key = key_begin + (int64_t)t * PKV + kr + (NT / L::CPRK) * i;
            if (key >= a.N) key = a.N - 1;
            rk[i] = *reinterpret_cast<const u32x4*>(Kg + (key * a.Hkv + g) * (int64_t)D + kc * 8);
        }
    };
    auto store_tile = [&](int stage) {
#pragma unroll
        for (int i = 0; i < KCH; ++i) *reinterpret_cast<u32x4*>(sK[stage] + L::koff(kr + (NT / L::CPRK) * i, kc)) = rk[i];
    };

    float m_run[RB], l_run[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) { m_run[rb] = -INFINITY; l_run[rb] = 0.f; }

    const int64_t first_masked = a.N - a.P + 1;   // candidates from here on are hidden from some probe row
    if (n_tiles > 0) { load_tile(0); store_tile(0); }
    __syncthreads();
    for (int t = 0; t < n_tiles; ++t) {
        if (t + 1 < n_tiles) load_tile(t + 1);
        const char* sk = sK[t & 1];
        const int64_t key0 = key_begin + (int64_t)t * PKV;
        const bool need_mask = key0 + PKV > first_masked || key0 + PKV > a.N;
        if (PASS == 1) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                f32x16 s[2];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        bf16x8 kf = *reinterpret_cast<const bf16x8*>(sk + L::koff(kb * 32 + l32, 2 * ks + lh));
                        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[rb][ks], s[kb], 0, 0, 0);
                    }
                }
                // lane: probe row = column l32; keys = kb*32 + 8*(r/4) + 4*lh + r%4
                float mx = -INFINITY;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float v = s[kb][r];
                        if (need_mask) {
                            int64_t key = key0 + kb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                            if (key > vis_last[rb]) v = -INFINITY;
                        }
                        s[kb][r] = v;
                        mx = fmaxf(mx, v);
                    }
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run[rb], mx);
                const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
                float sum = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(s[kb][r] - m_use);
                l_run[rb] = l_run[rb] * __builtin_amdgcn_exp2f(m_run[rb] - m_use) + sum;
                m_run[rb] = m_new;
            }
        } else {
            float ksum[2] = {0.f, 0.f};
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    f32x16 s = coff[rb];
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        bf16x8 kf = *reinterpret_cast<const bf16x8*>(sk + L::koff(kb * 32 + l32, 2 * ks + lh));
                        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][ks], kf, s, 0, 0, 0);
                    }
                    // lane: key = column kb*32 + l32; rows = rb*32 + 8*(r/4) + 4*lh + r%4
                    const int krel = (int)(key0 + kb * 32 + l32 - (a.N - a.P));   // position inside the probe window (< 0: before it)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float pv = __builtin_amdgcn_exp2f(s[r]);
                        if (need_mask && krel >= (int)((pvis[rb][r >> 1] >> (16 * (r & 1))) & 0xffffu)) pv = 0.f;
                        ksum[kb] += pv;
                    }
                    // one block at a time: interleaved, the blocks' accumulators and exponentials do not fit the registers
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                float v = ksum[kb] + __shfl_xor(ksum[kb], 32);
                if (lh == 0) sRed[wave][kb * 32 + l32] = v;
            }
            __syncthreads();
            if (tid < PKV) {
                int64_t key = key0 + tid;
                if (key < a.N) {
                    float tot = sRed[0][tid];
#pragma unroll
                    for (int wv = 1; wv < NWV; ++wv) tot += sRed[wv][tid];   // fixed order
                    a.partial[(int64_t)g * Np + key] = tot;
                }
            }
        }
        if (t + 1 < n_tiles) store_tile((t + 1) & 1);
        __syncthreads();
    }
    if (PASS == 1) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            float l = l_run[rb] + __shfl_xor(l_run[rb], 32);
            int rr = wave * 32 * RB + rb * 32 + l32;
            if (lh == 0) {
                float* o = stats_part + (((int64_t)chunk * a.Hkv + g) * Rp + rr) * 2;
                o[0] = m_run[rb];
                o[1] = l;
            }
        }
    }
}

// stats[g][rr] = (M, 1/L) over the chunks; padded rows rr >= R get (huge, 0).  One wavefront per (g, rr):
// lane c takes chunks c, c + 64, ...; maximum and sum are reduced over a fixed shuffle tree (deterministic).
__global__ void __launch_bounds__(256) probe_combine_kernel(const float* __restrict__ stats_part, float* __restrict__ stats,
                                                            int nchunks, int Hkv, int Rp, int R) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= Hkv * Rp) return;
    const int g = i / Rp, rr = i % Rp;
    if (rr >= R) {   // padded rows weigh nothing
        if (lane == 0) { stats[2 * i] = 1e30f; stats[2 * i + 1] = 0.f; }
        return;
    }
    float M = -INFINITY;
    for (int c = lane; c < nchunks; c += 64) M = fmaxf(M, stats_part[(((int64_t)c * Hkv + g) * Rp + rr) * 2]);
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    float Lsum = 0.f;
    for (int c = lane; c < nchunks; c += 64) {
        const float* s = stats_part + (((int64_t)c * Hkv + g) * Rp + rr) * 2;
        if (s[0] != -INFINITY) Lsum += s[1] * __builtin_amdgcn_exp2f(s[0] - M);
    }
    for (int off = 32; off > 0; off >>= 1) Lsum += __shfl_xor(Lsum, off);
    if (lane == 0) {
        stats[2 * i] = M;
        stats[2 * i + 1] = Lsum > 0.f ? 1.0f / Lsum : 0.f;
    }
}

__global__ void probe_final_kernel(const float* __restrict__ part, float* __restrict__ S, int64_t N, int64_t Np, int Hkv,
                                   float inv_rows) {
    int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    float acc = 0.f;
    for (int g = 0; g < Hkv; ++g) acc += part[(int64_t)g * Np + n];
    S[n] = acc * inv_rows;
}

static inline int probe_rp(int P, int H, int Hkv) { int R = P * (H / Hkv); return (R + 127) / 128 * 128; }

size_t probe_scratch_floats(int64_t N, int P, int H, int Hkv) {
    // generic path: stats [P*H, 2].  Matrix-core path: stats_part [nchunks][Hkv][Rp][2] + stats [Hkv][Rp][2]
    // + part [Hkv][Np]
    int64_t Np = (N + 255) / 256 * 256;
    int64_t nchunks = (N + CHUNK - 1) / CHUNK;
    int64_t Rp = probe_rp(P, H, Hkv);
    const size_t windowed = (size_t)(2 * (int64_t)P * H + 64) + (size_t)(nchunks * Hkv * Rp * 2 + Hkv * Rp * 2 + Hkv * Np + 256);
    const size_t single = probe_p1_scratch_floats(N, H);   // the single-row probe uses the same region from its start
    return windowed > single ? windowed : single;
}

bool probe_mfma_supported(const ProbeArgs& a) {
    if (a.d != 128 && a.d != 64) return false;
    if (a.N <= 0 || a.P <= 0 || a.H % a.Hkv != 0) return false;
    if (probe_rp(a.P, a.H, a.Hkv) > 512) return false;
    auto al = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    return al(a.qp) && al(a.k);
}

template <int D, int RB, int NWV = 4>
static hipError_t launch_probe_t(const ProbeArgs& a, int Rp, hipStream_t s) {
    const int64_t Np = (a.N + 255) / 256 * 256;
    const int nchunks = (int)((a.N + CHUNK - 1) / CHUNK);
    const int R = a.P * (a.H / a.Hkv);
    float* stats_part = a.partial;
    float* stats = stats_part + (size_t)nchunks * a.Hkv * Rp * 2;
    float* part = stats + (size_t)a.Hkv * Rp * 2;
    ProbeArgs b = a;
    b.partial = part;
    const float want = attention_mfma_q_scale(D);
    const float qmul = (a.q_scale != 0.f) ? want / a.q_scale : want;   // exactly 1 when the producer applied `want`
    dim3 grid(nchunks, a.Hkv), block(256), pblock(64 * NWV);
    probe_mfma_kernel<D, RB, 1, NWV><<<grid, pblock, 0, s>>>(b, Rp, Np, qmul, stats_part, nullptr);
    probe_combine_kernel<<<dim3((a.Hkv * Rp + 3) / 4), block, 0, s>>>(stats_part, stats, nchunks, a.Hkv, Rp, R);
    probe_mfma_kernel<D, RB, 2, NWV><<<grid, pblock, 0, s>>>(b, Rp, Np, qmul, nullptr, stats);
    probe_final_kernel<<<dim3((unsigned)((a.N + 255) / 256)), block, 0, s>>>(part, a.S, a.N, Np, a.Hkv, 1.0f / (float)(a.P * a.H));
    return hipGetLastError();
}

hipError_t launch_probe_mfma(const ProbeArgs& a, hipStream_t s) {
    const int Rp = probe_rp(a.P, a.H, a.Hkv);
    const int rb = Rp / 128;
    if (a.d == 128) {
        if (rb == 1) return launch_probe_t<128, 1>(a, Rp, s);
        if (rb == 2) return launch_probe_t<128, 2>(a, Rp, s);
        if (rb == 3) return launch_probe_t<128, 3>(a, Rp, s);
        return launch_probe_t<128, 2, 8>(a, Rp, s);   // 512 rows: 8 wavefronts x 64 rows keep two wavefronts per SIMD
    }
    if (rb == 1) return launch_probe_t<64, 1>(a, Rp, s);
    if (rb == 2) return launch_probe_t<64, 2>(a, Rp, s);
    if (rb == 3) return launch_probe_t<64, 3>(a, Rp, s);
    return launch_probe_t<64, 2, 8>(a, Rp, s);
}

}  // namespace spts
