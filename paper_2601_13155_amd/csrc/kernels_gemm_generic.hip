// Shape-agnostic C = A * B^T (A [M,K] rows optionally gathered, B [N,K]) with fp32 accumulation and
// the SPTS epilogues.  Serves the fp32 configuration and any shape the matrix-core kernel does not
// take (dimensions that are not tile multiples).  64x64 output tile, 256 threads, 4x4 per thread.
#include "spts_internal.h"

namespace spts {

constexpr int GT = 64;   // tile edge
constexpr int GK = 16;   // k step

template <typename T, bool DUAL>
__global__ void __launch_bounds__(256) gemm_generic_kernel(GemmArgs a) {
    __shared__ float As[GK][GT + 1];
    __shared__ float Bs[GK][GT + 1];
    __shared__ float Bs1[DUAL ? GK : 1][GT + 1];
    __shared__ float As1[DUAL ? GK : 1][GT + 1];
    __shared__ float red[GT][17];

    const T* A = (const T*)a.A;
    const T* A1 = a.A1 ? (const T*)a.A1 : A;
    const T* B0 = (const T*)a.B0;
    const T* B1 = (const T*)a.B1;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t row0 = (int64_t)blockIdx.y * GT;
    const int col0 = blockIdx.x * GT;

    float acc[4][4] = {}, acc1[4][4] = {};

    // loader mapping: thread loads element (r = tid / 16 + 16 * i, kk = tid % 16)
    const int lk = threadIdx.x & 15, lr = threadIdx.x >> 4;
    for (int k0 = 0; k0 < a.K; k0 += GK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int r = lr + 16 * i;
            int64_t grow = row0 + r;
            int kk = k0 + lk;
            float va = 0.f, va1 = 0.f, vb = 0.f, vb1 = 0.f;
            if (grow < a.M && kk < a.K) {
                int64_t srow = a.a_idx ? (int64_t)a.a_idx[grow] : grow;
                va = to_f32(A[srow * a.lda + kk]);
                if (DUAL) va1 = to_f32(A1[srow * a.lda + kk]);
            }
            int gcol = col0 + r;
            if (gcol < a.N && kk < a.K) {
                vb = to_f32(B0[(int64_t)gcol * a.ldb + kk]);
                if (DUAL) vb1 = to_f32(B1[(int64_t)gcol * a.ldb + kk]);
            }
            As[lk][r] = va;
            Bs[lk][r] = vb;
            if (DUAL) { Bs1[lk][r] = vb1; As1[lk][r] = va1; }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GK; ++kk) {
            float av[4], av1[4], bv[4], bv1[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { av[i] = As[kk][ty * 4 + i]; bv[i] = Bs[kk][tx * 4 + i]; if (DUAL) { bv1[i] = Bs1[kk][tx * 4 + i]; av1[i] = As1[kk][ty * 4 + i]; } }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
                    if (DUAL) acc1[i][j] = fmaf(av1[i], bv1[j], acc1[i][j]);
                }
        }
        __syncthreads();
    }

    if (a.epi == EPI_SUMSQ) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float ssq = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) { int gcol = col0 + tx * 4 + j; if (gcol < a.N) ssq += acc[i][j] * acc[i][j]; }
            red[ty * 4 + i][tx] = ssq;
        }
        __syncthreads();
        if (threadIdx.x < GT) {
            int64_t grow = row0 + threadIdx.x;
            if (grow < a.M) {
                float t = 0.f;
                for (int j = 0; j < 16; ++j) t += red[threadIdx.x][j];
                a.part[grow * a.part_ld + blockIdx.x] = t;
            }
        }
        return;
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int64_t grow = row0 + ty * 4 + i;
        if (grow >= a.M) continue;
        int64_t crow = a.c_idx ? (int64_t)a.c_idx[grow] : grow;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int gcol = col0 + tx * 4 + j;
            if (gcol >= a.N) continue;
            float v = acc[i][j];
            if (DUAL) { float g = v; v = g / (1.0f + expf(-g)) * acc1[i][j]; }
            if (a.epi == EPI_RESIDUAL) {
                T* c = (T*)a.C + crow * a.ldc + gcol;
                *c = from_f32<T>(to_f32(*c) + v);
            } else if (a.c_is_f32) {
                ((float*)a.C)[crow * a.ldc + gcol] = v;
            } else {
                T o = from_f32<T>(v);
                ((T*)a.C)[crow * a.ldc + gcol] = o;
                if (a.Ct) ((T*)a.Ct)[(int64_t)gcol * a.ldct + vt_key_slot(grow)] = o;
            }
        }
    }
}

hipError_t launch_gemm_generic(const GemmArgs& a, bool bf16, hipStream_t s) {
    if (a.M == 0 || a.N == 0) return hipSuccess;
    dim3 grid((unsigned)((a.N + GT - 1) / GT), (unsigned)((a.M + GT - 1) / GT)), block(256);
    bool dual = a.epi == EPI_SILU_MUL;
    if (bf16) {
        if (dual) gemm_generic_kernel<bf16_t, true><<<grid, block, 0, s>>>(a);
        else gemm_generic_kernel<bf16_t, false><<<grid, block, 0, s>>>(a);
    } else {
        if (dual) gemm_generic_kernel<float, true><<<grid, block, 0, s>>>(a);
        else gemm_generic_kernel<float, false><<<grid, block, 0, s>>>(a);
    }
    return hipGetLastError();
}

}  // namespace spts
