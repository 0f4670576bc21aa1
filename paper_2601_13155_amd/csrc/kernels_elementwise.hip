// Memory-bound helpers of the SPTS layer: rotary tables, RMSNorm, rotary application, row
// gather / scatter maps, score finishing.  All are HBM-bound streaming kernels: 16-byte accesses,
// one pass over the data.
#include "spts_internal.h"

#include <mutex>
#include <set>
#include <utility>

namespace spts {

static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

hipError_t ensure_dynamic_lds(const void* kernel, int bytes) {
    static std::mutex mtx;
    static std::set<std::pair<int, const void*>> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mtx);
    if (done.count({dev, kernel})) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.insert({dev, kernel});
    return e;
}

// ---------------------------------------------------------------- rotary table
// table[n, j] = (cos, sin)(pos[n] * base^(-2j/d)), j < d/2.  Angles are formed in fp64 so that
// positions up to 2^17 and beyond keep full fp32 accuracy in the stored cos/sin.
__global__ void rope_table_kernel(const int32_t* __restrict__ pos, int64_t N, int half, double neg2_over_d_log2base,
                                  float2* __restrict__ table) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N * half) return;
    int64_t n = i / half;
    int j = (int)(i - n * half);
    double theta = exp2((double)j * neg2_over_d_log2base);
    double ang = (double)pos[n] * theta;
    double s, c;
    sincos(ang, &s, &c);
    table[i] = make_float2((float)c, (float)s);
}

hipError_t launch_rope_table(const int32_t* pos, int64_t N, int d, float base, float2* table, hipStream_t s) {
    if (N == 0) return hipSuccess;
    int half = d / 2;
    double k = -2.0 / (double)d * log2((double)base);
    int64_t total = N * half;
    rope_table_kernel<<<dim3((unsigned)cdiv(total, 256)), dim3(256), 0, s>>>(pos, N, half, k, table);
    return hipGetLastError();
}

// ---------------------------------------------------------------- RMSNorm
// One workgroup of 256 threads per row; the row is read once into registers (D <= 256*32).
template <typename T> struct Vec16;
template <> struct Vec16<float> { static constexpr int n = 4; };
template <> struct Vec16<bf16_t> { static constexpr int n = 8; };

template <typename T>
__global__ void __launch_bounds__(256) rmsnorm_kernel(const T* __restrict__ x, const T* __restrict__ gamma, float eps,
                                                      T* __restrict__ out, int64_t N, int D) {
    constexpr int VN = Vec16<T>::n;
    constexpr int MAXV = 4;  // up to 4 vectors of 16 bytes per thread
    int64_t row = blockIdx.x;
    const T* xr = x + row * (int64_t)D;
    T* orow = out + row * (int64_t)D;
    float vals[MAXV * VN];
    int nvec = D / VN;  // host guarantees D % VN == 0 and nvec <= 256 * MAXV
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < MAXV; ++it) {
        int v = threadIdx.x + it * 256;
        if (v < nvec) {
            uint4 raw = *reinterpret_cast<const uint4*>(xr + (int64_t)v * VN);
            const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
            for (int q = 0; q < VN; ++q) { float f = to_f32(e[q]); vals[it * VN + q] = f; ss += f * f; }
        }
    }
    // block reduction
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    __shared__ float wsum[4];
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    float inv = 1.0f / sqrtf(tot / (float)D + eps);
#pragma unroll
    for (int it = 0; it < MAXV; ++it) {
        int v = threadIdx.x + it * 256;
        if (v < nvec) {
            uint4 graw = *reinterpret_cast<const uint4*>(gamma + (int64_t)v * VN);
            const T* g = reinterpret_cast<const T*>(&graw);
            uint4 o;
            T* oe = reinterpret_cast<T*>(&o);
#pragma unroll
            for (int q = 0; q < VN; ++q) oe[q] = from_f32<T>(vals[it * VN + q] * inv * to_f32(g[q]));
            *reinterpret_cast<uint4*>(orow + (int64_t)v * VN) = o;
        }
    }
}

// generic fallback for any D (scalar accesses)
template <typename T>
__global__ void __launch_bounds__(256) rmsnorm_any_kernel(const T* __restrict__ x, const T* __restrict__ gamma, float eps,
                                                          T* __restrict__ out, int64_t N, int D) {
    int64_t row = blockIdx.x;
    const T* xr = x + row * (int64_t)D;
    float ss = 0.f;
    for (int j = threadIdx.x; j < D; j += 256) { float f = to_f32(xr[j]); ss += f * f; }
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    __shared__ float wsum[4];
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    float inv = 1.0f / sqrtf(tot / (float)D + eps);
    for (int j = threadIdx.x; j < D; j += 256) out[row * (int64_t)D + j] = from_f32<T>(to_f32(xr[j]) * inv * to_f32(gamma[j]));
}

template <typename T>
static hipError_t rmsnorm_t(const void* x, const void* gamma, float eps, void* out, int64_t N, int D, hipStream_t s) {
    constexpr int VN = Vec16<T>::n;
    if (D % VN == 0 && D / VN <= 1024)
        rmsnorm_kernel<T><<<dim3((unsigned)N), dim3(256), 0, s>>>((const T*)x, (const T*)gamma, eps, (T*)out, N, D);
    else
        rmsnorm_any_kernel<T><<<dim3((unsigned)N), dim3(256), 0, s>>>((const T*)x, (const T*)gamma, eps, (T*)out, N, D);
    return hipGetLastError();
}

hipError_t launch_rmsnorm(const void* x, const void* gamma, float eps, void* out, int64_t N, int D, bool bf16, hipStream_t s) {
    if (N == 0) return hipSuccess;
    return bf16 ? rmsnorm_t<bf16_t>(x, gamma, eps, out, N, D, s) : rmsnorm_t<float>(x, gamma, eps, out, N, D, s);
}

// ---------------------------------------------------------------- rotary application
// in: fp32 [n, heads*d] (projection accumulators); out: T [n, heads*d].
template <typename T>
__global__ void rope_apply_kernel(const float* __restrict__ in, const float2* __restrict__ table,
                                  const int32_t* __restrict__ idx, int64_t row0, T* __restrict__ out, int64_t n,
                                  int heads, int d, float scale) {
    int half = d >> 1;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = n * heads * half;
    if (i >= total) return;
    int j = (int)(i % half);
    int64_t t = i / half;
    int h = (int)(t % heads);
    int64_t row = t / heads;
    int64_t trow = idx ? (int64_t)idx[row] : row + row0;
    float2 cs = table[trow * half + j];
    int64_t base = (row * heads + h) * (int64_t)d;
    float a = in[base + j], b = in[base + j + half];
    out[base + j] = from_f32<T>((a * cs.x - b * cs.y) * scale);
    out[base + j + half] = from_f32<T>((b * cs.x + a * cs.y) * scale);
}

hipError_t launch_rope_apply(const float* in, const float2* table, const int32_t* idx, int64_t row0, void* out,
                             int64_t n, int heads, int d, bool bf16, hipStream_t s, float scale) {
    if (n == 0) return hipSuccess;
    int64_t total = n * heads * (d / 2);
    dim3 g((unsigned)cdiv(total, 256)), b(256);
    if (bf16) rope_apply_kernel<bf16_t><<<g, b, 0, s>>>(in, table, idx, row0, (bf16_t*)out, n, heads, d, scale);
    else rope_apply_kernel<float><<<g, b, 0, s>>>(in, table, idx, row0, (float*)out, n, heads, d, scale);
    return hipGetLastError();
}

// ---------------------------------------------------------------- row gather / copies
// One wave per row chunk: rows are contiguous so every access is a full 16-byte lane access.
__global__ void __launch_bounds__(256) gather_rows16_kernel(const uint4* __restrict__ in, const int32_t* __restrict__ idx,
                                                            uint4* __restrict__ out, int64_t n, int64_t row_vec) {
    int64_t row = blockIdx.x;
    const uint4* src = in + (int64_t)idx[row] * row_vec;
    uint4* dst = out + row * row_vec;
    for (int64_t v = threadIdx.x; v < row_vec; v += 256) dst[v] = src[v];
}
__global__ void __launch_bounds__(256) gather_rows4_kernel(const uint32_t* __restrict__ in, const int32_t* __restrict__ idx,
                                                           uint32_t* __restrict__ out, int64_t n, int64_t row_words) {
    int64_t row = blockIdx.x;
    const uint32_t* src = in + (int64_t)idx[row] * row_words;
    uint32_t* dst = out + row * row_words;
    for (int64_t v = threadIdx.x; v < row_words; v += 256) dst[v] = src[v];
}

hipError_t launch_gather_rows(const void* in, const int32_t* idx, void* out, int64_t n, int64_t row_bytes, hipStream_t s) {
    if (n == 0) return hipSuccess;
    if (row_bytes % 16 == 0)
        gather_rows16_kernel<<<dim3((unsigned)n), dim3(256), 0, s>>>((const uint4*)in, idx, (uint4*)out, n, row_bytes / 16);
    else
        gather_rows4_kernel<<<dim3((unsigned)n), dim3(256), 0, s>>>((const uint32_t*)in, idx, (uint32_t*)out, n, row_bytes / 4);
    return hipGetLastError();
}

// Row gather with its bookkeeping in one launch: out[i, :] = in[idx[i], :] and, where wanted, pos_out[i] = pos_in[idx[i]]
// and old2new[idx[i]] = i.  A workgroup takes 1024 16-byte vectors (8 rows of 2 KB, 2 rows of 8 KB, ...): every lane has
// four independent loads (64 bytes) in flight before its first store.
__global__ void __launch_bounds__(256) gather_rows_maps_kernel(const u32x4* __restrict__ in, const int32_t* __restrict__ idx,
                                                               u32x4* __restrict__ out, int64_t n, int row_vec, int rows_per_wg,
                                                               const int32_t* __restrict__ pos_in, int32_t* __restrict__ pos_out,
                                                               int32_t* __restrict__ old2new) {
    const int64_t row0 = (int64_t)blockIdx.x * rows_per_wg;
    const int total = rows_per_wg * row_vec;      // vectors of this workgroup (<= 1024, or one row of any length)
    for (int base = 0; base < total; base += 1024) {
        u32x4 v[4];
        int64_t dst[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = base + u * 256 + (int)threadIdx.x;
            const int r = e / row_vec, c = e - r * row_vec;
            const int64_t row = row0 + r;
            dst[u] = -1;
            if (e < total && row < n) {
                v[u] = in[(int64_t)idx[row] * row_vec + c];
                dst[u] = row * row_vec + c;
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (dst[u] >= 0) out[dst[u]] = v[u];
    }
    if ((int)threadIdx.x < rows_per_wg) {
        const int64_t row = row0 + threadIdx.x;
        if (row < n) {
            const int32_t src = idx[row];
            if (pos_out) pos_out[row] = pos_in[src];
            if (old2new) old2new[src] = (int32_t)row;
        }
    }
}

hipError_t launch_gather_rows_maps(const void* in, const int32_t* idx, void* out, int64_t n, int64_t row_bytes,
                                   const int32_t* pos_in, int32_t* pos_out, int32_t* old2new, hipStream_t s) {
    if (n == 0) return hipSuccess;
    if (row_bytes % 16 != 0 || row_bytes / 16 > (int64_t)1 << 24) return hipErrorInvalidValue;
    const int row_vec = (int)(row_bytes / 16);
    int rows_per_wg = 1024 / row_vec;
    if (rows_per_wg < 1) rows_per_wg = 1;
    if (rows_per_wg > 256) rows_per_wg = 256;
    gather_rows_maps_kernel<<<dim3((unsigned)cdiv(n, rows_per_wg)), dim3(256), 0, s>>>((const u32x4*)in, idx, (u32x4*)out, n, row_vec,
                                                                                     rows_per_wg, pos_in, pos_out, old2new);
    return hipGetLastError();
}

__global__ void gather_i32_kernel(const int32_t* __restrict__ in, const int32_t* __restrict__ idx, int32_t* __restrict__ out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = in[idx[i]];
}
hipError_t launch_gather_i32(const int32_t* in, const int32_t* idx, int32_t* out, int64_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    gather_i32_kernel<<<dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s>>>(in, idx, out, n);
    return hipGetLastError();
}

__global__ void copy16_kernel(const uint4* __restrict__ in, uint4* __restrict__ out, int64_t nvec) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < nvec; i += stride) out[i] = in[i];
}
__global__ void copy4_kernel(const uint32_t* __restrict__ in, uint32_t* __restrict__ out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) out[i] = in[i];
}
hipError_t launch_copy_bytes(const void* in, void* out, int64_t bytes, hipStream_t s) {
    if (bytes == 0) return hipSuccess;
    if (bytes % 16 == 0) {
        int64_t nv = bytes / 16;
        int64_t blocks = cdiv(nv, 256); if (blocks > 8192) blocks = 8192;
        copy16_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const uint4*)in, (uint4*)out, nv);
    } else {
        int64_t nw = bytes / 4;
        int64_t blocks = cdiv(nw, 256); if (blocks > 8192) blocks = 8192;
        copy4_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const uint32_t*)in, (uint32_t*)out, nw);
    }
    return hipGetLastError();
}

__global__ void fill_i32_kernel(int32_t* p, int32_t v, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
hipError_t launch_fill_i32(int32_t* p, int32_t v, int64_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    fill_i32_kernel<<<dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s>>>(p, v, n);
    return hipGetLastError();
}
__global__ void iota_i32_kernel(int32_t* p, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = (int32_t)i;
}
hipError_t launch_iota_i32(int32_t* p, int64_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    iota_i32_kernel<<<dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s>>>(p, n);
    return hipGetLastError();
}
// idx[i] += seg_offsets[b] for the segment b whose output range [out_offsets[b], out_offsets[b+1]) holds i
// (per-sequence TopK writes indices relative to its sequence; the batched layer wants rows of the batch)
__global__ void add_segment_base_kernel(int32_t* __restrict__ idx, const int64_t* __restrict__ out_offsets,
                                        const int64_t* __restrict__ seg_offsets, int nseg, int64_t total) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int lo = 0, hi = nseg;   // last b with out_offsets[b] <= i
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (out_offsets[mid] <= i) lo = mid; else hi = mid;
    }
    idx[i] += (int32_t)seg_offsets[lo];
}
// dst[first + i] = chunk.v[i] for i < chunk.n: host integers travel as kernel arguments (captured by value at launch,
// so the host array may die as soon as the call returns, and nothing is staged or synchronised)
__global__ void write_i64_kernel(I64Chunk chunk, int64_t* __restrict__ dst, int64_t first) {
    const int i = threadIdx.x;
    if (i < chunk.n) dst[first + i] = chunk.v[i];
}

hipError_t launch_write_i64(const int64_t* host_vals, int64_t n, int64_t* dst, hipStream_t s) {
    for (int64_t first = 0; first < n; first += I64Chunk::CAP) {
        I64Chunk c;
        c.n = (int32_t)(n - first < I64Chunk::CAP ? n - first : I64Chunk::CAP);
        for (int i = 0; i < c.n; ++i) c.v[i] = host_vals[first + i];
        write_i64_kernel<<<dim3(1), dim3(I64Chunk::CAP), 0, s>>>(c, dst, first);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_add_segment_base(int32_t* idx, const int64_t* out_offsets, const int64_t* seg_offsets, int nseg, int64_t total,
                                   hipStream_t s) {
    if (total <= 0 || nseg <= 0) return hipSuccess;
    add_segment_base_kernel<<<dim3((unsigned)cdiv(total, 256)), dim3(256), 0, s>>>(idx, out_offsets, seg_offsets, nseg, total);
    return hipGetLastError();
}

__global__ void scatter_iota_kernel(const int32_t* __restrict__ idx, int32_t* __restrict__ old2new, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) old2new[idx[i]] = (int32_t)i;
}
hipError_t launch_scatter_iota(const int32_t* idx, int32_t* old2new, int64_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    scatter_iota_kernel<<<dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s>>>(idx, old2new, n);
    return hipGetLastError();
}

// ---------------------------------------------------------------- LTP score finishing
__global__ void finish_ffn_scores_kernel(const float* __restrict__ part, int nparts, const float* __restrict__ s_mha,
                                         float* __restrict__ c_ffn, float* __restrict__ s_ffn, int64_t N) {
    int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    float acc = 0.f;
    for (int j = 0; j < nparts; ++j) acc += part[n * nparts + j];  // fixed order: deterministic
    float c = sqrtf(acc);
    if (c_ffn) c_ffn[n] = c;
    if (s_ffn) s_ffn[n] = s_mha ? c * s_mha[n] : c;
}
hipError_t launch_finish_ffn_scores(const float* part, int nparts, const float* s_mha, float* c_ffn, float* s_ffn,
                                    int64_t N, hipStream_t s) {
    if (N == 0) return hipSuccess;
    finish_ffn_scores_kernel<<<dim3((unsigned)cdiv(N, 256)), dim3(256), 0, s>>>(part, nparts, s_mha, c_ffn, s_ffn, N);
    return hipGetLastError();
}

// C[n] = || z[n, :] ||_2 (and S^FFN = C * S^MHA): the proxy's output norm when U_down has orthonormal columns.  One
// wavefront per row, lane l takes elements l, l + 64, ...; a fixed shuffle tree (deterministic).
template <typename T>
__global__ void __launch_bounds__(256) row_norm_scores_kernel(const T* __restrict__ z, int r, const float* __restrict__ s_mha,
                                                              float* __restrict__ c_ffn, float* __restrict__ s_ffn, int64_t N) {
    const int lane = threadIdx.x & 63;
    const int64_t n = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const T* row = z + n * (int64_t)r;
    float acc = 0.f;
    if (r % 4 == 0) {   // rows are then whole groups of four elements, aligned to their size (z is 16-byte aligned)
        for (int j = lane * 4; j < r; j += 256) {
            float v[4];
            if (sizeof(T) == 2) {
                const uint2 raw = *reinterpret_cast<const uint2*>(row + j);
                v[0] = __uint_as_float(raw.x << 16); v[1] = __uint_as_float(raw.x & 0xffff0000u);
                v[2] = __uint_as_float(raw.y << 16); v[3] = __uint_as_float(raw.y & 0xffff0000u);
            } else {
                const float4 raw = *reinterpret_cast<const float4*>(row + j);
                v[0] = raw.x; v[1] = raw.y; v[2] = raw.z; v[3] = raw.w;
            }
            acc += v[0] * v[0]; acc += v[1] * v[1]; acc += v[2] * v[2]; acc += v[3] * v[3];
        }
    } else {
        for (int j = lane; j < r; j += 64) { const float v = to_f32(row[j]); acc += v * v; }
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0) {
        const float c = sqrtf(acc);
        if (c_ffn) c_ffn[n] = c;
        if (s_ffn) s_ffn[n] = s_mha ? c * s_mha[n] : c;
    }
}
hipError_t launch_row_norm_scores(const void* z, int r, bool bf16, const float* s_mha, float* c_ffn, float* s_ffn, int64_t N,
                                  hipStream_t s) {
    if (N == 0) return hipSuccess;
    dim3 g((unsigned)cdiv(N, 4)), b(256);
    if (bf16) row_norm_scores_kernel<bf16_t><<<g, b, 0, s>>>((const bf16_t*)z, r, s_mha, c_ffn, s_ffn, N);
    else row_norm_scores_kernel<float><<<g, b, 0, s>>>((const float*)z, r, s_mha, c_ffn, s_ffn, N);
    return hipGetLastError();
}

// ---------------------------------------------------------------- transpose with zero padding
// v [M, C] -> vt [C, ldvt] (keys in vt_key_slot order); 32x32 tiles through LDS so both sides are coalesced.
template <typename T>
__global__ void __launch_bounds__(256) transpose_pad_kernel(const T* __restrict__ v, T* __restrict__ vt, int64_t M, int C, int64_t ldvt) {
    __shared__ T tile[32][33];
    int64_t i0 = (int64_t)blockIdx.x * 32;
    int c0 = blockIdx.y * 32;
    int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        int64_t i = i0 + r; int c = c0 + tx;
        T val = from_f32<T>(0.f);
        if (i < M && c < C) val = v[i * C + c];
        tile[r][tx] = val;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        int c = c0 + r; int64_t i = i0 + tx;
        if (c < C && i < ldvt) vt[(int64_t)c * ldvt + vt_key_slot(i)] = tile[tx][r];
    }
}
hipError_t launch_transpose_pad(const void* v, void* vt, int64_t M, int C, int64_t ldvt, bool bf16, hipStream_t s) {
    if (ldvt == 0 || C == 0) return hipSuccess;
    dim3 g((unsigned)cdiv(ldvt, 32), (unsigned)cdiv(C, 32)), b(256);
    if (bf16) transpose_pad_kernel<bf16_t><<<g, b, 0, s>>>((const bf16_t*)v, (bf16_t*)vt, M, C, ldvt);
    else transpose_pad_kernel<float><<<g, b, 0, s>>>((const float*)v, (float*)vt, M, C, ldvt);
    return hipGetLastError();
}

// ---------------------------------------------------------------- slab-major copy of a row-major matrix
// out[(s * rows + r) * 32 + j] = W[r * K + 32 * s + j] (2-byte elements, K % 32 == 0): the 32 columns of K slab s of
// consecutive rows lie next to each other, 64 bytes per row.  One thread per 16-byte chunk.
__global__ void __launch_bounds__(256) pack_slab32_kernel(const u32x4* __restrict__ W, int64_t rows, int64_t chunks_per_row,
                                                          u32x4* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= rows * chunks_per_row) return;
    const int64_t r = i / chunks_per_row, c = i % chunks_per_row;
    out[((c >> 2) * rows + r) * 4 + (c & 3)] = W[i];
}

hipError_t launch_pack_slab32(const void* W, int64_t rows, int64_t K, void* out, hipStream_t s) {
    if (rows <= 0 || K <= 0 || K % 32 != 0) return hipErrorInvalidValue;
    const int64_t n = rows * (K / 8);
    pack_slab32_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>((const u32x4*)W, rows, K / 8, (u32x4*)out);
    return hipGetLastError();
}

}  // namespace spts
