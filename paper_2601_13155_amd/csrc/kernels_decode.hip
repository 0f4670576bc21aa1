// Decode phase over the per-layer KV caches left by the token-skipped prefill (Alg. 1 with
// Is_prefill_phase() false: both branches dense for the one new token; Sec. 3.2 last paragraph and
// the appendix on KV-cache flexibility say what a cache holds: the active pairs of the prefill plus
// every decoded token's pair).
//
// One token means every contraction is a matrix-vector product whose cost is reading the weights
// once, so the whole step is HBM-bound (8B-shaped model: 13.9 GB of bf16 weights per token):
//   * gemv_kernel: y = W x with W [R, K] row-major.  A workgroup of 4 wavefronts owns 2 rows (a gate
//     and an up row for the SwiGLU variant; 4 rows for Q/K/V) and splits K across its 256 lanes in
//     16-byte chunks, with several independent 16-byte weight loads per lane in flight before the first use; bf16
//     pairs are multiplied with v_dot2c_f32_bf16 (fp32 accumulate, no conversion instructions).
//     Lanes reduce by shuffles, wavefronts through LDS.  Up to three matrices that share x run as
//     one launch (Q, K, V).  Epilogues: store, SiLU(gate)*up, residual add, fp32 store (logits).
//   * decode_attn_kernel: flash-decoding.  Grid = (key splits, KV heads); 64/LPK keys per wavefront
//     step (LPK lanes hold one key row as 16-byte pieces), every lane group keeps its own running
//     (max, sum, weighted values) for all query heads of the KV head; groups, wavefronts and splits
//     are merged with the usual (max, sum) algebra in a fixed order (deterministic).
//   * small kernels: rotary embedding of q / k for the new position + cache append, merge of the
//     splits, argmax with ties to the lowest token id, table row gather.
#include "spts_internal.h"
#include "spts_lanes.h"

namespace spts {

// ------------------------------------------------------------------------------------------- GEMV
// 16-byte chunk of T -> chunk of T holding from_f32(x[e] * inv * gamma[e]) (RMSNorm's last step)
__device__ inline u32x4 norm_chunk(u32x4 xv, u32x4 gv, float inv, bf16_t) {
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float x0 = __uint_as_float(xv[i] << 16), x1 = __uint_as_float(xv[i] & 0xffff0000u);
        const float g0 = __uint_as_float(gv[i] << 16), g1 = __uint_as_float(gv[i] & 0xffff0000u);
        o[i] = (uint32_t)f32_to_bf16(x0 * inv * g0).v | ((uint32_t)f32_to_bf16(x1 * inv * g1).v << 16);
    }
    return o;
}
__device__ inline u32x4 norm_chunk(u32x4 xv, u32x4 gv, float inv, float) {
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = __float_as_uint(__uint_as_float(xv[i]) * inv * __uint_as_float(gv[i]));
    return o;
}
__device__ inline float chunk_sumsq(u32x4 v, bf16_t) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float a = __uint_as_float(v[i] << 16), b = __uint_as_float(v[i] & 0xffff0000u);
        s += a * a; s += b * b;
    }
    return s;
}
__device__ inline float chunk_sumsq(u32x4 v, float) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) { const float a = __uint_as_float(v[i]); s += a * a; }
    return s;
}

template <typename T, int MODE, bool NORM>
__global__ void __launch_bounds__(256) gemv_kernel(GemvArgs a) {
    constexpr int EPC = 16 / (int)sizeof(T);          // elements per 16-byte chunk
    constexpr int ROWS = (MODE == GEMV_RESID) ? 2 : (MODE == GEMV_SILU) ? 2 : 4;   // dot products per workgroup
    constexpr int NCH = 4;                            // chunks of x a lane may hold (fused norm)
    __shared__ float sred[4][ROWS];
    __shared__ float snorm[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // rows of this workgroup: ROWS consecutive rows of one matrix, or (SiLU) a gate row and the same up row.
    // Two rows per workgroup measured best where the epilogue allows it (O-proj 8.0 -> 7.5 us, down 19.7 -> 19.3 us,
    // gate/up 36.9 -> 35.3 us against four; one row and eight rows are slower); Q/K/V keep the four rows of two
    // rotary pairs
    const T* wrow[ROWS];
    int64_t out_row;      // first output element of this workgroup
    int which = 0;        // matrix the rows belong to
    if (MODE == GEMV_SILU) {
        out_row = (int64_t)blockIdx.x * (ROWS / 2);
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
            wrow[r] = (const T*)(r < ROWS / 2 ? a.W[0] : a.W[1]) + (out_row + (r % (ROWS / 2))) * a.K;
    } else if (MODE == GEMV_QKV_ROPE) {
        // Q and K blocks own the rows (j, j+1, j+d/2, j+d/2+1) of one head, so that both members of the
        // two rotary pairs are reduced by the same workgroup; V blocks own 4 consecutive rows
        int64_t blk = blockIdx.x;
        if (blk >= a.R[0] / 4) { blk -= a.R[0] / 4; which = 1; if (blk >= a.R[1] / 4) { blk -= a.R[1] / 4; which = 2; } }
        if (which < 2) {
            const int qd = a.head_dim / 4;                       // blocks per head
            out_row = (blk / qd) * a.head_dim + 2 * (blk % qd);  // j of the first pair
#pragma unroll
            for (int r = 0; r < ROWS; ++r)
                wrow[r] = (const T*)a.W[which] + (out_row + (r & 1) + (r >> 1) * (a.head_dim / 2)) * a.K;
        } else {
            out_row = blk * ROWS;
#pragma unroll
            for (int r = 0; r < ROWS; ++r) wrow[r] = (const T*)a.W[2] + (out_row + r) * a.K;
        }
    } else {
        int64_t row = (int64_t)blockIdx.x * ROWS;
        if (row >= a.R[0]) { row -= a.R[0]; which = 1; if (row >= a.R[1]) { row -= a.R[1]; which = 2; } }
        out_row = row;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) wrow[r] = (const T*)a.W[which] + (row + r) * a.K;
    }

    const int nchunks = a.K / EPC;
    const T* x = (const T*)a.x;
    float acc[ROWS];
    for (int r = 0; r < ROWS; ++r) acc[r] = 0.f;
    if (NORM) {
        // the weight loads do not depend on the norm: issue them first, then normalise x while they fly
        u32x4 wv[NCH][ROWS], xc[NCH], gc[NCH];
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int c = tid + 256 * i;
            if (c < nchunks) {
                xc[i] = *reinterpret_cast<const u32x4*>(x + (int64_t)c * EPC);
                gc[i] = *reinterpret_cast<const u32x4*>((const T*)a.gamma + (int64_t)c * EPC);
#pragma unroll
                for (int r = 0; r < ROWS; ++r) wv[i][r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wrow[r] + (int64_t)c * EPC));
            }
        }
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < NCH; ++i)
            if (tid + 256 * i < nchunks) ss += chunk_sumsq(xc[i], T{});
        ss = wave_sum(ss);
        if (lane == 0) snorm[wave] = ss;
        __syncthreads();
        const float inv = 1.0f / sqrtf((snorm[0] + snorm[1] + snorm[2] + snorm[3]) / (float)a.K + a.eps);
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int c = tid + 256 * i;
            if (c < nchunks) {
                const u32x4 xn = norm_chunk(xc[i], gc[i], inv, T{});
#pragma unroll
                for (int r = 0; r < ROWS; ++r) acc[r] = dot16(wv[i][r], xn, acc[r], T{});
            }
        }
    } else {
#pragma unroll 4
        for (int c = tid; c < nchunks; c += 256) {
            const u32x4 xv = *reinterpret_cast<const u32x4*>(x + (int64_t)c * EPC);
            u32x4 wv[ROWS];
#pragma unroll
            for (int r = 0; r < ROWS; ++r) wv[r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wrow[r] + (int64_t)c * EPC));
#pragma unroll
            for (int r = 0; r < ROWS; ++r) acc[r] = dot16(wv[r], xv, acc[r], T{});
        }
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        acc[r] = wave_sum(acc[r]);
        if (lane == 0) sred[wave][r] = acc[r];
    }
    __syncthreads();
    if (tid >= ROWS) return;
    const float v = sred[0][tid] + sred[1][tid] + sred[2][tid] + sred[3][tid];
    if (MODE == GEMV_SILU) {
        if (tid < ROWS / 2) {
            const float g = v;
            const float u = sred[0][tid + ROWS / 2] + sred[1][tid + ROWS / 2] + sred[2][tid + ROWS / 2] + sred[3][tid + ROWS / 2];
            const float h = g / (1.0f + __expf(-g)) * u;
            ((T*)a.y[0])[out_row + tid] = from_f32<T>(h);
        }
    } else if (MODE == GEMV_QKV_ROPE) {
        if (blockIdx.x == 0 && tid == 0 && a.pos_out) *a.pos_out = a.pos_val;
        if (which == 2) {
            ((T*)a.y[2])[out_row + tid] = from_f32<T>(v);
        } else {
            // tid: 0, 1 = first members (j, j+1), 2, 3 = their partners at +d/2
            const int half = a.head_dim / 2;
            const int j = (int)(out_row % a.head_dim) + (tid & 1);
            const float2 cs = a.rope[j];
            const float other = sred[0][tid ^ 2] + sred[1][tid ^ 2] + sred[2][tid ^ 2] + sred[3][tid ^ 2];
            const float res = tid < 2 ? v * cs.x - other * cs.y : v * cs.x + other * cs.y;
            ((T*)a.y[which])[out_row + (tid & 1) + (tid >> 1) * half] = from_f32<T>(res);
        }
    } else if (MODE == GEMV_RESID) {
        T* y = (T*)a.y[which] + out_row + tid;
        *y = from_f32<T>(to_f32(*y) + v);
    } else if (MODE == GEMV_F32) {
        ((float*)a.y[which])[out_row + tid] = v;
    } else {
        ((T*)a.y[which])[out_row + tid] = from_f32<T>(v);
    }
}

bool gemv_supported(const GemvArgs& a, bool bf16) {
    const int epc = bf16 ? 8 : 4;
    if (a.K <= 0 || a.K % epc != 0) return false;
    for (int i = 0; i < 3; ++i) {
        if (a.R[i] < 0 || a.R[i] % 4 != 0) return false;
        if (a.R[i] > 0 && (!a.W[i] || (reinterpret_cast<uintptr_t>(a.W[i]) & 15u))) return false;
    }
    if (!a.x || (reinterpret_cast<uintptr_t>(a.x) & 15u)) return false;
    if (a.gamma && ((reinterpret_cast<uintptr_t>(a.gamma) & 15u) || a.K / epc > 1024)) return false;
    return true;
}

template <typename T>
static hipError_t launch_gemv_t(const GemvArgs& a, hipStream_t s) {
    const int64_t rows = (int64_t)a.R[0] + a.R[1] + a.R[2];
    if (rows == 0) return hipSuccess;
    const dim3 b(256);
    const dim3 g((unsigned)(a.mode == GEMV_SILU ? a.R[0] : a.mode == GEMV_RESID ? rows / 2 : rows / 4));
    const bool n = a.gamma != nullptr;
    switch (a.mode) {
        case GEMV_STORE: if (n) gemv_kernel<T, GEMV_STORE, true><<<g, b, 0, s>>>(a); else gemv_kernel<T, GEMV_STORE, false><<<g, b, 0, s>>>(a); break;
        case GEMV_SILU: if (n) gemv_kernel<T, GEMV_SILU, true><<<g, b, 0, s>>>(a); else gemv_kernel<T, GEMV_SILU, false><<<g, b, 0, s>>>(a); break;
        case GEMV_RESID: if (n) return hipErrorInvalidValue; gemv_kernel<T, GEMV_RESID, false><<<g, b, 0, s>>>(a); break;
        case GEMV_F32: if (n) gemv_kernel<T, GEMV_F32, true><<<g, b, 0, s>>>(a); else gemv_kernel<T, GEMV_F32, false><<<g, b, 0, s>>>(a); break;
        case GEMV_QKV_ROPE:
            if (!a.rope || a.head_dim % 4 != 0 || a.R[0] % a.head_dim != 0 || a.R[1] % a.head_dim != 0) return hipErrorInvalidValue;
            if (n) gemv_kernel<T, GEMV_QKV_ROPE, true><<<g, b, 0, s>>>(a); else gemv_kernel<T, GEMV_QKV_ROPE, false><<<g, b, 0, s>>>(a);
            break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_gemv(const GemvArgs& a, bool bf16, hipStream_t s) {
    return bf16 ? launch_gemv_t<bf16_t>(a, s) : launch_gemv_t<float>(a, s);
}

// ------------------------------------------------------------------- GEMV over a few input vectors
// Y[b, r] = W[r, :] . X[b, :] for b < NB (a decode step over NB sequences): the weights are still read
// once, every weight chunk meets the NB input chunks in registers.  X [NB, K] and Y[i] [NB, R[i]] are
// row-major and contiguous.
// A wavefront owns RW rows on its own (RW/2 gate rows and the same up rows for the SiLU variant) and
// splits K over its 64 lanes; a workgroup is four such wavefronts on consecutive rows (they read the
// same input chunks at about the same time).  The RW*NB accumulators of a lane are reduced over the
// wavefront with a halving butterfly: at every step a lane hands half of its accumulators to its
// partner and adds the partner's other half, so 64 sums cost 63 exchanges instead of 64*6; lane
// (i << (6 - log2(RW*NB))) ends up with the total of accumulator i.
template <typename T, int MODE, int NB, int RW>
__global__ void __launch_bounds__(256) gemv_nb_kernel(GemvArgs a) {
    constexpr int EPC = 16 / (int)sizeof(T);
    constexpr int HR = RW / 2;
    constexpr int NA = RW * NB;                     // accumulators per lane (a power of two <= 64)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const T* wrow[RW];
    int64_t out_row;
    int which = 0;
    if (MODE == GEMV_SILU) {
        out_row = ((int64_t)blockIdx.x * 4 + wave) * HR;
#pragma unroll
        for (int r = 0; r < RW; ++r) wrow[r] = (const T*)(r < HR ? a.W[0] : a.W[1]) + (out_row + r % HR) * a.K;
    } else {
        int64_t row = ((int64_t)blockIdx.x * 4 + wave) * RW;
        if (row >= a.R[0]) { row -= a.R[0]; which = 1; if (row >= a.R[1]) { row -= a.R[1]; which = 2; } }
        out_row = row;
#pragma unroll
        for (int r = 0; r < RW; ++r) wrow[r] = (const T*)a.W[which] + (row + r) * a.K;
    }
    const int nchunks = a.K / EPC;
    const T* x = (const T*)a.x;
    float acc[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) acc[i] = 0.f;
#pragma unroll 2
    for (int c = lane; c < nchunks; c += 64) {
        u32x4 wv[RW], xv[NB];
#pragma unroll
        for (int r = 0; r < RW; ++r) wv[r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wrow[r] + (int64_t)c * EPC));
#pragma unroll
        for (int b = 0; b < NB; ++b) xv[b] = *reinterpret_cast<const u32x4*>(x + ((int64_t)b * a.K + (int64_t)c * EPC));
#pragma unroll
        for (int r = 0; r < RW; ++r)
#pragma unroll
            for (int b = 0; b < NB; ++b) acc[r * NB + b] = dot16(wv[r], xv[b], acc[r * NB + b], T{});
    }
    // halving butterfly over the 64 lanes
    int n = NA;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        if (n > 1) {
            const int half = n / 2;
            const bool up = (lane & off) != 0;
#pragma unroll
            for (int i = 0; i < NA / 2; ++i) {
                if (i < half) {
                    const float lo = acc[i], hi = acc[i + half];
                    acc[i] = (up ? hi : lo) + __shfl_xor(up ? lo : hi, off);
                }
            }
            n = half;
        } else {
            acc[0] += __shfl_xor(acc[0], off);
        }
    }
    constexpr int SH = NA == 64 ? 0 : NA == 32 ? 1 : NA == 16 ? 2 : NA == 8 ? 3 : NA == 4 ? 4 : NA == 2 ? 5 : 6;
    const float v = acc[0];
    const int idx = lane >> SH;                     // accumulator this lane holds the total of
    const int r = idx / NB, b = idx % NB;
    float u = 0.f;
    if (MODE == GEMV_SILU) u = __shfl(v, ((idx + HR * NB) % NA) << SH);   // the up row's total (read by the gate row's lane)
    if ((lane & ((1 << SH) - 1)) != 0) return;
    if (MODE == GEMV_SILU) {
        if (r < HR) ((T*)a.y[0])[(int64_t)b * a.R[0] + out_row + r] = from_f32<T>(v / (1.0f + __expf(-v)) * u);
    } else if (MODE == GEMV_RESID) {
        T* y = (T*)a.y[which] + (int64_t)b * a.R[which] + out_row + r;
        *y = from_f32<T>(to_f32(*y) + v);
    } else if (MODE == GEMV_F32) {
        ((float*)a.y[which])[(int64_t)b * a.R[which] + out_row + r] = v;
    } else {
        ((T*)a.y[which])[(int64_t)b * a.R[which] + out_row + r] = from_f32<T>(v);
    }
}

template <typename T, int NB, int RW>
static hipError_t launch_gemv_nb_tr(const GemvArgs& a, hipStream_t s) {
    const int64_t rows = (int64_t)a.R[0] + a.R[1] + a.R[2];
    const dim3 b(256);
    const dim3 g((unsigned)(a.mode == GEMV_SILU ? a.R[0] / (4 * (RW / 2)) : rows / (4 * RW)));
    switch (a.mode) {
        case GEMV_STORE: gemv_nb_kernel<T, GEMV_STORE, NB, RW><<<g, b, 0, s>>>(a); break;
        case GEMV_SILU: gemv_nb_kernel<T, GEMV_SILU, NB, RW><<<g, b, 0, s>>>(a); break;
        case GEMV_RESID: gemv_nb_kernel<T, GEMV_RESID, NB, RW><<<g, b, 0, s>>>(a); break;
        case GEMV_F32: gemv_nb_kernel<T, GEMV_F32, NB, RW><<<g, b, 0, s>>>(a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// rows per wavefront: 4 when every matrix has a multiple of 16 rows (8 outputs for the SiLU variant), else 2 (multiples
// of 8 / 4); row counts that divide neither are refused (the callers' shapes are multiples of 16)
template <typename T, int NB>
static hipError_t launch_gemv_nb_t(const GemvArgs& a, hipStream_t s) {
    const int64_t rows = (int64_t)a.R[0] + a.R[1] + a.R[2];
    if (rows == 0) return hipSuccess;
    auto divides = [&](int unit) { return a.R[0] % unit == 0 && a.R[1] % unit == 0 && a.R[2] % unit == 0; };
    const bool silu = a.mode == GEMV_SILU;
    if (divides(silu ? 8 : 16)) return launch_gemv_nb_tr<T, NB, 4>(a, s);
    if (divides(silu ? 4 : 8)) return launch_gemv_nb_tr<T, NB, 2>(a, s);
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------- the same on the matrix cores (bf16)
// Y[b, r] = W[r, :] . X[b, :] for up to 16 input vectors with v_mfma_f32_16x16x32_bf16: a weight row is an MFMA
// operand row (row = lane % 16, 8 consecutive k of group lane / 16) and an input vector is an operand column (lanes
// >= nb feed zeros).  No dot instructions, no lane reductions: the vector ALU only moves the 4 results per lane.
//
// The operand layout gives a row only 4 lanes, i.e. 64 bytes per load instruction, and weight streams read as
// half cache lines by two different instructions run at ~60 % of the rate of whole-line reads (measured: 4.1 against
// 6.4 TB/s on the 14336 x 4096 gate/up pair).  So the weights (and the input vectors, same shape: 16 rows with row
// stride K) go through LDS with direct-to-LDS loads whose lanes are laid out for memory, not for the matrix core:
// one instruction = 8 rows x one whole 128-byte line, two instructions = a 16-row strip x 64 k.  Fragments are then
// 16-byte LDS reads; the 16-byte chunk c of row r sits at slot c ^ (r >> 1) (the permutation is applied to the
// global addresses, since the hardware places lane l's 16 bytes at 16 * l), which spreads the 16 rows a fragment
// read touches over all banks.
//
// A workgroup of 4 wavefronts owns a strip of 16 rows (a gate strip and the same up strip for the SiLU variant)
// and splits K four ways (8 wavefronts with deeper or shallower rings measured the same or slower); every wavefront runs its own ring of DEPTH stages of 64 k (no workgroup barrier in the
// loop: a wavefront reads only what it loaded itself, after its own vmcnt wait).  The partial 16x16 tiles meet
// in LDS.  Needs K % 256 == 0 and row counts that are multiples of 16.
typedef __bf16 mfma_bf16x8 __attribute__((ext_vector_type(8)));
typedef float mfma_f32x4 __attribute__((ext_vector_type(4)));

constexpr int GEMV_MFMA_WAVES = 4;

template <int MODE, int XI>
__global__ void __launch_bounds__(GEMV_MFMA_WAVES * 64) gemv_mfma_kernel(GemvArgs a, int nb) {
    constexpr int NW = GEMV_MFMA_WAVES;
    constexpr int NS = MODE == GEMV_SILU ? 2 : 1;          // weight strips per workgroup (gate, up)
    constexpr int DEPTH = NS == 2 ? 3 : 4;                 // ring stages per wavefront (64 / 72 KB: two workgroups per CU)
    constexpr int NI = NS * 2 + XI;                        // direct-to-LDS loads per stage
    constexpr uint32_t STRIP_B = 2048, STAGE_B = (NS + 1) * STRIP_B, WAVE_B = DEPTH * STAGE_B;
    static_assert((DEPTH - 1) * NI <= 63, "vmcnt field");
    static_assert(NW * 64 >= 256 && (size_t)NW * WAVE_B >= (size_t)NW * NS * 16 * 17 * 4, "the partial tiles reuse the ring");
    extern __shared__ __attribute__((aligned(16))) char gsm[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, kg = lane >> 4;
    int64_t row0 = (int64_t)blockIdx.x * 16;
    int which = 0;
    const int nstage = a.K / (NW * 64);
    const int64_t kw = (int64_t)wave * nstage * 64;         // first k of this wavefront's contiguous share
    const char* wb[NS];
    if (MODE == GEMV_SILU) {
        wb[0] = (const char*)((const bf16_t*)a.W[0] + row0 * a.K + kw);
        wb[NS - 1] = (const char*)((const bf16_t*)a.W[1] + row0 * a.K + kw);
    } else {
        if (row0 >= a.R[0]) { row0 -= a.R[0]; which = 1; if (row0 >= a.R[1]) { row0 -= a.R[1]; which = 2; } }
        wb[0] = (const char*)((const bf16_t*)a.W[which] + row0 * a.K + kw);
    }
    const char* xb = (const char*)((const bf16_t*)a.x + kw);
    // load lanes: instruction j covers strip rows 8j .. 8j+7, lane -> (row 8j + lane / 8, slot lane % 8)
    uint32_t voff_w[2], voff_x[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = 8 * j + (lane >> 3), chunk = (lane & 7) ^ (r >> 1);
        const int xr = r < nb ? r : nb - 1;                 // rows beyond the batch: any valid row (their lanes feed zeros)
        voff_w[j] = (uint32_t)(((int64_t)r * a.K + chunk * 8) * 2);
        voff_x[j] = (uint32_t)(((int64_t)xr * a.K + chunk * 8) * 2);
    }
    const uint32_t ring = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)gsm + (uint32_t)wave * WAVE_B;
    auto issue = [&](int st) {                              // stage st -> ring slot st % DEPTH
        const uint32_t slot = ring + (uint32_t)(st % DEPTH) * STAGE_B;
        const int64_t koff = (int64_t)st * 128;
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int j = 0; j < 2; ++j) dma16s(voff_w[j], wb[s] + koff, slot + s * STRIP_B + j * 1024);
#pragma unroll
        for (int j = 0; j < XI; ++j) dma16s(voff_x[j], xb + koff, slot + NS * STRIP_B + j * 1024);
    };
    const int npre = nstage < DEPTH ? nstage : DEPTH;
    for (int st = 0; st < npre; ++st) issue(st);
    // fragment reads: lane (row l16, k group kg), half h of the stage -> chunk 4h + kg of its row
    const char* myring = gsm + (size_t)wave * WAVE_B;
    uint32_t foff[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) foff[h] = (uint32_t)(l16 * 128 + (((4 * h + kg) ^ (l16 >> 1)) * 16));
    const bool tok = l16 < nb;
    mfma_f32x4 acc[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) acc[s] = mfma_f32x4{0.f, 0.f, 0.f, 0.f};
    for (int st = 0; st < nstage; ++st) {
        // stages issued so far: min(nstage, st + DEPTH); all but the DEPTH - 1 youngest must have landed
        if (st + DEPTH <= nstage) SPTS_WAIT_VMCNT((DEPTH - 1) * NI); else SPTS_WAIT_VMCNT(0);
        asm volatile("" ::: "memory");
        const char* slot = myring + (size_t)(st % DEPTH) * STAGE_B;
        u32x4 wv[NS][2], xv[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int s = 0; s < NS; ++s) wv[s][h] = *reinterpret_cast<const u32x4*>(slot + s * STRIP_B + foff[h]);
            xv[h] = *reinterpret_cast<const u32x4*>(slot + NS * STRIP_B + foff[h]);
            if (!tok) xv[h] = u32x4{0u, 0u, 0u, 0u};
        }
        // the slot is refilled only after its fragments have arrived in registers
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (st + DEPTH < nstage) issue(st + DEPTH);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int s = 0; s < NS; ++s)
                acc[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(mfma_bf16x8, wv[s][h]),
                                                                 __builtin_bit_cast(mfma_bf16x8, xv[h]), acc[s], 0, 0, 0);
    }
    // every wavefront is done with its ring (nothing in flight: the last stage waited for vmcnt 0); the partial
    // tiles take its place.  Lane (token l16, row group kg) holds rows 4*kg .. 4*kg+3 of its tile.
    __syncthreads();
    float (*sred)[NS][16][17] = reinterpret_cast<float (*)[NS][16][17]>(gsm);
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int r = 0; r < 4; ++r) sred[wave][s][4 * kg + r][l16] = acc[s][r];
    __syncthreads();
    const int t = threadIdx.x;
    if (t >= 256) return;
    const int r = t >> 4, b = t & 15;
    if (b >= nb) return;
    float v = 0.f, u = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) { v += sred[w][0][r][b]; if (NS == 2) u += sred[w][NS - 1][r][b]; }
    if (MODE == GEMV_SILU) {
        ((bf16_t*)a.y[0])[(int64_t)b * a.R[0] + row0 + r] = f32_to_bf16(v / (1.0f + __expf(-v)) * u);
    } else if (MODE == GEMV_RESID) {
        bf16_t* y = (bf16_t*)a.y[which] + (int64_t)b * a.R[which] + row0 + r;
        *y = f32_to_bf16(bf16_to_f32(*y) + v);
    } else if (MODE == GEMV_F32) {
        ((float*)a.y[which])[(int64_t)b * a.R[which] + row0 + r] = v;
    } else {
        ((bf16_t*)a.y[which])[(int64_t)b * a.R[which] + row0 + r] = f32_to_bf16(v);
    }
}

bool gemv_mfma_supported(const GemvArgs& a, int nb) {
    if (nb < 1 || nb > 16 || a.gamma || a.K <= 0 || a.K % 256 != 0) return false;
    if (a.mode != GEMV_STORE && a.mode != GEMV_SILU && a.mode != GEMV_RESID && a.mode != GEMV_F32) return false;
    for (int i = 0; i < 3; ++i)
        if (a.R[i] < 0 || a.R[i] % 16 != 0) return false;
    // per-lane byte offsets are 32-bit: 16 rows of K elements
    if ((int64_t)16 * a.K * 2 >= ((int64_t)1 << 32)) return false;
    return true;
}

template <int MODE, int XI>
static hipError_t launch_gemv_mfma_t(const GemvArgs& a, int nb, unsigned grid, hipStream_t s) {
    constexpr int NS = MODE == GEMV_SILU ? 2 : 1, DEPTH = NS == 2 ? 3 : 4, NW = GEMV_MFMA_WAVES;
    const size_t lds = (size_t)NW * DEPTH * (NS + 1) * 2048;
    {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&gemv_mfma_kernel<MODE, XI>), (int)lds);
        if (e != hipSuccess) return e;
    }
    gemv_mfma_kernel<MODE, XI><<<dim3(grid), dim3(NW * 64), lds, s>>>(a, nb);
    return hipGetLastError();
}

template <int MODE>
static hipError_t launch_gemv_mfma_m(const GemvArgs& a, int nb, hipStream_t s) {
    const int64_t rows = MODE == GEMV_SILU ? (int64_t)a.R[0] : (int64_t)a.R[0] + a.R[1] + a.R[2];
    if (rows == 0) return hipSuccess;
    const unsigned grid = (unsigned)(rows / 16);
    return nb > 8 ? launch_gemv_mfma_t<MODE, 2>(a, nb, grid, s) : launch_gemv_mfma_t<MODE, 1>(a, nb, grid, s);
}

hipError_t launch_gemv_mfma(const GemvArgs& a, int nb, hipStream_t s) {
    switch (a.mode) {
        case GEMV_STORE: return launch_gemv_mfma_m<GEMV_STORE>(a, nb, s);
        case GEMV_SILU: return launch_gemv_mfma_m<GEMV_SILU>(a, nb, s);
        case GEMV_RESID: return launch_gemv_mfma_m<GEMV_RESID>(a, nb, s);
        case GEMV_F32: return launch_gemv_mfma_m<GEMV_F32>(a, nb, s);
        default: return hipErrorInvalidValue;
    }
}

// nb input vectors (1 <= nb <= 16).  bf16 with tile-friendly shapes runs on the matrix cores; otherwise the
// dot-product kernel, instantiated for 2, 4 and 8 vectors: other counts run as a sum of those (rows of X and Y are
// contiguous, so a group of vectors is the same call on shifted pointers)
hipError_t launch_gemv_nb(const GemvArgs& a, int nb, bool bf16, hipStream_t s) {
    if (nb < 1 || nb > DECODE_MAX_BATCH || a.gamma || a.mode == GEMV_QKV_ROPE) return hipErrorInvalidValue;
    if (bf16 && nb > 1 && gemv_mfma_supported(a, nb)) return launch_gemv_mfma(a, nb, s);
    const size_t eb = bf16 ? 2 : 4;
    int done = 0;
    while (done < nb) {
        const int left = nb - done;
        const int take = left >= 8 ? 8 : left >= 4 ? 4 : left >= 2 ? 2 : 1;
        GemvArgs g = a;
        g.x = (const char*)a.x + (size_t)done * a.K * eb;
        for (int i = 0; i < 3; ++i)
            if (a.y[i]) g.y[i] = (char*)a.y[i] + (size_t)done * a.R[i] * (a.mode == GEMV_F32 ? 4 : eb);
        hipError_t e;
        if (take == 1) e = launch_gemv(g, bf16, s);
        else if (bf16) e = take == 8 ? launch_gemv_nb_t<bf16_t, 8>(g, s) : take == 4 ? launch_gemv_nb_t<bf16_t, 4>(g, s) : launch_gemv_nb_t<bf16_t, 2>(g, s);
        else e = take == 8 ? launch_gemv_nb_t<float, 8>(g, s) : take == 4 ? launch_gemv_nb_t<float, 4>(g, s) : launch_gemv_nb_t<float, 2>(g, s);
        if (e != hipSuccess) return e;
        done += take;
    }
    return hipSuccess;
}

// ------------------------------------------------------------------- rotary table of one position
__global__ void decode_rope_row_kernel(int pos, int half, double neg2_over_d_log2base, float2* __restrict__ table) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= half) return;
    double sn, cs;
    sincos((double)pos * exp2((double)j * neg2_over_d_log2base), &sn, &cs);
    table[j] = make_float2((float)cs, (float)sn);
}

hipError_t launch_decode_rope_row(int pos, int d, float base, float2* table, hipStream_t s) {
    const int half = d / 2;
    decode_rope_row_kernel<<<dim3((unsigned)((half + 63) / 64)), dim3(64), 0, s>>>(pos, half, -2.0 / (double)d * log2((double)base),
                                                                                 table);
    return hipGetLastError();
}

// ------------------------------------------------------------------- rotary + cache append
// q [H, d] is rotated in place for position pos; k [Hkv, d] is rotated and written, with v, to row
// `row` of the cache; cache_pos[row] = pos.  Angles in fp64 like the prefill's rotary table.
template <typename T>
__global__ void decode_rope_append_kernel(T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, int pos,
                                          int H, int Hkv, int d, double neg2_over_d_log2base, T* __restrict__ cache_k,
                                          T* __restrict__ cache_v, int32_t* __restrict__ cache_pos, int64_t row) {
    const int half = d / 2;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) cache_pos[row] = pos;
    if (i >= (H + Hkv) * half) return;
    const int head = i / half, j = i % half;
    double sn, cs;
    sincos((double)pos * exp2((double)j * neg2_over_d_log2base), &sn, &cs);
    const float c = (float)cs, s = (float)sn;
    if (head < H) {
        T* p = q + (int64_t)head * d + j;
        const float a = to_f32(p[0]), b = to_f32(p[half]);
        p[0] = from_f32<T>(a * c - b * s);
        p[half] = from_f32<T>(b * c + a * s);
    } else {
        const int g = head - H;
        const T* p = k + (int64_t)g * d + j;
        const float a = to_f32(p[0]), b = to_f32(p[half]);
        T* o = cache_k + (row * Hkv + g) * (int64_t)d + j;
        o[0] = from_f32<T>(a * c - b * s);
        o[half] = from_f32<T>(b * c + a * s);
        T* ov = cache_v + (row * Hkv + g) * (int64_t)d + j;
        const T* pv = v + (int64_t)g * d + j;
        ov[0] = pv[0];
        ov[half] = pv[half];
    }
}

hipError_t launch_decode_rope_append(void* q, const void* k, const void* v, int pos, int H, int Hkv, int d, float base,
                                     void* cache_k, void* cache_v, int32_t* cache_pos, int64_t row, bool bf16, hipStream_t s) {
    const int n = (H + Hkv) * (d / 2);
    const double kk = -2.0 / (double)d * log2((double)base);
    const dim3 g((unsigned)((n + 255) / 256)), b(256);
    if (bf16)
        decode_rope_append_kernel<bf16_t><<<g, b, 0, s>>>((bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, pos, H, Hkv, d, kk,
                                                          (bf16_t*)cache_k, (bf16_t*)cache_v, cache_pos, row);
    else
        decode_rope_append_kernel<float><<<g, b, 0, s>>>((float*)q, (const float*)k, (const float*)v, pos, H, Hkv, d, kk,
                                                        (float*)cache_k, (float*)cache_v, cache_pos, row);
    return hipGetLastError();
}

// the same for a batch of sequences (blockIdx.y = sequence), from the fp32 sums of the projections: q32 [B, H, d],
// k32 / v32 [B, Hkv, d] -> q [B, H, d] and the new cache rows, rounded to T once, after the rotation (as the
// single-sequence GEMV's epilogue does); every sequence has its own cache, row and position (by-value descriptor: at
// most DECODE_MAX_BATCH sequences)
template <typename T>
__global__ void decode_rope_append_batched_kernel(const float* __restrict__ q32, const float* __restrict__ k32,
                                                  const float* __restrict__ v32, T* __restrict__ q, int H, int Hkv, int d,
                                                  double neg2_over_d_log2base, DecodeBatch db) {
    const int half = d / 2;
    const int b = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int pos = db.pos[b];
    const int64_t row = db.count[b];
    if (i == 0) db.cache_pos[b][row] = pos;
    if (i >= (H + Hkv) * half) return;
    const int head = i / half, j = i % half;
    double sn, cs;
    sincos((double)pos * exp2((double)j * neg2_over_d_log2base), &sn, &cs);
    const float c = (float)cs, s = (float)sn;
    if (head < H) {
        const int64_t o = ((int64_t)b * H + head) * d + j;
        const float x0 = q32[o], x1 = q32[o + half];
        q[o] = from_f32<T>(x0 * c - x1 * s);
        q[o + half] = from_f32<T>(x1 * c + x0 * s);
    } else {
        const int g = head - H;
        const int64_t i0 = ((int64_t)b * Hkv + g) * d + j;
        const float x0 = k32[i0], x1 = k32[i0 + half];
        T* o = (T*)db.cache_k[b] + (row * Hkv + g) * (int64_t)d + j;
        o[0] = from_f32<T>(x0 * c - x1 * s);
        o[half] = from_f32<T>(x1 * c + x0 * s);
        T* ov = (T*)db.cache_v[b] + (row * Hkv + g) * (int64_t)d + j;
        ov[0] = from_f32<T>(v32[i0]);
        ov[half] = from_f32<T>(v32[i0 + half]);
    }
}

hipError_t launch_decode_rope_append_batched(const float* q32, const float* k32, const float* v32, void* q, int H, int Hkv, int d,
                                             float base, const DecodeBatch& db, bool bf16, hipStream_t s) {
    if (db.n < 1 || db.n > DECODE_MAX_BATCH) return hipErrorInvalidValue;
    const int n = (H + Hkv) * (d / 2);
    const double kk = -2.0 / (double)d * log2((double)base);
    const dim3 g((unsigned)((n + 255) / 256), (unsigned)db.n), b(256);
    if (bf16)
        decode_rope_append_batched_kernel<bf16_t><<<g, b, 0, s>>>(q32, k32, v32, (bf16_t*)q, H, Hkv, d, kk, db);
    else
        decode_rope_append_batched_kernel<float><<<g, b, 0, s>>>(q32, k32, v32, (float*)q, H, Hkv, d, kk, db);
    return hipGetLastError();
}

// ------------------------------------------------------------------------- decode attention
// partial layout: part[((g * nsplit + split) * GRP_MAX + hg) * (d + 2)] = (max, sum, weighted values[d])
constexpr int GRP_MAX = 8;

// G: query heads per KV head the register arrays are sized for (>= H / Hkv)
template <typename T, int D, int G>
__device__ __forceinline__ void decode_attn_body(const T* __restrict__ q, const T* __restrict__ K, const T* __restrict__ V,
                                                 int64_t M, int H, int Hkv, float scale_log2e, float* __restrict__ part) {
    constexpr int EPC = 16 / (int)sizeof(T);
    constexpr int LPK = D / EPC;          // lanes that hold one key row
    constexpr int KPW = 64 / LPK;         // keys per wavefront step
    __shared__ float sm[4][G][2];
    __shared__ float sacc[4][G][D];

    const int split = blockIdx.x, nsplit = gridDim.x, g = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % LPK, kslot = lane / LPK;
    const int grp = H / Hkv;
    const int64_t per = (M + nsplit - 1) / nsplit;
    const int64_t m_begin = (int64_t)split * per;
    const int64_t m_end = m_begin + per < M ? m_begin + per : M;

    // this lane's piece of every query head of the group
    u32x4 qv[G];
#pragma unroll
    for (int hg = 0; hg < G; ++hg) {
        const int h = g * grp + (hg < grp ? hg : 0);
        qv[hg] = *reinterpret_cast<const u32x4*>(q + (int64_t)h * D + sub * EPC);
    }
    float mrun[G], lrun[G], acc[G][EPC];
#pragma unroll
    for (int hg = 0; hg < G; ++hg) {
        mrun[hg] = -INFINITY; lrun[hg] = 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[hg][e] = 0.f;
    }

    // keys of this lane: m_begin + wave*KPW + kslot + it * 4*KPW; the next pair is loaded before the
    // current one is used (rings of two or three more pairs in flight measured 25 % slower, at equal
    // occupancy)
    const T* Kg = K + (int64_t)g * D + sub * EPC;
    const T* Vg = V + (int64_t)g * D + sub * EPC;
    const int64_t rstride = (int64_t)Hkv * D;
    int64_t m = m_begin + wave * KPW + kslot;
    u32x4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
    if (m_begin < m_end) {
        const int64_t mc = m < m_end ? m : m_end - 1;
        kv = *reinterpret_cast<const u32x4*>(Kg + mc * rstride);
        vv = *reinterpret_cast<const u32x4*>(Vg + mc * rstride);
    }
    for (int64_t m0 = m_begin + wave * KPW; m0 < m_end; m0 += 4 * KPW, m += 4 * KPW) {
        const bool valid = m < m_end;
        const int64_t mn_ = m + 4 * KPW;
        const int64_t mnc = mn_ < m_end ? mn_ : m_end - 1;
        const u32x4 kvn = *reinterpret_cast<const u32x4*>(Kg + mnc * rstride);
        const u32x4 vvn = *reinterpret_cast<const u32x4*>(Vg + mnc * rstride);
        float vf[EPC];
#pragma unroll
        for (int e = 0; e < EPC; ++e) vf[e] = chunk_elem(vv, e, T{});
#pragma unroll
        for (int hg = 0; hg < G; ++hg) {
            if (hg < grp) {
                float s = group_sum<LPK>(dot16(kv, qv[hg], 0.f, T{}));
                s = valid ? s * scale_log2e : -INFINITY;
                const float mn = fmaxf(mrun[hg], s);
                const float mu = mn == -INFINITY ? 0.f : mn;
                // the running maximum rarely moves after the first keys: rescale only when it did for some lane
                if (__ballot(mn != mrun[hg]) != 0) {
                    const float alpha = __builtin_amdgcn_exp2f(mrun[hg] - mu);
                    lrun[hg] *= alpha;
#pragma unroll
                    for (int e = 0; e < EPC; ++e) acc[hg][e] *= alpha;
                    mrun[hg] = mn;
                }
                const float p = __builtin_amdgcn_exp2f(s - mu);
                lrun[hg] += p;
#pragma unroll
                for (int e = 0; e < EPC; ++e) acc[hg][e] = __builtin_fmaf(p, vf[e], acc[hg][e]);
            }
        }
        kv = kvn;
        vv = vvn;
    }
    // merge the KPW lane groups of the wavefront (lanes with equal `sub`)
#pragma unroll
    for (int hg = 0; hg < G; ++hg) {
        if (hg < grp) {
#pragma unroll
            for (int off = LPK; off < 64; off <<= 1) {
                const float mo = __shfl_xor(mrun[hg], off), lo = __shfl_xor(lrun[hg], off);
                const float mn = fmaxf(mrun[hg], mo);
                const float mu = mn == -INFINITY ? 0.f : mn;
                const float a0 = __builtin_amdgcn_exp2f(mrun[hg] - mu), a1 = __builtin_amdgcn_exp2f(mo - mu);
                lrun[hg] = lrun[hg] * a0 + lo * a1;
#pragma unroll
                for (int e = 0; e < EPC; ++e) acc[hg][e] = acc[hg][e] * a0 + __shfl_xor(acc[hg][e], off) * a1;
                mrun[hg] = mn;
            }
            if (kslot == 0) {
                if (sub == 0) { sm[wave][hg][0] = mrun[hg]; sm[wave][hg][1] = lrun[hg]; }
#pragma unroll
                for (int e = 0; e < EPC; ++e) sacc[wave][hg][sub * EPC + e] = acc[hg][e];
            }
        }
    }
    __syncthreads();
    // merge the 4 wavefronts: thread t < grp * D handles (hg, element)
    for (int t = tid; t < grp * D; t += 256) {
        const int hg = t / D, e = t % D;
        float mn = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mn = fmaxf(mn, sm[w][hg][0]);
        const float mu = mn == -INFINITY ? 0.f : mn;
        float l = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float aw = __builtin_amdgcn_exp2f(sm[w][hg][0] - mu);
            l += sm[w][hg][1] * aw;
            o += sacc[w][hg][e] * aw;
        }
        float* dst = part + (((int64_t)g * nsplit + split) * GRP_MAX + hg) * (D + 2);
        if (e == 0) { dst[0] = mn; dst[1] = l; }
        dst[2 + e] = o;
    }
}

template <typename T, int D, int G>
__global__ void __launch_bounds__(256) decode_attn_kernel(const T* __restrict__ q, const T* __restrict__ K,
                                                          const T* __restrict__ V, int64_t M, int H, int Hkv, float scale_log2e,
                                                          float* __restrict__ part) {
    decode_attn_body<T, D, G>(q, K, V, M, H, Hkv, scale_log2e, part);
}
// blockIdx.z = sequence: its query [H, D], its cache (count[b] + 1 pairs: the new pair is already appended) and its
// share of the partial buffer
template <typename T, int D, int G>
__global__ void __launch_bounds__(256) decode_attn_batched_kernel(const T* __restrict__ q, DecodeBatch db, int H, int Hkv,
                                                                  float scale_log2e, float* __restrict__ part, int64_t part_stride) {
    const int b = blockIdx.z;
    decode_attn_body<T, D, G>(q + (int64_t)b * H * D, (const T*)db.cache_k[b], (const T*)db.cache_v[b], db.count[b] + 1, H, Hkv,
                              scale_log2e, part + (int64_t)b * part_stride);
}

// out[h, e] = sum over splits of the weighted values / sum of sums.  One workgroup of 1024 threads per
// query head: thread s < 256 takes split s for the (max, sum) part; the weighted values are summed by
// 1024 / D thread groups that each walk a strided subset of the splits with independent loads.
template <typename T>
__global__ void __launch_bounds__(1024) decode_attn_merge_kernel(const float* __restrict__ part, int nsplit, int H, int Hkv, int D,
                                                                 T* __restrict__ out, int64_t part_stride) {
    __shared__ float sa[256];
    __shared__ float sw[16], sl[16];
    __shared__ float so[1024];
    const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = H / Hkv, g = h / grp, hg = h % grp;
    part += (int64_t)blockIdx.y * part_stride;      // blockIdx.y = sequence of a batched step
    out += (int64_t)blockIdx.y * H * D;
    const float* base = part + ((int64_t)g * nsplit * GRP_MAX + hg) * (D + 2);
    const int64_t stride = (int64_t)GRP_MAX * (D + 2);
    const float m = tid < nsplit ? base[tid * stride] : -INFINITY;       // nsplit <= 256: wavefronts 0-3
    const float l = tid < nsplit ? base[tid * stride + 1] : 0.f;
    float mx = m;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if (lane == 0) sw[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(sw[0], sw[1]), fmaxf(sw[2], sw[3]));
    const float mu = mx == -INFINITY ? 0.f : mx;
    const float a = __builtin_amdgcn_exp2f(m - mu);     // 0 for absent or empty splits
    if (tid < 256) sa[tid] = a;
    const float ls = wave_sum(l * a);
    if (lane == 0) sl[wave] = ls;
    __syncthreads();
    const float L = sl[0] + sl[1] + sl[2] + sl[3];
    const int ngroups = 1024 / D, grp_id = tid / D, e = tid % D;
    float o = 0.f;
    if (grp_id < ngroups) {
#pragma unroll 8
        for (int s = grp_id; s < nsplit; s += ngroups) o += base[s * stride + 2 + e] * sa[s];
    }
    so[tid] = o;
    __syncthreads();
    if (tid < D) {
        float t = 0.f;
        for (int k = 0; k < ngroups; ++k) t += so[k * D + tid];
        out[(int64_t)h * D + tid] = from_f32<T>(L > 0.f ? t / L : 0.f);
    }
}

// number of key splits per sequence: two workgroups per CU over the whole launch (measured best on 4.6K-13K cached
// pairs, one sequence: 32 / 64 / 128 / 256 splits of 8 KV heads take 14.6 / 11.7 / 12.8 / 14.3 us; 8 sequences of
// 8.3K pairs: 8 / 16 / 32 / 64 splits take 61 / 62 / 65 / 69 us, 4 splits 89 us), at least 64 keys each, and no
// more than the scratch buffer (scratch_floats, per sequence) holds
int decode_attn_splits(int64_t M, int Hkv, int d, size_t scratch_floats, int nseq) {
    int64_t s = 512 / ((int64_t)(Hkv > 0 ? Hkv : 1) * (nseq > 0 ? nseq : 1));
    if (s > (M + 63) / 64) s = (M + 63) / 64;
    const int64_t cap = (int64_t)(scratch_floats / ((size_t)Hkv * GRP_MAX * (d + 2)));
    if (s > cap) s = cap;
    if (s > 256) s = 256;
    if (s < 1) s = 1;
    return (int)s;
}
size_t decode_attn_min_scratch_floats(int Hkv, int d) { return (size_t)Hkv * GRP_MAX * (d + 2); }

bool decode_attn_supported(int H, int Hkv, int d, bool bf16) {
    (void)bf16;
    if (Hkv <= 0 || H % Hkv != 0 || H / Hkv > GRP_MAX) return false;
    return d == 16 || d == 32 || d == 64 || d == 128;
}

template <typename T>
static hipError_t launch_decode_attn_t(const T* q, const T* K, const T* V, int64_t M, int H, int Hkv, int d, float* part,
                                       size_t part_floats, T* out, hipStream_t s) {
    const int nsplit = decode_attn_splits(M, Hkv, d, part_floats, 1);
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)d);
    const dim3 g((unsigned)nsplit, (unsigned)Hkv), b(256);
    const int grp = H / Hkv;
#define SPTS_DEC_ATTN(D_)                                                                                      \
    if (grp <= 1) decode_attn_kernel<T, D_, 1><<<g, b, 0, s>>>(q, K, V, M, H, Hkv, scale_log2e, part);         \
    else if (grp <= 2) decode_attn_kernel<T, D_, 2><<<g, b, 0, s>>>(q, K, V, M, H, Hkv, scale_log2e, part);    \
    else if (grp <= 4) decode_attn_kernel<T, D_, 4><<<g, b, 0, s>>>(q, K, V, M, H, Hkv, scale_log2e, part);    \
    else decode_attn_kernel<T, D_, GRP_MAX><<<g, b, 0, s>>>(q, K, V, M, H, Hkv, scale_log2e, part);
    switch (d) {
        case 128: SPTS_DEC_ATTN(128) break;
        case 64: SPTS_DEC_ATTN(64) break;
        case 32: SPTS_DEC_ATTN(32) break;
        case 16: SPTS_DEC_ATTN(16) break;
        default: return hipErrorInvalidValue;
    }
#undef SPTS_DEC_ATTN
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    decode_attn_merge_kernel<T><<<dim3((unsigned)H), dim3(1024), 0, s>>>(part, nsplit, H, Hkv, d, out, 0);
    return hipGetLastError();
}

hipError_t launch_decode_attn(const void* q, const void* K, const void* V, int64_t M, int H, int Hkv, int d, float* part,
                              size_t part_floats, void* out, bool bf16, hipStream_t s) {
    if (M <= 0 || part_floats < decode_attn_min_scratch_floats(Hkv, d)) return hipErrorInvalidValue;
    if (bf16)
        return launch_decode_attn_t<bf16_t>((const bf16_t*)q, (const bf16_t*)K, (const bf16_t*)V, M, H, Hkv, d, part, part_floats,
                                            (bf16_t*)out, s);
    return launch_decode_attn_t<float>((const float*)q, (const float*)K, (const float*)V, M, H, Hkv, d, part, part_floats, (float*)out, s);
}

// the same for a batch of sequences in one launch (grid z = sequence); every sequence takes the same number of
// splits, chosen for the longest cache; out [B, H, d]
template <typename T>
static hipError_t launch_decode_attn_batched_t(const T* q, const DecodeBatch& db, int H, int Hkv, int d, float* part,
                                               size_t part_floats, T* out, hipStream_t s) {
    int64_t mmax = 1;
    for (int b = 0; b < db.n; ++b) mmax = db.count[b] + 1 > mmax ? db.count[b] + 1 : mmax;
    const int nsplit = decode_attn_splits(mmax, Hkv, d, part_floats / (size_t)db.n, db.n);
    const int64_t stride = (int64_t)Hkv * nsplit * GRP_MAX * (d + 2);
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)d);
    const dim3 g((unsigned)nsplit, (unsigned)Hkv, (unsigned)db.n), b(256);
    const int grp = H / Hkv;
#define SPTS_DEC_ATTN_B(D_)                                                                                                 \
    if (grp <= 1) decode_attn_batched_kernel<T, D_, 1><<<g, b, 0, s>>>(q, db, H, Hkv, scale_log2e, part, stride);           \
    else if (grp <= 2) decode_attn_batched_kernel<T, D_, 2><<<g, b, 0, s>>>(q, db, H, Hkv, scale_log2e, part, stride);      \
    else if (grp <= 4) decode_attn_batched_kernel<T, D_, 4><<<g, b, 0, s>>>(q, db, H, Hkv, scale_log2e, part, stride);      \
    else decode_attn_batched_kernel<T, D_, GRP_MAX><<<g, b, 0, s>>>(q, db, H, Hkv, scale_log2e, part, stride);
    switch (d) {
        case 128: SPTS_DEC_ATTN_B(128) break;
        case 64: SPTS_DEC_ATTN_B(64) break;
        case 32: SPTS_DEC_ATTN_B(32) break;
        case 16: SPTS_DEC_ATTN_B(16) break;
        default: return hipErrorInvalidValue;
    }
#undef SPTS_DEC_ATTN_B
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    decode_attn_merge_kernel<T><<<dim3((unsigned)H, (unsigned)db.n), dim3(1024), 0, s>>>(part, nsplit, H, Hkv, d, out, stride);
    return hipGetLastError();
}

hipError_t launch_decode_attn_batched(const void* q, const DecodeBatch& db, int H, int Hkv, int d, float* part, size_t part_floats,
                                      void* out, bool bf16, hipStream_t s) {
    if (db.n < 1 || db.n > DECODE_MAX_BATCH || part_floats / (size_t)db.n < decode_attn_min_scratch_floats(Hkv, d)) return hipErrorInvalidValue;
    if (bf16) return launch_decode_attn_batched_t<bf16_t>((const bf16_t*)q, db, H, Hkv, d, part, part_floats, (bf16_t*)out, s);
    return launch_decode_attn_batched_t<float>((const float*)q, db, H, Hkv, d, part, part_floats, (float*)out, s);
}

// ------------------------------------------------------------------------------ greedy head
// token = argmax of logits [V], ties to the lowest id; one workgroup
__global__ void __launch_bounds__(1024) argmax_kernel(const float* __restrict__ logits, int V, int32_t* __restrict__ token) {
    __shared__ float sv[16];
    __shared__ int si[16];
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = threadIdx.x; i < V; i += 1024) {
        const float v = logits[i];
        if (v > best || (v == best && i < bi)) { best = v; bi = i; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(best, off);
        const int oi = __shfl_xor(bi, off);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sv[wave] = best; si[wave] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w)
            if (sv[w] > best || (sv[w] == best && si[w] < bi)) { best = sv[w]; bi = si[w]; }
        *token = bi == 0x7fffffff ? 0 : bi;
    }
}

template <typename T>
__global__ void table_row_kernel(const T* __restrict__ table, const int32_t* __restrict__ token, int D, T* __restrict__ out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < D) out[i] = table[(int64_t)(*token) * D + i];
}

hipError_t launch_argmax_row(const float* logits, int V, int32_t* token, const void* table, int D, void* x_next, bool bf16,
                             hipStream_t s) {
    argmax_kernel<<<dim3(1), dim3(1024), 0, s>>>(logits, V, token);
    if (x_next) {
        const dim3 g((unsigned)((D + 255) / 256)), b(256);
        if (bf16) table_row_kernel<bf16_t><<<g, b, 0, s>>>((const bf16_t*)table, token, D, (bf16_t*)x_next);
        else table_row_kernel<float><<<g, b, 0, s>>>((const float*)table, token, D, (float*)x_next);
    }
    return hipGetLastError();
}

}  // namespace spts
