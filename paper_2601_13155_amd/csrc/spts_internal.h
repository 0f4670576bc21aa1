// Internal declarations shared by the HIP translation units of libspts (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spts {

// Native vector types for register staging (arrays of HIP's uint4 struct are not scalarised by the
// compiler and end up in scratch memory).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// ------------------------------------------------------------------ element types
struct bf16_t { uint16_t v; };

__host__ __device__ inline float bf16_to_f32(bf16_t h) {
    union { uint32_t u; float f; } c; c.u = ((uint32_t)h.v) << 16; return c.f;
}
// round-to-nearest-even; NaN stays NaN
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
    union { uint32_t u; float f; } c; c.f = f;
    uint32_t u = c.u;
    bf16_t r;
    if ((u & 0x7fffffffu) > 0x7f800000u) { r.v = (uint16_t)((u >> 16) | 0x40); return r; }
    u += 0x7fffu + ((u >> 16) & 1u);
    r.v = (uint16_t)(u >> 16);
    return r;
}
__device__ inline float to_f32(float v) { return v; }
__device__ inline float to_f32(bf16_t v) { return bf16_to_f32(v); }
// two floats -> packed bf16x2 with the hardware converter (v_cvt_pk_bf16_f32, round to nearest even)
typedef __bf16 hw_bf16x2 __attribute__((ext_vector_type(2)));
typedef float hw_f32x2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t cvt_pk_bf16(float a, float b) {
    hw_f32x2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, hw_bf16x2));
}
template <typename T> __device__ inline T from_f32(float v);
template <> __device__ inline float from_f32<float>(float v) { return v; }
template <> __device__ inline bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

// One direct-to-LDS load (gfx950 global_load_lds_dwordx4): every lane fetches 16 bytes from its own
// global address; the wavefront's 1 KB lands at lds_base + 16 * lane.  lds_base must be
// wavefront-uniform.  The compiler does not see these loads: the issuing code counts them itself
// (SPTS_WAIT_VMCNT) and publishes the data with a workgroup barrier.
__device__ inline void dma16(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off\n\t" ::"v"(gptr), "s"(lds_base) : "memory");
}
// The same load with the address split into a wavefront-uniform 64-bit base (SGPR pair) and a 32-bit
// unsigned per-lane byte offset.
__device__ inline void dma16s(uint32_t voff, const void* sbase, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n\t" ::"v"(voff), "s"(sbase), "s"(lds_base) : "memory");
}
// s_waitcnt vmcnt(n) only (expcnt / lgkmcnt fields left at "no wait")
#define SPTS_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 0xF) | (((n) >> 4) << 14))

// Key order of the transposed value copy V^T [Hkv*d, ld]: inside every aligned group of 16 keys the
// two middle quads are swapped (0-3, 8-11, 4-7, 12-15), which is the order the attention kernel's
// probability fragments come out of the matrix core, so a value fragment is one 16-byte read.
__host__ __device__ inline int64_t vt_key_slot(int64_t key) { return (key & ~(int64_t)12) | ((key & 4) << 1) | ((key & 8) >> 1); }

// Raises a kernel's dynamic-LDS limit once per (device, kernel); safe to call from several host threads.
hipError_t ensure_dynamic_lds(const void* kernel, int bytes);

// ------------------------------------------------------------------ GEMM (C = A * B^T)
enum GemmEpilogue : int {
    EPI_STORE = 0,      // C[row, col] = acc          (T, or fp32 when c_is_f32)
    EPI_SILU_MUL = 1,   // C[row, col] = silu(acc0) * acc1     (two B operands)
    EPI_RESIDUAL = 2,   // C[crow, col] = C[crow, col] + acc   (crow = c_idx ? c_idx[row] : row)
    EPI_SUMSQ = 3,      // part[row, col_block] = sum over the block's columns of acc^2
    EPI_ROPE = 4,       // C[row, col] = rotary(acc) with table row (rope_idx ? rope_idx[row] : row); MFMA path only
    EPI_ROPE_STORE = 5, // two products of the same A rows in one launch (MFMA path only): columns [0, n_split) = A * B0^T
                        // with the rotary epilogue -> C; columns [n_split, N) = A * B1^T stored plainly -> C2 (and Ct)
};

struct GemmArgs {
    const void* A; int64_t lda; const int32_t* a_idx;   // A [*, K] rows optionally gathered
    int64_t a_rows;                                     // with a_idx: rows of the gather source (every index is below it)
    const void* A1;                                     // EPI_SILU_MUL: A operand of the second product (null = A)
    const void* B0; const void* B1; int64_t ldb;        // B [N, K]; EPI_STORE with B1: columns [N/2, N) come from B1
    void* C; int64_t ldc; const int32_t* c_idx;         // output rows optionally scattered
    void* Ct; int64_t ldct;                             // optional transposed copy Ct[col, row]
    float* part; int32_t part_ld;                       // EPI_SUMSQ partial sums [M, part_ld]
    const float2* rope; int32_t head_dim;               // EPI_ROPE: cos/sin table [rows, head_dim/2]
    const int32_t* rope_idx;                            // table row = rope_idx ? rope_idx[row] : row
    float rope_scale;                                   // EPI_ROPE: the rotated values are multiplied by this before rounding (0 = 1)
    int32_t n_split; void* C2; int64_t ldc2;            // EPI_ROPE_STORE: first column of the second product, its output [M, N - n_split]
    int64_t b_rows1;                                    // EPI_ROPE_STORE with b_slab: rows of the slab-major B1 (b_rows: of B0)
    int64_t M; int32_t N; int32_t K;
    int32_t epi; int32_t c_is_f32;
    // tail split-K (matrix-core path; EPI_STORE / EPI_RESIDUAL / EPI_ROPE): the first `nfull` tiles (in
    // raster order) are computed whole; each of the remaining tiles is shared by `ksplit` workgroups,
    // every one taking a contiguous share of K and writing its raw fp32 accumulators to part32
    // (65536 floats per (tile, split), in accumulator-fragment order); a second kernel sums the
    // splits in split order and applies the epilogue.  With one workgroup resident per CU this turns
    // the last, partly filled round of tiles into a full round of short work units.
    // ksplit <= 1 disables it (nfull is then ignored).
    int32_t ksplit; int32_t nfull; float* part32;
    // slab-major operands (matrix-core path, 32-wide K slabs only): A stored [K/32][M][32], B0 / B1 stored [K/32][b_rows][32]
    // (pack_slab32 of the row-major matrix), so that the 16 rows a load instruction moves are 1 KB of whole cache lines
    // instead of 64-byte halves of 16 lines.  a_slab excludes a_idx (the packed copy is already gathered).
    int32_t a_slab; int32_t b_slab; int64_t b_rows;
    int32_t c_slab;   // EPI_SILU_MUL / EPI_STORE: C written slab-major [N/32][M][32] (the A operand of a following a_slab GEMM);
                      // no c_idx, no Ct
};
// Split plan for a GEMM of this shape on a 256-CU device: returns ksplit (1 = do not split) and
// sets *nfull; needs (tiles - nfull) * ksplit * 65536 floats of part32.
int gemm_pick_split(int64_t M, int32_t N, int32_t K, int epi, int32_t* nfull);

hipError_t launch_gemm_generic(const GemmArgs& a, bool bf16, hipStream_t s);
// true when the matrix-core kernel can serve these arguments (alignment / divisibility)
bool gemm_mfma_supported(const GemmArgs& a);
hipError_t launch_gemm_mfma(const GemmArgs& a, hipStream_t s);
// number of column blocks a EPI_SUMSQ launch writes per row
int gemm_sumsq_blocks(int32_t N, bool mfma);

// ------------------------------------------------------------------ proxy hidden layer (register-stationary rows)
// h[n, c] = silu(t_g[n, :] . Vg[c, :]) * (t_u[n, :] . Vu[c, :]) for n < N, c < Dlow, written slab-major [Dlow/32][N][32].
// t_g / t_u: element (n, k) at base + n * t_row_pitch + (k / 32) * t_slab_pitch + (k % 32) * 2 bytes (covers a row-major
// [N, 2r] matrix and a slab-major one); Vg_s / Vu_s: slab-major copies [r/32][Dlow][32] of the factors.
struct ProxyHiddenArgs {
    const void* tg; const void* tu; int64_t t_row_pitch, t_slab_pitch;
    const void* Vg_s; const void* Vu_s;
    void* hp;
    int64_t N; int32_t Dlow; int32_t r;
};
bool proxy_hidden_supported(const ProxyHiddenArgs& a);
hipError_t launch_proxy_hidden(const ProxyHiddenArgs& a, hipStream_t s);

// ------------------------------------------------------------------ elementwise / data movement
// slab-major copy of a row-major [rows, K] matrix of 2-byte elements: out[(s * rows + r) * 32 + j] = W[r * K + 32 * s + j]
hipError_t launch_pack_slab32(const void* W, int64_t rows, int64_t K, void* out, hipStream_t s);
hipError_t launch_rope_table(const int32_t* pos, int64_t N, int d, float base, float2* table, hipStream_t s);
hipError_t launch_rmsnorm(const void* x, const void* gamma, float eps, void* out, int64_t N, int D, bool bf16, hipStream_t s);
// out[n, h, :] = scale * rotary(in_f32[n, h, :]) with table row (idx ? idx[n] : n + row0)
hipError_t launch_rope_apply(const float* in, const float2* table, const int32_t* idx, int64_t row0, void* out,
                             int64_t n, int heads, int d, bool bf16, hipStream_t s, float scale = 1.0f);
// out[i, :] = in[idx[i], :]   (row_bytes multiple of 4)
hipError_t launch_gather_rows(const void* in, const int32_t* idx, void* out, int64_t n, int64_t row_bytes, hipStream_t s);
// out[i, :] = in[idx[i], :] (row_bytes multiple of 16) and, in the same launch, pos_out[i] = pos_in[idx[i]] (when pos_out) and
// old2new[idx[i]] = i (when old2new)
hipError_t launch_gather_rows_maps(const void* in, const int32_t* idx, void* out, int64_t n, int64_t row_bytes,
                                   const int32_t* pos_in, int32_t* pos_out, int32_t* old2new, hipStream_t s);
hipError_t launch_gather_i32(const int32_t* in, const int32_t* idx, int32_t* out, int64_t n, hipStream_t s);
hipError_t launch_copy_bytes(const void* in, void* out, int64_t bytes, hipStream_t s);
hipError_t launch_fill_i32(int32_t* p, int32_t v, int64_t n, hipStream_t s);
hipError_t launch_iota_i32(int32_t* p, int64_t n, hipStream_t s);
// n host int64 values -> device array dst, in chunks passed by value as kernel arguments (no host staging buffer, no
// synchronisation, safe under stream capture)
struct I64Chunk { static constexpr int CAP = 256; int64_t v[CAP]; int32_t n; };
hipError_t launch_write_i64(const int64_t* host_vals, int64_t n, int64_t* dst, hipStream_t s);
// idx[i] += seg_offsets[b] for i in [out_offsets[b], out_offsets[b+1]); device descriptor arrays
hipError_t launch_add_segment_base(int32_t* idx, const int64_t* out_offsets, const int64_t* seg_offsets, int nseg, int64_t total,
                                   hipStream_t s);
// old2new[idx[i]] = i
hipError_t launch_scatter_iota(const int32_t* idx, int32_t* old2new, int64_t n, hipStream_t s);
// c = sqrt(sum_j part[n, j]); s_ffn = c * (s_mha ? s_mha[n] : 1)
hipError_t launch_finish_ffn_scores(const float* part, int nparts, const float* s_mha, float* c_ffn, float* s_ffn,
                                    int64_t N, hipStream_t s);
// c_ffn[n] = ||z[n, :]||_2, s_ffn[n] = c_ffn[n] * s_mha[n] (s_mha may be null); z [N, r] row-major
hipError_t launch_row_norm_scores(const void* z, int r, bool bf16, const float* s_mha, float* c_ffn, float* s_ffn, int64_t N,
                                  hipStream_t s);
// vt[c, vt_key_slot(i)] = v[i, c]  (v [M, C] -> vt [C, ldvt]); keys i in [M, ldvt) are zero-filled
hipError_t launch_transpose_pad(const void* v, void* vt, int64_t M, int C, int64_t ldvt, bool bf16, hipStream_t s);

// ------------------------------------------------------------------ TopK
// `batch` independent problems: scores [batch, N] -> idx_out [batch, k], every row ascending.
// With segment descriptors (device arrays) problem b is scores[offsets[b] .. offsets[b+1]) with budget
// min(k[b], length), written to idx_out + out_offsets[b] as indices local to the segment; N is then the
// longest segment.
struct TopkSegments { const int64_t* offsets; const int64_t* k; const int64_t* out_offsets; };
hipError_t launch_topk(const float* scores, int64_t N, int64_t k, int protect_last, int32_t* idx_out,
                       int batch, hipStream_t s, TopkSegments seg = TopkSegments{nullptr, nullptr, nullptr});

// One problem spread over many workgroups (a launch per radix pass + one for the ordered compaction); `scratch`:
// TOPK_MULTI_SCRATCH_BYTES of device memory, 256-byte aligned, contents irrelevant on entry (every word that is
// read was written earlier in the same call); calls sharing a scratch must not overlap.  N <= TOPK_MULTI_MAX_N.
constexpr int TOPK_MULTI_MAX_WG = 128;
constexpr int64_t TOPK_MULTI_MAX_N = (int64_t)TOPK_MULTI_MAX_WG * 8192;
constexpr int64_t TOPK_MULTI_MIN_N = 20000;   // shorter rows: one workgroup with the keys in registers is as fast (measured crossover)
constexpr size_t TOPK_MULTI_SCRATCH_BYTES = 2 * (size_t)TOPK_MULTI_MAX_WG * 256 * 4 + (size_t)TOPK_MULTI_MAX_WG * 4 + 64;
// device address of this GPU's file-scope scratch array of TOPK_MULTI_SCRATCH_BYTES (looked up once per device, then cached)
hipError_t topk_static_scratch(void** out);
hipError_t launch_topk_multi(const float* scores, int64_t N, int64_t k, int protect_last, int32_t* idx_out, void* scratch,
                             hipStream_t s);

// ------------------------------------------------------------------ attention
struct AttnArgs {
    const void* q;  // [Mq, H, d]
    const void* k;  // [Mk, Hkv, d]
    const void* v;  // [Mk, Hkv, d]
    const void* vt; // [Hkv*d, ldvt] transposed values (MFMA path), may be null for the generic path
    int64_t ldvt;
    const int32_t* qpos; const int32_t* kpos;  // ascending absolute positions
    void* out;      // [Mq, H, d]
    int64_t Mq, Mk; int H, Hkv, d;
    int out_slab;   // matrix-core path only: out written slab-major [H*d/32][Mq][32] (A operand of an a_slab GEMM)
    float q_scale;  // factor the producer of q already folded into it (0 or 1 = none).  The matrix-core kernel wants
                    // attention_mfma_q_scale(d) and folds in what is missing, at the price of a second bf16 rounding of q
};
// log2(e) / sqrt(d): with q carrying this factor the matrix-core kernel's logits are exponents of 2 as they leave the MFMA
float attention_mfma_q_scale(int d);
hipError_t launch_attention_generic(const AttnArgs& a, bool bf16, hipStream_t s);
bool attention_mfma_supported(const AttnArgs& a);
hipError_t launch_attention_mfma(const AttnArgs& a, hipStream_t s);

// probe: qp [P, H, d], k [N, Hkv, d] -> S[N]; scratch floats: 2*P*H (+ Hkv*N for the MFMA path)
struct ProbeArgs {
    const void* qp; const void* k; float* S; float* stats; float* partial;
    int64_t N; int P, H, Hkv, d;
    float q_scale;   // factor the producer of qp already folded into it (0 or 1 = none), as for AttnArgs
};
hipError_t launch_probe_generic(const ProbeArgs& a, bool bf16, hipStream_t s);
bool probe_mfma_supported(const ProbeArgs& a);
hipError_t launch_probe_mfma(const ProbeArgs& a, hipStream_t s);
size_t probe_scratch_floats(int64_t N, int P, int H, int Hkv);
// single probe row (P = 1): a scan of K with one query per head; scratch: probe_p1_scratch_floats(N, H) floats
bool probe_p1_supported(const ProbeArgs& a);
size_t probe_p1_scratch_floats(int64_t N, int H);
hipError_t launch_probe_p1(const ProbeArgs& a, float* scratch, bool bf16, hipStream_t s);

// out[r] = mean of the k largest |vals[r, 0..n)|, rows of T with leading dimension ld (elements)
hipError_t launch_topk_mean(const void* vals, int64_t ld, int64_t rows, int64_t n, int64_t k, float* out, bool bf16,
                            hipStream_t s);

// ------------------------------------------------------------------ decode phase (one new token)
enum GemvMode : int {
    GEMV_STORE = 0,   // y[r] = W[r,:].x                     (T)
    GEMV_SILU = 1,    // y[r] = silu(W0[r,:].x) * W1[r,:].x  (T; R[0] rows each)
    GEMV_RESID = 2,   // y[r] += W[r,:].x                    (T, read-modify-write)
    GEMV_F32 = 3,     // y[r] = W[r,:].x                     (fp32)
    GEMV_QKV_ROPE = 4, // W[0], W[1]: rotary embedding of the products for one position (table `rope`), W[2]: plain store
};
// Up to three row-major matrices W[i] [R[i], K] that share the input vector x [K]; y[i] [R[i]].
// R[i] % 4 == 0, K a multiple of the 16-byte chunk; GEMV_SILU uses W[0] (gate), W[1] (up), y[0].
// gamma != NULL: x is the raw hidden state and every workgroup applies RMSNorm(x; gamma, eps) to it
// first (same arithmetic as the RMSNorm kernel); needs K <= 1024 chunks of 16 bytes.
struct GemvArgs {
    const void* W[3]; void* y[3]; int32_t R[3];
    const void* x; int32_t K; int mode;
    const void* gamma; float eps;
    const float2* rope; int32_t head_dim;   // GEMV_QKV_ROPE: (cos, sin)[head_dim / 2] of the token's position
    int32_t* pos_out; int32_t pos_val;      // GEMV_QKV_ROPE: *pos_out = pos_val (the cache row's position), when not NULL
};
bool gemv_supported(const GemvArgs& a, bool bf16);
hipError_t launch_gemv(const GemvArgs& a, bool bf16, hipStream_t s);
// (cos, sin) of one position for the decode GEMV's rotary epilogue: table[j] = (cos, sin)(pos * base^(-2j/d))
hipError_t launch_decode_rope_row(int pos, int d, float base, float2* table, hipStream_t s);
// rotary embedding of q [H, d] in place and of k [Hkv, d] into cache row `row`, v copied to that row
hipError_t launch_decode_rope_append(void* q, const void* k, const void* v, int pos, int H, int Hkv, int d, float base,
                                     void* cache_k, void* cache_v, int32_t* cache_pos, int64_t row, bool bf16, hipStream_t s);
// out [H, d] = softmax(q K^T / sqrt(d)) V over the M cached pairs K, V [M, Hkv, d]; part: fp32 scratch
bool decode_attn_supported(int H, int Hkv, int d, bool bf16);
size_t decode_attn_min_scratch_floats(int Hkv, int d);
hipError_t launch_decode_attn(const void* q, const void* K, const void* V, int64_t M, int H, int Hkv, int d, float* part,
                              size_t part_floats, void* out, bool bf16, hipStream_t s);
// A decode step over a few sequences at once: by-value descriptor of their caches (device pointers), the row
// each appends to (= its current count) and the new token's position.
constexpr int DECODE_MAX_BATCH = 16;
struct DecodeBatch {
    void* cache_k[DECODE_MAX_BATCH]; void* cache_v[DECODE_MAX_BATCH]; int32_t* cache_pos[DECODE_MAX_BATCH];
    int64_t count[DECODE_MAX_BATCH]; int32_t pos[DECODE_MAX_BATCH]; int32_t n;
};
// Y[b, r] = W[r, :] . X[b, :] for nb <= DECODE_MAX_BATCH input vectors (X [nb, K], Y[i] [nb, R[i]] contiguous); modes STORE, SILU,
// RESID, F32; no fused norm
hipError_t launch_gemv_nb(const GemvArgs& a, int nb, bool bf16, hipStream_t s);
// fp32 projection sums q32 [n, H, d], k32 / v32 [n, Hkv, d] -> q [n, H, d] rotated, k rotated / v copied into row count[b] of
// sequence b's cache; one rounding to the element type, after the rotation
hipError_t launch_decode_rope_append_batched(const float* q32, const float* k32, const float* v32, void* q, int H, int Hkv, int d,
                                             float base, const DecodeBatch& db, bool bf16, hipStream_t s);
// out [n, H, d]: attention of sequence b's query over its count[b] + 1 cached pairs
hipError_t launch_decode_attn_batched(const void* q, const DecodeBatch& db, int H, int Hkv, int d, float* part, size_t part_floats,
                                      void* out, bool bf16, hipStream_t s);
// token = argmax(logits [V]) with ties to the lowest id; x_next [D] = table[token, :] (skipped when NULL)
hipError_t launch_argmax_row(const float* logits, int V, int32_t* token, const void* table, int D, void* x_next, bool bf16,
                             hipStream_t s);

}  // namespace spts
