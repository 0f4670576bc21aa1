// C ABI of libspts: argument validation, workspace carving and the launch sequence of each call.
// No arithmetic of the method lives here; every step runs in the kernels of this library.
#include "../../include/spts.h"
#include "spts_internal.h"

#include <algorithm>
#include <new>
#include <vector>

using namespace spts;

namespace {

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

struct Workspace {
    size_t rope, xn, kall, tmp32, qp, probe, S, C, SF, part, idxA, idxF, posA, q, khat, vhat, vt, att, t, z, big, misc, seg, topk;
    size_t total;
};

struct Limits { int64_t max_tokens; int32_t max_probe, max_r, max_dlow; };

Workspace carve(const spts_model_desc& m, const Limits& L) {
    Workspace w{};
    const size_t b = m.dtype == SPTS_BF16 ? 2 : 4;
    const size_t Nm = (size_t)L.max_tokens;
    const size_t Np = (Nm + 255) / 256 * 256;  // row padding for tile-granular kernels
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    w.rope = take(Np * (size_t)(m.d / 2) * sizeof(float2));
    w.xn = take(Np * m.D * b);
    w.kall = take(Np * (size_t)m.Hkv * m.d * b);
    w.tmp32 = take(Np * (size_t)m.H * m.d * 4);
    w.qp = take((size_t)(L.max_probe + 256) * m.H * m.d * b);
    w.probe = take(probe_scratch_floats(L.max_tokens, L.max_probe, m.H, m.Hkv) * 4);
    w.S = take(Np * 4);
    w.C = take(Np * 4);
    w.SF = take(Np * 4);
    w.part = take(Np * (size_t)((m.D + 63) / 64) * 4);
    w.idxA = take(Np * 4);
    w.idxF = take(Np * 4);
    w.posA = take(Np * 4);
    w.q = take(Np * (size_t)m.H * m.d * b);
    w.khat = take(Np * (size_t)m.Hkv * m.d * b);
    w.vhat = take(Np * (size_t)m.Hkv * m.d * b);
    w.vt = take((size_t)m.Hkv * m.d * (Np + 256) * b);
    w.att = take(Np * (size_t)m.H * m.d * b);
    w.t = take(Np * (size_t)(2 * L.max_r) * b);
    w.z = take(Np * (size_t)L.max_r * b);
    size_t inner = (size_t)(m.Dff > L.max_dlow ? m.Dff : L.max_dlow);
    w.big = take(Np * inner * b);
    w.misc = take(4096);
    w.seg = take(3 * (size_t)(SPTS_MAX_BATCH + 1) * sizeof(int64_t));   // segment descriptors of a batched call
    w.topk = take(TOPK_MULTI_SCRATCH_BYTES);                             // tables of the chip-wide TopK
    w.total = off;
    return w;
}

bool model_ok(const spts_model_desc* m, int* status) {
    if (!m) { *status = SPTS_EINVAL; return false; }
    if (m->dtype != SPTS_F32 && m->dtype != SPTS_BF16) { *status = SPTS_EDTYPE; return false; }
    if (m->D <= 0 || m->H <= 0 || m->Hkv <= 0 || m->d <= 0 || m->Dff <= 0) { *status = SPTS_EINVAL; return false; }
    if (m->H % m->Hkv != 0 || (m->d & 1) || m->d > 256) { *status = SPTS_ESHAPE; return false; }
    if (!(m->rms_eps >= 0.f) || !(m->rope_base > 0.f)) { *status = SPTS_EINVAL; return false; }
    *status = SPTS_OK;
    return true;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

struct spts_ctx {
    spts_model_desc m;
    Limits lim;
    hipStream_t stream;
    char* ws;
    Workspace off;
    bool bf16;
    int last_hip;
    int64_t dec_rope_pos = -1;   // position whose (cos, sin) row sits at the start of the rotary table (decode), -1 = none
    // per-phase timing (spts_profile_*): events recorded around the launches of each phase
    bool prof_on = false;
    std::vector<hipEvent_t> ev_pool;
    size_t ev_used = 0;
    struct Rec { int phase; hipEvent_t a, b; };
    std::vector<Rec> recs;
    double phase_ms[32] = {};
    int64_t phase_n[32] = {};
    template <typename T> T* p(size_t o) const { return reinterpret_cast<T*>(ws + o); }
};

enum PhaseId {
    PH_ROPE_TABLE = 0, PH_RMSNORM, PH_K_PROJ, PH_PROBE_Q, PH_PROBE_ATTN, PH_TOPK, PH_GATHER, PH_Q_PROJ, PH_V_PROJ,
    PH_ATTENTION, PH_O_PROJ, PH_PROXY_IN, PH_PROXY_MID, PH_PROXY_Z, PH_PROXY_OUT, PH_FFN_GATE_UP, PH_FFN_DOWN,
    PH_COMPACT, PH_DEC_NORM, PH_DEC_QKV, PH_DEC_ROPE_APPEND, PH_DEC_ATTN, PH_DEC_O, PH_DEC_GATE_UP, PH_DEC_DOWN, PH_DEC_HEAD,
    PH_BUILD_SALIENCY, PH_BUILD_TOPMEAN, PH_QV_PROJ,
    PH_COUNT
};
static const char* const kPhaseNames[PH_COUNT] = {
    "rope_table", "rmsnorm", "k_proj", "probe_q", "probe_attn", "topk", "gather", "q_proj", "v_proj",
    "attention", "o_proj", "proxy_in", "proxy_mid", "proxy_z", "proxy_out", "ffn_gate_up", "ffn_down", "compact",
    "dec_rmsnorm", "dec_qkv", "dec_rope_append", "dec_attention", "dec_o_proj", "dec_gate_up", "dec_down", "dec_head",
    "build_saliency", "build_topmean", "qv_proj"};

// Brackets the launches issued during its lifetime with two events when profiling is on.
struct PhaseScope {
    spts_ctx* c; int rec = -1;
    PhaseScope(spts_ctx* ctx, int phase) : c(ctx) {
        if (!c->prof_on) return;
        hipEvent_t e[2];
        for (int i = 0; i < 2; ++i) {
            if (c->ev_used == c->ev_pool.size()) {
                hipEvent_t n;
                if (hipEventCreate(&n) != hipSuccess) return;
                c->ev_pool.push_back(n);
            }
            e[i] = c->ev_pool[c->ev_used++];
        }
        if (hipEventRecord(e[0], c->stream) != hipSuccess) return;
        c->recs.push_back({phase, e[0], e[1]});
        rec = (int)c->recs.size() - 1;
    }
    ~PhaseScope() { if (rec >= 0) (void)hipEventRecord(c->recs[rec].b, c->stream); }
};
#define PHASE(ctx, id) PhaseScope phase_scope__(ctx, id)

#define SPTS_HIP(ctx, expr)                                                   \
    do {                                                                      \
        hipError_t e__ = (expr);                                              \
        if (e__ != hipSuccess) { (ctx)->last_hip = (int)e__; return SPTS_EHIP; } \
    } while (0)
#define SPTS_TRY(expr)                       \
    do {                                     \
        int s__ = (expr);                    \
        if (s__ != SPTS_OK) return s__;      \
    } while (0)

namespace {

// ---- dispatch helpers -------------------------------------------------------------------------
// matrix-core launch; the partly filled last round of tiles is split over K through the fp32 staging buffer
int run_gemm_mfma(spts_ctx* c, GemmArgs a) {
    int32_t nfull = 0;
    const int ks = gemm_pick_split(a.M, a.N, a.K, a.epi, &nfull);
    if (ks > 1) {
        const int64_t tiles = (a.M + 255) / 256 * (a.N / 256);
        const size_t need = (size_t)(tiles - nfull) * ks * 65536 * sizeof(float);
        const size_t have = (size_t)((c->lim.max_tokens + 255) / 256 * 256) * c->m.H * c->m.d * sizeof(float);
        if (need <= have) { a.ksplit = ks; a.nfull = nfull; a.part32 = c->p<float>(c->off.tmp32); }
    }
    SPTS_HIP(c, launch_gemm_mfma(a, c->stream));
    return SPTS_OK;
}

int run_gemm(spts_ctx* c, const GemmArgs& a) {
    if (c->bf16 && gemm_mfma_supported(a)) return run_gemm_mfma(c, a);
    SPTS_HIP(c, launch_gemm_generic(a, c->bf16, c->stream));
    return SPTS_OK;
}

GemmArgs gemm_args(const void* A, int64_t lda, const int32_t* a_idx, const void* B, int64_t ldb, void* C, int64_t ldc,
                   int64_t M, int32_t N, int32_t K, int epi = EPI_STORE) {
    GemmArgs g{};
    g.A = A; g.lda = lda; g.a_idx = a_idx; g.B0 = B; g.B1 = nullptr; g.ldb = ldb; g.C = C; g.ldc = ldc;
    g.M = M; g.N = N; g.K = K; g.epi = epi;
    return g;
}

// B (one weight matrix, or the gate / up pair) through its slab-major copy when the caller gave one and the
// matrix-core kernel serves the call with it; otherwise g keeps the row-major pointers
void prefer_slab(const spts_ctx* c, GemmArgs& g, const void* s0, const void* s1, int64_t rows, int64_t rows1 = 0) {
    if (!c->bf16 || !s0 || (g.B1 && !s1)) return;
    GemmArgs t = g;
    t.B0 = s0; if (g.B1) t.B1 = s1;
    t.b_slab = 1; t.b_rows = rows; t.b_rows1 = rows1;
    if (gemm_mfma_supported(t)) g = t;
}

// The FFN's hidden activations in slab-major layout when both matrix-core GEMMs take it: gate/up writes them that way
// and down reads its A operand as whole cache lines (the buffer is the library's own, so the layout is free)
void hidden_slab(const spts_ctx* c, GemmArgs& gate_up, GemmArgs& down) {
    if (!c->bf16) return;
    GemmArgs tg = gate_up, td = down;
    tg.c_slab = 1; td.a_slab = 1;
    if (gemm_mfma_supported(tg) && gemm_mfma_supported(td)) { gate_up = tg; down = td; }
}

// Factor the prefill folds into the queries it stores (probe window and active rows): in bf16 log2(e)/sqrt(d), applied
// to the fp32 accumulators before their one rounding; in fp32 none.
float query_store_scale(const spts_ctx* c) { return c->bf16 ? attention_mfma_q_scale(c->m.d) : 1.0f; }

// out[rows, heads*d] = out_scale * rotary(A * B^T); table row of output row i is (tidx ? tidx[i] : i + row0); b_slab:
// optional slab-major copy of B (heads*d rows)
int run_gemm_rope(spts_ctx* c, GemmArgs g, int heads, const int32_t* tidx, int64_t row0, void* out, const void* b_slab = nullptr,
                  float out_scale = 1.0f) {
    const float2* table = c->p<float2>(c->off.rope);
    GemmArgs f = g;
    f.epi = EPI_ROPE; f.C = out; f.rope = table + row0 * (c->m.d / 2); f.rope_idx = tidx; f.head_dim = c->m.d;
    f.rope_scale = out_scale;
    prefer_slab(c, f, b_slab, nullptr, g.N);
    if (c->bf16 && gemm_mfma_supported(f)) return run_gemm_mfma(c, f);
    g.C = c->p<float>(c->off.tmp32); g.c_is_f32 = 1; g.epi = EPI_STORE;
    SPTS_TRY(run_gemm(c, g));
    SPTS_HIP(c, launch_rope_apply(c->p<float>(c->off.tmp32), table, tidx, row0, out, g.M, heads, c->m.d, c->bf16, c->stream, out_scale));
    return SPTS_OK;
}

int check_weights_attn(const spts_layer_weights* w) {
    if (!w || !w->Wq || !w->Wk || !w->gamma1) return SPTS_EINVAL;
    if (!aligned16(w->Wq) || !aligned16(w->Wk) || !aligned16(w->gamma1)) return SPTS_EALIGN;
    return SPTS_OK;
}
int check_weights_proxy(const spts_ctx* c, const spts_layer_weights* w) {
    if (!w || !w->gamma2 || !w->Ug || !w->Vg || !w->Uu || !w->Vu || !w->Ud || !w->Vd) return SPTS_EINVAL;
    if (w->r <= 0 || w->Dlow <= 0) return SPTS_EINVAL;
    if (w->r > c->lim.max_r || w->Dlow > c->lim.max_dlow) return SPTS_EWORKSPACE;
    const void* ps[] = {w->gamma2, w->Ug, w->Vg, w->Uu, w->Vu, w->Ud, w->Vd, w->Vg_s, w->Vu_s, w->Vd_s, w->Ug_s, w->Uu_s};   // the copies may be NULL
    for (const void* p : ps) if (!aligned16(p)) return SPTS_EALIGN;
    return SPTS_OK;
}
int check_weights_full(const spts_ctx* c, const spts_layer_weights* w, bool need_proxy) {
    SPTS_TRY(check_weights_attn(w));
    if (!w->Wv || !w->Wo || !w->Wgate || !w->Wup || !w->Wdown || !w->gamma2) return SPTS_EINVAL;
    const void* ps[] = {w->Wv, w->Wo, w->Wgate, w->Wup, w->Wdown, w->gamma2,
                        w->Wq_s, w->Wk_s, w->Wv_s, w->Wo_s, w->Wgate_s, w->Wup_s, w->Wdown_s};   // the copies may be NULL
    for (const void* p : ps) if (!aligned16(p)) return SPTS_EALIGN;
    if (need_proxy) SPTS_TRY(check_weights_proxy(c, w));
    return SPTS_OK;
}

// ---- PAP probe: norm, keys, probe queries, scores ----------------------------------------------
// scores of the candidates [row0, row0 + n) of the rows that norm_keys_impl prepared: the last P of them
// are the probe queries, k_rows points at the keys of row row0
int probe_scores_rows(spts_ctx* c, int64_t row0, int64_t n, const spts_layer_weights* w, int P, const void* k_rows, float* s_out) {
    const auto& m = c->m;
    const int QD = m.H * m.d;
    const size_t eb = c->bf16 ? 2 : 4;
    const char* xn_probe = c->p<char>(c->off.xn) + (size_t)(row0 + n - P) * m.D * eb;
    ProbeArgs pa{};
    pa.qp = c->p<void>(c->off.qp); pa.k = k_rows; pa.S = s_out;
    pa.stats = c->p<float>(c->off.probe);
    pa.partial = c->p<float>(c->off.probe) + (2 * (size_t)P * m.H + 64);
    pa.N = n; pa.P = P; pa.H = m.H; pa.Hkv = m.Hkv; pa.d = m.d;
    const bool p1 = probe_p1_supported(pa);
    const bool pmf = !p1 && c->bf16 && probe_mfma_supported(pa);
    // bf16: the queries leave the projection already multiplied by log2(e)/sqrt(d), before their one rounding (the
    // matrix-core kernels then get exponents of 2 straight from the MFMA; the other kernels divide their scale by it)
    pa.q_scale = query_store_scale(c);
    GemmArgs gq = gemm_args(xn_probe, m.D, nullptr, w->Wq, m.D, nullptr, QD, P, QD, m.D);
    { PHASE(c, PH_PROBE_Q); SPTS_TRY(run_gemm_rope(c, gq, m.H, nullptr, row0 + n - P, c->p<void>(c->off.qp), w->Wq_s, pa.q_scale)); }
    PHASE(c, PH_PROBE_ATTN);
    if (p1) SPTS_HIP(c, launch_probe_p1(pa, c->p<float>(c->off.probe), c->bf16, c->stream));
    else if (pmf) SPTS_HIP(c, launch_probe_mfma(pa, c->stream));
    else SPTS_HIP(c, launch_probe_generic(pa, c->bf16, c->stream));
    return SPTS_OK;
}

// leaves xn (normalised x) and the rotary table in the workspace for the caller
int probe_attn_impl(spts_ctx* c, const void* x, const int32_t* pos, int64_t N, const spts_layer_weights* w, int P,
                    bool want_scores, void* k_out, float* s_out) {
    const auto& m = c->m;
    c->dec_rope_pos = -1;   // the prefill's table overwrites the decode row
    { PHASE(c, PH_ROPE_TABLE); SPTS_HIP(c, launch_rope_table(pos, N, m.d, m.rope_base, c->p<float2>(c->off.rope), c->stream)); }
    { PHASE(c, PH_RMSNORM); SPTS_HIP(c, launch_rmsnorm(x, w->gamma1, m.rms_eps, c->p<void>(c->off.xn), N, m.D, c->bf16, c->stream)); }
    const int KV = m.Hkv * m.d;
    GemmArgs gk = gemm_args(c->p<void>(c->off.xn), m.D, nullptr, w->Wk, m.D, nullptr, KV, N, KV, m.D);
    { PHASE(c, PH_K_PROJ); SPTS_TRY(run_gemm_rope(c, gk, m.Hkv, nullptr, 0, k_out, w->Wk_s)); }
    if (!want_scores) return SPTS_OK;
    return probe_scores_rows(c, 0, N, w, P, k_out, s_out);
}

// ---- LTP probe on an already normalised xn2 [N, D] ---------------------------------------------
int proxy_scores_impl(spts_ctx* c, const void* xn2, int64_t N, const spts_layer_weights* w, const float* s_mha,
                      float* c_ffn, float* s_ffn) {
    const auto& m = c->m;
    const int r = w->r, Dlow = w->Dlow;
    const size_t eb = c->bf16 ? 2 : 4;
    char* t = c->p<char>(c->off.t);  // [N, 2r]: columns [0,r) = x Ug, [r,2r) = x Uu
    // hp = silu(tg Vg) * (tu Vu)   [N, Dlow]
    GemmArgs g3 = gemm_args(t, 2 * r, nullptr, w->Vg, r, c->p<void>(c->off.big), Dlow, N, Dlow, r, EPI_SILU_MUL);
    g3.B1 = w->Vu; g3.A1 = t + (size_t)r * eb;
    prefer_slab(c, g3, w->Vg_s, w->Vu_s, Dlow);
    // z = hp Vd^T   [N, r]
    GemmArgs g4 = gemm_args(c->p<void>(c->off.big), Dlow, nullptr, w->Vd, Dlow, c->p<void>(c->off.z), r, N, r, Dlow);
    prefer_slab(c, g4, w->Vd_s, nullptr, r);
    hidden_slab(c, g3, g4);
    {
        PHASE(c, PH_PROXY_IN);
        // one launch for both factors when the matrix-core kernel takes it (columns [0,r) from Ug, [r,2r) from Uu)
        GemmArgs g12 = gemm_args(xn2, m.D, nullptr, w->Ug, m.D, t, 2 * r, N, 2 * r, m.D);
        g12.B1 = w->Uu;
        prefer_slab(c, g12, w->Ug_s, w->Uu_s, r);
        if (c->bf16 && gemm_mfma_supported(g12)) {
            // t slab-major between the two launches when both take it: [2r/32][N][32], t_u starts r/32 slabs in
            GemmArgs s12 = g12, s3 = g3;
            s12.c_slab = 1;
            s3.a_slab = 1; s3.A1 = t + (size_t)(r / 32) * (size_t)N * 64;
            if (r % 32 == 0 && gemm_mfma_supported(s12) && gemm_mfma_supported(s3)) { g12 = s12; g3 = s3; }
            SPTS_TRY(run_gemm_mfma(c, g12));
        } else {
            GemmArgs g1 = gemm_args(xn2, m.D, nullptr, w->Ug, m.D, t, 2 * r, N, r, m.D);
            SPTS_TRY(run_gemm(c, g1));
            GemmArgs g2 = gemm_args(xn2, m.D, nullptr, w->Uu, m.D, t + (size_t)r * eb, 2 * r, N, r, m.D);
            SPTS_TRY(run_gemm(c, g2));
        }
    }
    {
        PHASE(c, PH_PROXY_MID);
        // hidden layer: the register-stationary kernel when the projection behind it reads the hidden state slab-major
        // and the factors come with their slab-major copies; else the dual-product GEMM
        ProxyHiddenArgs ph{};
        ph.Vg_s = w->Vg_s; ph.Vu_s = w->Vu_s; ph.hp = c->p<void>(c->off.big); ph.N = N; ph.Dlow = Dlow; ph.r = r;
        if (g3.a_slab) { ph.tg = t; ph.tu = t + (size_t)(r / 32) * (size_t)N * 64; ph.t_row_pitch = 64; ph.t_slab_pitch = N * 64; }
        else { ph.tg = t; ph.tu = t + (size_t)r * eb; ph.t_row_pitch = (int64_t)2 * r * eb; ph.t_slab_pitch = 64; }
        if (c->bf16 && g4.a_slab && proxy_hidden_supported(ph)) SPTS_HIP(c, launch_proxy_hidden(ph, c->stream));
        else SPTS_TRY(run_gemm(c, g3));
    }
    { PHASE(c, PH_PROXY_Z); SPTS_TRY(run_gemm(c, g4)); }
    if (w->Ud_orthonormal) {
        // ||z Ud^T|| = ||z|| when the columns of Ud are orthonormal (what a truncated SVD with Sigma folded into V
        // gives): the output projection is not evaluated at all
        PHASE(c, PH_PROXY_OUT);
        SPTS_HIP(c, launch_row_norm_scores(c->p<void>(c->off.z), r, c->bf16, s_mha, c_ffn, s_ffn, N, c->stream));
        return SPTS_OK;
    }
    // o = z Ud^T [N, D] is never stored: per-block sums of squares, then the square root
    GemmArgs g5 = gemm_args(c->p<void>(c->off.z), r, nullptr, w->Ud, r, nullptr, 0, N, m.D, r, EPI_SUMSQ);
    bool mf = c->bf16 && gemm_mfma_supported(g5);
    int nb = gemm_sumsq_blocks(m.D, mf);
    g5.part = c->p<float>(c->off.part); g5.part_ld = nb;
    PHASE(c, PH_PROXY_OUT);
    SPTS_TRY(run_gemm(c, g5));
    SPTS_HIP(c, launch_finish_ffn_scores(c->p<float>(c->off.part), nb, s_mha, c_ffn, s_ffn, N, c->stream));
    return SPTS_OK;
}

// out[i, :] = in[idx[i], :] with the position gather and the old->new map (each optional) in the same launch when rows
// are whole 16-byte vectors, else as separate launches
int gather_rows_maps(spts_ctx* c, const void* in, const int32_t* idx, void* out, int64_t n, int64_t row_bytes,
                     const int32_t* pos_in, int32_t* pos_out, int32_t* old2new) {
    if (row_bytes % 16 == 0) {
        SPTS_HIP(c, launch_gather_rows_maps(in, idx, out, n, row_bytes, pos_in, pos_out, old2new, c->stream));
        return SPTS_OK;
    }
    SPTS_HIP(c, launch_gather_rows(in, idx, out, n, row_bytes, c->stream));
    if (pos_out) SPTS_HIP(c, launch_gather_i32(pos_in, idx, pos_out, n, c->stream));
    if (old2new) SPTS_HIP(c, launch_scatter_iota(idx, old2new, n, c->stream));
    return SPTS_OK;
}

// TopK of one score row: longer rows are spread over the chip (a launch per radix pass), short ones stay in one workgroup
int run_topk(spts_ctx* c, const float* scores, int64_t N, int64_t k, int protect_last, int32_t* idx_out) {
    if (N >= TOPK_MULTI_MIN_N && N <= TOPK_MULTI_MAX_N)
        SPTS_HIP(c, launch_topk_multi(scores, N, k, protect_last, idx_out, c->p<void>(c->off.topk), c->stream));
    else
        SPTS_HIP(c, launch_topk(scores, N, k, protect_last, idx_out, 1, c->stream));
    return SPTS_OK;
}

int common_call_checks(const spts_ctx* c, int64_t N) {
    if (!c) return SPTS_EINVAL;
    if (N < 0) return SPTS_EINVAL;
    if (N > c->lim.max_tokens) return SPTS_EWORKSPACE;
    if (N > 0x7fffffff) return SPTS_ESHAPE;
    return SPTS_OK;
}

}  // namespace

extern "C" {

const char* spts_strerror(int status) {
    switch (status) {
        case SPTS_OK: return "ok";
        case SPTS_EINVAL: return "invalid argument";
        case SPTS_ESHAPE: return "unsupported shape";
        case SPTS_EALIGN: return "pointer not 16-byte aligned";
        case SPTS_EWORKSPACE: return "workspace too small for this call";
        case SPTS_EDTYPE: return "unsupported dtype";
        case SPTS_EHIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

size_t spts_workspace_bytes(const spts_model_desc* model, int64_t max_tokens, int32_t max_probe, int32_t max_r,
                            int32_t max_dlow) {
    int st;
    if (!model_ok(model, &st)) return 0;
    if (max_tokens <= 0 || max_probe <= 0 || max_r <= 0 || max_dlow <= 0) return 0;
    Limits L{max_tokens, max_probe, max_r, max_dlow};
    return carve(*model, L).total;
}

int spts_create(spts_ctx** ctx, const spts_model_desc* model, void* hip_stream, void* workspace, size_t workspace_bytes,
                int64_t max_tokens, int32_t max_probe, int32_t max_r, int32_t max_dlow) {
    if (!ctx) return SPTS_EINVAL;
    *ctx = nullptr;
    int st;
    if (!model_ok(model, &st)) return st;
    if (max_tokens <= 0 || max_probe <= 0 || max_r <= 0 || max_dlow <= 0 || !workspace) return SPTS_EINVAL;
    if (!aligned16(workspace)) return SPTS_EALIGN;
    Limits L{max_tokens, max_probe, max_r, max_dlow};
    Workspace w = carve(*model, L);
    if (workspace_bytes < w.total) return SPTS_EWORKSPACE;
    spts_ctx* c = new (std::nothrow) spts_ctx();
    if (!c) return SPTS_EINVAL;
    c->m = *model; c->lim = L; c->stream = (hipStream_t)hip_stream; c->ws = (char*)workspace; c->off = w;
    c->bf16 = model->dtype == SPTS_BF16; c->last_hip = 0;
    *ctx = c;
    return SPTS_OK;
}

void spts_destroy(spts_ctx* ctx) {
    if (!ctx) return;
    for (hipEvent_t e : ctx->ev_pool) (void)hipEventDestroy(e);
    delete ctx;
}

int spts_profile_begin(spts_ctx* c) {
    if (!c) return SPTS_EINVAL;
    c->recs.clear();
    c->ev_used = 0;
    for (int i = 0; i < PH_COUNT; ++i) { c->phase_ms[i] = 0.0; c->phase_n[i] = 0; }
    c->prof_on = true;
    return SPTS_OK;
}

int spts_profile_end(spts_ctx* c) {
    if (!c) return SPTS_EINVAL;
    c->prof_on = false;
    SPTS_HIP(c, hipStreamSynchronize(c->stream));
    for (const auto& r : c->recs) {
        float ms = 0.f;
        SPTS_HIP(c, hipEventElapsedTime(&ms, r.a, r.b));
        c->phase_ms[r.phase] += ms;
        c->phase_n[r.phase] += 1;
    }
    c->recs.clear();
    c->ev_used = 0;
    return SPTS_OK;
}

int spts_profile_count(const spts_ctx* c) { return c ? (int)PH_COUNT : 0; }

int spts_profile_get(const spts_ctx* c, int i, const char** name, double* total_ms, int64_t* launches) {
    if (!c || i < 0 || i >= PH_COUNT) return SPTS_EINVAL;
    if (name) *name = kPhaseNames[i];
    if (total_ms) *total_ms = c->phase_ms[i];
    if (launches) *launches = c->phase_n[i];
    return SPTS_OK;
}

int spts_last_hip_error(const spts_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

int spts_uses_mfma(const spts_ctx* ctx) {
    if (!ctx || !ctx->bf16) return 0;
    const auto& m = ctx->m;
    GemmArgs g = gemm_args((const void*)16, m.D, nullptr, (const void*)16, m.D, (void*)16, m.Dff, 256, m.Dff, m.D);
    return gemm_mfma_supported(g) ? 1 : 0;
}

int spts_probe_attn(spts_ctx* c, const void* x, const int32_t* pos, int64_t N, const spts_layer_weights* w,
                    int32_t probe_len, void* k_out, float* s_mha) {
    SPTS_TRY(common_call_checks(c, N));
    if (N == 0) return SPTS_OK;
    if (!x || !pos || !k_out || !s_mha) return SPTS_EINVAL;
    if (!aligned16(x) || !aligned16(pos) || !aligned16(k_out) || !aligned16(s_mha)) return SPTS_EALIGN;
    SPTS_TRY(check_weights_attn(w));
    if (probe_len < 1 || probe_len > N) return SPTS_EINVAL;
    if (probe_len > c->lim.max_probe) return SPTS_EWORKSPACE;
    return probe_attn_impl(c, x, pos, N, w, probe_len, true, k_out, s_mha);
}

int spts_probe_ffn(spts_ctx* c, const void* x, int64_t N, const spts_layer_weights* w, const float* s_mha, float* c_ffn,
                   float* s_ffn) {
    SPTS_TRY(common_call_checks(c, N));
    if (N == 0) return SPTS_OK;
    if (!x || !s_ffn) return SPTS_EINVAL;
    if (!aligned16(x) || !aligned16(s_ffn) || (s_mha && !aligned16(s_mha)) || (c_ffn && !aligned16(c_ffn))) return SPTS_EALIGN;
    SPTS_TRY(check_weights_proxy(c, w));
    { PHASE(c, PH_RMSNORM); SPTS_HIP(c, launch_rmsnorm(x, w->gamma2, c->m.rms_eps, c->p<void>(c->off.xn), N, c->m.D, c->bf16, c->stream)); }
    return proxy_scores_impl(c, c->p<void>(c->off.xn), N, w, s_mha, c_ffn, s_ffn);
}

int spts_select_topk(spts_ctx* c, const float* scores, int64_t N, int64_t k, int32_t protect_last, int32_t* idx_out) {
    SPTS_TRY(common_call_checks(c, N));
    if (k < 0 || k > N) return SPTS_EINVAL;
    if (k == 0) return SPTS_OK;
    if (!scores || !idx_out) return SPTS_EINVAL;
    if (!aligned16(scores) || !aligned16(idx_out)) return SPTS_EALIGN;
    PHASE(c, PH_TOPK);
    return run_topk(c, scores, N, k, protect_last, idx_out);
}

static_assert(SPTS_TOPK_STATIC_MAX_N <= TOPK_MULTI_MAX_N, "the static scratch's tables cover the documented maximum");

int spts_select_topk_static(void* hip_stream, const float* scores, int64_t N, int64_t k, int32_t protect_last, int32_t* idx_out) {
    if (N < 0 || k < 0 || k > N) return SPTS_EINVAL;
    if (N > SPTS_TOPK_STATIC_MAX_N) return SPTS_ESHAPE;
    if (k == 0) return SPTS_OK;
    if (!scores || !idx_out) return SPTS_EINVAL;
    if (!aligned16(scores) || !aligned16(idx_out)) return SPTS_EALIGN;
    void* scr = nullptr;
    if (topk_static_scratch(&scr) != hipSuccess) return SPTS_EHIP;
    if (launch_topk_multi(scores, N, k, protect_last, idx_out, scr, (hipStream_t)hip_stream) != hipSuccess) return SPTS_EHIP;
    return SPTS_OK;
}

int spts_select_topk_batched(spts_ctx* c, const float* scores, int64_t N, int64_t k, int32_t protect_last, int32_t batch,
                             int32_t* idx_out) {
    SPTS_TRY(common_call_checks(c, N));
    if (k < 0 || k > N || batch < 0 || batch > 65535) return SPTS_EINVAL;
    if (k == 0 || batch == 0) return SPTS_OK;
    if (!scores || !idx_out) return SPTS_EINVAL;
    if (!aligned16(scores) || !aligned16(idx_out)) return SPTS_EALIGN;
    PHASE(c, PH_TOPK);
    SPTS_HIP(c, launch_topk(scores, N, k, protect_last, idx_out, batch, c->stream));
    return SPTS_OK;
}

int spts_decode_layer(spts_ctx* c, void* x, int32_t pos, const spts_layer_weights* w, spts_kv_out* cache) {
    if (!c || !x || !w || !cache) return SPTS_EINVAL;
    if (pos < 0 || cache->count < 0 || cache->count >= cache->capacity) return SPTS_EINVAL;
    if (!cache->k || !cache->v || !cache->pos) return SPTS_EINVAL;
    if (!w->Wq || !w->Wk || !w->Wv || !w->Wo || !w->gamma1 || !w->Wgate || !w->Wup || !w->Wdown || !w->gamma2) return SPTS_EINVAL;
    if (!aligned16(x) || !aligned16(cache->k) || !aligned16(cache->v) || !aligned16(cache->pos) || !aligned16(w->gamma1) ||
        !aligned16(w->gamma2))
        return SPTS_EALIGN;
    const auto& m = c->m;
    const int QD = m.H * m.d, KV = m.Hkv * m.d;
    void* xn = c->p<void>(c->off.xn);
    void* q = c->p<void>(c->off.q);
    void* kx = c->p<void>(c->off.khat);
    void* vx = c->p<void>(c->off.vhat);
    void* att = c->p<void>(c->off.att);
    void* hbuf = c->p<void>(c->off.big);
    float* part = c->p<float>(c->off.tmp32);
    const size_t part_floats = (c->off.qp - c->off.tmp32) / sizeof(float);

    // the two RMSNorms run inside the GEMVs that consume them when the row fits the kernel's registers
    GemvArgs qkv{}; qkv.mode = GEMV_STORE; qkv.x = xn; qkv.K = m.D;
    qkv.W[0] = w->Wq; qkv.W[1] = w->Wk; qkv.W[2] = w->Wv; qkv.R[0] = QD; qkv.R[1] = KV; qkv.R[2] = KV;
    qkv.y[0] = q; qkv.y[1] = kx; qkv.y[2] = vx;
    GemvArgs o{}; o.mode = GEMV_RESID; o.x = att; o.K = QD; o.W[0] = w->Wo; o.R[0] = m.D; o.y[0] = x;
    GemvArgs gu{}; gu.mode = GEMV_SILU; gu.x = xn; gu.K = m.D; gu.W[0] = w->Wgate; gu.W[1] = w->Wup; gu.R[0] = m.Dff; gu.y[0] = hbuf;
    GemvArgs dn{}; dn.mode = GEMV_RESID; dn.x = hbuf; dn.K = m.Dff; dn.W[0] = w->Wdown; dn.R[0] = m.D; dn.y[0] = x;
    if (!gemv_supported(qkv, c->bf16) || !gemv_supported(o, c->bf16) || !gemv_supported(dn, c->bf16)) return SPTS_ESHAPE;
    {   // the SiLU variant addresses two matrices through W[0], W[1] with R[0] rows each
        GemvArgs chk = gu; chk.R[1] = m.Dff;
        if (!gemv_supported(chk, c->bf16)) return SPTS_ESHAPE;
    }
    if (!decode_attn_supported(m.H, m.Hkv, m.d, c->bf16)) return SPTS_ESHAPE;
    if (part_floats < decode_attn_min_scratch_floats(m.Hkv, m.d)) return SPTS_EWORKSPACE;

    hipStream_t st = c->stream;
    const int64_t row = cache->count;
    bool fuse_norm;
    {
        GemvArgs t = qkv; t.x = x; t.gamma = w->gamma1; t.eps = m.rms_eps;
        fuse_norm = gemv_supported(t, c->bf16);
    }
    if (fuse_norm) {   // pays for Q/K/V (one launch less); the gate/up product is faster with the leaner plain kernel
        qkv.x = x; qkv.gamma = w->gamma1; qkv.eps = m.rms_eps;
    } else {
        PHASE(c, PH_DEC_NORM); SPTS_HIP(c, launch_rmsnorm(x, w->gamma1, m.rms_eps, xn, 1, m.D, c->bf16, st));
    }
    const size_t eb = c->bf16 ? 2 : 4;
    if (m.d % 4 == 0) {
        // rotary embedding in the GEMV's epilogue: q goes to the workspace, the rotated key and the value straight into
        // row `row` of the cache.  The (cos, sin) row of this position is shared by all layers of the token.
        if (c->dec_rope_pos != pos) {
            PHASE(c, PH_DEC_ROPE_APPEND);
            SPTS_HIP(c, launch_decode_rope_row(pos, m.d, m.rope_base, c->p<float2>(c->off.rope), st));
            c->dec_rope_pos = pos;
        }
        qkv.mode = GEMV_QKV_ROPE; qkv.rope = c->p<float2>(c->off.rope); qkv.head_dim = m.d;
        qkv.y[1] = (char*)cache->k + (size_t)row * KV * eb;
        qkv.y[2] = (char*)cache->v + (size_t)row * KV * eb;
        qkv.pos_out = cache->pos + row; qkv.pos_val = pos;
        PHASE(c, PH_DEC_QKV); SPTS_HIP(c, launch_gemv(qkv, c->bf16, st));
    } else {
        { PHASE(c, PH_DEC_QKV); SPTS_HIP(c, launch_gemv(qkv, c->bf16, st)); }
        PHASE(c, PH_DEC_ROPE_APPEND);
        SPTS_HIP(c, launch_decode_rope_append(q, kx, vx, pos, m.H, m.Hkv, m.d, m.rope_base, cache->k, cache->v, cache->pos, row,
                                              c->bf16, st));
    }
    { PHASE(c, PH_DEC_ATTN);
      SPTS_HIP(c, launch_decode_attn(q, cache->k, cache->v, row + 1, m.H, m.Hkv, m.d, part, part_floats, att, c->bf16, st)); }
    { PHASE(c, PH_DEC_O); SPTS_HIP(c, launch_gemv(o, c->bf16, st)); }
    { PHASE(c, PH_DEC_NORM); SPTS_HIP(c, launch_rmsnorm(x, w->gamma2, m.rms_eps, xn, 1, m.D, c->bf16, st)); }
    { PHASE(c, PH_DEC_GATE_UP); SPTS_HIP(c, launch_gemv(gu, c->bf16, st)); }
    { PHASE(c, PH_DEC_DOWN); SPTS_HIP(c, launch_gemv(dn, c->bf16, st)); }
    cache->count = row + 1;
    return SPTS_OK;
}

int spts_greedy_token(spts_ctx* c, const void* x, const void* gamma_f, const void* table, int32_t V, int32_t* token_out,
                      float* logits_out, void* x_next) {
    if (!c || !x || !gamma_f || !table || !token_out || V <= 0) return SPTS_EINVAL;
    if (!aligned16(x) || !aligned16(gamma_f) || !aligned16(table) || (logits_out && !aligned16(logits_out)) ||
        (x_next && !aligned16(x_next)))
        return SPTS_EALIGN;
    const auto& m = c->m;
    float* logits = logits_out;
    if (!logits) {
        if ((size_t)V * sizeof(float) > c->off.misc - c->off.big) return SPTS_EWORKSPACE;
        logits = c->p<float>(c->off.big);
    }
    void* xn = c->p<void>(c->off.xn);
    GemvArgs g{}; g.mode = GEMV_F32; g.x = xn; g.K = m.D; g.W[0] = table; g.R[0] = V; g.y[0] = logits;
    if (!gemv_supported(g, c->bf16)) return SPTS_ESHAPE;
    PHASE(c, PH_DEC_HEAD);
    // separate norm: over a table of this size the plain kernel streams faster than the fused one
    SPTS_HIP(c, launch_rmsnorm(x, gamma_f, m.rms_eps, xn, 1, m.D, c->bf16, c->stream));
    SPTS_HIP(c, launch_gemv(g, c->bf16, c->stream));
    SPTS_HIP(c, launch_argmax_row(logits, V, token_out, table, m.D, x_next, c->bf16, c->stream));
    return SPTS_OK;
}

int spts_decode_layer_batched(spts_ctx* c, void* x, const int32_t* pos, int32_t batch, const spts_layer_weights* w,
                              spts_kv_out* caches) {
    if (!c || batch < 0 || batch > SPTS_MAX_DECODE_BATCH) return SPTS_EINVAL;
    if (batch == 0) return SPTS_OK;
    if (!x || !pos || !w || !caches) return SPTS_EINVAL;
    if (!w->Wq || !w->Wk || !w->Wv || !w->Wo || !w->gamma1 || !w->Wgate || !w->Wup || !w->Wdown || !w->gamma2) return SPTS_EINVAL;
    if (!aligned16(x) || !aligned16(w->gamma1) || !aligned16(w->gamma2)) return SPTS_EALIGN;
    if (batch > c->lim.max_tokens) return SPTS_EWORKSPACE;
    DecodeBatch db{};
    db.n = batch;
    for (int b = 0; b < batch; ++b) {
        const spts_kv_out& kc = caches[b];
        if (pos[b] < 0 || kc.count < 0 || kc.count >= kc.capacity || !kc.k || !kc.v || !kc.pos) return SPTS_EINVAL;
        if (!aligned16(kc.k) || !aligned16(kc.v) || !aligned16(kc.pos)) return SPTS_EALIGN;
        for (int o = 0; o < b; ++o)
            if (caches[o].k == kc.k) return SPTS_EINVAL;   // one cache per sequence
        db.cache_k[b] = kc.k; db.cache_v[b] = kc.v; db.cache_pos[b] = kc.pos; db.count[b] = kc.count; db.pos[b] = pos[b];
    }
    const auto& m = c->m;
    const int QD = m.H * m.d, KV = m.Hkv * m.d;
    void* xn = c->p<void>(c->off.xn);
    void* q = c->p<void>(c->off.q);
    void* att = c->p<void>(c->off.att);
    void* hbuf = c->p<void>(c->off.big);
    float* part = c->p<float>(c->off.tmp32);
    const size_t part_floats = (c->off.qp - c->off.tmp32) / sizeof(float);
    // the projections leave fp32 sums (in the FFN's hidden buffer, free until gate/up); the rotary kernel rounds once
    float* q32 = c->p<float>(c->off.big);
    float* k32 = q32 + (size_t)batch * QD;
    float* v32 = k32 + (size_t)batch * KV;
    GemvArgs qkv{}; qkv.mode = GEMV_F32; qkv.x = xn; qkv.K = m.D;
    qkv.W[0] = w->Wq; qkv.W[1] = w->Wk; qkv.W[2] = w->Wv; qkv.R[0] = QD; qkv.R[1] = KV; qkv.R[2] = KV;
    qkv.y[0] = q32; qkv.y[1] = k32; qkv.y[2] = v32;
    GemvArgs o{}; o.mode = GEMV_RESID; o.x = att; o.K = QD; o.W[0] = w->Wo; o.R[0] = m.D; o.y[0] = x;
    GemvArgs gu{}; gu.mode = GEMV_SILU; gu.x = xn; gu.K = m.D; gu.W[0] = w->Wgate; gu.W[1] = w->Wup; gu.R[0] = m.Dff; gu.y[0] = hbuf;
    GemvArgs dn{}; dn.mode = GEMV_RESID; dn.x = hbuf; dn.K = m.Dff; dn.W[0] = w->Wdown; dn.R[0] = m.D; dn.y[0] = x;
    if (!gemv_supported(qkv, c->bf16) || !gemv_supported(o, c->bf16) || !gemv_supported(dn, c->bf16)) return SPTS_ESHAPE;
    {
        GemvArgs chk = gu; chk.R[1] = m.Dff;
        if (!gemv_supported(chk, c->bf16)) return SPTS_ESHAPE;
    }
    if (!decode_attn_supported(m.H, m.Hkv, m.d, c->bf16)) return SPTS_ESHAPE;
    if (part_floats / (size_t)batch < decode_attn_min_scratch_floats(m.Hkv, m.d)) return SPTS_EWORKSPACE;
    hipStream_t st = c->stream;
    c->dec_rope_pos = -1;
    { PHASE(c, PH_DEC_NORM); SPTS_HIP(c, launch_rmsnorm(x, w->gamma1, m.rms_eps, xn, batch, m.D, c->bf16, st)); }
    { PHASE(c, PH_DEC_QKV); SPTS_HIP(c, launch_gemv_nb(qkv, batch, c->bf16, st)); }
    { PHASE(c, PH_DEC_ROPE_APPEND);
      SPTS_HIP(c, launch_decode_rope_append_batched(q32, k32, v32, q, m.H, m.Hkv, m.d, m.rope_base, db, c->bf16, st)); }
    { PHASE(c, PH_DEC_ATTN); SPTS_HIP(c, launch_decode_attn_batched(q, db, m.H, m.Hkv, m.d, part, part_floats, att, c->bf16, st)); }
    { PHASE(c, PH_DEC_O); SPTS_HIP(c, launch_gemv_nb(o, batch, c->bf16, st)); }
    { PHASE(c, PH_DEC_NORM); SPTS_HIP(c, launch_rmsnorm(x, w->gamma2, m.rms_eps, xn, batch, m.D, c->bf16, st)); }
    { PHASE(c, PH_DEC_GATE_UP); SPTS_HIP(c, launch_gemv_nb(gu, batch, c->bf16, st)); }
    { PHASE(c, PH_DEC_DOWN); SPTS_HIP(c, launch_gemv_nb(dn, batch, c->bf16, st)); }
    for (int b = 0; b < batch; ++b) caches[b].count += 1;
    return SPTS_OK;
}

int spts_greedy_token_batched(spts_ctx* c, const void* x, const void* gamma_f, const void* table, int32_t V, int32_t batch,
                              int32_t* token_out, float* logits_out, void* x_next) {
    if (!c || batch < 0 || batch > SPTS_MAX_DECODE_BATCH) return SPTS_EINVAL;
    if (batch == 0) return SPTS_OK;
    if (!x || !gamma_f || !table || !token_out || V <= 0) return SPTS_EINVAL;
    if (!aligned16(x) || !aligned16(gamma_f) || !aligned16(table) || (logits_out && !aligned16(logits_out)) ||
        (x_next && !aligned16(x_next)))
        return SPTS_EALIGN;
    const auto& m = c->m;
    if (batch > c->lim.max_tokens) return SPTS_EWORKSPACE;
    float* logits = logits_out;
    if (!logits) {
        if ((size_t)V * batch * sizeof(float) > c->off.misc - c->off.big) return SPTS_EWORKSPACE;
        logits = c->p<float>(c->off.big);
    }
    void* xn = c->p<void>(c->off.xn);
    GemvArgs g{}; g.mode = GEMV_F32; g.x = xn; g.K = m.D; g.W[0] = table; g.R[0] = V; g.y[0] = logits;
    if (!gemv_supported(g, c->bf16)) return SPTS_ESHAPE;
    const size_t eb = c->bf16 ? 2 : 4;
    PHASE(c, PH_DEC_HEAD);
    SPTS_HIP(c, launch_rmsnorm(x, gamma_f, m.rms_eps, xn, batch, m.D, c->bf16, c->stream));
    SPTS_HIP(c, launch_gemv_nb(g, batch, c->bf16, c->stream));
    for (int b = 0; b < batch; ++b)
        SPTS_HIP(c, launch_argmax_row(logits + (size_t)b * V, V, token_out + b, table, m.D,
                                      x_next ? (char*)x_next + (size_t)b * m.D * eb : nullptr, c->bf16, c->stream));
    return SPTS_OK;
}

int spts_pack_slab32(spts_ctx* c, const void* W, int64_t rows, int64_t K, void* out) {
    if (!c || !W || !out || rows <= 0 || K <= 0) return SPTS_EINVAL;
    if (!aligned16(W) || !aligned16(out)) return SPTS_EALIGN;
    if (K % 32 != 0) return SPTS_ESHAPE;
    SPTS_HIP(c, launch_pack_slab32(W, rows, K, out, c->stream));
    return SPTS_OK;
}

int spts_select_topk_segmented(spts_ctx* c, const float* scores, const int64_t* seg_offsets, const int64_t* seg_k,
                               const int64_t* out_offsets, int32_t batch, int64_t max_len, int32_t protect_last,
                               int32_t* idx_out) {
    SPTS_TRY(common_call_checks(c, max_len));
    if (batch < 0 || batch > 65535) return SPTS_EINVAL;
    if (batch == 0 || max_len == 0) return SPTS_OK;
    if (!scores || !seg_offsets || !seg_k || !out_offsets || !idx_out) return SPTS_EINVAL;
    if (!aligned16(scores) || !aligned16(idx_out) || (reinterpret_cast<uintptr_t>(seg_offsets) & 7u) ||
        (reinterpret_cast<uintptr_t>(seg_k) & 7u) || (reinterpret_cast<uintptr_t>(out_offsets) & 7u))
        return SPTS_EALIGN;
    PHASE(c, PH_TOPK);
    SPTS_HIP(c, launch_topk(scores, max_len, 0, protect_last, idx_out, batch, c->stream,
                            TopkSegments{seg_offsets, seg_k, out_offsets}));
    return SPTS_OK;
}

int spts_channel_importance(spts_ctx* c, const void* x_cal, int64_t T, const spts_layer_weights* w, int64_t k,
                            float* importance_out) {
    SPTS_TRY(common_call_checks(c, T));
    if (!x_cal || !w || !w->Wgate || !w->Wup || !importance_out) return SPTS_EINVAL;
    if (T < 1 || k < 1 || k > T) return SPTS_EINVAL;
    if (!aligned16(x_cal) || !aligned16(w->Wgate) || !aligned16(w->Wup) || !aligned16(importance_out)) return SPTS_EALIGN;
    const auto& m = c->m;
    void* zt = c->p<void>(c->off.big);   // Z^T [Dff, T]: channel-major, so that a channel's saliencies are one row
    GemmArgs g = gemm_args(w->Wgate, m.D, nullptr, x_cal, m.D, zt, T, m.Dff, (int32_t)T, m.D, EPI_SILU_MUL);
    g.A1 = w->Wup; g.B1 = x_cal;
    { PHASE(c, PH_BUILD_SALIENCY); SPTS_TRY(run_gemm(c, g)); }
    PHASE(c, PH_BUILD_TOPMEAN);
    SPTS_HIP(c, launch_topk_mean(zt, T, m.Dff, T, k, importance_out, c->bf16, c->stream));
    return SPTS_OK;
}

int spts_msdp_compact(spts_ctx* c, const void* x_in, const int32_t* pos_in, const float* s_mha, int64_t N, int64_t N_next,
                      int32_t protect_last, void* x_out, int32_t* pos_out, int32_t* map_new2old, int32_t* map_old2new) {
    SPTS_TRY(common_call_checks(c, N));
    if (N_next < 0) return SPTS_EINVAL;
    const int64_t keep = N_next < N ? N_next : N;
    if (N == 0) return SPTS_OK;
    if (map_old2new) {
        if (!aligned16(map_old2new)) return SPTS_EALIGN;
    }
    if (keep > 0) {
        if (!x_in || !pos_in || !s_mha || !x_out || !pos_out || !map_new2old) return SPTS_EINVAL;
        if (!aligned16(x_in) || !aligned16(pos_in) || !aligned16(s_mha) || !aligned16(x_out) || !aligned16(pos_out) ||
            !aligned16(map_new2old))
            return SPTS_EALIGN;
        const size_t row_bytes = (size_t)c->m.D * (c->bf16 ? 2 : 4);
        const char* a = (const char*)x_in; const char* b = (const char*)x_out;
        if (a < b + (size_t)keep * row_bytes && b < a + (size_t)N * row_bytes) return SPTS_EINVAL;  // overlap
    }
    PHASE(c, PH_COMPACT);
    if (map_old2new) SPTS_HIP(c, launch_fill_i32(map_old2new, -1, N, c->stream));
    if (keep == 0) return SPTS_OK;
    SPTS_TRY(run_topk(c, s_mha, N, keep, protect_last, map_new2old));
    const int64_t row_bytes = (int64_t)c->m.D * (c->bf16 ? 2 : 4);
    return gather_rows_maps(c, x_in, map_new2old, x_out, keep, row_bytes, pos_in, pos_out, map_old2new);
}

int spts_msdp_compact_batched(spts_ctx* c, const void* x_in, const int32_t* pos_in, const float* s_mha,
                              const int64_t* seq_offsets, int32_t batch, const int64_t* n_next, int32_t protect_last,
                              void* x_out, int32_t* pos_out, int32_t* map_new2old, int32_t* map_old2new) {
    if (!c || batch < 0 || batch > SPTS_MAX_BATCH) return SPTS_EINVAL;
    if (batch == 0) return SPTS_OK;
    if (!seq_offsets || !n_next || seq_offsets[0] != 0) return SPTS_EINVAL;
    const int64_t N = seq_offsets[batch];
    SPTS_TRY(common_call_checks(c, N));
    std::vector<int64_t> desc(3 * (size_t)(batch + 1));
    int64_t* dOff = desc.data(); int64_t* dK = dOff + (batch + 1); int64_t* dOut = dK + (batch + 1);
    int64_t max_len = 0;
    dOut[0] = 0;
    for (int b = 0; b < batch; ++b) {
        const int64_t nb = seq_offsets[b + 1] - seq_offsets[b];
        if (nb < 0 || n_next[b] < 0) return SPTS_EINVAL;
        dOff[b] = seq_offsets[b];
        dK[b] = n_next[b] < nb ? n_next[b] : nb;
        dOut[b + 1] = dOut[b] + dK[b];
        max_len = std::max(max_len, nb);
    }
    dOff[batch] = N; dK[batch] = 0;
    const int64_t keep = dOut[batch];
    if (N == 0) return SPTS_OK;
    if (map_old2new && !aligned16(map_old2new)) return SPTS_EALIGN;
    if (keep > 0) {
        if (!x_in || !pos_in || !s_mha || !x_out || !pos_out || !map_new2old) return SPTS_EINVAL;
        if (!aligned16(x_in) || !aligned16(pos_in) || !aligned16(s_mha) || !aligned16(x_out) || !aligned16(pos_out) ||
            !aligned16(map_new2old))
            return SPTS_EALIGN;
        const size_t row_bytes = (size_t)c->m.D * (c->bf16 ? 2 : 4);
        const char* a = (const char*)x_in; const char* b = (const char*)x_out;
        if (a < b + (size_t)keep * row_bytes && b < a + (size_t)N * row_bytes) return SPTS_EINVAL;  // overlap
    }
    PHASE(c, PH_COMPACT);
    if (map_old2new) SPTS_HIP(c, launch_fill_i32(map_old2new, -1, N, c->stream));
    if (keep == 0) return SPTS_OK;
    // the descriptors travel by value as kernel arguments: no staging copy of a host array that dies with this call
    int64_t* seg = c->p<int64_t>(c->off.seg);
    SPTS_HIP(c, launch_write_i64(desc.data(), (int64_t)desc.size(), seg, c->stream));
    const TopkSegments segs{seg, seg + (batch + 1), seg + 2 * (batch + 1)};
    SPTS_HIP(c, launch_topk(s_mha, max_len, 0, protect_last, map_new2old, batch, c->stream, segs));
    SPTS_HIP(c, launch_add_segment_base(map_new2old, segs.out_offsets, segs.offsets, batch, keep, c->stream));
    const int64_t row_bytes = (int64_t)c->m.D * (c->bf16 ? 2 : 4);
    return gather_rows_maps(c, x_in, map_new2old, x_out, keep, row_bytes, pos_in, pos_out, map_old2new);
}

int spts_layer_prefill(spts_ctx* c, void* x, const int32_t* pos, int64_t N, const spts_layer_weights* w,
                       const spts_layer_cfg* cfg, spts_kv_out* kv, float* s_mha, int32_t* idx_attn, int32_t* idx_ffn) {
    SPTS_TRY(common_call_checks(c, N));
    if (!cfg) return SPTS_EINVAL;
    if (cfg->m_attn < 0 || cfg->m_ffn < 0) return SPTS_EINVAL;
    if (kv) kv->count = 0;
    if (N == 0) return SPTS_OK;
    if (!x || !pos) return SPTS_EINVAL;
    if (!aligned16(x) || !aligned16(pos)) return SPTS_EALIGN;
    const bool skip = cfg->skip != 0;
    SPTS_TRY(check_weights_full(c, w, skip));
    if (skip) {
        if (cfg->probe_len < 1 || cfg->probe_len > N) return SPTS_EINVAL;
        if (cfg->probe_len > c->lim.max_probe) return SPTS_EWORKSPACE;
        if ((s_mha && !aligned16(s_mha)) || (idx_attn && !aligned16(idx_attn)) || (idx_ffn && !aligned16(idx_ffn)))
            return SPTS_EALIGN;
    }
    const auto& m = c->m;
    const int64_t Ma = skip ? (cfg->m_attn < N ? cfg->m_attn : N) : N;
    const int64_t Mf = skip ? (cfg->m_ffn < N ? cfg->m_ffn : N) : N;
    const bool full_kv = !skip || cfg->kv_mode == 1;
    const int64_t Mk = full_kv ? N : Ma;
    if (kv) {
        if (Ma > 0) {
            if (!kv->k || !kv->v || !kv->pos) return SPTS_EINVAL;
            if (!aligned16(kv->k) || !aligned16(kv->v) || !aligned16(kv->pos)) return SPTS_EALIGN;
            if (kv->capacity < Mk) return SPTS_EINVAL;
        }
    }
    const int KV = m.Hkv * m.d, QD = m.H * m.d;
    const size_t eb = c->bf16 ? 2 : 4;
    hipStream_t st = c->stream;
    void* xn = c->p<void>(c->off.xn);

    // ------------------------------------------------ attention block (Alg. 1, PAP block / dense branch)
    float* S = s_mha ? s_mha : c->p<float>(c->off.S);
    int32_t* idxA = nullptr;
    void* kall = (kv && full_kv && Ma > 0) ? kv->k : c->p<void>(c->off.kall);
    SPTS_TRY(probe_attn_impl(c, x, pos, N, w, skip ? cfg->probe_len : 0, skip, kall, S));
    if (skip) {
        idxA = idx_attn ? idx_attn : c->p<int32_t>(c->off.idxA);
        PHASE(c, PH_TOPK);
        SPTS_TRY(run_topk(c, S, N, Ma, cfg->protect_last, idxA));
    }
    if (Ma > 0) {
        const int32_t* qpos = pos;
        const int32_t* kpos = pos;
        void* kk = kall;
        void* vv;
        if (skip) {
            // K-hat = K[T_a] and the active positions, straight into the cache when there is one: one launch
            int32_t* posA = (kv && !full_kv) ? kv->pos : c->p<int32_t>(c->off.posA);
            PHASE(c, PH_GATHER);
            if (!full_kv) {
                kk = kv ? kv->k : c->p<void>(c->off.khat);
                SPTS_TRY(gather_rows_maps(c, kall, idxA, kk, Ma, (int64_t)KV * eb, pos, posA, nullptr));
                kpos = posA;
            } else {
                SPTS_HIP(c, launch_gather_i32(pos, idxA, posA, Ma, st));
            }
            qpos = posA;
        }
        if (full_kv && kv) SPTS_HIP(c, launch_copy_bytes(pos, kv->pos, N * 4, st));
        vv = kv ? kv->v : c->p<void>(c->off.vhat);
        AttnArgs aa{};
        aa.q = c->p<void>(c->off.q); aa.k = kk; aa.v = vv; aa.qpos = qpos; aa.kpos = kpos; aa.out = c->p<void>(c->off.att);
        aa.Mq = Ma; aa.Mk = Mk; aa.H = m.H; aa.Hkv = m.Hkv; aa.d = m.d;
        aa.ldvt = (Mk + 255) / 256 * 256; aa.vt = c->p<void>(c->off.vt);
        const bool amf = c->bf16 && attention_mfma_supported(aa);
        // queries of the active rows (rows gathered through idxA inside the GEMM's A loads), stored with the factor of
        // query_store_scale()
        aa.q_scale = query_store_scale(c);
        GemmArgs gq = gemm_args(xn, m.D, idxA, w->Wq, m.D, nullptr, QD, Ma, QD, m.D);
        gq.a_rows = N;
        GemmArgs gv = gemm_args(xn, m.D, full_kv ? nullptr : idxA, w->Wv, m.D, vv, KV, Mk, KV, m.D);
        gv.a_rows = N;
        // Queries and values of the same rows (active queries against their own keys, or the dense branch) leave one
        // launch when the matrix-core kernels take everything: columns [0, H*d) rotary queries, [H*d, H*d + Hkv*d)
        // values with their transposed copy.  One grid of (H + Hkv) * d / 256 column tiles instead of two, one tail.
        bool merged = false;
        if (amf && Mk == Ma && gv.a_idx == gq.a_idx) {
            GemmArgs f = gq;
            f.epi = EPI_ROPE_STORE; f.N = QD + KV; f.n_split = QD; f.B1 = w->Wv;
            f.C = c->p<void>(c->off.q); f.ldc = QD; f.C2 = vv; f.ldc2 = KV;
            f.rope = c->p<float2>(c->off.rope); f.rope_idx = idxA; f.head_dim = m.d; f.rope_scale = aa.q_scale;
            f.Ct = c->p<void>(c->off.vt); f.ldct = aa.ldvt;
            prefer_slab(c, f, w->Wq_s, w->Wv_s, QD, KV);
            if (gemm_mfma_supported(f)) {
                PHASE(c, PH_QV_PROJ);
                SPTS_TRY(run_gemm_mfma(c, f));
                merged = true;
            }
        }
        if (!merged) {
            { PHASE(c, PH_Q_PROJ); SPTS_TRY(run_gemm_rope(c, gq, m.H, idxA, 0, c->p<void>(c->off.q), w->Wq_s, aa.q_scale)); }
            prefer_slab(c, gv, w->Wv_s, nullptr, KV);
            bool vt_done = false;
            if (amf) {
                // the matrix-core projection writes the transposed copy (keys contiguous) in its epilogue
                GemmArgs gvt = gv; gvt.Ct = c->p<void>(c->off.vt); gvt.ldct = aa.ldvt;
                if (gemm_mfma_supported(gvt)) { gv = gvt; vt_done = true; }
            }
            PHASE(c, PH_V_PROJ);
            SPTS_TRY(run_gemm(c, gv));
            if (amf && !vt_done) SPTS_HIP(c, launch_transpose_pad(vv, c->p<void>(c->off.vt), Mk, KV, aa.ldvt, c->bf16, st));
        }
        if (kv) kv->count = Mk;
        // x[T_a] += att * Wo^T; the attention output (a buffer of the library's own) goes slab-major when the matrix-core
        // attention writes it and the matrix-core GEMM reads it
        GemmArgs go = gemm_args(c->p<void>(c->off.att), QD, nullptr, w->Wo, QD, x, m.D, Ma, m.D, QD, EPI_RESIDUAL);
        go.c_idx = idxA;
        prefer_slab(c, go, w->Wo_s, nullptr, m.D);
        if (amf) {
            GemmArgs t = go; t.a_slab = 1;
            if (gemm_mfma_supported(t)) { go = t; aa.out_slab = 1; }
        }
        {
            PHASE(c, PH_ATTENTION);
            if (amf) SPTS_HIP(c, launch_attention_mfma(aa, st));
            else SPTS_HIP(c, launch_attention_generic(aa, c->bf16, st));
        }
        { PHASE(c, PH_O_PROJ); SPTS_TRY(run_gemm(c, go)); }
    }

    // ------------------------------------------------ FFN block (Alg. 1, LTP block / dense branch)
    if (Mf == 0) return SPTS_OK;
    { PHASE(c, PH_RMSNORM); SPTS_HIP(c, launch_rmsnorm(x, w->gamma2, m.rms_eps, xn, N, m.D, c->bf16, st)); }
    int32_t* idxF = nullptr;
    if (skip && Mf >= N) {
        // the budget covers every candidate: TopK of all N is the whole set whatever the scores are, so the
        // proxy is not run and the FFN takes the rows in place
        if (idx_ffn) SPTS_HIP(c, launch_iota_i32(idx_ffn, N, st));
    } else if (skip) {
        float* SF = c->p<float>(c->off.SF);
        SPTS_TRY(proxy_scores_impl(c, xn, N, w, S, nullptr, SF));
        idxF = idx_ffn ? idx_ffn : c->p<int32_t>(c->off.idxF);
        PHASE(c, PH_TOPK);
        SPTS_TRY(run_topk(c, SF, N, Mf, cfg->protect_last, idxF));
    }
    GemmArgs gh = gemm_args(xn, m.D, idxF, w->Wgate, m.D, c->p<void>(c->off.big), m.Dff, Mf, m.Dff, m.D, EPI_SILU_MUL);
    gh.a_rows = N;
    gh.B1 = w->Wup;
    prefer_slab(c, gh, w->Wgate_s, w->Wup_s, m.Dff);
    GemmArgs gd = gemm_args(c->p<void>(c->off.big), m.Dff, nullptr, w->Wdown, m.Dff, x, m.D, Mf, m.D, m.Dff, EPI_RESIDUAL);
    gd.c_idx = idxF;
    prefer_slab(c, gd, w->Wdown_s, nullptr, m.D);
    hidden_slab(c, gh, gd);
    { PHASE(c, PH_FFN_GATE_UP); SPTS_TRY(run_gemm(c, gh)); }
    { PHASE(c, PH_FFN_DOWN); SPTS_TRY(run_gemm(c, gd)); }
    return SPTS_OK;
}

int spts_layer_prefill_batched(spts_ctx* c, void* x, const int32_t* pos, const int64_t* seq_offsets, int32_t batch,
                               const spts_layer_weights* w, int32_t skip, int32_t probe_len, const int64_t* m_attn, const int64_t* m_ffn,
                               int32_t protect_last, spts_kv_out* kv, float* s_mha, int32_t* idx_attn, int32_t* idx_ffn) {
    if (!c || batch < 0 || batch > SPTS_MAX_BATCH) return SPTS_EINVAL;
    if (batch == 0) return SPTS_OK;
    if (!seq_offsets || seq_offsets[0] != 0) return SPTS_EINVAL;
    if (skip && (!m_attn || !m_ffn)) return SPTS_EINVAL;
    const int64_t N = seq_offsets[batch];
    SPTS_TRY(common_call_checks(c, N));
    if (!x || !pos) return SPTS_EINVAL;
    if (!aligned16(x) || !aligned16(pos)) return SPTS_EALIGN;
    if ((s_mha && !aligned16(s_mha)) || (idx_attn && !aligned16(idx_attn)) || (idx_ffn && !aligned16(idx_ffn))) return SPTS_EALIGN;
    SPTS_TRY(check_weights_full(c, w, skip != 0));
    if (skip) {
        if (probe_len < 1) return SPTS_EINVAL;
        if (probe_len > c->lim.max_probe) return SPTS_EWORKSPACE;
    }
    const auto& m = c->m;
    const int KV = m.Hkv * m.d, QD = m.H * m.d;
    const size_t eb = c->bf16 ? 2 : 4;
    // host-side plan: per sequence its length, budgets and the start of its slice in the index lists
    std::vector<int64_t> desc(3 * (size_t)(batch + 1));
    int64_t* dOff = desc.data();                 // [batch+1] first row of each sequence
    int64_t* dKa = dOff + (batch + 1);            // [batch]   attention budgets (then reused for the FFN)
    int64_t* dOut = dKa + (batch + 1);            // [batch+1] first entry of each sequence in the index list
    std::vector<int64_t> ma(batch), mf(batch), oa(batch + 1), of(batch + 1);
    oa[0] = of[0] = 0;
    for (int b = 0; b < batch; ++b) {
        const int64_t nb = seq_offsets[b + 1] - seq_offsets[b];
        if (nb < 0) return SPTS_EINVAL;
        if (skip && (nb < probe_len || m_attn[b] < 0 || m_ffn[b] < 0)) return SPTS_EINVAL;   // every sequence holds its probe rows
        ma[b] = skip && m_attn[b] < nb ? m_attn[b] : nb;   // dense layer: every row is active
        mf[b] = skip && m_ffn[b] < nb ? m_ffn[b] : nb;
        oa[b + 1] = oa[b] + ma[b];
        of[b + 1] = of[b] + mf[b];
        if (kv) {
            kv[b].count = 0;
            if (ma[b] > 0) {
                if (!kv[b].k || !kv[b].v || !kv[b].pos) return SPTS_EINVAL;
                if (!aligned16(kv[b].k) || !aligned16(kv[b].v) || !aligned16(kv[b].pos)) return SPTS_EALIGN;
                if (kv[b].capacity < ma[b]) return SPTS_EINVAL;
            }
        }
    }
    const int64_t MaT = oa[batch], MfT = of[batch];
    hipStream_t st = c->stream;
    void* xn = c->p<void>(c->off.xn);
    int64_t* seg = c->p<int64_t>(c->off.seg);
    auto upload = [&](const std::vector<int64_t>& k, const std::vector<int64_t>& out) -> hipError_t {
        for (int b = 0; b <= batch; ++b) { dOff[b] = seq_offsets[b]; dOut[b] = out[b]; if (b < batch) dKa[b] = k[b]; }
        dKa[batch] = 0;
        // the descriptors of the previous selection may still be read by work in flight: the small kernels that write the
        // new ones (values passed by value as kernel arguments) are stream-ordered behind it
        return launch_write_i64(desc.data(), (int64_t)desc.size(), seg, st);
    };
    const TopkSegments segs{seg, seg + (batch + 1), seg + 2 * (batch + 1)};
    int64_t max_len = 0;
    for (int b = 0; b < batch; ++b) max_len = std::max<int64_t>(max_len, seq_offsets[b + 1] - seq_offsets[b]);

    // ------------------------------------------------ attention block: PAP per sequence, projections over the batch
    float* S = s_mha ? s_mha : c->p<float>(c->off.S);
    void* kall = c->p<void>(c->off.kall);
    SPTS_TRY(probe_attn_impl(c, x, pos, N, w, 0, false, kall, nullptr));
    for (int b = 0; skip && b < batch; ++b) {
        const int64_t r0 = seq_offsets[b], nb = seq_offsets[b + 1] - r0;
        SPTS_TRY(probe_scores_rows(c, r0, nb, w, probe_len, (const char*)kall + (size_t)r0 * KV * eb, S + r0));
    }
    // dense layer (the else-branches of Alg. 1): no selection, the "active rows" are the rows themselves
    int32_t* idxA = !skip ? nullptr : idx_attn ? idx_attn : c->p<int32_t>(c->off.idxA);
    if (skip) {
        PHASE(c, PH_TOPK);
        SPTS_HIP(c, upload(ma, oa));
        SPTS_HIP(c, launch_topk(S, max_len, 0, protect_last, idxA, batch, st, segs));
        SPTS_HIP(c, launch_add_segment_base(idxA, segs.out_offsets, segs.offsets, batch, MaT, st));
    }
    if (MaT > 0) {
        const int32_t* posA = pos;
        const char* khat = (const char*)kall;
        char* vhat = c->p<char>(c->off.vhat);
        if (skip) {
            PHASE(c, PH_GATHER);
            SPTS_TRY(gather_rows_maps(c, kall, idxA, c->p<void>(c->off.khat), MaT, (int64_t)KV * eb, pos, c->p<int32_t>(c->off.posA), nullptr));
            posA = c->p<int32_t>(c->off.posA);
            khat = c->p<char>(c->off.khat);
        }
        auto attn_args = [&](int b) {
            AttnArgs aa{};
            aa.q = c->p<char>(c->off.q) + (size_t)oa[b] * QD * eb;
            aa.k = khat + (size_t)oa[b] * KV * eb; aa.v = vhat + (size_t)oa[b] * KV * eb;
            aa.qpos = posA + oa[b]; aa.kpos = posA + oa[b];
            aa.out = c->p<char>(c->off.att) + (size_t)oa[b] * QD * eb;
            aa.Mq = ma[b]; aa.Mk = ma[b]; aa.H = m.H; aa.Hkv = m.Hkv; aa.d = m.d;
            aa.ldvt = (ma[b] + 255) / 256 * 256; aa.vt = c->p<void>(c->off.vt);
            return aa;
        };
        const float q_scale = query_store_scale(c);
        GemmArgs gq = gemm_args(xn, m.D, idxA, w->Wq, m.D, nullptr, QD, MaT, QD, m.D);
        gq.a_rows = N;
        { PHASE(c, PH_Q_PROJ); SPTS_TRY(run_gemm_rope(c, gq, m.H, idxA, 0, c->p<void>(c->off.q), w->Wq_s, q_scale)); }
        GemmArgs gv = gemm_args(xn, m.D, idxA, w->Wv, m.D, vhat, KV, MaT, KV, m.D);
        gv.a_rows = N;
        prefer_slab(c, gv, w->Wv_s, nullptr, KV);
        { PHASE(c, PH_V_PROJ); SPTS_TRY(run_gemm(c, gv)); }
        for (int b = 0; b < batch; ++b) {
            if (ma[b] == 0) continue;
            AttnArgs aa = attn_args(b);
            aa.q_scale = q_scale;
            const bool amf = c->bf16 && attention_mfma_supported(aa);
            PHASE(c, PH_ATTENTION);
            if (amf) {
                SPTS_HIP(c, launch_transpose_pad(aa.v, c->p<void>(c->off.vt), ma[b], KV, aa.ldvt, c->bf16, st));
                SPTS_HIP(c, launch_attention_mfma(aa, st));
            } else {
                SPTS_HIP(c, launch_attention_generic(aa, c->bf16, st));
            }
            if (kv) {
                SPTS_HIP(c, launch_copy_bytes(aa.k, kv[b].k, ma[b] * (int64_t)KV * eb, st));
                SPTS_HIP(c, launch_copy_bytes(aa.v, kv[b].v, ma[b] * (int64_t)KV * eb, st));
                SPTS_HIP(c, launch_copy_bytes(posA + oa[b], kv[b].pos, ma[b] * 4, st));
                kv[b].count = ma[b];
            }
        }
        GemmArgs go = gemm_args(c->p<void>(c->off.att), QD, nullptr, w->Wo, QD, x, m.D, MaT, m.D, QD, EPI_RESIDUAL);
        go.c_idx = idxA;
        prefer_slab(c, go, w->Wo_s, nullptr, m.D);
        { PHASE(c, PH_O_PROJ); SPTS_TRY(run_gemm(c, go)); }
    }

    // ------------------------------------------------ FFN block: proxy over the batch, TopK per sequence
    if (MfT == 0) return SPTS_OK;
    { PHASE(c, PH_RMSNORM); SPTS_HIP(c, launch_rmsnorm(x, w->gamma2, m.rms_eps, xn, N, m.D, c->bf16, st)); }
    float* SF = c->p<float>(c->off.SF);
    if (skip) SPTS_TRY(proxy_scores_impl(c, xn, N, w, S, nullptr, SF));
    int32_t* idxF = !skip ? nullptr : idx_ffn ? idx_ffn : c->p<int32_t>(c->off.idxF);
    if (skip) {
        PHASE(c, PH_TOPK);
        SPTS_HIP(c, upload(mf, of));
        SPTS_HIP(c, launch_topk(SF, max_len, 0, protect_last, idxF, batch, st, segs));
        SPTS_HIP(c, launch_add_segment_base(idxF, segs.out_offsets, segs.offsets, batch, MfT, st));
    }
    GemmArgs gh = gemm_args(xn, m.D, idxF, w->Wgate, m.D, c->p<void>(c->off.big), m.Dff, MfT, m.Dff, m.D, EPI_SILU_MUL);
    gh.a_rows = N;
    gh.B1 = w->Wup;
    prefer_slab(c, gh, w->Wgate_s, w->Wup_s, m.Dff);
    GemmArgs gd = gemm_args(c->p<void>(c->off.big), m.Dff, nullptr, w->Wdown, m.Dff, x, m.D, MfT, m.D, m.Dff, EPI_RESIDUAL);
    gd.c_idx = idxF;
    prefer_slab(c, gd, w->Wdown_s, nullptr, m.D);
    hidden_slab(c, gh, gd);
    { PHASE(c, PH_FFN_GATE_UP); SPTS_TRY(run_gemm(c, gh)); }
    { PHASE(c, PH_FFN_DOWN); SPTS_TRY(run_gemm(c, gd)); }
    return SPTS_OK;
}

}  // extern "C"
