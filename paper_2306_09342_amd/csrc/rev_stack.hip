// Host side of librevstack: argument checks, workspace layout, the per-block
// recompute (R_i) and gradient (V_i) kernel sequences, and the two schedules
// of the paper's Sec. 3.2 (Reprop: one stream) and Sec. 3.3 (PaReprop: the
// recomputation chain on a second stream, ordered against the gradient chain
// by events and a double-buffered activation slot).
#include "common.h"

#include <mutex>
#include <vector>

namespace rev {

// ---------------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------------
static thread_local std::string g_err;
void set_error(const std::string& msg) { g_err = msg; }
int hip_fail(hipError_t e, const char* what, const char* file, int line) {
    g_err = std::string(hipGetErrorString(e)) + " in " + what + " (" + file + ":" + std::to_string(line) + ")";
    return REV_EHIP;
}

// ---------------------------------------------------------------------------------
// per-family timing
// ---------------------------------------------------------------------------------
struct ProfRec { Kind kind; hipEvent_t e0, e1; };
static bool g_prof_on = false;
static std::vector<ProfRec> g_prof_recs;
static double g_prof_ms[K_COUNT];
static int64_t g_prof_n[K_COUNT];
static double g_prof_work[K_COUNT];
static const char* g_kind_names[K_COUNT] = {"gemm_nt", "gemm_wgrad", "attn_fwd", "attn_bwd", "ln_fwd",
                                            "ln_bwd", "colsum", "reduce", "convert", "optimizer"};
static const int g_kind_flops[K_COUNT] = {1, 1, 1, 1, 0, 0, 0, 0, 0, 0};

bool profiling() { return g_prof_on; }

ProfScope::ProfScope(Kind k, hipStream_t s, double work) : kind(k), stream(s), rec(nullptr) {
    if (!g_prof_on) return;
    ProfRec r;
    r.kind = k;
    if (hipEventCreate(&r.e0) != hipSuccess) return;
    if (hipEventCreate(&r.e1) != hipSuccess) { (void)hipEventDestroy(r.e0); return; }
    (void)hipEventRecord(r.e0, s);
    g_prof_recs.push_back(r);
    g_prof_work[k] += work;
    rec = (void*)(uintptr_t)g_prof_recs.size();   // index + 1
}
ProfScope::~ProfScope() {
    if (rec) (void)hipEventRecord(g_prof_recs[(uintptr_t)rec - 1].e1, stream);
}

// ---------------------------------------------------------------------------------
// configuration and packed-parameter layout
// ---------------------------------------------------------------------------------
enum { T_LN1G = 0, T_LN1B, T_WQKV, T_BQKV, T_WPROJ, T_BPROJ, T_LN2G, T_LN2B, T_WFC1, T_BFC1, T_WFC2, T_BFC2, T_COUNT };

static int64_t tensor_count(const rev_cfg& c, int t) {
    const int64_t D = c.d_model, Dm = c.d_mlp;
    switch (t) {
        case T_WQKV: return 3 * D * D;
        case T_BQKV: return 3 * D;
        case T_WPROJ: return D * D;
        case T_WFC1: case T_WFC2: return D * Dm;
        case T_BFC1: return Dm;
        default: return D;
    }
}
static int64_t tensor_offset(const rev_cfg& c, int t) {
    int64_t off = 0;
    for (int i = 0; i < t; ++i) off += tensor_count(c, i);
    return off;
}
static int64_t block_params(const rev_cfg& c) { return tensor_offset(c, T_COUNT); }

static int check_cfg(const rev_cfg* c) {
    if (!c) { set_error("cfg is null"); return REV_EINVAL; }
    if (c->n_blocks <= 0 || c->d_model <= 0 || c->n_heads <= 0 || c->d_mlp <= 0 || c->seq_len <= 0 || c->batch <= 0) {
        set_error("cfg: every size must be positive"); return REV_EINVAL;
    }
    if (c->mode != REV_MODE_FP32 && c->mode != REV_MODE_BF16) { set_error("cfg: unknown mode"); return REV_EINVAL; }
    if (c->d_model % c->n_heads != 0) { set_error("cfg: d_model must be divisible by n_heads"); return REV_EINVAL; }
    const int dh = c->d_model / c->n_heads;
    if (c->d_model % 8 != 0 || c->d_mlp % 8 != 0 || dh % 8 != 0) {
        set_error("cfg: d_model, d_mlp and head_dim must be multiples of 8"); return REV_EINVAL;
    }
    if (dh > 128) { set_error("cfg: head_dim must be <= 128"); return REV_EINVAL; }
    if (c->d_model > 8192 || c->d_mlp > 32768) { set_error("cfg: d_model <= 8192 and d_mlp <= 32768"); return REV_EINVAL; }
    // launch-grid limits: the attention kernels put (sample, head) pairs on the grid's y axis and the plain-ALU
    // GEMM 64-row strips of tokens; y holds at most 65535
    if ((int64_t)c->batch * c->seq_len > (int64_t)65535 * 64) {
        set_error("cfg: batch*seq_len must be <= 4194240"); return REV_EINVAL;
    }
    if ((int64_t)c->batch * c->n_heads > 65535) { set_error("cfg: batch*n_heads must be <= 65535"); return REV_EINVAL; }
    if (!(c->ln_eps >= 0.f)) { set_error("cfg: ln_eps must be >= 0"); return REV_EINVAL; }
    return REV_OK;
}

// ---------------------------------------------------------------------------------
// workspace layout (byte offsets, every region 256-byte aligned)
// ---------------------------------------------------------------------------------

struct Layout {
    int64_t slot[2];
    int64_t s_n2, s_h, s_a, s_n1, s_qkv, s_o, s_lse, s_st1, s_st2;   // relative to a slot
    int64_t ring[3][2];
    int64_t cot[2][2];     // float32 cotangent levels
    int64_t cot2b[2];      // act-typed copy of the stream-2 cotangent (bf16 mode)
    int64_t gy1b[2];       // act-typed copy of gY1 (bf16 mode), by block parity
    int64_t dh[2], dqkv[2]; // by block parity: read by the weight-gradient kernels of the block
    int64_t dn, dO, delta;
    int64_t part_ln[2], part_col[2], part_wg[4];   // one per deferred reduction of a block
    int64_t total;
    int64_t part_wg_elems[4];
    int64_t slot_bytes;
    int ring_levels;
};

// compact = the layout of the sequential schedule (and of the forward map): nothing of block i-1
// is produced while block i is still being consumed, so one activation slot, two residual levels and
// one copy of each per-block gradient temporary are enough.  The full layout doubles those, which is
// the extra memory the parallel schedule pays (Sec. 3.3, Sec. 4.2).
static Layout make_layout(const rev_cfg& c, bool compact) {
    Layout L = {};
    const int64_t M = (int64_t)c.batch * c.seq_len, D = c.d_model, Dm = c.d_mlp;
    const int64_t es = (c.mode == REV_MODE_BF16) ? 2 : 4;
    int64_t off = 0;
    auto take = [&](int64_t bytes) { int64_t o = off; off += (bytes + 255) / 256 * 256; return o; };
    // one activation slot
    {
        int64_t base = off;
        L.s_n2 = take(M * D * es) - base;
        L.s_h = take(M * Dm * es) - base;
        L.s_a = take(M * Dm * es) - base;
        L.s_n1 = take(M * D * es) - base;
        L.s_qkv = take(M * 3 * D * es) - base;
        L.s_o = take(M * D * es) - base;
        L.s_lse = take((int64_t)c.batch * c.n_heads * c.seq_len * 4) - base;
        L.s_st1 = take(M * 2 * 4) - base;
        L.s_st2 = take(M * 2 * 4) - base;
        L.slot_bytes = off - base;
        L.slot[0] = base;
        L.slot[1] = compact ? base : take(L.slot_bytes);
    }
    L.ring_levels = compact ? 2 : 3;
    for (int r = 0; r < L.ring_levels; ++r)
        for (int s = 0; s < 2; ++s) L.ring[r][s] = take(M * D * 4);
    for (int r = 0; r < 2; ++r)
        for (int s = 0; s < 2; ++s) L.cot[r][s] = take(M * D * 4);
    if (c.mode == REV_MODE_BF16) {
        L.cot2b[0] = take(M * D * es);
        L.cot2b[1] = take(M * D * es);
        L.gy1b[0] = take(M * D * es);
        L.gy1b[1] = compact ? L.gy1b[0] : take(M * D * es);
    }
    for (int r = 0; r < 2; ++r) {
        L.dh[r] = (compact && r) ? L.dh[0] : take(M * Dm * es);
        L.dqkv[r] = (compact && r) ? L.dqkv[0] : take(M * 3 * D * es);
    }
    L.dn = take(M * D * es);
    L.dO = take(M * D * es);
    L.delta = take((int64_t)c.batch * c.n_heads * c.seq_len * 4);
    L.part_ln[0] = take(ln_bwd_partial_elems((int)M, (int)D) * 4);
    L.part_ln[1] = take(ln_bwd_partial_elems((int)M, (int)D) * 4);
    {
        // [0]: fc1 bias gradient (column-sum strips of the GELU' epilogue, or a plain column sum);
        // [1]: QKV bias gradient; also the top block's fc2 bias gradient
        int64_t e0 = colsum_partial_elems((int)M, (int)Dm);
        int64_t e0b = (int64_t)gemm_colsum_strips_max((int)M) * Dm;
        if (e0b > e0) e0 = e0b;
        int64_t e1 = colsum_partial_elems((int)M, (int)(3 * D));
        int64_t e1b = colsum_partial_elems((int)M, (int)D);
        if (e1b > e1) e1 = e1b;
        L.part_col[0] = take(e0 * 4);
        L.part_col[1] = take(e1 * 4);
    }
    if (c.mode == REV_MODE_BF16) {
        // scratch for the pieces of the four weight gradients (fc2, fc1, proj, qkv), which go out as one launch: none
        // where their tiles fill the device without cutting the token range
        const int nn[4] = {(int)D, (int)Dm, (int)D, (int)(3 * D)}, kk[4] = {(int)Dm, (int)D, (int)D, (int)D};
        const int S = wgrad_group_ranges((int)M, nn, kk, 4);
        for (int w = 0; w < 4; ++w) {
            L.part_wg_elems[w] = S > 1 ? (int64_t)S * nn[w] * kk[w] : 0;
            L.part_wg[w] = take((L.part_wg_elems[w] > 0 ? L.part_wg_elems[w] : 64) * 4);
        }
    }
    L.total = off;
    return L;
}

// ---------------------------------------------------------------------------------
// event pool (the only state kept between calls)
// ---------------------------------------------------------------------------------
// A two-stream call leases a set of events that no other call holds while it enqueues, so calls issued
// from several host threads (on their own workspaces and streams) never record or wait on each other's
// events.  The lease ends when the enqueue returns: a wait that is already enqueued refers to the record
// that preceded it, so a later call may record the same event again without disturbing it.
static std::mutex g_ev_mu;
static std::vector<hipEvent_t> g_ev_free;
struct EventLease {
    std::vector<hipEvent_t> ev;
    int take(int n) {
        std::lock_guard<std::mutex> lk(g_ev_mu);
        while ((int)ev.size() < n) {
            hipEvent_t e;
            if (!g_ev_free.empty()) {
                e = g_ev_free.back();
                g_ev_free.pop_back();
            } else {
                REV_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
            }
            ev.push_back(e);
        }
        return REV_OK;
    }
    ~EventLease() {
        std::lock_guard<std::mutex> lk(g_ev_mu);
        g_ev_free.insert(g_ev_free.end(), ev.begin(), ev.end());
    }
};

// ---------------------------------------------------------------------------------
// the per-block kernel sequences
// ---------------------------------------------------------------------------------
#define RC(expr) do { int _rc = (expr); if (_rc != REV_OK) return _rc; } while (0)

template <typename T> struct Ops;
template <> struct Ops<float> {
    static int nt(hipStream_t s, const float* A, int64_t lda, const float* B, int64_t ldb, int M, int N, int K, const Epi& e) {
        return gemm_nt_f32(s, A, lda, B, ldb, M, N, K, e);
    }
    static int wgrad(hipStream_t s, const float* G, int64_t ldg, const float* A, int64_t lda, int M, int N, int K,
                     float* dW, float* part, int64_t pe, RedSeg* defer) {
        return gemm_wgrad_f32(s, G, ldg, A, lda, M, N, K, dW, part, pe, defer);
    }
};
template <> struct Ops<bf16> {
    static int nt(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb, int M, int N, int K, const Epi& e) {
        return gemm_nt_bf16(s, A, lda, B, ldb, M, N, K, e);
    }
    static int wgrad(hipStream_t s, const bf16* G, int64_t ldg, const bf16* A, int64_t lda, int M, int N, int K,
                     float* dW, float* part, int64_t pe, RedSeg* defer) {
        return gemm_wgrad_bf16(s, G, ldg, A, lda, M, N, K, dW, part, pe, defer);
    }
};

template <typename T>
struct Runner {
    static constexpr bool kBf16 = sizeof(T) == 2;
    rev_cfg c;
    Layout L;
    char* ws;
    const T* params;
    float* dparams;
    int M, D, Dm, H, dh, B, Tn;
    bool solo;      // one stream: every kernel has the device to itself
    const int* key_len = nullptr;   // optional key-padding mask: valid keys per sample (device, [batch])

    Runner(const rev_cfg& cfg, const void* p, float* dp, void* w, bool compact)
        : c(cfg), L(make_layout(cfg, compact)), ws((char*)w), params((const T*)p), dparams(dp), solo(compact) {
        M = c.batch * c.seq_len; D = c.d_model; Dm = c.d_mlp; H = c.n_heads; dh = D / H; B = c.batch; Tn = c.seq_len;
    }
    Epi epi0() const { Epi e = {}; e.solo = solo; return e; }
    template <typename U> U* at(int64_t off) const { return reinterpret_cast<U*>(ws + off); }
    const T* P(int blk, int t) const { return params + (int64_t)blk * block_params(c) + tensor_offset(c, t); }
    float* G(int blk, int t) const { return dparams + (int64_t)blk * block_params(c) + tensor_offset(c, t); }
    struct Slot { T *n2, *h, *a, *n1, *qkv, *o; float *lse, *st1, *st2; };
    Slot slot(int i) const {
        int64_t b = L.slot[i & 1];
        return {at<T>(b + L.s_n2), at<T>(b + L.s_h), at<T>(b + L.s_a), at<T>(b + L.s_n1), at<T>(b + L.s_qkv),
                at<T>(b + L.s_o), at<float>(b + L.s_lse), at<float>(b + L.s_st1), at<float>(b + L.s_st2)};
    }

    // F branch pieces up to the projection input: n1, qkv, o, lse from x2
    int f_pre(hipStream_t s, int blk, const float* x2, const Slot& sl) {
        RC((ln_forward<T, T>(s, x2, P(blk, T_LN1G), P(blk, T_LN1B), c.ln_eps, sl.n1, sl.st1, M, D)));
        Epi e = epi0(); e.kind = EPI_BIAS; e.out = sl.qkv; e.bias = P(blk, T_BQKV); e.ldo = 3 * D;
        RC(Ops<T>::nt(s, sl.n1, D, P(blk, T_WQKV), D, M, 3 * D, D, e));
        RC((attention_forward<T>(s, sl.qkv, sl.o, sl.lse, B, Tn, H, dh, key_len)));
        return REV_OK;
    }
    // out1 = in1 + sign * (o Wp^T + bp)
    int f_post(hipStream_t s, int blk, const Slot& sl, const float* in1, float* out1, float sign) {
        Epi e = epi0(); e.kind = EPI_RESIDUAL; e.outf = out1; e.res = in1; e.bias = P(blk, T_BPROJ); e.sign = sign; e.ldo = D;
        return Ops<T>::nt(s, sl.o, D, P(blk, T_WPROJ), D, M, D, D, e);
    }
    // out2 = in2 + sign * G(y1); the pre-activation of the MLP is kept only where a backward step will read it
    int g_branch(hipStream_t s, int blk, const float* y1, const Slot& sl, const float* in2, float* out2, float sign,
                 bool keep_h = true) {
        RC((ln_forward<T, T>(s, y1, P(blk, T_LN2G), P(blk, T_LN2B), c.ln_eps, sl.n2, sl.st2, M, D)));
        Epi e = epi0(); e.kind = EPI_BIAS_GELU; e.out = keep_h ? sl.h : nullptr; e.out2 = sl.a; e.bias = P(blk, T_BFC1); e.ldo = Dm;
        RC(Ops<T>::nt(s, sl.n2, D, P(blk, T_WFC1), D, M, Dm, D, e));
        Epi r = epi0(); r.kind = EPI_RESIDUAL; r.outf = out2; r.res = in2; r.bias = P(blk, T_BFC2); r.sign = sign; r.ldo = D;
        return Ops<T>::nt(s, sl.a, Dm, P(blk, T_WFC2), Dm, M, D, Dm, r);
    }

    // forward of block blk (0-based): (x1,x2) -> (y1,y2)
    int forward_block(hipStream_t s, int blk, const float* x1, const float* x2, float* y1, float* y2) {
        Slot sl = slot(0);
        RC(f_pre(s, blk, x2, sl));
        RC(f_post(s, blk, sl, x1, y1, 1.f));
        return g_branch(s, blk, y1, sl, x2, y2, 1.f, false);
    }

    // R_i: (y1,y2) -> (x1,x2) and the slot of block blk
    int recompute(hipStream_t s, int blk, const float* y1, const float* y2, float* x1, float* x2) {
        Slot sl = slot(blk);
        RC(g_branch(s, blk, y1, sl, y2, x2, -1.f));
        RC(f_pre(s, blk, x2, sl));
        return f_post(s, blk, sl, y1, x1, -1.f);
    }

    // dA[M,Kin] = dC[M,Nout] * W[Nout,Kin], the weight read as it is stored
    int dgrad(hipStream_t s, int blk, int wt, const T* dC, int Nout, int Kin, const Epi& e) {
        if constexpr (kBf16) {
            return gemm_nn_bf16(s, dC, Nout, P(blk, wt), Kin, M, Kin, Nout, e);
        } else {
            return gemm_nn_f32(s, dC, Nout, P(blk, wt), Kin, M, Kin, Nout, e);
        }
    }

    // V_i is issued as two kernel sequences.
    //   grad_d: the input-gradient chain (everything the next block down waits for) plus the cheap
    //           vector/bias gradients that fall out of its kernels;
    //   grad_w: the four weight-gradient GEMMs, which only consume what grad_d and R_i produced.
    // Under PaReprop grad_w rides on the recompute stream, so it overlaps the chain of the same block.
    // y1: first stream of the block's outputs, x2: second stream of its inputs.
    // d1, d2: incoming cotangents (float32); d2b: act-typed copy of d2.
    // o1, o2: outgoing cotangents; o2b: act-typed copy of o2 (nullable).
    // ev (nullable): 3 events recorded on s when dh / gY1 / dqkv are complete.
    T* gy1_act(int blk, float* o1) const { return kBf16 ? at<T>(L.gy1b[blk & 1]) : reinterpret_cast<T*>(o1); }

    int grad_d(hipStream_t s, int blk, const float* y1, const float* x2, const float* d1, const float* d2,
               const T* d2b, float* o1, float* o2, T* o2b, const hipEvent_t* ev) {
        Slot sl = slot(blk);
        T* dhb = at<T>(L.dh[blk & 1]);
        T* dqkv = at<T>(L.dqkv[blk & 1]);
        T* dn = at<T>(L.dn);
        T* dO = at<T>(L.dO);
        float* pcol0 = at<float>(L.part_col[0]);
        float* pcol1 = at<float>(L.part_col[1]);
        T* gy1b = gy1_act(blk, o1);
        // second stages of the block's fixed-order sums are gathered and run as one launch at the end
        RedSeg segs[4];
        int nseg = 0;

        // ---- G branch: dh = (dY2 W2) * gelu'(h); the bias gradient of fc1 (column sums of dh) rides
        // in the epilogue of the matrix-core kernel, otherwise it is a separate pass
        Epi e = epi0(); e.kind = EPI_GELU_BWD; e.out = dhb; e.aux = sl.h; e.ldo = Dm;
        bool fused_db1 = false;
        if constexpr (kBf16) fused_db1 = gemm_bf16_fast_path(d2b, D, P(blk, T_WFC2), Dm, Dm, D, e);
        if (fused_db1) e.colsum = pcol0;
        RC(dgrad(s, blk, T_WFC2, d2b, D, Dm, e));
        if (ev) REV_HIP(hipEventRecord(ev[0], s));
        if (fused_db1) segs[nseg++] = {pcol0, G(blk, T_BFC1), nullptr, (int64_t)Dm, (int64_t)Dm, (int64_t)Dm, gemm_colsum_strips(M)};
        else RC(colsum<T>(s, dhb, Dm, M, Dm, G(blk, T_BFC1), pcol0, &segs[nseg++]));
        Epi p = epi0(); p.kind = EPI_PLAIN; p.out = dn; p.ldo = D;
        RC(dgrad(s, blk, T_WFC1, dhb, Dm, D, p));
        // gY1 = dY1 + LN2bwd(dn); its column sums are the bias gradient of the projection
        RC((ln_backward<T, T>(s, dn, y1, sl.st2, P(blk, T_LN2G), d1, o1, kBf16 ? gy1b : nullptr,
                              G(blk, T_LN2G), G(blk, T_BPROJ), at<float>(L.part_ln[0]), M, D, &segs[nseg++])));
        if (ev) REV_HIP(hipEventRecord(ev[1], s));
        // ---- F branch
        Epi q = epi0(); q.kind = EPI_PLAIN; q.out = dO; q.ldo = D;
        RC(dgrad(s, blk, T_WPROJ, gy1b, D, D, q));
        RC((attention_backward<T>(s, sl.qkv, sl.o, dO, sl.lse, dqkv, at<float>(L.delta), B, Tn, H, dh, key_len, solo)));
        if (ev) REV_HIP(hipEventRecord(ev[2], s));
        Epi r = epi0(); r.kind = EPI_PLAIN; r.out = dn; r.ldo = D;
        RC(dgrad(s, blk, T_WQKV, dqkv, 3 * D, D, r));
        RC(colsum<T>(s, dqkv, 3 * D, M, 3 * D, G(blk, T_BQKV), pcol1, &segs[nseg++]));
        // dX2 = dY2 + LN1bwd(dn); dX2 is the block below's dY2, so its column sums are that block's
        // fc2 bias gradient
        RC((ln_backward<T, T>(s, dn, x2, sl.st1, P(blk, T_LN1G), d2, o2, kBf16 ? o2b : nullptr,
                              G(blk, T_LN1G), blk > 0 ? G(blk - 1, T_BFC2) : nullptr, at<float>(L.part_ln[1]), M, D,
                              &segs[nseg++])));
        return reduce_multi(s, segs, nseg);
    }

    // ev (nullable): events to wait for on s before the kernels that read dY2 copy / dh / gY1 / dqkv
    // (4 events); done_w2 (nullable) is recorded after the fc2 weight gradient.
    int grad_w(hipStream_t s, int blk, const T* d2b, float* o1, const hipEvent_t* ev, hipEvent_t done_w2) {
        Slot sl = slot(blk);
        T* dhb = at<T>(L.dh[blk & 1]);
        T* dqkv = at<T>(L.dqkv[blk & 1]);
        float* pwg[4] = {nullptr, nullptr, nullptr, nullptr};
        if constexpr (kBf16) for (int w = 0; w < 4; ++w) pwg[w] = at<float>(L.part_wg[w]);
        T* gy1b = gy1_act(blk, o1);
        RedSeg segs[4];
        if constexpr (kBf16) {
            // all four in one launch: together their tiles fill the device without cutting the token range (or with
            // fewer cuts), which saves the float32 pieces and most of their reduction
            const WgradItem items[4] = {
                {d2b, D, sl.a, Dm, D, Dm, G(blk, T_WFC2), pwg[0], L.part_wg_elems[0]},
                {dhb, Dm, sl.n2, D, Dm, D, G(blk, T_WFC1), pwg[1], L.part_wg_elems[1]},
                {gy1b, D, sl.o, D, D, D, G(blk, T_WPROJ), pwg[2], L.part_wg_elems[2]},
                {dqkv, 3 * D, sl.n1, D, 3 * D, D, G(blk, T_WQKV), pwg[3], L.part_wg_elems[3]}};
            if (ev) for (int k = 0; k < 4; ++k) REV_HIP(hipStreamWaitEvent(s, ev[k], 0));
            RC(gemm_wgrad_bf16_group(s, items, 4, M, segs));
            if (done_w2) REV_HIP(hipEventRecord(done_w2, s));
            RedSeg live4[4];
            int n4 = 0;
            for (int w = 0; w < 4; ++w)
                if (segs[w].P > 0) live4[n4++] = segs[w];
            return reduce_multi(s, live4, n4);
        }
        if (ev) REV_HIP(hipStreamWaitEvent(s, ev[0], 0));
        RC(Ops<T>::wgrad(s, d2b, D, sl.a, Dm, M, D, Dm, G(blk, T_WFC2), pwg[0], L.part_wg_elems[0], &segs[0]));
        if (done_w2) REV_HIP(hipEventRecord(done_w2, s));
        if (ev) REV_HIP(hipStreamWaitEvent(s, ev[1], 0));
        RC(Ops<T>::wgrad(s, dhb, Dm, sl.n2, D, M, Dm, D, G(blk, T_WFC1), pwg[1], L.part_wg_elems[1], &segs[1]));
        if (ev) REV_HIP(hipStreamWaitEvent(s, ev[2], 0));
        RC(Ops<T>::wgrad(s, gy1b, D, sl.o, D, M, D, D, G(blk, T_WPROJ), pwg[2], L.part_wg_elems[2], &segs[2]));
        if (ev) REV_HIP(hipStreamWaitEvent(s, ev[3], 0));
        RC(Ops<T>::wgrad(s, dqkv, 3 * D, sl.n1, D, M, 3 * D, D, G(blk, T_WQKV), pwg[3], L.part_wg_elems[3], &segs[3]));
        // one launch for the split reductions of all four
        RedSeg live[4];
        int nseg = 0;
        for (int w = 0; w < 4; ++w)
            if (segs[w].P > 0) live[nseg++] = segs[w];
        return reduce_multi(s, live, nseg);
    }

    // residual level `lvl` (0..N): stream s1/s2 pointers
    struct Ptrs { const float* in1; const float* in2; float* out1; float* out2; };
    float* res(int lvl, int st, float* x_out1, float* x_out2) const {
        if (lvl == 0 && st == 0 && x_out1) return x_out1;
        if (lvl == 0 && st == 1 && x_out2) return x_out2;
        return at<float>(L.ring[lvl % L.ring_levels][st]);
    }

    // schedule: 0 = Reprop, 1 = PaReprop, 2 = R chain only, 3 = V chain only
    //
    // PaReprop, stream by stream (block indices 1-based, N at the top):
    //   sr:  R_N | R_{N-1}  W_N | R_{N-2}  W_{N-1} | ...      (W_i = grad_w of block i)
    //   sv:  D_N | D_{N-1}      | D_{N-2}          | ...      (D_i = grad_d of block i)
    // Orderings across the streams (events):
    //   D_i  after R_i                      (activations of block i exist)
    //   D_i  after W_{i+2}                  (dh/dqkv/gY1 buffers of the same parity are free again)
    //   D_i  after the fc2 weight gradient of W_{i+1}   (it reads the dY2 copy that D_i's last kernel rewrites)
    //   R_i  after D_{i+2}                  (slot i mod 2 and ring level i+2 are free; W_{i+2} precedes R_i on sr)
    //   W_i after the kernels of D_i that produce its cotangent operands (bf16 mode: one launch for the four GEMMs,
    //   so after all of them; float32 mode: each GEMM after its own)
    // and sv finally waits for W_1, so everything is ordered before later work on sv.
    int backward(int schedule, const float* Y1, const float* Y2, const float* dY1, const float* dY2,
                 float* dX1, float* dX2, float* X1o, float* X2o, hipStream_t sv, hipStream_t sr) {
        const int N = c.n_blocks;
        const bool doR = schedule != 3, doV = schedule != 2;
        // per block: 0 R done, 1 D done, 2 W done, 3 dY2 copy ready (= D start), 4 dh, 5 gY1, 6 dqkv, 7 fc2 wgrad done
        constexpr int EPB = 8;
        EventLease lease;
        std::vector<hipEvent_t>& ev = lease.ev;
        auto E = [&](int i, int k) { return ev[(i - 1) * EPB + k]; };
        if (schedule == 1) {
            RC(lease.take(EPB * N + 1));
            REV_HIP(hipEventRecord(ev[EPB * N], sv));            // fork
            REV_HIP(hipStreamWaitEvent(sr, ev[EPB * N], 0));
        } else {
            sr = sv;
        }
        const T* top2b = nullptr;
        if (doV) {
            // fc2 bias gradient of the top block: column sums of the incoming dY2 (lower blocks get
            // theirs from the LayerNorm-backward kernel that produces their dY2)
            RC(colsum<float>(sv, dY2, D, M, D, G(N - 1, T_BFC2), at<float>(L.part_col[1])));
            if constexpr (kBf16) {
                T* b = at<T>(L.cot2b[N & 1]);
                RC(convert_f32_to_bf16(sv, dY2, b, (int64_t)M * D));
                top2b = b;
            } else {
                top2b = reinterpret_cast<const T*>(dY2);
            }
        }
        auto run_R = [&](int i) -> int {   // i = N..1 (1-based block index)
            const float* y1 = (i == N) ? Y1 : res(i, 0, X1o, X2o);
            const float* y2 = (i == N) ? Y2 : res(i, 1, X1o, X2o);
            return recompute(sr, i - 1, y1, y2, res(i - 1, 0, X1o, X2o), res(i - 1, 1, X1o, X2o));
        };
        auto d2b_of = [&](int i) -> const T* {
            if constexpr (kBf16) return (i == N) ? top2b : at<T>(L.cot2b[i & 1]);
            else return reinterpret_cast<const T*>((i == N) ? dY2 : at<float>(L.cot[i & 1][1]));
        };
        auto o1_of = [&](int i) -> float* { return (i == 1) ? dX1 : at<float>(L.cot[(i - 1) & 1][0]); };
        auto run_D = [&](int i, const hipEvent_t* evs) -> int {
            const float* y1 = (i == N) ? Y1 : res(i, 0, X1o, X2o);
            const float* x2 = res(i - 1, 1, X1o, X2o);
            const float* d1 = (i == N) ? dY1 : at<float>(L.cot[i & 1][0]);
            const float* d2 = (i == N) ? dY2 : at<float>(L.cot[i & 1][1]);
            float* o2 = (i == 1) ? dX2 : at<float>(L.cot[(i - 1) & 1][1]);
            T* o2b = nullptr;
            if constexpr (kBf16) o2b = (i == 1) ? nullptr : at<T>(L.cot2b[(i - 1) & 1]);
            return grad_d(sv, i - 1, y1, x2, d1, d2, d2b_of(i), o1_of(i), o2, o2b, evs);
        };
        if (schedule == 1) {
            RC(run_R(N));
            REV_HIP(hipEventRecord(E(N, 0), sr));
            for (int i = N; i >= 1; --i) {
                // ---- D_i on the gradient stream
                REV_HIP(hipStreamWaitEvent(sv, E(i, 0), 0));
                if (i + 2 <= N) REV_HIP(hipStreamWaitEvent(sv, E(i + 2, 2), 0));
                if (i + 1 <= N) REV_HIP(hipStreamWaitEvent(sv, E(i + 1, 7), 0));
                REV_HIP(hipEventRecord(E(i, 3), sv));
                const hipEvent_t dev[3] = {E(i, 4), E(i, 5), E(i, 6)};
                RC(run_D(i, dev));
                REV_HIP(hipEventRecord(E(i, 1), sv));
                // ---- R_{i-1}, then W_i, on the recompute stream
                if (i - 1 >= 1) {
                    if (i + 1 <= N) REV_HIP(hipStreamWaitEvent(sr, E(i + 1, 1), 0));
                    RC(run_R(i - 1));
                    REV_HIP(hipEventRecord(E(i - 1, 0), sr));
                }
                const hipEvent_t wev[4] = {E(i, 3), E(i, 4), E(i, 5), E(i, 6)};
                RC(grad_w(sr, i - 1, d2b_of(i), o1_of(i), wev, E(i, 7)));
                REV_HIP(hipEventRecord(E(i, 2), sr));
            }
            REV_HIP(hipStreamWaitEvent(sv, E(1, 2), 0));          // join (W_2 precedes W_1 on sr)
        } else {
            for (int i = N; i >= 1; --i) {
                if (doR) RC(run_R(i));
                if (doV) {
                    RC(run_D(i, nullptr));
                    RC(grad_w(sv, i - 1, d2b_of(i), o1_of(i), nullptr, nullptr));
                }
            }
        }
        return REV_OK;
    }

    int forward(const float* X1, const float* X2, float* Y1, float* Y2, hipStream_t s) {
        const int N = c.n_blocks;
        for (int i = 1; i <= N; ++i) {
            const float* x1 = (i == 1) ? X1 : at<float>(L.ring[(i - 1) % L.ring_levels][0]);
            const float* x2 = (i == 1) ? X2 : at<float>(L.ring[(i - 1) % L.ring_levels][1]);
            float* y1 = (i == N) ? Y1 : at<float>(L.ring[i % L.ring_levels][0]);
            float* y2 = (i == N) ? Y2 : at<float>(L.ring[i % L.ring_levels][1]);
            RC(forward_block(s, i - 1, x1, x2, y1, y2));
        }
        return REV_OK;
    }
};

static int check_common(const rev_cfg* cfg, const void* ws, int64_t ws_bytes, bool compact) {
    RC(check_cfg(cfg));
    if (!ws) { set_error("workspace is null"); return REV_EINVAL; }
    if (((uintptr_t)ws & 255) != 0) { set_error("workspace must be 256-byte aligned"); return REV_EINVAL; }
    Layout L = make_layout(*cfg, compact);
    if (ws_bytes < L.total) {
        set_error("workspace too small: need " + std::to_string(L.total) + " bytes, got " + std::to_string(ws_bytes));
        return REV_EWORKSPACE;
    }
    return REV_OK;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

static int backward_entry(int schedule, const rev_cfg* cfg, const void* params, const float* Y1, const float* Y2,
                          const float* dY1, const float* dY2, float* dX1, float* dX2, float* X1o, float* X2o,
                          float* dparams, void* ws, int64_t ws_bytes, void* sv, void* sr,
                          const int32_t* key_len = nullptr) {
    const bool compact = schedule == 0;          // the sequential schedule runs in the smaller layout
    RC(check_common(cfg, ws, ws_bytes, compact));
    if (!params || !Y1 || !Y2 || !dY1 || !dY2 || !dX1 || !dX2 || !dparams) {
        set_error("a required pointer is null"); return REV_EINVAL;
    }
    if (!aligned16(params) || !aligned16(Y1) || !aligned16(Y2) || !aligned16(dY1) || !aligned16(dY2) || !aligned16(dX1) ||
        !aligned16(dX2) || !aligned16(dparams) || !aligned16(X1o) || !aligned16(X2o)) {
        set_error("every buffer must be 16-byte aligned"); return REV_EINVAL;
    }
    if (schedule == 1 && sv == sr) { set_error("PaReprop needs two different streams"); return REV_EINVAL; }
    if (((uintptr_t)key_len & 3) != 0) { set_error("key_len must be 4-byte aligned"); return REV_EINVAL; }
    if (cfg->mode == REV_MODE_BF16) {
        Runner<bf16> r(*cfg, params, dparams, ws, compact);
        r.key_len = key_len;
        return r.backward(schedule, Y1, Y2, dY1, dY2, dX1, dX2, X1o, X2o, (hipStream_t)sv, (hipStream_t)sr);
    }
    Runner<float> r(*cfg, params, dparams, ws, compact);
    r.key_len = key_len;
    return r.backward(schedule, Y1, Y2, dY1, dY2, dX1, dX2, X1o, X2o, (hipStream_t)sv, (hipStream_t)sr);
}

// ---------------------------------------------------------------------------------
// file-scope scratch of the allocation-free entry point
// ---------------------------------------------------------------------------------
// The workspace of rev_stack_backward_reprop_static: every GPU the library runs on holds its own copy of this
// array from the moment the code object is loaded until the process ends.  In host code the name `scratch` is only
// a stand-in for the symbol: the device address is looked up once per device and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[REV_STATIC_WORKSPACE_BYTES];

static std::mutex g_scratch_mu;
static std::vector<void*> g_scratch_ptr;     // indexed by device ordinal; nullptr = not looked up yet

// device address of `scratch` on the current device
static int scratch_address(void** out) {
    int dev = 0;
    REV_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if ((int)g_scratch_ptr.size() <= dev) g_scratch_ptr.resize(dev + 1, nullptr);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        REV_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p & 255) != 0) { set_error("static workspace: bad symbol address"); return REV_EHIP; }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return REV_OK;
}

}  // namespace rev

using namespace rev;

extern "C" {

int rev_stack_check_cfg(const rev_cfg* cfg) { return check_cfg(cfg); }

int64_t rev_stack_param_count(const rev_cfg* cfg) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    return block_params(*cfg) * cfg->n_blocks;
}

int64_t rev_stack_param_offset(const rev_cfg* cfg, int32_t block, int32_t tensor, int64_t* count) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (block < 0 || block >= cfg->n_blocks || tensor < 0 || tensor >= T_COUNT) {
        set_error("param_offset: block or tensor index out of range"); return REV_EINVAL;
    }
    if (count) *count = tensor_count(*cfg, tensor);
    return block_params(*cfg) * block + tensor_offset(*cfg, tensor);
}

int64_t rev_stack_workspace_bytes(const rev_cfg* cfg) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    return make_layout(*cfg, false).total;
}

int64_t rev_stack_workspace_bytes_reprop(const rev_cfg* cfg) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    return make_layout(*cfg, true).total;
}

int64_t rev_stack_slot_bytes(const rev_cfg* cfg) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    return make_layout(*cfg, true).slot_bytes;
}

static int forward_entry(const rev_cfg* cfg, const void* params, const float* X1, const float* X2, float* Y1, float* Y2,
                         void* ws, int64_t ws_bytes, void* stream, const int32_t* key_len) {
    RC(check_common(cfg, ws, ws_bytes, true));
    if (!params || !X1 || !X2 || !Y1 || !Y2) { set_error("a required pointer is null"); return REV_EINVAL; }
    if (!aligned16(params) || !aligned16(X1) || !aligned16(X2) || !aligned16(Y1) || !aligned16(Y2)) {
        set_error("every buffer must be 16-byte aligned"); return REV_EINVAL;
    }
    if (((uintptr_t)key_len & 3) != 0) { set_error("key_len must be 4-byte aligned"); return REV_EINVAL; }
    if (cfg->mode == REV_MODE_BF16) {
        Runner<bf16> r(*cfg, params, nullptr, ws, true);
        r.key_len = key_len;
        return r.forward(X1, X2, Y1, Y2, (hipStream_t)stream);
    }
    Runner<float> r(*cfg, params, nullptr, ws, true);
    r.key_len = key_len;
    return r.forward(X1, X2, Y1, Y2, (hipStream_t)stream);
}

int rev_stack_forward(const rev_cfg* cfg, const void* params, const float* X1, const float* X2, float* Y1, float* Y2,
                      void* ws, int64_t ws_bytes, void* stream) {
    return forward_entry(cfg, params, X1, X2, Y1, Y2, ws, ws_bytes, stream, nullptr);
}

int rev_stack_forward_masked(const rev_cfg* cfg, const void* params, const float* X1, const float* X2,
                             const int32_t* key_len, float* Y1, float* Y2, void* ws, int64_t ws_bytes, void* stream) {
    if (!key_len) { set_error("key_len is null"); return REV_EINVAL; }
    return forward_entry(cfg, params, X1, X2, Y1, Y2, ws, ws_bytes, stream, key_len);
}

int rev_stack_backward_reprop(const rev_cfg* cfg, const void* params, const float* Y1, const float* Y2,
                              const float* dY1, const float* dY2, float* dX1, float* dX2, float* X1_out, float* X2_out,
                              float* dparams, void* ws, int64_t ws_bytes, void* stream) {
    return backward_entry(0, cfg, params, Y1, Y2, dY1, dY2, dX1, dX2, X1_out, X2_out, dparams, ws, ws_bytes, stream, stream);
}

int rev_stack_backward_reprop_static(const rev_cfg* cfg, const void* params, const float* Y1, const float* Y2,
                                     const float* dY1, const float* dY2, float* dX1, float* dX2, float* X1_out,
                                     float* X2_out, float* dparams, void* stream) {
    RC(check_cfg(cfg));
    const int64_t need = make_layout(*cfg, true).total;
    if (need > (int64_t)REV_STATIC_WORKSPACE_BYTES) {
        set_error("static workspace too small for this shape: the sequential schedule needs " + std::to_string(need) +
                  " bytes, the built-in buffer holds " + std::to_string((int64_t)REV_STATIC_WORKSPACE_BYTES) +
                  "; use rev_stack_backward_reprop with a caller-provided workspace");
        return REV_EWORKSPACE;
    }
    void* ws = nullptr;
    RC(scratch_address(&ws));
    return backward_entry(0, cfg, params, Y1, Y2, dY1, dY2, dX1, dX2, X1_out, X2_out, dparams, ws,
                          (int64_t)REV_STATIC_WORKSPACE_BYTES, stream, stream);
}

int rev_stack_backward_pareprop(const rev_cfg* cfg, const void* params, const float* Y1, const float* Y2,
                                const float* dY1, const float* dY2, float* dX1, float* dX2, float* X1_out, float* X2_out,
                                float* dparams, void* ws, int64_t ws_bytes, void* stream_grad, void* stream_recompute) {
    return backward_entry(1, cfg, params, Y1, Y2, dY1, dY2, dX1, dX2, X1_out, X2_out, dparams, ws, ws_bytes,
                          stream_grad, stream_recompute);
}

int rev_stack_backward_reprop_masked(const rev_cfg* cfg, const void* params, const float* Y1, const float* Y2,
                                     const int32_t* key_len, const float* dY1, const float* dY2, float* dX1, float* dX2,
                                     float* X1_out, float* X2_out, float* dparams, void* ws, int64_t ws_bytes,
                                     void* stream) {
    if (!key_len) { set_error("key_len is null"); return REV_EINVAL; }
    return backward_entry(0, cfg, params, Y1, Y2, dY1, dY2, dX1, dX2, X1_out, X2_out, dparams, ws, ws_bytes, stream, stream,
                          key_len);
}

int rev_stack_backward_pareprop_masked(const rev_cfg* cfg, const void* params, const float* Y1, const float* Y2,
                                       const int32_t* key_len, const float* dY1, const float* dY2, float* dX1, float* dX2,
                                       float* X1_out, float* X2_out, float* dparams, void* ws, int64_t ws_bytes,
                                       void* stream_grad, void* stream_recompute) {
    if (!key_len) { set_error("key_len is null"); return REV_EINVAL; }
    return backward_entry(1, cfg, params, Y1, Y2, dY1, dY2, dX1, dX2, X1_out, X2_out, dparams, ws, ws_bytes,
                          stream_grad, stream_recompute, key_len);
}

int rev_stack_backward_chain(const rev_cfg* cfg, const void* params, const float* Y1, const float* Y2,
                             const float* dY1, const float* dY2, float* dX1, float* dX2, float* X1_out, float* X2_out,
                             float* dparams, void* ws, int64_t ws_bytes, void* stream, int32_t chain) {
    if (chain != 0 && chain != 1) { set_error("chain must be 0 or 1"); return REV_EINVAL; }
    return backward_entry(chain == 0 ? 2 : 3, cfg, params, Y1, Y2, dY1, dY2, dX1, dX2, X1_out, X2_out, dparams, ws,
                          ws_bytes, stream, stream);
}

int rev_sgd_step(int64_t n, float* master, void* params_bf16, const float* grad, float lr, void* stream) {
    if (n <= 0) { set_error("sgd: n must be positive"); return REV_EINVAL; }
    if (!master || !grad) { set_error("sgd: a required pointer is null"); return REV_EINVAL; }
    if (!(lr >= 0.f)) { set_error("sgd: need lr >= 0"); return REV_EINVAL; }
    if (!aligned16(master) || !aligned16(grad) || ((uintptr_t)params_bf16 & 7) != 0) {
        set_error("sgd: float32 buffers must be 16-byte aligned, the bf16 copy 8-byte aligned"); return REV_EINVAL;
    }
    return sgd_step((hipStream_t)stream, n, master, params_bf16, grad, lr);
}

int rev_adamw_step(int64_t n, float* master, void* params_bf16, const float* grad, float* m, float* v,
                   int32_t step, float lr, float beta1, float beta2, float eps, float weight_decay, void* stream) {
    if (n <= 0) { set_error("adamw: n must be positive"); return REV_EINVAL; }
    if (!master || !grad || !m || !v) { set_error("adamw: a required pointer is null"); return REV_EINVAL; }
    if (step < 1) { set_error("adamw: the step counter starts at 1"); return REV_EINVAL; }
    if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f) || !(lr >= 0.f) ||
        !(weight_decay >= 0.f)) {
        set_error("adamw: need 0 <= beta < 1, eps >= 0, lr >= 0, weight_decay >= 0"); return REV_EINVAL;
    }
    if (!aligned16(master) || !aligned16(grad) || !aligned16(m) || !aligned16(v) || ((uintptr_t)params_bf16 & 7) != 0) {
        set_error("adamw: float32 buffers must be 16-byte aligned, the bf16 copy 8-byte aligned"); return REV_EINVAL;
    }
    return adamw_step((hipStream_t)stream, n, master, params_bf16, grad, m, v, step, lr, beta1, beta2, eps, weight_decay);
}

int rev_profile_begin(void) {
    for (auto& r : g_prof_recs) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
    g_prof_recs.clear();
    for (int k = 0; k < K_COUNT; ++k) { g_prof_ms[k] = 0; g_prof_n[k] = 0; g_prof_work[k] = 0; }
    g_prof_on = true;
    return REV_OK;
}

int rev_profile_end(void) {
    g_prof_on = false;
    REV_HIP(hipDeviceSynchronize());
    for (auto& r : g_prof_recs) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.e0, r.e1) == hipSuccess) { g_prof_ms[r.kind] += ms; g_prof_n[r.kind] += 1; }
        (void)hipEventDestroy(r.e0);
        (void)hipEventDestroy(r.e1);
    }
    g_prof_recs.clear();
    return REV_OK;
}

int rev_profile_kinds(void) { return K_COUNT; }
const char* rev_profile_name(int kind) { return (kind >= 0 && kind < K_COUNT) ? g_kind_names[kind] : ""; }
int rev_profile_is_flops(int kind) { return (kind >= 0 && kind < K_COUNT) ? g_kind_flops[kind] : 0; }
int rev_profile_get(int kind, double* total_ms, int64_t* launches, double* work) {
    if (kind < 0 || kind >= K_COUNT) { set_error("profile_get: bad kind"); return REV_EINVAL; }
    if (total_ms) *total_ms = g_prof_ms[kind];
    if (launches) *launches = g_prof_n[kind];
    if (work) *work = g_prof_work[kind];
    return REV_OK;
}

const char* rev_last_error(void) { return g_err.c_str(); }

}  // extern "C"
